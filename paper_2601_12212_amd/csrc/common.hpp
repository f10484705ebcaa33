// Device-side helpers shared by the gfx950 kernels: order-preserving keys, wave64
// reductions, bf16 access.  Wavefront size is 64 everywhere.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#define DT_WAVE 64

namespace dt {

typedef unsigned long long u64;
typedef uint32_t u32;

// ---- order-preserving integer image of a float (larger float <=> larger key) ----------
// -0 is folded onto +0 so that the integer order agrees with the float order exactly.
__device__ __forceinline__ u32 ord32(float f) {
    u32 u = __float_as_uint(f);
    if (u == 0x80000000u) u = 0u;
    return u ^ ((u >> 31) ? 0xFFFFFFFFu : 0x80000000u);
}
__device__ __forceinline__ float unord32(u32 k) {
    u32 u = (k & 0x80000000u) ? (k ^ 0x80000000u) : ~k;
    return __uint_as_float(u);
}
// 64-bit key of (value, index): larger value first, then SMALLER index.  Keys of distinct
// indices are distinct, so "greater key" is a strict total order.
__device__ __forceinline__ u64 make_key(float v, u32 idx) {
    return ((u64)ord32(v) << 32) | (u64)(0xFFFFFFFFu - idx);
}
__device__ __forceinline__ float key_val(u64 k) { return unord32((u32)(k >> 32)); }
__device__ __forceinline__ u32 key_idx(u64 k) { return 0xFFFFFFFFu - (u32)k; }

__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) { return __uint_as_float((u32)b << 16); }

// ---- wave64 primitives -------------------------------------------------------------------
__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & 63); }

__device__ __forceinline__ u32 lanes_below(u64 mask) {  // number of set bits of mask below this lane
    return __builtin_amdgcn_mbcnt_hi((u32)(mask >> 32), __builtin_amdgcn_mbcnt_lo((u32)mask, 0u));
}

// Wave-wide reductions with DPP row shifts and row broadcasts: six VALU steps, no LDS
// traffic.  The total lands in lane 63 and is broadcast from there, so the result is uniform.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int dpp_mov(int ident, int v) {
    return __builtin_amdgcn_update_dpp(ident, v, CTRL, ROW_MASK, 0xf, false);
}
#define DT_DPP_REDUCE(v, ident, OP, TO_I, FROM_I)                          \
    v = OP(v, FROM_I(dpp_mov<0x111, 0xf>(TO_I(ident), TO_I(v))));          \
    v = OP(v, FROM_I(dpp_mov<0x112, 0xf>(TO_I(ident), TO_I(v))));          \
    v = OP(v, FROM_I(dpp_mov<0x114, 0xf>(TO_I(ident), TO_I(v))));          \
    v = OP(v, FROM_I(dpp_mov<0x118, 0xf>(TO_I(ident), TO_I(v))));          \
    v = OP(v, FROM_I(dpp_mov<0x142, 0xa>(TO_I(ident), TO_I(v))));          \
    v = OP(v, FROM_I(dpp_mov<0x143, 0xc>(TO_I(ident), TO_I(v))));

__device__ __forceinline__ float f_add(float a, float b) { return a + b; }
__device__ __forceinline__ u32 u_max(u32 a, u32 b) { return a > b ? a : b; }
__device__ __forceinline__ int i_max(int a, int b) { return a > b ? a : b; }
__device__ __forceinline__ int i_add(int a, int b) { return a + b; }
__device__ __forceinline__ int id_i(int x) { return x; }
__device__ __forceinline__ int u2i(u32 x) { return (int)x; }
__device__ __forceinline__ u32 i2u(int x) { return (u32)x; }

__device__ __forceinline__ float wave_max(float v) {
    DT_DPP_REDUCE(v, -INFINITY, fmaxf, __float_as_int, __int_as_float)
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}
__device__ __forceinline__ float wave_sum(float v) {
    DT_DPP_REDUCE(v, 0.f, f_add, __float_as_int, __int_as_float)
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}
__device__ __forceinline__ u32 wave_max_u32(u32 v) {
    DT_DPP_REDUCE(v, 0u, u_max, u2i, i2u)
    return (u32)__builtin_amdgcn_readlane((int)v, 63);
}
__device__ __forceinline__ int wave_max_i32(int v) {
    DT_DPP_REDUCE(v, (int)0x80000000, i_max, id_i, id_i)
    return __builtin_amdgcn_readlane(v, 63);
}
__device__ __forceinline__ int wave_sum_i32(int v) {
    DT_DPP_REDUCE(v, 0, i_add, id_i, id_i)
    return __builtin_amdgcn_readlane(v, 63);
}
// inclusive prefix sum over the lanes of a wave (the same row shifts and row broadcasts)
__device__ __forceinline__ int wave_scan_incl_i32(int v) {
    DT_DPP_REDUCE(v, 0, i_add, id_i, id_i)
    return v;
}
// 64-bit maximum: the high words first, then the low words of the lanes that hold that high word.
__device__ __forceinline__ u64 wave_max_u64(u64 v) {
    const u32 hi = wave_max_u32((u32)(v >> 32));
    const u32 lo = wave_max_u32((u32)(v >> 32) == hi ? (u32)v : 0u);
    return ((u64)hi << 32) | lo;
}
__device__ __forceinline__ u64 shfl_xor_u64(u64 v, int o) {
    u32 lo = __shfl_xor((u32)v, o, 64), hi = __shfl_xor((u32)(v >> 32), o, 64);
    return ((u64)hi << 32) | lo;
}
__device__ __forceinline__ u64 readlane_u64(u64 v, int lane) {
    u32 lo = __builtin_amdgcn_readlane((u32)v, lane), hi = __builtin_amdgcn_readlane((u32)(v >> 32), lane);
    return ((u64)hi << 32) | lo;
}

// Philox4x32-10 (Salmon et al., SC'11): first output word for counter (c0,c1,c2,c3), key (k0,k1).
__device__ __forceinline__ u32 philox4x32_10_word0(u32 c0, u32 c1, u32 c2, u32 c3, u32 k0, u32 k1) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const u32 hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        const u32 hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        const u32 n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    return c0;
}
__device__ __forceinline__ float philox_uniform(u64 seed, u64 step, u32 seq, u32 node) {
    u32 x = philox4x32_10_word0(node, seq, (u32)step, (u32)(step >> 32), (u32)seed, (u32)(seed >> 32));
    return (float)(x >> 8) * (1.0f / 16777216.0f);
}

// (max, sum of exp relative to max) pairs: the associative combine of log-sum-exp partials.
__device__ __forceinline__ void lse_combine(float &m, float &s, float m2, float s2) {
    float M = fmaxf(m, m2);
    if (M == -INFINITY) { m = M; s = 0.f; return; }
    s = s * __expf(m - M) + s2 * __expf(m2 - M);
    m = M;
}

}  // namespace dt
