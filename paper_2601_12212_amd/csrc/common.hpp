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

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ u64 shfl_xor_u64(u64 v, int o) {
    u32 lo = __shfl_xor((u32)v, o, 64), hi = __shfl_xor((u32)(v >> 32), o, 64);
    return ((u64)hi << 32) | lo;
}
__device__ __forceinline__ u64 wave_max_u64(u64 v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        u64 w = shfl_xor_u64(v, o);
        v = w > v ? w : v;
    }
    return v;
}
__device__ __forceinline__ u64 readlane_u64(u64 v, int lane) {
    u32 lo = __builtin_amdgcn_readlane((u32)v, lane), hi = __builtin_amdgcn_readlane((u32)(v >> 32), lane);
    return ((u64)hi << 32) | lo;
}

// (max, sum of exp relative to max) pairs: the associative combine of log-sum-exp partials.
__device__ __forceinline__ void lse_combine(float &m, float &s, float m2, float s2) {
    float M = fmaxf(m, m2);
    if (M == -INFINITY) { m = M; s = 0.f; return; }
    s = s * __expf(m - M) + s2 * __expf(m2 - M);
    m = M;
}

}  // namespace dt
