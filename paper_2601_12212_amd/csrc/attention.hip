// Tree-masked attention of the tree tokens against [KV prefix | tree keys].
//
// bf16 path (MFMA).  Query rows of one kv head are the (node, group head) pairs, packed as
// the N dimension of S^T = K Q^T so that every lane owns ONE query column of the 32x32
// score block: the softmax statistics are lane-local plus one exchange with lane^32.  The
// probabilities come out of the S^T accumulator in exactly the register layout the B
// operand of O^T = V^T P^T wants, so P never leaves registers.  K tiles are staged in LDS
// row-major, V tiles transposed ([d][key], key order permuted to match the accumulator
// layout).  The prefix may be split across workgroups (partial max / sum / O, merged by a
// second kernel) when a batch offers too few (sequence, kv head, row tile) items to fill
// the chip.  The ancestor bitset is applied only to key blocks that contain tree keys.
//
// fp32 path: plain ALU kernel, one wave per (node, head); a correctness path for small
// problems and for head sizes the MFMA path does not cover.
#include "common.hpp"
#include "kernels.hpp"

namespace dt {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

#define ATT_KB 32           // keys per block
#define ATT_ROWS_PER_WAVE 32
#define ATT_WAVES 4
#define ATT_MTILE (ATT_ROWS_PER_WAVE * ATT_WAVES)
#define K_PITCH (128 + 8)   // bf16 elements per K row in LDS (272 B: conflict-free 16 B reads)
#define VT_PITCH 40         // bf16 elements per V^T row in LDS (80 B)
#define ATT_MAX_SPLITS 16

// position of key kk (0..31) inside a V^T row: 16-byte unit (step, lane half) then index,
// mirroring which accumulator registers of S^T a lane holds (rows 8*(i/4) + 4*half + i%4).
__device__ __forceinline__ int vt_pos(int kk) {
    const int step = kk >> 4, q = kk & 15;
    const int half = (q >> 2) & 1, idx = ((q >> 3) << 2) | (q & 3);
    return step * 16 + half * 8 + idx;
}

struct Partial {
    float *o;    // [batch, splits, TT_cap, Hq, D]
    float2 *ml;  // [batch, splits, TT_cap, Hq]  (running max of scale*score, sum)
};

template <int D>
__global__ __launch_bounds__(256) void attn_mfma_kernel(AttnArgs a, int splits, Partial part) {
    static_assert(D == 128, "head dim");
    constexpr int KSTEPS = D / 16, DBLK = D / 32;
    const int G = a.Hq / a.Hkv;
    const int b = blockIdx.z / splits, sp = blockIdx.z % splits, h = blockIdx.y;
    const int N = min(max(a.n_nodes[b], 1), a.TT_cap);
    const int M = N * G;
    const int m0 = blockIdx.x * ATT_MTILE;
    if (m0 >= M) return;
    const int L = max(a.prefix_len[b], 0);
    const int Tk = L + N;
    const int nb = (Tk + ATT_KB - 1) / ATT_KB;
    const int per = (nb + splits - 1) / splits;
    const int kb0 = sp * per, kb1 = min(nb, kb0 + per);

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int half = lane >> 5, col = lane & 31;
    const int mq = m0 + w * ATT_ROWS_PER_WAVE + col;  // this lane's query row
    const bool qvalid = mq < M;
    const int node = qvalid ? mq / G : 0;
    const int hq = h * G + (qvalid ? mq % G : 0);

    __shared__ __attribute__((aligned(16))) __bf16 s_k[ATT_KB * K_PITCH];
    __shared__ __attribute__((aligned(16))) __bf16 s_vt[D * VT_PITCH];

    // ---- Q as the B operand of S^T = K Q^T: k-step s, lane half g -> d = 16 s + 8 g .. +8 --
    bf16x8 qreg[KSTEPS];
    {
        const __bf16 *qp = (const __bf16 *)a.q + (((int64_t)b * a.TT_cap + node) * a.Hq + hq) * D;
#pragma unroll
        for (int s = 0; s < KSTEPS; ++s) {
            if (qvalid) qreg[s] = *(const bf16x8 *)(qp + 16 * s + 8 * half);
            else
#pragma unroll
                for (int e = 0; e < 8; ++e) qreg[s][e] = (__bf16)0.f;
        }
    }
    const u64 mask0 = a.anc_mask[((int64_t)b * a.TT_cap + node) * DT_MASK_WORDS];
    const u64 mask1 = a.anc_mask[((int64_t)b * a.TT_cap + node) * DT_MASK_WORDS + 1];

    f32x16 oacc[DBLK];
#pragma unroll
    for (int db = 0; db < DBLK; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[db][i] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;
    const float c = a.scale * 1.4426950408889634f;

    const __bf16 *kpre = (const __bf16 *)a.k_prefix[b], *vpre = (const __bf16 *)a.v_prefix[b];
    const __bf16 *ktree = (const __bf16 *)a.k_tree + (int64_t)b * a.TT_cap * a.Hkv * D;
    const __bf16 *vtree = (const __bf16 *)a.v_tree + (int64_t)b * a.TT_cap * a.Hkv * D;

    // staging role of this thread: key row tid/8 of the block, 16 d's starting at (tid%8)*16
    const int skey = tid >> 3, sd0 = (tid & 7) * 16;

    for (int kb = kb0; kb < kb1; ++kb) {
        // ---- stage K (row-major) and V (transposed) of this key block ---------------------
        {
            const int t = kb * ATT_KB + skey;
            bf16x8 k0, k1, v0, v1;
            if (t < Tk) {
                const __bf16 *kp, *vp;
                if (t < L) {
                    const int64_t off = (int64_t)t * a.kv_stride_tok + (int64_t)h * a.kv_stride_head + sd0;
                    kp = kpre + off; vp = vpre + off;
                } else {
                    const int64_t off = ((int64_t)(t - L) * a.Hkv + h) * D + sd0;
                    kp = ktree + off; vp = vtree + off;
                }
                k0 = *(const bf16x8 *)kp; k1 = *(const bf16x8 *)(kp + 8);
                v0 = *(const bf16x8 *)vp; v1 = *(const bf16x8 *)(vp + 8);
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) { k0[e] = k1[e] = v0[e] = v1[e] = (__bf16)0.f; }
            }
            *(bf16x8 *)(s_k + skey * K_PITCH + sd0) = k0;
            *(bf16x8 *)(s_k + skey * K_PITCH + sd0 + 8) = k1;
            const int pos = vt_pos(skey);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                s_vt[(sd0 + e) * VT_PITCH + pos] = v0[e];
                s_vt[(sd0 + 8 + e) * VT_PITCH + pos] = v1[e];
            }
        }
        __syncthreads();

        // ---- S^T block: 32 keys x 32 queries ---------------------------------------------------
        f32x16 sacc;
#pragma unroll
        for (int i = 0; i < 16; ++i) sacc[i] = 0.f;
#pragma unroll
        for (int s = 0; s < KSTEPS; ++s) {
            const bf16x8 ka = *(const bf16x8 *)(s_k + col * K_PITCH + 16 * s + 8 * half);
            sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qreg[s], sacc, 0, 0, 0);
        }
        // ---- mask, online softmax (this lane: one query, 16 of the 32 keys) ---------------
        const int tbase = kb * ATT_KB;
        const bool has_tree = tbase + ATT_KB > L;
        float mloc = -INFINITY;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int t = tbase + 8 * (i >> 2) + 4 * half + (i & 3);
            bool vis = true;
            if (has_tree) {
                const int j = t - L;
                if (j >= 0) vis = j < N && (((j < 64 ? mask0 : mask1) >> (j & 63)) & 1ull);
            }
            sacc[i] = vis ? sacc[i] : -INFINITY;
            mloc = fmaxf(mloc, sacc[i]);
        }
        mloc = fmaxf(mloc, __shfl_xor(mloc, 32, 64));
        const float m_new = fmaxf(m_run, mloc);
        const float m_use = m_new == -INFINITY ? 0.f : m_new;
        const float alpha = __builtin_amdgcn_exp2f((m_run - m_use) * c);  // m_run = -inf -> 0
        float psum = 0.f;
        bf16x8 pb[2];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const float p = __builtin_amdgcn_exp2f((sacc[i] - m_use) * c);
            psum += p;
            pb[i >> 3][i & 7] = (__bf16)p;
        }
        l_run = l_run * alpha + psum;
        m_run = m_new;
#pragma unroll
        for (int db = 0; db < DBLK; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) oacc[db][i] *= alpha;
        // ---- O^T += V^T P^T ------------------------------------------------------------------------
#pragma unroll
        for (int db = 0; db < DBLK; ++db)
#pragma unroll
            for (int st = 0; st < 2; ++st) {
                const bf16x8 va = *(const bf16x8 *)(s_vt + (32 * db + col) * VT_PITCH + st * 16 + half * 8);
                oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pb[st], oacc[db], 0, 0, 0);
            }
        __syncthreads();
    }

    // ---- epilogue -------------------------------------------------------------------------------
    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    if (!qvalid) return;
    const int64_t row = ((int64_t)b * a.TT_cap + node) * a.Hq + hq;
    if (splits == 1) {
        const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
        __bf16 *op = (__bf16 *)a.out + row * D;
#pragma unroll
        for (int db = 0; db < DBLK; ++db)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                bf16x4 o4;
#pragma unroll
                for (int e = 0; e < 4; ++e) o4[e] = (__bf16)(oacc[db][q4 * 4 + e] * inv);
                *(bf16x4 *)(op + 32 * db + 8 * q4 + 4 * half) = o4;
            }
    } else {
        const int64_t prow = (((int64_t)b * splits + sp) * a.TT_cap + node) * a.Hq + hq;
        float *op = part.o + prow * D;
#pragma unroll
        for (int db = 0; db < DBLK; ++db)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                float4 o4 = make_float4(oacc[db][q4 * 4], oacc[db][q4 * 4 + 1], oacc[db][q4 * 4 + 2],
                                        oacc[db][q4 * 4 + 3]);
                *(float4 *)(op + 32 * db + 8 * q4 + 4 * half) = o4;
            }
        if (half == 0) part.ml[prow] = make_float2(m_run, l_tot);
    }
}

// Merge the per-split partials: one thread per (row, 4 output columns).
template <int D>
__global__ __launch_bounds__(256) void attn_combine_kernel(AttnArgs a, int splits, Partial part) {
    const int b = blockIdx.y;
    const int N = min(max(a.n_nodes[b], 1), a.TT_cap);
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int c4 = (int)(idx % (D / 4));
    const int64_t r = idx / (D / 4);  // row inside the sequence: node * Hq + head
    if (r >= (int64_t)N * a.Hq) return;
    const float c = a.scale * 1.4426950408889634f;
    float M = -INFINITY;
    for (int sp = 0; sp < splits; ++sp)
        M = fmaxf(M, part.ml[((int64_t)b * splits + sp) * a.TT_cap * a.Hq + r].x);
    const float Mu = M == -INFINITY ? 0.f : M;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    float l = 0.f;
    for (int sp = 0; sp < splits; ++sp) {
        const int64_t prow = ((int64_t)b * splits + sp) * a.TT_cap * a.Hq + r;
        const float2 ml = part.ml[prow];
        if (ml.y <= 0.f) continue;
        const float wgt = __builtin_amdgcn_exp2f((ml.x - Mu) * c);
        const float4 o = *(const float4 *)(part.o + prow * D + c4 * 4);
        acc.x += o.x * wgt; acc.y += o.y * wgt; acc.z += o.z * wgt; acc.w += o.w * wgt;
        l += ml.y * wgt;
    }
    const float inv = l > 0.f ? 1.0f / l : 0.f;
    bf16x4 o4;
    o4[0] = (__bf16)(acc.x * inv); o4[1] = (__bf16)(acc.y * inv);
    o4[2] = (__bf16)(acc.z * inv); o4[3] = (__bf16)(acc.w * inv);
    *(bf16x4 *)((__bf16 *)a.out + ((int64_t)b * a.TT_cap * a.Hq + r) * D + c4 * 4) = o4;
}

// ------------------------------------------------------------------------------ fp32 path --
// One wave per (node, head).  Keys are taken 64 at a time: lane j scores key j, the wave
// agrees on the running maximum, then lane c accumulates output columns c, c+64.
template <typename T>
__device__ __forceinline__ float ld(const T *p);
template <>
__device__ __forceinline__ float ld<float>(const float *p) { return *p; }
template <>
__device__ __forceinline__ float ld<uint16_t>(const uint16_t *p) { return bf16_bits_to_float(*p); }

template <typename T>
__global__ __launch_bounds__(64) void attn_simple_kernel(AttnArgs a) {
    const int node = blockIdx.x, hq = blockIdx.y, b = blockIdx.z, lane = threadIdx.x;
    const int N = min(max(a.n_nodes[b], 1), a.TT_cap);
    if (node >= N) return;
    const int D = a.D, G = a.Hq / a.Hkv, h = hq / G;
    const int L = max(a.prefix_len[b], 0), Tk = L + N;
    const int64_t row = ((int64_t)b * a.TT_cap + node) * a.Hq + hq;
    const T *q = (const T *)a.q + row * D;
    const T *kpre = (const T *)a.k_prefix[b], *vpre = (const T *)a.v_prefix[b];
    const T *ktree = (const T *)a.k_tree + (int64_t)b * a.TT_cap * a.Hkv * D;
    const T *vtree = (const T *)a.v_tree + (int64_t)b * a.TT_cap * a.Hkv * D;
    const u64 mask0 = a.anc_mask[((int64_t)b * a.TT_cap + node) * DT_MASK_WORDS];
    const u64 mask1 = a.anc_mask[((int64_t)b * a.TT_cap + node) * DT_MASK_WORDS + 1];

    __shared__ float s_q[128];
    for (int cidx = lane; cidx < D; cidx += 64) s_q[cidx] = ld(q + cidx);
    __syncthreads();

    float m_run = -INFINITY, l_run = 0.f, o0 = 0.f, o1 = 0.f;
    for (int t0 = 0; t0 < Tk; t0 += 64) {
        const int t = t0 + lane;
        bool vis = t < Tk;
        if (vis && t >= L) {
            const int j = t - L;
            vis = ((j < 64 ? mask0 : mask1) >> (j & 63)) & 1ull;
        }
        float s = -INFINITY;
        if (vis) {
            const T *kp = t < L ? kpre + (int64_t)t * a.kv_stride_tok + (int64_t)h * a.kv_stride_head
                                : ktree + ((int64_t)(t - L) * a.Hkv + h) * D;
            float dot = 0.f;
            for (int cidx = 0; cidx < D; ++cidx) dot = fmaf(s_q[cidx], ld(kp + cidx), dot);
            s = dot * a.scale;
        }
        const float m_new = fmaxf(m_run, wave_max(s));
        if (m_new == -INFINITY) continue;
        const float alpha = __expf(m_run - m_new);
        const float p = vis ? __expf(s - m_new) : 0.f;
        l_run = l_run * alpha + wave_sum(p);
        o0 *= alpha; o1 *= alpha;
        m_run = m_new;
        const int cnt = min(64, Tk - t0);
        for (int j = 0; j < cnt; ++j) {
            const float pj = __shfl(p, j, 64);
            if (pj == 0.f) continue;
            const int tj = t0 + j;
            const T *vp = tj < L ? vpre + (int64_t)tj * a.kv_stride_tok + (int64_t)h * a.kv_stride_head
                                 : vtree + ((int64_t)(tj - L) * a.Hkv + h) * D;
            if (lane < D) o0 = fmaf(pj, ld(vp + lane), o0);
            if (lane + 64 < D) o1 = fmaf(pj, ld(vp + lane + 64), o1);
        }
    }
    const float inv = l_run > 0.f ? 1.0f / l_run : 0.f;
    if (sizeof(T) == 4) {
        float *op = (float *)a.out + row * D;
        if (lane < D) op[lane] = o0 * inv;
        if (lane + 64 < D) op[lane + 64] = o1 * inv;
    } else {
        __bf16 *op = (__bf16 *)a.out + row * D;
        if (lane < D) op[lane] = (__bf16)(o0 * inv);
        if (lane + 64 < D) op[lane + 64] = (__bf16)(o1 * inv);
    }
}

// ------------------------------------------------------------------------------- launchers --
static size_t split_bytes(int batch, int TT_cap, int Hq, int D) {
    return (size_t)batch * TT_cap * Hq * ((size_t)D * 4 + 8);
}

size_t attn_workspace_bytes(int batch, int TT_cap, int Hq, int D) {
    // room for 8 splits, capped at 256 MiB (the launcher uses fewer splits if scratch is short)
    size_t want = split_bytes(batch, TT_cap, Hq, D) * 8;
    const size_t cap = (size_t)256 << 20;
    return want < cap ? want : cap;
}

int attn_launch(const AttnArgs &a, hipStream_t st, hipError_t *err) {
    *err = hipSuccess;
    if (a.batch <= 0) return DT_OK;
    const bool mfma = a.dtype == DT_BF16 && a.D == 128 && a.kv_stride_tok % 8 == 0 && a.kv_stride_head % 8 == 0;
    if (!mfma) {
        if (a.D > 128) return DT_ERR_LIMIT;
        dim3 grid(a.TT_cap, a.Hq, a.batch);
        ProfScope prof(KID_ATTN, st);
        if (a.dtype == DT_BF16) hipLaunchKernelGGL(attn_simple_kernel<uint16_t>, grid, dim3(64), 0, st, a);
        else hipLaunchKernelGGL(attn_simple_kernel<float>, grid, dim3(64), 0, st, a);
        *err = hipGetLastError();
        return *err == hipSuccess ? DT_OK : DT_ERR_HIP;
    }
    const int G = a.Hq / a.Hkv;
    const int mtiles = (a.TT_cap * G + ATT_MTILE - 1) / ATT_MTILE;
    const int base_wgs = a.batch * a.Hkv * mtiles;
    const int nb_max = (a.max_prefix_len + a.TT_cap + ATT_KB - 1) / ATT_KB;
    int splits = 1;
    if (base_wgs < 512) splits = (512 + base_wgs - 1) / base_wgs;
    if (splits > ATT_MAX_SPLITS) splits = ATT_MAX_SPLITS;
    if (splits > nb_max / 2) splits = nb_max / 2 > 0 ? nb_max / 2 : 1;
    const size_t per = split_bytes(a.batch, a.TT_cap, a.Hq, a.D);
    if (splits > 1 && (size_t)splits * per > a.ws_bytes) splits = (int)(a.ws_bytes / per);
    if (splits < 1) splits = 1;
    Partial part;
    part.o = (float *)a.ws;
    part.ml = (float2 *)((char *)a.ws + (size_t)a.batch * splits * a.TT_cap * a.Hq * a.D * 4);
    dim3 grid(mtiles, a.Hkv, a.batch * splits);
    {
        ProfScope prof(KID_ATTN, st);
        hipLaunchKernelGGL(attn_mfma_kernel<128>, grid, dim3(256), 0, st, a, splits, part);
    }
    *err = hipGetLastError();
    if (*err != hipSuccess) return DT_ERR_HIP;
    if (splits > 1) {
        const int64_t items = (int64_t)a.TT_cap * a.Hq * (a.D / 4);
        dim3 cgrid((unsigned)((items + 255) / 256), a.batch);
        {
            ProfScope prof(KID_ATTN_COMBINE, st);
            hipLaunchKernelGGL(attn_combine_kernel<128>, cgrid, dim3(256), 0, st, a, splits, part);
        }
        *err = hipGetLastError();
        if (*err != hipSuccess) return DT_ERR_HIP;
    }
    return DT_OK;
}

}  // namespace dt
