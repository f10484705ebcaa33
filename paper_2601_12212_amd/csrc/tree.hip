// Tree kernel: layer-wise expansion, rerank, and emission of the node arrays and the
// ancestor bitsets.  One workgroup per sequence; the whole candidate pool (at most
// k + (d-1)k^2 = 7200 scores) lives in LDS.
//
// Selections ("the n best by (score desc, pool index asc)") are done without sorting:
// a bitwise bisection over the order-preserving integer image of the score finds the n-th
// largest score, then one pass in pool-index order takes everything above it and the first
// few equal to it.  For up to 1024 candidates one wave does this from registers with
// ballots only (no barrier inside the 32 steps).
#include "common.hpp"
#include "kernels.hpp"

namespace dt {

#define DT_P_MAX (DT_K_MAX + (DT_D_MAX - 1) * DT_K_MAX * DT_K_MAX)

struct Cut {
    u32 thr;      // key of the n-th best candidate
    int need_eq;  // how many candidates with key == thr are taken (lowest pool indices first)
};

__device__ __forceinline__ u32 score_key(float s) { return ord32(s); }
#define KEY_NEG_INF 0x007FFFFFu

// keep-th largest key among score[0..n), n <= 1024; executed by one full wave.
__device__ __forceinline__ Cut wave_cut(const float *score, int n, int keep) {
    const int lane = lane_id();
    u32 it[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) {
        int i = j * 64 + lane;
        it[j] = i < n ? score_key(score[i]) : 0u;
    }
    u32 t = 0;
    for (int bit = 31; bit >= 0; --bit) {
        const u32 cand = t | (1u << bit);
        int cnt = 0;
#pragma unroll
        for (int j = 0; j < 16; ++j)
            if (j * 64 < n) cnt += __popcll(__ballot(it[j] >= cand));
        if (cnt >= keep) t = cand;
    }
    int gt = 0;
#pragma unroll
    for (int j = 0; j < 16; ++j)
        if (j * 64 < n) gt += __popcll(__ballot(it[j] > t));
    Cut c;
    c.thr = t;
    c.need_eq = keep - gt;
    return c;
}

__device__ __forceinline__ int block_sum_256(int v, int *s_red) {
    const int lane = lane_id(), w = threadIdx.x >> 6;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    __syncthreads();
    if (lane == 0) s_red[w] = v;
    __syncthreads();
    return s_red[0] + s_red[1] + s_red[2] + s_red[3];
}

// Same cut for any n, by the whole workgroup (barriers inside every step).
__device__ __forceinline__ Cut block_cut(const float *score, int n, int keep, int *s_red) {
    u32 t = 0;
    for (int bit = 31; bit >= 0; --bit) {
        const u32 cand = t | (1u << bit);
        int cnt = 0;
        for (int i = threadIdx.x; i < n; i += 256) cnt += score_key(score[i]) >= cand ? 1 : 0;
        if (block_sum_256(cnt, s_red) >= keep) t = cand;
    }
    int gt = 0;
    for (int i = threadIdx.x; i < n; i += 256) gt += score_key(score[i]) > t ? 1 : 0;
    Cut c;
    c.thr = t;
    c.need_eq = keep - block_sum_256(gt, s_red);
    return c;
}

__device__ __forceinline__ int count_viable_wave(const float *score, int n) {
    int cnt = 0;
    for (int base = 0; base < n; base += 64) {
        int i = base + lane_id();
        cnt += __popcll(__ballot(i < n && score[i] > -INFINITY));
    }
    return cnt;
}

// Visit the selected candidates of score[0..n) in ascending index; f(i, position).  One wave.
template <typename F>
__device__ __forceinline__ int wave_enumerate(const float *score, int n, Cut c, F f) {
    int pos = 0, eq_seen = 0;
    for (int base = 0; base < n; base += 64) {
        const int i = base + lane_id();
        const u32 key = i < n ? score_key(score[i]) : 0u;
        const bool eq = i < n && key == c.thr;
        const u64 meq = __ballot(eq);
        const bool take = (i < n && key > c.thr) || (eq && eq_seen + (int)lanes_below(meq) < c.need_eq);
        const u64 m = __ballot(take);
        if (take) f(i, pos + (int)lanes_below(m));
        pos += __popcll(m);
        eq_seen += __popcll(meq);
    }
    return pos;
}

struct Decoded {
    int level, slot, rank, row;
};
__device__ __forceinline__ Decoded decode(int p, int k) {
    Decoded d;
    if (p < k) {
        d.level = 1; d.slot = 0; d.rank = p; d.row = 0;
    } else {
        int q = p - k, kk = k * k;
        int l2 = q / kk, rem = q - l2 * kk;
        d.level = l2 + 2; d.slot = rem / k; d.rank = rem - d.slot * k;
        d.row = 1 + l2 * k + d.slot;
    }
    return d;
}

__global__ __launch_bounds__(256) void tree_kernel(TreeArgs a) {
    const int b = blockIdx.x, tid = threadIdx.x, w = tid >> 6;
    const dt_params prm = a.params[b];
    const int TT = min(max(prm.TT, 1), a.TT_cap), d = min(max(prm.d, 1), DT_D_MAX);
    const int k = min(max(prm.k, 1), min(DT_K_MAX, a.V));
    const int64_t r0 = a.row_off[b];
    const float *tv = a.top_val + r0 * DT_K_MAX;
    const int32_t *ti = a.top_id + r0 * DT_K_MAX;
    const float *lse = a.lse + r0;
    const int64_t o = (int64_t)b * a.TT_cap;

    __shared__ float s_score[DT_P_MAX];
    __shared__ int16_t s_node[DT_P_MAX];
    __shared__ int8_t s_slot[DT_P_MAX];
    __shared__ int s_exp[DT_D_MAX][DT_K_MAX];
    __shared__ int s_nexp;
    __shared__ int s_red[4];
    __shared__ Cut s_cut;

    if (tid == 0) {
        a.tokens[o] = a.root_token[b];
        a.parents[o] = -1;
        a.depth[o] = 0;
        a.score[o] = 0.f;
        a.logp[o] = 0.f;
        a.src_row[o] = 0;
        a.anc_mask[o * DT_MASK_WORDS] = 1ull;
        a.anc_mask[o * DT_MASK_WORDS + 1] = 0ull;
    }
    if (TT == 1) {
        if (tid == 0) a.n_nodes[b] = 1;
        return;
    }
    const int P = k + (d - 1) * k * k;
    for (int p = tid; p < P; p += 256) {
        s_score[p] = -INFINITY;
        s_node[p] = -1;
        s_slot[p] = -1;
    }
    __syncthreads();
    if (tid < k) {
        float v = tv[tid];
        s_score[tid] = v > -INFINITY ? v - lse[0] : -INFINITY;
    }
    __syncthreads();

    // ---- expansion, level by level -----------------------------------------------------------
    for (int l = 1; l < d; ++l) {
        const int lo = l == 1 ? 0 : k + (l - 2) * k * k;
        const int n = l == 1 ? k : k * k;
        if (w == 0) {
            const float *sc = s_score + lo;
            int keep = min(k, count_viable_wave(sc, n));
            int n_exp = 0;
            if (keep > 0) {
                Cut c = wave_cut(sc, n, keep);
                int *exp_l = s_exp[l];
                n_exp = wave_enumerate(sc, n, c, [&](int i, int pos) {
                    exp_l[pos] = lo + i;
                    s_slot[lo + i] = (int8_t)pos;
                });
            }
            if (lane_id() == 0) s_nexp = n_exp;
        }
        __syncthreads();
        const int n_exp = s_nexp;
        if (n_exp == 0) break;
        const int nlo = k + (l - 1) * k * k;
        for (int t = tid; t < n_exp * k; t += 256) {
            int s = t / k, r = t - s * k;
            int row = 1 + (l - 1) * k + s;
            float v = tv[row * DT_K_MAX + r];
            if (v > -INFINITY) s_score[nlo + s * k + r] = s_score[s_exp[l][s]] + (v - lse[row]);
        }
        __syncthreads();
    }

    __syncthreads();  // every wave has read s_nexp before it is reused below

    // ---- rerank: the TT-1 best of the whole pool ----------------------------------------------
    Cut cut;
    int keep;
    if (P <= 1024) {
        if (w == 0) {
            int kp = min(TT - 1, count_viable_wave(s_score, P));
            Cut c;
            c.thr = 0xFFFFFFFFu;
            c.need_eq = 0;
            if (kp > 0) c = wave_cut(s_score, P, kp);
            if (lane_id() == 0) { s_cut = c; s_nexp = kp; }
        }
        __syncthreads();
        cut = s_cut;
        keep = s_nexp;
    } else {
        int v = 0;
        for (int i = tid; i < P; i += 256) v += s_score[i] > -INFINITY ? 1 : 0;
        keep = min(TT - 1, block_sum_256(v, s_red));
        cut.thr = 0xFFFFFFFFu;
        cut.need_eq = 0;
        if (keep > 0) cut = block_cut(s_score, P, keep, s_red);
    }
    if (w == 0 && keep > 0)
        wave_enumerate(s_score, P, cut, [&](int i, int pos) { s_node[i] = (int16_t)(pos + 1); });
    __syncthreads();
    if (tid == 0) a.n_nodes[b] = keep + 1;

    // ---- emission -------------------------------------------------------------------------------
    for (int p = tid; p < P; p += 256) {
        const int n = s_node[p];
        if (n < 0) continue;
        const Decoded dc = decode(p, k);
        const float v = tv[dc.row * DT_K_MAX + dc.rank];
        int par_pool = dc.level == 1 ? -1 : s_exp[dc.level - 1][dc.slot];
        a.tokens[o + n] = ti[dc.row * DT_K_MAX + dc.rank];
        a.parents[o + n] = par_pool < 0 ? 0 : max((int)s_node[par_pool], 0);
        a.depth[o + n] = dc.level;
        a.score[o + n] = s_score[p];
        a.logp[o + n] = v - lse[dc.row];
        a.src_row[o + n] = s_slot[p] >= 0 ? 1 + (dc.level - 1) * k + s_slot[p] : -1;
        u64 m0 = 1ull, m1 = 0ull;  // the root
        int nn = n, pp = par_pool;
        for (int guard = 0; guard <= DT_D_MAX; ++guard) {
            if (nn < 64) m0 |= 1ull << nn; else m1 |= 1ull << (nn - 64);
            if (pp < 0) break;
            nn = max((int)s_node[pp], 0);
            const Decoded dp = decode(pp, k);
            pp = dp.level == 1 ? -1 : s_exp[dp.level - 1][dp.slot];
        }
        a.anc_mask[(o + n) * DT_MASK_WORDS] = m0;
        a.anc_mask[(o + n) * DT_MASK_WORDS + 1] = m1;
    }
}

hipError_t tree_launch(const TreeArgs &a, hipStream_t st) {
    if (a.batch <= 0) return hipSuccess;
    ProfScope prof(KID_TREE, st);
    hipLaunchKernelGGL(tree_kernel, dim3(a.batch), dim3(256), 0, st, a);
    return hipGetLastError();
}

}  // namespace dt
