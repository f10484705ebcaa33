// Acceptance kernel: per-node accept decision (greedy arg max match, or stochastic
// min(1, P_T/P_d) against a Philox uniform), then the longest accepted root path via the
// ancestor bitsets, and the bonus token.  One workgroup per sequence.  The vocabulary
// rows themselves were reduced by the row kernels; this kernel merges their per-chunk
// partials (arg max key, and (max, sum) of row/T for the stochastic mode).
#include "common.hpp"
#include "kernels.hpp"

namespace dt {

__device__ __forceinline__ float load_logit(const void *base, int dtype, int64_t idx) {
    return dtype == DT_BF16 ? bf16_bits_to_float(((const uint16_t *)base)[idx]) : ((const float *)base)[idx];
}

// The up to 32 consecutive entries id0 .. id0 + epl - 1 of a row that a thread owns (epl a multiple of 8; entries
// at or past `hi`, and octets past epl, read as -inf), as four octets.  Every load is unconditional, so that all
// of a thread's loads are in flight together (a load inside a branch is waited for inside that branch): an
// aligned bf16 octet that lies wholly inside the range is one 16-byte load, any other octet asks for the row's
// first entries instead and is patched with element loads afterwards (at most one octet of a chunk straddles the
// end of the row).  vec_ok: the row is 16-byte aligned and holds at least 8 entries.
__device__ __forceinline__ void load_logits32(const void *row, int dtype, int id0, int epl, int hi, bool vec_ok,
                                              float x[4][8]) {
    if (dtype == DT_BF16 && vec_ok) {  // uniform
        uint4 raw[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int id = id0 + 8 * j;
            const bool full = 8 * j < epl && id + 8 <= hi;
            raw[j] = *(const uint4 *)((const uint16_t *)row + (full ? id : 0));
        }
        __builtin_amdgcn_sched_barrier(0);  // every request is out before the first conversion
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const u32 wds[4] = {raw[j].x, raw[j].y, raw[j].z, raw[j].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                x[j][2 * e] = __uint_as_float(wds[e] << 16);
                x[j][2 * e + 1] = __uint_as_float(wds[e] & 0xFFFF0000u);
            }
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int id = id0 + 8 * j;
            if (!(8 * j < epl && id + 8 <= hi)) {
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    x[j][e] = 8 * j < epl && id + e < hi ? load_logit(row, dtype, id + e) : -INFINITY;
            }
        }
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int id = id0 + 8 * j + e;
                x[j][e] = load_logit(row, dtype, 8 * j < epl && id < hi ? id : 0);
            }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int id = id0 + 8 * j + e;
                x[j][e] = 8 * j < epl && id < hi ? x[j][e] : -INFINITY;
            }
    }
}

// Inverse-CDF sample of softmax(row g / T) at the uniform u, by the whole workgroup (256 threads; contains
// barriers).  The row kernel left (max, sum exp((x - max)/T)) of every chunk of the row: their masses
// relative to the row maximum Mrow, accumulated in double, locate the chunk that holds the crossing; only
// that chunk is read again (thread t owns `epl` <= 32 consecutive ids), element masses in fp32, running sums in
// double.  The comparison is "cumulative mass > u * total", the un-normalised form of the cdf > u test;
// it differs from an all-double evaluation by ~1e-6 in probability.  The result is left in *s_out.
__device__ __forceinline__ void sample_row_block(const AcceptArgs &a, int64_t g, float Mrow, float u, float inv_t,
                                                 double *s_wtot, int *s_out) {
    const int tid = threadIdx.x, lane = lane_id(), w = tid >> 6, S = a.S;
    const void *row = (const char *)a.target + g * a.row_stride * (a.dtype == DT_BF16 ? 2 : 4);
    const float cexp = 1.4426950408889634f * inv_t;
    // chunk c in lane c (S <= 64), every wave for itself
    double mass = 0.0;
    if (lane < S) {
        const float2 p = a.part_ms[g * S + lane];
        if (p.y > 0.f) mass = (double)p.y * (double)__builtin_amdgcn_exp2f((p.x - Mrow) * cexp);
    }
    double cum = mass;  // inclusive scan over the chunks
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const double t = __shfl_up(cum, off, 64);
        if (lane >= off) cum += t;
    }
    const double Z = __shfl(cum, 63, 64);
    const double target_mass = (double)u * Z;
    // first chunk whose cumulative mass passes the target; if rounding leaves none, the last with mass
    const u64 passed = __ballot(cum > target_mass), massy = __ballot(mass > 0.0);
    const int cstar = passed ? (int)__builtin_ctzll(passed) : massy ? 63 - (int)__builtin_clzll(massy) : 0;
    const double before = __shfl(cum - mass, cstar, 64);
    const int epl = a.chunk_elems / 256;
    const int lo = cstar * a.chunk_elems, hi = min(a.V, lo + a.chunk_elems);
    const int id0 = lo + tid * epl;
    const bool vec_ok = ((uintptr_t)row & 15) == 0 && a.V >= 8;  // id0 is a multiple of 8
    // a thread owns at most 32 entries (four octets): all asked for at once and kept, the thread that
    // holds the crossing walks its registers and nothing is read twice
    float x[4][8];
    load_logits32(row, a.dtype, id0, epl, hi, vec_ok, x);
    double mine = 0.0;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int e = 0; e < 8; ++e) mine += (double)__builtin_amdgcn_exp2f((x[j][e] - Mrow) * cexp);  // past epl: + 0
    double incl = mine;  // inclusive scan over the lanes of the wave
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const double t = __shfl_up(incl, off, 64);
        if (lane >= off) incl += t;
    }
    __syncthreads();  // s_wtot / *s_out may still be read from an earlier use
    if (lane == 63) s_wtot[w] = incl;
    if (tid == 0) *s_out = -1;
    __syncthreads();
    double run = before;
    for (int q = 0; q < w; ++q) run += s_wtot[q];
    const bool cross = run + incl > target_mass;
    const u64 m = __ballot(cross);
    // the first crossing thread of the first crossing wave
    bool earlier = false;
    {
        double r2 = before;
        for (int q = 0; q < w; ++q) {
            r2 += s_wtot[q];
            earlier = earlier || r2 > target_mass;
        }
    }
    if (!earlier && m && lane == (int)__builtin_ctzll(m)) {
        double cm = run + incl - mine;
        int id = min(id0 + epl, hi) - 1;
        bool done = false;
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                cm += (double)__builtin_amdgcn_exp2f((x[j][e] - Mrow) * cexp);
                if (!done && cm > target_mass) { id = id0 + 8 * j + e; done = true; }
            }
        *s_out = id;
    }
    __syncthreads();
    if (tid == 0 && *s_out < 0) {
        // the chunk's re-computed mass falls just short of the crossing (rounding), or the row
        // carries no mass at all: last token of the chunk that carries mass, else token 0
        int id = hi - 1;
        while (id > lo && !(__builtin_amdgcn_exp2f((load_logit(row, a.dtype, id) - Mrow) * cexp) > 0.f)) --id;
        *s_out = Z > 0.0 ? id : 0;
    }
    __syncthreads();
}

// Target-sampled verification: node i of sequence b draws the target's own next token from
// softmax(row i / T) at the uniform of its depth.  One workgroup per (sequence, node).
__global__ __launch_bounds__(256) void node_sample_kernel(AcceptArgs a) {
    const int b = blockIdx.x / a.TT_cap, i = blockIdx.x % a.TT_cap, lane = lane_id();
    const int N = min(max(a.n_nodes[b], 1), a.TT_cap);
    if (i >= N) return;
    const int64_t g = (int64_t)b * a.TT_cap + i;
    __shared__ double s_wtot[4];
    __shared__ int s_out;
    // the row maximum: the largest of the chunks' best keys
    u64 key = lane < a.S ? a.part_keys[g * a.S + lane] : 0ull;
    key = wave_max_u64(key);
    const int dep = min(max(a.depth[g], 0), DT_D_MAX);
    const float u = philox_uniform(a.seed, a.step, (u32)b, 0x80000000u + (u32)dep);
    sample_row_block(a, g, key_val(key), u, 1.0f / a.temperature, s_wtot, &s_out);
    if (threadIdx.x == 0) a.samples[g] = s_out;
}

__global__ __launch_bounds__(256) void accept_kernel(AcceptArgs a) {
    const int b = blockIdx.x, tid = threadIdx.x, lane = lane_id(), w = tid >> 6;
    const int N = min(max(a.n_nodes[b], 1), a.TT_cap);
    const int64_t o = (int64_t)b * a.TT_cap;
    const bool stochastic = a.mode == DT_ACCEPT_STOCHASTIC;
    const bool sampled = a.mode == DT_ACCEPT_SAMPLED;  // node_sample_kernel has drawn every node's token
    const float inv_t = stochastic ? 1.0f / a.temperature : 1.0f;
    const int S = a.S;

    __shared__ int s_amax[DT_TT_MAX];
    __shared__ float s_rowmax[DT_TT_MAX];
    __shared__ float s_lse[DT_TT_MAX];
    __shared__ u64 s_acc[2];
    __shared__ int s_best[4];
    __shared__ double s_wtot[4];
    __shared__ int s_bonus;

    // ---- everything a node needs later is requested now, so the loads overlap the merge -------
    int my_tok = 0, my_par = 0, my_dep = 0;
    u64 my_m0 = 0ull, my_m1 = 0ull;
    float my_logp = 0.f;
    if (tid < N) {
        my_tok = a.tokens[o + tid];
        my_par = a.parents[o + tid];
        my_dep = a.depth[o + tid];
        my_m0 = a.anc_mask[(o + tid) * DT_MASK_WORDS];
        my_m1 = a.anc_mask[(o + tid) * DT_MASK_WORDS + 1];
        if (stochastic) my_logp = a.logp[o + tid];
    }

    // ---- merge the row partials: four adjacent lanes share a row, each takes every fourth chunk --
    {
        const float cexp = 1.4426950408889634f * inv_t;
        const int part = tid & 3;
        for (int i0 = 0; i0 < N; i0 += 64) {
            const int i = i0 + (tid >> 2);
            const int64_t g = o + min(i, N - 1);
            u64 best = 0ull;
            float M = -INFINITY, Ssum = 0.f;
            for (int c0 = part; c0 < S; c0 += 16) {  // four chunks per trip to memory
                u64 key[4];
                float2 p[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int c = min(c0 + 4 * u, S - 1);  // past the end: the last chunk again, ignored below
                    key[u] = a.part_keys[g * S + c];
                    if (stochastic) p[u] = a.part_ms[g * S + c];
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    if (c0 + 4 * u >= S) continue;
                    best = key[u] > best ? key[u] : best;
                    if (stochastic) {
                        const float M2 = fmaxf(M, p[u].x);
                        if (M2 != -INFINITY)
                            Ssum = Ssum * __builtin_amdgcn_exp2f((M - M2) * cexp) +
                                   p[u].y * __builtin_amdgcn_exp2f((p[u].x - M2) * cexp);
                        M = M2;
                    }
                }
            }
#pragma unroll
            for (int off = 1; off <= 2; off <<= 1) {  // the four lanes of the row
                const u64 ob = shfl_xor_u64(best, off);
                best = ob > best ? ob : best;
                if (stochastic) {
                    const float M2 = __shfl_xor(M, off, 64), S2 = __shfl_xor(Ssum, off, 64);
                    const float Mn = fmaxf(M, M2);
                    if (Mn != -INFINITY)
                        Ssum = Ssum * __builtin_amdgcn_exp2f((M - Mn) * cexp) + S2 * __builtin_amdgcn_exp2f((M2 - Mn) * cexp);
                    M = Mn;
                }
            }
            if (part == 0 && i < N) {
                const int choice = sampled ? a.samples[o + i] : (int)key_idx(best);
                s_amax[i] = choice;
                s_rowmax[i] = key_val(best);
                s_lse[i] = stochastic ? M * inv_t + __logf(Ssum) : 0.f;
                if (a.node_argmax) a.node_argmax[o + i] = choice;
            }
        }
    }
    __syncthreads();

    // ---- per-node accept bit ----------------------------------------------------------------
    if (tid < DT_TT_MAX) {  // waves 0 and 1: wave w owns bits [64w, 64w+64)
        bool acc = false;
        if (tid < N) {
            if (tid == 0) {
                acc = true;
            } else {
                const int p = min(max(my_par, 0), N - 1);
                if (!stochastic) {
                    acc = my_tok == s_amax[p];
                } else if (my_tok >= 0 && my_tok < a.V) {
                    const float x = load_logit(a.target, a.dtype, (o + p) * a.row_stride + my_tok);
                    const float lpT = x * inv_t - s_lse[p];
                    const float alpha = fminf(1.0f, __expf(lpT - my_logp));
                    const float u = philox_uniform(a.seed, a.step, (u32)b, (u32)tid);
                    acc = u < alpha;
                }
            }
        }
        const u64 m = __ballot(acc);
        if (lane == 0) s_acc[w] = m;
    }
    __syncthreads();

    // ---- deepest node whose ancestors are all accepted; ties -> lowest index -------------
    if (tid < DT_TT_MAX) {
        int key = -1;
        if (tid < N) {
            const bool ok = ((my_m0 & ~s_acc[0]) | (my_m1 & ~s_acc[1])) == 0ull;
            if (ok) key = (my_dep << 8) | (255 - tid);
        }
        key = wave_max_i32(key);
        if (lane == 0) s_best[w] = key;
    }
    __syncthreads();
    const int bkey = max(s_best[0], s_best[1]);
    const int best = 255 - (bkey & 255);
    const int len = bkey >> 8;

    // ---- the accepted path: exactly the nodes in the ancestor set of `best`, which its owner
    //      thread publishes (the accept bits in s_acc are no longer needed) -----------------------
    if (tid == best) { s_acc[0] = my_m0; s_acc[1] = my_m1; }
    if (tid <= DT_D_MAX && tid > len) {  // unused slots; slot len of out_tokens is the bonus token
        a.path_nodes[(int64_t)b * (DT_D_MAX + 1) + tid] = -1;
        a.out_tokens[(int64_t)b * (DT_D_MAX + 1) + tid] = -1;
    }
    __syncthreads();
    if (tid < N) {
        const bool on_path = ((tid < 64 ? s_acc[0] : s_acc[1]) >> (tid & 63)) & 1ull;
        if (on_path && my_dep <= DT_D_MAX) {
            a.path_nodes[(int64_t)b * (DT_D_MAX + 1) + my_dep] = tid;
            if (tid > 0) a.out_tokens[(int64_t)b * (DT_D_MAX + 1) + my_dep - 1] = my_tok;
        }
    }
    if (tid == 0) { a.accept_len[b] = len; a.best_node[b] = best; }

    // ---- bonus token --------------------------------------------------------------------------
    if (!stochastic) {
        if (tid == 0) s_bonus = s_amax[best];
    } else {
        // inverse CDF of softmax(row best / T) at the bonus uniform
        sample_row_block(a, o + best, s_rowmax[best], philox_uniform(a.seed, a.step, (u32)b, 0xFFFFFFFFu), inv_t,
                         s_wtot, &s_bonus);
    }
    __syncthreads();

    if (tid == 0 && len <= DT_D_MAX) a.out_tokens[(int64_t)b * (DT_D_MAX + 1) + len] = s_bonus;
}

hipError_t accept_launch(const AcceptArgs &a, hipStream_t st) {
    if (a.batch <= 0) return hipSuccess;
    if (a.mode == DT_ACCEPT_SAMPLED) {
        launch_kernel(KID_NODE_SAMPLE, st, node_sample_kernel, dim3(a.batch * a.TT_cap), dim3(256), 0, a);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    launch_kernel(KID_ACCEPT, st, accept_kernel, dim3(a.batch), dim3(256), 0, a);
    return hipGetLastError();
}

}  // namespace dt
