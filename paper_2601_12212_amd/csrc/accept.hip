// Acceptance kernel: per-node accept decision (greedy arg max match, or stochastic
// min(1, P_T/P_d) against a Philox uniform), then the longest accepted root path via the
// ancestor bitsets, and the bonus token.  One workgroup per sequence.  The vocabulary
// rows themselves were reduced by the row kernels; this kernel merges their per-chunk
// partials (arg max key, and (max, sum) of row/T for the stochastic mode).
#include "common.hpp"
#include "kernels.hpp"

namespace dt {

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

__device__ __forceinline__ float load_logit(const void *base, int dtype, int64_t idx) {
    return dtype == DT_BF16 ? bf16_bits_to_float(((const uint16_t *)base)[idx]) : ((const float *)base)[idx];
}

__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

__global__ __launch_bounds__(256) void accept_kernel(AcceptArgs a) {
    const int b = blockIdx.x, tid = threadIdx.x, lane = lane_id(), w = tid >> 6;
    const int N = min(max(a.n_nodes[b], 1), a.TT_cap);
    const int64_t o = (int64_t)b * a.TT_cap;
    const bool stochastic = a.mode == DT_ACCEPT_STOCHASTIC;
    const float inv_t = stochastic ? 1.0f / a.temperature : 1.0f;

    __shared__ int s_amax[DT_TT_MAX];
    __shared__ float s_rowmax[DT_TT_MAX];
    __shared__ float s_lse[DT_TT_MAX];
    __shared__ u64 s_acc[2];
    __shared__ int s_best[4];
    __shared__ double s_wtot[4];
    __shared__ int s_bonus;

    // ---- merge the row partials: wave w takes rows w, w+4, ...; lane c holds chunk c (S <= 64) --
    {
        const float cexp = 1.4426950408889634f * inv_t;
#pragma unroll 4
        for (int i = w; i < N; i += 4) {
            const int64_t g = o + i;
            const u64 key = lane < a.S ? a.part_keys[g * a.S + lane] : 0ull;
            const u64 best = wave_max_u64(key);
            float lse_i = 0.f;
            if (stochastic) {
                float2 p = lane < a.S ? a.part_ms[g * a.S + lane] : make_float2(-INFINITY, 0.f);
                const float M = wave_max(p.x);
                const float Mu = M == -INFINITY ? 0.f : M;
                const float term = p.y > 0.f ? p.y * __builtin_amdgcn_exp2f((p.x - Mu) * cexp) : 0.f;
                lse_i = M * inv_t + __logf(wave_sum(term));
            }
            if (lane == 0) {
                s_amax[i] = (int)key_idx(best);
                s_rowmax[i] = key_val(best);
                s_lse[i] = lse_i;
                if (a.node_argmax) a.node_argmax[g] = (int)key_idx(best);
            }
        }
    }
    if (tid < 2) s_acc[tid] = 0ull;
    __syncthreads();

    // ---- per-node accept bit ----------------------------------------------------------------
    if (tid < DT_TT_MAX) {  // waves 0 and 1: wave w owns bits [64w, 64w+64)
        bool acc = false;
        if (tid < N) {
            if (tid == 0) {
                acc = true;
            } else {
                const int p = min(max(a.parents[o + tid], 0), N - 1);
                const int tok = a.tokens[o + tid];
                if (!stochastic) {
                    acc = tok == s_amax[p];
                } else if (tok >= 0 && tok < a.V) {
                    const float x = load_logit(a.target, a.dtype, (o + p) * a.row_stride + tok);
                    const float lpT = x * inv_t - s_lse[p];
                    const float alpha = fminf(1.0f, __expf(lpT - a.logp[o + tid]));
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
            const u64 m0 = a.anc_mask[(o + tid) * DT_MASK_WORDS], m1 = a.anc_mask[(o + tid) * DT_MASK_WORDS + 1];
            const bool ok = ((m0 & ~s_acc[0]) | (m1 & ~s_acc[1])) == 0ull;
            if (ok) key = (a.depth[o + tid] << 8) | (255 - tid);
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) key = max(key, __shfl_xor(key, off, 64));
        if (lane == 0) s_best[w] = key;
    }
    __syncthreads();
    const int bkey = max(s_best[0], s_best[1]);
    const int best = 255 - (bkey & 255);
    const int len = bkey >> 8;

    // ---- bonus token --------------------------------------------------------------------------
    if (!stochastic) {
        if (tid == 0) s_bonus = s_amax[best];
    } else {
        // inverse CDF of softmax(row/T) at the bonus uniform, in double.  Wave w owns the
        // contiguous span [w*span, (w+1)*span) of the row, walked in steps of 64 lanes x 8.
        const void *row = (const char *)a.target + (o + best) * a.row_stride * (a.dtype == DT_BF16 ? 2 : 4);
        const double T = (double)a.temperature;
        const double mT = (double)s_rowmax[best] / T;
        const int span = ((a.V + 2047) / 2048) * 512;
        const int lo = w * span, hi = min(a.V, lo + span);
        double tot = 0.0;
        for (int base = lo + lane * 8; base < hi; base += 512)
            for (int e = 0; e < 8; ++e)
                if (base + e < hi) tot += exp((double)load_logit(row, a.dtype, base + e) / T - mT);
        tot = wave_sum_f64(tot);
        if (lane == 0) s_wtot[w] = tot;
        if (tid == 0) s_bonus = -1;
        __syncthreads();
        const double Z = s_wtot[0] + s_wtot[1] + s_wtot[2] + s_wtot[3];
        const double target_mass = (double)philox_uniform(a.seed, a.step, (u32)b, 0xFFFFFFFFu) * Z;
        double before = 0.0;
        for (int q = 0; q < w; ++q) before += s_wtot[q];
        // the wave whose span contains the crossing walks it again
        if (before <= target_mass && (target_mass < before + s_wtot[w])) {
            double run = before;
            for (int sb = lo; sb < hi; sb += 512) {
                const int base = sb + lane * 8;
                double p[8], mine = 0.0;
                for (int e = 0; e < 8; ++e) {
                    p[e] = base + e < hi ? exp((double)load_logit(row, a.dtype, base + e) / T - mT) : 0.0;
                    mine += p[e];
                }
                double incl = mine;  // inclusive scan over lanes
#pragma unroll
                for (int off = 1; off < 64; off <<= 1) {
                    double t = __shfl_up(incl, off, 64);
                    if (lane >= off) incl += t;
                }
                const double step_total = __shfl(incl, 63, 64);
                if (run + step_total > target_mass) {
                    const u64 m = __ballot(run + incl > target_mass);
                    const int first = __ffsll((long long)m) - 1;
                    if (lane == first) {
                        double c = run + incl - mine;
                        int id = base + 7;
                        for (int e = 0; e < 8; ++e) {
                            c += p[e];
                            if (c > target_mass) { id = base + e; break; }
                        }
                        s_bonus = min(id, a.V - 1);
                    }
                    break;
                }
                run += step_total;
            }
        }
        __syncthreads();
        if (tid == 0 && s_bonus < 0) {
            // the uniform lies above the rounded total mass: last token that carries mass
            int id = a.V - 1;
            while (id > 0 && !(exp((double)load_logit(row, a.dtype, id) / T - mT) > 0.0)) --id;
            s_bonus = id;
        }
    }
    __syncthreads();

    // ---- walk and outputs ---------------------------------------------------------------------
    if (tid == 0) {
        a.accept_len[b] = len;
        a.best_node[b] = best;
        int32_t *path = a.path_nodes + (int64_t)b * (DT_D_MAX + 1);
        int32_t *outt = a.out_tokens + (int64_t)b * (DT_D_MAX + 1);
        for (int s = 0; s <= DT_D_MAX; ++s) { path[s] = -1; outt[s] = -1; }
        int i = best;
        for (int guard = 0; guard <= DT_D_MAX && i >= 0; ++guard) {
            const int dpt = min(max(a.depth[o + i], 0), DT_D_MAX);
            path[dpt] = i;
            if (i > 0) outt[dpt - 1] = a.tokens[o + i];
            i = i > 0 ? a.parents[o + i] : -1;
        }
        if (len <= DT_D_MAX) outt[len] = s_bonus;
    }
}

hipError_t accept_launch(const AcceptArgs &a, hipStream_t st) {
    if (a.batch <= 0) return hipSuccess;
    ProfScope prof(KID_ACCEPT, st);
    hipLaunchKernelGGL(accept_kernel, dim3(a.batch), dim3(256), 0, st, a);
    return hipGetLastError();
}

}  // namespace dt
