// Action selection on the device: the policy MLP on the concatenated hidden-state vector, the
// action cache of Algorithm 1, and the (TT, d, k) of the chosen action written straight into the
// device array that dt_build_tree / dt_expand_level read -- no host round trip between the policy
// and the step.
//
// Layer 1 is a [batch, F] x [F, H] product with F ~ 12k: the weight matrix (6 MB in fp32) is the only
// real traffic.  It is cut along F into slices of POLICY_KS inputs, one workgroup per slice, thread
// (o, part) accumulating output o over half of the slice for up to eight sequences at a time (the
// inputs sit in LDS and are read as broadcasts; the [in][out] weight layout makes every wave read
// contiguous rows).  The partial sums are added up in slice order by the second kernel (one
// workgroup per sequence), which also runs the two small layers, picks the action and keeps the cache.
// Sequences whose cached action is still valid cost nothing but the cache update.
#include "common.hpp"
#include "kernels.hpp"

namespace dt {

#define POLICY_BCH 8

__device__ __forceinline__ bool policy_needed(const PolicyArgs &a, int b) {
    return a.cache_step[b] == 0 || a.cached_action[b] < 0;
}

__global__ __launch_bounds__(256) void policy_layer1_kernel(PolicyArgs a) {
    const int H = a.H, tid = threadIdx.x;
    const int o = tid % H, part = tid / H;  // blockDim.x = 2 H
    const int k0 = blockIdx.x * POLICY_KS;
    const int half = POLICY_KS / 2;
    __shared__ float s_x[POLICY_BCH][POLICY_KS];
    __shared__ float s_acc[POLICY_BCH][128];
    __shared__ int s_need[POLICY_BCH];
    // This thread's weights do not depend on the batch: asked for first, so that the one trip to memory
    // they cost overlaps the cache flags and the inputs (rows past F: the last row again, zeroed at use).
    float wreg[POLICY_KS / 2];
#pragma unroll
    for (int i = 0; i < POLICY_KS / 2; ++i) wreg[i] = a.W1[(int64_t)min(k0 + part * half + i, a.F - 1) * H + o];
    for (int b0 = 0; b0 < a.batch; b0 += POLICY_BCH) {
        const int nb = min(POLICY_BCH, a.batch - b0);
        // the inputs are read before the flags that say which sequences need them are back
        float xv[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = tid + u * (int)blockDim.x;
            xv[u] = 0.f;
            if (i < nb * POLICY_KS) {
                const int64_t idx = (int64_t)(b0 + i / POLICY_KS) * a.feat_stride + min(k0 + i % POLICY_KS, a.F - 1);
                xv[u] = a.feat_dtype == DT_BF16 ? bf16_bits_to_float(((const uint16_t *)a.feat)[idx])
                                                : ((const float *)a.feat)[idx];
            }
        }
        if (tid < POLICY_BCH) s_need[tid] = tid < nb && policy_needed(a, b0 + tid);
        __syncthreads();
        bool any = false;
        for (int j = 0; j < nb; ++j) any = any || s_need[j];
        if (any) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = tid + u * (int)blockDim.x;
                if (i < nb * POLICY_KS) {
                    const int j = i / POLICY_KS, kk = i % POLICY_KS;
                    s_x[j][kk] = (s_need[j] && k0 + kk < a.F) ? xv[u] : 0.f;
                }
            }
            __syncthreads();
            float acc[POLICY_BCH];
#pragma unroll
            for (int j = 0; j < POLICY_BCH; ++j) acc[j] = 0.f;
#pragma unroll
            for (int i = 0; i < POLICY_KS / 2; ++i) {
                const int kk = part * half + i;
                const float w = k0 + kk < a.F ? wreg[i] : 0.f;
#pragma unroll
                for (int j = 0; j < POLICY_BCH; ++j) acc[j] = fmaf(w, s_x[j][kk], acc[j]);
            }
            if (part == 1)
#pragma unroll
                for (int j = 0; j < POLICY_BCH; ++j) s_acc[j][o] = acc[j];
            __syncthreads();
            if (part == 0)
                for (int j = 0; j < nb; ++j)
                    if (s_need[j]) a.partial[((int64_t)blockIdx.x * a.batch + b0 + j) * H + o] = acc[j] + s_acc[j][o];
        }
        __syncthreads();
    }
}

// s + sum_i x[i] * w[i * stride], i = 0 .. n-1 in order, n a multiple of 64: the sixty-four weights of a
// batch are requested together, so a layer of 128 inputs costs two trips to memory and not one per few terms.
__device__ __forceinline__ float dot_strided(float s, const float *x, const float *w, int n, int stride) {
    for (int i0 = 0; i0 < n; i0 += 64) {
        float wv[64];
#pragma unroll
        for (int i = 0; i < 64; ++i) wv[i] = w[(int64_t)(i0 + i) * stride];
#pragma unroll
        for (int i = 0; i < 64; ++i) s = fmaf(x[i0 + i], wv[i], s);
    }
    return s;
}

__global__ __launch_bounds__(256) void policy_head_kernel(PolicyArgs a) {
    const int b = blockIdx.x, tid = threadIdx.x, lane = lane_id(), w = tid >> 6;
    const int H = a.H, A = a.A;
    __shared__ float s_h1[128], s_h2[128];
    __shared__ float s_run[4][128];
    __shared__ u64 s_key[4];
    __shared__ double s_wtot[4];
    __shared__ int s_act;
    const bool need = policy_needed(a, b);
    if (need) {
        {
            // the slices' partial sums, in a fixed order: 256 / H threads per output take consecutive runs
            // of slices (thirty-two requests in flight each), the runs are added up in order
            const int o = tid % H, r = tid / H, R = 256 / H;
            const int per = (a.S + R - 1) / R, s0 = r * per, s1 = min(a.S, s0 + per);
            float s = 0.f;
            for (int sl = s0; sl < s1; sl += 32) {
                float v[32];
#pragma unroll
                for (int i = 0; i < 32; ++i)
                    v[i] = a.partial[((int64_t)min(sl + i, s1 - 1) * a.batch + b) * H + o];
#pragma unroll
                for (int i = 0; i < 32; ++i) s += sl + i < s1 ? v[i] : 0.f;
            }
            s_run[r][o] = s;
        }
        __syncthreads();
        if (tid < H) {
            float s = a.b1[tid];
            for (int r = 0; r < 256 / H; ++r) s += s_run[r][tid];
            s_h1[tid] = tanhf(s);
        }
        __syncthreads();
        if (tid < H) s_h2[tid] = tanhf(dot_strided(a.b2[tid], s_h1, a.W2 + tid, H, H));
        __syncthreads();
        float logit = -INFINITY;
        if (tid < A) {
            const float s = dot_strided(a.b3[tid], s_h2, a.W3 + tid, H, A);
            logit = s;
            if (a.logits_out) a.logits_out[(int64_t)b * A + tid] = s;
        }
        // largest logit, ties -> lowest action
        u64 key = tid < A ? make_key(logit, (u32)tid) : 0ull;
        key = wave_max_u64(key);
        if (lane == 0) s_key[w] = key;
        __syncthreads();
        u64 k01 = s_key[0] > s_key[1] ? s_key[0] : s_key[1], k23 = s_key[2] > s_key[3] ? s_key[2] : s_key[3];
        const u64 best = k01 > k23 ? k01 : k23;
        if (a.mode == 0) {
            if (tid == 0) s_act = (int)key_idx(best);
        } else {
            // a sample of softmax(logits): inverse CDF in double at the Philox uniform of this decision
            const double p = tid < A ? exp((double)logit - (double)key_val(best)) : 0.0;
            double incl = p;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const double t = __shfl_up(incl, off, 64);
                if (lane >= off) incl += t;
            }
            if (lane == 63) s_wtot[w] = incl;
            if (tid == 0) s_act = A - 1;
            __syncthreads();
            double before = 0.0;
            for (int q = 0; q < w; ++q) before += s_wtot[q];
            const double Z = s_wtot[0] + s_wtot[1] + s_wtot[2] + s_wtot[3];
            const double target = (double)philox_uniform(a.seed, a.step, (u32)b, 0xFFFFFFFEu) * Z;
            const bool cross = tid < A && before + incl > target;
            const u64 m = __ballot(cross);
            if (before <= target && m && lane == (int)__builtin_ctzll(m)) s_act = tid;  // first crossing wave only
        }
        __syncthreads();
    }
    if (tid == 0) {
        int cs = a.cache_step[b], act;
        if (need) {
            act = s_act;
            a.cached_action[b] = act;
            cs = 1;
        } else {
            act = a.cached_action[b];
            cs += 1;
        }
        if (cs >= a.N) cs = 0;
        a.cache_step[b] = cs;
        act = min(max(act, 0), A - 1);
        a.params_out[b] = a.table[act];
        if (a.action_out) a.action_out[b] = act;
        if (a.queried_out) a.queried_out[b] = need ? 1 : 0;
    }
}

// Reward of the step that has just been verified and, at the end of a cache interval, its average over
// the interval.  One thread per sequence; float arithmetic (an interval has at most a few dozen terms).
__global__ __launch_bounds__(256) void reward_kernel(RewardArgs a) {
    const int b = blockIdx.x * 256 + threadIdx.x;
    if (b >= a.batch) return;
    const float secs = a.elapsed_dev ? a.elapsed_dev[b] : a.elapsed;
    const float tokens = (float)(max(a.accept_len[b], 0) + a.count_bonus);
    const float sum = a.reward_sum[b] + tokens / secs;
    const int steps = a.reward_steps[b] + 1;
    if (a.cache_step[b] == 0) {  // the action cache has closed its interval with this step
        a.reward_avg[b] = sum / (float)steps;
        a.interval_done[b] = 1;
        a.reward_sum[b] = 0.f;
        a.reward_steps[b] = 0;
    } else {
        a.interval_done[b] = 0;
        a.reward_sum[b] = sum;
        a.reward_steps[b] = steps;
    }
}

hipError_t reward_launch(const RewardArgs &a, hipStream_t st) {
    if (a.batch <= 0) return hipSuccess;
    launch_kernel(KID_REWARD, st, reward_kernel, dim3((a.batch + 255) / 256), dim3(256), 0, a);
    return hipGetLastError();
}

hipError_t policy_launch(const PolicyArgs &a, hipStream_t st) {
    if (a.batch <= 0) return hipSuccess;
    launch_kernel(KID_POLICY_L1, st, policy_layer1_kernel, dim3(a.S), dim3(2 * a.H), 0, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    launch_kernel(KID_POLICY_HEAD, st, policy_head_kernel, dim3(a.batch), dim3(256), 0, a);
    return hipGetLastError();
}

}  // namespace dt
