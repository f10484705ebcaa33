// Row kernels: top-k and log-sum-exp over vocabulary rows (draft rows: k best + lse;
// target rows: arg max, and lse of row/T for stochastic acceptance).
//
// A row is cut into chunks of 256*8*NL elements; one workgroup reduces one chunk held
// entirely in registers (one coalesced 16-byte load per lane per 8 bf16 elements), and a
// second small kernel merges the per-chunk partials of a row.  Selection is exact under
// the total order (value desc, id asc): the k-th largest lane maximum bounds the k-th
// largest element from below, elements at or above that bound are ranked by their 64-bit
// (value, id) keys; a slow exact path covers rows with so many ties that the candidate
// list overflows.
#include "common.hpp"
#include "kernels.hpp"

namespace dt {

// ---------------------------------------------------------------- row -> (valid, k) ----
struct RowMeta {
    bool valid;
    int k;
};

__device__ __forceinline__ RowMeta row_meta(const RowArgs &a, int64_t g) {
    RowMeta m;
    m.valid = true;
    m.k = a.k_uniform;
    if (a.mode == ROWS_DRAFT) {
        // sequence b with row_off[b] <= g < row_off[b+1]
        int lo = 0, hi = a.batch;
        while (hi - lo > 1) {
            int mid = (lo + hi) >> 1;
            if (a.row_off[mid] <= g) lo = mid; else hi = mid;
        }
        int r = (int)(g - a.row_off[lo]);
        dt_params p = a.params[lo];
        int TT = min(max(p.TT, 1), a.TT_cap), d = min(max(p.d, 1), DT_D_MAX);
        int k = min(max(p.k, 1), min(DT_K_MAX, a.V));
        m.k = k;
        m.valid = (TT > 1) && (r < 1 + (d - 1) * k) && (g < a.row_off[lo + 1]);
    } else if (a.mode == ROWS_TARGET) {
        int b = (int)(g / a.TT_cap), i = (int)(g % a.TT_cap);
        m.k = 1;
        m.valid = i < a.n_nodes[b];
    }
    return m;
}

// ---------------------------------------------- rank a short LDS list, keep the k best --
// list[0..n) distinct keys, n <= 64*IPL.  The key of rank r < k is handed to emit(r, key).
template <int IPL, typename Emit>
__device__ __forceinline__ void rank_emit(const u64 *list, int n, int k, Emit emit) {
    const int lane = lane_id();
    u64 mine[IPL];
    int rank[IPL];
#pragma unroll
    for (int q = 0; q < IPL; ++q) {
        int i = lane + 64 * q;
        mine[q] = i < n ? list[i] : 0ull;
        rank[q] = 0;
    }
    for (int i = 0; i < n; ++i) {
        u64 o = list[i];  // same address in every lane: LDS broadcast
#pragma unroll
        for (int q = 0; q < IPL; ++q) rank[q] += (o > mine[q]) ? 1 : 0;
    }
#pragma unroll
    for (int q = 0; q < IPL; ++q)
        if (lane + 64 * q < n && rank[q] < k) emit(rank[q], mine[q]);
}

// k-th largest of one 32-bit key per lane (k <= 64), by bitwise bisection over ballots.
// LOWBIT: lowest key bit that can differ between lanes (16 for keys derived from bf16).
template <int LOWBIT>
__device__ __forceinline__ u32 wave_kth_largest(u32 key, int k) {
    u32 t = 0;
    for (int bit = 31; bit >= LOWBIT; --bit) {
        u32 cand = t | (1u << bit);
        int cnt = __popcll(__ballot(key >= cand));
        if (cnt >= k) t = cand;
    }
    if (LOWBIT > 0 && !(t >> 31)) t |= (1u << LOWBIT) - 1u;  // negative floats: low key bits are all ones
    return t;
}

// ------------------------------------------------------------------- chunk kernel -----
// LDS per workgroup: candidate lists (4 waves x 64), wave results (4 x 32), merge list (128).
template <int NL, bool BF16, bool VEC>
__global__ __launch_bounds__(256) void row_chunk_kernel(RowArgs a) {
    constexpr int E = 8 * NL;
    constexpr int CH = 256 * E;
    const int64_t g = blockIdx.y;
    const int c = blockIdx.x;
    const RowMeta meta = row_meta(a, g);
    if (!meta.valid) return;
    const int k = meta.k;
    const int lane = lane_id(), w = threadIdx.x >> 6;
    const int V = a.V;

    __shared__ u64 s_cand[4][64];
    __shared__ u64 s_wout[4][DT_K_MAX];
    __shared__ u64 s_merge[128];
    __shared__ float s_m[4], s_s[4];

    // ---- load the chunk: element (n, e) of this lane has id = base + n*512 + e ----------
    const int base = c * CH + w * (64 * E) + lane * 8;
    float x[E];
    if (BF16) {
        const uint16_t *row = (const uint16_t *)a.logits + g * a.row_stride;
#pragma unroll
        for (int n = 0; n < NL; ++n) {
            int id0 = base + n * 512;
            if (VEC && id0 + 8 <= V) {
                uint4 r = *(const uint4 *)(row + id0);
                u32 rr[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
                for (int p = 0; p < 4; ++p) {
                    x[n * 8 + 2 * p] = __uint_as_float(rr[p] << 16);
                    x[n * 8 + 2 * p + 1] = __uint_as_float(rr[p] & 0xFFFF0000u);
                }
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    x[n * 8 + e] = id0 + e < V ? bf16_bits_to_float(row[id0 + e]) : -INFINITY;
            }
        }
    } else {
        const float *row = (const float *)a.logits + g * a.row_stride;
#pragma unroll
        for (int n = 0; n < NL; ++n) {
            int id0 = base + n * 512;
            if (VEC && id0 + 8 <= V) {
                float4 r0 = *(const float4 *)(row + id0), r1 = *(const float4 *)(row + id0 + 4);
                x[n * 8 + 0] = r0.x; x[n * 8 + 1] = r0.y; x[n * 8 + 2] = r0.z; x[n * 8 + 3] = r0.w;
                x[n * 8 + 4] = r1.x; x[n * 8 + 5] = r1.y; x[n * 8 + 6] = r1.z; x[n * 8 + 7] = r1.w;
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) x[n * 8 + e] = id0 + e < V ? row[id0 + e] : -INFINITY;
            }
        }
    }

    // ---- lane maximum -----------------------------------------------------------------------
    float mx = x[0];
#pragma unroll
    for (int j = 1; j < E; ++j) mx = fmaxf(mx, x[j]);

    // ---- partial log-sum-exp of x * inv_t, relative to the lane maximum -------------------
    if (a.want_lse) {
        const float cexp = 1.4426950408889634f * a.inv_t;
        const float mref = mx == -INFINITY ? 0.f : mx;
        const float nm = -mref * cexp;
        float s = 0.f;
#pragma unroll
        for (int j = 0; j < E; ++j) s += __builtin_amdgcn_exp2f(fmaf(x[j], cexp, nm));
        const float M = wave_max(mx);
        const float Mref = M == -INFINITY ? 0.f : M;
        float term = s > 0.f ? s * __builtin_amdgcn_exp2f((mref - Mref) * cexp) : 0.f;
        term = wave_sum(term);
        if (lane == 0) { s_m[w] = M; s_s[w] = term; }
    }

    // ---- wave-level exact top-k ---------------------------------------------------------------
    float T;
    if (k == 1) {
        T = wave_max(mx);
    } else {
        T = unord32(wave_kth_largest<BF16 ? 16 : 0>(ord32(mx), k));
    }
    int n_c = 0;
#pragma unroll
    for (int j = 0; j < E; ++j) {
        const bool hit = x[j] >= T;
        const u64 m = __ballot(hit);
        if (m) {
            if (hit) {
                int slot = n_c + (int)lanes_below(m);
                if (slot < 64) s_cand[w][slot] = make_key(x[j], (u32)(base + (j >> 3) * 512 + (j & 7)));
            }
            n_c += __popcll(m);
        }
    }
    if (n_c <= 64) {
        u64 *wout = s_wout[w];
        rank_emit<1>(s_cand[w], n_c, k, [&](int r, u64 key) { wout[r] = key; });
    } else {
        // too many elements tie with the bound: k rounds of exact extract-max
        u64 prev = ~0ull;
        for (int r = 0; r < k; ++r) {
            u64 best = 0ull;
#pragma unroll
            for (int j = 0; j < E; ++j) {
                u64 key = make_key(x[j], (u32)(base + (j >> 3) * 512 + (j & 7)));
                if (key < prev && key > best) best = key;
            }
            best = wave_max_u64(best);
            if (lane == 0) s_wout[w][r] = best;
            prev = best;
        }
    }
    __syncthreads();

    // ---- workgroup merge by wave 0, partial results to scratch ----------------------------
    if (w == 0) {
        const int64_t slot = g * gridDim.x + c;
        u64 *out = a.part_keys + slot * a.key_stride;
        if (k == 1) {
            u64 best = lane < 4 ? s_wout[lane][0] : 0ull;
            best = wave_max_u64(best);
            if (lane == 0) out[0] = best;
        } else {
            u64 bound = lane < 4 ? s_wout[lane][k - 1] : 0ull;
            bound = wave_max_u64(bound);  // the best wave's k-th key: at least k keys are >= it
            int n = 0;
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                int i = lane + 64 * q;
                u64 key = i < 4 * k ? s_wout[i / k][i % k] : 0ull;
                bool hit = i < 4 * k && key >= bound;
                u64 m = __ballot(hit);
                if (hit) s_merge[n + (int)lanes_below(m)] = key;
                n += __popcll(m);
            }
            rank_emit<2>(s_merge, n, k, [&](int r, u64 key) { out[r] = key; });
        }
        if (a.want_lse && lane == 0) {
            float M = s_m[0], S = s_s[0];
#pragma unroll
            for (int q = 1; q < 4; ++q) {
                float M2 = fmaxf(M, s_m[q]);
                if (M2 != -INFINITY) {
                    const float cexp = 1.4426950408889634f * a.inv_t;
                    S = S * __builtin_amdgcn_exp2f((M - M2) * cexp) + s_s[q] * __builtin_amdgcn_exp2f((s_m[q] - M2) * cexp);
                }
                M = M2;
            }
            a.part_ms[slot] = make_float2(M, S);
        }
    }
}

// -------------------------------------------------------------------- merge kernel ------
// One wave per row: merge the S per-chunk lists (each k keys, best first) into the row's
// top-k, and the S (max, sum) pairs into the row's log-sum-exp.  S <= 64.
__global__ __launch_bounds__(64) void row_merge_kernel(RowArgs a, int S, float *top_val, int32_t *top_id,
                                                       float *lse, int out_stride) {
    const int64_t g = blockIdx.x;
    const RowMeta meta = row_meta(a, g);
    if (!meta.valid) return;
    const int k = meta.k, lane = lane_id();
    const u64 *lists = a.part_keys + g * S * a.key_stride;
    __shared__ u64 s_all[64 * DT_K_MAX];  // list c at [c*k, c*k+k)
    __shared__ u64 s_list[256];

    const int n_items = S * k;
    for (int i = lane; i < n_items; i += 64) s_all[i] = lists[(i / k) * a.key_stride + (i % k)];

    if (a.want_lse && lse) {
        const float cexp = 1.4426950408889634f * a.inv_t;
        float M = -INFINITY, Ssum = 0.f;
        if (lane < S) {
            float2 p = a.part_ms[g * S + lane];
            M = p.x;
            Ssum = p.y;
        }
        const float Mw = wave_max(M);
        float term = (Ssum > 0.f) ? Ssum * __builtin_amdgcn_exp2f((M - Mw) * cexp) : 0.f;
        term = wave_sum(term);
        if (lane == 0) lse[g] = (Mw == -INFINITY) ? -INFINITY : Mw * a.inv_t + __logf(term);
    }

    float *tv = top_val + g * out_stride;
    int32_t *ti = top_id ? top_id + g * out_stride : nullptr;
    const int V = a.V;
    auto emit = [&](int r, u64 key) {
        float v = key_val(key);
        u32 id = key_idx(key);
        bool viable = (v > -INFINITY) && (id < (u32)V);
        tv[r] = viable ? v : -INFINITY;
        if (ti) ti[r] = viable ? (int32_t)id : -1;
    };

    // Lower bound of the k-th best key: (a) the best list's k-th key, (b) the k-th largest of
    // the first q keys of every list (S*q >= k keys).  At least k keys are >= either.
    const int q = (k + S - 1) / S;
    const int nh = S * q;  // < k + S <= 96
    u64 bound = lane < S ? s_all[lane * k + k - 1] : 0ull;
    {
        u64 kth = 0ull;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            int i = lane + 64 * h;
            u64 mine = i < nh ? s_all[(i / q) * k + (i % q)] : 0ull;
            int rank = 0;
            for (int j = 0; j < nh; ++j) rank += (s_all[(j / q) * k + (j % q)] > mine) ? 1 : 0;
            if (i < nh && rank == k - 1) kth = mine;
        }
        bound = kth > bound ? kth : bound;
    }
    bound = wave_max_u64(bound);

    int n = 0;
    for (int base = 0; base < n_items; base += 64) {
        int i = base + lane;
        u64 key = i < n_items ? s_all[i] : 0ull;
        bool hit = i < n_items && key >= bound;
        u64 m = __ballot(hit);
        int slot = n + (int)lanes_below(m);
        if (hit && slot < 256) s_list[slot] = key;
        n += __popcll(m);
    }
    if (n <= 256) {
        rank_emit<4>(s_list, n, k, emit);
    } else {
        // adversarial spread of the top keys over the lists: rank every key against all
        for (int base = 0; base < n_items; base += 64) {
            int i = base + lane;
            u64 mine = i < n_items ? s_all[i] : 0ull;
            int rank = 0;
            for (int j = 0; j < n_items; ++j) rank += (s_all[j] > mine) ? 1 : 0;
            if (i < n_items && rank < k) emit(rank, mine);
        }
    }
}

// ------------------------------------------------------------------------ launchers ------
template <int NL>
static hipError_t launch_chunk(const RowArgs &a, int64_t n_rows, bool vec, hipStream_t st) {
    const int CH = 256 * 8 * NL;
    dim3 grid((a.V + CH - 1) / CH, (unsigned)n_rows);
    if (a.dtype == DT_BF16) {
        if (vec) hipLaunchKernelGGL((row_chunk_kernel<NL, true, true>), grid, dim3(256), 0, st, a);
        else hipLaunchKernelGGL((row_chunk_kernel<NL, true, false>), grid, dim3(256), 0, st, a);
    } else {
        if (vec) hipLaunchKernelGGL((row_chunk_kernel<NL, false, true>), grid, dim3(256), 0, st, a);
        else hipLaunchKernelGGL((row_chunk_kernel<NL, false, false>), grid, dim3(256), 0, st, a);
    }
    return hipGetLastError();
}

int rows_chunks_per_row(int V, int nl) { return (V + 256 * 8 * nl - 1) / (256 * 8 * nl); }

int rows_pick_nl(int64_t n_rows, int V) {
    // enough workgroups to cover the chip several times over, else smaller chunks
    for (int nl = 4; nl > 1; nl >>= 1)
        if (n_rows * rows_chunks_per_row(V, nl) >= 2048) return nl;
    return 1;
}

hipError_t rows_launch_chunks(const RowArgs &a, int64_t n_rows, int nl, hipStream_t st) {
    if (n_rows <= 0) return hipSuccess;
    const int esz = a.dtype == DT_BF16 ? 2 : 4;
    const bool vec = ((uintptr_t)a.logits % 16 == 0) && ((a.row_stride * esz) % 16 == 0);
    ProfScope prof(a.mode == ROWS_DRAFT ? KID_ROWS_DRAFT : a.mode == ROWS_TARGET ? KID_ROWS_TARGET : KID_ROWS_UNIFORM, st);
    switch (nl) {
        case 4: return launch_chunk<4>(a, n_rows, vec, st);
        case 2: return launch_chunk<2>(a, n_rows, vec, st);
        default: return launch_chunk<1>(a, n_rows, vec, st);
    }
}

hipError_t rows_launch_merge(const RowArgs &a, int64_t n_rows, int S, float *top_val, int32_t *top_id,
                             float *lse, int out_stride, hipStream_t st) {
    if (n_rows <= 0) return hipSuccess;
    ProfScope prof(KID_ROWS_MERGE, st);
    hipLaunchKernelGGL(row_merge_kernel, dim3((unsigned)n_rows), dim3(64), 0, st, a, S, top_val, top_id, lse,
                       out_stride);
    return hipGetLastError();
}

}  // namespace dt
