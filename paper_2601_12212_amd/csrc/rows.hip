// Row kernels: top-k and log-sum-exp over vocabulary rows (draft rows: k best + lse;
// target rows: arg max, and lse of row/T for stochastic acceptance).
//
// Top-k rows take two passes.  The first is a pure stream: a row is cut into chunks of
// 256*8*NL elements, each lane reads 8*NL of them with coalesced 16-byte loads and leaves
// only its maximum (plus one (max, sum-exp) pair per wave).  The second works on those lane
// maxima, 8*NL times fewer than the logits: the k-th largest lane maximum bounds the k-th
// largest element from below, so only the ~k lanes that reach it are read again and their
// elements ranked by 64-bit (value, id) keys -- exact under (value desc, id asc).  Rows
// dominated by ties fall back to a slow exact loop.
#include "common.hpp"
#include "kernels.hpp"

namespace dt {


// ---------------------------------------------------------------- row -> (valid, k) ----
struct RowMeta {
    bool valid;
    int k;
    int64_t out;  // row index of the results (top-k values, ids, lse)
};

__device__ __forceinline__ RowMeta row_meta(const RowArgs &a, int64_t g) {
    RowMeta m;
    m.valid = true;
    m.k = a.k_uniform;
    m.out = g;
    if (a.mode == ROWS_LEVEL) {
        // level-at-a-time build: row s of sequence b in this call is the row of the s-th node expanded
        // one level up (level 1: the root's row); its results go to the sequence's row slot in the state
        const int b = (int)(g / a.rows_per_seq), s = (int)(g % a.rows_per_seq);
        const dt_params p = a.params[b];
        const int TT = min(max(p.TT, 1), a.TT_cap), d = min(max(p.d, 1), DT_D_MAX);
        const int k = min(max(p.k, 1), min(DT_K_MAX, a.V));
        const int cnt = a.level == 1 ? 1 : min(max(a.n_exp_prev[b], 0), k);
        m.k = k;
        m.valid = TT > 1 && a.level <= d && s < cnt;
        m.out = (int64_t)b * a.state_rows + (a.level == 1 ? 0 : 1 + (a.level - 2) * k + s);
    } else if (a.mode == ROWS_DRAFT) {
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
        m.out = (int64_t)lo * DT_STATE_ROWS + r;  // results in the sequence's own block of rows
    } else if (a.mode == ROWS_TARGET) {
        int b = (int)(g / a.TT_cap), i = (int)(g % a.TT_cap);
        m.k = 1;
        m.valid = i < a.n_nodes[b];
    }
    return m;
}

// ------------------------------------------------- rank at most 64 keys, keep the k best --
// Keys are held one per lane (lanes >= n hold 0) and are distinct.  Each lane ranks its key by
// comparing against every lane's key through readlane: no LDS traffic, no wait inside the loop.
// The key of rank r < k is handed to emit(r, key).
template <typename Emit>
__device__ __forceinline__ void rank_emit_lanes(u64 mine, int n, int k, Emit emit) {
    int rank = 0;
    for (int i = 0; i < n; ++i) rank += (readlane_u64(mine, i) > mine) ? 1 : 0;
    if (lane_id() < n && rank < k) emit(rank, mine);
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

// -------------------------------------------------------------------- chunk loading -----
// Element (n, e) of a lane, n < NL, e < 8, has id = base + n*512 + e with
// base = chunk*256*8*NL + wave*64*8*NL + lane*8: one coalesced 16-byte load per (lane, n).
// Two halves, so that a kernel can put other waits (the row's metadata) between them:
// chunk_request asks for a lane's NL 16-byte groups (32-byte for fp32), unconditionally, so that they are in
// flight together -- a load inside a branch is waited for inside that branch, and the NL trips to memory would
// follow one another.  A lane whose eight elements do not all lie inside the row asks for the row's first eight
// instead (V >= 8 on the vector path); chunk_finish converts what arrived and patches those lanes (at most one
// lane of a row straddles its end) with element loads.  Without VEC everything happens in chunk_finish.
template <int NL, bool BF16>
struct RawChunk {
    uint4 r[BF16 ? NL : 2 * NL];
};
template <int NL, bool BF16, bool VEC>
__device__ __forceinline__ void chunk_request(const RowArgs &a, int64_t g, int base, RawChunk<NL, BF16> &raw) {
    if (!VEC) return;
    const int V = a.V;
    if (BF16) {
        const uint16_t *row = (const uint16_t *)a.logits + g * a.row_stride;
#pragma unroll
        for (int n = 0; n < NL; ++n) {
            const int id0 = base + n * 512;
            raw.r[n] = *(const uint4 *)(row + (id0 + 8 <= V ? id0 : 0));
        }
    } else {
        const float *row = (const float *)a.logits + g * a.row_stride;
#pragma unroll
        for (int n = 0; n < NL; ++n) {
            const int id0 = base + n * 512, idv = id0 + 8 <= V ? id0 : 0;
            raw.r[2 * n] = *(const uint4 *)(row + idv);
            raw.r[2 * n + 1] = *(const uint4 *)(row + idv + 4);
        }
    }
    __builtin_amdgcn_sched_barrier(0);  // every request is out before anything that follows
}
template <int NL, bool BF16, bool VEC>
__device__ __forceinline__ void chunk_finish(const RowArgs &a, int64_t g, int base, const RawChunk<NL, BF16> &raw,
                                             float (&x)[8 * NL]) {
    const int V = a.V;
    if (BF16) {
        const uint16_t *row = (const uint16_t *)a.logits + g * a.row_stride;
        if (VEC) {
#pragma unroll
            for (int n = 0; n < NL; ++n) {
                const u32 rr[4] = {raw.r[n].x, raw.r[n].y, raw.r[n].z, raw.r[n].w};
#pragma unroll
                for (int p = 0; p < 4; ++p) {
                    x[n * 8 + 2 * p] = __uint_as_float(rr[p] << 16);
                    x[n * 8 + 2 * p + 1] = __uint_as_float(rr[p] & 0xFFFF0000u);
                }
            }
        }
#pragma unroll
        for (int n = 0; n < NL; ++n) {
            const int id0 = base + n * 512;
            if (!VEC || id0 + 8 > V) {
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    x[n * 8 + e] = id0 + e < V ? bf16_bits_to_float(row[id0 + e]) : -INFINITY;
            }
        }
    } else {
        const float *row = (const float *)a.logits + g * a.row_stride;
        if (VEC) {
#pragma unroll
            for (int n = 0; n < NL; ++n) {
                const uint4 r0 = raw.r[2 * n], r1 = raw.r[2 * n + 1];
                x[n * 8 + 0] = __uint_as_float(r0.x); x[n * 8 + 1] = __uint_as_float(r0.y);
                x[n * 8 + 2] = __uint_as_float(r0.z); x[n * 8 + 3] = __uint_as_float(r0.w);
                x[n * 8 + 4] = __uint_as_float(r1.x); x[n * 8 + 5] = __uint_as_float(r1.y);
                x[n * 8 + 6] = __uint_as_float(r1.z); x[n * 8 + 7] = __uint_as_float(r1.w);
            }
        }
#pragma unroll
        for (int n = 0; n < NL; ++n) {
            const int id0 = base + n * 512;
            if (!VEC || id0 + 8 > V) {
#pragma unroll
                for (int e = 0; e < 8; ++e) x[n * 8 + e] = id0 + e < V ? row[id0 + e] : -INFINITY;
            }
        }
    }
}

// (max, sum of exp((x - max) * inv_t)) of a wave's elements, from the lane maxima.
template <int E>
__device__ __forceinline__ float2 wave_lse_partial(const float (&x)[E], float mx, float inv_t) {
    const float cexp = 1.4426950408889634f * inv_t;
    const float mref = mx == -INFINITY ? 0.f : mx;
    const float nm = -mref * cexp;
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < E; ++j) s += __builtin_amdgcn_exp2f(fmaf(x[j], cexp, nm));
    const float M = wave_max(mx);
    const float Mref = M == -INFINITY ? 0.f : M;
    float term = s > 0.f ? s * __builtin_amdgcn_exp2f((mref - Mref) * cexp) : 0.f;
    return make_float2(M, wave_sum(term));
}

// ------------------------------------------------------------ streaming kernel (top-k rows) --
// Pure stream: every wave reads its 64*8*NL elements once and leaves behind one maximum per
// lane and one (max, sum) pair per wave.  No LDS, no barrier.  All selection happens later on
// the lane maxima, which are 8*NL times fewer than the logits.
template <int NL, bool BF16, bool VEC>
__global__ __launch_bounds__(256) void row_stream_kernel(RowArgs a) {
    constexpr int E = 8 * NL;
    // workgroup (chunk c, row g): the chunk rides in grid x, the row in y and -- past 65,535 rows -- z
    // (no division in front of the loads: a streaming workgroup's life is one trip to memory long)
    const int64_t g = (int64_t)blockIdx.z * gridDim.y + blockIdx.y;
    const int c = blockIdx.x;
    const int lane = lane_id(), w = threadIdx.x >> 6;
    const int base = c * (256 * E) + w * (64 * E) + lane * 8;
    if (g >= a.n_rows) return;
    // early: the row's elements are on their way while the (dependent, scalar) reads of its metadata are waited for
    float x[E];
    RawChunk<NL, BF16> raw;
    if (a.early_load) chunk_request<NL, BF16, VEC>(a, g, base, raw);
    const RowMeta meta = row_meta(a, g);
    if (!meta.valid) return;
    if (!a.early_load) chunk_request<NL, BF16, VEC>(a, g, base, raw);
    chunk_finish<NL, BF16, VEC>(a, g, base, raw, x);
    float mx = x[0];
#pragma unroll
    for (int j = 1; j < E; ++j) mx = fmaxf(mx, x[j]);
    const int64_t wslot = (g * gridDim.x + c) * 4 + w;
    a.lane_max[wslot * 64 + lane] = mx;
    if (a.want_lse) {
        const float2 p = wave_lse_partial<E>(x, mx, a.inv_t);
        if (lane == 0) a.part_ms[wslot] = p;
    }
}

// ------------------------------------------------------------- selection kernel (top-k rows) --
// One workgroup per row, working on the row's S*256 lane maxima:
//   1. every thread takes the maximum of its S lane maxima; each wave finds the k-th largest of
//      its 64 thread maxima (ballot bisection); the largest of the four, T0, is a lower bound of
//      the row's k-th largest lane maximum (loose: up to a few hundred lane maxima reach it);
//   2. the lane maxima >= T0 go into a histogram over their distance from T0 in steps of the upper
//      16 key bits (for bf16 data: in representable values), and a scan from the top names the bin
//      of the k-th largest lane maximum.  Its lower edge T1 is a lower bound of the row's k-th
//      largest ELEMENT (k different lanes hold an element >= T1), and only lanes whose maximum
//      reaches T1 ("hot" lanes: k of them plus ties at the edge) can hold a winner;
//   3. the hot lanes' 8*NL elements are read again (they sit in L2), elements >= T1 are keyed
//      by (value, id) and ranked by counting.
// More than 128 hot lanes or candidates (rows dominated by ties, fewer than k finite entries)
// switch to an exact but slow extract-max loop over the whole row.
#define SEL_CAP 128
__device__ __forceinline__ float load_elem(const RowArgs &a, int64_t g, int id) {
    if (a.dtype == DT_BF16) return bf16_bits_to_float(((const uint16_t *)a.logits)[g * a.row_stride + id]);
    return ((const float *)a.logits)[g * a.row_stride + id];
}

template <bool BF16>
__global__ __launch_bounds__(256) void row_select_kernel(RowArgs a, int nl, int S, int vec, float *top_val,
                                                         int32_t *top_id, float *lse, int out_stride) {
    const int64_t g = blockIdx.x;
    const int tid = threadIdx.x, lane = lane_id(), w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int V = a.V, E = 8 * nl;
    const int n_lanes = S * 256;
    const float *lm = a.lane_max + g * n_lanes;
    // the lane maxima do not depend on the row's metadata (two dependent global reads): ask for them
    // first, and wave 3 for the row's (max, sum) partials.  Rows that turn out to be dead have their
    // slots in the workspace all the same.
    float it[16];
    if (S <= 16) {
#pragma unroll
        for (int j = 0; j < 16; ++j) it[j] = lm[min(j, S - 1) * 256 + tid];
    }
    const bool lse_wave = w == 3 && a.want_lse && lse;
    float2 pm = make_float2(-INFINITY, 0.f);
    if (lse_wave && S <= 16) pm = a.part_ms[g * S * 4 + min(lane, S * 4 - 1)];
    const RowMeta meta = row_meta(a, g);
    if (!meta.valid) return;
    const int k = meta.k;

    __shared__ float s_T[4];
    __shared__ __attribute__((aligned(16))) u32 s_hist[256];
    __shared__ int s_hot[SEL_CAP];
    __shared__ int s_h;
    __shared__ u64 s_fin[SEL_CAP];
    __shared__ int s_n2;
    __shared__ u64 s_best[4];

    float *tv = top_val + meta.out * out_stride;
    int32_t *ti = top_id ? top_id + meta.out * out_stride : nullptr;
    auto emit = [&](int r, u64 key) {
        float v = key_val(key);
        u32 id = key_idx(key);
        bool viable = (v > -INFINITY) && (id < (u32)V);
        tv[r] = viable ? v : -INFINITY;
        if (ti) ti[r] = viable ? (int32_t)id : -1;
    };

    // ---- 1. thread maxima, per-wave k-th largest, T0 ------------------------------------------
    float tmax = -INFINITY;
    if (S <= 16) {
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            it[j] = j < S ? it[j] : -INFINITY;
            tmax = fmaxf(tmax, it[j]);
        }
    } else {
        for (int j = 0; j < S; ++j) tmax = fmaxf(tmax, lm[j * 256 + tid]);
    }
    const float Tw = unord32(wave_kth_largest<BF16 ? 16 : 0>(ord32(tmax), k));
    if (lane == 0) s_T[w] = Tw;
    if (tid == 0) { s_n2 = 0; s_h = 0; }
    s_hist[tid] = 0u;
    __syncthreads();
    const float T0 = fmaxf(fmaxf(s_T[0], s_T[1]), fmaxf(s_T[2], s_T[3]));

    // ---- 2. histogram of the lane maxima >= T0; its scan from the top gives T1 ------------------
    const u32 key0 = ord32(T0) >> 16;
    if (S <= 16) {
#pragma unroll
        for (int j = 0; j < 16; ++j)
            if (it[j] >= T0) atomicAdd(&s_hist[min((ord32(it[j]) >> 16) - key0, 255u)], 1u);
    } else {
        for (int j = 0; j < S; ++j) {
            const float v = lm[j * 256 + tid];
            if (v >= T0) atomicAdd(&s_hist[min((ord32(v) >> 16) - key0, 255u)], 1u);
        }
    }
    __syncthreads();
    // every wave by itself: lane L holds bins 4(63-L) .. 4(63-L)+3, so an ascending lane scan walks the
    // bins downwards; at least k lane maxima reach T0, so the scan finds its bin
    int n_hot;      // lane maxima >= T1
    float T1;
    {
        const uint4 hb = *(const uint4 *)&s_hist[4 * (63 - lane)];
        const int c4 = (int)(hb.x + hb.y + hb.z + hb.w);
        const int incl = wave_scan_incl_i32(c4);
        const u64 m = __ballot(incl >= k);
        const int ls = m ? (int)__builtin_ctzll(m) : 63;
        int acc = __builtin_amdgcn_readlane(incl - c4, ls);
        const int h3 = __builtin_amdgcn_readlane((int)hb.w, ls), h2 = __builtin_amdgcn_readlane((int)hb.z, ls),
                  h1 = __builtin_amdgcn_readlane((int)hb.y, ls), h0 = __builtin_amdgcn_readlane((int)hb.x, ls);
        int dg;
        if (acc + h3 >= k) { dg = 3; acc += h3; }
        else if (acc + h3 + h2 >= k) { dg = 2; acc += h3 + h2; }
        else if (acc + h3 + h2 + h1 >= k) { dg = 1; acc += h3 + h2 + h1; }
        else { dg = 0; acc += h3 + h2 + h1 + h0; }
        n_hot = acc;
        // the lower edge of that bin: the smallest float whose upper 16 key bits are the bin's (bin 255 also
        // holds everything farther up: its lower edge still bounds all of it)
        T1 = unord32((key0 + (u32)(4 * (63 - ls) + dg)) << 16);
        T1 = fmaxf(T1, T0);  // bin 0 starts at T0 itself, not at the edge below it
    }
    bool slow = n_hot > SEL_CAP || n_hot < k;  // uniform over the workgroup

    // ---- the row's log-sum-exp, by wave 3: called where the other waves wait for memory anyway ----------
    bool lse_done = false;
    auto row_lse = [&]() {
        lse_done = true;
        if (!lse_wave) return;
        const float cexp = 1.4426950408889634f * a.inv_t;
        float M = -INFINITY, Ssum = 0.f;
        if (S <= 16) {
            if (lane < S * 4) { M = pm.x; Ssum = pm.y; }
        } else {
            for (int i = lane; i < S * 4; i += 64) {
                const float2 p = a.part_ms[g * S * 4 + i];
                const float M2 = fmaxf(M, p.x);
                if (M2 != -INFINITY)
                    Ssum = Ssum * __builtin_amdgcn_exp2f((M - M2) * cexp) + p.y * __builtin_amdgcn_exp2f((p.x - M2) * cexp);
                M = M2;
            }
        }
        const float Mw = wave_max(M);
        float term = (Ssum > 0.f) ? Ssum * __builtin_amdgcn_exp2f((M - Mw) * cexp) : 0.f;
        term = wave_sum(term);
        if (lane == 0) lse[meta.out] = (Mw == -INFINITY) ? -INFINITY : Mw * a.inv_t + __logf(term);
    };

    if (!slow) {
        // ---- 3. the hot lanes, in any order: a thread reserves room for its hits with one LDS add ----
        {
            int mine = 0;
            if (S <= 16) {
#pragma unroll
                for (int j = 0; j < 16; ++j) mine += it[j] >= T1 ? 1 : 0;
                if (mine > 0) {
                    int at = atomicAdd(&s_h, mine);
#pragma unroll
                    for (int j = 0; j < 16; ++j)
                        if (it[j] >= T1) { if (at < SEL_CAP) s_hot[at] = j * 256 + tid; ++at; }
                }
            } else {
                for (int j = 0; j < S; ++j)
                    if (lm[j * 256 + tid] >= T1) {
                        const int at = atomicAdd(&s_h, 1);
                        if (at < SEL_CAP) s_hot[at] = j * 256 + tid;
                    }
            }
        }
        __syncthreads();
        const int h = min(s_h, SEL_CAP);
        const int nl_log2 = nl == 4 ? 2 : nl == 2 ? 1 : 0;  // chunk multipliers are 1, 2 or 4
        if (h * nl <= 192) row_lse();  // wave 3 has no hot lane to re-read: it merges while the others wait for theirs
        // ---- 4. re-read the hot lanes: (hot lane, load n) pairs spread over the threads ----
        for (int q = tid; q < h * nl; q += 256) {
            const int gl = s_hot[q >> nl_log2], n = q & (nl - 1);
            const int c = gl >> 8, ww = (gl >> 6) & 3, l = gl & 63;
            const int id0 = c * (256 * E) + ww * (64 * E) + l * 8 + n * 512;
            float xv[8];
            if (BF16 && vec && id0 + 8 <= V) {
                const uint4 r = *(const uint4 *)((const uint16_t *)a.logits + g * a.row_stride + id0);
                const u32 rr[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
                for (int p = 0; p < 4; ++p) {
                    xv[2 * p] = __uint_as_float(rr[p] << 16);
                    xv[2 * p + 1] = __uint_as_float(rr[p] & 0xFFFF0000u);
                }
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) xv[e] = load_elem(a, g, min(id0 + e, V - 1));
#pragma unroll
                for (int e = 0; e < 8; ++e) xv[e] = id0 + e < V ? xv[e] : -INFINITY;
            }
            int hits = 0;
#pragma unroll
            for (int e = 0; e < 8; ++e) hits += xv[e] >= T1 ? 1 : 0;
            if (hits > 0) {
                int slot = atomicAdd(&s_n2, hits);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    if (xv[e] >= T1) {
                        if (slot < SEL_CAP) s_fin[slot] = make_key(xv[e], (u32)(id0 + e));
                        ++slot;
                    }
                }
            }
        }
        if (h * nl > 192) row_lse();
        __syncthreads();
        const int n2 = s_n2;
        if (n2 <= SEL_CAP) {
            // ---- 5. candidate t ranks itself against all n2 keys (LDS broadcasts, eight in flight) ----
            if (tid < SEL_CAP && (tid & ~63) < n2) {  // the waves that hold a candidate
                const u64 mine = tid < n2 ? s_fin[tid] : 0ull;
                int r0 = 0, r1 = 0;
                for (int j0 = 0; j0 < n2; j0 += 8) {
                    u64 o[8];
#pragma unroll
                    for (int j = 0; j < 8; ++j) o[j] = s_fin[min(j0 + j, SEL_CAP - 1)];
#pragma unroll
                    for (int j = 0; j < 8; j += 2) {  // s_fin[n2 ..] may hold anything: masked
                        r0 += j0 + j < n2 && o[j] > mine ? 1 : 0;
                        r1 += j0 + j + 1 < n2 && o[j + 1] > mine ? 1 : 0;
                    }
                }
                if (tid < n2 && r0 + r1 < k) emit(r0 + r1, mine);
            }
            return;
        }
        slow = true;
    }

    // ---- exact fallback: k rounds of "largest key below the previous winner" ----------------
    if (!lse_done) row_lse();
    u64 prev = ~0ull;
    for (int r = 0; r < k; ++r) {
        u64 best = 0ull;
        for (int id = tid; id < V; id += 256) {
            const u64 key = make_key(load_elem(a, g, id), (u32)id);
            if (key < prev && key > best) best = key;
        }
        best = wave_max_u64(best);
        __syncthreads();
        if (lane == 0) s_best[w] = best;
        __syncthreads();
        u64 b01 = s_best[0] > s_best[1] ? s_best[0] : s_best[1];
        u64 b23 = s_best[2] > s_best[3] ? s_best[2] : s_best[3];
        best = b01 > b23 ? b01 : b23;
        if (tid == 0) {
            if (best != 0ull) emit(r, best);
            else { tv[r] = -INFINITY; if (ti) ti[r] = -1; }
        }
        prev = best;  // 0 once the row is exhausted: nothing is below it, later slots stay empty
    }
}

// ------------------------------------------------------------- arg max kernel (target rows) --
// k = 1: every workgroup leaves the best (value, id) key of its chunk, and optionally the
// (max, sum) pair of row/T; the acceptance kernel merges the chunks of a row.
template <int NL, bool BF16, bool VEC>
__global__ __launch_bounds__(256) void row_argmax_kernel(RowArgs a) {
    constexpr int E = 8 * NL;
    const int64_t g = (int64_t)blockIdx.z * gridDim.y + blockIdx.y;
    const int c = blockIdx.x;
    const int lane = lane_id(), w = threadIdx.x >> 6;
    __shared__ u64 s_wout[4];
    __shared__ float s_m[4], s_s[4];

    const int base = c * (256 * E) + w * (64 * E) + lane * 8;
    if (g >= a.n_rows) return;
    // early: the row's elements are on their way while the (dependent, scalar) reads of its metadata are waited for
    float x[E];
    RawChunk<NL, BF16> raw;
    if (a.early_load) chunk_request<NL, BF16, VEC>(a, g, base, raw);
    const RowMeta meta = row_meta(a, g);
    if (!meta.valid) return;
    if (!a.early_load) chunk_request<NL, BF16, VEC>(a, g, base, raw);
    chunk_finish<NL, BF16, VEC>(a, g, base, raw, x);
    float mx = x[0];
#pragma unroll
    for (int j = 1; j < E; ++j) mx = fmaxf(mx, x[j]);
    if (a.want_lse) {
        const float2 p = wave_lse_partial<E>(x, mx, a.inv_t);
        if (lane == 0) { s_m[w] = p.x; s_s[w] = p.y; }
    }
    // the wave's best key: lanes holding the wave maximum find their first such element
    const float T = wave_max(mx);
    u64 key = 0ull;
    if (mx == T) {
        int jbest = 0;
#pragma unroll
        for (int j = E - 1; j >= 0; --j) jbest = x[j] == T ? j : jbest;
        key = make_key(T, (u32)(base + (jbest >> 3) * 512 + (jbest & 7)));
    }
    key = wave_max_u64(key);
    if (lane == 0) s_wout[w] = key;
    __syncthreads();
    if (threadIdx.x == 0) {
        const int64_t slot = g * gridDim.x + c;
        u64 b01 = s_wout[0] > s_wout[1] ? s_wout[0] : s_wout[1];
        u64 b23 = s_wout[2] > s_wout[3] ? s_wout[2] : s_wout[3];
        a.part_keys[slot] = b01 > b23 ? b01 : b23;
        if (a.want_lse) {
            const float cexp = 1.4426950408889634f * a.inv_t;
            float M = s_m[0], S = s_s[0];
#pragma unroll
            for (int q = 1; q < 4; ++q) {
                float M2 = fmaxf(M, s_m[q]);
                if (M2 != -INFINITY)
                    S = S * __builtin_amdgcn_exp2f((M - M2) * cexp) + s_s[q] * __builtin_amdgcn_exp2f((s_m[q] - M2) * cexp);
                M = M2;
            }
            a.part_ms[slot] = make_float2(M, S);
        }
    }
}

// ------------------------------------------------------------------------ launchers ------

int rows_chunks_per_row(int V, int nl) { return (V + 256 * 8 * nl - 1) / (256 * 8 * nl); }

// Chunk multiplier for the top-k rows: the smallest that keeps a row within 16 chunks (so that
// the selection kernel holds its lane maxima in registers); 4 beyond that.
int rows_topk_nl(int V) {
    for (int nl = 1; nl <= 4; nl <<= 1)
        if (rows_chunks_per_row(V, nl) <= 16) return nl;
    return 4;
}

// Chunk multiplier for the arg max rows: few, fat chunks (the acceptance kernel merges the
// chunks of a row, and measured kernel time does not depend on the chunk size), but at least
// about one workgroup per compute unit.
int rows_pick_nl(int64_t n_rows, int V) {
    for (int nl = 4; nl > 1; nl >>= 1)
        if (n_rows * rows_chunks_per_row(V, nl) >= 256) return nl;
    return 1;
}

// (chunks, rows) as a launch grid: rows beyond what grid y holds continue in z; the last z-slab may
// overhang, its workgroups leave at once
static dim3 rows_grid(int chunks, int64_t n_rows) {
    const int64_t ny = n_rows < 65535 ? n_rows : 65535;
    return dim3((unsigned)chunks, (unsigned)ny, (unsigned)((n_rows + ny - 1) / ny));
}

static bool rows_vec_ok(const RowArgs &a) {
    const int esz = a.dtype == DT_BF16 ? 2 : 4;
    return ((uintptr_t)a.logits % 16 == 0) && ((a.row_stride * esz) % 16 == 0) && a.V >= 8;
}

#define DT_ROWS_DISPATCH(KID, KERNEL, NLV, GRID)                                                          \
    do {                                                                                                  \
        dim3 grid = GRID;                                                                                 \
        if (a.dtype == DT_BF16) {                                                                         \
            if (vec) launch_kernel(KID, st, KERNEL<NLV, true, true>, grid, dim3(256), 0, a);              \
            else launch_kernel(KID, st, KERNEL<NLV, true, false>, grid, dim3(256), 0, a);                 \
        } else {                                                                                          \
            if (vec) launch_kernel(KID, st, KERNEL<NLV, false, true>, grid, dim3(256), 0, a);             \
            else launch_kernel(KID, st, KERNEL<NLV, false, false>, grid, dim3(256), 0, a);                \
        }                                                                                                 \
    } while (0)

// top-k rows, pass 1: lane maxima and (max, sum) partials
// Launches of at most this many workgroups are latency bound: their rows are read before they are known
// to be live.  Larger ones are bandwidth bound, and the bytes of a dead row would cost time.
static const int64_t EARLY_LOAD_WGS = 2048;

hipError_t rows_launch_stream(const RowArgs &a_in, int64_t n_rows, int nl, hipStream_t st) {
    if (n_rows <= 0) return hipSuccess;
    RowArgs a = a_in;
    // every row of a draft or uniform launch is live unless the caller's row_off leaves gaps
    a.early_load = a.mode == ROWS_DRAFT || a.mode == ROWS_UNIFORM || n_rows * rows_chunks_per_row(a.V, nl) <= EARLY_LOAD_WGS;
    const bool vec = rows_vec_ok(a);
    const int kid = a.mode == ROWS_DRAFT ? KID_ROWS_DRAFT : KID_ROWS_UNIFORM;
    a.n_rows = n_rows;
#define STREAM_GRID(NLV) rows_grid(rows_chunks_per_row(a.V, NLV), n_rows)
    switch (nl) {
        case 4: DT_ROWS_DISPATCH(kid, row_stream_kernel, 4, STREAM_GRID(4)); break;
        case 2: DT_ROWS_DISPATCH(kid, row_stream_kernel, 2, STREAM_GRID(2)); break;
        default: DT_ROWS_DISPATCH(kid, row_stream_kernel, 1, STREAM_GRID(1)); break;
    }
#undef STREAM_GRID
    return hipGetLastError();
}

// top-k rows, pass 2: selection on the lane maxima
hipError_t rows_launch_select(const RowArgs &a, int64_t n_rows, int nl, float *top_val, int32_t *top_id, float *lse,
                              int out_stride, hipStream_t st) {
    if (n_rows <= 0) return hipSuccess;
    const int S = rows_chunks_per_row(a.V, nl);
    const int vec = rows_vec_ok(a) ? 1 : 0;
    if (a.dtype == DT_BF16)
        launch_kernel(KID_ROWS_MERGE, st, row_select_kernel<true>, dim3((unsigned)n_rows), dim3(256), 0, a, nl, S,
                      vec, top_val, top_id, lse, out_stride);
    else
        launch_kernel(KID_ROWS_MERGE, st, row_select_kernel<false>, dim3((unsigned)n_rows), dim3(256), 0, a, nl, S,
                      vec, top_val, top_id, lse, out_stride);
    return hipGetLastError();
}

// arg max rows (target logits)
hipError_t rows_launch_argmax(const RowArgs &a_in, int64_t n_rows, int nl, hipStream_t st) {
    if (n_rows <= 0) return hipSuccess;
    RowArgs a = a_in;
    a.early_load = n_rows * rows_chunks_per_row(a.V, nl) <= EARLY_LOAD_WGS;
    const bool vec = rows_vec_ok(a);
    a.n_rows = n_rows;
#define STREAM_GRID(NLV) rows_grid(rows_chunks_per_row(a.V, NLV), n_rows)
    switch (nl) {
        case 4: DT_ROWS_DISPATCH(KID_ROWS_TARGET, row_argmax_kernel, 4, STREAM_GRID(4)); break;
        case 2: DT_ROWS_DISPATCH(KID_ROWS_TARGET, row_argmax_kernel, 2, STREAM_GRID(2)); break;
        default: DT_ROWS_DISPATCH(KID_ROWS_TARGET, row_argmax_kernel, 1, STREAM_GRID(1)); break;
    }
#undef STREAM_GRID
    return hipGetLastError();
}

}  // namespace dt
