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

#ifdef DT_TIMESTAMPS
__device__ unsigned long long dt_dbg_stamps[64];
#define STAMP(i) do { if (threadIdx.x == 0 && blockIdx.x == 0) dt_dbg_stamps[i] = __builtin_amdgcn_s_memtime(); } while (0)
#else
#define STAMP(i) do {} while (0)
#endif

#define DT_P_MAX (DT_K_MAX + (DT_D_MAX - 1) * DT_K_MAX * DT_K_MAX)

struct Cut {
    u32 thr;      // key of the n-th best candidate
    int need_eq;  // how many candidates with key == thr are taken (lowest pool indices first)
};

__device__ __forceinline__ u32 score_key(float s) { return ord32(s); }
#define KEY_NEG_INF 0x007FFFFFu

// Selection of the `keep_max` best of score[0..n) (n <= 64*ITEMS) by one full wave, entirely from
// registers: count the viable ones, find the keep-th largest key by bisection two bits at a time
// (three independent probe counts per step, all on ballots), then visit the winners in ascending
// index: f(index, position).  Absent items hold key 0, which no probe (>= 1) ever counts.
template <int ITEMS, typename F>
__device__ __forceinline__ int wave_select_t(const float *score, int n, int keep_max, Cut *cut_out, u32 *scratch, F f) {
    const int lane = lane_id();
    u32 it[ITEMS];
    int viable = 0;
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
        const int i = j * 64 + lane;
        it[j] = i < n ? score_key(score[i]) : 0u;
        viable += __popcll(__ballot(it[j] > KEY_NEG_INF));
    }
    const int keep = min(keep_max, viable);
    Cut c;
    c.thr = 0xFFFFFFFFu;
    c.need_eq = 0;
    bool decided = false;
    if (keep > 0 && viable <= keep_max) {
        // everything viable is kept (a level whose parents propose no more than k candidates in all)
        c.thr = KEY_NEG_INF;
        decided = true;
    }
    if (keep > 0 && !decided) {
        u32 t = 0;
        if (ITEMS <= 2) {
            // few registers per lane: two bits per step (three independent probe counts)
#pragma unroll 1
            for (int bit = 30; bit >= 0; bit -= 2) {
                const u32 c1 = t | (1u << bit), c2 = t | (2u << bit), c3 = t | (3u << bit);
                int n1 = 0, n2 = 0, n3 = 0;
#pragma unroll
                for (int j = 0; j < ITEMS; ++j) {
                    n1 += __popcll(__ballot(it[j] >= c1));
                    n2 += __popcll(__ballot(it[j] >= c2));
                    n3 += __popcll(__ballot(it[j] >= c3));
                }
                t = n3 >= keep ? c3 : n2 >= keep ? c2 : n1 >= keep ? c1 : t;
            }
        } else {
            // many registers per lane: settle the upper 16 key bits on all of them, then only the
            // handful of keys that share that prefix (compacted to one per lane) decide the rest
#pragma unroll 1
            for (int bit = 31; bit >= 16; --bit) {
                const u32 c1 = t | (1u << bit);
                int n1 = 0;
#pragma unroll
                for (int j = 0; j < ITEMS; ++j) n1 += __popcll(__ballot(it[j] >= c1));
                t = n1 >= keep ? c1 : t;
            }
            int above = 0, nb = 0;
            u32 bk = 0u;  // boundary key of this lane
            bool one_per_lane = true;
#pragma unroll
            for (int j = 0; j < ITEMS; ++j) {
                above += __popcll(__ballot((it[j] >> 16) > (t >> 16)));
                const bool bnd = (it[j] >> 16) == (t >> 16);
                const u64 m = __ballot(bnd);
                // lane q takes the q-th boundary key: hand it over through LDS-free readlane
                // is not possible for a variable source, so stage through the scratch list
                if (bnd) {
                    const int slot = nb + (int)lanes_below(m);
                    if (slot < 64) scratch[slot] = it[j];
                }
                nb += __popcll(m);
            }
            one_per_lane = nb <= 64;
            const int need = keep - above;
            if (one_per_lane) {
                bk = lane < nb ? scratch[lane] : 0u;
#pragma unroll 1
                for (int bit = 15; bit >= 0; --bit) {
                    const u32 c1 = t | (1u << bit);
                    t = __popcll(__ballot(bk >= c1)) >= need ? c1 : t;
                }
            } else {
#pragma unroll 1
                for (int bit = 15; bit >= 0; --bit) {
                    const u32 c1 = t | (1u << bit);
                    int n1 = 0;
#pragma unroll
                    for (int j = 0; j < ITEMS; ++j) n1 += __popcll(__ballot(it[j] >= c1));
                    t = n1 >= keep ? c1 : t;
                }
            }
        }
        int gt = 0;
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) gt += __popcll(__ballot(it[j] > t));
        c.thr = t;
        c.need_eq = keep - gt;
    }
    if (cut_out) *cut_out = c;
    int pos = 0, eq_seen = 0;
    if (keep > 0) {
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) {
            const int i = j * 64 + lane;
            const bool eq = it[j] == c.thr;
            const u64 meq = __ballot(eq);
            const bool take = it[j] > c.thr || (eq && eq_seen + (int)lanes_below(meq) < c.need_eq);
            const u64 m = __ballot(take);
            if (take) f(i, pos + (int)lanes_below(m));
            pos += __popcll(m);
            eq_seen += __popcll(meq);
        }
    }
    return pos;
}
// scratch: 64 LDS words private to the calling wave
template <typename F>
__device__ __forceinline__ int wave_select(const float *score, int n, int keep_max, Cut *cut_out, u32 *scratch, F f) {
    if (n <= 64) return wave_select_t<1>(score, n, keep_max, cut_out, scratch, f);
    if (n <= 128) return wave_select_t<2>(score, n, keep_max, cut_out, scratch, f);
    if (n <= 256) return wave_select_t<4>(score, n, keep_max, cut_out, scratch, f);
    if (n <= 512) return wave_select_t<8>(score, n, keep_max, cut_out, scratch, f);
    return wave_select_t<16>(score, n, keep_max, cut_out, scratch, f);
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
    const int64_t r0 = a.row_off ? a.row_off[b] : (int64_t)b * a.seq_rows;
    const int xl = a.expand_level;  // > 0: only the nodes of level xl that are expanded next
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
    __shared__ u32 s_scratch[64];

    STAMP(0);
    if (xl > 0 && (TT == 1 || xl >= d)) {  // nothing is drafted below level d
        if (tid == 0) { a.n_expand[b] = 0; a.state_n_exp[b] = 0; }
        return;
    }
    if (tid == 0 && xl == 0) {
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
    // candidates through level d, or through level xl when only that level's choice is wanted (the
    // rows of deeper levels do not exist yet)
    const int P = xl > 0 ? k + (xl - 1) * k * k : k + (d - 1) * k * k;
    // Every candidate's own log-probability is known up front: the draft row that would
    // produce pool index p is fixed by p alone (only its parent is decided later).  Park
    // lp in s_score; the level loop turns it into the cumulative score in place.
    for (int p = tid; p < P; p += 256) {
        const Decoded dc = decode(p, k);
        const float v = tv[dc.row * DT_K_MAX + dc.rank];
        s_score[p] = v > -INFINITY ? v - lse[dc.row] : -INFINITY;
        s_node[p] = -1;
        s_slot[p] = -1;
    }
    __syncthreads();
    STAMP(1);

    // ---- expansion, level by level -----------------------------------------------------------
    int p_end = k;  // pool indices below p_end hold real scores (levels computed so far)
    const int l_end = xl > 0 ? xl + 1 : d;
    for (int l = 1; l < l_end; ++l) {
        const int lo = l == 1 ? 0 : k + (l - 2) * k * k;
        const int n = l == 1 ? k : k * k;
        if (w == 0) {
            int *exp_l = s_exp[l];
            const int n_exp = wave_select(s_score + lo, n, k, nullptr, s_scratch, [&](int i, int pos) {
                exp_l[pos] = lo + i;
                s_slot[lo + i] = (int8_t)pos;
            });
            if (lane_id() == 0) s_nexp = n_exp;
        }
        STAMP(2 + 2 * l);
        __syncthreads();
        const int n_exp = s_nexp;
        if (l == xl) {
            // ---- what the draft model is handed for its next pass: node s of the chosen set ----------
            if (tid < n_exp) {
                const int pi = s_exp[l][tid];
                const Decoded dc = decode(pi, k);
                const int64_t e = (int64_t)b * DT_K_MAX + tid;
                a.exp_token[e] = ti[dc.row * DT_K_MAX + dc.rank];
                a.exp_parent_slot[e] = l == 1 ? -1 : dc.slot;
                const int own = 1 + (l - 1) * k + tid;
                a.exp_row[e] = own;
                a.exp_pos[e] = (a.prefix_len ? max(a.prefix_len[b], 0) : 0) + l;
                // draft-side mask over draft rows: the root's row, the rows of the ancestors, its own
                u64 m0 = 1ull, m1 = 0ull, m2 = 0ull, m3 = 0ull;
                auto set = [&](int r) {
                    const u64 bit = 1ull << (r & 63);
                    const int wd = r >> 6;
                    m0 |= wd == 0 ? bit : 0ull; m1 |= wd == 1 ? bit : 0ull;
                    m2 |= wd == 2 ? bit : 0ull; m3 |= wd == 3 ? bit : 0ull;
                };
                set(own);
                int pp = l == 1 ? -1 : s_exp[l - 1][dc.slot];
                for (int guard = 0; guard < DT_D_MAX && pp >= 0; ++guard) {
                    const Decoded dp = decode(pp, k);
                    set(1 + (dp.level - 1) * k + s_slot[pp]);
                    pp = dp.level == 1 ? -1 : s_exp[dp.level - 1][dp.slot];
                }
                a.exp_mask[e * 4] = m0; a.exp_mask[e * 4 + 1] = m1;
                a.exp_mask[e * 4 + 2] = m2; a.exp_mask[e * 4 + 3] = m3;
            }
            if (tid == 0) { a.n_expand[b] = n_exp; a.state_n_exp[b] = n_exp; }
            return;
        }
        if (n_exp == 0) break;
        const int nlo = k + (l - 1) * k * k;
        for (int t = tid; t < k * k; t += 256) {
            const int s = t / k;
            // slots beyond the expanded set own no node: their candidates do not exist
            s_score[nlo + t] = s < n_exp ? s_score[s_exp[l][s]] + s_score[nlo + t] : -INFINITY;
        }
        p_end = nlo + k * k;
        __syncthreads();
        STAMP(3 + 2 * l);
    }

    if (xl > 0) {  // an earlier level had nothing viable to expand
        if (tid == 0) { a.n_expand[b] = 0; a.state_n_exp[b] = 0; }
        return;
    }
    __syncthreads();  // every wave has read s_nexp before it is reused below

    // ---- rerank: the TT-1 best of the whole pool ----------------------------------------------
    Cut cut;
    int keep;
    if (p_end <= 1024) {
        if (w == 0) {
            const int kp = wave_select(s_score, p_end, TT - 1, nullptr, s_scratch,
                                       [&](int i, int pos) { s_node[i] = (int16_t)(pos + 1); });
            if (lane_id() == 0) s_nexp = kp;
        }
        __syncthreads();
        keep = s_nexp;
    } else {
        int v = 0;
        for (int i = tid; i < p_end; i += 256) v += s_score[i] > -INFINITY ? 1 : 0;
        keep = min(TT - 1, block_sum_256(v, s_red));
        cut.thr = 0xFFFFFFFFu;
        cut.need_eq = 0;
        if (keep > 0) cut = block_cut(s_score, p_end, keep, s_red);
    }
    STAMP(20);
    if (p_end > 1024) {
        if (w == 0 && keep > 0)
            wave_enumerate(s_score, p_end, cut, [&](int i, int pos) { s_node[i] = (int16_t)(pos + 1); });
        __syncthreads();
    }
    if (tid == 0) a.n_nodes[b] = keep + 1;
    STAMP(21);

    // ---- emission -------------------------------------------------------------------------------
    for (int p = tid; p < p_end; p += 256) {
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
    STAMP(22);
}

#ifdef DT_TIMESTAMPS
extern "C" int dt_debug_stamps(unsigned long long *out) {
    return (int)hipMemcpyFromSymbol(out, HIP_SYMBOL(dt_dbg_stamps), sizeof(unsigned long long) * 64);
}
#endif

hipError_t tree_launch(const TreeArgs &a, hipStream_t st) {
    if (a.batch <= 0) return hipSuccess;
    launch_kernel(KID_TREE, st, tree_kernel, dim3(a.batch), dim3(256), 0, a);
    return hipGetLastError();
}

}  // namespace dt
