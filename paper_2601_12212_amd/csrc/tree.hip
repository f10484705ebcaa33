// Tree kernel: layer-wise expansion, rerank, and emission of the node arrays and the
// ancestor bitsets.  One workgroup of eight waves per sequence; the whole candidate pool (at most
// k + (d-1)k^2 = 7200 scores) lives in LDS.
//
// Selections ("the n best by (score desc, pool index asc)") never sort.
//  * A level of up to 128 candidates (k <= 11) is ranked by counting: every candidate counts the candidates with
//    a larger key, the work split over the waves by (64 candidates) x (a slice of the others), the
//    others read as LDS broadcasts.  Every wave then forms the chosen set by itself from the partial
//    counts, so the next level's scores follow without another barrier.
//  * Everything else (larger levels, the rerank over the pool, exact ties that straddle a cut) is cut by
//    score buckets: one LDS histogram over floor(-8 score) and one scan name the bucket that holds the
//    cut, the few candidates inside it rank themselves one against the other, everything in a better
//    bucket is taken; one workgroup-wide prefix count hands out positions in pool-index order (of equal
//    keys the lowest indices first).  A bucket too crowded for that goes through a radix selection over
//    the order-preserving integer image of the score (four 8-bit digits, one histogram and one barrier
//    per digit, every wave scanning the 256 bins by itself).
#include "common.hpp"
#include "kernels.hpp"

namespace dt {


#define DT_P_MAX (DT_K_MAX + (DT_D_MAX - 1) * DT_K_MAX * DT_K_MAX)
#ifndef TREE_NT
#define TREE_NT 512               // threads of the workgroup
#endif
#define TREE_NW (TREE_NT / 64)    // its waves
#define COUNT_MAX 128             // largest level ranked by counting (beyond it the bucket cut is faster: measured)
#define BUCKET_CAP 64             // most candidates of one score bucket that are ranked one against the other

__device__ __forceinline__ u32 score_key(float s) { return ord32(s); }
#define KEY_NEG_INF 0x007FFFFFu   // key of -inf: a candidate that does not exist

// x / dv for 0 <= x < 8192 and 1 <= dv <= 1024 with inv = 1.0f / dv (any rounding within two ulp):
// (x + 0.5) / dv is at least 0.5 / dv away from every integer, far more than the product's error.
__device__ __forceinline__ int fdiv(int x, float inv) { return (int)(((float)x + 0.5f) * inv); }

struct Decoded {
    int level, slot, rank, row;
};
struct PoolShape {
    int k, kk;
    float inv_k, inv_kk;
};
__device__ __forceinline__ PoolShape pool_shape(int k) {
    PoolShape s;
    s.k = k; s.kk = k * k;
    s.inv_k = 1.0f / (float)k; s.inv_kk = 1.0f / (float)(k * k);
    return s;
}
// pool index -> (level, slot of the parent in its level's expanded set, rank in the parent's row, draft row)
__device__ __forceinline__ Decoded decode(int p, const PoolShape &s) {
    Decoded d;
    if (p < s.k) {
        d.level = 1; d.slot = 0; d.rank = p; d.row = 0;
    } else {
        const int q = p - s.k;
        const int l2 = fdiv(q, s.inv_kk), rem = q - l2 * s.kk;
        d.level = l2 + 2; d.slot = fdiv(rem, s.inv_k); d.rank = rem - d.slot * s.k;
        d.row = 1 + l2 * s.k + d.slot;
    }
    return d;
}

struct TreeLds {
    float score[DT_P_MAX];         // lp of a candidate, then its cumulative score
    float lp[DT_P_MAX];            // its own log-probability and token, kept for the emission: the
    int tok[DT_P_MAX];             // kernel then ends without another trip to memory
    int16_t node[DT_P_MAX];        // node number after the rerank, -1: not kept
    int8_t slot[DT_P_MAX];         // slot in its level's expanded set, -1: not expanded
    int exp[DT_D_MAX][DT_K_MAX];   // pool index of slot s of level l
    u32 key[2][COUNT_MAX];         // keys of the level being ranked by counting (levels alternate)
    int rank[2][COUNT_MAX];        // how many keys of the level lie above each (summed by LDS adds)
    u32 hist[4][256];              // one histogram per radix digit
    int wtot[TREE_NW];             // per-wave totals of the position scan
    u64 mem[BUCKET_CAP];           // (key, index) of the candidates in the bucket that holds the cut
    int memn;
};

// ---- radix selection ---------------------------------------------------------------------------------
// Key of the keep-th best of score[0..n), keep = min(keep_max, #viable): returns keep (uniform), thr and
// need_eq = how many candidates with key == thr belong to the chosen set.  Whole workgroup; ends
// with every thread past the last barrier it contains.
__device__ __forceinline__ int block_radix_cut(const float *score, int n, int keep_max, TreeLds &S, u32 &thr,
                                               int &need_eq) {
    const int tid = threadIdx.x, lane = lane_id();
    for (int i = tid; i < 4 * 256; i += TREE_NT) (&S.hist[0][0])[i] = 0u;
    __syncthreads();
    u32 prefix = 0;
    int above = 0, keep = 0;
    thr = 0xFFFFFFFFu;
    need_eq = 0;
#pragma unroll 1
    for (int p = 0; p < 4; ++p) {
        const int shift = 24 - 8 * p;
        for (int i = tid; i < n; i += TREE_NT) {
            const u32 key = score_key(score[i]);
            const bool in = key > KEY_NEG_INF && (p == 0 || (key >> (shift + 8)) == (prefix >> (shift + 8)));
            if (in) atomicAdd(&S.hist[p][(key >> shift) & 255u], 1u);
        }
        __syncthreads();
        // every wave: lane L holds bins 4(63-L) .. 4(63-L)+3, so an ascending lane scan walks the bins downwards
        const uint4 h = *(const uint4 *)&S.hist[p][4 * (63 - lane)];
        const int c = (int)(h.x + h.y + h.z + h.w);
        const int incl = wave_scan_incl_i32(c);
        if (p == 0) {
            keep = min(keep_max, __builtin_amdgcn_readlane(incl, 63));
            if (keep <= 0) return 0;
        }
        const int need = keep - above;  // rank of the wanted key among those sharing the digits found so far
        const u64 m = __ballot(incl >= need);
        const int ls = __ffsll((long long)m) - 1;
        int acc = __builtin_amdgcn_readlane(incl - c, ls);
        const int h3 = __builtin_amdgcn_readlane((int)h.w, ls), h2 = __builtin_amdgcn_readlane((int)h.z, ls),
                  h1 = __builtin_amdgcn_readlane((int)h.y, ls);
        int dg;
        if (acc + h3 >= need) dg = 3;
        else {
            acc += h3;
            if (acc + h2 >= need) dg = 2;
            else {
                acc += h2;
                if (acc + h1 >= need) dg = 1;
                else { acc += h1; dg = 0; }
            }
        }
        above += acc;
        prefix |= (u32)(4 * (63 - ls) + dg) << shift;
        const int hd = dg == 3 ? h3 : dg == 2 ? h2 : dg == 1 ? h1 : __builtin_amdgcn_readlane((int)h.x, ls);
        if (keep - above == hd && p < 3 && prefix != 0u) {
            // every key that shares these digits belongs to the set: cut just below the smallest of them
            thr = prefix - 1u;
            need_eq = 0;
            return keep;
        }
    }
    thr = prefix;
    need_eq = keep - above;
    return keep;
}

// Positions in ascending index of the chosen candidates of score[0..n): those above thr and the first
// need_eq of those equal to it; f(index, position).  Returns how many were chosen (uniform).  Whole
// workgroup; one barrier inside, none after the calls of f.
template <typename F>
__device__ __forceinline__ int block_enumerate(const float *score, int n, u32 thr, int need_eq, TreeLds &S, F f) {
    const int tid = threadIdx.x, lane = lane_id(), w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int C = (n + TREE_NT - 1) / TREE_NT;  // consecutive candidates per thread
    const int i0 = tid * C;
    int own = 0;  // low half: keys above thr, high half: keys equal to thr
    for (int c = 0; c < C; ++c) {
        const int i = i0 + c;
        const u32 kv = score_key(score[min(i, n - 1)]);
        const u32 key = i < n ? kv : 0u;
        own += (key > thr ? 1 : 0) + (key == thr ? 0x10000 : 0);
    }
    const int incl = wave_scan_incl_i32(own);
    if (lane == 63) S.wtot[w] = incl;
    __syncthreads();
    int base = 0, total = 0;
#pragma unroll
    for (int v = 0; v < TREE_NW; ++v) {
        const int t = S.wtot[v];
        base += v < w ? t : 0;
        total += t;
    }
    int before = base + incl - own;
    for (int c = 0; c < C; ++c) {
        const int i = i0 + c;
        const u32 kv = score_key(score[min(i, n - 1)]);
        const u32 key = i < n ? kv : 0u;
        const int gt = before & 0xFFFF, eq = before >> 16;
        if (key > thr || (key == thr && eq < need_eq)) f(i, gt + min(eq, need_eq));
        before += (key > thr ? 1 : 0) + (key == thr ? 0x10000 : 0);
    }
    return (total & 0xFFFF) + min(total >> 16, need_eq);
}

// Positions of flagged candidates: thread t owns candidates [t C, t C + C) and their flags (bit c of
// `flags`); f(index, position) for every flagged one, positions counted in ascending index.  Returns
// the number of flagged candidates (uniform).  Whole workgroup; one barrier inside.
template <typename F>
__device__ __forceinline__ int block_positions(int C, u32 flags, TreeLds &S, F f) {
    const int tid = threadIdx.x, lane = lane_id(), w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int own = __popc(flags);
    const int incl = wave_scan_incl_i32(own);
    if (lane == 63) S.wtot[w] = incl;
    __syncthreads();
    int base = 0, total = 0;
#pragma unroll
    for (int v = 0; v < TREE_NW; ++v) {
        const int t = S.wtot[v];
        base += v < w ? t : 0;
        total += t;
    }
    int pos = base + incl - own;
    for (int c = 0; c < C; ++c)
        if ((flags >> c) & 1u) f(tid * C + c, pos++);
    return total;
}

// The keep_max best of score[0..n) (fewer if fewer are viable), visited in ascending index.  Whole
// workgroup; the calls of f are followed by a barrier.
//
// Scores are log-probabilities, so floor(-8 score), capped at 255, spreads them over buckets that are
// ordered like the scores.  One histogram and one scan name the bucket that holds the cut; the few
// candidates inside it are ranked one against the other by (key desc, index asc), everything in a better
// bucket is taken.  A bucket with more than BUCKET_CAP candidates (many equal scores, or scores below
// -32) goes through the radix selection instead.  CT: candidates per thread when known at compile time
// (their scores then stay in registers), 0: any number up to 32.
// (clamped as a float first: converting a float beyond the int range would be undefined)
__device__ __forceinline__ int score_bucket(float sc) { return max((int)fminf(sc * -8.0f, 255.0f), 0); }
__device__ __forceinline__ u64 member_key(u32 key, int i) { return ((u64)key << 32) | (u32)(0x7FFFFFFF - i); }

template <int CT, typename F>
__device__ __forceinline__ int block_select_t(const float *score, int n, int keep_max, TreeLds &S, F f) {
    const int tid = threadIdx.x, lane = lane_id();
    const int C = CT > 0 ? CT : (n + TREE_NT - 1) / TREE_NT;  // consecutive candidates per thread
    constexpr int CR = CT > 0 ? CT : 1;
    float sc[CR];
    if (tid < 256) S.hist[0][tid] = 0u;
    if (tid < BUCKET_CAP) S.mem[tid] = 0ull;
    if (tid == 0) S.memn = 0;
    __syncthreads();
    if (CT > 0) {
#pragma unroll
        for (int c = 0; c < CR; ++c) sc[c] = score[min(tid * CT + c, n - 1)];
#pragma unroll
        for (int c = 0; c < CR; ++c) {
            if (tid * CT + c >= n) sc[c] = -INFINITY;
            if (sc[c] > -INFINITY) atomicAdd(&S.hist[0][score_bucket(sc[c])], 1u);
        }
    } else {
        for (int c = 0; c < C; ++c) {
            const int i = tid * C + c;
            const float v = score[min(i, n - 1)];
            if (i < n && v > -INFINITY) atomicAdd(&S.hist[0][score_bucket(v)], 1u);
        }
    }
    __syncthreads();
    // every wave: lane L holds buckets 4L .. 4L+3, best scores first
    const uint4 h = *(const uint4 *)&S.hist[0][4 * lane];
    const int c4 = (int)(h.x + h.y + h.z + h.w);
    const int incl = wave_scan_incl_i32(c4);
    const int keep = min(keep_max, __builtin_amdgcn_readlane(incl, 63));
    if (keep <= 0) return 0;
    const int ls = __ffsll((long long)__builtin_amdgcn_ballot_w64(incl >= keep)) - 1;
    int above = __builtin_amdgcn_readlane(incl - c4, ls);
    const int h0 = __builtin_amdgcn_readlane((int)h.x, ls), h1 = __builtin_amdgcn_readlane((int)h.y, ls),
              h2 = __builtin_amdgcn_readlane((int)h.z, ls), h3 = __builtin_amdgcn_readlane((int)h.w, ls);
    int dg, hB;
    if (above + h0 >= keep) { dg = 0; hB = h0; }
    else {
        above += h0;
        if (above + h1 >= keep) { dg = 1; hB = h1; }
        else {
            above += h1;
            if (above + h2 >= keep) { dg = 2; hB = h2; }
            else { above += h2; dg = 3; hB = h3; }
        }
    }
    const int B = 4 * ls + dg;
    const int need = keep - above;  // how many of bucket B belong to the set: 1 .. hB
    if (hB > BUCKET_CAP) {
        u32 thr;
        int need_eq;
        if (block_radix_cut(score, n, keep_max, S, thr, need_eq) <= 0) return 0;
        const int taken = block_enumerate(score, n, thr, need_eq, S, f);
        __syncthreads();
        return taken;
    }
    // flags of the candidates in better buckets, and of those in bucket B
    u32 sure = 0u, inb = 0u;
    if (CT > 0) {
#pragma unroll
        for (int c = 0; c < CR; ++c) {
            const int bk = score_bucket(sc[c]);
            const bool ok = sc[c] > -INFINITY;
            sure |= (ok && bk < B ? 1u : 0u) << c;
            inb |= (ok && bk == B ? 1u : 0u) << c;
        }
    } else {
        for (int c = 0; c < C; ++c) {
            const int i = tid * C + c;
            const float v = score[min(i, n - 1)];
            const int bk = score_bucket(v);
            const bool ok = i < n && v > -INFINITY;
            sure |= (ok && bk < B ? 1u : 0u) << c;
            inb |= (ok && bk == B ? 1u : 0u) << c;
        }
    }
    if (need < hB) {  // the cut runs through bucket B: its members rank themselves
        auto key_of = [&](int c) { return member_key(score_key(CT > 0 ? sc[CT > 0 ? c : 0] : score[tid * C + c]), tid * C + c); };
        if (CT > 0) {
#pragma unroll
            for (int c = 0; c < CR; ++c)
                if ((inb >> c) & 1u) S.mem[atomicAdd(&S.memn, 1)] = key_of(c);
        } else {
            for (int c = 0; c < C; ++c)
                if ((inb >> c) & 1u) S.mem[atomicAdd(&S.memn, 1)] = key_of(c);
        }
        __syncthreads();
        if (inb) {
            // entries past the hB members are zero and rank below every member
            auto rank_of = [&](u64 mine) {
                int rank = 0;
                for (int j0 = 0; j0 < hB; j0 += 8) {
                    u64 o[8];
#pragma unroll
                    for (int j = 0; j < 8; ++j) o[j] = S.mem[j0 + j];
#pragma unroll
                    for (int j = 0; j < 8; ++j) rank += o[j] > mine ? 1 : 0;
                }
                return rank;
            };
            if (CT > 0) {
#pragma unroll
                for (int c = 0; c < CR; ++c)
                    if (((inb >> c) & 1u) && rank_of(key_of(c)) < need) sure |= 1u << c;
            } else {
                for (int c = 0; c < C; ++c)
                    if (((inb >> c) & 1u) && rank_of(key_of(c)) < need) sure |= 1u << c;
            }
        }
    } else {
        sure |= inb;
    }
    const int taken = block_positions(C, sure, S, f);
    __syncthreads();
    return taken;
}
template <typename F>
__device__ __forceinline__ int block_select(const float *score, int n, int keep_max, TreeLds &S, F f) {
    if (n <= TREE_NT) return block_select_t<1>(score, n, keep_max, S, f);
    if (n <= 2 * TREE_NT) return block_select_t<2>(score, n, keep_max, S, f);
    return block_select_t<0>(score, n, keep_max, S, f);
}

// c_i += (o_i > mine) for the four keys of o.  Written out so that the four compares go to four scalar
// register pairs and the four adds-with-carry follow them: no result is needed by the next instruction,
// where the compiler's own sequence (compare into VCC, add from VCC) waits on every pair.
__device__ __forceinline__ void count_above4(const uint4 o, u32 mine, int &c0, int &c1, int &c2, int &c3) {
    u64 m0, m1, m2, m3;
    asm(
        "v_cmp_gt_u32_e64 %[m0], %[ox], %[mine]\n\t"
        "v_cmp_gt_u32_e64 %[m1], %[oy], %[mine]\n\t"
        "v_cmp_gt_u32_e64 %[m2], %[oz], %[mine]\n\t"
        "v_cmp_gt_u32_e64 %[m3], %[ow], %[mine]\n\t"
        "v_addc_co_u32_e64 %[c0], %[m0], 0, %[c0], %[m0]\n\t"
        "v_addc_co_u32_e64 %[c1], %[m1], 0, %[c1], %[m1]\n\t"
        "v_addc_co_u32_e64 %[c2], %[m2], 0, %[c2], %[m2]\n\t"
        "v_addc_co_u32_e64 %[c3], %[m3], 0, %[c3], %[m3]\n\t"
        : [c0] "+v"(c0), [c1] "+v"(c1), [c2] "+v"(c2), [c3] "+v"(c3), [m0] "=&s"(m0), [m1] "=&s"(m1),
          [m2] "=&s"(m2), [m3] "=&s"(m3)
        : [ox] "v"(o.x), [oy] "v"(o.y), [oz] "v"(o.z), [ow] "v"(o.w), [mine] "v"(mine));
}

// ---- ranking a level by counting ---------------------------------------------------------------------
// key[0 .. 64 G) holds the keys of the level's n candidates (zero beyond n), G = ceil(n / 64) <= 2, and
// rank[0 .. 64 G) is zero.  Wave w counts, for the 64 candidates of group w % G, the keys above
// theirs within slice w / G of the level, and adds that to their rank.  Ties are counted as "not above",
// so candidates of equal key share a rank; the caller detects a tie that straddles the cut by the size
// of the chosen set.
template <int G>
__device__ __forceinline__ void level_count(const u32 *key, int *rank) {
    static_assert(G == 1 || G == 2, "groups of 64 candidates");
    constexpr int H = G == 1 ? TREE_NW : TREE_NW / 2;  // slices
    constexpr int PER = 64 * G / H;                                           // keys per slice (padding included)
    const int lane = lane_id(), w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (w < G * H) {
        const int g = w % G, h = w / G;
        const u32 mine = key[g * 64 + lane];
        const uint4 *other = (const uint4 *)&key[h * PER];
        int c0 = 0, c1 = 0, c2 = 0, c3 = 0;
#pragma unroll
        for (int j = 0; j < PER / 4; ++j) count_above4(other[j], mine, c0, c1, c2, c3);
        atomicAdd(&rank[g * 64 + lane], (c0 + c1) + (c2 + c3));
    }
}
// Every wave by itself, after the barrier that follows level_count: the chosen set of the level (rank
// below k among the viable candidates; all of them when n <= k, rank then is not read), positions in
// ascending index.  Returns the size of the set, or -1 when equal keys straddle the cut (nothing has
// been written then).  f(index, position) is called by every wave for every chosen candidate.
template <int G, typename F>
__device__ __forceinline__ int level_choose(const u32 *key, const int *rank, int n, int k, F f) {
    const int lane = lane_id();
    u64 m[G];
    int chosen = 0, viable = 0;
    u32 ky[G];
    int rk[G];
#pragma unroll
    for (int q = 0; q < G; ++q) {  // all loads first
        ky[q] = key[q * 64 + lane];
        rk[q] = n <= k ? 0 : rank[q * 64 + lane];
    }
#pragma unroll
    for (int q = 0; q < G; ++q) {
        const bool ok = ky[q] > KEY_NEG_INF;
        m[q] = __builtin_amdgcn_ballot_w64(ok && rk[q] < k);
        viable += __popcll(__builtin_amdgcn_ballot_w64(ok));
        chosen += __popcll(m[q]);
    }
    if (chosen != min(k, viable)) return -1;
    int before = 0;
#pragma unroll
    for (int q = 0; q < G; ++q) {
        if ((m[q] >> lane) & 1ull) f(q * 64 + lane, before + (int)lanes_below(m[q]));
        before += __popcll(m[q]);
    }
    return chosen;
}

__global__ __launch_bounds__(TREE_NT) void tree_kernel(TreeArgs a) {
    const int b = blockIdx.x, tid = threadIdx.x;
    // Row results of sequence b: rows b * seq_rows .. (the same block layout for the one-shot build and
    // the level-at-a-time state), so nothing about them depends on the sequence's parameters.  The first
    // 64 rows are requested before the parameters have arrived: one trip to memory instead of two.
    const int64_t r0 = (int64_t)b * a.seq_rows;
    const float *tv = a.top_val + r0 * DT_K_MAX;
    const int32_t *ti = a.top_id + r0 * DT_K_MAX;
    const float *lse = a.lse + r0;
    constexpr int EARLY = 4;  // entries per thread read ahead: rows 0 .. EARLY * TREE_NT / DT_K_MAX - 1
    float ev[EARLY], el[EARLY];
    int et[EARLY];
#pragma unroll
    for (int j = 0; j < EARLY; ++j) {
        const int e = tid + j * TREE_NT;  // entry (row e / 32, rank e % 32)
        ev[j] = tv[e];
        et[j] = ti[e];
        el[j] = lse[e / DT_K_MAX];
    }
    const dt_params prm = a.params[b];
    // one-shot build: rows past the span the sequence owns were never reduced; they count as rows
    // without a viable token (the level-at-a-time state has no such span: its rows arrive level by level)
    const int64_t span = a.row_off ? a.row_off[b + 1] - a.row_off[b] : (int64_t)DT_STATE_ROWS;
    const int TT = min(max(prm.TT, 1), a.TT_cap), d = min(max(prm.d, 1), DT_D_MAX);
    const int k = min(max(prm.k, 1), min(DT_K_MAX, a.V));
    const int xl = a.expand_level;  // > 0: only the nodes of level xl that are expanded next
    const int64_t o = (int64_t)b * a.TT_cap;
    const PoolShape ps = pool_shape(k);
    const int kk = k * k;

    extern __shared__ __attribute__((aligned(16))) unsigned char s_dyn[];  // 116 KB: more than a static array may hold
    TreeLds &S = *reinterpret_cast<TreeLds *>(s_dyn);

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
    // Candidates through level d, or through level xl when only that level's choice is wanted (the
    // rows of deeper levels do not exist yet).  Every candidate's own log-probability is known up front: the draft row that would
    // produce pool index p is fixed by p alone (only its parent is decided later).  Park
    // lp in the score array; the level loop turns it into the cumulative score in place.
    // Entry (row, rank) with rank < k is candidate p = rank (row 0) or k + (row - 1) k + rank.
    const int R = xl > 0 ? 1 + (xl - 1) * k : 1 + (d - 1) * k;  // rows that hold candidates
    const int owned = (int)min(max(span, (int64_t)0), (int64_t)DT_STATE_ROWS);
    auto place = [&](int e, float v, int token, float row_lse) {
        const int row = e / DT_K_MAX, rank = e % DT_K_MAX;
        if (row < R && rank < k) {
            const int p = row == 0 ? rank : k + (row - 1) * k + rank;
            const float own = v - row_lse;
            const float lp = v > -INFINITY && row < owned ? own : -INFINITY;
            S.score[p] = lp;
            S.lp[p] = own;
            S.tok[p] = token;
            S.node[p] = -1;
            S.slot[p] = -1;
            if (row == 0) S.key[1][p] = score_key(lp);  // level 1 is chosen first
        }
    };
#pragma unroll
    for (int j = 0; j < EARLY; ++j) place(tid + j * TREE_NT, ev[j], et[j], el[j]);
    for (int e = tid + EARLY * TREE_NT; e < R * DT_K_MAX; e += TREE_NT) place(e, tv[e], ti[e], lse[e / DT_K_MAX]);
    if (tid < 64 && tid >= k) S.key[1][tid] = 0u;
    for (int t = tid; t < COUNT_MAX; t += TREE_NT) S.rank[0][t] = 0;
    __syncthreads();

    // ---- expansion, level by level -----------------------------------------------------------
    int p_end = k;  // pool indices below p_end hold real scores (levels computed so far)
    const int l_end = xl > 0 ? xl + 1 : d;
    // token count of Algorithm 2's expansion loop: the root plus the viable candidates proposed so far
    int tok_count = a.early_stop ? 1 + __syncthreads_count(tid < k && S.score[tid] > -INFINITY) : 0;
    for (int l = 1; l < l_end; ++l) {
        if (a.early_stop && tok_count >= TT) break;  // uniform: no further level is expanded
        const int lo = l == 1 ? 0 : k + (l - 2) * kk;
        const int n = l == 1 ? k : kk;
        int *exp_l = S.exp[l];
        auto put = [&](int i, int pos) {
            exp_l[pos] = lo + i;
            S.slot[lo + i] = (int8_t)pos;
        };
        int n_exp = -1;
        if (n <= COUNT_MAX) {
            // (after the barrier that published the keys) count, publish the ranks, choose in every wave
            const u32 *key = S.key[l & 1];
            int *rank = S.rank[l & 1];
            const int G = (n + 63) >> 6;
            if (n > k) {  // otherwise every viable candidate is chosen
                if (G == 1) level_count<1>(key, rank);
                else level_count<2>(key, rank);
                __syncthreads();
            }
            if (G == 1) n_exp = level_choose<1>(key, rank, n, k, put);
            else n_exp = level_choose<2>(key, rank, n, k, put);
        }
        if (n_exp < 0) n_exp = block_select(S.score + lo, n, k, S, put);
        if (l == xl) {
            // ---- what the draft model is handed for its next pass: node s of the chosen set ----------
            if (tid < n_exp) {
                const int pi = exp_l[tid];
                const Decoded dc = decode(pi, ps);
                const int64_t e = (int64_t)b * DT_K_MAX + tid;
                a.exp_token[e] = S.tok[pi];
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
                // the slot of an expanded candidate is read from S.exp, which every wave wrote for itself
                int lv = l, sl = dc.slot;  // level of the current node, slot of its parent
                for (int guard = 0; guard < DT_D_MAX && lv > 1; ++guard) {
                    set(1 + (lv - 2) * k + sl);
                    const Decoded dp = decode(S.exp[lv - 1][sl], ps);
                    --lv;
                    sl = dp.slot;
                }
                a.exp_mask[e * 4] = m0; a.exp_mask[e * 4 + 1] = m1;
                a.exp_mask[e * 4 + 2] = m2; a.exp_mask[e * 4 + 3] = m3;
            }
            if (tid == 0) { a.n_expand[b] = n_exp; a.state_n_exp[b] = n_exp; }
            return;
        }
        if (n_exp == 0) break;
        // next level: score = score[parent] + lp, and the keys for its ranking.  exp_l is read by the
        // wave that wrote it (every wave writes the whole set) or after block_select's barrier.
        const int nlo = k + (l - 1) * kk;
        const int npad = kk <= COUNT_MAX ? ((kk + 63) & ~63) : kk;
        int fresh = 0;  // viable candidates this thread has just scored (at most two: kk <= 2 TREE_NT)
        for (int t = tid; t < npad; t += TREE_NT) {
            const int tc = min(t, kk - 1);
            const int s = fdiv(tc, ps.inv_k);
            // slots beyond the expanded set own no node: their candidates do not exist
            const float par = S.score[exp_l[min(s, n_exp - 1)]], own = S.score[nlo + tc];
            const float sc = s < n_exp ? par + own : -INFINITY;
            if (t < kk) S.score[nlo + t] = sc;
            fresh += t < kk && sc > -INFINITY;
            if (kk <= COUNT_MAX) {  // the other pair of arrays: slower waves may still be choosing from this level's
                S.key[(l + 1) & 1][t] = t < kk ? score_key(sc) : 0u;
                S.rank[(l + 1) & 1][t] = 0;
            }
        }
        p_end = nlo + kk;
        if (a.early_stop) tok_count += __syncthreads_count(fresh >= 1) + __syncthreads_count(fresh >= 2);
        else __syncthreads();
    }

    if (xl > 0) {  // an earlier level had nothing viable to expand, or the token count ended the expansion
        if (tid == 0) { a.n_expand[b] = 0; a.state_n_exp[b] = 0; }
        return;
    }
    __syncthreads();  // the level loop may have been left right after a wave-local choice

    // ---- rerank: the TT-1 best of the whole pool ----------------------------------------------
    const int keep = block_select(S.score, p_end, TT - 1, S, [&](int i, int pos) { S.node[i] = (int16_t)(pos + 1); });
    if (tid == 0) a.n_nodes[b] = keep + 1;

    // ---- emission -------------------------------------------------------------------------------
    for (int p = tid; p < p_end; p += TREE_NT) {
        const int n = S.node[p];
        if (n < 0) continue;
        const Decoded dc = decode(p, ps);
        int par_pool = dc.level == 1 ? -1 : S.exp[dc.level - 1][dc.slot];
        a.tokens[o + n] = S.tok[p];
        a.parents[o + n] = par_pool < 0 ? 0 : max((int)S.node[par_pool], 0);
        a.depth[o + n] = dc.level;
        a.score[o + n] = S.score[p];
        a.logp[o + n] = S.lp[p];
        a.src_row[o + n] = S.slot[p] >= 0 ? 1 + (dc.level - 1) * k + S.slot[p] : -1;
        u64 m0 = 1ull, m1 = 0ull;  // the root
        int nn = n, pp = par_pool;
        for (int guard = 0; guard <= DT_D_MAX; ++guard) {
            if (nn < 64) m0 |= 1ull << nn; else m1 |= 1ull << (nn - 64);
            if (pp < 0) break;
            nn = max((int)S.node[pp], 0);
            const Decoded dp = decode(pp, ps);
            pp = dp.level == 1 ? -1 : S.exp[dp.level - 1][dp.slot];
        }
        a.anc_mask[(o + n) * DT_MASK_WORDS] = m0;
        a.anc_mask[(o + n) * DT_MASK_WORDS + 1] = m1;
    }
}


// LDS beyond 64 KB has to be asked for, once per device (dt_init)
hipError_t tree_init() {
    return hipFuncSetAttribute((const void *)tree_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sizeof(TreeLds));
}

hipError_t tree_launch(const TreeArgs &a, hipStream_t st) {
    if (a.batch <= 0) return hipSuccess;
    launch_kernel(KID_TREE, st, tree_kernel, dim3(a.batch), dim3(TREE_NT), sizeof(TreeLds), a);
    return hipGetLastError();
}

}  // namespace dt
