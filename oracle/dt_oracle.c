/*
 * dt_oracle.c -- plain CPU oracle for one draft-tree speculative step.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, by-eye-checkable statement of
 * what the GPU library must compute.  It shares no code, header, table or helper
 * with the HIP path and the product never calls it: only the tests, the smoke
 * check and the CPU-baseline leg of the benchmark do.
 *
 * What it follows (paper: "Speculative Sampling with Reinforcement Learning"):
 *   - Section 3.2 "Draft Tree Expansion": layer-wise expansion, at each layer the
 *     top-k nodes by global acceptance value V_i (product of draft confidences
 *     along the path, kept here as a sum of log-probabilities) are expanded.
 *   - Section 3.2 "Confidence-Based Candidate Reranking": after expansion every
 *     token of the tree is re-ranked by V_i and the best TT go to verification.
 *   - Appendix B, Algorithm 2, the drafting block (expansion loop, then rerank and
 *     verify); Section 4 "Action Space": (TT, d, k) are upper limits.
 *   - Section 3.2 "Verification Phase" / "Acceptance Criterion": the target scores
 *     every tree token conditioned on its own path (tree attention); a draft token
 *     is accepted with probability min(1, P_T / P_d); Section 3.1: greedy decoding
 *     takes the arg max, which is the temperature-0 limit used in the experiments.
 *
 * Readings taken where the paper is silent (all listed in the design notes):
 *   TT counts the root; d = number of draft levels below the root; the TT limit
 *   binds at the rerank only; confidence = draft softmax probability; ties are
 *   broken by (logit desc, token id asc) inside a row and by (score desc, pool
 *   index asc) across rows; expanded nodes are handed their draft rows in
 *   ascending pool index; stochastic acceptance is applied per node with its own
 *   uniform, then the deepest all-accepted path wins (ties: lowest node index).
 *
 * Arithmetic: inputs are upcast exactly; sums (log-sum-exp, dot products, CDF) are
 * accumulated in double; log-probabilities and scores are rounded to float exactly
 * once per operation: lp = fl32(x - lse), score = fl32(score[parent] + lp).
 *
 *   - Appendix, "System Profiling and Overhead Analysis": after verification the
 *     "input update" brings the KV cache to the state the next step starts from --
 *     the accepted tokens stay, the rejected ones are discarded, and positions
 *     continue from the new length (ref_commit_rows).
 *   - Section 3.3 "Addressing the Challenges with Re-SpS" and Algorithm 1: the state is the
 *     concatenation of three hidden-state vectors, the policy is a small MLP (Appendix A,
 *     "Network Architecture"), a chosen action is reused for N decision points; Appendix A,
 *     "Action Space in Implementation": the table of actions (ref_action_table,
 *     ref_policy_logits, ref_policy_step); Section 3.1 "Reward Function" and the averaged reward
 *     of Section 3.3 (ref_reward_step).
 *
 * Pins: every function here is pinned by tests (library sorts, closed forms,
 * brute-force enumeration of token strings and of root-to-leaf paths, float64
 * dense-mask attention, Philox known-answer vectors).  Not pinned: that the
 * per-node stochastic rule preserves the target distribution (it is not claimed).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define REF_OK 0
#define REF_ERR_ARG (-1)
#define REF_ERR_INTERNAL (-9)

#define REF_F32 0
#define REF_BF16 1

#define REF_TT_MAX 128
#define REF_D_MAX 8
#define REF_K_MAX 32

/* ---------------------------------------------------------------- helpers */

static float elem(const void *base, int dtype, int64_t idx)
{
    if (dtype == REF_F32)
        return ((const float *)base)[idx];
    uint32_t u = (uint32_t)((const uint16_t *)base)[idx] << 16; /* bf16 -> f32, exact */
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* round-to-nearest-even float -> bf16 -> float (finite inputs) */
static float round_bf16(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    u = (u + 0x7FFFu + ((u >> 16) & 1u)) & 0xFFFF0000u;
    memcpy(&f, &u, 4);
    return f;
}

typedef struct {
    float x;
    int32_t id;
} item_t;

/* total order of a row: larger logit first, then smaller token id */
static int cmp_item(const void *pa, const void *pb)
{
    const item_t *a = (const item_t *)pa, *b = (const item_t *)pb;
    if (a->x > b->x) return -1;
    if (a->x < b->x) return 1;
    return (a->id > b->id) - (a->id < b->id);
}

/* ------------------------------------------------- A1: row top-k + row LSE */

/*
 * One vocabulary row (Algorithm 2: "select highest V_i children"): the k largest
 * logits under (logit desc, id asc), and lse = log sum_v exp(x_v).
 * Entries equal to -inf are not viable: their slot gets value -inf and id -1.
 * Returns the number of viable entries among the k (or a negative error).
 */
int ref_row_reduce(const void *row, int dtype, int V, int k,
                   float *top_val, int32_t *top_id, float *lse_out)
{
    if (!row || V < 1 || k < 1 || k > V) return REF_ERR_ARG;
    item_t *it = (item_t *)malloc(sizeof(item_t) * (size_t)V);
    if (!it) return REF_ERR_INTERNAL;
    float m = -INFINITY;
    for (int v = 0; v < V; ++v) {
        it[v].x = elem(row, dtype, v);
        it[v].id = v;
        if (it[v].x > m) m = it[v].x;
    }
    float lse = -INFINITY;
    if (m > -INFINITY) {
        double s = 0.0;
        for (int v = 0; v < V; ++v) s += exp((double)it[v].x - (double)m);
        lse = (float)((double)m + log(s));
    }
    qsort(it, (size_t)V, sizeof(item_t), cmp_item);
    int viable = 0;
    for (int r = 0; r < k; ++r) {
        if (it[r].x > -INFINITY) {
            if (top_val) top_val[r] = it[r].x;
            if (top_id) top_id[r] = it[r].id;
            ++viable;
        } else {
            if (top_val) top_val[r] = -INFINITY;
            if (top_id) top_id[r] = -1;
        }
    }
    if (lse_out) *lse_out = lse;
    free(it);
    return viable;
}

/* Same, for n_rows rows laid out with a row stride (in elements). */
int ref_topk_rows(const void *logits, int dtype, int64_t n_rows, int V, int64_t row_stride, int k,
                  float *top_val, int32_t *top_id, float *lse)
{
    if (!logits || n_rows < 0 || row_stride < V) return REF_ERR_ARG;
    int esz = dtype == REF_F32 ? 4 : 2;
    int rc = REF_OK;
#pragma omp parallel for schedule(dynamic)
    for (int64_t r = 0; r < n_rows; ++r) {
        const char *row = (const char *)logits + r * row_stride * esz;
        int v = ref_row_reduce(row, dtype, V, k, top_val + r * k, top_id + r * k, lse + r);
        if (v < 0) rc = v;
    }
    return rc;
}

/* ------------------------------------------ A2-A4: expansion, rerank, emit */

typedef struct {
    int viable;
    float score;     /* cumulative log-probability root -> this candidate */
    float lp;        /* its own draft log-probability */
    int32_t tok;
    int parent_pool; /* pool index of the parent candidate, -1 = root */
    int level;       /* 1..d */
    int from_row;    /* draft row whose top-k produced it */
    int own_row;     /* draft row it was handed when expanded, else -1 */
    int own_slot;    /* its slot in its level's expanded set, else -1 */
} cand_t;

typedef struct {
    float score;
    int idx;
} key_t_;

/* total order across rows: larger score first, then smaller pool index */
static int cmp_key(const void *pa, const void *pb)
{
    const key_t_ *a = (const key_t_ *)pa, *b = (const key_t_ *)pb;
    if (a->score > b->score) return -1;
    if (a->score < b->score) return 1;
    return (a->idx > b->idx) - (a->idx < b->idx);
}

/*
 * Keep the `keep` best of the viable candidates pool[lo..hi).  kept[] (indexed by
 * pool index) is set to 1 for them.  *margin is lowered to the smallest score gap
 * between a kept and a dropped candidate that come from different draft rows (the
 * only comparisons whose outcome depends on the rounding of a row's lse).
 */
static int select_best(const cand_t *pool, int lo, int hi, int keep, unsigned char *kept, float *margin)
{
    int n = 0;
    key_t_ *keys = (key_t_ *)malloc(sizeof(key_t_) * (size_t)(hi - lo + 1));
    if (!keys) return REF_ERR_INTERNAL;
    for (int i = lo; i < hi; ++i)
        if (pool[i].viable) {
            keys[n].score = pool[i].score;
            keys[n].idx = i;
            ++n;
        }
    qsort(keys, (size_t)n, sizeof(key_t_), cmp_key);
    if (keep > n) keep = n;
    for (int a = 0; a < keep; ++a) kept[keys[a].idx] = 1;
    for (int a = 0; a < keep; ++a)
        for (int b = keep; b < n; ++b)
            if (pool[keys[a].idx].from_row != pool[keys[b].idx].from_row) {
                float gap = keys[a].score - keys[b].score;
                if (gap < *margin) *margin = gap;
            }
    free(keys);
    return keep;
}

/*
 * Build the draft tree of one sequence from its draft-logit rows.
 *
 * rows: row 0 is the root's next-token row; row 1 + (l-1)*k + s belongs to the
 *       s-th expanded node (ascending pool index) of level l, l = 1..d-1.
 * Outputs, node order = root, then kept candidates in ascending pool index:
 *   tokens, parents (node index, root -1), depth, score, logp, src_row (the row a
 *   node was handed, -1 if never expanded), anc_mask[node][W] with W = ceil(TT_cap/64)
 *   (bit j set iff j is the node itself or one of its ancestors), n_nodes,
 *   min_margin (see select_best; +inf if no such comparison occurred).
 * Optional (all three NULL or all three given), what a draft model sitting between the levels
 * is told after level l = 1..d-1 (Algorithm 2: the nodes chosen at a level are the draft
 * model's next inputs), indexed [l*REF_K_MAX + slot]:
 *   exp_count[l]     number of nodes of level l that are expanded (exp_count[0] = 0)
 *   exp_tok          their tokens, in slot order (= ascending pool index)
 *   exp_parent_slot  slot of the parent in level l-1's expanded set (-1: the root)
 *   exp_mask[..][4]  draft-side tree mask over draft rows: bit r set iff draft row r belongs to
 *                    the node itself or to one of its ancestors (row 0 = the root)
 * early_stop != 0: the token-count exit of Algorithm 2's expansion loop.  token_count starts at 1
 *   (the root) and grows by the candidates each expansion proposes (the root's k, then up to k per
 *   expanded node); no further level is expanded once token_count >= TT.  Levels never expanded
 *   report exp_count = 0 and their rows are not read.  With early_stop == 0, TT binds only at the
 *   rerank (Section 3.2: the rerank sees every token of the finished tree).
 */
int ref_build_tree(const void *rows, int dtype, int V, int64_t row_stride, int n_rows_avail,
                   int TT, int d, int k, int32_t root_token, int TT_cap,
                   int32_t *n_nodes, int32_t *tokens, int32_t *parents, int32_t *depth,
                   float *score, float *logp, int32_t *src_row, uint64_t *anc_mask,
                   float *min_margin, int32_t *exp_count, int32_t *exp_tok, int32_t *exp_parent_slot,
                   uint64_t *exp_mask, int early_stop)
{
    if (!rows || !n_nodes || !tokens || !parents || !depth || !score || !logp || !src_row || !anc_mask)
        return REF_ERR_ARG;
    if (TT_cap < 1 || TT_cap > REF_TT_MAX || TT < 1 || TT > TT_cap) return REF_ERR_ARG;
    if (d < 1 || d > REF_D_MAX || k < 1 || k > REF_K_MAX || k > V) return REF_ERR_ARG;
    if (row_stride < V || n_rows_avail < 1 + (d - 1) * k) return REF_ERR_ARG;

    const int W = (TT_cap + 63) / 64;
    const int P = k + (d - 1) * k * k;
    const int esz = dtype == REF_F32 ? 4 : 2;
    float margin = INFINITY;
    int rc = REF_OK;

    cand_t *pool = (cand_t *)calloc((size_t)P, sizeof(cand_t));
    unsigned char *kept = (unsigned char *)calloc((size_t)P, 1);
    int *node_of = (int *)malloc(sizeof(int) * (size_t)P);
    float tv[REF_K_MAX];
    int32_t ti[REF_K_MAX];
    if (!pool || !kept || !node_of) { rc = REF_ERR_INTERNAL; goto done; }
    for (int i = 0; i < P; ++i) { pool[i].own_row = -1; pool[i].own_slot = -1; pool[i].parent_pool = -1; }
    if (exp_count) {
        if (!exp_tok || !exp_parent_slot || !exp_mask) { rc = REF_ERR_ARG; goto done; }
        for (int l = 0; l < REF_D_MAX; ++l) exp_count[l] = 0;
    }

    /* node 0: the root */
    tokens[0] = root_token; parents[0] = -1; depth[0] = 0; score[0] = 0.0f; logp[0] = 0.0f;
    src_row[0] = 0;
    for (int w = 0; w < W; ++w) anc_mask[w] = 0;
    anc_mask[0] = 1ull;
    *n_nodes = 1;

    if (TT > 1) {
        /* level 1: the root's row */
        float lse;
        int nv = ref_row_reduce(rows, dtype, V, k, tv, ti, &lse);
        if (nv < 0) { rc = nv; goto done; }
        for (int r = 0; r < nv; ++r) {
            cand_t *c = &pool[r];
            c->viable = 1; c->tok = ti[r]; c->lp = tv[r] - lse; c->score = c->lp;
            c->parent_pool = -1; c->level = 1; c->from_row = 0;
        }
        int lo = 0, hi = k; /* pool range of the current level */
        int token_count = 1 + nv; /* the root and the candidates proposed so far (Algorithm 2) */
        for (int l = 1; l < d; ++l) {
            /* Algorithm 2 leaves the expansion loop once the tree holds TT tokens; applied on request only */
            if (early_stop && token_count >= TT) break;
            /* choose the nodes of level l to expand: its k best by score */
            unsigned char *exp_flag = (unsigned char *)calloc((size_t)P, 1);
            if (!exp_flag) { rc = REF_ERR_INTERNAL; goto done; }
            int n_exp = select_best(pool, lo, hi, k, exp_flag, &margin);
            if (n_exp < 0) { free(exp_flag); rc = n_exp; goto done; }
            int nlo = k + (l - 1) * k * k, nhi = nlo + k * k;
            int slot = 0;
            for (int i = lo; i < hi; ++i) { /* ascending pool index -> slot -> draft row */
                if (!exp_flag[i]) continue;
                int row = 1 + (l - 1) * k + slot;
                pool[i].own_row = row;
                pool[i].own_slot = slot;
                if (exp_count) {
                    int e = l * REF_K_MAX + slot;
                    exp_tok[e] = pool[i].tok;
                    exp_parent_slot[e] = pool[i].parent_pool < 0 ? -1 : pool[pool[i].parent_pool].own_slot;
                    for (int w = 0; w < 4; ++w) exp_mask[(size_t)e * 4 + w] = 0;
                    exp_mask[(size_t)e * 4] = 1ull; /* the root's row */
                    for (int j = i; j >= 0; j = pool[j].parent_pool) /* the node and its ancestors */
                        exp_mask[(size_t)e * 4 + pool[j].own_row / 64] |= 1ull << (pool[j].own_row % 64);
                    exp_count[l] = slot + 1;
                }
                const char *rp = (const char *)rows + (int64_t)row * row_stride * esz;
                int nvr = ref_row_reduce(rp, dtype, V, k, tv, ti, &lse);
                if (nvr < 0) { free(exp_flag); rc = nvr; goto done; }
                for (int r = 0; r < nvr; ++r) {
                    cand_t *c = &pool[nlo + slot * k + r];
                    c->viable = 1; c->tok = ti[r]; c->lp = tv[r] - lse;
                    c->score = pool[i].score + c->lp;
                    c->parent_pool = i; c->level = l + 1; c->from_row = row;
                }
                token_count += nvr;
                ++slot;
            }
            free(exp_flag);
            if (n_exp == 0) break; /* no viable candidate to expand */
            lo = nlo; hi = nhi;
        }
        /* rerank the whole pool, keep the best TT-1 */
        int nk = select_best(pool, 0, P, TT - 1, kept, &margin);
        if (nk < 0) { rc = nk; goto done; }
        /* emit in ascending pool index */
        int n = 1;
        for (int i = 0; i < P; ++i) {
            node_of[i] = -1;
            if (!kept[i]) continue;
            int par = 0;
            if (pool[i].parent_pool >= 0) {
                par = node_of[pool[i].parent_pool];
                if (par < 0) { rc = REF_ERR_INTERNAL; goto done; } /* kept set not ancestor-closed */
            }
            node_of[i] = n;
            tokens[n] = pool[i].tok; parents[n] = par; depth[n] = pool[i].level;
            score[n] = pool[i].score; logp[n] = pool[i].lp; src_row[n] = pool[i].own_row;
            for (int w = 0; w < W; ++w) anc_mask[(size_t)n * W + w] = anc_mask[(size_t)par * W + w];
            anc_mask[(size_t)n * W + n / 64] |= 1ull << (n % 64);
            ++n;
        }
        *n_nodes = n;
    }
    if (min_margin) *min_margin = margin;
done:
    free(pool); free(kept); free(node_of);
    return rc;
}

/* ------------------------------------------------------ A5: tree attention */

/*
 * Tree-masked attention of one sequence, written out from its definition: node i,
 * query head h (kv head g = h / (Hq/Hkv)) attends to all L prefix keys and to the
 * tree keys j with bit j of anc_mask[i] set.
 *   q [N,Hq,D], k_tree/v_tree [N,Hkv,D] contiguous; prefix element (t,g,c) at
 *   t*stride_tok + g*stride_head + c.
 * If n_samples > 0 only the listed (node, head) pairs are computed and out is
 * [n_samples, D]; else out is [N,Hq,D].  out is float; for bf16 inputs it is
 * rounded to the bf16 grid (round to nearest even).
 */
int ref_tree_attention(int dtype, int Hq, int Hkv, int D, float scale,
                       const void *q, const void *k_tree, const void *v_tree, int N,
                       const void *k_prefix, const void *v_prefix, int L,
                       int64_t stride_tok, int64_t stride_head,
                       const uint64_t *anc_mask, int TT_cap,
                       const int32_t *sample_node, const int32_t *sample_head, int n_samples,
                       float *out)
{
    if (!q || !k_tree || !v_tree || !anc_mask || !out) return REF_ERR_ARG;
    if (L > 0 && (!k_prefix || !v_prefix)) return REF_ERR_ARG;
    if (Hq < 1 || Hkv < 1 || Hq % Hkv || D < 1 || N < 1 || N > TT_cap || TT_cap > REF_TT_MAX || L < 0)
        return REF_ERR_ARG;
    const int W = (TT_cap + 63) / 64, G = Hq / Hkv;
    const int64_t n_out = n_samples > 0 ? n_samples : (int64_t)N * Hq;
    int rc = REF_OK;
#pragma omp parallel for schedule(dynamic)
    for (int64_t o = 0; o < n_out; ++o) {
        int i = n_samples > 0 ? sample_node[o] : (int)(o / Hq);
        int h = n_samples > 0 ? sample_head[o] : (int)(o % Hq);
        if (i < 0 || i >= N || h < 0 || h >= Hq) { rc = REF_ERR_ARG; continue; }
        int g = h / G;
        int nkeys = L + N;
        double *s = (double *)malloc(sizeof(double) * (size_t)nkeys);
        double *acc = (double *)calloc((size_t)D, sizeof(double));
        if (!s || !acc) { rc = REF_ERR_INTERNAL; free(s); free(acc); continue; }
        double smax = -INFINITY;
        for (int t = 0; t < nkeys; ++t) {
            int visible = 1;
            if (t >= L) {
                int j = t - L;
                visible = (int)((anc_mask[(size_t)i * W + j / 64] >> (j % 64)) & 1ull);
            }
            if (!visible) { s[t] = -INFINITY; continue; }
            double dot = 0.0;
            for (int c = 0; c < D; ++c) {
                float kv = t < L ? elem(k_prefix, dtype, t * stride_tok + g * stride_head + c)
                                 : elem(k_tree, dtype, ((int64_t)(t - L) * Hkv + g) * D + c);
                dot += (double)elem(q, dtype, ((int64_t)i * Hq + h) * D + c) * (double)kv;
            }
            s[t] = (double)scale * dot;
            if (s[t] > smax) smax = s[t];
        }
        double denom = 0.0;
        for (int t = 0; t < nkeys; ++t) {
            if (s[t] == -INFINITY) continue;
            double p = exp(s[t] - smax);
            denom += p;
            for (int c = 0; c < D; ++c) {
                float vv = t < L ? elem(v_prefix, dtype, t * stride_tok + g * stride_head + c)
                                 : elem(v_tree, dtype, ((int64_t)(t - L) * Hkv + g) * D + c);
                acc[c] += p * (double)vv;
            }
        }
        for (int c = 0; c < D; ++c) {
            float r = (float)(acc[c] / denom);
            out[o * D + c] = dtype == REF_BF16 ? round_bf16(r) : r;
        }
        free(s); free(acc);
    }
    return rc;
}

/* ------------------------------------------------------------ Philox4x32-10 */

/* Counter-based generator of Salmon et al. (SC'11), 4 words of 32 bits, 10 rounds. */
void ref_philox4x32(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3], k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0, p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* uniform in [0,1) with 24 bits: node index, sequence index and step form the counter */
float ref_uniform(uint64_t seed, uint64_t step, uint32_t seq, uint32_t node)
{
    uint32_t ctr[4] = {node, seq, (uint32_t)step, (uint32_t)(step >> 32)};
    uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint32_t r[4];
    ref_philox4x32(ctr, key, r);
    return (float)(r[0] >> 8) * (1.0f / 16777216.0f);
}

/* ------------------------------------------------- A6-A7: acceptance, walk */

static int row_argmax(const void *row, int dtype, int V)
{
    int best = 0;
    float bx = elem(row, dtype, 0);
    for (int v = 1; v < V; ++v) {
        float x = elem(row, dtype, v);
        if (x > bx) { bx = x; best = v; } /* strict: ties keep the lowest id */
    }
    return best;
}

/* log sum_v exp(x_v / T), accumulated in double */
static double row_lse_t(const void *row, int dtype, int V, double T)
{
    double m = -INFINITY;
    for (int v = 0; v < V; ++v) {
        double x = (double)elem(row, dtype, v) / T;
        if (x > m) m = x;
    }
    double s = 0.0;
    for (int v = 0; v < V; ++v) s += exp((double)elem(row, dtype, v) / T - m);
    return m + log(s);
}

/*
 * Inverse-CDF sample of softmax(row / T) at the uniform u, the CDF accumulated in double: the first
 * id with cdf > u (if rounding leaves none: the last id that carries mass).  *margin is lowered to
 * the distance of u to the edges of the chosen bin.
 */
static int row_sample_t(const void *row, int dtype, int V, double T, double u, double *margin)
{
    double l = row_lse_t(row, dtype, V, T);
    double cdf = 0.0, prev = 0.0;
    int last_pos = 0;
    for (int v = 0; v < V; ++v) {
        double p = exp((double)elem(row, dtype, v) / T - l);
        if (p > 0.0) last_pos = v;
        prev = cdf;
        cdf += p;
        if (cdf > u) {
            if (cdf - u < *margin) *margin = cdf - u;
            if (v > 0 && u - prev < *margin) *margin = u - prev;
            return v;
        }
    }
    return last_pos;
}

/*
 * Verify one sequence's tree against the target logits (row i = target's next-token
 * logits after node i) and walk the longest accepted path.
 *   mode 0 (greedy): node i>0 is accepted iff tokens[i] == argmax of its parent's row.
 *   mode 1 (stochastic): accepted iff u_i < min(1, P_T(tokens[i]) / P_d(tokens[i])),
 *     P_T = softmax(target[parent]/T), P_d = exp(logp[i]), u_i = ref_uniform(.., node i).
 *   mode 2 (target-sampled, distribution preserving): every node i draws the target's own next
 *     token y_i ~ softmax(target[i]/T) by inverse CDF at u = ref_uniform(.., node 0x80000000 + depth[i])
 *     (one uniform per depth: at most one node per depth lies on the walk); node i>0 is accepted iff
 *     tokens[i] == y_parent, and the bonus token is y_best.  With the children of a node being a fixed
 *     set (the draft's top-k, not samples), this is what sibling-by-sibling rejection sampling with
 *     residual renormalisation reduces to: child x_1 is accepted with probability p(x_1), after its
 *     rejection x_2 with p(x_2)/(1-p(x_1)), ..., i.e. child x_j overall with probability p(x_j), and
 *     otherwise the token comes from p restricted to the non-children -- exactly one draw from p.  The
 *     emitted tokens are therefore the target's own autoregressive samples for the same uniforms.
 *     node_argmax then receives y_i instead of the arg max.
 * ok[i] = accepted[i] and ok[parent]; best = deepest ok node, ties -> lowest index.
 * out_tokens = draft tokens along root->best (root excluded) followed by the bonus
 * token: greedy arg max of row best, or the inverse-CDF sample of softmax(row best/T)
 * at u = ref_uniform(.., node 0xFFFFFFFF).  path_nodes/out_tokens have d_cap+1 slots,
 * unused slots are -1.  node_argmax (may be NULL) gets the arg max of every row.
 * accepted (may be NULL) gets the per-node accept flags.
 * min_margin (may be NULL): stochastic only, the smallest |u_i - alpha_i| over nodes
 * with alpha_i < 1 and the distance of the bonus uniform to its CDF bin edges; mode 2: the
 * smallest distance of a uniform to its CDF bin edges over the nodes whose draw decides the
 * output (the nodes with all ancestors accepted).  node_margin (may be NULL; mode 2 only):
 * that distance for every node.
 */
int ref_accept(int mode, float temperature, const void *target, int dtype, int V, int64_t row_stride,
               int N, const int32_t *tokens, const int32_t *parents, const int32_t *depth,
               const float *logp, int d_cap, uint64_t seed, uint64_t step, uint32_t seq,
               int32_t *accept_len, int32_t *best_node, int32_t *path_nodes, int32_t *out_tokens,
               int32_t *node_argmax, uint8_t *accepted, float *min_margin, float *node_margin)
{
    if (!target || !tokens || !parents || !depth || !accept_len || !best_node || !path_nodes || !out_tokens)
        return REF_ERR_ARG;
    if (N < 1 || N > REF_TT_MAX || V < 1 || row_stride < V || d_cap < 1 || d_cap > REF_D_MAX) return REF_ERR_ARG;
    if (mode != 0 && mode != 1 && mode != 2) return REF_ERR_ARG;
    if (mode == 1 && !logp) return REF_ERR_ARG;
    if (mode != 0 && !(temperature > 0.0f)) return REF_ERR_ARG;
    const int esz = dtype == REF_F32 ? 4 : 2;
    int amax[REF_TT_MAX];
    unsigned char acc[REF_TT_MAX], ok[REF_TT_MAX];
    double margin = INFINITY;
    double nmargin[REF_TT_MAX];

#pragma omp parallel for schedule(dynamic)
    for (int i = 0; i < N; ++i)
        amax[i] = row_argmax((const char *)target + (int64_t)i * row_stride * esz, dtype, V);

    acc[0] = 1;
    if (mode == 0) {
        for (int i = 1; i < N; ++i) acc[i] = tokens[i] == amax[parents[i]];
    } else if (mode == 2) {
        double T = (double)temperature;
        for (int i = 0; i < N; ++i) {
            if (depth[i] < 0 || depth[i] > REF_D_MAX) return REF_ERR_ARG;
            double u = (double)ref_uniform(seed, step, seq, 0x80000000u + (uint32_t)depth[i]);
            nmargin[i] = INFINITY;
            amax[i] = row_sample_t((const char *)target + (int64_t)i * row_stride * esz, dtype, V, T, u, &nmargin[i]);
        }
        for (int i = 1; i < N; ++i) acc[i] = tokens[i] == amax[parents[i]];
    } else {
        double T = (double)temperature;
        double lse[REF_TT_MAX];
#pragma omp parallel for schedule(dynamic)
        for (int i = 0; i < N; ++i)
            lse[i] = row_lse_t((const char *)target + (int64_t)i * row_stride * esz, dtype, V, T);
        for (int i = 1; i < N; ++i) {
            int p = parents[i];
            if (tokens[i] < 0 || tokens[i] >= V) return REF_ERR_ARG;
            const char *prow = (const char *)target + (int64_t)p * row_stride * esz;
            double lpT = (double)elem(prow, dtype, tokens[i]) / T - lse[p];
            double alpha = exp(lpT - (double)logp[i]);
            if (alpha > 1.0) alpha = 1.0;
            double u = (double)ref_uniform(seed, step, seq, (uint32_t)i);
            acc[i] = u < alpha;
            if (alpha < 1.0 && fabs(u - alpha) < margin) margin = fabs(u - alpha);
        }
    }

    int best = 0;
    ok[0] = 1;
    for (int i = 1; i < N; ++i) {
        if (parents[i] < 0 || parents[i] >= i) return REF_ERR_ARG;
        ok[i] = acc[i] && ok[parents[i]];
        if (ok[i] && depth[i] > depth[best]) best = i; /* strict: ties keep the lowest index */
    }
    if (mode == 2)
        for (int i = 0; i < N; ++i) {
            if (ok[i] && nmargin[i] < margin) margin = nmargin[i];
            if (node_margin) node_margin[i] = (float)nmargin[i];
        }
    int len = depth[best];
    if (len > d_cap) return REF_ERR_ARG;
    for (int s = 0; s <= d_cap; ++s) { path_nodes[s] = -1; out_tokens[s] = -1; }
    for (int i = best; i >= 0; i = parents[i]) {
        path_nodes[depth[i]] = i;
        if (i > 0) out_tokens[depth[i] - 1] = tokens[i];
    }

    int bonus;
    if (mode == 0 || mode == 2) {
        bonus = amax[best];
    } else {
        double T = (double)temperature;
        const char *brow = (const char *)target + (int64_t)best * row_stride * esz;
        double l = row_lse_t(brow, dtype, V, T);
        double u = (double)ref_uniform(seed, step, seq, 0xFFFFFFFFu);
        double cdf = 0.0, prev = 0.0;
        int last_pos = 0;
        bonus = -1;
        for (int v = 0; v < V; ++v) {
            double p = exp((double)elem(brow, dtype, v) / T - l);
            if (p > 0.0) last_pos = v;
            prev = cdf;
            cdf += p;
            if (cdf > u) { bonus = v; break; }
        }
        if (bonus < 0) { bonus = last_pos; } /* u above the rounded total: last token with mass */
        else {
            double m1 = cdf - u, m2 = u - prev;
            if (m1 < margin) margin = m1;
            if (bonus > 0 && m2 < margin) margin = m2;
        }
    }
    out_tokens[len] = bonus;
    *accept_len = len;
    *best_node = best;
    if (node_argmax) for (int i = 0; i < N; ++i) node_argmax[i] = amax[i];
    if (accepted) for (int i = 0; i < N; ++i) accepted[i] = acc[i];
    if (min_margin) *min_margin = (float)margin;
    return REF_OK;
}

/* ------------------------------------------------------------- input update (KV commit) */

/*
 * "Input update" after verification (Appendix, System Profiling and Overhead Analysis): the
 * KV cache keeps the accepted tokens and discards the rejected ones.  The keys/values of
 * all tree tokens were produced by the verification pass into a buffer of their own, so
 * "discard" means: only the rows on the accepted path are appended to the cache.
 *
 * One sequence, one cache tensor (K or V of one layer):
 *   cache       element (t, g, c) at t*stride_tok + g*stride_head + c; rows 0..L-1 hold the prefix
 *   cap         rows the cache can hold
 *   tree        [N, Hkv, D] rows of the tree tokens (row 0 = root)
 *   path_nodes  path_nodes[0..len] = root .. deepest accepted node (output of ref_accept)
 * Cache row L+s receives tree row path_nodes[s], s = 0..len, for as long as the row fits
 * (L+s < cap).  *new_len = min(cap, L+len+1): the position of the next root (the bonus token),
 * whose own keys/values are computed by the next step.
 */
int ref_commit_rows(void *cache, int dtype, int64_t cap, int64_t L, int64_t stride_tok, int64_t stride_head,
                    int Hkv, int D, const void *tree, int N, const int32_t *path_nodes, int len,
                    int64_t *new_len)
{
    if (!cache || !tree || !path_nodes || !new_len) return REF_ERR_ARG;
    if (L < 0 || L > cap || len < 0 || len > REF_D_MAX || N < 1 || Hkv < 1 || D < 1) return REF_ERR_ARG;
    size_t esz = dtype == REF_F32 ? 4 : 2;
    for (int s = 0; s <= len; ++s) {
        int node = path_nodes[s];
        if (node < 0 || node >= N) return REF_ERR_ARG;
        int64_t t = L + s;
        if (t >= cap) break;
        for (int g = 0; g < Hkv; ++g)
            for (int c = 0; c < D; ++c)
                memcpy((char *)cache + (size_t)(t * stride_tok + g * stride_head + c) * esz,
                       (const char *)tree + ((size_t)((int64_t)node * Hkv + g) * D + c) * esz, esz);
    }
    *new_len = L + len + 1 < cap ? L + len + 1 : cap;
    return REF_OK;
}

/* ------------------------------------------------- action selection (policy + action cache) */

/*
 * Action table (Appendix A, "Action Space in Implementation"): all (TT, d, k) with
 * TT in {32,48,64,80,96,128}, d in {3..8}, k in {8,12,16,20,32}, kept only if TT <= k^(d-1).
 * Order (the paper gives none): TT-major, then d, then k.  out holds 3 ints per action.
 * Returns the number of actions written (at most cap).
 */
int ref_action_table(int32_t *out, int cap)
{
    static const int TTs[] = {32, 48, 64, 80, 96, 128}, ds[] = {3, 4, 5, 6, 7, 8}, ks[] = {8, 12, 16, 20, 32};
    int n = 0;
    for (int a = 0; a < 6; ++a)
        for (int b = 0; b < 6; ++b)
            for (int c = 0; c < 5; ++c) {
                double lim = pow((double)ks[c], (double)(ds[b] - 1));
                if ((double)TTs[a] > lim) continue;
                if (n < cap) { out[3 * n] = TTs[a]; out[3 * n + 1] = ds[b]; out[3 * n + 2] = ks[c]; }
                ++n;
            }
    return n;
}

/*
 * Policy network (Appendix A, "Network Architecture": an MLP with two hidden layers of H units on
 * the state s_t = the three concatenated hidden-state vectors, Section 3.3; the defaults of the PPO
 * implementation the paper names: tanh activations, one linear layer onto the action logits).
 * Weight matrices are stored [in][out] row-major: W1 [F][H], W2 [H][H], W3 [H][A].
 * Everything in double; logits[A] out.
 */
int ref_policy_logits(const float *feat, int F, int H, int A, const float *W1, const float *b1, const float *W2,
                      const float *b2, const float *W3, const float *b3, double *logits)
{
    if (!feat || !W1 || !b1 || !W2 || !b2 || !W3 || !b3 || !logits || F < 1 || H < 1 || A < 1) return REF_ERR_ARG;
    double *h1 = (double *)malloc(sizeof(double) * (size_t)H), *h2 = (double *)malloc(sizeof(double) * (size_t)H);
    if (!h1 || !h2) { free(h1); free(h2); return REF_ERR_INTERNAL; }
    for (int o = 0; o < H; ++o) {
        double s = (double)b1[o];
        for (int i = 0; i < F; ++i) s += (double)feat[i] * (double)W1[(size_t)i * H + o];
        h1[o] = tanh(s);
    }
    for (int o = 0; o < H; ++o) {
        double s = (double)b2[o];
        for (int i = 0; i < H; ++i) s += h1[i] * (double)W2[(size_t)i * H + o];
        h2[o] = tanh(s);
    }
    for (int a = 0; a < A; ++a) {
        double s = (double)b3[a];
        for (int i = 0; i < H; ++i) s += h2[i] * (double)W3[(size_t)i * A + a];
        logits[a] = s;
    }
    free(h1); free(h2);
    return REF_OK;
}

/*
 * One decision point of Algorithm 1 ("Re-SpS with Action Caching") for one sequence.
 *   cache_step, cached_action: in/out (start: 0 and -1 = nothing cached)
 *   logits: the policy's action logits for the current state (read only when the policy is queried)
 *   mode 0: the action of largest logit, ties -> lowest index; mode 1: a sample of softmax(logits) by
 *   inverse CDF (double) at the Philox uniform with node index 0xFFFFFFFE
 * The policy is queried iff cache_step == 0 or nothing is cached; the chosen action is then used for
 * N consecutive decision points (cache_step counts them and is reset once it reaches N).
 * Returns the action; *queried tells whether the policy was used; *margin (may be NULL) is lowered to
 * the gap that decided a queried action (top-2 logit gap, or distance of the uniform to the CDF edges).
 */
int ref_policy_step(int *cache_step, int *cached_action, const double *logits, int A, int N, int mode,
                    uint64_t seed, uint64_t step, uint32_t seq, int *queried, double *margin)
{
    if (!cache_step || !cached_action || !queried || A < 1 || N < 1) return REF_ERR_ARG;
    if (*cache_step == 0 || *cached_action < 0) {
        if (!logits) return REF_ERR_ARG;
        int best = 0;
        for (int a = 1; a < A; ++a)
            if (logits[a] > logits[best]) best = a;
        int act = best;
        if (mode == 0) {
            for (int a = 0; a < A; ++a)
                if (a != best && margin && logits[best] - logits[a] < *margin) *margin = logits[best] - logits[a];
        } else {
            double Z = 0.0;
            for (int a = 0; a < A; ++a) Z += exp(logits[a] - logits[best]);
            double u = (double)ref_uniform(seed, step, seq, 0xFFFFFFFEu), cdf = 0.0, prev = 0.0;
            act = -1;
            for (int a = 0; a < A; ++a) {
                prev = cdf;
                cdf += exp(logits[a] - logits[best]) / Z;
                if (cdf > u) { act = a; break; }
            }
            if (act < 0) act = A - 1;
            else if (margin) {
                if (cdf - u < *margin) *margin = cdf - u;
                if (act > 0 && u - prev < *margin) *margin = u - prev;
            }
        }
        *cached_action = act;
        *cache_step = 1;
        *queried = 1;
    } else {
        *cache_step += 1;
        *queried = 0;
    }
    int act = *cached_action;
    if (*cache_step >= N) *cache_step = 0;
    return act;
}

/*
 * Reward of a decision point and its average over the cache interval (Section 3.1 "Reward Function":
 * accepted tokens divided by the elapsed time of the drafting/verification step; Section 3.3,
 * "multi-step action persistence": the reward is averaged over the N decoding steps of the cache
 * interval; Algorithm 1: the reward is computed after verification, before the cache step is reset).
 *
 * Called once per decoding step, after ref_policy_step and the verification of that step:
 *   cache_step     the cache step as ref_policy_step left it (0 = this step was the last of its interval)
 *   tokens         accepted tokens of the step (the caller decides whether the bonus token counts)
 *   elapsed        seconds the step took (> 0)
 *   sum, steps     in/out accumulators of the running interval (start: 0, 0)
 * Adds tokens / elapsed to the interval's sum.  When the interval ends, *avg = sum / steps (steps = N for
 * a full interval; a generation that started in the middle of one averages over what it saw), *done = 1
 * and the accumulators return to zero; otherwise *done = 0 and *avg is left alone.
 */
int ref_reward_step(int cache_step, double tokens, double elapsed, double *sum, int *steps, double *avg, int *done)
{
    if (!sum || !steps || !avg || !done || !(elapsed > 0.0) || cache_step < 0 || *steps < 0) return REF_ERR_ARG;
    *sum += tokens / elapsed;
    *steps += 1;
    if (cache_step == 0) {
        *avg = *sum / (double)*steps;
        *done = 1;
        *sum = 0.0;
        *steps = 0;
    } else {
        *done = 0;
    }
    return REF_OK;
}

