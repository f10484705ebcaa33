/*
 * dt.h -- C ABI of the draft-tree speculative step for AMD MI355X (gfx950).
 *
 * One speculative step of an EAGLE-style decoder whose tree limits (TT, d, k) are chosen
 * anew on every call, as the RL policy of "Speculative Sampling with Reinforcement
 * Learning" (Re-SpS) does:  dt_build_tree -> [target forward, whose attention is
 * dt_tree_attention] -> dt_accept   (paper: Algorithm 1, "Construct draft tree DT using
 * (TT, d, k)", "Verify DT with M_t"; Appendix B, Algorithm 2, drafting block).
 *
 * Conventions for every entry point
 *   - Returns DT_OK or a negative dt_status.  Never throws, aborts, allocates, frees or
 *     synchronises.  Arguments are validated on the host before anything is launched; that
 *     includes the launch grids (see the limits below): a call that would need a grid the
 *     hardware cannot take returns DT_ERR_LIMIT and launches nothing.
 *   - One-time set-up per device: see dt_init().  Apart from that the library keeps no state
 *     (the optional dt_profile_* timing aside) and its entry points may be called from several
 *     threads, on different streams, as long as calls that share a workspace are ordered.
 *   - All tensor pointers are DEVICE pointers owned by the caller.  Scalars are host values.
 *   - `stream` is the caller's hipStream_t (as void*; NULL = the default stream).  Work is
 *     enqueued on it and the call returns immediately; outputs are valid once the stream
 *     has reached that point.
 *   - `ws` is caller-owned device scratch of at least dt_workspace_bytes() bytes, 256-byte
 *     aligned; its contents need not survive between calls.  Calls that share one workspace
 *     must be ordered on one stream.
 *   - Per-sequence limits live in a DEVICE array of dt_params so that a policy running on
 *     the GPU can set them without a host round trip.  Values are clamped on the device
 *     to 1 <= TT <= TT_cap, 1 <= d <= DT_D_MAX, 1 <= k <= min(DT_K_MAX, V).
 *   - Logits must not contain NaN or +inf; -inf marks a token that can never be proposed.
 *   - Tie-breaks: inside a row larger logit first, then smaller token id; across rows
 *     larger cumulative score first, then smaller pool index (see dt_build_tree).
 */
#ifndef DT_H
#define DT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Limits: maxima of the action space in the paper's Appendix A
 * (TT in {32..128}, d in {3..8}, k in {8..32}). */
#define DT_TT_MAX 128
#define DT_D_MAX 8
#define DT_K_MAX 32
#define DT_MASK_WORDS (DT_TT_MAX / 64) /* uint64 words per node in anc_mask */

typedef struct {
    int32_t TT; /* upper limit on tree tokens, root included  (paper Section 4, action space) */
    int32_t d;  /* upper limit on tree depth = draft levels below the root */
    int32_t k;  /* children proposed per expanded node and nodes expanded per level */
} dt_params;

typedef enum { DT_F32 = 0, DT_BF16 = 1 } dt_dtype;
typedef enum { DT_ACCEPT_GREEDY = 0, DT_ACCEPT_STOCHASTIC = 1, DT_ACCEPT_SAMPLED = 2 } dt_accept_mode;

typedef enum {
    DT_OK = 0,
    DT_ERR_INVALID_ARG = -1, /* null pointer, negative size, misaligned pointer, bad enum */
    DT_ERR_LIMIT = -2,       /* a size exceeds a compiled limit (TT_cap, k, head dim, ...) */
    DT_ERR_WORKSPACE = -3,   /* ws too small or NULL */
    DT_ERR_DTYPE = -4,       /* dtype/shape combination without a kernel */
    DT_ERR_HIP = -5          /* a HIP call failed; see dt_last_hip_error() */
} dt_status;

/*
 * One-time set-up for the CURRENT device: asks the runtime for the device's number of compute
 * units (launch shapes depend on it), gives the kernels that use more than 64 KB of LDS leave
 * to do so (hipFuncSetAttribute) and looks up the device's address of the library's own
 * scratch (dt_topk_rows_static).  No allocation, no launch, no stream operation.
 * Thread-safe and idempotent; every launching entry point does the same on its first call on a
 * device, so calling dt_init() is optional -- but a caller that records its first call into a
 * HIP graph, or calls from several threads at once at start-up, may prefer to have it done
 * beforehand.  (The set-up calls are legal while a stream is being captured: they enqueue
 * nothing.)  At most 64 devices per process.  Returns DT_OK or DT_ERR_HIP.
 */
int dt_init(void);

const char *dt_status_string(int status);
/* hipError_t of the last failing HIP call made by this library on this thread (0 if none). */
int dt_last_hip_error(void);
const char *dt_hip_error_string(int hip_error); /* HIP's own text for that code */

/*
 * Scratch size that suffices for any of the calls below with
 *   batch sequences, total_rows draft rows (all sequences), vocabulary V,
 *   node rows padded to TT_cap per sequence, Hq query heads of dimension D.
 * Host-only computation.
 */
int dt_workspace_bytes(int batch, int64_t total_rows, int V, int TT_cap, int Hq, int D, size_t *bytes);

/*
 * Row top-k and row log-sum-exp (paper Algorithm 2: each expanded node proposes its k
 * most confident children; Section 3.2: confidence = draft probability).
 *   logits   [n_rows, row_stride] elements of type t, row r at logits + r*row_stride; V <= row_stride.
 *   top_val  [n_rows, k] float : the k largest logits of the row, best first
 *   top_id   [n_rows, k] int32 : their token ids; equal logits are ordered by ascending id
 *   lse      [n_rows]   float  : log sum_v exp(logits[r, v])
 * Slots beyond the number of finite entries of a row hold (-inf, -1).
 * Errors: k < 1 or k > min(DT_K_MAX, V) -> DT_ERR_LIMIT; V beyond 524,288 or more than 2^31 - 1
 * rows in one call -> DT_ERR_LIMIT.
 */
int dt_topk_rows(void *stream, const void *logits, dt_dtype t, int64_t n_rows, int V, int64_t row_stride,
                 int k, float *top_val, int32_t *top_id, float *lse, void *ws, size_t ws_bytes);

/*
 * dt_topk_rows for callers that cannot allocate device memory and hold no workspace: code that runs
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same inputs, outputs,
 * kernels and results as dt_topk_rows; the scratch (lane maxima and log-sum-exp partials) lives in
 * device memory that belongs to the library -- DT_STATIC_SCRATCH_BYTES per device that runs it, held
 * until the process ends -- and the call makes no allocation of any kind.
 * Limit: rows * ceil(V / c) * 1056 bytes must fit (c = 2048, 4096 or 8192: the smallest that keeps a row
 * within 16 chunks, 8192 beyond that): 496 rows of a 128,256-entry vocabulary, 1,986 of 32,000.
 * More -> DT_ERR_LIMIT, nothing is launched.  Other errors as dt_topk_rows.
 * All calls on one device share that device's scratch, which keeps the previous call's contents (none
 * of it needs clearing): calls that overlap on one device -- different streams, or graphs that replay
 * concurrently -- race; order them.
 */
#define DT_STATIC_SCRATCH_BYTES (8u << 20)
int dt_topk_rows_static(void *stream, const void *logits, dt_dtype t, int64_t n_rows, int V, int64_t row_stride,
                        int k, float *top_val, int32_t *top_id, float *lse);

/*
 * Draft-tree construction for a batch (paper Section 3.2 "Draft Tree Expansion" and
 * "Confidence-Based Candidate Reranking"; Algorithm 2, expansion loop and rerank).
 *
 * Input rows.  Sequence b owns draft rows row_off[b] .. row_off[b+1]-1 of draft_logits
 * and uses the first 1 + (d-1)*k of them: local row 0 is the next-token row of the root;
 * local row 1 + (l-1)*k + s is the next-token row of the s-th expanded node of level l
 * (l = 1..d-1), expanded nodes of a level being numbered in ascending pool index.
 * total_rows = row_off[batch] as a host value (sizes the launch; draft_logits holds that many rows,
 * all of which may be read, also those a sequence does not use).  A sequence that owns fewer than
 * 1 + (d-1)*k rows is built as if the missing rows held no viable token (all -inf): the nodes that
 * would have been handed those rows get no children.
 *
 * Method.  Level-l candidates are the top-k tokens of every expanded level-(l-1) node;
 * score = score[parent] + (logit - lse of its row), one float add per level.  The k best
 * candidates of a level (score desc, pool index asc) are expanded.  Pool index of the
 * rank-r child of slot s at level l: r for l = 1, else k + (l-2)k^2 + s*k + r.  Finally the
 * best min(TT-1, pool size) candidates of the whole pool are kept (same order).
 *
 * Outputs, per sequence b at offset b*TT_cap (b*TT_cap*DT_MASK_WORDS for anc_mask);
 * node 0 is the root, nodes 1.. are the kept candidates in ascending pool index, so
 * parents precede children and depth is non-decreasing:
 *   n_nodes [batch]           number of nodes N <= TT
 *   tokens  [batch, TT_cap]   token id (node 0: root_token[b])
 *   parents [batch, TT_cap]   node index of the parent, -1 for the root
 *   depth   [batch, TT_cap]   level, 0 for the root
 *   score   [batch, TT_cap]   cumulative draft log-probability
 *   logp    [batch, TT_cap]   the node's own draft log-probability (0 for the root)
 *   src_row [batch, TT_cap]   local draft row the node was handed (root 0), -1 if not expanded
 *   anc_mask[batch, TT_cap, DT_MASK_WORDS] bit j of node i set iff j == i or j is an ancestor of i
 * Entries at index >= n_nodes[b] are left untouched.
 *
 * flags: 0, or DT_TREE_EARLY_STOP for the token-count exit of Algorithm 2's expansion loop: the count
 * starts at 1 (the root) and grows by the viable candidates every expansion proposes (the root's k, then
 * up to k per expanded node); no further level is expanded once it has reached TT.  The rows of levels
 * that are then never expanded are still streamed (their number is not known before the launch) but no
 * result depends on them.  Without the flag TT binds at the rerank only (Section 3.2: all tokens of the
 * tree are reranked).
 * Errors: TT_cap < 1 or > DT_TT_MAX, V < 1 -> DT_ERR_LIMIT; unknown flag bits -> DT_ERR_INVALID_ARG;
 * ws too small -> DT_ERR_WORKSPACE.
 */
#define DT_TREE_EARLY_STOP 1
int dt_build_tree(void *stream, int batch, const dt_params *params, const void *draft_logits, dt_dtype t,
                  int V, int64_t row_stride, const int64_t *row_off, int64_t total_rows,
                  const int32_t *root_token, int TT_cap, int32_t *n_nodes, int32_t *tokens,
                  int32_t *parents, int32_t *depth, float *score, float *logp, int32_t *src_row,
                  uint64_t *anc_mask, void *ws, size_t ws_bytes, int flags);

/*
 * Tree-masked attention of the tree tokens for ONE layer (paper Section 3.2 "Verification
 * Phase": the target evaluates all draft tokens in one pass; Section 2: tree attention).
 * Node i of sequence b, query head h (kv head h / (Hq/Hkv)) attends to the prefix_len[b]
 * prefix keys and to the tree keys j with bit j of anc_mask[b, i] set:
 *   out[b,i,h,:] = softmax_j(scale * q[b,i,h,:] . K_j) V_j
 *   q, out         [batch, TT_cap, Hq, D]  type t (rows >= n_nodes[b] are neither read nor written)
 *   k_tree, v_tree [batch, TT_cap, Hkv, D] type t
 *   k_prefix[b], v_prefix[b] : device arrays (length batch) of device pointers; element
 *       (token, kv head, c) at token*kv_stride_tok + head*kv_stride_head + c (strides in elements);
 *       [token, kv head, D] and [kv head, token, D] caches are both expressed by the two strides.
 *       The pointers themselves must be 16-byte aligned (they live in device memory, so the host
 *       cannot check them; the kernels read 16 bytes at a time from them)
 *   max_prefix_len : host upper bound of prefix_len[] (sizes the launch)
 * Arithmetic: bf16 inputs, fp32 accumulation, fp32 softmax, output rounded to bf16; fp32 inputs are
 * handled entirely in fp32.  bf16 with D == 128 and both strides multiples of 8 elements runs on the
 * matrix cores; every other combination with D <= 128 runs on a plain vector-ALU kernel (correct, slow).
 * Errors: Hq % Hkv != 0, scale <= 0, negative strides, q / k_tree / v_tree / out not 16-byte aligned
 * -> DT_ERR_INVALID_ARG; D > 128, batch > 8191 or Hq > 65535 -> DT_ERR_LIMIT.
 */
int dt_tree_attention(void *stream, int batch, dt_dtype t, int Hq, int Hkv, int D, float scale,
                      const void *q, const void *k_tree, const void *v_tree, const int32_t *n_nodes,
                      const void *const *k_prefix, const void *const *v_prefix, const int32_t *prefix_len,
                      int max_prefix_len, int64_t kv_stride_tok, int64_t kv_stride_head,
                      const uint64_t *anc_mask, int TT_cap, void *out, void *ws, size_t ws_bytes);

/*
 * Acceptance and longest accepted walk (paper Section 3.2 "Acceptance Criterion";
 * Section 3.1 greedy decoding).  target_logits row (b, i) = the target's next-token
 * logits after node i, at target_logits + (b*TT_cap + i)*row_stride.  The buffer holds all
 * batch*TT_cap rows: rows at and past n_nodes[b] never reach a result, but a small launch may read them.
 *   greedy     : node i > 0 accepted iff tokens[i] == argmax(row of its parent), ties -> lowest id
 *   stochastic : accepted iff u_i < min(1, P_T(tokens[i]) / P_d(tokens[i])), P_T = softmax(row of
 *                parent / temperature), P_d = exp(logp[i]); u_i is the first word of
 *                Philox4x32-10(counter = (i, b, step lo, step hi), key = (seed lo, seed hi)),
 *                mapped to [0,1) as (word >> 8) * 2^-24.
 *   sampled    : distribution-preserving verification for trees whose children are a fixed set (the
 *                draft's top-k): every node i draws the target's own next token y_i from
 *                softmax(row i / temperature) by inverse CDF at the Philox uniform with node index
 *                0x80000000 + depth[i]; node i > 0 is accepted iff tokens[i] == y of its parent, and
 *                the bonus token is y_best.  (Sibling-by-sibling rejection with renormalised residuals
 *                accepts child x with probability p(x) overall and otherwise draws from p outside the
 *                children: one draw from p.)  The emitted tokens are the target's autoregressive
 *                samples for the same uniforms.  node_argmax then holds y_i.
 * The walk ends at `best`, the deepest node all of whose ancestors (and itself) are accepted,
 * ties -> lowest node index.  Outputs per sequence:
 *   accept_len [batch]               depth of best = number of accepted draft tokens
 *   best_node  [batch]
 *   path_nodes [batch, DT_D_MAX+1]   root .. best, unused slots -1
 *   out_tokens [batch, DT_D_MAX+1]   accepted draft tokens, then the bonus token (greedy: argmax of
 *                                    row best; stochastic: inverse-CDF sample of softmax(row best /
 *                                    temperature) at the uniform with node index 0xFFFFFFFF), then -1
 *   node_argmax[batch, TT_cap]       argmax of every node row (may be NULL)
 * Errors: stochastic / sampled with temperature <= 0, stochastic with logp NULL -> DT_ERR_INVALID_ARG;
 * batch*TT_cap beyond 2^31 - 1 rows -> DT_ERR_LIMIT.
 */
int dt_accept(void *stream, int batch, dt_accept_mode mode, float temperature, const void *target_logits,
              dt_dtype t, int V, int64_t row_stride, const int32_t *n_nodes, const int32_t *tokens,
              const int32_t *parents, const int32_t *depth, const float *logp, const uint64_t *anc_mask,
              int TT_cap, uint64_t philox_seed, uint64_t philox_step, int32_t *accept_len,
              int32_t *best_node, int32_t *path_nodes, int32_t *out_tokens, int32_t *node_argmax,
              void *ws, size_t ws_bytes);

/*
 * The same tree, built one level at a time, for a draft model that sits between the levels
 * (paper Appendix B, Algorithm 2: every pass of the expansion loop runs the draft model on the
 * nodes chosen one level up, then chooses the next ones).  Call pattern per step:
 *     for level = 1 .. max d:   [draft model] -> dt_expand_level(level, logits of this pass)
 *     dt_finish_tree            -> the outputs of dt_build_tree
 * `state` (dt_level_state_bytes(batch) bytes, 256-byte aligned, caller-owned, contents opaque, need not
 * be cleared) carries the row results from call to call; all calls of one step use the same batch,
 * params, V and TT_cap.
 *
 * dt_expand_level, level l: level_logits holds the rows of this pass, sequence b's row s at
 * level_logits + (b*R + s)*row_stride with R = 1 for level 1 (the root's next-token row) and
 * R = rows_per_seq (>= every k, <= DT_K_MAX) otherwise; row s belongs to the s-th node that the
 * previous call reported for sequence b (rows at and past that call's n_expand[b] are ignored, but
 * belong to the buffer, which holds batch*R rows: a small launch may read them).
 * The call scores the candidates of level l and reports the nodes of level l that are expanded
 * next, in slot order (= ascending pool index):
 *   n_expand        [batch]            how many (0 when l >= d, TT == 1, nothing is viable, or -- with
 *                                      DT_TREE_EARLY_STOP -- the token count has reached TT)
 *   exp_token       [batch, DT_K_MAX]  their tokens
 *   exp_parent_slot [batch, DT_K_MAX]  slot of the parent in the previous call's list (-1: the root)
 *   exp_row         [batch, DT_K_MAX]  the draft row each is handed, 1 + (l-1)k + slot
 *   exp_pos         [batch, DT_K_MAX]  position id prefix_len[b] + l (prefix_len may be NULL: l)
 *   exp_mask        [batch, DT_K_MAX, 4]  draft-side tree mask over draft rows (bit r: row r belongs to
 *                                      the node or one of its ancestors; row 0 = root)
 * Workspace: dt_workspace_bytes(batch, batch*R, V, TT_cap, 1, 1) bytes.
 * dt_finish_tree reranks and emits exactly what dt_build_tree would from the same rows.
 * flags as for dt_build_tree, the same value in every call of a step: with DT_TREE_EARLY_STOP the draft
 * model's loop ends at the first level whose n_expand is 0 everywhere, which is what the flag is for.
 * Errors as dt_build_tree; level outside 1..DT_D_MAX, rows_per_seq outside 1..DT_K_MAX or a
 * misaligned state -> DT_ERR_INVALID_ARG.
 */
int dt_level_state_bytes(int batch, size_t *bytes);
int dt_expand_level(void *stream, int batch, int level, const dt_params *params, const void *level_logits, dt_dtype t,
                    int V, int64_t row_stride, int rows_per_seq, const int32_t *prefix_len, int TT_cap, void *state,
                    int32_t *n_expand, int32_t *exp_token, int32_t *exp_parent_slot, int32_t *exp_row, int32_t *exp_pos,
                    uint64_t *exp_mask, void *ws, size_t ws_bytes, int flags);
int dt_finish_tree(void *stream, int batch, const dt_params *params, int V, const int32_t *root_token, int TT_cap,
                   const void *state, int32_t *n_nodes, int32_t *tokens, int32_t *parents, int32_t *depth, float *score,
                   float *logp, int32_t *src_row, uint64_t *anc_mask, int flags);

/*
 * Action selection on the device (paper Section 3.3 and Algorithm 1 "Re-SpS with Action Caching";
 * Appendix A "Action Space in Implementation", "Network Architecture").
 *
 * dt_action_table (host): writes the actions (TT, d, k) of the printed value sets that pass the printed
 * filter TT <= k^(d-1), in the order TT, then d, then k, into table[0 .. min(capacity, *n_actions));
 * *n_actions is their number (177).  The caller copies the table to the device.
 *
 * dt_policy_step: one decision point for every sequence.  If nothing is cached for sequence b
 * (cached_action[b] < 0) or its interval is over (cache_step[b] == 0) the policy is evaluated on
 * features[b] = the concatenated hidden-state vectors (F values, type feat_t, row stride feat_stride):
 *     logits = W3^T tanh(W2^T tanh(W1^T x + b1) + b2) + b3          (fp32, weights [in][out] row-major:
 *     W1 [F,H], W2 [H,H], W3 [H,n_actions]; H in {64,128}; n_actions <= 256)
 * and the action is the largest logit (ties -> lowest index) or, with sample = 1, the inverse-CDF
 * sample of softmax(logits) at the Philox uniform with node index 0xFFFFFFFE (see dt_accept); it is
 * cached and cache_step[b] = 1.  Otherwise the cached action is used again and cache_step[b] += 1.
 * cache_step[b] returns to 0 when it reaches cache_interval, so an action serves cache_interval
 * consecutive decision points.  Outputs: params_out[b] = action_table[action] (a device array that
 * dt_build_tree / dt_expand_level take as `params`: no host round trip), action_out[b], queried_out[b]
 * (1 if the policy ran), logits_out[b, n_actions] (written only where the policy ran); the last
 * three may be NULL.  Start of a generation: cache_step = 0, cached_action = -1.
 * Workspace: dt_policy_workspace_bytes(batch, F, H), 256-byte aligned.
 * Errors: H not 64/128 or n_actions > 256 -> DT_ERR_LIMIT; null pointers, cache_interval < 1,
 * feat_stride < F -> DT_ERR_INVALID_ARG.
 */
int dt_action_table(dt_params *table, int capacity, int *n_actions);
int dt_policy_workspace_bytes(int batch, int F, int H, size_t *bytes);
int dt_policy_step(void *stream, int batch, dt_dtype feat_t, const void *features, int64_t feat_stride, int F, int H,
                   int n_actions, const float *W1, const float *b1, const float *W2, const float *b2, const float *W3,
                   const float *b3, const dt_params *action_table, int cache_interval, int sample, uint64_t philox_seed,
                   uint64_t philox_step, int32_t *cache_step, int32_t *cached_action, dt_params *params_out,
                   int32_t *action_out, int32_t *queried_out, float *logits_out, void *ws, size_t ws_bytes);

/*
 * Reward bookkeeping of Algorithm 1 (paper Section 3.1 "Reward Function": accepted tokens divided by the
 * elapsed time of the drafting/verification step; Section 3.3, multi-step action persistence: the reward is
 * averaged over the N decoding steps of the cache interval; Algorithm 1: computed after verification, before
 * the cache step is reset).  Call once per decoding step, after dt_policy_step and dt_accept of that step:
 *     reward = (accept_len[b] + count_bonus) / seconds,  seconds = elapsed_per_seq[b] (device, may be NULL)
 *              or else elapsed_seconds (host); count_bonus (0 or 1) says whether the bonus token counts as
 *              an accepted token (the paper does not say: 1 makes the reward the step's emitted tokens / s)
 *     reward_sum[b] += reward; reward_steps[b] += 1                    (device accumulators, start at 0)
 *     if cache_step[b] == 0 (dt_policy_step has closed the interval with this step):
 *         reward_avg[b] = reward_sum[b] / reward_steps[b], interval_done[b] = 1, accumulators back to 0
 *     else interval_done[b] = 0 and reward_avg[b] is left alone.
 * reward_steps is N for a full interval; a generation that begins inside one averages over what it saw.
 * Float arithmetic.  Errors: null pointers, count_bonus not 0/1, no positive time -> DT_ERR_INVALID_ARG.
 */
int dt_reward_step(void *stream, int batch, const int32_t *accept_len, int count_bonus, float elapsed_seconds,
                   const float *elapsed_per_seq, const int32_t *cache_step, float *reward_sum, int32_t *reward_steps,
                   float *reward_avg, int32_t *interval_done);

/*
 * Input update after verification (paper Appendix, "System Profiling and Overhead Analysis": the
 * input update brings the KV cache to the state of the next step -- accepted tokens kept, rejected
 * ones discarded, positions continued).  For every sequence b, layer l and both of K and V, the tree
 * rows of the accepted path are appended to the prefix cache:
 *     cache_l,b row prefix_len[b] + s  <-  tree_l row (b, path_nodes[b, s]),   s = 0 .. accept_len[b]
 * for as long as the row fits (row < prefix_cap[b]); nothing else in the cache is touched.
 *   k_tree, v_tree    device arrays [n_layers] of device pointers to [batch, TT_cap, Hkv, D] (type t)
 *   k_prefix,v_prefix device arrays [n_layers * batch] (layer-major) of device pointers to the caches;
 *                     element (token t, kv head g, c) at t*kv_stride_tok + g*kv_stride_head + c
 *   prefix_len,prefix_cap  [batch] valid rows and capacity in rows of every cache of sequence b
 *   n_nodes, path_nodes [batch, DT_D_MAX+1], accept_len, out_tokens [batch, DT_D_MAX+1]: as written
 *                     by dt_build_tree / dt_accept
 *   new_prefix_len [batch]  out: min(prefix_cap, prefix_len + accept_len + 1), the position of the next
 *                     root; must not alias prefix_len (every workgroup reads the old length)
 *   next_root_token [batch] out, may be NULL: the bonus token out_tokens[b, accept_len[b]]
 * 16-byte copies are used when D*sizeof(t), both strides and all base pointers allow it.  No workspace.
 * Errors: null pointers, new_prefix_len == prefix_len, non-positive sizes -> DT_ERR_INVALID_ARG;
 * TT_cap outside 1..DT_TT_MAX or n_layers > 65535 -> DT_ERR_LIMIT.
 */
int dt_commit(void *stream, int batch, int n_layers, dt_dtype t, int Hkv, int D, const void *const *k_tree,
              const void *const *v_tree, void *const *k_prefix, void *const *v_prefix, const int32_t *prefix_len,
              const int32_t *prefix_cap, int64_t kv_stride_tok, int64_t kv_stride_head, const int32_t *n_nodes,
              const int32_t *path_nodes, const int32_t *accept_len, const int32_t *out_tokens, int TT_cap,
              int32_t *new_prefix_len, int32_t *next_root_token);

/*
 * Optional per-kernel timing, for measurement only (off by default; not part of the step).
 * dt_profile_enable(n > 0) pre-creates n HIP event pairs and switches timing on: every kernel
 * launched by the calls above then carries an event pair on its dispatch that records the
 * kernel's own begin and end (not usable while the stream is being captured into a graph).
 * dt_profile_enable(0) switches it off.  dt_profile_read sums, for one kernel id
 * (0 draft row chunks, 1 row merge, 2 tree, 3 attention, 4 attention combine, 5 target row
 * chunks, 6 accept, 7 dt_topk_rows chunks, 8 commit, 9 policy layer 1, 10 policy head, 11 per-node target samples,
 * 12 reward), the elapsed milliseconds of the launches recorded
 * since the last enable, waiting for them to finish.  Not thread-safe.
 */
int dt_profile_enable(int max_launches);
int dt_profile_read(int kernel_id, double *total_ms, int *launches);
const char *dt_profile_kernel_name(int kernel_id);

#ifdef __cplusplus
}
#endif
#endif /* DT_H */
