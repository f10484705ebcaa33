// Internal interfaces between the C ABI (api.cpp) and the kernel files.
#pragma once
#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/dt.h"

namespace dt {

// ---------------------------------------------------------- per-kernel timing (profile.cpp)
// Off by default.  When switched on (dt_profile_enable), every kernel is launched with a pair
// of pre-created HIP events attached to its dispatch (hipExtLaunchKernelGGL), which record the
// kernel's own begin and end; dt_profile_read sums the elapsed times per kernel id.
enum KernelId { KID_ROWS_DRAFT = 0, KID_ROWS_MERGE, KID_TREE, KID_ATTN, KID_ATTN_COMBINE, KID_ROWS_TARGET,
                KID_ACCEPT, KID_ROWS_UNIFORM, KID_COMMIT, KID_POLICY_L1, KID_POLICY_HEAD, KID_NODE_SAMPLE, KID_REWARD, KID_COUNT };
bool prof_next(int kid, hipEvent_t *start, hipEvent_t *stop);  // false when timing is off

template <typename F, typename... Args>
inline void launch_kernel(int kid, hipStream_t st, F kernel, dim3 grid, dim3 block, size_t lds, Args... args) {
    hipEvent_t e0, e1;
    if (prof_next(kid, &e0, &e1)) hipExtLaunchKernelGGL(kernel, grid, block, (unsigned)lds, st, e0, e1, 0, args...);
    else hipLaunchKernelGGL(kernel, grid, block, (unsigned)lds, st, args...);
}

// ------------------------------------------------------------------ row kernels (rows.hip)
enum RowMode { ROWS_UNIFORM = 0, ROWS_DRAFT = 1, ROWS_TARGET = 2, ROWS_LEVEL = 3 };
#define DT_STATE_ROWS (1 + (DT_D_MAX - 1) * DT_K_MAX)  // draft rows a sequence can own

struct RowArgs {
    const void *logits;
    int dtype;           // dt_dtype
    int V;
    int64_t row_stride;  // elements
    int mode;            // RowMode: which rows of the launch are live and their k
    int k_uniform;       // ROWS_UNIFORM
    int batch;           // ROWS_DRAFT
    const dt_params *params;
    const int64_t *row_off;
    int TT_cap;           // ROWS_DRAFT (clamp), ROWS_TARGET (rows per sequence)
    const int32_t *n_nodes;  // ROWS_TARGET
    int want_lse;
    float inv_t;          // 1 / temperature applied inside the exponentials
    unsigned long long *part_keys;  // arg max rows: [rows, S] best key of every chunk
    float *lane_max;      // top-k rows: [rows, S*256] one maximum per lane
    float2 *part_ms;      // (max, sum exp((x-max)*inv_t)): [rows, S] (arg max rows), [rows, S*4] (top-k rows)
    // ROWS_LEVEL: rows of one level of every sequence, results scattered into the build state
    int level, rows_per_seq, state_rows;
    const int32_t *n_exp_prev;  // [batch] nodes expanded one level up
    int64_t n_rows;  // set by the launch functions: rows of the launch (the grid may overhang)
    // set by the launch functions: read a row's chunk before the row is known to be live (the loads then
    // overlap the reads that decide it; the row is inside the caller's buffer either way)
    int early_load;
};

int rows_chunks_per_row(int V, int nl);
int rows_topk_nl(int V);                    // chunk multiplier of the top-k passes
int rows_pick_nl(int64_t n_rows, int V);    // chunk multiplier of the arg max pass
hipError_t rows_launch_stream(const RowArgs &a, int64_t n_rows, int nl, hipStream_t st);
hipError_t rows_launch_select(const RowArgs &a, int64_t n_rows, int nl, float *top_val, int32_t *top_id, float *lse,
                              int out_stride, hipStream_t st);
hipError_t rows_launch_argmax(const RowArgs &a, int64_t n_rows, int nl, hipStream_t st);

// ------------------------------------------------------------------ tree kernel (tree.hip)
struct TreeArgs {
    int batch;
    const dt_params *params;
    int V;
    const int32_t *root_token;
    int TT_cap;
    const float *top_val;  // [batch, seq_rows, DT_K_MAX]: row results of sequence b start at row b * seq_rows
    const int32_t *top_id;
    const float *lse;      // [batch, seq_rows]
    const int64_t *row_off;  // one-shot build: [batch+1] draft rows a sequence owns; null: all of its block
    int32_t *n_nodes, *tokens, *parents, *depth, *src_row;
    float *score, *logp;
    unsigned long long *anc_mask;
    int64_t seq_rows;
    int early_stop;         // expansion also ends once the root and the candidates proposed so far number TT
    // level-at-a-time build
    int expand_level;       // 0: whole tree; l > 0: only the set of level-l nodes to expand
    const int32_t *prefix_len;  // may be null (positions then count from 0)
    int32_t *n_expand, *state_n_exp, *exp_token, *exp_parent_slot, *exp_row, *exp_pos;  // [batch(, DT_K_MAX)]
    unsigned long long *exp_mask;  // [batch, DT_K_MAX, 4]
};
hipError_t tree_init();  // once per device, before the first launch
hipError_t tree_launch(const TreeArgs &a, hipStream_t st);

// -------------------------------------------------------------- attention (attention.hip)
struct AttnArgs {
    int batch, dtype, Hq, Hkv, D;
    float scale;
    const void *q, *k_tree, *v_tree;
    const int32_t *n_nodes;
    const void *const *k_prefix;
    const void *const *v_prefix;
    const int32_t *prefix_len;
    int max_prefix_len;
    int64_t kv_stride_tok, kv_stride_head;
    const unsigned long long *anc_mask;
    int TT_cap;
    void *out;
    void *ws;
    size_t ws_bytes;
    int n_cu;  // compute units of the device the launch goes to
};
size_t attn_workspace_bytes(int batch, int TT_cap, int Hq, int D, int n_cu);
hipError_t attn_init();  // once per device, before the first launch
int attn_launch(const AttnArgs &a, hipStream_t st, hipError_t *err);  // returns dt_status

// ------------------------------------------------------------------- accept (accept.hip)
struct AcceptArgs {
    int batch, mode;
    float temperature;
    const void *target;
    int dtype, V;
    int64_t row_stride;
    const int32_t *n_nodes, *tokens, *parents, *depth;
    const float *logp;
    const unsigned long long *anc_mask;
    int TT_cap;
    unsigned long long seed, step;
    int32_t *accept_len, *best_node, *path_nodes, *out_tokens, *node_argmax;
    const unsigned long long *part_keys;  // [batch*TT_cap, S]
    const float2 *part_ms;
    int S;            // chunks per row
    int chunk_elems;  // vocabulary entries per chunk
    int32_t *samples; // [batch*TT_cap] target-sampled mode: the token every node drew
};
hipError_t accept_launch(const AcceptArgs &a, hipStream_t st);

// --------------------------------------------------------------- input update (commit.hip)
struct CommitArgs {
    int batch, n_layers, dtype, Hkv, D;
    const void *const *k_tree;   // [n_layers] -> [batch, TT_cap, Hkv, D]
    const void *const *v_tree;
    void *const *k_prefix;       // [n_layers * batch], layer-major
    void *const *v_prefix;
    const int32_t *prefix_len, *prefix_cap;
    int64_t kv_stride_tok, kv_stride_head;
    const int32_t *n_nodes, *path_nodes, *accept_len, *out_tokens;
    int TT_cap;
    int vec16;                   // rows of D elements and both strides are multiples of 16 bytes
    int32_t *new_prefix_len, *next_root_token;
};
hipError_t commit_launch(const CommitArgs &a, hipStream_t st);

// ------------------------------------------------------------ action selection (policy.hip)
#define POLICY_KS 64  // inputs of layer 1 per workgroup
struct PolicyArgs {
    int batch, feat_dtype, F, H, A, N, mode;
    const void *feat;
    int64_t feat_stride;
    const float *W1, *b1, *W2, *b2, *W3, *b3;  // weights [in][out]
    const dt_params *table;                    // [A]
    unsigned long long seed, step;
    int32_t *cache_step, *cached_action;       // [batch] in/out
    dt_params *params_out;
    int32_t *action_out, *queried_out;         // may be null
    float *logits_out;                         // [batch, A], may be null
    float *partial;                            // [S, batch, H]
    int S;
};
hipError_t policy_launch(const PolicyArgs &a, hipStream_t st);

struct RewardArgs {
    int batch, count_bonus;
    float elapsed;             // seconds of the step, used when elapsed_dev is null
    const float *elapsed_dev;  // [batch] or null
    const int32_t *accept_len, *cache_step;
    float *reward_sum, *reward_avg;
    int32_t *reward_steps, *interval_done;
};
hipError_t reward_launch(const RewardArgs &a, hipStream_t st);

}  // namespace dt
