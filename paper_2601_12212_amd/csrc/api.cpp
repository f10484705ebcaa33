// C ABI of the library: argument validation on host values, scratch layout, launches.
// No allocation, no synchronisation, no exceptions.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdint>
#include <mutex>

#include "kernels.hpp"

namespace {

thread_local int g_last_hip = 0;

// ---- one-time set-up per device (dt_init) ---------------------------------------------------------
// Kernels that use more than 64 KB of LDS have to be given leave once per device, and the launch
// shapes depend on the device's number of compute units.  Both are settled here, under a lock, by
// dt_init() or by the first launching call on a device; afterwards the launch path only reads.
constexpr int MAX_DEVICES = 64;
struct DeviceState {
    std::atomic<int> ready{0};
    int n_cu = 0;
    void *scratch = nullptr;  // this device's copy of g_scratch
};

// Scratch of dt_topk_rows_static: device memory that belongs to the library, so that the call needs no
// workspace and allocates nothing.  Every device that runs the library holds its own copy, at its own
// address, until the process ends.  In host code the array's name is only a handle for
// hipGetSymbolAddress: the address kernels and copies use is the one kept per device in DeviceState.
static __device__ __align__(256) unsigned char g_scratch[DT_STATIC_SCRATCH_BYTES];
DeviceState g_dev[MAX_DEVICES];
std::mutex g_init_mu;

// status; *n_cu = compute units of the current device
int ensure_init(int *n_cu) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) { g_last_hip = (int)e; (void)hipGetLastError(); return DT_ERR_HIP; }
    if (dev < 0 || dev >= MAX_DEVICES) return DT_ERR_LIMIT;
    DeviceState &d = g_dev[dev];
    if (!d.ready.load(std::memory_order_acquire)) {
        std::lock_guard<std::mutex> lock(g_init_mu);
        if (!d.ready.load(std::memory_order_relaxed)) {
            int n = 0;
            e = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev);
            if (e == hipSuccess) e = dt::tree_init();
            if (e == hipSuccess) e = dt::attn_init();
            void *sp = nullptr;
            if (e == hipSuccess) e = hipGetSymbolAddress(&sp, HIP_SYMBOL(g_scratch));
            if (e != hipSuccess || n < 1 || !sp) { g_last_hip = (int)e; (void)hipGetLastError(); return DT_ERR_HIP; }
            d.n_cu = n;
            d.scratch = sp;
            d.ready.store(1, std::memory_order_release);
        }
    }
    if (n_cu) *n_cu = d.n_cu;
    return DT_OK;
}

// the current device's copy of the library-owned scratch (after ensure_init succeeded on it)
void *device_scratch() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return nullptr;
    return g_dev[dev].ready.load(std::memory_order_acquire) ? g_dev[dev].scratch : nullptr;
}

// compute units for sizing a workspace: of the current device if there is one, else of an MI355X
// (the size is then an upper bound for any smaller part)
int cu_count_for_sizing() {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) == hipSuccess && dev >= 0 && dev < MAX_DEVICES) {
        if (g_dev[dev].ready.load(std::memory_order_acquire)) return g_dev[dev].n_cu;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0) return n;
    }
    (void)hipGetLastError();
    return 256;
}

// launch grids: x up to 2^31 - 1 workgroups, y and z up to 65535; rows ride in y and z (65535^2 of them),
// and the row selection takes one workgroup per row in x
constexpr int64_t GRID_X_MAX = 2147483647ll;
constexpr int GRID_YZ_MAX = 65535;

inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

inline bool bad_dtype(int t) { return t != DT_F32 && t != DT_BF16; }

// Smallest chunk multiplier that keeps a row within 64 chunks (the merge handles <= 64 lists).
inline int min_nl(int V) {
    for (int nl = 1; nl <= 4; nl <<= 1)
        if (dt::rows_chunks_per_row(V, nl) <= 64) return nl;
    return 0;
}
inline int pick_nl(int64_t n_rows, int V) {
    int a = dt::rows_pick_nl(n_rows, V), b = min_nl(V);
    return a > b ? a : b;
}
inline int max_chunks(int V) { return dt::rows_chunks_per_row(V, min_nl(V)); }

struct ArgmaxScratch {  // arg max rows: [rows, S] keys, [rows, S] (max, sum) pairs
    unsigned long long *keys;
    float2 *ms;
    size_t bytes;
};
inline ArgmaxScratch argmax_scratch(void *ws, int64_t rows, int S) {
    ArgmaxScratch r;
    size_t kb = align_up((size_t)rows * S * 8);
    r.keys = (unsigned long long *)ws;
    r.ms = (float2 *)((char *)ws + kb);
    r.bytes = kb + align_up((size_t)rows * S * 8);
    return r;
}
struct TopkScratch {  // top-k rows: [rows, S*256] lane maxima, [rows, S*4] (max, sum) pairs
    float *lane_max;
    float2 *ms;
    size_t bytes;
};
inline TopkScratch topk_scratch(void *ws, int64_t rows, int S) {
    TopkScratch r;
    size_t lb = align_up((size_t)rows * S * 256 * 4);
    r.lane_max = (float *)ws;
    r.ms = (float2 *)((char *)ws + lb);
    r.bytes = lb + align_up((size_t)rows * S * 4 * 8);
    return r;
}
inline bool topk_v_ok(int V) { return V >= 1 && dt::rows_chunks_per_row(V, dt::rows_topk_nl(V)) <= 64; }

struct LevelState {  // row results of one sequence after the other, then the per-sequence counts
    float *top_val;    // [batch, DT_STATE_ROWS, DT_K_MAX]
    int32_t *top_id;
    float *lse;        // [batch, DT_STATE_ROWS]
    int32_t *n_exp;    // [batch] nodes expanded at the last level processed
    size_t bytes;
};
inline LevelState level_state(void *st, int batch) {
    LevelState r;
    char *p = (char *)st;
    const size_t rows = (size_t)batch * DT_STATE_ROWS;
    size_t off = 0;
    r.top_val = (float *)(p + off); off += align_up(rows * DT_K_MAX * 4);
    r.top_id = (int32_t *)(p + off); off += align_up(rows * DT_K_MAX * 4);
    r.lse = (float *)(p + off); off += align_up(rows * 4);
    r.n_exp = (int32_t *)(p + off); off += align_up((size_t)batch * 4);
    r.bytes = off;
    return r;
}

inline int hip_fail(hipError_t e) {
    g_last_hip = (int)e;
    return DT_ERR_HIP;
}

}  // namespace

extern "C" {

const char *dt_status_string(int s) {
    switch (s) {
        case DT_OK: return "ok";
        case DT_ERR_INVALID_ARG: return "invalid argument";
        case DT_ERR_LIMIT: return "size exceeds a compiled limit";
        case DT_ERR_WORKSPACE: return "workspace missing or too small";
        case DT_ERR_DTYPE: return "no kernel for this dtype/shape";
        case DT_ERR_HIP: return "HIP call failed";
        default: return "unknown status";
    }
}

int dt_init(void) { return ensure_init(nullptr); }

int dt_last_hip_error(void) { return g_last_hip; }
const char *dt_hip_error_string(int code) { return hipGetErrorString((hipError_t)code); }

int dt_workspace_bytes(int batch, int64_t total_rows, int V, int TT_cap, int Hq, int D, size_t *bytes) {
    if (!bytes || batch < 0 || total_rows < 0 || Hq < 0 || D < 0) return DT_ERR_INVALID_ARG;
    if (V < 1 || TT_cap < 1 || TT_cap > DT_TT_MAX || min_nl(V) == 0 || !topk_v_ok(V)) return DT_ERR_LIMIT;
    const int S = max_chunks(V);
    const int St = dt::rows_chunks_per_row(V, dt::rows_topk_nl(V));
    // build: lane maxima + (max, sum) partials + merged top-k (values, ids) + lse
    const size_t state_rows = (size_t)batch * DT_STATE_ROWS;  // merged results: one block of rows per sequence
    size_t build = topk_scratch(nullptr, total_rows, St).bytes + 2 * align_up(state_rows * DT_K_MAX * 4) +
                   align_up(state_rows * 4);
    size_t accept = argmax_scratch(nullptr, (int64_t)batch * TT_cap, S).bytes + align_up((size_t)batch * TT_cap * 4);
    size_t attn = dt::attn_workspace_bytes(batch, TT_cap, Hq, D, cu_count_for_sizing());
    size_t m = build > accept ? build : accept;
    m = m > attn ? m : attn;
    *bytes = m + 256;
    return DT_OK;
}

int dt_topk_rows(void *stream, const void *logits, dt_dtype t, int64_t n_rows, int V, int64_t row_stride, int k,
                 float *top_val, int32_t *top_id, float *lse, void *ws, size_t ws_bytes) {
    if (!logits || !top_val || !top_id || !lse || n_rows < 0 || bad_dtype(t) || row_stride < V)
        return DT_ERR_INVALID_ARG;
    if (!topk_v_ok(V) || k < 1 || k > DT_K_MAX || k > V) return DT_ERR_LIMIT;
    if (n_rows == 0) return DT_OK;
    const int nl = dt::rows_topk_nl(V), S = dt::rows_chunks_per_row(V, nl);
    if (n_rows > GRID_X_MAX) return DT_ERR_LIMIT;
    if (!ws || (uintptr_t)ws % 256) return DT_ERR_WORKSPACE;
    TopkScratch rs = topk_scratch(ws, n_rows, S);
    if (rs.bytes > ws_bytes) return DT_ERR_WORKSPACE;
    if (int rc = ensure_init(nullptr)) return rc;
    dt::RowArgs a = {};
    a.logits = logits; a.dtype = t; a.V = V; a.row_stride = row_stride;
    a.mode = dt::ROWS_UNIFORM; a.k_uniform = k;
    a.want_lse = 1; a.inv_t = 1.0f;
    a.lane_max = rs.lane_max; a.part_ms = rs.ms;
    hipStream_t st = (hipStream_t)stream;
    (void)hipGetLastError();  // a stale error left by another HIP user of this process is not ours
    hipError_t e = dt::rows_launch_stream(a, n_rows, nl, st);
    if (e != hipSuccess) return hip_fail(e);
    e = dt::rows_launch_select(a, n_rows, nl, top_val, top_id, lse, k, st);
    if (e != hipSuccess) return hip_fail(e);
    return DT_OK;
}

int dt_topk_rows_static(void *stream, const void *logits, dt_dtype t, int64_t n_rows, int V, int64_t row_stride, int k,
                        float *top_val, int32_t *top_id, float *lse) {
    // the argument checks of dt_topk_rows come first, so that both calls refuse the same inputs alike
    if (!logits || !top_val || !top_id || !lse || n_rows < 0 || bad_dtype(t) || row_stride < V)
        return DT_ERR_INVALID_ARG;
    if (!topk_v_ok(V) || k < 1 || k > DT_K_MAX || k > V) return DT_ERR_LIMIT;
    if (n_rows == 0) return DT_OK;
    const int S = dt::rows_chunks_per_row(V, dt::rows_topk_nl(V));
    if (n_rows > GRID_X_MAX) return DT_ERR_LIMIT;
    if (topk_scratch(nullptr, n_rows, S).bytes > (size_t)DT_STATIC_SCRATCH_BYTES) return DT_ERR_LIMIT;
    if (int rc = ensure_init(nullptr)) return rc;
    void *ws = device_scratch();
    if (!ws) return DT_ERR_HIP;
    // nothing in this scratch has to start from zero: every word the selection reads is written by the
    // streaming pass of the same call
    return dt_topk_rows(stream, logits, t, n_rows, V, row_stride, k, top_val, top_id, lse, ws, DT_STATIC_SCRATCH_BYTES);
}

int dt_build_tree(void *stream, int batch, const dt_params *params, const void *draft_logits, dt_dtype t, int V,
                  int64_t row_stride, const int64_t *row_off, int64_t total_rows, const int32_t *root_token,
                  int TT_cap, int32_t *n_nodes, int32_t *tokens, int32_t *parents, int32_t *depth, float *score,
                  float *logp, int32_t *src_row, uint64_t *anc_mask, void *ws, size_t ws_bytes, int flags) {
    if (batch < 0 || total_rows < 0 || bad_dtype(t) || (flags & ~DT_TREE_EARLY_STOP)) return DT_ERR_INVALID_ARG;
    if (batch == 0) return DT_OK;
    if (!params || !draft_logits || !row_off || !root_token || !n_nodes || !tokens || !parents || !depth ||
        !score || !logp || !src_row || !anc_mask || row_stride < V)
        return DT_ERR_INVALID_ARG;
    if (!topk_v_ok(V) || TT_cap < 1 || TT_cap > DT_TT_MAX) return DT_ERR_LIMIT;
    if (total_rows < batch) return DT_ERR_INVALID_ARG;  // every sequence owns at least its root row
    const int nl = dt::rows_topk_nl(V), S = dt::rows_chunks_per_row(V, nl);
    if (total_rows > GRID_X_MAX) return DT_ERR_LIMIT;
    if (!ws || (uintptr_t)ws % 256) return DT_ERR_WORKSPACE;
    char *wsd = (char *)ws;
    TopkScratch rs = topk_scratch(wsd, total_rows, S);
    size_t off = rs.bytes;
    // merged row results: sequence b's row r at row b * DT_STATE_ROWS + r, the layout the tree kernel reads
    const size_t state_rows = (size_t)batch * DT_STATE_ROWS;
    float *top_val = (float *)(wsd + off); off += align_up(state_rows * DT_K_MAX * 4);
    int32_t *top_id = (int32_t *)(wsd + off); off += align_up(state_rows * DT_K_MAX * 4);
    float *lse = (float *)(wsd + off); off += align_up(state_rows * 4);
    if (off > ws_bytes) return DT_ERR_WORKSPACE;
    if (int rc = ensure_init(nullptr)) return rc;

    dt::RowArgs a = {};
    a.logits = draft_logits; a.dtype = t; a.V = V; a.row_stride = row_stride;
    a.mode = dt::ROWS_DRAFT; a.batch = batch; a.params = params; a.row_off = row_off; a.TT_cap = TT_cap;
    a.want_lse = 1; a.inv_t = 1.0f;
    a.lane_max = rs.lane_max; a.part_ms = rs.ms;
    hipStream_t st = (hipStream_t)stream;
    (void)hipGetLastError();  // a stale error left by another HIP user of this process is not ours
    hipError_t e = dt::rows_launch_stream(a, total_rows, nl, st);
    if (e != hipSuccess) return hip_fail(e);
    e = dt::rows_launch_select(a, total_rows, nl, top_val, top_id, lse, DT_K_MAX, st);
    if (e != hipSuccess) return hip_fail(e);

    dt::TreeArgs ta = {};
    ta.batch = batch; ta.params = params; ta.V = V; ta.seq_rows = DT_STATE_ROWS; ta.root_token = root_token;
    ta.TT_cap = TT_cap; ta.top_val = top_val; ta.top_id = top_id; ta.lse = lse; ta.row_off = row_off;
    ta.early_stop = flags & DT_TREE_EARLY_STOP;
    ta.n_nodes = n_nodes; ta.tokens = tokens; ta.parents = parents; ta.depth = depth; ta.src_row = src_row;
    ta.score = score; ta.logp = logp; ta.anc_mask = (unsigned long long *)anc_mask;
    e = dt::tree_launch(ta, st);
    if (e != hipSuccess) return hip_fail(e);
    return DT_OK;
}

int dt_tree_attention(void *stream, int batch, dt_dtype t, int Hq, int Hkv, int D, float scale, const void *q,
                      const void *k_tree, const void *v_tree, const int32_t *n_nodes, const void *const *k_prefix,
                      const void *const *v_prefix, const int32_t *prefix_len, int max_prefix_len,
                      int64_t kv_stride_tok, int64_t kv_stride_head, const uint64_t *anc_mask, int TT_cap,
                      void *out, void *ws, size_t ws_bytes) {
    if (batch < 0 || bad_dtype(t)) return DT_ERR_INVALID_ARG;
    if (batch == 0) return DT_OK;
    if (!q || !k_tree || !v_tree || !n_nodes || !k_prefix || !v_prefix || !prefix_len || !anc_mask || !out)
        return DT_ERR_INVALID_ARG;
    if (Hq < 1 || Hkv < 1 || Hq % Hkv || D < 1 || max_prefix_len < 0 || !(scale > 0.0f) || kv_stride_tok < 0 ||
        kv_stride_head < 0)
        return DT_ERR_INVALID_ARG;
    if (TT_cap < 1 || TT_cap > DT_TT_MAX || D > 128 || batch > GRID_YZ_MAX / 8 || Hq > GRID_YZ_MAX) return DT_ERR_LIMIT;
    if ((uintptr_t)q % 16 || (uintptr_t)k_tree % 16 || (uintptr_t)v_tree % 16 || (uintptr_t)out % 16)
        return DT_ERR_INVALID_ARG;
    if (ws && (uintptr_t)ws % 256) return DT_ERR_WORKSPACE;
    int n_cu = 0;
    if (int rc = ensure_init(&n_cu)) return rc;
    dt::AttnArgs a = {};
    a.n_cu = n_cu;
    a.batch = batch; a.dtype = t; a.Hq = Hq; a.Hkv = Hkv; a.D = D; a.scale = scale;
    a.q = q; a.k_tree = k_tree; a.v_tree = v_tree; a.n_nodes = n_nodes;
    a.k_prefix = k_prefix; a.v_prefix = v_prefix; a.prefix_len = prefix_len; a.max_prefix_len = max_prefix_len;
    a.kv_stride_tok = kv_stride_tok; a.kv_stride_head = kv_stride_head;
    a.anc_mask = (const unsigned long long *)anc_mask; a.TT_cap = TT_cap; a.out = out;
    a.ws = ws; a.ws_bytes = ws ? ws_bytes : 0;
    hipError_t e = hipSuccess;
    (void)hipGetLastError();  // a stale error left by another HIP user of this process is not ours
    int rc = dt::attn_launch(a, (hipStream_t)stream, &e);
    if (rc == DT_ERR_HIP) return hip_fail(e);
    return rc;
}

int dt_accept(void *stream, int batch, dt_accept_mode mode, float temperature, const void *target_logits, dt_dtype t,
              int V, int64_t row_stride, const int32_t *n_nodes, const int32_t *tokens, const int32_t *parents,
              const int32_t *depth, const float *logp, const uint64_t *anc_mask, int TT_cap, uint64_t philox_seed,
              uint64_t philox_step, int32_t *accept_len, int32_t *best_node, int32_t *path_nodes,
              int32_t *out_tokens, int32_t *node_argmax, void *ws, size_t ws_bytes) {
    if (batch < 0 || bad_dtype(t)) return DT_ERR_INVALID_ARG;
    if (mode != DT_ACCEPT_GREEDY && mode != DT_ACCEPT_STOCHASTIC && mode != DT_ACCEPT_SAMPLED) return DT_ERR_INVALID_ARG;
    if (batch == 0) return DT_OK;
    if (!target_logits || !n_nodes || !tokens || !parents || !depth || !anc_mask || !accept_len || !best_node ||
        !path_nodes || !out_tokens || row_stride < V)
        return DT_ERR_INVALID_ARG;
    if (mode == DT_ACCEPT_STOCHASTIC && !logp) return DT_ERR_INVALID_ARG;
    if (mode != DT_ACCEPT_GREEDY && !(temperature > 0.0f)) return DT_ERR_INVALID_ARG;
    if (V < 1 || min_nl(V) == 0 || TT_cap < 1 || TT_cap > DT_TT_MAX) return DT_ERR_LIMIT;
    const int64_t rows = (int64_t)batch * TT_cap;
    const int nl = pick_nl(rows, V), S = dt::rows_chunks_per_row(V, nl);
    if (rows > GRID_X_MAX) return DT_ERR_LIMIT;
    if (!ws || (uintptr_t)ws % 256) return DT_ERR_WORKSPACE;
    ArgmaxScratch rs = argmax_scratch(ws, rows, S);
    int32_t *samples = (int32_t *)((char *)ws + rs.bytes);  // target-sampled mode: one token per node
    if (rs.bytes + align_up((size_t)rows * 4) > ws_bytes) return DT_ERR_WORKSPACE;
    if (int rc = ensure_init(nullptr)) return rc;

    dt::RowArgs a = {};
    a.logits = target_logits; a.dtype = t; a.V = V; a.row_stride = row_stride;
    a.mode = dt::ROWS_TARGET; a.batch = batch; a.TT_cap = TT_cap; a.n_nodes = n_nodes;
    a.want_lse = mode != DT_ACCEPT_GREEDY; a.inv_t = mode != DT_ACCEPT_GREEDY ? 1.0f / temperature : 1.0f;
    a.part_keys = rs.keys; a.part_ms = rs.ms;
    hipStream_t st = (hipStream_t)stream;
    (void)hipGetLastError();  // a stale error left by another HIP user of this process is not ours
    hipError_t e = dt::rows_launch_argmax(a, rows, nl, st);
    if (e != hipSuccess) return hip_fail(e);

    dt::AcceptArgs aa = {};
    aa.batch = batch; aa.mode = mode; aa.temperature = temperature; aa.target = target_logits; aa.dtype = t;
    aa.V = V; aa.row_stride = row_stride; aa.n_nodes = n_nodes; aa.tokens = tokens; aa.parents = parents;
    aa.depth = depth; aa.logp = logp; aa.anc_mask = (const unsigned long long *)anc_mask; aa.TT_cap = TT_cap;
    aa.seed = philox_seed; aa.step = philox_step; aa.accept_len = accept_len; aa.best_node = best_node;
    aa.path_nodes = path_nodes; aa.out_tokens = out_tokens; aa.node_argmax = node_argmax;
    aa.part_keys = rs.keys; aa.part_ms = rs.ms; aa.S = S; aa.chunk_elems = 256 * 8 * nl; aa.samples = samples;
    e = dt::accept_launch(aa, st);
    if (e != hipSuccess) return hip_fail(e);
    return DT_OK;
}

int dt_level_state_bytes(int batch, size_t *bytes) {
    if (!bytes || batch < 0) return DT_ERR_INVALID_ARG;
    *bytes = level_state(nullptr, batch).bytes;
    return DT_OK;
}

int dt_expand_level(void *stream, int batch, int level, const dt_params *params, const void *level_logits, dt_dtype t,
                    int V, int64_t row_stride, int rows_per_seq, const int32_t *prefix_len, int TT_cap, void *state,
                    int32_t *n_expand, int32_t *exp_token, int32_t *exp_parent_slot, int32_t *exp_row, int32_t *exp_pos,
                    uint64_t *exp_mask, void *ws, size_t ws_bytes, int flags) {
    if (batch < 0 || bad_dtype(t) || level < 1 || level > DT_D_MAX || (flags & ~DT_TREE_EARLY_STOP)) return DT_ERR_INVALID_ARG;
    if (batch == 0) return DT_OK;
    if (!params || !level_logits || !state || !n_expand || !exp_token || !exp_parent_slot || !exp_row || !exp_pos ||
        !exp_mask || row_stride < V || (uintptr_t)state % 256)
        return DT_ERR_INVALID_ARG;
    if (rows_per_seq < 1 || rows_per_seq > DT_K_MAX) return DT_ERR_INVALID_ARG;
    if (!topk_v_ok(V) || TT_cap < 1 || TT_cap > DT_TT_MAX) return DT_ERR_LIMIT;
    const int rps = level == 1 ? 1 : rows_per_seq;
    const int64_t total_rows = (int64_t)batch * rps;
    const int nl = dt::rows_topk_nl(V), S = dt::rows_chunks_per_row(V, nl);
    if (!ws || (uintptr_t)ws % 256) return DT_ERR_WORKSPACE;
    TopkScratch rs = topk_scratch(ws, total_rows, S);
    if (rs.bytes > ws_bytes) return DT_ERR_WORKSPACE;
    if (total_rows > GRID_X_MAX) return DT_ERR_LIMIT;
    if (int rc = ensure_init(nullptr)) return rc;
    LevelState ls = level_state(state, batch);

    dt::RowArgs a = {};
    a.logits = level_logits; a.dtype = t; a.V = V; a.row_stride = row_stride;
    a.mode = dt::ROWS_LEVEL; a.batch = batch; a.params = params; a.TT_cap = TT_cap;
    a.level = level; a.rows_per_seq = rps; a.state_rows = DT_STATE_ROWS; a.n_exp_prev = ls.n_exp;
    a.want_lse = 1; a.inv_t = 1.0f;
    a.lane_max = rs.lane_max; a.part_ms = rs.ms;
    hipStream_t st = (hipStream_t)stream;
    (void)hipGetLastError();  // a stale error left by another HIP user of this process is not ours
    hipError_t e = dt::rows_launch_stream(a, total_rows, nl, st);
    if (e != hipSuccess) return hip_fail(e);
    e = dt::rows_launch_select(a, total_rows, nl, ls.top_val, ls.top_id, ls.lse, DT_K_MAX, st);
    if (e != hipSuccess) return hip_fail(e);

    dt::TreeArgs ta = {};
    ta.batch = batch; ta.params = params; ta.V = V; ta.seq_rows = DT_STATE_ROWS;
    ta.TT_cap = TT_cap; ta.top_val = ls.top_val; ta.top_id = ls.top_id; ta.lse = ls.lse;
    ta.expand_level = level; ta.prefix_len = prefix_len; ta.n_expand = n_expand; ta.state_n_exp = ls.n_exp;
    ta.exp_token = exp_token; ta.exp_parent_slot = exp_parent_slot; ta.exp_row = exp_row; ta.exp_pos = exp_pos;
    ta.exp_mask = (unsigned long long *)exp_mask;
    ta.early_stop = flags & DT_TREE_EARLY_STOP;
    e = dt::tree_launch(ta, st);
    if (e != hipSuccess) return hip_fail(e);
    return DT_OK;
}

int dt_finish_tree(void *stream, int batch, const dt_params *params, int V, const int32_t *root_token, int TT_cap,
                   const void *state, int32_t *n_nodes, int32_t *tokens, int32_t *parents, int32_t *depth, float *score,
                   float *logp, int32_t *src_row, uint64_t *anc_mask, int flags) {
    if (batch < 0 || (flags & ~DT_TREE_EARLY_STOP)) return DT_ERR_INVALID_ARG;
    if (batch == 0) return DT_OK;
    if (!params || !root_token || !state || !n_nodes || !tokens || !parents || !depth || !score || !logp || !src_row ||
        !anc_mask || (uintptr_t)state % 256)
        return DT_ERR_INVALID_ARG;
    if (V < 1 || TT_cap < 1 || TT_cap > DT_TT_MAX) return DT_ERR_LIMIT;
    if (int rc = ensure_init(nullptr)) return rc;
    LevelState ls = level_state((void *)state, batch);
    dt::TreeArgs ta = {};
    ta.batch = batch; ta.params = params; ta.V = V; ta.seq_rows = DT_STATE_ROWS;
    ta.root_token = root_token; ta.TT_cap = TT_cap; ta.top_val = ls.top_val; ta.top_id = ls.top_id; ta.lse = ls.lse;
    ta.n_nodes = n_nodes; ta.tokens = tokens; ta.parents = parents; ta.depth = depth; ta.src_row = src_row;
    ta.score = score; ta.logp = logp; ta.anc_mask = (unsigned long long *)anc_mask;
    ta.early_stop = flags & DT_TREE_EARLY_STOP;
    (void)hipGetLastError();  // a stale error left by another HIP user of this process is not ours
    hipError_t e = dt::tree_launch(ta, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(e);
    return DT_OK;
}

int dt_action_table(dt_params *table, int capacity, int *n_actions) {
    // Appendix A, "Action Space in Implementation": the printed value sets, combinations with
    // TT > k^(d-1) filtered out; enumeration order TT, then d, then k
    static const int TTs[] = {32, 48, 64, 80, 96, 128}, ds[] = {3, 4, 5, 6, 7, 8}, ks[] = {8, 12, 16, 20, 32};
    if (!n_actions || capacity < 0 || (capacity > 0 && !table)) return DT_ERR_INVALID_ARG;
    int n = 0;
    for (int TT : TTs)
        for (int d : ds)
            for (int k : ks) {
                long long lim = 1;  // k^(d-1), saturated well above every TT
                for (int i = 1; i < d && lim < (1 << 20); ++i) lim *= k;
                if (TT > lim) continue;
                if (n < capacity) { table[n].TT = TT; table[n].d = d; table[n].k = k; }
                ++n;
            }
    *n_actions = n;
    return DT_OK;
}

int dt_policy_workspace_bytes(int batch, int F, int H, size_t *bytes) {
    if (!bytes || batch < 0 || F < 1 || H < 1) return DT_ERR_INVALID_ARG;
    const size_t S = ((size_t)F + POLICY_KS - 1) / POLICY_KS;
    *bytes = align_up(S * (size_t)batch * H * 4) + 256;
    return DT_OK;
}

int dt_policy_step(void *stream, int batch, dt_dtype feat_t, const void *features, int64_t feat_stride, int F, int H,
                   int n_actions, const float *W1, const float *b1, const float *W2, const float *b2, const float *W3,
                   const float *b3, const dt_params *action_table, int cache_interval, int sample, uint64_t philox_seed,
                   uint64_t philox_step, int32_t *cache_step, int32_t *cached_action, dt_params *params_out,
                   int32_t *action_out, int32_t *queried_out, float *logits_out, void *ws, size_t ws_bytes) {
    if (batch < 0 || bad_dtype(feat_t)) return DT_ERR_INVALID_ARG;
    if (batch == 0) return DT_OK;
    if (!features || !W1 || !b1 || !W2 || !b2 || !W3 || !b3 || !action_table || !cache_step || !cached_action ||
        !params_out || feat_stride < F || F < 1 || cache_interval < 1 || (sample != 0 && sample != 1))
        return DT_ERR_INVALID_ARG;
    if ((H != 64 && H != 128) || n_actions < 1 || n_actions > 256) return DT_ERR_LIMIT;
    size_t need = 0;
    dt_policy_workspace_bytes(batch, F, H, &need);
    if (!ws || (uintptr_t)ws % 256 || ws_bytes < need) return DT_ERR_WORKSPACE;
    dt::PolicyArgs a = {};
    a.batch = batch; a.feat_dtype = feat_t; a.F = F; a.H = H; a.A = n_actions; a.N = cache_interval; a.mode = sample;
    a.feat = features; a.feat_stride = feat_stride;
    a.W1 = W1; a.b1 = b1; a.W2 = W2; a.b2 = b2; a.W3 = W3; a.b3 = b3; a.table = action_table;
    a.seed = philox_seed; a.step = philox_step; a.cache_step = cache_step; a.cached_action = cached_action;
    a.params_out = params_out; a.action_out = action_out; a.queried_out = queried_out; a.logits_out = logits_out;
    a.partial = (float *)ws; a.S = (F + POLICY_KS - 1) / POLICY_KS;
    (void)hipGetLastError();  // a stale error left by another HIP user of this process is not ours
    hipError_t e = dt::policy_launch(a, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(e);
    return DT_OK;
}

int dt_reward_step(void *stream, int batch, const int32_t *accept_len, int count_bonus, float elapsed_seconds,
                   const float *elapsed_per_seq, const int32_t *cache_step, float *reward_sum, int32_t *reward_steps,
                   float *reward_avg, int32_t *interval_done) {
    if (batch < 0) return DT_ERR_INVALID_ARG;
    if (batch == 0) return DT_OK;
    if (!accept_len || !cache_step || !reward_sum || !reward_steps || !reward_avg || !interval_done ||
        (count_bonus != 0 && count_bonus != 1) || (!elapsed_per_seq && !(elapsed_seconds > 0.0f)))
        return DT_ERR_INVALID_ARG;
    dt::RewardArgs a = {};
    a.batch = batch; a.count_bonus = count_bonus; a.elapsed = elapsed_seconds; a.elapsed_dev = elapsed_per_seq;
    a.accept_len = accept_len; a.cache_step = cache_step; a.reward_sum = reward_sum; a.reward_steps = reward_steps;
    a.reward_avg = reward_avg; a.interval_done = interval_done;
    (void)hipGetLastError();  // a stale error left by another HIP user of this process is not ours
    hipError_t e = dt::reward_launch(a, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(e);
    return DT_OK;
}

int dt_commit(void *stream, int batch, int n_layers, dt_dtype t, int Hkv, int D, const void *const *k_tree,
              const void *const *v_tree, void *const *k_prefix, void *const *v_prefix, const int32_t *prefix_len,
              const int32_t *prefix_cap, int64_t kv_stride_tok, int64_t kv_stride_head, const int32_t *n_nodes,
              const int32_t *path_nodes, const int32_t *accept_len, const int32_t *out_tokens, int TT_cap,
              int32_t *new_prefix_len, int32_t *next_root_token) {
    if (batch < 0 || n_layers < 0 || bad_dtype(t)) return DT_ERR_INVALID_ARG;
    if (batch == 0 || n_layers == 0) return DT_OK;
    if (!k_tree || !v_tree || !k_prefix || !v_prefix || !prefix_len || !prefix_cap || !n_nodes || !path_nodes ||
        !accept_len || !out_tokens || !new_prefix_len || new_prefix_len == prefix_len)
        return DT_ERR_INVALID_ARG;
    if (Hkv < 1 || D < 1 || kv_stride_tok < 1 || kv_stride_head < 1) return DT_ERR_INVALID_ARG;
    if (TT_cap < 1 || TT_cap > DT_TT_MAX || n_layers > 65535) return DT_ERR_LIMIT;
    dt::CommitArgs a = {};
    a.batch = batch; a.n_layers = n_layers; a.dtype = t; a.Hkv = Hkv; a.D = D;
    a.k_tree = k_tree; a.v_tree = v_tree; a.k_prefix = k_prefix; a.v_prefix = v_prefix;
    a.prefix_len = prefix_len; a.prefix_cap = prefix_cap; a.kv_stride_tok = kv_stride_tok; a.kv_stride_head = kv_stride_head;
    a.n_nodes = n_nodes; a.path_nodes = path_nodes; a.accept_len = accept_len; a.out_tokens = out_tokens; a.TT_cap = TT_cap;
    const int esz = t == DT_BF16 ? 2 : 4;
    a.vec16 = (D * esz) % 16 == 0 && (kv_stride_tok * esz) % 16 == 0 && (kv_stride_head * esz) % 16 == 0;
    a.new_prefix_len = new_prefix_len; a.next_root_token = next_root_token;
    (void)hipGetLastError();  // a stale error left by another HIP user of this process is not ours
    hipError_t e = dt::commit_launch(a, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(e);
    return DT_OK;
}

}  // extern "C"
