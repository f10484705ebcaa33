// Optional per-kernel timing (used by the benchmark to report the achieved bandwidth of
// individual kernels): HIP events attached to each kernel dispatch record its begin and end.
// Events are created when profiling is switched on, never on the launch path.
#include <hip/hip_runtime.h>

#include <vector>

#include "kernels.hpp"

namespace {
struct Pair {
    hipEvent_t a, b;
};
bool g_on = false;
std::vector<Pair> g_pool;            // pre-created pairs
std::vector<int> g_used[dt::KID_COUNT];  // indices into g_pool, per kernel id
size_t g_next = 0;
}  // namespace

namespace dt {
bool prof_next(int kid, hipEvent_t *start, hipEvent_t *stop) {
    if (!g_on || g_next >= g_pool.size()) return false;
    const int idx = (int)g_next++;
    *start = g_pool[idx].a;
    *stop = g_pool[idx].b;
    g_used[kid].push_back(idx);
    return true;
}
}  // namespace dt

extern "C" {

int dt_profile_enable(int max_launches) {
    for (int k = 0; k < dt::KID_COUNT; ++k) g_used[k].clear();
    g_next = 0;
    if (max_launches <= 0) { g_on = false; return DT_OK; }
    while ((int)g_pool.size() < max_launches) {
        Pair p;
        if (hipEventCreate(&p.a) != hipSuccess || hipEventCreate(&p.b) != hipSuccess) return DT_ERR_HIP;
        g_pool.push_back(p);
    }
    g_on = true;
    return DT_OK;
}

int dt_profile_read(int kernel_id, double *total_ms, int *launches) {
    if (kernel_id < 0 || kernel_id >= dt::KID_COUNT || !total_ms || !launches) return DT_ERR_INVALID_ARG;
    double tot = 0.0;
    for (int idx : g_used[kernel_id]) {
        float ms = 0.f;
        if (hipEventSynchronize(g_pool[idx].b) != hipSuccess) return DT_ERR_HIP;
        if (hipEventElapsedTime(&ms, g_pool[idx].a, g_pool[idx].b) != hipSuccess) return DT_ERR_HIP;
        tot += ms;
    }
    *total_ms = tot;
    *launches = (int)g_used[kernel_id].size();
    return DT_OK;
}

const char *dt_profile_kernel_name(int kernel_id) {
    static const char *names[] = {"rows_draft_chunk", "rows_merge", "tree", "attention", "attention_combine",
                                  "rows_target_chunk", "accept", "rows_uniform_chunk", "commit", "policy_layer1", "policy_head", "node_sample",
                                  "reward"};
    return (kernel_id >= 0 && kernel_id < dt::KID_COUNT) ? names[kernel_id] : "?";
}
}
