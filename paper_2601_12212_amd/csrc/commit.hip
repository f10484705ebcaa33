// Input update after verification: the K/V rows of the accepted path (root .. deepest accepted
// node) are appended to every layer's prefix cache; rejected tree tokens are simply never copied.
// One workgroup per (sequence, layer, K or V): at most DT_D_MAX + 1 rows of Hkv * D elements each,
// moved in 16-byte pieces when the layout allows it.  The new prefix length (= position of the next
// root, the bonus token) and the next root token are written by the workgroups of layer 0.
#include "common.hpp"
#include "kernels.hpp"

namespace dt {

template <typename T>
__device__ __forceinline__ void copy_rows(const CommitArgs &a, const T *tree, T *cache, int L, int rows, const int *node,
                                          int per_head /* units of T per head */) {
    // unit u of a row = (head g, piece c); the cache strides are given in elements, T holds `epu` of them
    const int epu = sizeof(T) / (a.dtype == DT_BF16 ? 2 : 4);
    const int64_t stok = a.kv_stride_tok / epu, shead = a.kv_stride_head / epu;
    const int per_row = a.Hkv * per_head;
    for (int i = threadIdx.x; i < rows * per_row; i += blockDim.x) {
        const int s = i / per_row, u = i % per_row, g = u / per_head, c = u % per_head;
        cache[(int64_t)(L + s) * stok + (int64_t)g * shead + c] = tree[((int64_t)node[s] * a.Hkv + g) * per_head + c];
    }
}

__global__ __launch_bounds__(256) void commit_kernel(CommitArgs a) {
    const int b = blockIdx.x, layer = blockIdx.y, kv = blockIdx.z;
    __shared__ int s_node[DT_D_MAX + 1];
    const int N = min(max(a.n_nodes[b], 1), a.TT_cap);
    const int len = min(max(a.accept_len[b], 0), DT_D_MAX);
    const int cap = max(a.prefix_cap[b], 0);
    const int L = min(max(a.prefix_len[b], 0), cap);
    const int rows = min(len + 1, cap - L);  // rows that still fit
    if ((int)threadIdx.x <= len)  // a node index outside the tree (bad input) is clamped, never followed
        s_node[threadIdx.x] = min(max(a.path_nodes[(int64_t)b * (DT_D_MAX + 1) + threadIdx.x], 0), N - 1);
    __syncthreads();
    if (layer == 0 && kv == 0 && threadIdx.x == 0) {
        a.new_prefix_len[b] = L + rows;
        if (a.next_root_token) a.next_root_token[b] = a.out_tokens[(int64_t)b * (DT_D_MAX + 1) + len];
    }
    if (rows <= 0) return;
    const void *tree = (kv ? a.v_tree : a.k_tree)[layer];
    void *cache = (kv ? a.v_prefix : a.k_prefix)[(int64_t)layer * a.batch + b];
    const int esz = a.dtype == DT_BF16 ? 2 : 4;
    const int64_t tree_seq = (int64_t)b * a.TT_cap * a.Hkv * a.D;  // elements before this sequence's tree rows
    const char *tp = (const char *)tree + tree_seq * esz;
    const bool vec = a.vec16 && ((uintptr_t)tp % 16 == 0) && ((uintptr_t)cache % 16 == 0);
    if (vec) copy_rows<uint4>(a, (const uint4 *)tp, (uint4 *)cache, L, rows, s_node, a.D * esz / 16);
    else if (esz == 2) copy_rows<uint16_t>(a, (const uint16_t *)tp, (uint16_t *)cache, L, rows, s_node, a.D);
    else copy_rows<uint32_t>(a, (const uint32_t *)tp, (uint32_t *)cache, L, rows, s_node, a.D);
}

hipError_t commit_launch(const CommitArgs &a, hipStream_t st) {
    if (a.batch <= 0 || a.n_layers <= 0) return hipSuccess;
    launch_kernel(KID_COMMIT, st, commit_kernel, dim3(a.batch, a.n_layers, 2), dim3(256), 0, a);
    return hipGetLastError();
}

}  // namespace dt
