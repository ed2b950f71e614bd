// Visibility-mask builder: ancestor closure of the token graph, one work-group per sequence.
//
// Paper Section 4.1 lets a flattened token attend only to its ancestors; on the merged graph of Section 5.3
// that set is the closure over all parent edges.  Rows live in LDS as packed 64-bit words and are relaxed
//     row[i] <- bit(i) | OR_{p in parents(i)} row[p]
// for all (node, word) items in parallel until nothing changes.  Nodes are in topological order, so the
// relaxation reaches its (unique) fixed point after at most depth+1 sweeps; the loop is also hard-bounded by
// the node count, so every wave leaves the kernel.  A sweep costs one LDS round trip and one barrier.
#include "gsd_internal.h"

namespace gsd {

constexpr int kMaskThreads = 1024;
constexpr int kEdgeCacheInts = 6144;   // per-sequence parent lists are staged in LDS when they fit

__global__ __launch_bounds__(kMaskThreads) void build_mask_kernel(
    int32_t max_nodes, int32_t words_per_row, const int32_t *__restrict__ node_offsets,
    const int32_t *__restrict__ parent_offsets, const int32_t *__restrict__ parent_idx,
    uint64_t *__restrict__ mask, int32_t *__restrict__ dag_error_flag) {
    extern __shared__ uint64_t rows[];                       // [n][W]
    __shared__ int32_t edge_cache[kEdgeCacheInts];
    __shared__ int32_t off_cache[GSD_MAX_NODES_PER_SEQ + 1];

    const int b = blockIdx.x;
    const int W = words_per_row;
    const int64_t base = node_offsets[b];
    int n = node_offsets[b + 1] - node_offsets[b];
    bool bad = false;
    if (n > max_nodes) {                                     // caller's bound was wrong: flag, process what fits
        n = max_nodes;
        bad = true;
    }
    if (n <= 0) return;
    const int items = n * W;
    const int32_t e0 = parent_offsets[base];
    const int32_t e1 = parent_offsets[base + n];
    const bool cached = (e1 - e0) <= kEdgeCacheInts;

    for (int i = threadIdx.x; i <= n; i += kMaskThreads) off_cache[i] = parent_offsets[base + i] - e0;
    if (cached)
        for (int e = threadIdx.x; e < e1 - e0; e += kMaskThreads) edge_cache[e] = parent_idx[e0 + e];
    for (int idx = threadIdx.x; idx < items; idx += kMaskThreads) {
        const int i = idx / W, w = idx - i * W;
        rows[idx] = (w == (i >> 6)) ? (uint64_t(1) << (i & 63)) : uint64_t(0);
    }
    __syncthreads();
    const int32_t *edges = cached ? edge_cache : (parent_idx + e0);

    // Each thread owns up to kItemsPerThread (node, word) items and keeps the first kRegParents parent ids of
    // each in registers, so a sweep is a handful of independent LDS reads; convergence is signalled through three
    // rotating LDS flags (set in sweep s, read after its barrier, cleared during sweep s+1 for sweep s+2).
    constexpr int kItemsPerThread = (GSD_MAX_NODES_PER_SEQ * 8 + kMaskThreads - 1) / kMaskThreads;   // 4096 words max
    constexpr int kRegParents = 4;
    int item_node[kItemsPerThread], item_word[kItemsPerThread], item_deg[kItemsPerThread];
    int item_par[kItemsPerThread][kRegParents];
#pragma unroll
    for (int q = 0; q < kItemsPerThread; ++q) {
        const int idx = threadIdx.x + q * kMaskThreads;
        item_node[q] = -1;
        item_word[q] = 0;
        item_deg[q] = 0;
#pragma unroll
        for (int x = 0; x < kRegParents; ++x) item_par[q][x] = -1;
        if (idx < items) {
            const int i = idx / W;
            item_node[q] = i;
            item_word[q] = idx - i * W;
            const int e_lo = off_cache[i], e_hi = off_cache[i + 1];
            item_deg[q] = e_hi - e_lo;
#pragma unroll
            for (int x = 0; x < kRegParents; ++x) {
                if (e_lo + x < e_hi) {
                    const int pp = edges[e_lo + x];
                    if (pp >= 0 && pp < i) item_par[q][x] = pp;
                    else if (pp != -1) bad = true;
                }
            }
        }
    }
    __shared__ int changed_flag[3];
    if (threadIdx.x < 3) changed_flag[threadIdx.x] = 0;
    __syncthreads();

    for (int sweep = 0; sweep <= n; ++sweep) {
        bool changed = false;
#pragma unroll
        for (int q = 0; q < kItemsPerThread; ++q) {
            const int i = item_node[q];
            if (i < 0) continue;
            const int w = item_word[q];
            const int idx = i * W + w;
            const uint64_t cur = rows[idx];
            uint64_t acc = cur;
#pragma unroll
            for (int x = 0; x < kRegParents; ++x)
                if (item_par[q][x] >= 0) acc |= rows[item_par[q][x] * W + w];
            for (int e = off_cache[i] + kRegParents; e < off_cache[i] + item_deg[q]; ++e) {   // rare: more parents
                const int pp = edges[e];
                if (pp >= 0 && pp < i) acc |= rows[pp * W + w];
                else if (pp != -1) bad = true;
            }
            if (acc != cur) {
                rows[idx] = acc;
                changed = true;
            }
        }
        const int slot = sweep % 3;
        if (changed) changed_flag[slot] = 1;
        if (threadIdx.x == 0) changed_flag[(sweep + 1) % 3] = 0;
        __syncthreads();
        if (changed_flag[slot] == 0) break;       // uniform: everybody reads the same flag after the barrier
    }

    uint64_t *out = mask + base * W;
    for (int idx = threadIdx.x; idx < items; idx += kMaskThreads) out[idx] = rows[idx];
    if (bad && dag_error_flag) *dag_error_flag = 1;
}

hipError_t launch_build_mask(int32_t batch, int32_t max_nodes, int32_t words_per_row, const int32_t *node_offsets,
                             const int32_t *parent_offsets, const int32_t *parent_idx, uint64_t *mask,
                             int32_t *dag_error_flag, hipStream_t stream) {
    const size_t lds = size_t(max_nodes) * words_per_row * sizeof(uint64_t);
    hipLaunchKernelGGL(build_mask_kernel, dim3(batch), dim3(kMaskThreads), lds, stream, max_nodes, words_per_row,
                       node_offsets, parent_offsets, parent_idx, mask, dag_error_flag);
    return hipGetLastError();
}

}  // namespace gsd
