// KV-cache commit of the accepted path (paper Section 7.1: the cache update is a cost of its own).
//
// Per sequence, layer and K|V the accepted draft rows are compacted in place behind the prefix:
//     row P+j <- row P+path[j],  j = 0 .. accept_len-1,  path strictly increasing so path[j] >= j.
// HBM-bound: 2 * accept_len * row_bytes bytes per (sequence, layer, K|V).  A thread owns one 16-byte column of
// the rows and walks j upwards in groups of kGroup: it loads the group's source rows, then stores them.  Because
// a destination j is never above its source and sources only grow, a row is always read (by this thread, in this
// column) before anything overwrites it; different columns never touch each other's bytes, so no
// synchronisation is needed at all.
#include "gsd_internal.h"

namespace gsd {

constexpr int kCommitThreads = 256;
constexpr int kGroup = 8;

__global__ __launch_bounds__(kCommitThreads) void commit_kv_kernel(
    int32_t max_nodes, int vecs_per_row, char *__restrict__ k, char *__restrict__ v, int64_t token_stride,
    int64_t layer_stride, const int64_t *__restrict__ kv_offsets, const int32_t *__restrict__ prefix_lens,
    const int32_t *__restrict__ accept_len, const int32_t *__restrict__ accept_path,
    int32_t *__restrict__ new_prefix_lens) {
    const int b = blockIdx.z >> 1;
    const int which = blockIdx.z & 1;
    const int layer = blockIdx.y;
    const int col = blockIdx.x * kCommitThreads + threadIdx.x;
    int len = accept_len[b];
    if (len > max_nodes) len = max_nodes;
    const int P = prefix_lens[b];
    if (which == 0 && layer == 0 && col == 0) new_prefix_lens[b] = P + (len > 0 ? len : 0);
    if (col >= vecs_per_row || len <= 0) return;

    char *rows = (which ? v : k) + layer * layer_stride + (kv_offsets[b] + P) * token_stride + int64_t(col) * 16;
    const int32_t *path = accept_path + int64_t(b) * max_nodes;
    for (int j0 = 0; j0 < len; j0 += kGroup) {
        uint4 held[kGroup];
        bool move[kGroup];
#pragma unroll
        for (int x = 0; x < kGroup; ++x) {
            const int j = j0 + x;
            move[x] = false;
            if (j < len) {
                const int s = path[j];
                if (s > j && s < max_nodes) {              // s == j: already in place
                    held[x] = *reinterpret_cast<const uint4 *>(rows + int64_t(s) * token_stride);
                    move[x] = true;
                }
            }
        }
#pragma unroll
        for (int x = 0; x < kGroup; ++x)
            if (move[x]) *reinterpret_cast<uint4 *>(rows + int64_t(j0 + x) * token_stride) = held[x];
    }
}

hipError_t launch_commit_kv(int32_t batch, int32_t max_nodes, int32_t num_layers, int64_t row_bytes, void *k, void *v,
                            int64_t token_stride, int64_t layer_stride, const int64_t *kv_offsets,
                            const int32_t *prefix_lens, const int32_t *accept_len, const int32_t *accept_path,
                            int32_t *new_prefix_lens, hipStream_t stream) {
    const int vecs = int(row_bytes / 16);
    dim3 grid((vecs + kCommitThreads - 1) / kCommitThreads, num_layers, batch * 2);
    hipLaunchKernelGGL(commit_kv_kernel, grid, dim3(kCommitThreads), 0, stream, max_nodes, vecs, (char *)k, (char *)v,
                       token_stride, layer_stride, kv_offsets, prefix_lens, accept_len, accept_path, new_prefix_lens);
    return hipGetLastError();
}

}  // namespace gsd
