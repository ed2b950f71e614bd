// KV-cache commit of the accepted path (paper Section 7.1: the cache update is a cost of its own).
//
// Per sequence, layer and K|V the accepted draft rows are compacted in place behind the prefix:
//     row P+j <- row P+path[j],  j = 0 .. accept_len-1,  path strictly increasing so path[j] >= j.
// HBM-bound: 2 * (rows that move) * row_bytes bytes per (sequence, layer, K|V).  A work-group owns up to 256 of the
// 16-byte columns of one (sequence, layer, K|V) and takes the destination rows in chunks of 4096/columns rows: every
// thread loads its 16 (row, column) pieces of the chunk, all loads in flight at once, the work-group meets at a
// barrier, then every thread stores.  In place is safe: a source row is never below its destination and sources only
// grow, so a chunk reads rows at or above its first destination row and writes only its own destination rows after
// the barrier, and the chunks that follow read only rows above those.  Different columns never touch each other's
// bytes.  Rows already in place (path[j] == j) are neither read nor written.
#include "gsd_internal.h"

namespace gsd {

constexpr int kCommitThreads = 256;
constexpr int kPieces = 16;                                   // 16-byte pieces a thread holds between load and store
constexpr int kChunkPieces = kCommitThreads * kPieces;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // (HIP's uint4 class keeps such arrays out of registers)

__global__ __launch_bounds__(kCommitThreads) void commit_kv_kernel(
    int32_t max_nodes, int vecs_per_row, char *__restrict__ k, char *__restrict__ v, int64_t token_stride,
    int64_t layer_stride, const int64_t *__restrict__ kv_offsets, const int32_t *__restrict__ prefix_lens,
    const int32_t *__restrict__ accept_len, const int32_t *__restrict__ accept_path,
    int32_t *__restrict__ new_prefix_lens) {
    __shared__ int32_t src_of[GSD_MAX_NODES_PER_SEQ];         // source row of destination row j, or -1: nothing to move
    const int b = blockIdx.z >> 1;
    const int which = blockIdx.z & 1;
    const int layer = blockIdx.y;
    const int col0 = blockIdx.x * kCommitThreads;
    const int cols = min(kCommitThreads, vecs_per_row - col0);          // >= 1 by the grid's construction
    // every index this work-group needs is fetched in one round trip: the path entries do not wait for the length
    static_assert(GSD_MAX_NODES_PER_SEQ <= 2 * kCommitThreads, "two path entries per thread cover a sequence");
    const int32_t *path = accept_path + int64_t(b) * max_nodes;
    const int j_a = threadIdx.x, j_b = threadIdx.x + kCommitThreads;
    const int32_t s_a = j_a < max_nodes ? path[j_a] : -1;
    const int32_t s_b = j_b < max_nodes ? path[j_b] : -1;
    int len = accept_len[b];
    const int P = prefix_lens[b];
    const int64_t seq_row0 = kv_offsets[b];
    if (len > max_nodes) len = max_nodes;
    if (which == 0 && layer == 0 && blockIdx.x == 0 && threadIdx.x == 0) new_prefix_lens[b] = P + (len > 0 ? len : 0);
    if (len <= 0) return;                                               // uniform for the work-group

    if (j_a < len) src_of[j_a] = (s_a > j_a && s_a < max_nodes) ? s_a : -1;     // s == j: already in place
    if (j_b < len) src_of[j_b] = (s_b > j_b && s_b < max_nodes) ? s_b : -1;
    __syncthreads();

    char *rows = (which ? v : k) + layer * layer_stride + (seq_row0 + P) * token_stride + int64_t(col0) * 16;
    const int rows_per_chunk = kChunkPieces / cols;                     // >= kPieces
    for (int j0 = 0; j0 < len; j0 += rows_per_chunk) {
        const int pieces = min(rows_per_chunk, len - j0) * cols;
        u32x4 held[kPieces];
        int64_t dst[kPieces];                                           // byte offset of the destination, -1: no store
        // loads without branches: a piece that does not exist or does not move reads its own destination instead
#pragma unroll
        for (int x = 0; x < kPieces; ++x) {
            const int idx = min(int(threadIdx.x) + x * kCommitThreads, pieces - 1);
            const int r = idx / cols, c = idx - r * cols;
            const int j = j0 + r;
            const int s = src_of[j];
            const bool moves = s >= 0 && int(threadIdx.x) + x * kCommitThreads < pieces;
            dst[x] = moves ? int64_t(j) * token_stride + c * 16 : -1;
            held[x] = *reinterpret_cast<const u32x4 *>(rows + int64_t(moves ? s : j) * token_stride + c * 16);
        }
        __syncthreads();                                                // every source of the chunk has been read
#pragma unroll
        for (int x = 0; x < kPieces; ++x)
            if (dst[x] >= 0) *reinterpret_cast<u32x4 *>(rows + dst[x]) = held[x];
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
