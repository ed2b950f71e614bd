// Un-merging a token graph into a token tree (paper Section 5.4), one work-group per sequence.
//
// The tree has one node per root path of the graph.  With c[i] = number of root paths ending at graph node i,
//     c[i] = sum over parents p of i of (p == root ? 1 : c[p]),
// the replicas of node i are numbered first[i] .. first[i]+c[i]-1 with first = exclusive prefix sum of c, and the
// replica reached through parent slot s from the r-th replica of that parent p is
//     first[i] + (sum of c over the earlier slots) + r,      with tree parent  first[p] + r   (root: -1).
// So nothing is enumerated: counts are settled in LDS level by level (nodes are in topological order, so that
// takes depth+1 sweeps; the loop is hard-bounded by the node count), a scan gives `first`, and
// every tree node below the cap finds its (origin, slot, r) by a binary search and a walk over one parent list.
// Counts saturate at 2^62, far above any cap, so sums never wrap.
#include "gsd_internal.h"

namespace gsd {

constexpr int kUnmergeThreads = 512;                      // one thread per graph node
constexpr uint64_t kPathCap = uint64_t(1) << 62;

__device__ __forceinline__ uint64_t sat_add(uint64_t a, uint64_t b) {
    const uint64_t s = a + b;                             // a, b <= 2^62: no wrap
    return s > kPathCap ? kPathCap : s;
}

// Path counts and their exclusive scan for the calling work-group's sequence.  cnt[0..n), first[0..n]; returns
// true if a malformed edge was met.  All threads of the work-group must call it.
// Level-synchronous: a node adds up its parents' counts once, in the first sweep that finds all of them final
// (done_at[p] = sweep in which cnt[p] became final, compared against the current sweep so that only counts
// finished before the last barrier are used).  The first four parents of a node sit in registers, an absent one
// reading slot n (final from the start, count 0), so a sweep's reads carry no branch per parent.
__device__ bool count_paths(int n, int64_t base, const int32_t *__restrict__ parent_offsets,
                            const int32_t *__restrict__ parent_idx, uint64_t *cnt /* [n+1] */, uint64_t *first,
                            int32_t *done_at /* [n+1] */, int *flags) {
    constexpr int kRegParents = 4;
    const int i = threadIdx.x;
    const bool active = i < n;
    bool bad = false;
    int e_lo = 0, e_hi = 0;
    int par[kRegParents];                                  // slot in cnt / done_at: a parent id, or n
    uint64_t roots = 0;                                    // edges from the root among the first four
#pragma unroll
    for (int x = 0; x < kRegParents; ++x) par[x] = n;
    if (active) {
        e_lo = parent_offsets[base + i];
        e_hi = parent_offsets[base + i + 1];
        if (e_hi > e_lo) {
            int p[kRegParents];
#pragma unroll
            for (int x = 0; x < kRegParents; ++x) p[x] = parent_idx[min(e_lo + x, e_hi - 1)];
#pragma unroll
            for (int x = 0; x < kRegParents; ++x) {
                if (e_lo + x >= e_hi) continue;
                if (p[x] == -1) roots += 1;
                else if (p[x] >= 0 && p[x] < i) par[x] = p[x];
                else bad = true;
            }
        }
        cnt[i] = 0;
        done_at[i] = 0x7fffffff;
    }
    if (i == 0) {
        cnt[n] = 0;
        done_at[n] = -1;
    }
    if (i < 3) flags[i] = 0;
    __syncthreads();
    const bool more = active && e_hi - e_lo > kRegParents;     // rare: a node with more than four parents
    bool mine_done = !active;
    for (int sweep = 0; sweep <= n; ++sweep) {
        bool finished = false;
        if (!mine_done) {
            bool ready = true;
#pragma unroll
            for (int x = 0; x < kRegParents; ++x) ready &= done_at[par[x]] < sweep;
            if (more) {
                for (int e = e_lo + kRegParents; e < e_hi; ++e) {
                    const int p = parent_idx[e];
                    if (p >= 0 && p < i) ready &= done_at[p] < sweep;
                }
            }
            if (ready) {
                uint64_t acc = roots;
#pragma unroll
                for (int x = 0; x < kRegParents; ++x) acc = sat_add(acc, cnt[par[x]]);
                if (more) {
                    for (int e = e_lo + kRegParents; e < e_hi; ++e) {
                        const int p = parent_idx[e];
                        if (p == -1) acc = sat_add(acc, 1);
                        else if (p >= 0 && p < i) acc = sat_add(acc, cnt[p]);
                        else bad = true;
                    }
                }
                cnt[i] = acc;
                done_at[i] = sweep;
                mine_done = true;
                finished = true;
            }
        }
        const int slot = sweep % 3;
        if (finished) flags[slot] = 1;
        if (i == 0) flags[(sweep + 1) % 3] = 0;
        __syncthreads();
        if (flags[slot] == 0) break;                      // uniform: read after the barrier
    }
    // exclusive scan (saturating addition is associative on [0, 2^62]); first[n] = total.  Within a wave by shuffles,
    // across waves through the eight wave totals.
    __shared__ uint64_t wave_total[kUnmergeThreads / 64];
    const int lane = i & 63, wave = i >> 6;
    uint64_t v = i < n ? cnt[i] : 0;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint64_t up = __shfl_up(static_cast<unsigned long long>(v), d, 64);
        if (lane >= d) v = sat_add(v, up);
    }
    if (lane == 63) wave_total[wave] = v;
    __syncthreads();
    uint64_t before = 0;
#pragma unroll
    for (int w = 0; w < kUnmergeThreads / 64; ++w)
        if (w < wave) before = sat_add(before, wave_total[w]);
    first[i + 1] = sat_add(before, v);
    if (i == 0) first[0] = 0;
    __syncthreads();
    return bad;
}

__global__ __launch_bounds__(kUnmergeThreads) void unmerge_count_kernel(
    int32_t max_nodes, const int32_t *__restrict__ node_offsets, const int32_t *__restrict__ parent_offsets,
    const int32_t *__restrict__ parent_idx, int64_t *__restrict__ path_count, int32_t *__restrict__ dag_error_flag) {
    __shared__ uint64_t cnt[kUnmergeThreads + 1];
    __shared__ uint64_t first[kUnmergeThreads + 1];
    __shared__ int32_t done_at[kUnmergeThreads + 1];
    __shared__ int flags[3];
    const int b = blockIdx.x;
    const int64_t base = node_offsets[b];
    int n = node_offsets[b + 1] - node_offsets[b];
    bool bad = false;
    if (n > max_nodes) {
        n = max_nodes;
        bad = true;
    }
    if (n < 0) n = 0;
    bad |= count_paths(n, base, parent_offsets, parent_idx, cnt, first, done_at, flags);
    if (threadIdx.x == 0) path_count[b] = int64_t(first[n]);
    if (bad && dag_error_flag) *dag_error_flag = 1;
}

__global__ __launch_bounds__(kUnmergeThreads) void unmerge_fill_kernel(
    int32_t batch, int32_t max_nodes, int32_t max_tree_nodes, const int32_t *__restrict__ node_offsets,
    const int32_t *__restrict__ parent_offsets, const int32_t *__restrict__ parent_idx,
    const int64_t *__restrict__ path_count, int32_t *__restrict__ tree_node_offsets,
    int32_t *__restrict__ tree_parent, int32_t *__restrict__ tree_parent_offsets, int32_t *__restrict__ tree_origin) {
    __shared__ uint64_t cnt[kUnmergeThreads + 1];
    __shared__ uint64_t first[kUnmergeThreads + 1];
    __shared__ int32_t done_at[kUnmergeThreads + 1];
    __shared__ int flags[3];
    __shared__ int wave_sum[kUnmergeThreads / 64];
    const int b = blockIdx.x;

    // packed position of this sequence's tree: sum of the capped sizes of the sequences before it
    int mine = 0;
    for (int s = threadIdx.x; s < b; s += kUnmergeThreads) {
        const int64_t c = path_count[s];
        mine += int(c < max_tree_nodes ? c : max_tree_nodes);
    }
    for (int d = 32; d > 0; d >>= 1) mine += __shfl_xor(mine, d);
    if ((threadIdx.x & 63) == 0) wave_sum[threadIdx.x >> 6] = mine;
    __syncthreads();
    int tree_base = 0;
    for (int w = 0; w < kUnmergeThreads / 64; ++w) tree_base += wave_sum[w];

    const int64_t base = node_offsets[b];
    int n = node_offsets[b + 1] - node_offsets[b];
    if (n > max_nodes) n = max_nodes;
    if (n < 0) n = 0;
    count_paths(n, base, parent_offsets, parent_idx, cnt, first, done_at, flags);
    const uint64_t total = first[n];
    const int n_tree = int(total < uint64_t(max_tree_nodes) ? total : uint64_t(max_tree_nodes));

    if (threadIdx.x == 0) {
        tree_node_offsets[b] = tree_base;
        if (b == batch - 1) {
            tree_node_offsets[batch] = tree_base + n_tree;
            if (tree_parent_offsets) tree_parent_offsets[tree_base + n_tree] = tree_base + n_tree;
        }
    }
    for (int t = threadIdx.x; t < n_tree; t += kUnmergeThreads) {
        // origin = the last node i with first[i] <= t  (nodes without root paths have empty ranges)
        int lo = 0, hi = n;                               // invariant: first[lo] <= t < first[hi]
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (first[mid] <= uint64_t(t)) lo = mid;
            else hi = mid;
        }
        const int i = lo;
        uint64_t r = uint64_t(t) - first[i];
        int parent = -1;
        for (int e = parent_offsets[base + i]; e < parent_offsets[base + i + 1]; ++e) {
            const int p = parent_idx[e];
            uint64_t c;
            if (p == -1) c = 1;
            else if (p >= 0 && p < i) c = cnt[p];
            else continue;
            if (r < c) {
                parent = p == -1 ? -1 : int(first[p] + r);
                break;
            }
            r -= c;
        }
        tree_parent[tree_base + t] = parent;
        tree_origin[tree_base + t] = i;
        if (tree_parent_offsets) tree_parent_offsets[tree_base + t] = tree_base + t;
    }
}

hipError_t launch_unmerge(int32_t batch, int32_t max_nodes, int32_t max_tree_nodes, const int32_t *node_offsets,
                          const int32_t *parent_offsets, const int32_t *parent_idx, int32_t *tree_node_offsets,
                          int32_t *tree_parent, int32_t *tree_parent_offsets, int32_t *tree_origin,
                          int64_t *path_count, int32_t *dag_error_flag, hipStream_t stream) {
    hipLaunchKernelGGL(unmerge_count_kernel, dim3(batch), dim3(kUnmergeThreads), 0, stream, max_nodes, node_offsets,
                       parent_offsets, parent_idx, path_count, dag_error_flag);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    hipLaunchKernelGGL(unmerge_fill_kernel, dim3(batch), dim3(kUnmergeThreads), 0, stream, batch, max_nodes,
                       max_tree_nodes, node_offsets, parent_offsets, parent_idx, path_count, tree_node_offsets,
                       tree_parent, tree_parent_offsets, tree_origin);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------- row gather
template <typename Vec>
__global__ __launch_bounds__(256) void gather_rows_kernel(int64_t rows, int vecs_per_row, const char *__restrict__ src,
                                                          int64_t src_rows, int64_t src_stride,
                                                          const int32_t *__restrict__ index, char *__restrict__ dst,
                                                          int64_t dst_stride) {
    // blockIdx.x walks rows (grid-stride), threads walk a row's vectors
    for (int64_t r = blockIdx.x; r < rows; r += gridDim.x) {
        const int64_t s = index[r];
        if (s < 0 || s >= src_rows) continue;
        const Vec *in = reinterpret_cast<const Vec *>(src + s * src_stride);
        Vec *out = reinterpret_cast<Vec *>(dst + r * dst_stride);
        for (int c = threadIdx.x; c < vecs_per_row; c += 256) out[c] = in[c];
    }
}

hipError_t launch_gather_rows(int64_t rows, int64_t row_bytes, const void *src, int64_t src_rows,
                              int64_t src_stride, const int32_t *index, void *dst, int64_t dst_stride,
                              hipStream_t stream) {
    const bool wide = row_bytes % 16 == 0 && src_stride % 16 == 0 && dst_stride % 16 == 0 &&
                      reinterpret_cast<uintptr_t>(src) % 16 == 0 && reinterpret_cast<uintptr_t>(dst) % 16 == 0;
    const int grid = int(rows < 65536 ? rows : 65536);
    if (wide)
        hipLaunchKernelGGL(gather_rows_kernel<uint4>, dim3(grid), dim3(256), 0, stream, rows, int(row_bytes / 16),
                           (const char *)src, src_rows, src_stride, index, (char *)dst, dst_stride);
    else
        hipLaunchKernelGGL(gather_rows_kernel<uint32_t>, dim3(grid), dim3(256), 0, stream, rows, int(row_bytes / 4),
                           (const char *)src, src_rows, src_stride, index, (char *)dst, dst_stride);
    return hipGetLastError();
}

}  // namespace gsd
