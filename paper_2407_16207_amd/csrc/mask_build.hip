// Visibility-mask builder: ancestor closure of the token graph, one work-group per sequence.
//
// Paper Section 4.1 lets a flattened token attend only to its ancestors; on the merged graph of Section 5.3
// that set is the closure over all parent edges.  Rows live in LDS as packed 64-bit words and are relaxed
//     row[i] <- bit(i) | OR_{p in parents(i)} row[p]
// in data-flow order: a node takes its parents' rows as soon as they are final and publishes its own with a flag;
// every wavefront polls the flags of its own nodes' parents, no work-group barrier inside the loop.  Nodes are in
// topological order, so the lowest unfinished node is always ready, and the loop is bounded on top of that, so every
// wave leaves the kernel.  One thread per node holds the node's whole row (W words) and its first four parent ids in
// registers; a poll is four narrow LDS reads (are my parents final?), then, once, the wide reads of the parents' rows.
#include "gsd_internal.h"

namespace gsd {

constexpr int kEdgeCacheInts = 6144;   // per-sequence parent lists are staged in LDS when they fit

template <int W>
__global__ __launch_bounds__(GSD_MAX_NODES_PER_SEQ) void build_mask_kernel(
    int32_t max_nodes, int32_t words_per_row, const int32_t *__restrict__ node_offsets,
    const int32_t *__restrict__ parent_offsets, const int32_t *__restrict__ parent_idx, uint64_t *__restrict__ mask,
    int32_t *__restrict__ dag_error_flag) {
    __shared__ __attribute__((aligned(16))) uint64_t rows[GSD_MAX_NODES_PER_SEQ * W];     // [n][W]
    __shared__ int32_t edge_cache[kEdgeCacheInts];
    __shared__ int32_t off_cache[GSD_MAX_NODES_PER_SEQ + 1];
    __shared__ int32_t done_at[GSD_MAX_NODES_PER_SEQ + 1];

    const int b = blockIdx.x;
    const int threads = blockDim.x;                          // >= max_nodes: one node per thread
    const int64_t base = node_offsets[b];
    int n = node_offsets[b + 1] - node_offsets[b];
    bool bad = false;
    if (n > max_nodes) {                                     // caller's bound was wrong: flag, process what fits
        n = max_nodes;
        bad = true;
    }
    if (n <= 0) return;
    const int32_t e0 = parent_offsets[base];
    const int32_t e1 = parent_offsets[base + n];
    const bool cached = (e1 - e0) <= kEdgeCacheInts;

    for (int i = threadIdx.x; i <= n; i += threads) off_cache[i] = parent_offsets[base + i] - e0;
    if (cached)
        for (int e = threadIdx.x; e < e1 - e0; e += threads) edge_cache[e] = parent_idx[e0 + e];
    __syncthreads();

    const int i = threadIdx.x;
    const bool active = i < n;
    constexpr int kRegParents = 4;
    // The first four parents live in registers as two indices each, so that a sweep's reads carry no branches (a
    // branch per parent serialises the LDS round trips): an absent parent reads the node's own row (OR-ing it in
    // changes nothing) and slot n of done_at, which is final from the start.
    int par_row[kRegParents], par_done[kRegParents];
    int e_lo = 0, e_hi = 0;
    uint64_t r[W];
#pragma unroll
    for (int w = 0; w < W; ++w) r[w] = 0;
#pragma unroll
    for (int x = 0; x < kRegParents; ++x) {
        par_row[x] = active ? i : 0;
        par_done[x] = n;
    }
    // parent e of this sequence, from the LDS copy or (sequences with more edges than the cache holds) from memory
    auto edge_at = [&](int e) -> int { return cached ? edge_cache[e] : parent_idx[e0 + e]; };
    if (active) {
        e_lo = off_cache[i];
        e_hi = off_cache[i + 1];
#pragma unroll
        for (int x = 0; x < kRegParents; ++x) {
            if (e_lo + x < e_hi) {
                const int pp = edge_at(e_lo + x);
                if (pp >= 0 && pp < i) {
                    par_row[x] = pp;
                    par_done[x] = pp;
                } else if (pp != -1) {
                    bad = true;
                }
            }
        }
#pragma unroll
        for (int w = 0; w < W; ++w) {
            r[w] = (w == (i >> 6)) ? (uint64_t(1) << (i & 63)) : uint64_t(0);
            rows[i * W + w] = r[w];
        }
        done_at[i] = 0;
    }
    if (threadIdx.x == 0) done_at[n] = 1;
    __syncthreads();
    const bool more = active && e_hi - e_lo > kRegParents;     // rare: a node with more than four parents

    // Data flow instead of sweeps with barriers: a node takes its parents' rows as soon as all of them are final
    // (done_at[p] != 0, published after the row itself; LDS operations of a wave complete in order), and is final
    // itself from then on.  Every wave polls on its own; the wavefronts of a work-group are all resident, nodes are in
    // topological order and only earlier nodes are ever waited for, so the lowest unfinished node is always ready and
    // every poll of its wave finishes it: the loop ends after at most depth+1 productive polls per wave.  It is bounded
    // all the same (kPollLimit polls; a wave that hits the bound reports the graph as bad and writes what it has).
    auto is_final = [&](int node) -> bool {     // relaxed LDS read that the compiler may neither cache nor drop
        return __hip_atomic_load(&done_at[node], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) != 0;
    };
    bool mine_done = !active;
    constexpr int kPollLimit = 1 << 16;
    for (int poll = 0; poll < kPollLimit; ++poll) {
        if (!mine_done) {
            bool ready = true;
#pragma unroll
            for (int x = 0; x < kRegParents; ++x) ready &= is_final(par_done[x]);
            if (more) {
                for (int e = e_lo + kRegParents; e < e_hi; ++e) {
                    const int pp = edge_at(e);
                    if (pp >= 0 && pp < i) ready &= is_final(pp);
                    else if (pp != -1) bad = true;
                }
            }
            if (ready) {
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");     // the rows are read after their flags
#pragma unroll
                for (int x = 0; x < kRegParents; ++x)
#pragma unroll
                    for (int w = 0; w < W; ++w) r[w] |= rows[par_row[x] * W + w];
                if (more) {
                    for (int e = e_lo + kRegParents; e < e_hi; ++e) {
                        const int pp = edge_at(e);
                        if (pp >= 0 && pp < i) {
#pragma unroll
                            for (int w = 0; w < W; ++w) r[w] |= rows[pp * W + w];
                        }
                    }
                }
#pragma unroll
                for (int w = 0; w < W; ++w) rows[i * W + w] = r[w];
                __hip_atomic_store(&done_at[i], 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);   // after the row
                mine_done = true;
            }
        }
        if (__all(mine_done)) break;              // wave-uniform
    }
    if (!mine_done) bad = true;                   // poll limit reached (never, with the guarantees above)

    if (active) {
        uint64_t *out = mask + (base + i) * words_per_row;
#pragma unroll
        for (int w = 0; w < W; ++w) out[w] = r[w];
        for (int w = W; w < words_per_row; ++w) out[w] = 0;   // rows wider than any node id can reach
    }
    if (bad && dag_error_flag) *dag_error_flag = 1;
}

hipError_t launch_build_mask(int32_t batch, int32_t max_nodes, int32_t words_per_row, const int32_t *node_offsets,
                             const int32_t *parent_offsets, const int32_t *parent_idx, uint64_t *mask,
                             int32_t *dag_error_flag, hipStream_t stream) {
    const dim3 grid(batch), block((max_nodes + 63) / 64 * 64);
#define GSD_MASK_CASE(WORDS)                                                                                         \
    case WORDS:                                                                                                      \
        hipLaunchKernelGGL(build_mask_kernel<WORDS>, grid, block, 0, stream, max_nodes, words_per_row, node_offsets,  \
                           parent_offsets, parent_idx, mask, dag_error_flag);                                        \
        break;
    // words computed per row: no node id reaches past word GSD_MAX_NODES_PER_SEQ/64 - 1, wider rows are zero-filled
    static_assert(GSD_MAX_NODES_PER_SEQ == 512, "the cases below cover 512 / 64 = 8 words");
    switch (words_per_row < 8 ? words_per_row : 8) {
        GSD_MASK_CASE(1) GSD_MASK_CASE(2) GSD_MASK_CASE(3) GSD_MASK_CASE(4)
        GSD_MASK_CASE(5) GSD_MASK_CASE(6) GSD_MASK_CASE(7) GSD_MASK_CASE(8)
        default: return hipErrorInvalidValue;
    }
#undef GSD_MASK_CASE
    return hipGetLastError();
}

}  // namespace gsd
