// Visibility-mask builder: ancestor closure of the token graph, one work-group per sequence.
//
// Paper Section 4.1 lets a flattened token attend only to its ancestors; on the merged graph of Section 5.3
// that set is the closure over all parent edges.  Rows live in LDS as packed 32-bit words and are relaxed
//     row[i] <- bit(i) | OR_{p in parents(i)} row[p]
// in data-flow order: a node takes its parents' rows as soon as they are final and publishes its own with a flag;
// no work-group barrier inside the closure.  The chain of dependent layers is what the kernel's time consists of, and a
// single wavefront issues one instruction every few cycles however few of its lanes are busy, so a node is not one lane
// but a group of L lanes, one per 32-bit word of its row: a layer then costs a handful of instructions (each lane reads
// one word per parent, ORs them and writes one word) instead of a row's worth.  A wavefront holds 64 / L nodes (a
// "chunk"), the chunks are dealt round-robin to the work-group's wavefronts, and a wavefront takes its chunks in
// ascending order.  Nodes are in topological order and only earlier nodes are ever waited for: the lowest unfinished
// node is ready, and its wavefront is working either on its chunk or on an earlier one, whose nodes are all finished
// or ready as well; so every poll loop ends.  It is bounded on top of that, so every wave leaves the kernel.
#include "gsd_internal.h"

namespace gsd {

constexpr int kEdgeCacheInts = 6144;   // per-sequence parent lists are staged in LDS when they fit
constexpr int kMaskThreads = 512;

template <int W>
__global__ __launch_bounds__(kMaskThreads) void build_mask_kernel(
    int32_t max_nodes, int32_t words_per_row, const int32_t *__restrict__ node_offsets,
    const int32_t *__restrict__ parent_offsets, const int32_t *__restrict__ parent_idx, uint64_t *__restrict__ mask,
    int32_t *__restrict__ dag_error_flag) {
    constexpr int D = 2 * W;                                           // 32-bit words of a row
    constexpr int L = D <= 2 ? 2 : D <= 4 ? 4 : D <= 8 ? 8 : 16;       // lanes of a node (a power of two)
    constexpr int G = 64 / L;                                          // nodes of a wavefront's chunk
    constexpr int kWaves = kMaskThreads / 64;
    __shared__ __attribute__((aligned(16))) uint32_t rows[GSD_MAX_NODES_PER_SEQ * D];     // [n][D]
    __shared__ int32_t edge_cache[kEdgeCacheInts];
    __shared__ int32_t off_cache[GSD_MAX_NODES_PER_SEQ + 1];
    __shared__ int32_t done_at[GSD_MAX_NODES_PER_SEQ + 1];

    const int b = blockIdx.x;
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

    for (int i = threadIdx.x; i <= n; i += kMaskThreads) {
        off_cache[i] = parent_offsets[base + i] - e0;
        done_at[i] = i == n ? 1 : 0;                         // slot n: final from the start, what an absent parent reads
    }
    if (cached)
        for (int e = threadIdx.x; e < e1 - e0; e += kMaskThreads) edge_cache[e] = parent_idx[e0 + e];
    __syncthreads();

    // parent e of this sequence, from the LDS copy or (sequences with more edges than the cache holds) from memory
    auto edge_at = [&](int e) -> int { return cached ? edge_cache[e] : parent_idx[e0 + e]; };
    // No instruction: the compiler keeps the LDS accesses before it before those after it, and reads LDS again after it.
    auto in_this_order = [] { asm volatile("" ::: "memory"); };
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int d = lane % L;                                  // this lane's word of the row
    const int slot = lane / L;                               // this lane's node within the chunk
    constexpr int kRegParents = 4;
    constexpr int kPollLimit = 1 << 16;
    const int chunks = (n + G - 1) / G;
    for (int c = wave; c < chunks; c += kWaves) {            // uniform per wavefront
        const int i = c * G + slot;
        const bool active = i < n && d < D;
        // The first four parents live in registers as two indices each, so that a poll's reads carry no branches: an
        // absent parent reads the node's own word, which holds nothing yet (OR-ing it in changes nothing), and slot n
        // of done_at, which is final from the start.
        int par_row[kRegParents], par_done[kRegParents];
        int e_lo = 0, e_hi = 0;
#pragma unroll
        for (int x = 0; x < kRegParents; ++x) {
            par_row[x] = active ? i : 0;
            par_done[x] = n;
        }
        uint32_t mine = 0;
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
            mine = d == (i >> 5) ? 1u << (i & 31) : 0u;
            rows[i * D + d] = 0;
        }
        const bool more = active && e_hi - e_lo > kRegParents;     // rare: a node with more than four parents
        bool mine_done = !active;
        for (int poll = 0; poll < kPollLimit; ++poll) {
            if (!mine_done) {
                // One batch of LDS reads per poll: the parents' flags, then, without waiting for them, this lane's
                // word of the parents' rows.  The LDS unit serves a wavefront's instructions in the order they were
                // issued (and the owner of a row writes the row before the flag), so a row word read after a flag that
                // turned out to be set is final; if a flag was not set the words are thrown away.
                in_this_order();
                int fin[kRegParents];
#pragma unroll
                for (int x = 0; x < kRegParents; ++x) fin[x] = done_at[par_done[x]];
                in_this_order();
                uint32_t got = 0;
#pragma unroll
                for (int x = 0; x < kRegParents; ++x) got |= rows[par_row[x] * D + d];
                bool ready = true;
#pragma unroll
                for (int x = 0; x < kRegParents; ++x) ready &= fin[x] != 0;
                if (more) {
                    for (int e = e_lo + kRegParents; e < e_hi; ++e) {
                        const int pp = edge_at(e);
                        if (pp >= 0 && pp < i) {
                            in_this_order();
                            const int f = done_at[pp];
                            in_this_order();
                            got |= rows[pp * D + d];
                            ready &= f != 0;
                        } else if (pp != -1) {
                            bad = true;
                        }
                    }
                }
                if (ready) {
                    mine |= got;
                    rows[i * D + d] = mine;
                    // The flag after the row: the lanes of a node take the same decision (same parents, and a flag
                    // comes from one instruction for all of them), so all words of the row are written by the one
                    // instruction above, and the flag by a later one.
                    in_this_order();
                    if (d == 0) done_at[i] = 1;
                    in_this_order();
                    mine_done = true;
                }
            }
            if (__all(mine_done)) break;          // wave-uniform
        }
        if (!mine_done) {                         // poll limit reached (never, with the guarantees above): publish what
            bad = true;                           // there is, so that nobody waits for this node for as long again
            rows[i * D + d] = mine;
            in_this_order();
            if (d == 0) done_at[i] = 1;
            in_this_order();
        }
    }
    __syncthreads();

    // rows to memory, one 64-bit word per thread and turn; words that no node id can reach are zero
    for (int x = threadIdx.x; x < n * words_per_row; x += kMaskThreads) {
        const int i = x / words_per_row, w = x - i * words_per_row;
        uint64_t v = 0;
        if (w < W) v = uint64_t(rows[i * D + 2 * w]) | (uint64_t(rows[i * D + 2 * w + 1]) << 32);
        mask[(base + i) * words_per_row + w] = v;
    }
    if (bad && dag_error_flag) *dag_error_flag = 1;
}

hipError_t launch_build_mask(int32_t batch, int32_t max_nodes, int32_t words_per_row, const int32_t *node_offsets,
                             const int32_t *parent_offsets, const int32_t *parent_idx, uint64_t *mask,
                             int32_t *dag_error_flag, hipStream_t stream) {
    const dim3 grid(batch), block(kMaskThreads);
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
