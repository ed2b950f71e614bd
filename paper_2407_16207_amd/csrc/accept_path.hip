// Longest accepted root path per sequence (deterministic verification, paper Sections 3 and 4.1).
//
// An edge p -> i is accepted iff tokens[i] equals the LLM's choice after p (pred[p], or root_pred for the
// root); the first mismatch on a hypothesis discards everything after it, and the longest accepted path from
// the root is taken.  One work-group per sequence: L[i] (nodes on the longest accepted root path ending at i,
// -1 if none) is relaxed over all nodes in parallel until it stops changing (at most depth+1 sweeps because
// the nodes are in topological order; hard bound = node count), then the best end node is reduced and one
// thread walks the back-pointers.  Ties: smallest end node id, then the smallest-id qualifying parent.
#include "gsd_internal.h"

namespace gsd {

constexpr int kAcceptThreads = 512;
constexpr int kAcceptEdgeCache = 6144;

__global__ __launch_bounds__(kAcceptThreads) void accept_kernel(
    int32_t max_nodes, const int32_t *__restrict__ node_offsets, const int32_t *__restrict__ parent_offsets,
    const int32_t *__restrict__ parent_idx, const int32_t *__restrict__ tokens, const int32_t *__restrict__ pred,
    const int32_t *__restrict__ root_pred, int32_t *__restrict__ accept_len, int32_t *__restrict__ accept_path,
    int32_t *__restrict__ bonus_token) {
    __shared__ int32_t L[GSD_MAX_NODES_PER_SEQ];
    __shared__ int32_t pred_s[GSD_MAX_NODES_PER_SEQ];
    __shared__ int32_t tok_s[GSD_MAX_NODES_PER_SEQ];
    __shared__ int32_t path_s[GSD_MAX_NODES_PER_SEQ];
    __shared__ int32_t back_s[GSD_MAX_NODES_PER_SEQ];
    __shared__ int32_t off_cache[GSD_MAX_NODES_PER_SEQ + 1];
    __shared__ int32_t edge_cache[kAcceptEdgeCache];
    __shared__ uint32_t wave_best[kAcceptThreads / 64];
    __shared__ int32_t len_s;

    const int b = blockIdx.x;
    const int64_t base = node_offsets[b];
    int n = node_offsets[b + 1] - node_offsets[b];
    if (n > max_nodes) n = max_nodes;
    if (n < 0) n = 0;
    const int32_t rp = root_pred[b];
    const int32_t e0 = parent_offsets[base];
    const int32_t e1 = parent_offsets[base + n];
    const bool cached = (e1 - e0) <= kAcceptEdgeCache;

    for (int i = threadIdx.x; i <= n; i += kAcceptThreads) off_cache[i] = parent_offsets[base + i] - e0;
    if (cached)
        for (int e = threadIdx.x; e < e1 - e0; e += kAcceptThreads) edge_cache[e] = parent_idx[e0 + e];
    for (int i = threadIdx.x; i < n; i += kAcceptThreads) {
        L[i] = -1;
        pred_s[i] = pred[base + i];
        tok_s[i] = tokens[base + i];
    }
    __syncthreads();
    // parent e of this sequence, from the LDS copy or (sequences with more edges than the cache holds) from memory
    auto edge_at = [&](int e) -> int { return cached ? edge_cache[e] : parent_idx[e0 + e]; };

    // One thread per node (kAcceptThreads >= GSD_MAX_NODES_PER_SEQ).  Whether an edge is accepted never changes,
    // so it is decided once; the first four parents of a node stay in registers as (id, accepted), which leaves a
    // sweep with four independent LDS reads and no branch per parent (branches serialise the round trips).
    static_assert(kAcceptThreads >= GSD_MAX_NODES_PER_SEQ, "one thread per node");
    constexpr int kRegParents = 4;
    const int i = threadIdx.x;
    const bool active = i < n;
    int par[kRegParents];          // parent id; -1 = root; -2 = no such edge, or not accepted
    int e_lo = 0, e_hi = 0;
    int32_t my_tok = 0;
#pragma unroll
    for (int x = 0; x < kRegParents; ++x) par[x] = -2;
    // is edge p -> i accepted (p is a well-formed parent of i)?
    auto accepted = [&](int p) -> bool { return my_tok == (p == -1 ? rp : pred_s[p]); };
    if (active) {
        e_lo = off_cache[i];
        e_hi = off_cache[i + 1];
        my_tok = tok_s[i];
#pragma unroll
        for (int x = 0; x < kRegParents; ++x) {
            if (e_lo + x < e_hi) {
                const int p = edge_at(e_lo + x);
                if (p >= -1 && p < i && accepted(p)) par[x] = p;
            }
        }
    }
    const bool more = active && e_hi - e_lo > kRegParents;     // rare: a node with more than four parents

    int32_t mine = -1;             // L[i]
    for (int sweep = 0; sweep <= n; ++sweep) {
        int changed = 0;
        if (active) {
            int32_t best = mine;
#pragma unroll
            for (int x = 0; x < kRegParents; ++x) {
                const int32_t l = L[par[x] >= 0 ? par[x] : i];
                const int32_t lp = par[x] >= 0 ? l : (par[x] == -1 ? 0 : -1);
                if (lp >= 0 && lp + 1 > best) best = lp + 1;
            }
            if (more) {
                for (int e = e_lo + kRegParents; e < e_hi; ++e) {
                    const int p = edge_at(e);
                    if (p < -1 || p >= i || !accepted(p)) continue;
                    const int32_t lp = (p == -1) ? 0 : L[p];
                    if (lp >= 0 && lp + 1 > best) best = lp + 1;
                }
            }
            if (best != mine) {
                mine = best;
                L[i] = best;
                changed = 1;
            }
        }
        if (!__syncthreads_or(changed)) break;
    }

    // back pointer of every accepted node: the smallest-id accepted parent that ends a path one node shorter
    // (the root, id -1, is the smallest)
    if (active && mine > 0) {
        int32_t chosen = 0x7fffffff;
#pragma unroll
        for (int x = 0; x < kRegParents; ++x) {
            const int32_t l = L[par[x] >= 0 ? par[x] : i];
            const int32_t lp = par[x] >= 0 ? l : (par[x] == -1 ? 0 : -1);
            if (lp == mine - 1 && par[x] < chosen) chosen = par[x];
        }
        if (more) {
            for (int e = e_lo + kRegParents; e < e_hi; ++e) {
                const int p = edge_at(e);
                if (p < -1 || p >= i || !accepted(p)) continue;
                const int32_t lp = (p == -1) ? 0 : L[p];
                if (lp == mine - 1 && p < chosen) chosen = p;
            }
        }
        back_s[i] = chosen;
    }

    // best end node: largest L, then smallest id.  key = L * 1024 + (1023 - i), 0 = nothing accepted.
    uint32_t key = 0;
    if (active && mine > 0) key = uint32_t(mine) * 1024u + uint32_t(1023 - i);
    for (int off = 32; off > 0; off >>= 1) {
        const uint32_t other = __shfl_xor(key, off, 64);
        key = other > key ? other : key;
    }
    if ((threadIdx.x & 63) == 0) wave_best[threadIdx.x >> 6] = key;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t k = 0;
        for (int w = 0; w < kAcceptThreads / 64; ++w) k = wave_best[w] > k ? wave_best[w] : k;
        const int32_t len = int32_t(k / 1024u);
        int32_t v = (len > 0) ? int32_t(1023u - (k % 1024u)) : -1;
        len_s = len;
        accept_len[b] = len;
        bonus_token[b] = (len > 0) ? pred_s[v] : rp;
        for (int pos = len - 1; pos >= 0 && v >= 0 && v < n; --pos) {   // L drops by one per step: the root's child sits at pos 0
            path_s[pos] = v;
            v = back_s[v];
        }
    }
    __syncthreads();
    const int32_t len = len_s;
    int32_t *out = accept_path + int64_t(b) * max_nodes;
    for (int x = threadIdx.x; x < max_nodes; x += kAcceptThreads) out[x] = (x < len) ? path_s[x] : -1;
}

hipError_t launch_accept(int32_t batch, int32_t max_nodes, const int32_t *node_offsets,
                         const int32_t *parent_offsets, const int32_t *parent_idx, const int32_t *tokens,
                         const int32_t *pred, const int32_t *root_pred, int32_t *accept_len, int32_t *accept_path,
                         int32_t *bonus_token, hipStream_t stream) {
    hipLaunchKernelGGL(accept_kernel, dim3(batch), dim3(kAcceptThreads), 0, stream, max_nodes, node_offsets,
                       parent_offsets, parent_idx, tokens, pred, root_pred, accept_len, accept_path, bonus_token);
    return hipGetLastError();
}

}  // namespace gsd
