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
    const int32_t *edges = cached ? edge_cache : (parent_idx + e0);

    for (int sweep = 0; sweep <= n; ++sweep) {
        int changed = 0;
        for (int i = threadIdx.x; i < n; i += kAcceptThreads) {
            const int32_t tok = tok_s[i];
            int32_t best = L[i];
            for (int e = off_cache[i]; e < off_cache[i + 1]; ++e) {
                const int p = edges[e];
                if (p < -1 || p >= i) continue;
                const int32_t lp = (p == -1) ? 0 : L[p];
                const int32_t choice = (p == -1) ? rp : pred_s[p];
                if (lp >= 0 && tok == choice && lp + 1 > best) best = lp + 1;
            }
            if (best != L[i]) {
                L[i] = best;
                changed = 1;
            }
        }
        if (!__syncthreads_or(changed)) break;
    }

    // best end node: largest L, then smallest id.  key = L * 1024 + (1023 - i), 0 = nothing accepted.
    uint32_t key = 0;
    for (int i = threadIdx.x; i < n; i += kAcceptThreads) {
        const int32_t l = L[i];
        if (l > 0) {
            const uint32_t k = uint32_t(l) * 1024u + uint32_t(1023 - i);
            key = k > key ? k : key;
        }
    }
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
        for (int pos = len - 1; pos >= 0; --pos) {
            path_s[pos] = v;
            int32_t chosen = 0x7fffffff;
            for (int e = off_cache[v]; e < off_cache[v + 1]; ++e) {
                const int p = edges[e];
                if (p < -1 || p >= v) continue;
                const int32_t lp = (p == -1) ? 0 : L[p];
                const int32_t choice = (p == -1) ? rp : pred_s[p];
                if (lp == pos && tok_s[v] == choice && p < chosen) chosen = p;
            }
            if (chosen == 0x7fffffff || chosen < 0) break;   // reached the root (pos == 0)
            v = chosen;
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
