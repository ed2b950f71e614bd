// Draft-side construction of the token graph from a drafted token tree (paper Sections 4.2, 5.2, 5.3): probability
// pruning, sibling pruning, tau-gram redundancy, merging.  One work-group per sequence, one thread per tree node.
//
// Whether a node exists depends on its parent having been expanded, which depends on the parent not being redundant,
// which depends on which EARLIER nodes exist: the construction is sequential across layers, so the work-group walks
// the tree layer by layer (nodes come breadth first: a layer is a run of consecutive ids).  Within a layer everything
// is parallel: existence comes from the layer above; the first occurrence of a node's tau-gram is found by scanning
// all earlier existing nodes and comparing the tau tokens along the two ancestor chains exactly (no hashing: at most
// 512 nodes, so the quadratic scan is a few thousand LDS reads per thread).  A redundant node whose first occurrence
// lies in its own layer is merged into it: the children of that node get one more parent.
// Two launches: the first only counts nodes and edges per sequence, the second repeats the construction and writes
// the packed graph behind the sequences before it (the library keeps no scratch memory).
#include "gsd_internal.h"

namespace gsd {

constexpr int kGraphThreads = 512;

struct GraphLds {
    int32_t par[GSD_MAX_NODES_PER_SEQ];
    int32_t tok[GSD_MAX_NODES_PER_SEQ];
    float q[GSD_MAX_NODES_PER_SEQ];
    int32_t depth[GSD_MAX_NODES_PER_SEQ];
    int32_t flags[GSD_MAX_NODES_PER_SEQ];      // bit0 prob, bit1 sibling, bit2 redundant, bit3 no merge edge, bit8 exists
    int32_t merged_to[GSD_MAX_NODES_PER_SEQ];  // first occurrence this node is merged into, or -1
    uint32_t sib_max[GSD_MAX_NODES_PER_SEQ + 1];   // float bits of the largest child probability, slot p+1
    int32_t scan[GSD_MAX_NODES_PER_SEQ];
    int32_t bad;
    int32_t max_depth;
};

// Runs the construction for the calling work-group's sequence; afterwards flags (bit8 = exists), merged_to and depth
// are final.  Returns the node count through n_out.
__device__ void construct(GraphLds &s, int n, int64_t base, const int32_t *__restrict__ tree_parent,
                          const int32_t *__restrict__ tokens, const float *__restrict__ draft_prob, int tau,
                          float theta_prob, float theta_sib) {
    const int i = threadIdx.x;
    if (i == 0) {
        s.bad = 0;
        s.max_depth = 0;
    }
    s.sib_max[i] = 0;
    if (i == 0) s.sib_max[GSD_MAX_NODES_PER_SEQ] = 0;
    if (i < n) {
        s.par[i] = tree_parent[base + i];
        s.tok[i] = tokens[base + i];
        s.q[i] = draft_prob[base + i];
        s.depth[i] = 0;
        s.flags[i] = 0;
        s.merged_to[i] = -1;
    }
    __syncthreads();
    if (i < n) {
        int p = s.par[i];
        if (p < -1 || p >= i) {               // malformed: treated as hanging off a node that does not exist
            s.bad = 1;
            p = -2;
            s.par[i] = -2;
        }
        if (p >= -1) atomicMax(&s.sib_max[p + 1], __float_as_uint(fmaxf(s.q[i], 0.f)));
    }
    __syncthreads();
    // depths by relaxation (a chain can be as long as the sequence)
    for (int sweep = 0; sweep <= n; ++sweep) {
        int changed = 0;
        if (i < n && s.depth[i] == 0) {
            const int p = s.par[i];
            const int d = p == -1 ? 1 : (p >= 0 && s.depth[p] > 0 ? s.depth[p] + 1 : 0);
            if (d > 0) {
                s.depth[i] = d;
                changed = 1;
            }
        }
        if (!__syncthreads_or(changed)) break;
    }
    if (i < n) {
        if (i > 0 && s.depth[i] < s.depth[i - 1]) s.bad = 1;       // not breadth first
        atomicMax(&s.max_depth, s.depth[i]);
    }
    __syncthreads();
    const int max_depth = s.max_depth;
    const int my_depth = i < n ? s.depth[i] : 0;
    for (int layer = 1; layer <= max_depth; ++layer) {
        // existence and the two pruning rules: everything they need is in the layer above
        if (my_depth == layer) {
            const int p = s.par[i];
            const bool ex = p == -1 || (p >= 0 && (s.flags[p] & 0x100) && (s.flags[p] & 0xf) == 0);
            int f = 0;
            if (ex) {
                f = 0x100;
                if (s.q[i] < theta_prob) f |= 1;
                if (s.q[i] < theta_sib * __uint_as_float(s.sib_max[p + 1])) f |= 2;
            }
            s.flags[i] = f;
        }
        __syncthreads();
        // redundancy: the earliest existing earlier node with the same tau-gram (existence of this layer is known now;
        // the redundancy of nodes of this layer does not change whether THEY exist, only whether they are expanded)
        if (my_depth == layer && (s.flags[i] & 0x100) && layer >= tau) {
            int first = -1;
            for (int j = 0; j < i && first < 0; ++j) {
                if (!(s.flags[j] & 0x100) || s.depth[j] < tau) continue;
                int a = i, c = j;
                bool same = true;
                for (int t = 0; t < tau; ++t) {
                    if (s.tok[a] != s.tok[c]) {
                        same = false;
                        break;
                    }
                    a = s.par[a];
                    c = s.par[c];
                }
                if (same) first = j;
            }
            if (first >= 0) {
                if (s.depth[first] == layer) {
                    s.merged_to[i] = first;
                    s.flags[i] |= 4;
                } else {
                    s.flags[i] |= 4 | 8;
                }
            }
        }
        __syncthreads();
    }
}

// inclusive scan of `value` over the work-group's threads in LDS; returns this thread's inclusive prefix
__device__ int block_scan(int32_t *buf, int value) {
    const int i = threadIdx.x;
    buf[i] = value;
    __syncthreads();
    for (int d = 1; d < kGraphThreads; d <<= 1) {
        const int add = i >= d ? buf[i - d] : 0;
        __syncthreads();
        buf[i] += add;
        __syncthreads();
    }
    return buf[i];
}

// number of parents of existing node i in the graph: its tree parent plus the nodes merged into that parent
__device__ int extra_parents(const GraphLds &s, int n, int i) {
    const int f = s.par[i];
    if (f < 0) return 0;
    int cnt = 0;
    for (int r = f + 1; r < n && s.depth[r] == s.depth[f]; ++r) cnt += (s.merged_to[r] == f);
    return cnt;
}

__global__ __launch_bounds__(kGraphThreads) void graph_count_kernel(
    int32_t max_nodes, const int32_t *__restrict__ node_offsets, const int32_t *__restrict__ tree_parent,
    const int32_t *__restrict__ tokens, const float *__restrict__ draft_prob, int tau, float theta_prob, float theta_sib,
    int32_t *__restrict__ counts /* [B][2]: nodes, edges */, int32_t *__restrict__ error_flag) {
    __shared__ GraphLds s;
    const int b = blockIdx.x;
    const int64_t base = node_offsets[b];
    int n = node_offsets[b + 1] - node_offsets[b];
    bool bad = false;
    if (n > max_nodes) {
        n = max_nodes;
        bad = true;
    }
    if (n < 0) n = 0;
    construct(s, n, base, tree_parent, tokens, draft_prob, tau, theta_prob, theta_sib);
    const int i = threadIdx.x;
    const bool ex = i < n && (s.flags[i] & 0x100);
    const int nodes = block_scan(s.scan, ex ? 1 : 0);
    const int total_nodes = s.scan[kGraphThreads - 1];
    __syncthreads();
    const int edges = block_scan(s.scan, ex ? 1 + extra_parents(s, n, i) : 0);
    const int total_edges = s.scan[kGraphThreads - 1];
    (void)nodes;
    (void)edges;
    if (i == 0) {
        counts[2 * b] = total_nodes;
        counts[2 * b + 1] = total_edges;
        if ((bad || s.bad) && error_flag) atomicOr(error_flag, 1);
    }
}

__global__ __launch_bounds__(kGraphThreads) void graph_fill_kernel(
    int32_t batch, int32_t max_nodes, const int32_t *__restrict__ node_offsets, const int32_t *__restrict__ tree_parent,
    const int32_t *__restrict__ tokens, const float *__restrict__ draft_prob, int tau, float theta_prob, float theta_sib,
    const int32_t *__restrict__ counts, int32_t *__restrict__ graph_node_offsets, int32_t *__restrict__ parent_offsets,
    int32_t *__restrict__ parent_idx, int64_t edge_capacity, int32_t *__restrict__ origin,
    int32_t *__restrict__ flags_out, int32_t *__restrict__ error_flag) {
    __shared__ GraphLds s;
    __shared__ int32_t red[2][kGraphThreads / 64];
    const int b = blockIdx.x;
    const int i = threadIdx.x;
    // packed position of this sequence: sums over the sequences before it
    int nb = 0, eb = 0;
    for (int x = i; x < b; x += kGraphThreads) {
        nb += counts[2 * x];
        eb += counts[2 * x + 1];
    }
    for (int d = 32; d > 0; d >>= 1) {
        nb += __shfl_xor(nb, d);
        eb += __shfl_xor(eb, d);
    }
    if ((i & 63) == 0) {
        red[0][i >> 6] = nb;
        red[1][i >> 6] = eb;
    }
    __syncthreads();
    int node_base = 0, edge_base = 0;
    for (int w = 0; w < kGraphThreads / 64; ++w) {
        node_base += red[0][w];
        edge_base += red[1][w];
    }

    const int64_t base = node_offsets[b];
    int n = node_offsets[b + 1] - node_offsets[b];
    if (n > max_nodes) n = max_nodes;
    if (n < 0) n = 0;
    construct(s, n, base, tree_parent, tokens, draft_prob, tau, theta_prob, theta_sib);
    const bool ex = i < n && (s.flags[i] & 0x100);
    const int my_new = block_scan(s.scan, ex ? 1 : 0) - 1;           // new id of an existing node
    const int total_nodes = s.scan[kGraphThreads - 1];
    __syncthreads();
    // new ids of all nodes are needed below: keep them where depth is no longer read... depth IS read by
    // extra_parents, so the ids go into q's storage (reinterpreted) once q is done with
    int32_t *new_id = reinterpret_cast<int32_t *>(s.q);
    __syncthreads();
    if (i < n) new_id[i] = ex ? my_new : -1;
    __syncthreads();
    const int my_edges = ex ? 1 + extra_parents(s, n, i) : 0;
    const int edge_end = block_scan(s.scan, my_edges);
    const int total_edges = s.scan[kGraphThreads - 1];
    if (ex) {
        const int g = node_base + my_new;
        origin[g] = i;
        flags_out[g] = s.flags[i] & 0xf;
        parent_offsets[g] = edge_base + edge_end - my_edges;
        int64_t e = int64_t(edge_base) + edge_end - my_edges;
        const int f = s.par[i];
        bool over = false;
        auto put = [&](int32_t v) {
            if (e < edge_capacity) parent_idx[e] = v; else over = true;
            ++e;
        };
        put(f < 0 ? -1 : new_id[f]);
        if (f >= 0)
            for (int r = f + 1; r < n && s.depth[r] == s.depth[f]; ++r)
                if (s.merged_to[r] == f) put(new_id[r]);
        if (over && error_flag) atomicOr(error_flag, 2);
    }
    if (i == 0) {
        graph_node_offsets[b] = node_base;
        if (b == batch - 1) {
            graph_node_offsets[batch] = node_base + total_nodes;
            parent_offsets[node_base + total_nodes] = edge_base + total_edges;
        }
    }
}

hipError_t launch_build_graph(int32_t batch, int32_t max_nodes, const int32_t *node_offsets, const int32_t *tree_parent,
                              const int32_t *tokens, const float *draft_prob, int32_t tau, float theta_prob,
                              float theta_sib, int32_t *counts, int32_t *graph_node_offsets, int32_t *parent_offsets,
                              int32_t *parent_idx, int64_t edge_capacity, int32_t *origin, int32_t *flags,
                              int32_t *error_flag, hipStream_t stream) {
    hipLaunchKernelGGL(graph_count_kernel, dim3(batch), dim3(kGraphThreads), 0, stream, max_nodes, node_offsets,
                       tree_parent, tokens, draft_prob, tau, theta_prob, theta_sib, counts, error_flag);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    hipLaunchKernelGGL(graph_fill_kernel, dim3(batch), dim3(kGraphThreads), 0, stream, batch, max_nodes, node_offsets,
                       tree_parent, tokens, draft_prob, tau, theta_prob, theta_sib, counts, graph_node_offsets,
                       parent_offsets, parent_idx, edge_capacity, origin, flags, error_flag);
    return hipGetLastError();
}

}  // namespace gsd
