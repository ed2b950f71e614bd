// Draft-side construction of the token graph from a drafted token tree (paper Sections 4.2, 5.2, 5.3): probability
// pruning, sibling pruning, tau-gram redundancy, merging.  One work-group per sequence, one thread per tree node.
//
// Whether a node exists depends on its parent having been expanded, which depends on the parent not being redundant,
// which depends on which EARLIER nodes exist: the construction is sequential across layers, so the work-group walks
// the tree layer by layer (nodes come breadth first: a layer is a run of consecutive ids).  Within a layer everything
// is parallel: existence comes from the layer above, and the first occurrence of a node's tau-gram is a lookup.
// Before the walk every node gets the exact equivalence class of its tau-gram among ALL tree nodes (no hashing):
// class_t(i) = the smallest j <= i with tok[j] == tok[i] and class_(t-1)(parent j) == class_(t-1)(parent i), built
// level by level with one all-pairs comparison per level (the candidates of a wave sit one per lane and are
// broadcast with readlane, so the comparison touches no memory).  During the walk the smallest existing node of
// every class is kept in a table (atomic min by the layer's existing nodes), so "the earliest existing earlier node
// with the same tau-gram" is one read.
//
// Merging (Section 5.3: an edge from the redundant node R to the first occurrence F of its tau-gram, so that what
// follows F is reused below R) makes R one more parent of every child of F, unless R already descends from F in the
// graph built so far: that would close a cycle, and R then stays a bare leaf.  Which nodes exist does not depend on
// these decisions, but the decisions depend on each other in generation order (an edge drawn for one node changes
// who descends from whom for the next), so after the walk the redundant nodes are taken one at a time, in id order,
// against per-node ancestor bit rows in LDS: one bit test, then every descendant of F takes over R's ancestors, one
// barrier per redundant node.  An edge from a later layer into an earlier one breaks the generation order as a
// topological order: the fill kernel renumbers the graph by level (longest distance from the root, by relaxation),
// nodes of one level in generation order.
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
    int32_t flags[GSD_MAX_NODES_PER_SEQ];      // bit0 prob, bit1 sibling, bit2 redundant, bit3 no merge edge, bit8 exists, bit9 merged
    int32_t merged_to[GSD_MAX_NODES_PER_SEQ];  // first occurrence of a redundant node's tau-gram, or -1
    uint32_t sib_max[GSD_MAX_NODES_PER_SEQ + 1];   // float bits of the largest child probability, slot p+1
    int32_t scan[GSD_MAX_NODES_PER_SEQ];
    int32_t cls[GSD_MAX_NODES_PER_SEQ];        // class of the node's tau-gram (an earlier-or-equal node id), -1 if none
    int32_t first_ex[GSD_MAX_NODES_PER_SEQ];   // per class: smallest existing node seen so far
    int32_t merge_cnt[GSD_MAX_NODES_PER_SEQ];  // nodes merged into this one (merge edges actually drawn)
    uint64_t anc[GSD_MAX_NODES_PER_SEQ * 8];   // ancestor bit row of every node in the graph built so far (itself included)
    int32_t bad;
    int32_t max_depth;
};
constexpr int kFlagExists = 0x100;             // internal flag bits, above the four that are returned
constexpr int kFlagMerged = 0x200;             // redundant node whose merge edges are drawn

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
    s.first_ex[i] = 0x7fffffff;
    s.merge_cnt[i] = 0;
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

    // tau-gram classes, level by level.  At level t a node with depth >= t has the key (its token, the level t-1
    // class of its parent); its class is the smallest node id with the same key.  Wave w holds nodes 64w .. 64w+63
    // and only ever needs candidates below that, 64 at a time, one per lane.
    const int lane = i & 63;
    int my_cls = -1;                                   // class at the level just finished (level 0: everyone alike)
    const int32_t my_tok = i < n ? s.tok[i] : 0;
    const int my_par = i < n ? s.par[i] : -2;
    const int levels = tau <= max_depth ? tau : 0;     // no chain reaches tau nodes: nothing is ever redundant
    for (int t = 1; t <= levels; ++t) {
        const int my_prev = t == 1 ? 0 : (my_par >= 0 ? s.cls[my_par] : -1);     // class of the parent one level down
        const bool my_valid = my_depth >= t;
        s.scan[i] = my_prev;                           // staged so that the candidates can be fetched one per lane
        __syncthreads();                               // (also: everyone has read the previous level's classes)
        int found = my_valid ? i : -1;
        for (int c0 = 0; c0 <= (i | 63) && c0 < n; c0 += 64) {      // uniform per wave
            const int j = c0 + lane;
            const int32_t cand_tok = j < n ? s.tok[j] : 0;
            const int32_t cand_prev = j < n ? s.scan[j] : -1;
            const int cand_valid = (j < n && s.depth[j] >= t) ? 1 : 0;
            for (int l = 0; l < 64; ++l) {
                const int32_t tj = __builtin_amdgcn_readlane(cand_tok, l);
                const int32_t pj = __builtin_amdgcn_readlane(cand_prev, l);
                const int vj = __builtin_amdgcn_readlane(cand_valid, l);
                const int jj = c0 + l;
                if (my_valid && vj && jj < found && tj == my_tok && pj == my_prev) found = jj;
            }
        }
        my_cls = found;
        s.cls[i] = my_cls;
        __syncthreads();                               // classes of this level published, staging area free again
    }

    for (int layer = 1; layer <= max_depth; ++layer) {
        // existence and the two pruning rules: everything they need is in the layer above
        bool ex = false;
        if (my_depth == layer) {
            const int p = s.par[i];
            ex = p == -1 || (p >= 0 && (s.flags[p] & kFlagExists) && (s.flags[p] & 0xf) == 0);
            int f = 0;
            if (ex) {
                f = kFlagExists;
                if (s.q[i] < theta_prob) f |= 1;
                if (s.q[i] < theta_sib * __uint_as_float(s.sib_max[p + 1])) f |= 2;
            }
            s.flags[i] = f;
            // redundancy: the earliest existing earlier node with the same tau-gram.  The existing nodes of this layer
            // enter the table first (their redundancy does not change whether THEY exist, only whether they are
            // expanded), then every one of them looks its class up.
            if (ex && layer >= tau) atomicMin(&s.first_ex[my_cls], i);
        }
        __syncthreads();
        if (my_depth == layer && ex && layer >= tau) {
            const int first = s.first_ex[my_cls];
            if (first < i) {
                s.merged_to[i] = first;
                s.flags[i] |= 4;
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

// After construct(): takes the redundant nodes in id order and decides for each whether its merge edges are drawn
// (kFlagMerged, merge_cnt of the first occurrence) or it descends from its first occurrence (bit 3).  Leaves the
// ancestor rows of the finished graph in s.anc.  Uses s.cls (free after construct) for the list of redundant nodes.
__device__ void decide_merges(GraphLds &s, int n) {
    const int i = threadIdx.x;
    const bool ex = i < n && (s.flags[i] & kFlagExists);
    uint64_t *row = s.anc + i * 8;
#pragma unroll
    for (int w = 0; w < 8; ++w) row[w] = 0;
    __syncthreads();
    const int max_depth = s.max_depth;
    for (int layer = 1; layer <= max_depth; ++layer) {      // tree ancestors: the parent's row plus the node itself
        if (ex && s.depth[i] == layer) {
            const int p = s.par[i];
            if (p >= 0) {
#pragma unroll
                for (int w = 0; w < 8; ++w) row[w] = s.anc[p * 8 + w];
            }
            row[i >> 6] |= uint64_t(1) << (i & 63);
        }
        __syncthreads();
    }
    const bool red = ex && (s.flags[i] & 4);
    const int pos = block_scan(s.scan, red ? 1 : 0) - 1;
    const int n_red = s.scan[kGraphThreads - 1];
    __syncthreads();
    if (red) s.cls[pos] = i;
    __syncthreads();
    for (int k = 0; k < n_red; ++k) {                       // uniform trip count and operands
        const int r = s.cls[k], f = s.merged_to[r];
        const bool cyclic = (s.anc[r * 8 + (f >> 6)] >> (f & 63)) & 1;
        if (!cyclic) {
            // r is no descendant of f, so nobody writes r's row in this step; every other row is written by its owner
            if (ex && i != f && ((row[f >> 6] >> (f & 63)) & 1)) {
#pragma unroll
                for (int w = 0; w < 8; ++w) row[w] |= s.anc[r * 8 + w];
            }
            if (i == r) {
                s.flags[i] |= kFlagMerged;
                s.merge_cnt[f] += 1;
            }
        } else if (i == r) {
            s.flags[i] |= 8;
        }
        __syncthreads();
    }
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
    decide_merges(s, n);
    const int i = threadIdx.x;
    const bool ex = i < n && (s.flags[i] & kFlagExists);
    const int nodes = block_scan(s.scan, ex ? 1 : 0);
    const int total_nodes = s.scan[kGraphThreads - 1];
    __syncthreads();
    const int edges = block_scan(s.scan, ex ? 1 + (s.par[i] >= 0 ? s.merge_cnt[s.par[i]] : 0) : 0);
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
    decide_merges(s, n);
    const bool ex = i < n && (s.flags[i] & kFlagExists);
    const bool merger = ex && (s.flags[i] & kFlagMerged);
    const int my_par = i < n ? s.par[i] : -2;
    const int my_first = merger ? s.merged_to[i] : -1;
    // Storage that construct() and decide_merges() are done with is used again from here on:
    int32_t *level = s.tok;                 // longest distance from the root, in edges below the root's children
    int32_t *group_level = s.first_ex;      // per node f: the largest level among f and the nodes merged into it
    int32_t *new_id = reinterpret_cast<int32_t *>(s.q);
    int32_t *list_off = reinterpret_cast<int32_t *>(s.sib_max);     // per f: where its mergers' new ids start in `list`
    int32_t *list = s.cls;                  // new ids of the mergers of every f, ascending within an f
    __syncthreads();
    level[i] = ex ? s.depth[i] - 1 : -1;
    group_level[i] = -1;
    __syncthreads();
    // levels by relaxation: they start at the tree depth, a lower bound, and only grow; a sweep that moves nothing
    // ends it (at most one sweep per node of the longest path, and never more than n + 1)
    for (int sweep = 0; sweep <= n; ++sweep) {
        if (ex) atomicMax(&group_level[i], level[i]);
        if (merger) atomicMax(&group_level[my_first], level[i]);
        __syncthreads();
        int changed = 0;
        if (ex && my_par >= 0) {
            const int l = 1 + group_level[my_par];
            if (l > level[i]) {
                level[i] = l;
                changed = 1;
            }
        }
        if (!__syncthreads_or(changed)) break;
    }
    // new id = rank by (level, id) among the existing nodes
    int my_new = -1;
    if (ex) {
        my_new = 0;
        const int li = level[i];
        for (int j = 0; j < n; ++j) {
            const int lj = level[j];
            my_new += (lj >= 0 && (lj < li || (lj == li && j < i))) ? 1 : 0;
        }
    }
    new_id[i] = my_new;
    (void)block_scan(s.scan, ex ? 1 : 0);
    const int total_nodes = s.scan[kGraphThreads - 1];
    __syncthreads();
    // the mergers of every first occurrence, sorted by new id
    const int cnt_i = i < n ? s.merge_cnt[i] : 0;
    const int off_end = block_scan(s.scan, cnt_i);
    __syncthreads();
    list_off[i] = off_end - cnt_i;
    __syncthreads();
    if (merger) {
        int before = 0;
        for (int j = 0; j < n; ++j)
            before += ((s.flags[j] & kFlagMerged) && s.merged_to[j] == my_first && new_id[j] < my_new) ? 1 : 0;
        list[list_off[my_first] + before] = my_new;
    }
    __syncthreads();
    // edges, in the order of the new ids
    const int my_edges = ex ? 1 + (my_par >= 0 ? s.merge_cnt[my_par] : 0) : 0;
    int32_t *by_rank = s.depth;             // depth is not read any more
    by_rank[i] = 0;
    __syncthreads();
    if (ex) by_rank[my_new] = my_edges;
    __syncthreads();
    (void)block_scan(s.scan, by_rank[i]);
    const int total_edges = s.scan[kGraphThreads - 1];
    if (ex) {
        const int g = node_base + my_new;
        origin[g] = i;
        flags_out[g] = s.flags[i] & 0xf;
        int64_t e = int64_t(edge_base) + s.scan[my_new] - my_edges;
        parent_offsets[g] = int32_t(e);
        bool over = false;
        auto put = [&](int32_t v) {
            if (e < edge_capacity) parent_idx[e] = v; else over = true;
            ++e;
        };
        if (my_par < 0) {
            put(-1);
        } else {                                // the tree parent's new id merged into the sorted ids of its mergers
            const int pid = new_id[my_par];
            const int k = s.merge_cnt[my_par];
            const int32_t *m = list + list_off[my_par];
            int x = 0;
            for (; x < k && m[x] < pid; ++x) put(m[x]);
            put(pid);
            for (; x < k; ++x) put(m[x]);
        }
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
