// Draft-side construction of the token graph from a drafted token tree (paper Sections 4.2, 5.2, 5.3): probability
// pruning, sibling pruning, tau-gram redundancy, merging.  One work-group per sequence, one thread per tree node.
//
// Whether a node exists depends on its parent having been expanded, which depends on the parent not being redundant,
// which depends on which EARLIER nodes exist: the construction is sequential across layers, so the work-group walks
// the tree layer by layer (nodes come breadth first: a layer is a run of consecutive ids).  Within a layer everything
// is parallel: existence comes from the layer above, and the first occurrence of a node's tau-gram is a lookup.
// Before the walk every node gets the exact equivalence class of its tau-gram among ALL tree nodes:
// class_t(i) = the smallest j with tok[j] == tok[i] and class_(t-1)(parent j) == class_(t-1)(parent i), built level
// by level through an open-addressed table in LDS whose slots hold the full 64-bit key (token, class of the parent
// one level down), so two nodes share a slot only if their keys are equal: hashing picks where to look, never what
// is equal, and the smallest id of a slot does not depend on the order of arrival.  During the walk the smallest
// existing node of every class is kept in a table (atomic min by the layer's existing nodes), so "the earliest
// existing earlier node with the same tau-gram" is one read.
//
// Merging (Section 5.3: an edge from the redundant node R to the first occurrence F of its tau-gram, so that what
// follows F is reused below R) makes R one more parent of every child of F, unless R already descends from F in the
// graph built so far: that would close a cycle, and R then stays a bare leaf.  Which nodes exist does not depend on
// these decisions, but the decisions depend on each other in generation order (an edge drawn for one node changes
// who descends from whom for the next), so after the walk the redundant nodes are taken one at a time, in id order.
// The decisions only ever ask whether one node's first occurrence is an ancestor of another redundant node, so one
// wave keeps exactly those bits in registers (a row per redundant node, a column per pair) and runs the whole
// sequence with lane broadcasts, no LDS traffic and no barrier in between.
// An edge from a later layer into an earlier one breaks the generation order as a topological order: the fill kernel
// renumbers the graph by level (longest distance from the root, by relaxation), nodes of one level in generation
// order (a counting sort: ballots within a wave, one scan over the per-wave counts).
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
    // 32 KB used three times over: the key table of the tau-gram classes, then (merge decisions) per node the set of
    // redundant nodes it is the first occurrence for, word-major, then the counting tables of the renumbering
    uint64_t pool[GSD_MAX_NODES_PER_SEQ * 8];
    int32_t wave_tot[16];
    int32_t bad;
    int32_t max_depth;
};
constexpr int kFlagExists = 0x100;             // internal flag bits, above the four that are returned
constexpr int kFlagMerged = 0x200;             // redundant node whose merge edges are drawn

// Runs the construction for the calling work-group's sequence; afterwards flags (bit8 = exists), merged_to and depth
// are final.
__device__ __forceinline__ void construct(GraphLds &s, int n, int64_t base, const int32_t *__restrict__ tree_parent,
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
    // depth = nodes on the way up to the root; a parent is an earlier node, so the walk ends within i + 1 steps, and
    // a node that hangs off a malformed one never reaches the root and keeps depth 0
    if (i < n) {
        int d = 0, a = i;
        while (a >= 0) {
            ++d;
            a = s.par[a];
        }
        s.depth[i] = a == -1 ? d : 0;
    }
    __syncthreads();
    if (i < n) {
        if (i > 0 && s.depth[i] < s.depth[i - 1]) s.bad = 1;       // not breadth first
        atomicMax(&s.max_depth, s.depth[i]);
    }
    __syncthreads();
    const int max_depth = s.max_depth;
    const int my_depth = i < n ? s.depth[i] : 0;

    // tau-gram classes, level by level.  At level t a node with depth >= t has the key (its token, the level t-1
    // class of its parent); its class is the smallest node id with the same key.  The nodes with a key claim a slot
    // of the table by compare-and-swap on the key itself (linear probing; at most 512 keys in 2048 slots, so a free
    // slot always turns up) and leave the minimum of their ids there.
    constexpr int kSlots = 2048;
    constexpr unsigned long long kEmpty = ~0ull;       // no key looks like this: the low half is a class + 1 <= 512
    unsigned long long *slot_key = reinterpret_cast<unsigned long long *>(s.pool);
    int32_t *slot_min = reinterpret_cast<int32_t *>(s.pool + kSlots);
    int my_cls = -1;                                   // class at the level just finished (level 0: everyone alike)
    const int32_t my_tok = i < n ? s.tok[i] : 0;
    const int my_par = i < n ? s.par[i] : -2;
    const int levels = tau <= max_depth ? tau : 0;     // no chain reaches tau nodes: nothing is ever redundant
    for (int t = 1; t <= levels; ++t) {
        const int my_prev = t == 1 ? 0 : (my_par >= 0 ? s.cls[my_par] : -1);     // class of the parent one level down
        const bool my_valid = my_depth >= t;
        for (int x = i; x < kSlots; x += kGraphThreads) {
            slot_key[x] = kEmpty;
            slot_min[x] = 0x7fffffff;
        }
        __syncthreads();                               // (also: everyone has read the previous level's classes)
        int slot = -1;
        if (my_valid) {
            const unsigned long long key = (static_cast<unsigned long long>(static_cast<uint32_t>(my_tok)) << 32) |
                                           static_cast<uint32_t>(my_prev + 1);
            uint32_t h = (static_cast<uint32_t>(my_tok) * 0x9E3779B1u) ^ (static_cast<uint32_t>(my_prev + 1) * 0x85EBCA6Bu);
            h = (h ^ (h >> 15)) & (kSlots - 1);
            for (int probe = 0; probe < kSlots; ++probe) {
                const unsigned long long seen = atomicCAS(&slot_key[h], kEmpty, key);
                if (seen == kEmpty || seen == key) {
                    slot = int(h);
                    break;
                }
                h = (h + 1) & (kSlots - 1);
            }
            if (slot >= 0) atomicMin(&slot_min[slot], i);
        }
        __syncthreads();
        my_cls = slot >= 0 ? slot_min[slot] : -1;
        s.cls[i] = my_cls;
        __syncthreads();                               // classes of this level published, table free again
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

// Inclusive scan of `value` over the work-group's threads: within a wave by shuffles, across waves through the
// eight wave totals.  Leaves every thread's inclusive prefix in buf[] (published by the closing barrier) and returns
// the caller's own.
__device__ __forceinline__ int block_scan(GraphLds &s, int32_t *buf, int value) {
    const int i = threadIdx.x, lane = i & 63, wave = i >> 6;
    int v = value;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int up = __shfl_up(v, d, 64);
        if (lane >= d) v += up;
    }
    if (lane == 63) s.wave_tot[wave] = v;
    __syncthreads();
#pragma unroll
    for (int w = 0; w < kGraphThreads / 64; ++w)
        if (w < wave) v += s.wave_tot[w];
    buf[i] = v;
    __syncthreads();
    return v;
}

// The decisions of decide_merges() for n_red <= 64 * NC redundant nodes, taken by one wave without touching LDS in
// between.  Pair k is the k-th redundant node R_k (in id order) with the first occurrence F_k of its tau-gram.
// All that the decisions ever look at is whether some F_k is an ancestor of some R_j, so the ancestor sets are kept
// as one bit per pair: lane j of chunk c holds the row of pair 64 c + j, bit k of it says "F_k is an ancestor of
// R_j".  Pair k in turn: its own bit k decides (set: R_k descends from F_k, no edges); otherwise every row with bit
// k set, that is every R below F_k, takes over the row of R_k, handed out with readlane.  Rows of earlier pairs and
// bits of earlier pairs are never looked at again, so the sweep leaves them alone.
// Before: col[w * GSD_MAX_NODES_PER_SEQ + a] = the pairs (bits of word w) whose F is node a.
template <int NC>
__device__ __forceinline__ void decide_in_one_wave(GraphLds &s, int n_red) {
    constexpr int W = 2 * NC;
    const int lane = threadIdx.x & 63;
    const uint32_t *col = reinterpret_cast<const uint32_t *>(s.pool);
    int r_of[NC], f_of[NC];
    uint32_t row[NC][W];
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        const int k = 64 * c + lane;
        r_of[c] = k < n_red ? s.cls[k] : -1;
        f_of[c] = k < n_red ? s.merged_to[r_of[c]] : 0;
#pragma unroll
        for (int w = 0; w < W; ++w) row[c][w] = 0;
        // tree ancestors of R (R itself is nobody's first occurrence: a first occurrence is never redundant)
        int a = k < n_red ? s.par[r_of[c]] : -1;
        while (a >= 0) {
#pragma unroll
            for (int w = 0; w < W; ++w) row[c][w] |= col[w * GSD_MAX_NODES_PER_SEQ + a];
            a = s.par[a];
        }
    }
    uint64_t drawn[NC];                                     // per chunk: the pairs whose edges are drawn (uniform)
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        drawn[c] = 0;
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int wk = 2 * c + half;                    // the word that holds the bits of these 32 pairs
            const int end = n_red - 64 * c < 32 * half + 32 ? n_red - 64 * c : 32 * half + 32;
            for (int l = 32 * half; l < end; ++l) {         // uniform
                const uint32_t bit = 1u << (l & 31);
                const uint32_t own = __builtin_amdgcn_readlane(row[c][wk], l);
                if (own & bit) continue;                    // R descends from F
                uint32_t r_row[W];
#pragma unroll
                for (int w = wk; w < W; ++w) r_row[w] = __builtin_amdgcn_readlane(row[c][w], l);
#pragma unroll
                for (int c2 = c; c2 < NC; ++c2) {
                    if (row[c2][wk] & bit) {
#pragma unroll
                        for (int w = wk; w < W; ++w) row[c2][w] |= r_row[w];
                    }
                }
                drawn[c] |= uint64_t(1) << l;
            }
        }
    }
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        if (r_of[c] >= 0) {
            const bool edges = (drawn[c] >> lane) & 1;
            s.flags[r_of[c]] |= edges ? kFlagMerged : 8;
            if (edges) atomicAdd(&s.merge_cnt[f_of[c]], 1);
        }
    }
}

// After construct(): takes the redundant nodes in id order and decides for each whether its merge edges are drawn
// (kFlagMerged, merge_cnt of the first occurrence) or it descends from its first occurrence (bit 3).
// Uses s.cls (free after construct) for the list of redundant nodes and s.pool for the table of first occurrences.
__device__ __forceinline__ void decide_merges(GraphLds &s, int n) {
    const int i = threadIdx.x;
    const bool red = i < n && (s.flags[i] & kFlagExists) && (s.flags[i] & 4);
    uint32_t *col = reinterpret_cast<uint32_t *>(s.pool);
#pragma unroll
    for (int w = 0; w < 16; ++w) col[w * GSD_MAX_NODES_PER_SEQ + i] = 0;
    const int pos = block_scan(s, s.scan, red ? 1 : 0) - 1;
    const int n_red = s.scan[kGraphThreads - 1];
    if (red) {
        s.cls[pos] = i;
        atomicOr(&col[(pos >> 5) * GSD_MAX_NODES_PER_SEQ + s.merged_to[i]], 1u << (pos & 31));
    }
    __syncthreads();
    if (i < 64 && n_red > 0) {                              // the first wave; the others wait for its decisions
        if (n_red <= 64) decide_in_one_wave<1>(s, n_red);
        else if (n_red <= 128) decide_in_one_wave<2>(s, n_red);
        else if (n_red <= 256) decide_in_one_wave<4>(s, n_red);
        else decide_in_one_wave<8>(s, n_red);
    }
    __syncthreads();
}

// Rank of the calling thread by (key, thread id) among the threads with `valid`; key in [0, GSD_MAX_NODES_PER_SEQ).
// A wave counts its threads per key with ballots (a thread's place among its wave's equals comes out of the same
// ballot), the counts go into table[key][wave], and a scan over the table in that order turns them into the first
// rank of every (key, wave).  Afterwards table[key * 8] is the number of valid threads with a smaller key, and
// `total` the number of valid threads.  `table`: 8 * GSD_MAX_NODES_PER_SEQ words.
__device__ __forceinline__ int stable_rank(GraphLds &s, int32_t *table, int key, bool valid, int &total) {
    constexpr int kWaves = kGraphThreads / 64;
    const int i = threadIdx.x, lane = i & 63, wave = i >> 6;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) table[i * kWaves + w] = 0;
    __syncthreads();
    int place = 0;
    uint64_t todo = __ballot(valid);
    while (todo != 0) {                                     // one turn per distinct key of the wave
        const int leader = __ffsll(static_cast<unsigned long long>(todo)) - 1;
        const int k = __builtin_amdgcn_readlane(key, leader);
        const uint64_t same = __ballot(valid && key == k);
        if (valid && key == k) place = __popcll(same & ((uint64_t(1) << lane) - 1));
        if (lane == leader) table[k * kWaves + wave] = __popcll(same);
        todo &= ~same;
    }
    __syncthreads();
    int cnt[kWaves], mine = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        cnt[w] = table[i * kWaves + w];
        mine += cnt[w];
    }
    int first = block_scan(s, s.scan, mine) - mine;         // threads with a smaller key
    total = s.scan[kGraphThreads - 1];
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        table[i * kWaves + w] = first;
        first += cnt[w];
    }
    __syncthreads();
    return valid ? table[key * kWaves + wave] + place : -1;     // (the caller meets at a barrier before the table is used again)
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
    const int nodes = block_scan(s, s.scan, ex ? 1 : 0);
    const int total_nodes = s.scan[kGraphThreads - 1];
    __syncthreads();
    const int edges = block_scan(s, s.scan, ex ? 1 + (s.par[i] >= 0 ? s.merge_cnt[s.par[i]] : 0) : 0);
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
    int32_t *table = reinterpret_cast<int32_t *>(s.pool);            // the ancestor rows are not needed any more
    int32_t *node_of = table + 8 * GSD_MAX_NODES_PER_SEQ;           // node with a given new id
    int total_nodes = 0;
    const int my_new = stable_rank(s, table, ex ? level[i] : 0, ex, total_nodes);
    new_id[i] = my_new;
    if (ex) node_of[my_new] = i;
    __syncthreads();
    // the mergers of every first occurrence, sorted by new id: with the threads standing in the order of the new ids,
    // a merger's place in the list of all mergers is its rank by (first occurrence, new id)
    const int node_r = i < total_nodes ? node_of[i] : -1;         // this thread stands for the node with new id i
    const bool v_merger = node_r >= 0 && (s.flags[node_r] & kFlagMerged);
    int total_mergers = 0;
    const int place = stable_rank(s, table, v_merger ? s.merged_to[node_r] : 0, v_merger, total_mergers);
    list_off[i] = table[i * (kGraphThreads / 64)];
    if (v_merger) list[place] = i;
    __syncthreads();
    // edges, in the order of the new ids
    const int my_edges = ex ? 1 + (my_par >= 0 ? s.merge_cnt[my_par] : 0) : 0;
    int32_t *by_rank = s.depth;             // depth is not read any more
    by_rank[i] = 0;
    __syncthreads();
    if (ex) by_rank[my_new] = my_edges;
    __syncthreads();
    (void)block_scan(s, s.scan, by_rank[i]);
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
