/*
 * gsd.h -- C ABI of the MI355X (gfx950) verification hot path of Graph-structured Speculative Decoding.
 *
 * One verifier pass over the flattened token graph (paper Sections 4.1, 5.3, 5.4) and the deterministic
 * acceptance step (Section 3):
 *
 *   gsd_build_mask            token graph (DAG) -> per-node visibility bitmask (ancestor closure)
 *   gsd_dag_attention         masked attention of every packed draft node over [context ; visible nodes]
 *   gsd_node_argmax           the verifier's own next token after every node (row argmax of the logits);
 *                             gsd_node_argmax_stats: the same sweep also leaves the softmax normalisers
 *   gsd_accept_longest_path   longest root path on which every drafted token equals the verifier's choice
 * and, around that pass,
 *   gsd_unmerge_to_tree       token graph -> token tree with replicated successors (Section 5.4), gsd_gather_rows
 *   gsd_commit_kv             accepted path -> contiguous context rows of the KV cache (Section 7.1)
 *   gsd_accept_stochastic     non-deterministic verification (Sections 3, 6.4), gsd_softmax_stats
 *   gsd_build_token_graph     drafted token tree -> pruned, merged token graph (Sections 4.2, 5.2, 5.3)
 *
 * Conventions common to all calls
 *   - Every data pointer is a DEVICE pointer owned by the caller; scalars and the descriptor struct are host
 *     values.  The library allocates nothing, frees nothing and keeps no state between calls.
 *   - Work is enqueued on `hip_stream` (a hipStream_t passed as void*, NULL = the default stream) and the call
 *     returns without synchronising.  Outputs are deterministic run to run (bit-identical).
 *   - Return value: GSD_OK or a GSD_ERR_* code.  Host-checkable mistakes (null pointer, non-positive size,
 *     unsupported head_dim, head counts that do not divide, words_per_row or workspace too small) are
 *     reported before anything is launched and leave all outputs untouched; gsd_last_error() then holds a
 *     detail string for the calling thread.  Mistakes only the device can see (a parent id that is not an
 *     earlier node, i.e. a graph that is not listed in topological order) are reported through `dag_error_flag`,
 *     never through the return value: the library does not wait for the device.
 *   - Packed nodes: sequence b owns packed rows node_offsets[b] .. node_offsets[b+1]-1, listed in a
 *     topological order of its graph; parent ids are sequence-local, -1 names the root (the context at the
 *     start of drafting, Section 4).
 */
#ifndef GSD_H
#define GSD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    GSD_OK = 0,
    GSD_ERR_INVALID_ARG = 1,
    GSD_ERR_UNSUPPORTED = 3,
    GSD_ERR_WORKSPACE = 4,
    GSD_ERR_HIP = 5
};

enum { GSD_F32 = 0, GSD_BF16 = 1 };

/* Limits of this build. */
#define GSD_MAX_NODES_PER_SEQ 512 /* nodes of one sequence (mask builder and acceptance keep a sequence in LDS) */

/* Static strings; never NULL. */
const char *gsd_status_string(int status);
/* Detail of the last error returned on this thread ("" if none). */
const char *gsd_last_error(void);
/* Library version string, e.g. "gsd-gfx950 0.1". */
const char *gsd_version(void);

/*
 * Visibility mask (Section 4.1: a flattened token attends only to its ancestors; Section 5.3: the token graph
 * is a DAG, so "ancestors" is the closure over ALL parent edges).  For every packed node t = node_offsets[b]+i
 *     mask[t][j/64] bit (j%64, LSB first) = 1  iff  j == i or node j of sequence b is an ancestor of node i.
 * The row is fully overwritten (bits at and beyond the sequence's node count are 0).  The root is not a bit:
 * the context is visible to every node.
 *
 *   batch            B >= 1
 *   max_nodes        upper bound on the nodes of any one sequence, 1..GSD_MAX_NODES_PER_SEQ
 *   node_offsets     [B+1] int32
 *   parent_offsets   [T+1] int32, CSR over packed nodes (T = node_offsets[B])
 *   parent_idx       [E]   int32, sequence-local parent id (< the child's id) or -1 for the root
 *   mask             [T][words_per_row] uint64, words_per_row >= ceil(max_nodes/64)
 *   dag_error_flag   [1] int32 or NULL; set to 1 (never cleared) if some parent id is >= its child or < -1;
 *                    such an edge is ignored.  Clear it before the call if you read it afterwards.
 */
int gsd_build_mask(int32_t batch, int32_t max_nodes, int32_t words_per_row, const int32_t *node_offsets,
                   const int32_t *parent_offsets, const int32_t *parent_idx, uint64_t *mask,
                   int32_t *dag_error_flag, void *hip_stream);

/*
 * DAG-masked attention (Sections 4.1 and 5.4: the verifier scores all hypotheses in one pass over the
 * flattened graph).  For packed node t of sequence b and query head h (KV head h / (Hq/Hkv)):
 *     O[t][h] = softmax_j( scale * <Q[t][h], K_j> ) . V_j     over j in  prefix rows 0..P_b-1 of sequence b
 *                                                              and draft rows whose bit is set in mask[t]
 * Sequence b's K/V rows are contiguous: row kv_offsets[b] + j for prefix position j < P_b, then row
 * kv_offsets[b] + P_b + i for draft node i.  Element (row, kv_head, d) lives at
 * row*kv_token_stride + kv_head*kv_head_stride + d (strides in elements; d is contiguous).  Q and O element
 * (t, h, d) lives at t*token_stride + h*head_stride + d.  Rows must be 16-byte aligned (pointers and strides
 * multiples of 8 elements for bf16, 4 for f32).
 *
 * dtype GSD_BF16: Q/K/V/O are bf16, both contractions run on the matrix cores with fp32 accumulation, softmax
 * in fp32, O rounded to nearest-even.  dtype GSD_F32: everything fp32.  head_dim must be 64 or 128.
 * lse (optional, [T][Hq] fp32): natural-log sum of exp of the scaled scores over the visible keys.
 *
 * Small problems are split along the KV prefix across work-groups and merged by a second kernel in a fixed
 * order; the partial results live in `workspace` (gsd_dag_attention_workspace() bytes, 0 if unsplit).
 */
typedef struct gsd_attn_desc {
    int32_t batch;         /* B */
    int32_t total_nodes;   /* T = node_offsets[B] (host copy) */
    int32_t max_nodes;     /* upper bound on nodes per sequence (sizes the grid) */
    int32_t max_prefix;    /* upper bound on prefix_lens[b] (sizes the KV split) */
    int32_t num_q_heads;   /* Hq */
    int32_t num_kv_heads;  /* Hkv, divides Hq */
    int32_t head_dim;      /* D: 64 or 128 */
    int32_t dtype;         /* GSD_F32 or GSD_BF16 */
    int32_t words_per_row; /* uint64 words per mask row, >= ceil(max_nodes/64) */
    int32_t num_splits;    /* KV splits: 0 = let the library choose, >= 1 = forced */
    float softmax_scale;   /* e.g. 1/sqrt(D) */
    int32_t wg_waves;      /* tuning: work-group shape of the bf16 kernel: 0 = let the library choose; 4 or 8 = that many
                              wavefronts of 32 query rows each; 64 = 4 wavefronts of 64 query rows each */
    const void *q;         /* [T][Hq][D] via strides */
    void *o;               /* same shape and dtype as q */
    float *lse;            /* [T][Hq] contiguous, or NULL */
    const void *k;
    const void *v;
    const int64_t *kv_offsets;   /* [B] */
    const int32_t *prefix_lens;  /* [B] */
    const int32_t *node_offsets; /* [B+1] */
    const uint64_t *mask;        /* [T][words_per_row] from gsd_build_mask */
    int64_t q_token_stride, q_head_stride;
    int64_t o_token_stride, o_head_stride;
    int64_t kv_token_stride, kv_head_stride;
    void *workspace;             /* device scratch for split partials, may be NULL when 0 bytes are needed */
    size_t workspace_bytes;
} gsd_attn_desc;

/* Bytes of workspace gsd_dag_attention needs for this descriptor (0 when it will not split).  Returns
 * (size_t)-1 if the descriptor is invalid (see gsd_last_error()).  Touches no device memory. */
size_t gsd_dag_attention_workspace(const gsd_attn_desc *desc);
/* Number of KV splits the library will use for this descriptor (>= 1), or -1 if invalid. */
int gsd_dag_attention_splits(const gsd_attn_desc *desc);
int gsd_dag_attention(const gsd_attn_desc *desc, void *hip_stream);

/*
 * gsd_dag_attention for callers that cannot allocate device memory or pass a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): the same kernels and the same results, but the
 * split-KV partials live in an array of GSD_STATIC_SCRATCH_BYTES inside the library, one copy per GPU, held until
 * the process ends.  desc->workspace and desc->workspace_bytes are ignored.  A descriptor whose partials
 * (gsd_dag_attention_workspace() bytes) exceed GSD_STATIC_SCRATCH_BYTES is rejected with GSD_ERR_WORKSPACE before
 * anything is launched.  Calls no allocating routine.  All calls on one GPU share that GPU's array: two calls that
 * overlap in time on one GPU (different streams, different threads) race and give wrong results; calls on one
 * stream are safe.  Nothing in the array has to start at zero: a launch writes every partial it later reads.
 */
#define GSD_STATIC_SCRATCH_BYTES (32u << 20)
int gsd_dag_attention_static(const gsd_attn_desc *desc, void *hip_stream);

/*
 * Deterministic verification, part 1 (Section 3: a drafted token is accepted only if the LLM would generate
 * the same): pred[r] = the lowest index holding the largest value of row r of the logits.  NaN never wins; a
 * row of only NaN gives 0.  logits element (r, x) lives at r*row_stride + x (elements).
 *   rows >= 1, vocab >= 1, dtype GSD_F32 or GSD_BF16, pred [rows] int32.
 */
int gsd_node_argmax(int32_t rows, int32_t vocab, int dtype, const void *logits, int64_t row_stride,
                    int32_t *pred, void *hip_stream);

/*
 * gsd_node_argmax and gsd_softmax_stats (below) in ONE pass over the logits: the verifier's own token after every
 * node (Section 3, deterministic verification) and the normaliser of its distribution there (Section 3, the
 * probabilities non-deterministic verification compares), for callers that want both without reading the logits
 * twice.  pred as gsd_node_argmax (bit-identical); row_max[r] = max_x logits[r][x], row_sumexp[r] = sum_x
 * exp(logits[r][x] - row_max[r]) in fp32 (same definition as gsd_softmax_stats; the summation order differs, so the
 * last bits may).  rows >= 1, vocab >= 1; pred [rows] int32; row_max, row_sumexp [rows] fp32.
 */
int gsd_node_argmax_stats(int32_t rows, int32_t vocab, int dtype, const void *logits, int64_t row_stride,
                          int32_t *pred, float *row_max, float *row_sumexp, void *hip_stream);

/*
 * Deterministic verification, part 2 (Sections 3 and 4.1): an edge p -> i is accepted iff tokens[i] equals
 * the LLM's choice after p (pred[p]; root_pred[b] when p is the root).  A root path is accepted iff all its
 * edges are: the first mismatch discards everything after it.  Per sequence the longest accepted root path
 * is returned; among equally long ones the end node with the smallest id wins and, walking back, the
 * smallest-id parent that continues a path of full length (the root counts as smallest).
 *
 *   total_nodes  T = node_offsets[B] (host copy; sizes the argmax launch)
 *   tokens       [T] int32 drafted token of every packed node
 *   logits       [T][vocab] or NULL.  When given, pred is first filled by gsd_node_argmax on the same stream.
 *   pred         [T] int32: output when logits != NULL, input otherwise
 *   root_pred    [B] int32: the LLM's choice right after the context
 *   accept_len   [B] int32: number of accepted draft nodes (0 if none)
 *   accept_path  [B][max_nodes] int32: sequence-local node ids from the root outwards, -1 padded
 *   bonus_token  [B] int32: the LLM's choice after the last accepted node (root_pred[b] if accept_len is 0):
 *                the token the LLM regenerates at the first rejection
 * Malformed parent ids (>= child or < -1) are ignored, as in gsd_build_mask.
 */
int gsd_accept_longest_path(int32_t batch, int32_t total_nodes, int32_t max_nodes, const int32_t *node_offsets,
                            const int32_t *parent_offsets, const int32_t *parent_idx, const int32_t *tokens,
                            const void *logits, int dtype, int32_t vocab, int64_t row_stride, int32_t *pred,
                            const int32_t *root_pred, int32_t *accept_len, int32_t *accept_path,
                            int32_t *bonus_token, void *hip_stream);

/*
 * Un-merging the token graph into a token tree (Section 5.4: before verification the graph is reverted to a
 * tree; the successors of a merged node are replicated).  The un-merged tree has one node per ROOT PATH of the
 * graph (root -> v1 -> ... -> vm along parent edges); the tree parent of a path is the path without its last
 * node, and the tree node stands for the graph node the path ends at (its ORIGIN: same token, same per-node
 * data).  Tree nodes of a sequence are numbered in this order: by origin id; paths with the same origin by the
 * position of their last edge in the origin's stored parent list; paths that also share that parent in the
 * order of their parent paths.  Parents precede children, so the output is itself a valid input of every call
 * in this header, and so is any prefix of it: a sequence's list is cut after max_tree_nodes entries (the number
 * of root paths can be exponential in the depth).
 *
 *   batch, max_nodes, node_offsets, parent_offsets, parent_idx: the graph, as for gsd_build_mask
 *   max_tree_nodes      cap on tree nodes per sequence, >= 1, batch * max_tree_nodes < 2^31
 *   tree_node_offsets   [B+1] int32 out: packed tree nodes of sequence b are rows [b] .. [b+1]-1
 *   tree_parent         [>= B*max_tree_nodes] int32 out: sequence-local TREE id of the parent, -1 = root.
 *                       Every tree node has one parent, so the tree's CSR parent_offsets are 0,1,2,...
 *   tree_parent_offsets [>= B*max_tree_nodes + 1] int32 out or NULL: those CSR offsets (entry g = g, g <= T')
 *   tree_origin         [>= B*max_tree_nodes] int32 out: sequence-local graph id of the node replicated
 *   path_count          [B] int64 out: number of root paths of sequence b = its tree size without the cap,
 *                       saturating at 2^62
 *   dag_error_flag      as for gsd_build_mask (a malformed edge is ignored)
 * Only entries below tree_node_offsets[B] are written.  Two launches on `hip_stream`; no host synchronisation:
 * read tree_node_offsets back to learn T' before sizing the calls that consume the tree.
 */
int gsd_unmerge_to_tree(int32_t batch, int32_t max_nodes, int32_t max_tree_nodes, const int32_t *node_offsets,
                        const int32_t *parent_offsets, const int32_t *parent_idx, int32_t *tree_node_offsets,
                        int32_t *tree_parent, int32_t *tree_parent_offsets, int32_t *tree_origin,
                        int64_t *path_count, int32_t *dag_error_flag, void *hip_stream);

/*
 * Row gather, dst[r] = src[index[r]] for r < rows: carries per-node data (queries, keys, values, tokens,
 * predictions) from graph nodes to their replicas in the un-merged tree (Section 5.4).
 *   row_bytes multiple of 4; src/dst strides in bytes, multiples of 4 and >= row_bytes; index [rows] int32,
 *   each in [0, src_rows) (an index outside that range leaves the destination row untouched).
 *   src and dst must not overlap.
 */
int gsd_gather_rows(int64_t rows, int64_t row_bytes, const void *src, int64_t src_rows, int64_t src_stride_bytes,
                    const int32_t *index, void *dst, int64_t dst_stride_bytes, void *hip_stream);

/*
 * KV-cache commit after acceptance (Section 7.1 finds the cache update to be a cost of its own next to drafting
 * and verifying).  The accepted draft tokens become context, everything else drafted in this iteration is
 * dropped: for every layer l, for K and for V, and every j < accept_len[b]
 *     row (kv_offsets[b] + P_b + j)  <-  row (kv_offsets[b] + P_b + accept_path[b][j])        (P_b = prefix_lens[b])
 * in place, reading every source row before any row that overwrites it, and new_prefix_lens[b] = P_b +
 * accept_len[b].  Rows past the new prefix keep whatever they held.  accept_path must be what
 * gsd_accept_longest_path returns (ids strictly increasing, so accept_path[b][j] >= j); an id outside
 * [j, max_nodes) skips that row.
 *
 *   max_nodes          1..GSD_MAX_NODES_PER_SEQ (more: GSD_ERR_UNSUPPORTED)
 *   num_layers >= 1; layer l of K starts at (char*)k + l*layer_stride_bytes (same for v)
 *   row_bytes          bytes of one token's K (or V) in one layer (all KV heads), multiple of 16
 *   token_stride_bytes distance between consecutive rows, multiple of 16, >= row_bytes
 *   k, v               16-byte aligned device pointers
 *   accept_path        [B][max_nodes] int32;  new_prefix_lens [B] int32, must not alias prefix_lens
 */
int gsd_commit_kv(int32_t batch, int32_t max_nodes, int32_t num_layers, int64_t row_bytes, void *k, void *v,
                  int64_t token_stride_bytes, int64_t layer_stride_bytes, const int64_t *kv_offsets,
                  const int32_t *prefix_lens, const int32_t *accept_len, const int32_t *accept_path,
                  int32_t *new_prefix_lens, void *hip_stream);

/*
 * Normaliser of a softmax over each row of logits, in one pass (running maximum and sum of exp(x - max), merged
 * across lanes): row_max[r] = max_x logits[r][x], row_sumexp[r] = sum_x exp(logits[r][x] - row_max[r]).  The
 * vocabulary-wide part of non-deterministic verification (Section 3: acceptance needs the LLM's probability
 * p(token) = exp(logit - max) / sumexp), the counterpart of gsd_node_argmax.  An all -inf row gives (-inf, 0).
 *   rows >= 1, vocab >= 1, dtype GSD_F32 or GSD_BF16, row_stride in elements; row_max, row_sumexp: [rows] fp32.
 */
int gsd_softmax_stats(int64_t rows, int32_t vocab, int dtype, const void *logits, int64_t row_stride, float *row_max,
                      float *row_sumexp, void *hip_stream);

/*
 * Non-deterministic verification on the token graph (Section 3: the i-th drafted token is accepted with probability
 * min(1, p/q), the first rejection discards the rest of its hypothesis and the LLM regenerates that token; Section
 * 6.4: the setting on token graphs, for which the paper states no rule of its own).  As built:
 *   - edge r -> i is accepted iff accept_u[i] < min(1, p_r(tokens[i]) / draft_prob[i]), p_r = softmax of the LLM's
 *     logits after r (the root's after the context); one coin per node, shared by all its parent edges;
 *   - the longest accepted root path is taken, ties as in gsd_accept_longest_path;
 *   - bonus_token is drawn after the path's end node r* by inverse CDF with resample_u[b] (the smallest token whose
 *     cumulative weight exceeds resample_u * total): from max(p - q, 0) at r* when r* has children in the graph
 *     (q = softmax of the draft model's logits after r*; p itself if that residual is empty), from p when it has none.
 * All four logits arrays share dtype, vocab and row_stride (elements).  Malformed parent ids and tokens outside
 * [0, vocab) never pass.  Launches four kernels on `hip_stream` (two normaliser passes, acceptance, draw).
 */
typedef struct gsd_stochastic_desc {
    int32_t batch, total_nodes, max_nodes, vocab, dtype;
    const int32_t *node_offsets;    /* [B+1] */
    const int32_t *parent_offsets;  /* [T+1] */
    const int32_t *parent_idx;      /* [E]   */
    const int32_t *tokens;          /* [T]   */
    const void *logits;             /* [T][vocab] LLM logits after each node */
    const void *root_logits;        /* [B][vocab] LLM logits after the context */
    const void *draft_logits;       /* [T][vocab] draft model's logits after each node */
    const void *root_draft_logits;  /* [B][vocab] */
    int64_t row_stride;
    const float *draft_prob;        /* [T] probability the draft model gave tokens[i] when it drafted node i, > 0 */
    const float *accept_u;          /* [T] uniforms in [0, 1) */
    const float *resample_u;        /* [B] uniforms in [0, 1) */
    float *row_max, *row_sumexp;    /* [T+B] out: softmax normalisers of `logits` rows, then of `root_logits` rows */
    int32_t *accept_len;            /* [B] out */
    int32_t *accept_path;           /* [B][max_nodes] out, -1 padded */
    int32_t *end_node;              /* [B] out: last node of the accepted path, -1 = the root */
    int32_t *bonus_token;           /* [B] out */
} gsd_stochastic_desc;
int gsd_accept_stochastic(const gsd_stochastic_desc *desc, void *hip_stream);

/*
 * Draft-side construction of the token graph (Section 4.2: probability and sibling pruning; Section 5.2: tau-redundant
 * nodes; Section 5.3: merging) from a drafted token TREE: per sequence, nodes in generation order (breadth first, so
 * depths never decrease along the ids), tree_parent[i] < i or -1, the drafted token of every node and the probability
 * the draft model gave it.  Visiting the nodes in that order:
 *   - a node exists only if its parent is the root or an existing node that was expanded;
 *   - it becomes a leaf if draft_prob < theta_prob, or if draft_prob < theta_sib * (largest draft_prob among its
 *     parent's children), both compared in fp32;
 *   - it is tau-redundant, and a leaf, if its depth is >= tau and its tau-gram (its token and those of its tau-1
 *     nearest ancestors in the tree) equals that of an earlier existing node; the earliest such node F is the first
 *     occurrence.  Merging: the redundant node R becomes one more parent of every child of F, whichever layer F lies
 *     in, so that what follows F is reused below R (the edge Section 5.3 draws from R to F).  The exception is an R
 *     that already descends from F in the graph built so far (all parent edges, earlier merge edges included): the
 *     reuse would close a cycle, a case the paper leaves open; such an R is a leaf without merge edges;
 *   - a node is expanded iff it is no leaf.
 * A merge into an earlier layer gives an existing node a parent that was generated after it, so the graph is renumbered
 * into a topological order: by level (0 for the children of the root, otherwise one more than the largest level among
 * the parents), nodes of one level in generation order.  Without such edges this is the generation order.  The output
 * is a valid graph for every call in this header.
 *
 *   tau >= 1; counts [B][2] int32 out (nodes and edges of each sequence's graph)
 *   graph_node_offsets [B+1], parent_offsets [T+1] (only the first T'+1 entries are written), parent_idx
 *   [edge_capacity] (new sequence-local ids, ascending within a node, -1 = root), origin [T] (tree id of each graph
 *   node), flags [T]: bit0 probability-pruned, bit1 sibling-pruned, bit2 redundant, bit3 redundant without merge edges (cyclic case)
 *   error_flag [1] or NULL: bit0 set on malformed input (a parent id >= its child or < -1, ids not breadth first, more
 *   than max_nodes nodes; such nodes are dropped), bit1 if edge_capacity was too small (parent_idx is then incomplete).
 *   Never cleared.  Two launches on `hip_stream`; read graph_node_offsets / parent_offsets back to size what follows.
 */
int gsd_build_token_graph(int32_t batch, int32_t max_nodes, int32_t tau, float theta_prob, float theta_sib,
                          const int32_t *node_offsets, const int32_t *tree_parent, const int32_t *tokens,
                          const float *draft_prob, int32_t *counts, int32_t *graph_node_offsets, int32_t *parent_offsets,
                          int32_t *parent_idx, int64_t edge_capacity, int32_t *origin, int32_t *flags,
                          int32_t *error_flag, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* GSD_H */
