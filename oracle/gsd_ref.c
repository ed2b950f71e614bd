/*
 * gsd_ref.c -- plain, slow CPU oracle for the verification hot path of Graph-structured Speculative
 * Decoding (GSD).  THIS IS TEST INFRASTRUCTURE: it exists so that the GPU library can be checked against
 * the paper's definitions.  It shares no code with the GPU path, is never tuned, and must never be called
 * from the product path (only tests, the smoke check and the benchmark's cpu_baseline leg use it).
 *
 * What it computes, and the passage each part follows:
 *
 *   gsd_ref_build_mask           Section 4.1 (tree attention: a flattened token may attend only to its
 *                                ancestors) applied to the token graph of Section 5.3 (a DAG): the
 *                                visibility set of node i is i itself plus every node from which i can be
 *                                reached over parent edges.  Written as a depth-first walk from each node.
 *   gsd_ref_dag_attention(_rows) Sections 4.1 / 5.4: one verifier pass over the flattened graph; node i's
 *                                query attends to the whole context (the root, Section 4) and to its
 *                                visible draft nodes.  Ordinary softmax attention written out in fp64.
 *   gsd_ref_node_argmax          Section 3, deterministic verification: the token the LLM itself would
 *                                generate after a node = first index of the row maximum of its logits.
 *   gsd_ref_accept_longest_path  Sections 3 and 4.1: a root path is accepted while every drafted token
 *                                equals the LLM's own choice after its predecessor; the first mismatch
 *                                discards the rest; the longest accepted path from the root is taken, and
 *                                the LLM's token after its last node is the regenerated ("bonus") token.
 *
 * Readings where the paper is silent: a node sees itself (so a chain is plain causal attention); every
 * node sees the whole prefix; the LLM's choice after the bare context is an input (root_pred); ties between
 * equally long accepted paths go to the smallest end node, then walking back to the smallest parent id (the
 * root counts as smallest); argmax ties go to the lowest index and NaN never wins.
 *
 * All pointers are host pointers.  Floating-point inputs are either fp32 (dtype 0) or bf16 bit patterns in
 * uint16 (dtype 1); both are widened exactly to fp64 before any arithmetic.
 */
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define GSD_REF_F32 0
#define GSD_REF_BF16 1

static double load_elt(const void *base, int dtype, int64_t idx) {
    if (dtype == GSD_REF_F32) return (double)((const float *)base)[idx];
    uint32_t bits = ((uint32_t)((const uint16_t *)base)[idx]) << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

/* Threads the row loops will use (for reporting next to timings). */
int gsd_ref_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------------------------------------ mask */

/* Marks node `i` and, recursively, all its ancestors in `seen` (depth-first over parent edges). */
static void visit_ancestors(int32_t i, int64_t node_base, const int32_t *parent_offsets,
                            const int32_t *parent_idx, uint8_t *seen, int32_t *bad) {
    if (seen[i]) return;
    seen[i] = 1;
    for (int32_t e = parent_offsets[node_base + i]; e < parent_offsets[node_base + i + 1]; ++e) {
        int32_t p = parent_idx[e];
        if (p == -1) continue;              /* the root: the context, always visible, not a mask bit */
        if (p < -1 || p >= i) {             /* not a topological order (or out of range): flag, ignore */
            *bad = 1;
            continue;
        }
        visit_ancestors(p, node_base, parent_offsets, parent_idx, seen, bad);
    }
}

/* mask[(node_offsets[b]+i)*W + j/64] bit (j%64) = 1 iff draft node j of sequence b is visible to node i. */
int gsd_ref_build_mask(int32_t batch, int32_t words_per_row, const int32_t *node_offsets,
                       const int32_t *parent_offsets, const int32_t *parent_idx, uint64_t *mask,
                       int32_t *dag_error_flag) {
    int32_t bad = 0;
    for (int32_t b = 0; b < batch; ++b) {
        int64_t base = node_offsets[b];
        int32_t n = node_offsets[b + 1] - node_offsets[b];
        if (n > words_per_row * 64) return -1;
        uint8_t *seen = (uint8_t *)malloc((size_t)(n > 0 ? n : 1));
        for (int32_t i = 0; i < n; ++i) {
            memset(seen, 0, (size_t)n);
            visit_ancestors(i, base, parent_offsets, parent_idx, seen, &bad);
            uint64_t *row = mask + (base + i) * words_per_row;
            for (int32_t w = 0; w < words_per_row; ++w) row[w] = 0;
            for (int32_t j = 0; j < n; ++j)
                if (seen[j]) row[j / 64] |= (uint64_t)1 << (j % 64);
        }
        free(seen);
    }
    if (dag_error_flag) *dag_error_flag = bad;
    return 0;
}

/* ------------------------------------------------------------------------------------------- attention */

typedef struct {
    int32_t batch, num_q_heads, num_kv_heads, head_dim, dtype, words_per_row;
    double scale;
    const void *q;              /* element (t,h,d) at t*q_token_stride + h*q_head_stride + d            */
    const void *k, *v;          /* element (row,hk,d) at row*kv_token_stride + hk*kv_head_stride + d    */
    int64_t q_token_stride, q_head_stride, kv_token_stride, kv_head_stride;
    const int64_t *kv_offsets;  /* [B] first K/V row of sequence b: P_b prefix rows, then its N_b draft rows */
    const int32_t *prefix_lens; /* [B] */
    const int32_t *node_offsets;/* [B+1] */
    const uint64_t *mask;       /* [T][W] */
} attn_args;

/* One output row: packed node t (sequence b, local id i), query head h.  out[D] fp64, *lse natural log. */
static void attention_row(const attn_args *a, int32_t b, int32_t i, int32_t h, double *out, double *lse,
                          double *score_buf, int64_t *key_buf) {
    const int32_t D = a->head_dim;
    const int32_t group = a->num_q_heads / a->num_kv_heads;
    const int32_t hk = h / group;
    const int64_t t = (int64_t)a->node_offsets[b] + i;
    const int32_t n = a->node_offsets[b + 1] - a->node_offsets[b];
    const int32_t P = a->prefix_lens[b];
    const uint64_t *row_mask = a->mask + t * a->words_per_row;

    /* the allowed keys: every prefix row, then the visible draft rows */
    int64_t nkeys = 0;
    for (int32_t j = 0; j < P; ++j) key_buf[nkeys++] = a->kv_offsets[b] + j;
    for (int32_t j = 0; j < n; ++j)
        if ((row_mask[j / 64] >> (j % 64)) & 1) key_buf[nkeys++] = a->kv_offsets[b] + P + j;

    double m = -INFINITY;
    for (int64_t x = 0; x < nkeys; ++x) {
        double s = 0.0;
        for (int32_t d = 0; d < D; ++d)
            s += load_elt(a->q, a->dtype, t * a->q_token_stride + (int64_t)h * a->q_head_stride + d) *
                 load_elt(a->k, a->dtype, key_buf[x] * a->kv_token_stride + (int64_t)hk * a->kv_head_stride + d);
        s *= a->scale;
        score_buf[x] = s;
        if (s > m) m = s;
    }
    double denom = 0.0;
    for (int32_t d = 0; d < D; ++d) out[d] = 0.0;
    for (int64_t x = 0; x < nkeys; ++x) {
        double w = exp(score_buf[x] - m);
        denom += w;
        for (int32_t d = 0; d < D; ++d)
            out[d] += w * load_elt(a->v, a->dtype,
                                   key_buf[x] * a->kv_token_stride + (int64_t)hk * a->kv_head_stride + d);
    }
    if (nkeys == 0) {                       /* cannot happen with a self bit; defined as zeros anyway */
        if (lse) *lse = -INFINITY;
        return;
    }
    for (int32_t d = 0; d < D; ++d) out[d] /= denom;
    if (lse) *lse = m + log(denom);
}

static int32_t max_keys(const attn_args *a) {
    int32_t best = 0;
    for (int32_t b = 0; b < a->batch; ++b) {
        int32_t x = a->prefix_lens[b] + (a->node_offsets[b + 1] - a->node_offsets[b]);
        if (x > best) best = x;
    }
    return best;
}

static attn_args pack_args(int32_t batch, int32_t num_q_heads, int32_t num_kv_heads, int32_t head_dim,
                           int32_t dtype, double scale, const void *q, int64_t q_token_stride,
                           int64_t q_head_stride, const void *k, const void *v, int64_t kv_token_stride,
                           int64_t kv_head_stride, const int64_t *kv_offsets, const int32_t *prefix_lens,
                           const int32_t *node_offsets, const uint64_t *mask, int32_t words_per_row) {
    attn_args a;
    a.batch = batch; a.num_q_heads = num_q_heads; a.num_kv_heads = num_kv_heads; a.head_dim = head_dim;
    a.dtype = dtype; a.words_per_row = words_per_row; a.scale = scale;
    a.q = q; a.k = k; a.v = v;
    a.q_token_stride = q_token_stride; a.q_head_stride = q_head_stride;
    a.kv_token_stride = kv_token_stride; a.kv_head_stride = kv_head_stride;
    a.kv_offsets = kv_offsets; a.prefix_lens = prefix_lens; a.node_offsets = node_offsets; a.mask = mask;
    return a;
}

/* All rows.  out[T][Hq][D] fp64 (contiguous), lse[T][Hq] fp64 or NULL. */
int gsd_ref_dag_attention(int32_t batch, int32_t num_q_heads, int32_t num_kv_heads, int32_t head_dim,
                          int32_t dtype, double scale, const void *q, int64_t q_token_stride,
                          int64_t q_head_stride, const void *k, const void *v, int64_t kv_token_stride,
                          int64_t kv_head_stride, const int64_t *kv_offsets, const int32_t *prefix_lens,
                          const int32_t *node_offsets, const uint64_t *mask, int32_t words_per_row,
                          double *out, double *lse) {
    if (num_kv_heads <= 0 || num_q_heads % num_kv_heads != 0) return -1;
    attn_args a = pack_args(batch, num_q_heads, num_kv_heads, head_dim, dtype, scale, q, q_token_stride,
                            q_head_stride, k, v, kv_token_stride, kv_head_stride, kv_offsets, prefix_lens,
                            node_offsets, mask, words_per_row);
    const int32_t mk = max_keys(&a);
    for (int32_t b = 0; b < batch; ++b) {
        const int32_t n = node_offsets[b + 1] - node_offsets[b];
#pragma omp parallel
        {
            double *score_buf = (double *)malloc(sizeof(double) * (size_t)(mk > 0 ? mk : 1));
            int64_t *key_buf = (int64_t *)malloc(sizeof(int64_t) * (size_t)(mk > 0 ? mk : 1));
#pragma omp for collapse(2) schedule(dynamic, 1)
            for (int32_t h = 0; h < num_q_heads; ++h)
                for (int32_t i = 0; i < n; ++i) {
                    int64_t t = (int64_t)node_offsets[b] + i;
                    attention_row(&a, b, i, h, out + (t * num_q_heads + h) * head_dim,
                                  lse ? lse + t * num_q_heads + h : NULL, score_buf, key_buf);
                }
            free(score_buf);
            free(key_buf);
        }
    }
    return 0;
}

/* A chosen subset of rows (for spot checks at sizes where all rows would take too long):
 * row r is (sequence row_b[r], local node row_i[r], query head row_h[r]); out[n_rows][D], lse[n_rows]. */
int gsd_ref_dag_attention_rows(int32_t batch, int32_t num_q_heads, int32_t num_kv_heads, int32_t head_dim,
                               int32_t dtype, double scale, const void *q, int64_t q_token_stride,
                               int64_t q_head_stride, const void *k, const void *v,
                               int64_t kv_token_stride, int64_t kv_head_stride, const int64_t *kv_offsets,
                               const int32_t *prefix_lens, const int32_t *node_offsets,
                               const uint64_t *mask, int32_t words_per_row, int64_t n_rows,
                               const int32_t *row_b, const int32_t *row_i, const int32_t *row_h,
                               double *out, double *lse) {
    if (num_kv_heads <= 0 || num_q_heads % num_kv_heads != 0) return -1;
    attn_args a = pack_args(batch, num_q_heads, num_kv_heads, head_dim, dtype, scale, q, q_token_stride,
                            q_head_stride, k, v, kv_token_stride, kv_head_stride, kv_offsets, prefix_lens,
                            node_offsets, mask, words_per_row);
    const int32_t mk = max_keys(&a);
    for (int64_t r = 0; r < n_rows; ++r) {
        if (row_b[r] < 0 || row_b[r] >= batch || row_h[r] < 0 || row_h[r] >= num_q_heads) return -1;
        if (row_i[r] < 0 || row_i[r] >= node_offsets[row_b[r] + 1] - node_offsets[row_b[r]]) return -1;
    }
#pragma omp parallel
    {
        double *score_buf = (double *)malloc(sizeof(double) * (size_t)(mk > 0 ? mk : 1));
        int64_t *key_buf = (int64_t *)malloc(sizeof(int64_t) * (size_t)(mk > 0 ? mk : 1));
#pragma omp for schedule(dynamic, 1)
        for (int64_t r = 0; r < n_rows; ++r)
            attention_row(&a, row_b[r], row_i[r], row_h[r], out + r * head_dim, lse ? lse + r : NULL,
                          score_buf, key_buf);
        free(score_buf);
        free(key_buf);
    }
    return 0;
}

/* ---------------------------------------------------------------------------------------------- argmax */

/* pred[r] = lowest index holding the largest non-NaN value of row r (0 if the whole row is NaN). */
int gsd_ref_node_argmax(int64_t rows, int32_t vocab, int32_t dtype, const void *logits, int64_t row_stride,
                        int32_t *pred) {
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        int32_t best = -1;
        double best_val = 0.0;
        for (int32_t x = 0; x < vocab; ++x) {
            double val = load_elt(logits, dtype, r * row_stride + x);
            if (isnan(val)) continue;
            if (best < 0 || val > best_val) {
                best = x;
                best_val = val;
            }
        }
        pred[r] = best < 0 ? 0 : best;
    }
    return 0;
}

/* ------------------------------------------------------------------------------------------ acceptance */

/*
 * For each sequence: path_len[i] = number of nodes on the longest accepted root path that ends at node i,
 * or -1 if no accepted path reaches i.  An edge p -> i is accepted iff tokens[i] equals the LLM's choice
 * after p (pred[p], or root_pred[b] when p is the root); a path is accepted iff all its edges are.
 * Outputs: accept_len[b], accept_path[b][0..len) (sequence-local ids from the root outwards, -1 padded to
 * max_nodes), bonus_token[b] = the LLM's choice after the path's last node (root_pred[b] if len == 0).
 */
int gsd_ref_accept_longest_path(int32_t batch, int32_t max_nodes, const int32_t *node_offsets,
                                const int32_t *parent_offsets, const int32_t *parent_idx,
                                const int32_t *tokens, const int32_t *pred, const int32_t *root_pred,
                                int32_t *accept_len, int32_t *accept_path, int32_t *bonus_token) {
    for (int32_t b = 0; b < batch; ++b) {
        const int64_t base = node_offsets[b];
        const int32_t n = node_offsets[b + 1] - node_offsets[b];
        if (n > max_nodes) return -1;
        int32_t *path_len = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
        int32_t best_len = 0, best_end = -1;
        for (int32_t i = 0; i < n; ++i) {
            int32_t L = -1;
            for (int32_t e = parent_offsets[base + i]; e < parent_offsets[base + i + 1]; ++e) {
                int32_t p = parent_idx[e];
                if (p < -1 || p >= i) continue;                  /* malformed edge: ignored */
                int32_t len_p = (p == -1) ? 0 : path_len[p];
                int32_t llm_choice = (p == -1) ? root_pred[b] : pred[base + p];
                if (len_p >= 0 && tokens[base + i] == llm_choice && len_p + 1 > L) L = len_p + 1;
            }
            path_len[i] = L;
            if (L > best_len) {                                  /* strict: the smallest id wins a tie */
                best_len = L;
                best_end = i;
            }
        }
        int32_t *out_path = accept_path + (int64_t)b * max_nodes;
        for (int32_t x = 0; x < max_nodes; ++x) out_path[x] = -1;
        accept_len[b] = best_len;
        bonus_token[b] = (best_end < 0) ? root_pred[b] : pred[base + best_end];
        int32_t v = best_end;
        for (int32_t pos = best_len - 1; pos >= 0; --pos) {
            out_path[pos] = v;
            /* smallest-id accepted parent whose own longest path is exactly one shorter */
            int32_t chosen = INT32_MAX;
            for (int32_t e = parent_offsets[base + v]; e < parent_offsets[base + v + 1]; ++e) {
                int32_t p = parent_idx[e];
                if (p < -1 || p >= v) continue;
                int32_t len_p = (p == -1) ? 0 : path_len[p];
                int32_t llm_choice = (p == -1) ? root_pred[b] : pred[base + p];
                if (len_p == pos && tokens[base + v] == llm_choice && p < chosen) chosen = p;
            }
            v = chosen;                                          /* -1 (root) exactly when pos == 0 */
        }
        free(path_len);
    }
    return 0;
}
