// C ABI of libgsd: argument validation, error reporting and dispatch to the kernel launchers.
// Everything a host can check is checked here, before any launch, so a bad call leaves its outputs untouched.
#include <cstdarg>
#include <cstdio>
#include <cstring>

#include "gsd_internal.h"

namespace {

thread_local char g_last_error[256] = "";

int fail(int code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_last_error, sizeof g_last_error, fmt, ap);
    va_end(ap);
    return code;
}

int hip_fail(hipError_t err, const char *what) {
    return fail(GSD_ERR_HIP, "%s: %s", what, hipGetErrorString(err));
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

int check_attn_desc(const gsd_attn_desc *d) {
    if (!d) return fail(GSD_ERR_INVALID_ARG, "descriptor is NULL");
    if (d->batch < 1 || d->total_nodes < 1 || d->max_nodes < 1 || d->max_prefix < 0)
        return fail(GSD_ERR_INVALID_ARG, "batch, total_nodes, max_nodes must be >= 1 and max_prefix >= 0");
    if (d->num_q_heads < 1 || d->num_kv_heads < 1 || d->num_q_heads % d->num_kv_heads != 0)
        return fail(GSD_ERR_INVALID_ARG, "num_kv_heads (%d) must divide num_q_heads (%d)", d->num_kv_heads,
                    d->num_q_heads);
    if (d->dtype != GSD_F32 && d->dtype != GSD_BF16) return fail(GSD_ERR_UNSUPPORTED, "dtype %d", d->dtype);
    if (d->head_dim != 64 && d->head_dim != 128)
        return fail(GSD_ERR_UNSUPPORTED, "head_dim %d (supported: 64, 128)", d->head_dim);
    if (d->max_nodes > GSD_MAX_NODES_PER_SEQ)
        return fail(GSD_ERR_UNSUPPORTED, "max_nodes %d exceeds %d", d->max_nodes, GSD_MAX_NODES_PER_SEQ);
    if (d->words_per_row < (d->max_nodes + 63) / 64)
        return fail(GSD_ERR_INVALID_ARG, "words_per_row %d too small for max_nodes %d", d->words_per_row,
                    d->max_nodes);
    if (d->num_splits < 0) return fail(GSD_ERR_INVALID_ARG, "num_splits must be >= 0");
    if (d->wg_waves != 0 && d->wg_waves != 4 && d->wg_waves != 8 && d->wg_waves != 64)
        return fail(GSD_ERR_INVALID_ARG, "wg_waves must be 0, 4, 8 or 64");
    if (!(d->softmax_scale > 0.f) || !(d->softmax_scale < 1e6f))
        return fail(GSD_ERR_INVALID_ARG, "softmax_scale must be positive and finite");
    return GSD_OK;
}

}  // namespace

extern "C" {

const char *gsd_status_string(int status) {
    switch (status) {
        case GSD_OK: return "ok";
        case GSD_ERR_INVALID_ARG: return "invalid argument";
        case GSD_ERR_UNSUPPORTED: return "unsupported configuration";
        case GSD_ERR_WORKSPACE: return "workspace too small";
        case GSD_ERR_HIP: return "HIP runtime error";
        default: return "unknown status";
    }
}

const char *gsd_last_error(void) { return g_last_error; }

const char *gsd_version(void) { return "gsd-gfx950 0.1"; }

int gsd_build_mask(int32_t batch, int32_t max_nodes, int32_t words_per_row, const int32_t *node_offsets,
                   const int32_t *parent_offsets, const int32_t *parent_idx, uint64_t *mask,
                   int32_t *dag_error_flag, void *hip_stream) {
    if (batch < 1 || max_nodes < 1) return fail(GSD_ERR_INVALID_ARG, "batch and max_nodes must be >= 1");
    if (max_nodes > GSD_MAX_NODES_PER_SEQ)
        return fail(GSD_ERR_UNSUPPORTED, "max_nodes %d exceeds %d", max_nodes, GSD_MAX_NODES_PER_SEQ);
    if (words_per_row < (max_nodes + 63) / 64)
        return fail(GSD_ERR_INVALID_ARG, "words_per_row %d too small for max_nodes %d", words_per_row, max_nodes);
    if (!node_offsets || !parent_offsets || !parent_idx || !mask)
        return fail(GSD_ERR_INVALID_ARG, "NULL pointer argument");
    hipError_t err = gsd::launch_build_mask(batch, max_nodes, words_per_row, node_offsets, parent_offsets,
                                            parent_idx, mask, dag_error_flag, (hipStream_t)hip_stream);
    return err == hipSuccess ? GSD_OK : hip_fail(err, "gsd_build_mask launch");
}

int gsd_dag_attention_splits(const gsd_attn_desc *desc) {
    if (check_attn_desc(desc) != GSD_OK) return -1;
    return desc->dtype == GSD_BF16 ? gsd::attention_bf16_splits(*desc) : 1;
}

size_t gsd_dag_attention_workspace(const gsd_attn_desc *desc) {
    if (check_attn_desc(desc) != GSD_OK) return (size_t)-1;
    if (desc->dtype != GSD_BF16) return 0;
    return gsd::attention_bf16_workspace(*desc, gsd::attention_bf16_splits(*desc));
}

}  // extern "C"

namespace {

// Shared by the two attention entry points: everything but where the split partials live.
int check_attn_buffers(const gsd_attn_desc &d) {
    if (!d.q || !d.o || !d.k || !d.v || !d.kv_offsets || !d.prefix_lens || !d.node_offsets || !d.mask)
        return fail(GSD_ERR_INVALID_ARG, "NULL pointer argument");
    const int64_t align = d.dtype == GSD_BF16 ? 8 : 4;
    if (!aligned16(d.q) || !aligned16(d.o) || !aligned16(d.k) || !aligned16(d.v))
        return fail(GSD_ERR_INVALID_ARG, "q, o, k, v must be 16-byte aligned");
    const int64_t strides[6] = {d.q_token_stride, d.q_head_stride, d.o_token_stride,
                                d.o_head_stride, d.kv_token_stride, d.kv_head_stride};
    for (int64_t s : strides)
        if (s < d.head_dim || s % align != 0)
            return fail(GSD_ERR_INVALID_ARG, "strides must be >= head_dim and multiples of %lld elements",
                        (long long)align);
    if (int64_t(d.total_nodes) * d.num_q_heads > (int64_t(1) << 30))
        return fail(GSD_ERR_UNSUPPORTED, "total_nodes * num_q_heads too large");
    if (d.dtype == GSD_BF16) {
        // the bf16 kernel addresses a sequence's K/V rows with 32-bit byte offsets from the sequence's first row
        const int64_t row_bytes = d.kv_token_stride * 2;
        if (row_bytes >= (int64_t(1) << 24) ||
            (int64_t(d.max_prefix) + d.max_nodes) * row_bytes >= (int64_t(1) << 31))
            return fail(GSD_ERR_UNSUPPORTED, "one sequence's K/V rows span 2 GiB or more (or a row stride >= 16 MiB)");
    }
    return GSD_OK;
}

}  // namespace

extern "C" {

int gsd_dag_attention(const gsd_attn_desc *desc, void *hip_stream) {
    int rc = check_attn_desc(desc);
    if (rc != GSD_OK) return rc;
    const gsd_attn_desc &d = *desc;
    rc = check_attn_buffers(d);
    if (rc != GSD_OK) return rc;
    hipStream_t stream = (hipStream_t)hip_stream;
    hipError_t err;
    if (d.dtype == GSD_F32) {
        err = gsd::launch_attention_f32(d, stream);
    } else {
        const int splits = gsd::attention_bf16_splits(d);
        const size_t need = gsd::attention_bf16_workspace(d, splits);
        if (need > 0 && (!d.workspace || d.workspace_bytes < need))
            return fail(GSD_ERR_WORKSPACE, "workspace of %zu bytes needed for %d KV splits, %zu given", need, splits,
                        d.workspace ? d.workspace_bytes : size_t(0));
        if (need > 0 && !aligned16(d.workspace)) return fail(GSD_ERR_INVALID_ARG, "workspace must be 16-byte aligned");
        err = gsd::launch_attention_bf16(d, splits, stream);
    }
    return err == hipSuccess ? GSD_OK : hip_fail(err, "gsd_dag_attention launch");
}

int gsd_dag_attention_static(const gsd_attn_desc *desc, void *hip_stream) {
    int rc = check_attn_desc(desc);
    if (rc != GSD_OK) return rc;
    gsd_attn_desc d = *desc;
    rc = check_attn_buffers(d);
    if (rc != GSD_OK) return rc;
    hipStream_t stream = (hipStream_t)hip_stream;
    hipError_t err;
    if (d.dtype == GSD_F32) {
        err = gsd::launch_attention_f32(d, stream);
    } else {
        const int splits = gsd::attention_bf16_splits(d);
        const size_t need = gsd::attention_bf16_workspace(d, splits);
        if (need > GSD_STATIC_SCRATCH_BYTES)
            return fail(GSD_ERR_WORKSPACE, "%zu bytes of split partials (%d KV splits) exceed the static scratch of %zu",
                        need, splits, size_t(GSD_STATIC_SCRATCH_BYTES));
        d.workspace = nullptr;
        d.workspace_bytes = 0;
        if (need > 0) {
            void *ptr = nullptr;
            err = gsd::attention_static_scratch(&ptr);
            if (err != hipSuccess) return hip_fail(err, "gsd_dag_attention_static scratch address");
            d.workspace = ptr;
            d.workspace_bytes = GSD_STATIC_SCRATCH_BYTES;
        }
        err = gsd::launch_attention_bf16(d, splits, stream);
    }
    return err == hipSuccess ? GSD_OK : hip_fail(err, "gsd_dag_attention_static launch");
}

int gsd_node_argmax(int32_t rows, int32_t vocab, int dtype, const void *logits, int64_t row_stride,
                    int32_t *pred, void *hip_stream) {
    if (rows < 1 || vocab < 1) return fail(GSD_ERR_INVALID_ARG, "rows and vocab must be >= 1");
    if (dtype != GSD_F32 && dtype != GSD_BF16) return fail(GSD_ERR_UNSUPPORTED, "dtype %d", dtype);
    if (!logits || !pred) return fail(GSD_ERR_INVALID_ARG, "NULL pointer argument");
    if (row_stride < vocab) return fail(GSD_ERR_INVALID_ARG, "row_stride %lld < vocab %d", (long long)row_stride, vocab);
    const uintptr_t elt = dtype == GSD_BF16 ? 2 : 4;
    if (reinterpret_cast<uintptr_t>(logits) % elt != 0) return fail(GSD_ERR_INVALID_ARG, "logits misaligned");
    hipError_t err = gsd::launch_node_argmax(rows, vocab, dtype, logits, row_stride, pred, nullptr, nullptr,
                                             (hipStream_t)hip_stream);
    return err == hipSuccess ? GSD_OK : hip_fail(err, "gsd_node_argmax launch");
}

int gsd_node_argmax_stats(int32_t rows, int32_t vocab, int dtype, const void *logits, int64_t row_stride,
                          int32_t *pred, float *row_max, float *row_sumexp, void *hip_stream) {
    if (rows < 1 || vocab < 1) return fail(GSD_ERR_INVALID_ARG, "rows and vocab must be >= 1");
    if (dtype != GSD_F32 && dtype != GSD_BF16) return fail(GSD_ERR_UNSUPPORTED, "dtype %d", dtype);
    if (!logits || !pred || !row_max || !row_sumexp) return fail(GSD_ERR_INVALID_ARG, "NULL pointer argument");
    if (row_stride < vocab) return fail(GSD_ERR_INVALID_ARG, "row_stride %lld < vocab %d", (long long)row_stride, vocab);
    const uintptr_t elt = dtype == GSD_BF16 ? 2 : 4;
    if (reinterpret_cast<uintptr_t>(logits) % elt != 0) return fail(GSD_ERR_INVALID_ARG, "logits misaligned");
    hipError_t err = gsd::launch_node_argmax(rows, vocab, dtype, logits, row_stride, pred, row_max, row_sumexp,
                                             (hipStream_t)hip_stream);
    return err == hipSuccess ? GSD_OK : hip_fail(err, "gsd_node_argmax_stats launch");
}

int gsd_accept_longest_path(int32_t batch, int32_t total_nodes, int32_t max_nodes, const int32_t *node_offsets,
                            const int32_t *parent_offsets, const int32_t *parent_idx, const int32_t *tokens,
                            const void *logits, int dtype, int32_t vocab, int64_t row_stride, int32_t *pred,
                            const int32_t *root_pred, int32_t *accept_len, int32_t *accept_path,
                            int32_t *bonus_token, void *hip_stream) {
    if (batch < 1 || max_nodes < 1 || total_nodes < 1)
        return fail(GSD_ERR_INVALID_ARG, "batch, total_nodes and max_nodes must be >= 1");
    if (max_nodes > GSD_MAX_NODES_PER_SEQ)
        return fail(GSD_ERR_UNSUPPORTED, "max_nodes %d exceeds %d", max_nodes, GSD_MAX_NODES_PER_SEQ);
    if (!node_offsets || !parent_offsets || !parent_idx || !tokens || !pred || !root_pred || !accept_len ||
        !accept_path || !bonus_token)
        return fail(GSD_ERR_INVALID_ARG, "NULL pointer argument");
    hipStream_t stream = (hipStream_t)hip_stream;
    if (logits) {
        const int rc = gsd_node_argmax(total_nodes, vocab, dtype, logits, row_stride, pred, hip_stream);
        if (rc != GSD_OK) return rc;
    }
    hipError_t err = gsd::launch_accept(batch, max_nodes, node_offsets, parent_offsets, parent_idx, tokens, pred,
                                        root_pred, accept_len, accept_path, bonus_token, stream);
    return err == hipSuccess ? GSD_OK : hip_fail(err, "gsd_accept_longest_path launch");
}

int gsd_unmerge_to_tree(int32_t batch, int32_t max_nodes, int32_t max_tree_nodes, const int32_t *node_offsets,
                        const int32_t *parent_offsets, const int32_t *parent_idx, int32_t *tree_node_offsets,
                        int32_t *tree_parent, int32_t *tree_parent_offsets, int32_t *tree_origin,
                        int64_t *path_count, int32_t *dag_error_flag, void *hip_stream) {
    if (batch < 1 || max_nodes < 1 || max_tree_nodes < 1)
        return fail(GSD_ERR_INVALID_ARG, "batch, max_nodes and max_tree_nodes must be >= 1");
    if (max_nodes > GSD_MAX_NODES_PER_SEQ)
        return fail(GSD_ERR_UNSUPPORTED, "max_nodes %d exceeds %d", max_nodes, GSD_MAX_NODES_PER_SEQ);
    if (int64_t(batch) * max_tree_nodes >= (int64_t(1) << 31))
        return fail(GSD_ERR_UNSUPPORTED, "batch * max_tree_nodes must stay below 2^31");
    if (!node_offsets || !parent_offsets || !parent_idx || !tree_node_offsets || !tree_parent || !tree_origin ||
        !path_count)
        return fail(GSD_ERR_INVALID_ARG, "NULL pointer argument");
    hipError_t err = gsd::launch_unmerge(batch, max_nodes, max_tree_nodes, node_offsets, parent_offsets, parent_idx,
                                         tree_node_offsets, tree_parent, tree_parent_offsets, tree_origin,
                                         path_count, dag_error_flag, (hipStream_t)hip_stream);
    return err == hipSuccess ? GSD_OK : hip_fail(err, "gsd_unmerge_to_tree launch");
}

int gsd_gather_rows(int64_t rows, int64_t row_bytes, const void *src, int64_t src_rows, int64_t src_stride_bytes,
                    const int32_t *index, void *dst, int64_t dst_stride_bytes, void *hip_stream) {
    if (rows < 1 || src_rows < 1 || row_bytes < 4)
        return fail(GSD_ERR_INVALID_ARG, "rows and src_rows must be >= 1 and row_bytes >= 4");
    if (row_bytes % 4 != 0 || src_stride_bytes % 4 != 0 || dst_stride_bytes % 4 != 0)
        return fail(GSD_ERR_INVALID_ARG, "row_bytes and strides must be multiples of 4");
    if (src_stride_bytes < row_bytes || dst_stride_bytes < row_bytes)
        return fail(GSD_ERR_INVALID_ARG, "strides must be >= row_bytes");
    if (row_bytes / 4 > INT32_MAX) return fail(GSD_ERR_UNSUPPORTED, "row_bytes too large");
    if (!src || !dst || !index) return fail(GSD_ERR_INVALID_ARG, "NULL pointer argument");
    if (reinterpret_cast<uintptr_t>(src) % 4 != 0 || reinterpret_cast<uintptr_t>(dst) % 4 != 0)
        return fail(GSD_ERR_INVALID_ARG, "src and dst must be 4-byte aligned");
    hipError_t err = gsd::launch_gather_rows(rows, row_bytes, src, src_rows, src_stride_bytes, index, dst,
                                             dst_stride_bytes, (hipStream_t)hip_stream);
    return err == hipSuccess ? GSD_OK : hip_fail(err, "gsd_gather_rows launch");
}

int gsd_commit_kv(int32_t batch, int32_t max_nodes, int32_t num_layers, int64_t row_bytes, void *k, void *v,
                  int64_t token_stride_bytes, int64_t layer_stride_bytes, const int64_t *kv_offsets,
                  const int32_t *prefix_lens, const int32_t *accept_len, const int32_t *accept_path,
                  int32_t *new_prefix_lens, void *hip_stream) {
    if (batch < 1 || max_nodes < 1 || num_layers < 1)
        return fail(GSD_ERR_INVALID_ARG, "batch, max_nodes and num_layers must be >= 1");
    if (batch > 32767 || num_layers > 65535)
        return fail(GSD_ERR_UNSUPPORTED, "batch <= 32767 and num_layers <= 65535 (grid limits)");
    if (max_nodes > GSD_MAX_NODES_PER_SEQ)
        return fail(GSD_ERR_UNSUPPORTED, "max_nodes %d exceeds %d", max_nodes, GSD_MAX_NODES_PER_SEQ);
    if (row_bytes < 16 || row_bytes % 16 != 0 || token_stride_bytes % 16 != 0 || token_stride_bytes < row_bytes)
        return fail(GSD_ERR_INVALID_ARG, "row_bytes and token_stride_bytes must be multiples of 16, stride >= row");
    if (row_bytes / 16 > INT32_MAX) return fail(GSD_ERR_UNSUPPORTED, "row_bytes too large");
    if (num_layers > 1 && (layer_stride_bytes % 16 != 0 || layer_stride_bytes < token_stride_bytes))
        return fail(GSD_ERR_INVALID_ARG, "layer_stride_bytes must be a multiple of 16 and >= token_stride_bytes");
    if (!k || !v || !kv_offsets || !prefix_lens || !accept_len || !accept_path || !new_prefix_lens)
        return fail(GSD_ERR_INVALID_ARG, "NULL pointer argument");
    if (!aligned16(k) || !aligned16(v)) return fail(GSD_ERR_INVALID_ARG, "k and v must be 16-byte aligned");
    if (new_prefix_lens == prefix_lens)
        return fail(GSD_ERR_INVALID_ARG, "new_prefix_lens must not alias prefix_lens");
    hipError_t err = gsd::launch_commit_kv(batch, max_nodes, num_layers, row_bytes, k, v, token_stride_bytes,
                                           layer_stride_bytes, kv_offsets, prefix_lens, accept_len, accept_path,
                                           new_prefix_lens, (hipStream_t)hip_stream);
    return err == hipSuccess ? GSD_OK : hip_fail(err, "gsd_commit_kv launch");
}

int gsd_softmax_stats(int64_t rows, int32_t vocab, int dtype, const void *logits, int64_t row_stride, float *row_max,
                      float *row_sumexp, void *hip_stream) {
    if (rows < 1 || rows > INT32_MAX || vocab < 1) return fail(GSD_ERR_INVALID_ARG, "rows and vocab must be >= 1");
    if (dtype != GSD_F32 && dtype != GSD_BF16) return fail(GSD_ERR_UNSUPPORTED, "dtype %d", dtype);
    if (!logits || !row_max || !row_sumexp) return fail(GSD_ERR_INVALID_ARG, "NULL pointer argument");
    if (row_stride < vocab) return fail(GSD_ERR_INVALID_ARG, "row_stride %lld < vocab %d", (long long)row_stride, vocab);
    const uintptr_t elt = dtype == GSD_BF16 ? 2 : 4;
    if (reinterpret_cast<uintptr_t>(logits) % elt != 0) return fail(GSD_ERR_INVALID_ARG, "logits misaligned");
    hipError_t err = gsd::launch_softmax_stats(rows, vocab, dtype, logits, row_stride, row_max, row_sumexp,
                                               (hipStream_t)hip_stream);
    return err == hipSuccess ? GSD_OK : hip_fail(err, "gsd_softmax_stats launch");
}

int gsd_accept_stochastic(const gsd_stochastic_desc *desc, void *hip_stream) {
    if (!desc) return fail(GSD_ERR_INVALID_ARG, "descriptor is NULL");
    const gsd_stochastic_desc &d = *desc;
    if (d.batch < 1 || d.total_nodes < 1 || d.max_nodes < 1 || d.vocab < 1)
        return fail(GSD_ERR_INVALID_ARG, "batch, total_nodes, max_nodes and vocab must be >= 1");
    if (d.max_nodes > GSD_MAX_NODES_PER_SEQ)
        return fail(GSD_ERR_UNSUPPORTED, "max_nodes %d exceeds %d", d.max_nodes, GSD_MAX_NODES_PER_SEQ);
    if (d.dtype != GSD_F32 && d.dtype != GSD_BF16) return fail(GSD_ERR_UNSUPPORTED, "dtype %d", d.dtype);
    if (d.row_stride < d.vocab)
        return fail(GSD_ERR_INVALID_ARG, "row_stride %lld < vocab %d", (long long)d.row_stride, d.vocab);
    if (!d.node_offsets || !d.parent_offsets || !d.parent_idx || !d.tokens || !d.logits || !d.root_logits ||
        !d.draft_logits || !d.root_draft_logits || !d.draft_prob || !d.accept_u || !d.resample_u || !d.row_max ||
        !d.row_sumexp || !d.accept_len || !d.accept_path || !d.end_node || !d.bonus_token)
        return fail(GSD_ERR_INVALID_ARG, "NULL pointer argument");
    const uintptr_t elt = d.dtype == GSD_BF16 ? 2 : 4;
    const void *rows4[4] = {d.logits, d.root_logits, d.draft_logits, d.root_draft_logits};
    for (const void *ptr : rows4)
        if (reinterpret_cast<uintptr_t>(ptr) % elt != 0) return fail(GSD_ERR_INVALID_ARG, "logits misaligned");
    hipError_t err = gsd::launch_accept_stochastic(d, (hipStream_t)hip_stream);
    return err == hipSuccess ? GSD_OK : hip_fail(err, "gsd_accept_stochastic launch");
}

int gsd_build_token_graph(int32_t batch, int32_t max_nodes, int32_t tau, float theta_prob, float theta_sib,
                          const int32_t *node_offsets, const int32_t *tree_parent, const int32_t *tokens,
                          const float *draft_prob, int32_t *counts, int32_t *graph_node_offsets, int32_t *parent_offsets,
                          int32_t *parent_idx, int64_t edge_capacity, int32_t *origin, int32_t *flags,
                          int32_t *error_flag, void *hip_stream) {
    if (batch < 1 || max_nodes < 1 || tau < 1) return fail(GSD_ERR_INVALID_ARG, "batch, max_nodes and tau must be >= 1");
    if (max_nodes > GSD_MAX_NODES_PER_SEQ)
        return fail(GSD_ERR_UNSUPPORTED, "max_nodes %d exceeds %d", max_nodes, GSD_MAX_NODES_PER_SEQ);
    if (!(theta_prob >= 0.f) || !(theta_sib >= 0.f)) return fail(GSD_ERR_INVALID_ARG, "thresholds must be >= 0");
    if (edge_capacity < 1) return fail(GSD_ERR_INVALID_ARG, "edge_capacity must be >= 1");
    if (!node_offsets || !tree_parent || !tokens || !draft_prob || !counts || !graph_node_offsets || !parent_offsets ||
        !parent_idx || !origin || !flags)
        return fail(GSD_ERR_INVALID_ARG, "NULL pointer argument");
    hipError_t err = gsd::launch_build_graph(batch, max_nodes, node_offsets, tree_parent, tokens, draft_prob, tau,
                                             theta_prob, theta_sib, counts, graph_node_offsets, parent_offsets,
                                             parent_idx, edge_capacity, origin, flags, error_flag,
                                             (hipStream_t)hip_stream);
    return err == hipSuccess ? GSD_OK : hip_fail(err, "gsd_build_token_graph launch");
}

}  // extern "C"
