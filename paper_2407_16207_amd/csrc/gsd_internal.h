// Internal declarations shared by the host API and the kernel translation units of libgsd (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gsd.h"

namespace gsd {

// Host-side launchers; every argument has been validated by the API layer.
hipError_t launch_build_mask(int32_t batch, int32_t max_nodes, int32_t words_per_row, const int32_t *node_offsets,
                             const int32_t *parent_offsets, const int32_t *parent_idx, uint64_t *mask,
                             int32_t *dag_error_flag, hipStream_t stream);

// row_max / row_sumexp: both NULL (argmax only) or both given (the same sweep also leaves the softmax normalisers)
hipError_t launch_node_argmax(int32_t rows, int32_t vocab, int dtype, const void *logits, int64_t row_stride,
                              int32_t *pred, float *row_max, float *row_sumexp, hipStream_t stream);

hipError_t launch_accept(int32_t batch, int32_t max_nodes, const int32_t *node_offsets,
                         const int32_t *parent_offsets, const int32_t *parent_idx, const int32_t *tokens,
                         const int32_t *pred, const int32_t *root_pred, int32_t *accept_len, int32_t *accept_path,
                         int32_t *bonus_token, hipStream_t stream);

hipError_t launch_attention_f32(const gsd_attn_desc &d, hipStream_t stream);

// bf16 MFMA path.  `splits` >= 1 as chosen by attention_bf16_splits(); partials (if splits > 1) go to workspace.
int attention_bf16_splits(const gsd_attn_desc &d);
size_t attention_bf16_workspace(const gsd_attn_desc &d, int splits);
hipError_t launch_attention_bf16(const gsd_attn_desc &d, int splits, hipStream_t stream);
// device address, on the current device, of the library's static scratch array of GSD_STATIC_SCRATCH_BYTES
hipError_t attention_static_scratch(void **ptr);

hipError_t launch_unmerge(int32_t batch, int32_t max_nodes, int32_t max_tree_nodes, const int32_t *node_offsets,
                          const int32_t *parent_offsets, const int32_t *parent_idx, int32_t *tree_node_offsets,
                          int32_t *tree_parent, int32_t *tree_parent_offsets, int32_t *tree_origin,
                          int64_t *path_count, int32_t *dag_error_flag, hipStream_t stream);

hipError_t launch_gather_rows(int64_t rows, int64_t row_bytes, const void *src, int64_t src_rows,
                              int64_t src_stride, const int32_t *index, void *dst, int64_t dst_stride,
                              hipStream_t stream);

hipError_t launch_commit_kv(int32_t batch, int32_t max_nodes, int32_t num_layers, int64_t row_bytes, void *k, void *v,
                            int64_t token_stride, int64_t layer_stride, const int64_t *kv_offsets,
                            const int32_t *prefix_lens, const int32_t *accept_len, const int32_t *accept_path,
                            int32_t *new_prefix_lens, hipStream_t stream);

// rows_after further rows are taken from logits_after (same stride); their results follow the first buffer's
hipError_t launch_softmax_stats(int64_t rows, int32_t vocab, int dtype, const void *logits, int64_t row_stride,
                                float *row_max, float *row_sumexp, hipStream_t stream, int64_t rows_after = 0,
                                const void *logits_after = nullptr);
hipError_t launch_accept_stochastic(const gsd_stochastic_desc &d, hipStream_t stream);

hipError_t launch_build_graph(int32_t batch, int32_t max_nodes, const int32_t *node_offsets, const int32_t *tree_parent,
                              const int32_t *tokens, const float *draft_prob, int32_t tau, float theta_prob,
                              float theta_sib, int32_t *counts, int32_t *graph_node_offsets, int32_t *parent_offsets,
                              int32_t *parent_idx, int64_t edge_capacity, int32_t *origin, int32_t *flags,
                              int32_t *error_flag, hipStream_t stream);

}  // namespace gsd
