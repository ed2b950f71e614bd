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

hipError_t launch_node_argmax(int32_t rows, int32_t vocab, int dtype, const void *logits, int64_t row_stride,
                              int32_t *pred, hipStream_t stream);

hipError_t launch_accept(int32_t batch, int32_t max_nodes, const int32_t *node_offsets,
                         const int32_t *parent_offsets, const int32_t *parent_idx, const int32_t *tokens,
                         const int32_t *pred, const int32_t *root_pred, int32_t *accept_len, int32_t *accept_path,
                         int32_t *bonus_token, hipStream_t stream);

hipError_t launch_attention_f32(const gsd_attn_desc &d, hipStream_t stream);

// bf16 MFMA path.  `splits` >= 1 as chosen by attention_bf16_splits(); partials (if splits > 1) go to workspace.
int attention_bf16_splits(const gsd_attn_desc &d);
size_t attention_bf16_workspace(const gsd_attn_desc &d, int splits);
hipError_t launch_attention_bf16(const gsd_attn_desc &d, int splits, hipStream_t stream);

}  // namespace gsd
