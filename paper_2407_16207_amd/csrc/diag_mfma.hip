// Measurement aid: a bare loop of the attention kernel's matrix instruction, two wavefronts per SIMD, operands
// taken from a caller buffer so that their statistics (zeros, normal deviates, ...) are the caller's choice.
#include "gsd_internal.h"

namespace gsd {

typedef __bf16 diag_bf16x8 __attribute__((ext_vector_type(8)));
typedef float diag_floatx16 __attribute__((ext_vector_type(16)));

__global__ __launch_bounds__(512) void diag_mfma_loop_kernel(const diag_bf16x8 *__restrict__ operands,
                                                             uint32_t fragments, int32_t iters,
                                                             float *__restrict__ sink) {
    const uint32_t t = blockIdx.x * 512u + threadIdx.x;
    diag_bf16x8 a[8], b[8];
#pragma unroll
    for (uint32_t f = 0; f < 8; ++f) {
        a[f] = operands[(16u * t + f) % fragments];
        b[f] = operands[(16u * t + 8u + f) % fragments];
    }
    diag_floatx16 acc[4];
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[q][j] = 0.f;
    for (int32_t it = 0; it < iters; ++it) {
#pragma unroll
        for (int idx = 0; idx < 16; ++idx)
            acc[idx & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[idx & 7], b[(idx >> 1) & 7], acc[idx & 3], 0, 0, 0);
    }
    float r = 0.f;
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int j = 0; j < 16; ++j) r += acc[q][j];
    sink[t] = r;
}

hipError_t launch_diag_mfma_loop(const void *operands, int64_t operand_bytes, int32_t work_groups, int32_t iters,
                                 float *sink, hipStream_t stream) {
    hipLaunchKernelGGL(diag_mfma_loop_kernel, dim3(work_groups), dim3(512), 0, stream,
                       reinterpret_cast<const diag_bf16x8 *>(operands), uint32_t(operand_bytes / 16), iters, sink);
    return hipGetLastError();
}

}  // namespace gsd
