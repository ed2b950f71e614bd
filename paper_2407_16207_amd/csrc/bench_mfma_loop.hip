// libgsd_bench.so: a measurement aid of bench.py, not part of the verification path and not part of libgsd.so.
// A bare loop of the attention kernel's matrix instruction (v_mfma_f32_32x32x16_bf16, fp32 accumulate), two
// wavefronts per SIMD, nothing else in the loop, operands taken from a caller buffer so that their statistics (zeros,
// normal deviates, ...) are the caller's choice: the clock the matrix pipe sustains depends on how much the operand
// bits toggle, and the benchmark reports that rate next to the attention kernel's.
//
//   int gsd_bench_mfma_loop(const void *operands, int64_t operand_bytes, int32_t work_groups, int32_t iters,
//                           float *sink, void *hip_stream);
// `work_groups` work-groups of 512 lanes; every lane first loads sixteen 16-byte operand fragments (eight A, eight B)
// from `operands`, fragment f of lane t at byte 16 * ((16*t + f) mod (operand_bytes/16)), then issues iters * 16
// matrix instructions that rotate through them, and finally stores the sum of its accumulators to sink[t] (so that
// the loop is not removed).  flops per launch = work_groups * 8 * iters * 16 * 32768.  operands: device, 16-byte
// aligned, operand_bytes a positive multiple of 16; sink: device, [work_groups*512] fp32; work_groups in [1, 65536],
// iters in [1, 1<<20].  Returns 0, 1 for an argument out of range, 2 for a launch failure.  No synchronisation.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {
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

}  // namespace

extern "C" int gsd_bench_mfma_loop(const void *operands, int64_t operand_bytes, int32_t work_groups, int32_t iters,
                                   float *sink, void *hip_stream) {
    if (!operands || !sink || operand_bytes < 16 || operand_bytes % 16 != 0 || operand_bytes / 16 > INT64_C(0xffffffff) ||
        reinterpret_cast<uintptr_t>(operands) % 16 != 0 || work_groups < 1 || work_groups > 65536 || iters < 1 ||
        iters > (1 << 20))
        return 1;
    hipLaunchKernelGGL(diag_mfma_loop_kernel, dim3(work_groups), dim3(512), 0, (hipStream_t)hip_stream,
                       reinterpret_cast<const diag_bf16x8 *>(operands), uint32_t(operand_bytes / 16), iters, sink);
    return hipGetLastError() == hipSuccess ? 0 : 2;
}
