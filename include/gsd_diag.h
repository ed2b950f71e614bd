/*
 * Measurement aids of libgsd.so.  Nothing here is a step of the verification path: these calls exist so that
 * the benchmark can report, next to the attention kernel's rate, what the matrix pipe of the chip it runs on
 * sustains for the same operand statistics (the sustained clock of the matrix pipe depends on how much the
 * operand bits toggle, so the rate of one and the same instruction stream differs between zero and random inputs).
 * Same conventions as gsd.h: device pointers owned by the caller, work enqueued on `hip_stream`, no
 * synchronisation, GSD_OK or a GSD_ERR_* code with gsd_last_error() holding the detail.
 */
#ifndef GSD_DIAG_H
#define GSD_DIAG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * A bare loop of the attention kernel's matrix instruction (v_mfma_f32_32x32x16_bf16, fp32 accumulate), two
 * wavefronts per SIMD, nothing else in the loop.  `work_groups` work-groups of 512 lanes; every lane first loads
 * sixteen 16-byte operand fragments (eight A, eight B) from `operands`, fragment f of lane t at byte
 * 16 * ((16*t + f) mod (operand_bytes/16)), then issues iters * 16 matrix instructions that rotate through them,
 * and finally stores the sum of its accumulators to sink[t] (so that the loop is not removed).
 *   flops per launch = work_groups * 8 * iters * 16 * 32768
 *   operands: device, operand_bytes >= 16 and a multiple of 16, 16-byte aligned; sink: device, [work_groups*512] fp32.
 *   work_groups in [1, 65536], iters in [1, 1<<20].
 */
int gsd_diag_mfma_loop(const void *operands, int64_t operand_bytes, int32_t work_groups, int32_t iters, float *sink,
                       void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif
