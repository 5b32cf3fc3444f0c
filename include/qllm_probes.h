/*
 * Measurement probes of libqllm: no part of the method and no part of its boundary.  They exist for callers
 * (the benchmark) that price the two hot kernels against what the machine delivers, next to the data-sheet
 * peaks.  DEVICE pointers; all conventions as in qllm.h.
 */
#ifndef QLLM_PROBES_H
#define QLLM_PROBES_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 *   qllm_probe_mfma    `workgroups` workgroups of 8 waves; every wave issues iters * 32 int8 matrix-core
 *                      operations (16 x 16 x 64 each, i.e. 2 * 16384 integer operations) on register
 *                      operands shaped like 4-bit codes and touches no memory.  sink: one device int32.
 *   qllm_probe_mfma_fp6  the same shape of loop with FP6 (E2M3) matrix-core operations, 16 x 16 x 128 each, on
 *                      operands whose 6-bit fields hold 4-bit codes.  sink: one device float.
 *   qllm_probe_stream  reads `bytes` (a multiple of 16) from src and writes bytes / 4 to dst: the 4 : 1
 *                      read : write mix of the fused kernel with bf16 input and 4-bit codes.
 * Errors: NULL / SHAPE / ALIGN (src 16-byte, dst 4-byte aligned) / HIP.
 */
int32_t qllm_probe_mfma(int32_t workgroups, int32_t iters, int32_t *sink, void *hip_stream);
int32_t qllm_probe_mfma_fp6(int32_t workgroups, int32_t iters, float *sink, void *hip_stream);
int32_t qllm_probe_stream(const void *src, void *dst, int64_t bytes, int32_t workgroups, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* QLLM_PROBES_H */
