/*
 * sdllm_diag.h -- diagnostics of the sdllm library that are NOT part of the decode step: what plain kernels
 * reach on the device, to read the roofline fractions of the hot-path kernels against.  Used by the benchmark.
 */
#ifndef SDLLM_DIAG_H
#define SDLLM_DIAG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ---------------------------------------------------------------------------------------
 * Device ceilings (diagnostics; not part of the decode step): what plain kernels reach on the
 * device, to read the roofline fractions of the hot-path kernels against.
 *   sdllm_probe_read       streams `bytes` (multiple of 16, > 0) of src once; sink: >= 4 bytes of
 *                          device memory that is practically never written
 *   sdllm_probe_copy       dst <- src, `bytes` (multiple of 16, > 0), bit for bit; no overlap
 *   sdllm_probe_mfma_bf16  2 workgroups of 4 waves per CU, each wave `iters` (>= 1) rounds of 8 independent
 *                          v_mfma_f32_16x16x32_bf16; operand_kind 0 = smooth small operand values,
 *                          1 = pseudo-random sign / exponent / mantissa bits (more power per
 *                          instruction, lower sustained clock).  *flops (HOST, optional) receives the
 *                          floating-point operations of one launch.
 * All three only enqueue one kernel on `stream`.  Errors: INVALID_ARG, HIP.
 * ------------------------------------------------------------------------------------- */
int sdllm_probe_read(const void* src, size_t bytes, void* sink, void* stream);
int sdllm_probe_copy(void* dst, const void* src, size_t bytes, void* stream);
int sdllm_probe_mfma_bf16(int32_t iters, int32_t operand_kind, void* sink, void* stream, double* flops);

#ifdef __cplusplus
}
#endif
#endif /* SDLLM_DIAG_H */
