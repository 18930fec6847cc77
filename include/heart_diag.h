/*
 * heart_diag.h -- diagnostics of libheart for roofline accounting.  Not part of the method
 * and not needed by a caller of the hot path (include/heart.h); used by the benchmark.
 * Conventions (device pointers, stream, return codes, heart_last_error) as in heart.h.
 */
#ifndef HEART_DIAG_H_
#define HEART_DIAG_H_

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * heart_ubench_mfma_bf16: n_workgroups workgroups of 4 wavefronts each issue 16 * iters
 *   v_mfma_f32_32x32x16_bf16 on register operands taken from a_bf16 / b_bf16 (device,
 *   8192 bf16 each, 16-byte aligned); FLOPs = n_workgroups * 4 * iters * 16 * 32768.
 *   The sustained clock of the chip depends on the operand bits, so timing this call
 *   with zeros and with data like a kernel's own gives the nominal and the attainable
 *   matrix-core rate.  sink: one float (device), practically never written.
 * heart_ubench_copy: plain device-to-device copy of `bytes` (multiple of 16); moves
 *   2 * bytes through HBM.  Reference for scaling hardware traffic counters.
 * heart_ubench_read: streams `bytes` (multiple of 16) from src with the access pattern of the
 *   pooling kernel (one workgroup per 32 KB, every load of a workgroup in flight at once,
 *   non-temporal) and reduces them to nothing; moves `bytes` through HBM.  What a read-only
 *   streaming kernel sustains on this chip.  sink: one 32-bit word (device), practically
 *   never written.
 */
int heart_ubench_mfma_bf16(const void *a_bf16, const void *b_bf16, int n_workgroups, int iters,
                           float *sink, void *stream);
int heart_ubench_copy(const void *src, void *dst, size_t bytes, void *stream);
int heart_ubench_read(const void *src, size_t bytes, unsigned *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* HEART_DIAG_H_ */
