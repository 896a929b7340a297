/*
 * tofu_probe.h -- two trivial device probes that measure what the machine attains, so that
 * a kernel's fraction of the published peak can also be read against an achievable one.
 * They are measurement aids exported by the same library; they take no part in the method.
 *
 * Both only enqueue one kernel on `hip_stream` (a hipStream_t passed as void*, NULL = the null
 * stream), never allocate or synchronise, and return TOFU_OK or a negative tofu_status_t
 * (tofu.h) with the reason in tofu_last_error().
 */
#ifndef TOFU_PROBE_H_
#define TOFU_PROBE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Pure matrix-pipe loop: `workgroups` workgroups of 4 wavefronts, each wavefront issuing
 * `iters` rounds of 8 independent fp32 32x32x2 MFMAs on registers (no memory traffic).
 * FLOP executed = workgroups * 4 * iters * 8 * 4096.
 *   sink : DEVICE pointer to at least one float; written only if an accumulator sum takes an
 *          impossible value (keeps the loop alive), so its content is otherwise untouched.
 * Errors: TOFU_ERR_INVALID_ARG for a null sink, iters < 1 or workgroups < 1.
 */
int tofu_probe_mfma(void* sink, int32_t iters, int32_t workgroups, void* hip_stream);

/*
 * Plain streaming copy of `bytes` bytes (16-byte vectors, one load and one store per vector)
 * from DEVICE `src` to DEVICE `dst`; the buffers must not overlap.  HBM traffic = 2 * bytes.
 * Errors: TOFU_ERR_INVALID_ARG for null pointers, bytes not a multiple of 16 or pointers not
 * 16-byte aligned.  bytes == 0 is a no-op.
 */
int tofu_probe_copy(void* dst, const void* src, size_t bytes, void* hip_stream);

#ifdef __cplusplus
}
#endif

#endif /* TOFU_PROBE_H_ */
