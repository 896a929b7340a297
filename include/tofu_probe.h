/*
 * tofu_probe.h -- trivial device probes that measure what the machine attains, so that
 * a kernel's fraction of the published peak can also be read against an achievable one.
 * They are measurement aids exported by the same library; they take no part in the method.
 *
 * Each only enqueues one kernel on `hip_stream` (a hipStream_t passed as void*, NULL = the null
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

/*
 * Read-only stream: reads `bytes` bytes from DEVICE `src` with nontemporal 16-byte loads (16 in
 * flight per lane) and writes nothing.  HBM traffic = bytes.
 *   sink : DEVICE pointer to at least one float; written only if a lane's sum takes one
 *          particular value (keeps the loads alive).
 * Errors: TOFU_ERR_INVALID_ARG for null pointers, bytes not a multiple of 16, src not 16-byte
 * aligned.  bytes == 0 is a no-op.
 */
int tofu_probe_read(const void* src, size_t bytes, void* sink, void* hip_stream);

/*
 * k:1 read:write stream, the traffic mix of a k-way output reduction: dst[i] = srcs[0][i] + ... +
 * srcs[k-1][i] over `bytes` bytes per array, nontemporal 16-byte loads and stores, nothing else
 * (no reducers, no unaligned head or tail).  `srcs` is a HOST array of k DEVICE pointers, k in
 * {1, 2, 4, 8}; with k = 1 this is a nontemporal copy.  HBM traffic = (k + 1) * bytes.  dst must
 * not overlap any source.
 * Errors: TOFU_ERR_INVALID_ARG for null or misaligned pointers, another k, bytes not a multiple
 * of 16.  bytes == 0 is a no-op.
 */
int tofu_probe_stream(void* dst, const void* const* srcs, int32_t k, size_t bytes, void* hip_stream);

#ifdef __cplusplus
}
#endif

#endif /* TOFU_PROBE_H_ */
