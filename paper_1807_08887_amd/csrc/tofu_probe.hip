// Device probes of attainable peaks (tofu_probe.h): a register-only fp32 MFMA loop and a plain
// 16-byte-vector streaming copy.  Measurement aids; no part of the method runs through them.
#include <hip/hip_runtime.h>

#include "tofu_internal.h"
#include "tofu_mfma.h"
#include "tofu_probe.h"

namespace tofu {

__global__ void __launch_bounds__(256) probe_mfma_kernel(float* sink, int iters) {
  constexpr int NACC = 8;
  acc16 acc[NACC];
#pragma unroll
  for (int i = 0; i < NACC; ++i) acc[i] = acc_zero();
  const float a = threadIdx.x * 1e-3f, b = 1.0f / (1 + threadIdx.x);
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < NACC; ++i) acc[i] = mfma_32x32x2(a, b, acc[i]);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < NACC; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) s += acc[i][v];
  if (s == -12345.678f) sink[0] = s;   // never true for these operands; keeps the loop from being removed
}

__global__ void __launch_bounds__(256) probe_copy_kernel(v4f32* __restrict__ dst, const v4f32* __restrict__ src, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) dst[i] = src[i];
}

}  // namespace tofu

extern "C" int tofu_probe_mfma(void* sink, int32_t iters, int32_t workgroups, void* hip_stream) {
  using namespace tofu;
  if (!sink || iters < 1 || workgroups < 1) return fail(TOFU_ERR_INVALID_ARG, "mfma probe needs a sink, iters >= 1 and workgroups >= 1");
  hipLaunchKernelGGL(probe_mfma_kernel, dim3(workgroups), dim3(256), 0, static_cast<hipStream_t>(hip_stream), static_cast<float*>(sink), iters);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(TOFU_ERR_HIP, "mfma probe launch failed: %s", hipGetErrorString(e));
  return TOFU_OK;
}

extern "C" int tofu_probe_copy(void* dst, const void* src, size_t bytes, void* hip_stream) {
  using namespace tofu;
  if (!dst || !src) return fail(TOFU_ERR_INVALID_ARG, "copy probe needs two device pointers");
  if (bytes % 16 || (reinterpret_cast<uintptr_t>(dst) | reinterpret_cast<uintptr_t>(src)) % 16)
    return fail(TOFU_ERR_INVALID_ARG, "copy probe needs 16-byte aligned pointers and a multiple of 16 bytes");
  if (bytes == 0) return TOFU_OK;
  const size_t n = bytes / 16;
  const size_t blocks = (n + 255) / 256 < 16384 ? (n + 255) / 256 : 16384;
  hipLaunchKernelGGL(probe_copy_kernel, dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                     static_cast<v4f32*>(dst), static_cast<const v4f32*>(src), n);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(TOFU_ERR_HIP, "copy probe launch failed: %s", hipGetErrorString(e));
  return TOFU_OK;
}
