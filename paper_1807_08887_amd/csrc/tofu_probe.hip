// Device probes of attainable peaks (tofu_probe.h): a register-only fp32 MFMA loop, a plain
// 16-byte-vector streaming copy, a read-only stream and a k:1 read:write stream.  Measurement
// aids; no part of the method runs through them.
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

// Read-only stream: one wavefront per workgroup, 16 nontemporal 16-byte loads in flight per lane.
__global__ void __launch_bounds__(64) probe_read_kernel(const v4f32* __restrict__ src, size_t n, float* sink) {
  constexpr int VPL = 16;
  const size_t base = (size_t)blockIdx.x * 64 * VPL;
  v4f32 acc = {0.f, 0.f, 0.f, 0.f};
  if (base + 64 * VPL <= n) {
    v4f32 v[VPL];
#pragma unroll
    for (int u = 0; u < VPL; ++u) v[u] = __builtin_nontemporal_load(src + base + u * 64 + threadIdx.x);
#pragma unroll
    for (int u = 0; u < VPL; ++u) acc += v[u];
  } else {
    for (size_t i = base + threadIdx.x; i < n; i += 64) acc += __builtin_nontemporal_load(src + i);
  }
  if (acc[0] + acc[1] + acc[2] + acc[3] == -12345.678f) sink[0] = acc[0];   // keeps the loads alive; practically never true
}

// k reads and one write per vector (the traffic mix of a k-way output reduction): one wavefront
// per workgroup, a contiguous chunk of 64 * 8 vectors read source by source (nontemporal).
struct ProbePtrs {
  const v4f32* p[8];
};
template <int K>
__global__ void __launch_bounds__(64) probe_stream_kernel(v4f32* __restrict__ dst, ProbePtrs src, size_t n) {
  constexpr int VPL = 8;
  const size_t base = (size_t)blockIdx.x * 64 * VPL;
  if (base + 64 * VPL <= n) {            // source by source: an 8 KB run of each
    v4f32 acc[VPL];
#pragma unroll
    for (int u = 0; u < VPL; ++u) acc[u] = __builtin_nontemporal_load(src.p[0] + base + u * 64 + threadIdx.x);
#pragma unroll
    for (int j = 1; j < K; ++j) {
      v4f32 t[VPL];
#pragma unroll
      for (int u = 0; u < VPL; ++u) t[u] = __builtin_nontemporal_load(src.p[j] + base + u * 64 + threadIdx.x);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int u = 0; u < VPL; ++u) acc[u] += t[u];
    }
#pragma unroll
    for (int u = 0; u < VPL; ++u) __builtin_nontemporal_store(acc[u], dst + base + u * 64 + threadIdx.x);
  } else {
    for (size_t i = base + threadIdx.x; i < n; i += 64) {
      v4f32 a = __builtin_nontemporal_load(src.p[0] + i);
#pragma unroll
      for (int j = 1; j < K; ++j) a += __builtin_nontemporal_load(src.p[j] + i);
      __builtin_nontemporal_store(a, dst + i);
    }
  }
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

extern "C" int tofu_probe_read(const void* src, size_t bytes, void* sink, void* hip_stream) {
  using namespace tofu;
  if (!src || !sink) return fail(TOFU_ERR_INVALID_ARG, "read probe needs a source and a sink");
  if (bytes % 16 || reinterpret_cast<uintptr_t>(src) % 16) return fail(TOFU_ERR_INVALID_ARG, "read probe needs a 16-byte aligned pointer and a multiple of 16 bytes");
  if (bytes == 0) return TOFU_OK;
  const size_t n = bytes / 16, blocks = (n + 1023) / 1024;
  if (blocks >= ((size_t)1 << 31)) return fail(TOFU_ERR_INVALID_ARG, "read probe: too many bytes for one launch");
  hipLaunchKernelGGL(probe_read_kernel, dim3((unsigned)blocks), dim3(64), 0, static_cast<hipStream_t>(hip_stream), static_cast<const v4f32*>(src), n,
                     static_cast<float*>(sink));
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(TOFU_ERR_HIP, "read probe launch failed: %s", hipGetErrorString(e));
  return TOFU_OK;
}

extern "C" int tofu_probe_stream(void* dst, const void* const* srcs, int32_t k, size_t bytes, void* hip_stream) {
  using namespace tofu;
  if (!dst || !srcs) return fail(TOFU_ERR_INVALID_ARG, "stream probe needs a destination and a source array");
  if (k != 1 && k != 2 && k != 4 && k != 8) return fail(TOFU_ERR_INVALID_ARG, "stream probe: k = %d is not 1, 2, 4 or 8", (int)k);
  if (bytes % 16 || reinterpret_cast<uintptr_t>(dst) % 16) return fail(TOFU_ERR_INVALID_ARG, "stream probe needs 16-byte aligned pointers and a multiple of 16 bytes");
  ProbePtrs p;
  for (int j = 0; j < 8; ++j) {
    const void* q = srcs[j < k ? j : 0];
    if (!q || reinterpret_cast<uintptr_t>(q) % 16) return fail(TOFU_ERR_INVALID_ARG, "stream probe: srcs[%d] is null or not 16-byte aligned", j < k ? j : 0);
    p.p[j] = static_cast<const v4f32*>(q);
  }
  if (bytes == 0) return TOFU_OK;
  const size_t n = bytes / 16;
  const size_t chunk = (size_t)64 * 8, blocks = (n + chunk - 1) / chunk;
  if (blocks >= ((size_t)1 << 31)) return fail(TOFU_ERR_INVALID_ARG, "stream probe: too many bytes for one launch");
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  v4f32* d = static_cast<v4f32*>(dst);
  switch (k) {
    case 1: hipLaunchKernelGGL(probe_stream_kernel<1>, dim3((unsigned)blocks), dim3(64), 0, s, d, p, n); break;
    case 2: hipLaunchKernelGGL(probe_stream_kernel<2>, dim3((unsigned)blocks), dim3(64), 0, s, d, p, n); break;
    case 4: hipLaunchKernelGGL(probe_stream_kernel<4>, dim3((unsigned)blocks), dim3(64), 0, s, d, p, n); break;
    default: hipLaunchKernelGGL(probe_stream_kernel<8>, dim3((unsigned)blocks), dim3(64), 0, s, d, p, n); break;
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(TOFU_ERR_HIP, "stream probe launch failed: %s", hipGetErrorString(e));
  return TOFU_OK;
}
