// Output reduction of partition-n-reduce (arXiv 1807.08887 Sec. 3.1, second way; Sec. 6):
// dst[i] = partials[0][i] + ... + partials[k-1][i], summed left to right in fp32 registers.
//
// Pure streaming: k reads and one write per element, no reuse, so the kernel is bound by HBM
// bandwidth.  Each lane owns 16-byte vectors, issues all k loads of a vector before the first
// add (k independent requests in flight per lane), and never uses atomics, so the result does
// not depend on the launch shape and is identical from run to run.
#include <hip/hip_runtime.h>

#include "tofu_internal.h"

namespace tofu {

constexpr int kMaxReduceK = 16;
typedef float v4f __attribute__((ext_vector_type(4)));

struct ReducePtrs {
  const float* p[kMaxReduceK];
};

constexpr int kReduceThreads = 512;
constexpr int kReduceMaxBlocks = 16384;
// Inputs are read with the streaming (nontemporal) hint: measured cold (inside the whole-step
// benchmark) it is the faster choice for both the 151 MB and the 531 MB reduction.
template <bool NT>
__device__ __forceinline__ v4f ld_vec(const v4f* p) {
  return NT ? __builtin_nontemporal_load(p) : *p;
}

template <int K, int UNROLL, bool NT>
__global__ void __launch_bounds__(kReduceThreads) reduce_kernel(float* __restrict__ dst, ReducePtrs src, int64_t n_vec, int64_t count) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  // main part: UNROLL vectors per trip, all loads first
  for (; i + (UNROLL - 1) * stride < n_vec; i += UNROLL * stride) {
    v4f v[UNROLL][K];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u)
#pragma unroll
      for (int j = 0; j < K; ++j) v[u][j] = ld_vec<NT>(reinterpret_cast<const v4f*>(src.p[j]) + i + u * stride);
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      v4f acc = v[u][0];
#pragma unroll
      for (int j = 1; j < K; ++j) acc += v[u][j];
      __builtin_nontemporal_store(acc, reinterpret_cast<v4f*>(dst) + i + u * stride);
    }
  }
  for (; i < n_vec; i += stride) {
    v4f acc = ld_vec<NT>(reinterpret_cast<const v4f*>(src.p[0]) + i);
#pragma unroll
    for (int j = 1; j < K; ++j) acc += ld_vec<NT>(reinterpret_cast<const v4f*>(src.p[j]) + i);
    __builtin_nontemporal_store(acc, reinterpret_cast<v4f*>(dst) + i);
  }
  // scalar tail (count not a multiple of 4, or the whole array when pointers are not 16-byte aligned)
  for (int64_t e = n_vec * 4 + (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < count; e += stride) {
    float acc = src.p[0][e];
#pragma unroll
    for (int j = 1; j < K; ++j) acc += src.p[j][e];
    dst[e] = acc;
  }
}

template <int K>
static void launch_k(float* dst, const ReducePtrs& src, int64_t n_vec, int64_t count, int blocks, bool nt, hipStream_t s) {
  constexpr int U = K <= 4 ? 4 : K <= 8 ? 2 : 1;
  if (nt) hipLaunchKernelGGL((reduce_kernel<K, U, true>), dim3(blocks), dim3(kReduceThreads), 0, s, dst, src, n_vec, count);
  else hipLaunchKernelGGL((reduce_kernel<K, U, false>), dim3(blocks), dim3(kReduceThreads), 0, s, dst, src, n_vec, count);
}

int launch_reduce(float* dst, const float* const* parts, int k, int64_t count, void* stream) {
  if (count == 0) return TOFU_OK;
  ReducePtrs src;
  bool aligned = (reinterpret_cast<uintptr_t>(dst) & 15) == 0;
  for (int j = 0; j < kMaxReduceK; ++j) {
    src.p[j] = parts[j < k ? j : 0];
    aligned = aligned && (reinterpret_cast<uintptr_t>(src.p[j]) & 15) == 0;
  }
  const int64_t n_vec = aligned ? count / 4 : 0;
  // Enough resident lanes to cover HBM latency, few enough that every lane streams several vectors.
  int64_t work = n_vec > 0 ? n_vec : count;
  int64_t want = (work + kReduceThreads - 1) / kReduceThreads;
  int blocks = (int)(want < kReduceMaxBlocks ? (want < 1 ? 1 : want) : kReduceMaxBlocks);
  const bool nt = true;
  hipStream_t s = static_cast<hipStream_t>(stream);
  switch (k) {
#define TOFU_CASE(K) case K: launch_k<K>(dst, src, n_vec, count, blocks, nt, s); break;
    TOFU_CASE(1) TOFU_CASE(2) TOFU_CASE(3) TOFU_CASE(4) TOFU_CASE(5) TOFU_CASE(6) TOFU_CASE(7) TOFU_CASE(8)
    TOFU_CASE(9) TOFU_CASE(10) TOFU_CASE(11) TOFU_CASE(12) TOFU_CASE(13) TOFU_CASE(14) TOFU_CASE(15) TOFU_CASE(16)
#undef TOFU_CASE
    default: return fail(TOFU_ERR_INVALID_ARG, "k = %d outside [1,%d]", k, kMaxReduceK);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(TOFU_ERR_HIP, "reduce launch failed: %s", hipGetErrorString(e));
  return TOFU_OK;
}

}  // namespace tofu

extern "C" int tofu_partition_reduce(void* dst, const void* const* partials, int32_t k, int64_t count, void* hip_stream) {
  using namespace tofu;
  if (k < 1 || k > kMaxReduceK) return fail(TOFU_ERR_INVALID_ARG, "k = %d outside [1,%d]", (int)k, kMaxReduceK);
  if (count < 0) return fail(TOFU_ERR_INVALID_ARG, "count = %lld is negative", (long long)count);
  if (count == 0) return TOFU_OK;
  if (!dst || !partials) return fail(TOFU_ERR_INVALID_ARG, "dst or partials is NULL");
  const char* d0 = static_cast<const char*>(dst);
  const int64_t bytes = count * (int64_t)sizeof(float);
  for (int j = 0; j < k; ++j) {
    if (!partials[j]) return fail(TOFU_ERR_INVALID_ARG, "partials[%d] is NULL", j);
    const char* pj = static_cast<const char*>(partials[j]);
    // dst may be exactly partials[0]; any other overlap with an input would race
    bool same = pj == d0;
    bool overlap = pj < d0 + bytes && d0 < pj + bytes;
    if (overlap && !(same && j == 0))
      return fail(TOFU_ERR_INVALID_ARG, "dst overlaps partials[%d]; only dst == partials[0] is allowed", j);
  }
  return launch_reduce(static_cast<float*>(dst), reinterpret_cast<const float* const*>(partials), k, count, hip_stream);
}
