// Output reduction of partition-n-reduce (arXiv 1807.08887 Sec. 3.1, second way; Sec. 6):
// dst[i] = partials[0][i] + ... + partials[k-1][i], summed left to right in fp32 registers.
// The extended entry point also offers the other built-in reducers of the operator description
// language (Sec. 4.1: Max, Min, Prod) and a pairwise order that follows the recursion's binary
// tree of workers (Sec. 5.2): fold(l, r) = fold(l, m) (+) fold(m, r), m = l + ceil((r - l) / 2).
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

// MODE: 0 sum left to right, 1 sum pairwise, 2 product left to right, 3 product pairwise, 4 max, 5 min
template <int MODE, typename T>
__device__ __forceinline__ T combine(T a, T b) {
  if constexpr (MODE <= 1) return a + b;
  else if constexpr (MODE <= 3) return a * b;
  else if constexpr (MODE == 4) return __builtin_elementwise_max(a, b);   // fmax semantics: a NaN operand is dropped
  else return __builtin_elementwise_min(a, b);
}
template <int MODE, int L, int R, typename T>
__device__ __forceinline__ T fold_tree(const T* v) {
  if constexpr (R - L == 1) return v[L];
  else {
    constexpr int M = L + (R - L + 1) / 2;
    return combine<MODE>(fold_tree<MODE, L, M>(v), fold_tree<MODE, M, R>(v));
  }
}
template <int MODE, int K, typename T>
__device__ __forceinline__ T fold(const T* v) {
  if constexpr (MODE == 1 || MODE == 3) return fold_tree<MODE, 0, K>(v);
  else {
    T acc = v[0];
#pragma unroll
    for (int j = 1; j < K; ++j) acc = combine<MODE>(acc, v[j]);
    return acc;
  }
}

template <int K, int UNROLL, bool NT, int MODE>
__global__ void __launch_bounds__(kReduceThreads) reduce_kernel(float* __restrict__ dst_all, ReducePtrs src_all, int64_t n_vec, int64_t count, int head) {
  // elements [head, head + 4 * n_vec) are whole aligned vectors; the `head` elements before them and the rest after are scalar work
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  float* dst = dst_all + head;
  ReducePtrs src;
#pragma unroll
  for (int j = 0; j < K; ++j) src.p[j] = src_all.p[j] + head;
  // main part: UNROLL vectors per trip, all loads first
  for (; i + (UNROLL - 1) * stride < n_vec; i += UNROLL * stride) {
    v4f v[UNROLL][K];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u)
#pragma unroll
      for (int j = 0; j < K; ++j) v[u][j] = ld_vec<NT>(reinterpret_cast<const v4f*>(src.p[j]) + i + u * stride);
#pragma unroll
    for (int u = 0; u < UNROLL; ++u)
      __builtin_nontemporal_store(fold<MODE, K>(v[u]), reinterpret_cast<v4f*>(dst) + i + u * stride);
  }
  for (; i < n_vec; i += stride) {
    v4f v[K];
#pragma unroll
    for (int j = 0; j < K; ++j) v[j] = ld_vec<NT>(reinterpret_cast<const v4f*>(src.p[j]) + i);
    __builtin_nontemporal_store(fold<MODE, K>(v), reinterpret_cast<v4f*>(dst) + i);
  }
  // scalar work: the head, the tail, or the whole array when the pointers do not share one 16-byte phase
  const int64_t left = count - n_vec * 4;
  for (int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; r < left; r += stride) {
    const int64_t e = r < head ? r : r + n_vec * 4;
    float v[K];
#pragma unroll
    for (int j = 0; j < K; ++j) v[j] = src_all.p[j][e];
    dst_all[e] = fold<MODE, K>(v);
  }
}

template <int K, int MODE>
static void launch_k(float* dst, const ReducePtrs& src, int64_t n_vec, int64_t count, int head, int blocks, hipStream_t s) {
  constexpr int U = K <= 4 ? 4 : K <= 8 ? 2 : 1;
  hipLaunchKernelGGL((reduce_kernel<K, U, true, MODE>), dim3(blocks), dim3(kReduceThreads), 0, s, dst, src, n_vec, count, head);
}

template <int MODE>
static bool launch_mode(int k, float* dst, const ReducePtrs& src, int64_t n_vec, int64_t count, int head, int blocks, hipStream_t s) {
  switch (k) {
#define TOFU_CASE(K) case K: launch_k<K, MODE>(dst, src, n_vec, count, head, blocks, s); return true;
    TOFU_CASE(1) TOFU_CASE(2) TOFU_CASE(3) TOFU_CASE(4) TOFU_CASE(5) TOFU_CASE(6) TOFU_CASE(7) TOFU_CASE(8)
    TOFU_CASE(9) TOFU_CASE(10) TOFU_CASE(11) TOFU_CASE(12) TOFU_CASE(13) TOFU_CASE(14) TOFU_CASE(15) TOFU_CASE(16)
#undef TOFU_CASE
    default: return false;
  }
}

int launch_reduce(float* dst, const float* const* parts, int k, int64_t count, void* stream) {
  return launch_reduce_mode(dst, parts, k, count, 0, stream);
}

int launch_reduce_mode(float* dst, const float* const* parts, int k, int64_t count, int mode, void* stream) {
  if (count == 0) return TOFU_OK;
  ReducePtrs src;
  // vector path: every pointer has the same offset into a 16-byte line (a whole number of floats);
  // the elements up to the next line start are done one by one
  const uintptr_t phase = reinterpret_cast<uintptr_t>(dst) & 15;
  bool aligned = phase % 4 == 0;
  for (int j = 0; j < kMaxReduceK; ++j) {
    src.p[j] = parts[j < k ? j : 0];
    aligned = aligned && (reinterpret_cast<uintptr_t>(src.p[j]) & 15) == phase;
  }
  int head = aligned ? (int)((16 - phase) % 16 / 4) : 0;
  if (head > count) head = (int)count;
  const int64_t n_vec = aligned ? (count - head) / 4 : 0;
  // Enough resident lanes to cover HBM latency, few enough that every lane streams several vectors.
  int64_t work = n_vec > 0 ? n_vec : count;
  int64_t want = (work + kReduceThreads - 1) / kReduceThreads;
  int blocks = (int)(want < kReduceMaxBlocks ? (want < 1 ? 1 : want) : kReduceMaxBlocks);
  hipStream_t s = static_cast<hipStream_t>(stream);
  bool ok = false;
  switch (mode) {
    case 0: ok = launch_mode<0>(k, dst, src, n_vec, count, head, blocks, s); break;
    case 1: ok = launch_mode<1>(k, dst, src, n_vec, count, head, blocks, s); break;
    case 2: ok = launch_mode<2>(k, dst, src, n_vec, count, head, blocks, s); break;
    case 3: ok = launch_mode<3>(k, dst, src, n_vec, count, head, blocks, s); break;
    case 4: ok = launch_mode<4>(k, dst, src, n_vec, count, head, blocks, s); break;
    case 5: ok = launch_mode<5>(k, dst, src, n_vec, count, head, blocks, s); break;
    default: break;
  }
  if (!ok) return fail(TOFU_ERR_INVALID_ARG, "k = %d outside [1,%d] or unknown reduction mode %d", k, kMaxReduceK, mode);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(TOFU_ERR_HIP, "reduce launch failed: %s", hipGetErrorString(e));
  return TOFU_OK;
}

}  // namespace tofu

namespace tofu {
static int check_reduce_args(void* dst, const void* const* partials, int32_t k, int64_t count) {
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
  return TOFU_OK;
}
}  // namespace tofu

extern "C" int tofu_partition_reduce(void* dst, const void* const* partials, int32_t k, int64_t count, void* hip_stream) {
  using namespace tofu;
  int rc = check_reduce_args(dst, partials, k, count);
  if (rc || count == 0) return rc;
  return launch_reduce(static_cast<float*>(dst), reinterpret_cast<const float* const*>(partials), k, count, hip_stream);
}

extern "C" int tofu_partition_reduce_ex(void* dst, const void* const* partials, int32_t k, int64_t count, int32_t reducer,
                                        int32_t order, void* hip_stream) {
  using namespace tofu;
  if (reducer < TOFU_REDUCE_SUM || reducer > TOFU_REDUCE_PROD) return fail(TOFU_ERR_INVALID_ARG, "unknown reducer %d", (int)reducer);
  if (order != TOFU_ORDER_LINEAR && order != TOFU_ORDER_TREE) return fail(TOFU_ERR_INVALID_ARG, "unknown reduction order %d", (int)order);
  int rc = check_reduce_args(dst, partials, k, count);
  if (rc || count == 0) return rc;
  const bool tree = order == TOFU_ORDER_TREE;
  const int mode = reducer == TOFU_REDUCE_SUM ? (tree ? 1 : 0) : reducer == TOFU_REDUCE_PROD ? (tree ? 3 : 2) : reducer == TOFU_REDUCE_MAX ? 4 : 5;
  return launch_reduce_mode(static_cast<float*>(dst), reinterpret_cast<const float* const*>(partials), k, count, mode, hip_stream);
}

extern "C" int tofu_partition_reduce_scatter(void* dst, const void* const* partials, int32_t k, int64_t count, int32_t shares,
                                             int32_t share, int32_t reducer, int32_t order, void* hip_stream) {
  using namespace tofu;
  if (reducer < TOFU_REDUCE_SUM || reducer > TOFU_REDUCE_PROD) return fail(TOFU_ERR_INVALID_ARG, "unknown reducer %d", (int)reducer);
  if (order != TOFU_ORDER_LINEAR && order != TOFU_ORDER_TREE) return fail(TOFU_ERR_INVALID_ARG, "unknown reduction order %d", (int)order);
  int rc = check_reduce_args(dst, partials, k, count);
  if (rc) return rc;
  if (shares < 1 || share < 0 || share >= shares) return fail(TOFU_ERR_INVALID_ARG, "share %d of %d is not a valid share", (int)share, (int)shares);
  // balanced cut of the flat index range, the same rule as for tensor dimensions; shares may be empty when count < shares
  const int64_t lo = (int64_t)((__int128)share * count / shares), hi = (int64_t)((__int128)(share + 1) * count / shares);
  if (hi == lo) return TOFU_OK;
  const float* parts[kMaxReduceK];
  for (int j = 0; j < k; ++j) parts[j] = static_cast<const float*>(partials[j]) + lo;
  const bool tree = order == TOFU_ORDER_TREE;
  const int mode = reducer == TOFU_REDUCE_SUM ? (tree ? 1 : 0) : reducer == TOFU_REDUCE_PROD ? (tree ? 3 : 2) : reducer == TOFU_REDUCE_MAX ? 4 : 5;
  return launch_reduce_mode(static_cast<float*>(dst) + lo, parts, k, hi - lo, mode, hip_stream);
}
