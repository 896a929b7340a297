// Output reduction of partition-n-reduce (arXiv 1807.08887 Sec. 3.1, second way; Sec. 6):
// dst[i] = partials[0][i] + ... + partials[k-1][i], summed left to right in fp32 registers.
// The extended entry point also offers the other built-in reducers of the operator description
// language (Sec. 4.1: Max, Min, Prod) and a pairwise order that follows the recursion's binary
// tree of workers (Sec. 5.2): fold(l, r) = fold(l, m) (+) fold(m, r), m = l + ceil((r - l) / 2).
//
// Pure streaming: k reads and one write per element, no reuse, so the kernel is bound by HBM
// bandwidth, and what decides the rate is the ORDER in which the requests reach the memory: a
// workgroup is one wavefront that owns a contiguous chunk of 64 * VPL 16-byte vectors (8 KB per
// input for VPL = 8) and reads it input by input -- the whole 8 KB run of input 0, then of input
// 1, ... -- folding as it goes.  Reading the same bytes vector by vector across the k inputs
// (1 KB from each in turn) measured 15 - 20 % slower (27.5 against 23.3 us for the 151 MB gate
// reduction, 96 against 84 us for the 531 MB one), and so did a grid-wide stride between a
// lane's vectors.  No atomics: the result does not depend on the launch shape and is identical
// from run to run.
#include <hip/hip_runtime.h>

#include "tofu_internal.h"

namespace tofu {

constexpr int kMaxReduceK = 16;
typedef float v4f __attribute__((ext_vector_type(4)));

struct ReducePtrs {
  const float* p[kMaxReduceK];
};

constexpr int kReduceThreads = 64;       // one wavefront per workgroup
// Inputs and output carry the streaming (nontemporal) hint: measured cold it is the faster
// choice for both the 151 MB and the 531 MB reduction.
__device__ __forceinline__ v4f ld_vec(const v4f* p) { return __builtin_nontemporal_load(p); }

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

// INPLACE: dst is the first input (in-place aggregation); every element is read and then written
// by the same lane, and the pointers carry no __restrict__.  Otherwise dst overlaps no input and
// says so, which lets the stores of finished vectors go out between the loads of later ones.
template <bool INPLACE> struct DstPtr { typedef float* __restrict__ type; };
template <> struct DstPtr<true> { typedef float* type; };

template <int K, int VPL, int MODE, bool INPLACE>
__global__ void __launch_bounds__(kReduceThreads) reduce_kernel(typename DstPtr<INPLACE>::type dst_all, ReducePtrs src_all, int64_t n_vec, int64_t count, int head) {
  // elements [head, head + 4 * n_vec) are whole aligned vectors; the `head` elements before them and the rest after are scalar work
  constexpr int CHUNK = kReduceThreads * VPL;
  constexpr bool PAIRWISE = MODE == 1 || MODE == 3;
  const int64_t base = (int64_t)blockIdx.x * CHUNK;
  if (base + CHUNK <= n_vec) {            // a whole chunk, input by input; the scheduling barriers keep that order
    v4f* d = reinterpret_cast<v4f*>(dst_all + head) + base + threadIdx.x;
    if constexpr (!PAIRWISE) {            // left to right (any order for max / min): fold as the inputs arrive
      v4f acc[VPL];
      {
        const v4f* p = reinterpret_cast<const v4f*>(src_all.p[0] + head) + base + threadIdx.x;
#pragma unroll
        for (int u = 0; u < VPL; ++u) acc[u] = ld_vec(p + u * kReduceThreads);
      }
#pragma unroll
      for (int j = 1; j < K; ++j) {
        const v4f* p = reinterpret_cast<const v4f*>(src_all.p[j] + head) + base + threadIdx.x;
        v4f t[VPL];
#pragma unroll
        for (int u = 0; u < VPL; ++u) t[u] = ld_vec(p + u * kReduceThreads);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < VPL; ++u) acc[u] = combine<MODE>(acc[u], t[u]);
      }
#pragma unroll
      for (int u = 0; u < VPL; ++u) __builtin_nontemporal_store(acc[u], d + u * kReduceThreads);
    } else {                              // pairwise: every input's value is kept until the tree is folded
      v4f v[VPL][K];
#pragma unroll
      for (int j = 0; j < K; ++j) {
        const v4f* p = reinterpret_cast<const v4f*>(src_all.p[j] + head) + base + threadIdx.x;
#pragma unroll
        for (int u = 0; u < VPL; ++u) v[u][j] = ld_vec(p + u * kReduceThreads);
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int u = 0; u < VPL; ++u) __builtin_nontemporal_store(fold<MODE, K>(v[u]), d + u * kReduceThreads);
    }
  } else {                                // the ragged last chunk, one vector at a time
    for (int64_t i = base + threadIdx.x; i < n_vec; i += kReduceThreads) {
      v4f v[K];
#pragma unroll
      for (int j = 0; j < K; ++j) v[j] = ld_vec(reinterpret_cast<const v4f*>(src_all.p[j] + head) + i);
      __builtin_nontemporal_store(fold<MODE, K>(v), reinterpret_cast<v4f*>(dst_all + head) + i);
    }
  }
  // scalar work: the head, the tail, or the whole array when the pointers do not share one 16-byte phase
  const int64_t left = count - n_vec * 4, stride = (int64_t)gridDim.x * kReduceThreads;
  for (int64_t r = (int64_t)blockIdx.x * kReduceThreads + threadIdx.x; r < left; r += stride) {
    const int64_t e = r < head ? r : r + n_vec * 4;
    float v[K];
#pragma unroll
    for (int j = 0; j < K; ++j) v[j] = src_all.p[j][e];
    dst_all[e] = fold<MODE, K>(v);
  }
}

// Vectors per lane: 8 (an 8 KB run per input and wavefront); the pairwise orders keep all k * VPL
// values in registers and take 4 when k > 8.
template <int K, int MODE> struct ReduceVpl { static constexpr int value = ((MODE == 1 || MODE == 3) && K > 8) ? 4 : 8; };

template <int K, int MODE>
static void launch_k(float* dst, const ReducePtrs& src, int64_t n_vec, int64_t count, int head, hipStream_t s) {
  constexpr int VPL = ReduceVpl<K, MODE>::value;
  constexpr int64_t chunk = (int64_t)kReduceThreads * VPL;
  // one workgroup per chunk of vectors; without a vector part (pointers out of phase) a grid-stride loop over elements
  int64_t blocks = n_vec > 0 ? (n_vec + chunk - 1) / chunk : (count + 4 * kReduceThreads - 1) / (4 * kReduceThreads);
  if (n_vec == 0 && blocks > 16384) blocks = 16384;
  if (dst == src.p[0]) hipLaunchKernelGGL((reduce_kernel<K, VPL, MODE, true>), dim3((unsigned)blocks), dim3(kReduceThreads), 0, s, dst, src, n_vec, count, head);
  else hipLaunchKernelGGL((reduce_kernel<K, VPL, MODE, false>), dim3((unsigned)blocks), dim3(kReduceThreads), 0, s, dst, src, n_vec, count, head);
}

template <int MODE>
static bool launch_mode(int k, float* dst, const ReducePtrs& src, int64_t n_vec, int64_t count, int head, hipStream_t s) {
  switch (k) {
#define TOFU_CASE(K) case K: launch_k<K, MODE>(dst, src, n_vec, count, head, s); return true;
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
  if (n_vec >= ((int64_t)1 << 31) * 64) return fail(TOFU_ERR_UNSUPPORTED, "reduce: more than 2^37 vectors in one call; split it");
  hipStream_t s = static_cast<hipStream_t>(stream);
  bool ok = false;
  switch (mode) {
    case 0: ok = launch_mode<0>(k, dst, src, n_vec, count, head, s); break;
    case 1: ok = launch_mode<1>(k, dst, src, n_vec, count, head, s); break;
    case 2: ok = launch_mode<2>(k, dst, src, n_vec, count, head, s); break;
    case 3: ok = launch_mode<3>(k, dst, src, n_vec, count, head, s); break;
    case 4: ok = launch_mode<4>(k, dst, src, n_vec, count, head, s); break;
    case 5: ok = launch_mode<5>(k, dst, src, n_vec, count, head, s); break;
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
