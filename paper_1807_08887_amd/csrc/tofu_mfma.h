// fp32 matrix-core primitives for gfx950 shared by the three contraction kernels.
//
// v_mfma_f32_32x32x2_f32: one wavefront multiplies a 32x2 block of A by a 2x32 block of B and
// accumulates into a 32x32 block of D (16 VGPRs per lane, 64 cycles on the matrix pipe).
//   lane l supplies  A[i = l % 32][k = l / 32]   and   B[k = l / 32][j = l % 32];
//   accumulator register v of lane l holds  D[i = 8*(v/4) + 4*(l/32) + v%4][j = l % 32].
// (Layout checked on the device against a host triple loop.)
#ifndef TOFU_MFMA_H_
#define TOFU_MFMA_H_

#include <hip/hip_runtime.h>

namespace tofu {

typedef float acc16 __attribute__((ext_vector_type(16)));
typedef float v4f32 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ acc16 mfma_32x32x2(float a, float b, acc16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

// Row (within the 32x32 block) held by accumulator register v of a lane in half `half` (= lane / 32).
__device__ __forceinline__ int acc_row(int v, int half) { return 8 * (v >> 2) + 4 * half + (v & 3); }

__device__ __forceinline__ acc16 acc_zero() {
  acc16 z;
#pragma unroll
  for (int i = 0; i < 16; ++i) z[i] = 0.f;
  return z;
}

}  // namespace tofu

#endif  // TOFU_MFMA_H_
