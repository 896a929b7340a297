// fp32 matrix-core and buffer-load primitives for gfx950 shared by the three contraction kernels.
//
// v_mfma_f32_32x32x2_f32: one wavefront multiplies a 32x2 block of A by a 2x32 block of B and
// accumulates into a 32x32 block of D (16 VGPRs per lane, 64 cycles on the matrix pipe).
//   lane l supplies  A[i = l % 32][k = l / 32]   and   B[k = l / 32][j = l % 32];
//   accumulator register v of lane l holds  D[i = 8*(v/4) + 4*(l/32) + v%4][j = l % 32].
// (Layout checked on the device against a host triple loop.)
#ifndef TOFU_MFMA_H_
#define TOFU_MFMA_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

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

constexpr uint32_t kNoOffset = 0xFFFFFFFFu;   // buffer offset that is out of range for every buffer

// Raw buffer loads: the descriptor carries base and size, a lane supplies a 32-bit byte offset
// and an out-of-range offset (kNoOffset marks zero padding and idle slots) reads as 0 without a
// branch; a scalar offset moves the whole wavefront to the current step of the K loop.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), (short)0, (int)bytes, 0x00020000);
}
__device__ __forceinline__ float buf_load(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff) {
  return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, (int)voff, (int)soff, 0));
}
__device__ __forceinline__ v4f32 buf_load4(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff) {
  return __builtin_bit_cast(v4f32, __builtin_amdgcn_raw_buffer_load_b128(r, (int)voff, (int)soff, 0));
}

}  // namespace tofu

#endif  // TOFU_MFMA_H_
