// Shard of a matrix multiplication (arXiv 1807.08887 Sec. 3.1: each worker runs the same
// operator on smaller inputs; Sec. 4.2: the smaller inputs are the regions of A and B the
// worker's index ranges touch).  C[m,n] = sum_{k in shard} A[m,k] * B[k,n] for (m,n) in the
// shard's output box.
//
// The operands are addressed through their element strides, so the backward GEMMs of the same
// layer (dX = dY * W^T, dW = X^T * dY; forward and backward form one group, Sec. 5.1) are the
// same call with a transposed view: TA / TB select the staging for an operand whose rows (A) or
// columns (B) are contiguous along the other index.
//
// Kernel: a BM x BN output tile per workgroup, K walked in steps of BK.  Each step stages
// A[BM x BK] and B[BK x BN] in LDS through registers, double-buffered so that the global loads
// of step t+1 are in flight while the matrix cores work on step t; one barrier per step.
// WM x WN wavefronts each own a (BM/WM) x (BN/WN) block of 32x32 MFMA tiles.  An operand whose
// global vectors run along k is kept row-major with the step's k values permuted so that the
// values a lane feeds to four successive MFMAs are one 16-byte LDS read (two 8-byte writes per
// global vector); an operand whose vectors run along the other index is kept k-major, written
// whole and read one float per MFMA.  Tall-skinny shards (the
// M = 128 LSTM gate GEMM) do not have enough output tiles to fill 256 CUs, so the kernel cuts
// its own K range into slices -- a partition-n-reduce inside the worker -- writes the slices to
// the caller's workspace and sums them in fixed order with the reduce kernel.
#include <hip/hip_runtime.h>

#include <mutex>
#include <type_traits>

#include "tofu_internal.h"
#include "tofu_mfma.h"

namespace tofu {

struct MatmulArgs {
  const float* A;   // element (m_lo, k_lo)
  const float* B;   // element (k_lo, n_lo)
  float* C;         // element (m_lo, n_lo) of the output, or slice 0 of the workspace
  int64_t a_rs, a_cs, b_rs, b_cs, c_rs, c_cs;   // row / column element strides
  int64_t c_slice;  // element stride between K slices of the workspace
  int m, n, k;      // shard extents
  int k_slice;      // K elements per slice (multiple of BK); slices = gridDim.y
  int tiles_n;      // number of tiles along n
  int accumulate;   // 1: the product is added to what the output box holds (only without K slices; the slice sum adds otherwise)
  int fast;         // 1: each operand contiguous along one index, 16-byte aligned, 32-bit offsets -> buffer vector loads
  uint32_t a_bytes, b_bytes;   // bytes spanned by the two input boxes (buffer bounds, fast path)
};

// TA: A is contiguous along m (a transposed view) instead of along k.
// TB: B is contiguous along k (a transposed view) instead of along n.
template <int BM, int BN, int BK, int WM, int WN, bool TA, bool TB>
struct MatmulCfg {
  static constexpr int kThreads = 64 * WM * WN;
  static constexpr int TM = BM / WM, TN = BN / WN;   // wavefront tile
  static constexpr int FM = TM / 32, FN = TN / 32;   // 32x32 MFMA tiles per wavefront
  // A tile.  TA (vectors along m): k-major As[k][m], written whole, read one float per MFMA.
  // Otherwise (vectors along k): m-major As[m][slot] with the step's k values permuted so that
  // the BK/2 values one lane feeds to successive MFMAs -- k = half, half + 2, half + 4, ... --
  // are consecutive: slot(k) = (k % 2) * BK/2 + k / 2.  A global vector k0..k0+3 is then two
  // 8-byte writes, and one 16-byte read serves four MFMA steps.  The pitch of BK + 4 floats
  // keeps rows 16-byte aligned and sends the eight lanes of a 128-byte read phase to
  // different banks.
  static constexpr int LDA = TA ? BM + 4 : BK + 4;
  static constexpr int kAStage = TA ? BK * LDA : BM * LDA;     // floats of one A buffer
  // B tile.  Vectors along n: k-major Bs[k][n], written whole.  TB (vectors along k): n-major
  // Bs[n][slot] with the same permuted k slots as A.
  static constexpr int LDB = TB ? BK + 4 : BN + 4;
  static constexpr int kBStage = TB ? BN * LDB : BK * LDB;     // floats of one B buffer
  static constexpr int kLdsFloats = 2 * (kAStage + kBStage);
  static constexpr int AV = BM * BK / 4 / kThreads;  // 16-byte vectors of A per thread per step
  static constexpr int BV = BK * BN / 4 / kThreads;
  static_assert(TM % 32 == 0 && TN % 32 == 0, "wavefront tile must be made of 32x32 blocks");
  static_assert(AV >= 1 && BV >= 1 && BM * BK / 4 % kThreads == 0 && BK * BN / 4 % kThreads == 0, "staging must divide evenly");
  static_assert(BK % 8 == 0, "BK must hold whole vectors and whole groups of four MFMA steps per half");
};

template <int BM, int BN, int BK, int WM, int WN, bool TA, bool TB>
__global__ void __launch_bounds__(64 * WM * WN) matmul_kernel(const MatmulArgs p) {
  using Cfg = MatmulCfg<BM, BN, BK, WM, WN, TA, TB>;
  constexpr int NT = Cfg::kThreads, LDA = Cfg::LDA, LDB = Cfg::LDB, FM = Cfg::FM, FN = Cfg::FN;
  __shared__ __attribute__((aligned(16))) float lds[Cfg::kLdsFloats];
  constexpr int AST = Cfg::kAStage, BST = Cfg::kBStage;
  float* As = lds;                      // [2][AST]: [BK][LDA] (TA) or [BM][LDA]
  float* Bs = lds + 2 * AST;            // [2][BST]: [BK][LDB] or (TB) [BN][LDB]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, half = lane >> 5;
  const int wm = wave / WN, wn = wave % WN;
  const int tile_m = blockIdx.x / p.tiles_n, tile_n = blockIdx.x % p.tiles_n;
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  const int k_begin = blockIdx.y * p.k_slice;
  const int k_end = min(p.k, k_begin + p.k_slice);
  const int steps = (k_end - k_begin + BK - 1) / BK;
  // Fast path: per-lane byte offsets are fixed; a K step only moves a scalar offset.  Vectors
  // that start past m or n read as zero (offset out of range); a vector that straddles the edge
  // may read a neighbouring row's values, which only reach accumulators that are never stored.
  uint32_t a_voff[Cfg::AV], b_voff[Cfg::BV];
#pragma unroll
  for (int i = 0; i < Cfg::AV; ++i) {
    const int idx = tid + i * NT;
    if (TA) {   // vector = rows m..m+3 of one k
      const int kk = idx / (BM / 4), mq = idx % (BM / 4);
      a_voff[i] = m0 + 4 * mq < p.m ? 4u * (uint32_t)((int64_t)kk * p.a_cs + m0 + 4 * mq) : kNoOffset;
    } else {    // vector = columns k..k+3 of one row
      const int row = idx / (BK / 4), q = idx % (BK / 4);
      a_voff[i] = m0 + row < p.m ? 4u * (uint32_t)((int64_t)(m0 + row) * p.a_rs + 4 * q) : kNoOffset;
    }
  }
#pragma unroll
  for (int i = 0; i < Cfg::BV; ++i) {
    const int idx = tid + i * NT;
    if (TB) {   // vector = rows k..k+3 of one column
      const int col = idx / (BK / 4), q = idx % (BK / 4);
      b_voff[i] = n0 + col < p.n ? 4u * (uint32_t)((int64_t)(n0 + col) * p.b_cs + 4 * q) : kNoOffset;
    } else {    // vector = columns n..n+3 of one row
      const int row = idx / (BN / 4), c = idx % (BN / 4);
      b_voff[i] = n0 + 4 * c < p.n ? 4u * (uint32_t)((int64_t)row * p.b_rs + n0 + 4 * c) : kNoOffset;
    }
  }
  const __amdgpu_buffer_rsrc_t a_rsrc = make_rsrc(p.A, p.a_bytes);
  const __amdgpu_buffer_rsrc_t b_rsrc = make_rsrc(p.B, p.b_bytes);

  v4f32 ra[Cfg::AV], rb[Cfg::BV];

  auto load_global = [&](int step) {
    const int k0 = k_begin + step * BK;
    const bool full_k = k0 + BK <= k_end;
    if (p.fast && full_k) {
      const uint32_t a_soff = 4u * (uint32_t)((int64_t)k0 * p.a_cs), b_soff = 4u * (uint32_t)((int64_t)k0 * p.b_rs);
#pragma unroll
      for (int i = 0; i < Cfg::AV; ++i) ra[i] = buf_load4(a_rsrc, a_voff[i], a_soff);
#pragma unroll
      for (int i = 0; i < Cfg::BV; ++i) rb[i] = buf_load4(b_rsrc, b_voff[i], b_soff);
    } else {    // guarded element loads into the same register layout
#pragma unroll
      for (int i = 0; i < Cfg::AV; ++i) {
        const int idx = tid + i * NT;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int mm = m0 + (TA ? 4 * (idx % (BM / 4)) + j : idx / (BK / 4));
          const int kk = k0 + (TA ? idx / (BM / 4) : 4 * (idx % (BK / 4)) + j);
          ra[i][j] = (mm < p.m && kk < k_end) ? p.A[(int64_t)mm * p.a_rs + (int64_t)kk * p.a_cs] : 0.f;
        }
      }
#pragma unroll
      for (int i = 0; i < Cfg::BV; ++i) {
        const int idx = tid + i * NT;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int kk = k0 + (TB ? 4 * (idx % (BK / 4)) + j : idx / (BN / 4));
          const int nn = n0 + (TB ? idx / (BK / 4) : 4 * (idx % (BN / 4)) + j);
          rb[i][j] = (kk < k_end && nn < p.n) ? p.B[(int64_t)kk * p.b_rs + (int64_t)nn * p.b_cs] : 0.f;
        }
      }
    }
  };
  auto store_a = [&](float* as, int i) {
    const int idx = tid + i * NT;
    if (TA) {
      *reinterpret_cast<v4f32*>(as + (idx / (BM / 4)) * LDA + 4 * (idx % (BM / 4))) = ra[i];
    } else {   // k = 4q, 4q+2 -> slots 2q, 2q+1 of the even half; k = 4q+1, 4q+3 -> the same slots of the odd half
      const int row = idx / (BK / 4), q = idx % (BK / 4);
      typedef float v2f32 __attribute__((ext_vector_type(2)));
      v2f32 even = {ra[i][0], ra[i][2]}, odd = {ra[i][1], ra[i][3]};
      *reinterpret_cast<v2f32*>(as + row * LDA + 2 * q) = even;
      *reinterpret_cast<v2f32*>(as + row * LDA + BK / 2 + 2 * q) = odd;
    }
  };
  auto store_b = [&](float* bs, int i) {
    const int idx = tid + i * NT;
    if (TB) {
      const int col = idx / (BK / 4), q = idx % (BK / 4);
      typedef float v2f32 __attribute__((ext_vector_type(2)));
      v2f32 even = {rb[i][0], rb[i][2]}, odd = {rb[i][1], rb[i][3]};
      *reinterpret_cast<v2f32*>(bs + col * LDB + 2 * q) = even;
      *reinterpret_cast<v2f32*>(bs + col * LDB + BK / 2 + 2 * q) = odd;
    } else {
      *reinterpret_cast<v4f32*>(bs + (idx / (BN / 4)) * LDB + 4 * (idx % (BN / 4))) = rb[i];
    }
  };
  auto store_lds = [&](int buf) {
#pragma unroll
    for (int i = 0; i < Cfg::AV; ++i) store_a(As + buf * AST, i);
#pragma unroll
    for (int i = 0; i < Cfg::BV; ++i) store_b(Bs + buf * BST, i);
  };

  acc16 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j) acc[i][j] = acc_zero();

  // Pipeline: the tiles of step t+1 are written to LDS during step t, and right after
  // each write the global loads of step t+2 are issued into the same registers, so every load has a
  // whole step to land.  The body is branch-free (the compiler can then count outstanding LDS
  // operations exactly): the last steps simply stage the final tiles again into the idle buffer.
  if (steps > 0) {
    load_global(0);
    store_lds(0);
    load_global(min(1, steps - 1));
  }
  __syncthreads();
  // Staging work of one step = AV tiles of A + BV tiles of B per lane.  In a HOT step each item
  // (write last step's registers to LDS, then reload them for the step after next) is issued
  // between two k-steps of the MFMA stream, so that no MFMA waits behind a block of staging
  // instructions.  Steps whose reload would touch a ragged K tail, and operands that need the
  // guarded element loads, stage in one block instead.
  constexpr int KS = BK / 2, NI = Cfg::AV + Cfg::BV, STRIDE = (KS - 2) / NI > 0 ? (KS - 2) / NI : 1;
  static_assert(1 + (NI - 1) * STRIDE < KS, "staging items must fit into one step");
  const int n_hot = !p.fast ? 0 : (k_end - k_begin) % BK == 0 ? steps : max(0, steps - 3);

  auto run_step = [&](int t, auto hot_tag) {
    constexpr bool HOT = decltype(hot_tag)::value;
    const int buf = t & 1;
    const float* as = TA ? As + buf * AST + wm * Cfg::TM + l32 + half * LDA
                         : As + buf * AST + (wm * Cfg::TM + l32) * LDA + half * (BK / 2);
    const float* bs = TB ? Bs + buf * BST + (wn * Cfg::TN + l32) * LDB + half * (BK / 2)
                         : Bs + buf * BST + wn * Cfg::TN + l32 + half * LDB;
    float* as_next = As + (buf ^ 1) * AST;
    float* bs_next = Bs + (buf ^ 1) * BST;
    const int nxt = min(t + 2, steps - 1), k0 = k_begin + nxt * BK;
    const uint32_t a_soff = 4u * (uint32_t)((int64_t)k0 * p.a_cs), b_soff = 4u * (uint32_t)((int64_t)k0 * p.b_rs);
    // operands of k-step s+1 are fetched before the MFMAs of k-step s are issued
    float a[2][FM], b[2][FN];
    v4f32 ag[2][FM], bg[2][FN];                // vectors along k: the values of four MFMA steps per 16-byte read
    auto fetch = [&](int s, float (&av)[FM], float (&bv)[FN]) {
      if constexpr (TA) {
#pragma unroll
        for (int i = 0; i < FM; ++i) av[i] = as[2 * s * LDA + i * 32];
      } else if (s % 4 == 0) {
#pragma unroll
        for (int i = 0; i < FM; ++i) ag[(s / 4) & 1][i] = *reinterpret_cast<const v4f32*>(as + i * 32 * LDA + s);
      }
      if constexpr (!TB) {
#pragma unroll
        for (int j = 0; j < FN; ++j) bv[j] = bs[2 * s * LDB + j * 32];
      } else if (s % 4 == 0) {
#pragma unroll
        for (int j = 0; j < FN; ++j) bg[(s / 4) & 1][j] = *reinterpret_cast<const v4f32*>(bs + j * 32 * LDB + s);
      }
    };
    fetch(0, a[0], b[0]);
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      if (s + 1 < KS) fetch(s + 1, a[(s + 1) & 1], b[(s + 1) & 1]);
      if (HOT) {
        if (s >= 1 && (s - 1) % STRIDE == 0 && (s - 1) / STRIDE < NI) {
          const int item = (s - 1) / STRIDE;
          if (item < Cfg::AV) {
            store_a(as_next, item);
            ra[item] = buf_load4(a_rsrc, a_voff[item], a_soff);
          } else {
            const int i = item - Cfg::AV;
            store_b(bs_next, i);
            rb[i] = buf_load4(b_rsrc, b_voff[i], b_soff);
          }
        }
      } else if (s == KS / 2) {
        store_lds(buf ^ 1);
        load_global(nxt);
      }
      __builtin_amdgcn_sched_barrier(0);       // keep fetch and staging ahead of the MFMAs they overlap with
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) acc[i][j] = mfma_32x32x2(TA ? a[s & 1][i] : ag[(s / 4) & 1][i][s % 4], TB ? bg[(s / 4) & 1][j][s % 4] : b[s & 1][j], acc[i][j]);
    }
    __syncthreads();
  };
  for (int t = 0; t < n_hot; ++t) run_step(t, std::true_type());
  for (int t = n_hot; t < steps; ++t) run_step(t, std::false_type());

  float* C = p.C + (int64_t)blockIdx.y * p.c_slice;
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j) {
      const int col = n0 + wn * Cfg::TN + j * 32 + l32;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = m0 + wm * Cfg::TM + i * 32 + acc_row(v, half);
        if (row < p.m && col < p.n) {
          float* c = C + (int64_t)row * p.c_rs + (int64_t)col * p.c_cs;
          *c = p.accumulate ? *c + acc[i][j][v] : acc[i][j][v];
        }
      }
    }
}

// Sum of the K slices held in the workspace ([slices][m][n], dense) into the output box, in
// fixed order; with `accumulate` the sum of the slices is then added to what the box holds.
// The output may be a strided block of a larger tensor.
__global__ void __launch_bounds__(256) slice_sum_kernel(float* __restrict__ C, int64_t c_rs, int64_t c_cs, const float* __restrict__ ws,
                                                         int slices, int m, int n, int vec, int accumulate) {
  const int64_t per_row = n / vec, items = (int64_t)m * per_row, slice = (int64_t)m * n;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < items; i += (int64_t)gridDim.x * blockDim.x) {
    const int64_t row = i / per_row, col = (i - row * per_row) * vec;
    const float* src = ws + row * n + col;
    if (vec == 4) {
      v4f32 acc = *reinterpret_cast<const v4f32*>(src);
      for (int j = 1; j < slices; ++j) acc += *reinterpret_cast<const v4f32*>(src + j * slice);
      v4f32* c = reinterpret_cast<v4f32*>(C + row * c_rs + col);
      *c = accumulate ? *c + acc : acc;
    } else {
      float acc = src[0];
      for (int j = 1; j < slices; ++j) acc += src[j * slice];
      float* c = C + row * c_rs + col * c_cs;
      *c = accumulate ? *c + acc : acc;
    }
  }
}

// ---- launch plan -------------------------------------------------------------------------
constexpr int kBM = 128, kBN = 64, kBK = 32, kWM = 2, kWN = 2;
constexpr int kTargetGroups = 512;   // two resident workgroups on each of the 256 compute units
constexpr int kMaxSplit = 16;        // the reduce kernel sums at most 16 inputs

int matmul_split_k(int64_t m, int64_t n, int64_t k) {
  int64_t tiles = ((m + kBM - 1) / kBM) * ((n + kBN - 1) / kBN);
  if (tiles >= kTargetGroups || k < 1024) return 1;
  int64_t s = kTargetGroups / tiles;
  if (s > kMaxSplit) s = kMaxSplit;
  while (s > 1 && k / s < 512) --s;   // keep every slice long enough to amortise its prologue
  return (int)s;
}

static int shard_matmul(const tofu_op_desc_t* op, const tofu_split_t* splits, int32_t nsplits, const tofu_tensor_t* A,
                        const tofu_tensor_t* B, const tofu_tensor_t* C, void* workspace, size_t workspace_bytes, void* hip_stream,
                        bool accumulate) {
  if (!op || op->kind != TOFU_OP_MATMUL) return fail(TOFU_ERR_INVALID_ARG, "operator description is not a matmul");
  tofu_region_t out_box, in_boxes[2];
  int32_t partial = 0;
  int rc = tofu_op_regions(op, splits, nsplits, &out_box, in_boxes, nullptr, nullptr, &partial);
  if (rc) return rc;
  if ((rc = check_tensor("A", A, 2, &in_boxes[0]))) return rc;
  if ((rc = check_tensor("B", B, 2, &in_boxes[1]))) return rc;
  if ((rc = check_tensor("C", C, 2, &out_box))) return rc;
  const int64_t m = out_box.hi[0] - out_box.lo[0], n = out_box.hi[1] - out_box.lo[1];
  const int64_t k = in_boxes[0].hi[1] - in_boxes[0].lo[1];
  if (m == 0 || n == 0) return TOFU_OK;
  if (m >= (1 << 30) || n >= (1 << 30) || k >= (1 << 30)) return fail(TOFU_ERR_UNSUPPORTED, "matmul shard extent exceeds 2^30");

  int64_t as[2], bs[2], cs[2];
  effective_strides(A, as);
  effective_strides(B, bs);
  effective_strides(C, cs);
  MatmulArgs p;
  p.A = element_ptr(A, as, in_boxes[0].lo);
  p.B = element_ptr(B, bs, in_boxes[1].lo);
  float* c_out = const_cast<float*>(element_ptr(C, cs, out_box.lo));
  p.a_rs = as[0]; p.a_cs = as[1]; p.b_rs = bs[0]; p.b_cs = bs[1];
  p.m = (int)m; p.n = (int)n; p.k = (int)k;
  p.tiles_n = (int)((n + kBN - 1) / kBN);
  const int tiles_m = (int)((m + kBM - 1) / kBM);
  const int64_t a_span = 1 + (m - 1) * as[0] + (k - 1) * as[1], b_span = 1 + (k - 1) * bs[0] + (n - 1) * bs[1];
  // Vector staging needs each operand contiguous along one index with the other stride a whole
  // number of vectors: A along k (plain) or along m (ta), B along n (plain) or along k (tb).
  const bool ta = as[1] != 1 && as[0] == 1, tb = bs[1] != 1 && bs[0] == 1;
  const int64_t a_ld = ta ? as[1] : as[0], b_ld = tb ? bs[1] : bs[0];
  p.fast = (ta || as[1] == 1) && (tb || bs[1] == 1) && a_ld >= 0 && b_ld >= 0 && a_ld % 4 == 0 && b_ld % 4 == 0 &&
           (reinterpret_cast<uintptr_t>(p.A) & 15) == 0 && (reinterpret_cast<uintptr_t>(p.B) & 15) == 0 &&
           a_span < ((int64_t)1 << 29) && b_span < ((int64_t)1 << 29);
  p.a_bytes = p.fast ? (uint32_t)(4 * a_span) : 0;
  p.b_bytes = p.fast ? (uint32_t)(4 * b_span) : 0;

  const int split = matmul_split_k(m, n, k);
  if (split > 1) {
    const size_t need = (size_t)split * (size_t)m * (size_t)n * sizeof(float);
    if (!workspace || workspace_bytes < need)
      return fail(TOFU_ERR_WORKSPACE_TOO_SMALL, "matmul shard needs %zu workspace bytes, got %zu", need, workspace ? workspace_bytes : (size_t)0);
    if (reinterpret_cast<uintptr_t>(workspace) & 15) return fail(TOFU_ERR_INVALID_ARG, "workspace must be 16-byte aligned");
    p.C = static_cast<float*>(workspace);
    p.accumulate = 0;
    p.c_rs = n; p.c_cs = 1; p.c_slice = m * n;
    p.k_slice = (int)(((k + split - 1) / split + kBK - 1) / kBK * kBK);
  } else {
    p.C = c_out;
    p.accumulate = accumulate ? 1 : 0;
    p.c_rs = cs[0]; p.c_cs = cs[1]; p.c_slice = 0;
    p.k_slice = (int)((k + kBK - 1) / kBK * kBK);
  }
  const int slices = (int)((k + p.k_slice - 1) / p.k_slice);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  void (*kern)(const MatmulArgs) = matmul_kernel<kBM, kBN, kBK, kWM, kWN, false, false>;   // also the guarded path for any strides
  if (p.fast && ta && tb) kern = matmul_kernel<kBM, kBN, kBK, kWM, kWN, true, true>;
  else if (p.fast && ta) kern = matmul_kernel<kBM, kBN, kBK, kWM, kWN, true, false>;
  else if (p.fast && tb) kern = matmul_kernel<kBM, kBN, kBK, kWM, kWN, false, true>;
  hipLaunchKernelGGL(kern, dim3(tiles_m * p.tiles_n, slices > 0 ? slices : 1), dim3(64 * kWM * kWN), 0, s, p);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(TOFU_ERR_HIP, "matmul launch failed: %s", hipGetErrorString(e));
  if (split > 1) {
    // sum the K slices in fixed order j = 0..slices-1 into the (possibly strided) output box
    const int vec = (n % 4 == 0 && cs[1] == 1 && cs[0] % 4 == 0 && (reinterpret_cast<uintptr_t>(c_out) & 15) == 0) ? 4 : 1;
    const int64_t items = m * (n / vec);
    const int blocks = (int)((items + 255) / 256 < 4096 ? (items + 255) / 256 : 4096);
    hipLaunchKernelGGL(slice_sum_kernel, dim3(blocks), dim3(256), 0, s, c_out, cs[0], cs[1], static_cast<const float*>(workspace),
                       slices, (int)m, (int)n, vec, accumulate ? 1 : 0);
    e = hipGetLastError();
    if (e != hipSuccess) return fail(TOFU_ERR_HIP, "matmul slice sum launch failed: %s", hipGetErrorString(e));
  }
  return TOFU_OK;
}

}  // namespace tofu

extern "C" int tofu_shard_matmul(const tofu_op_desc_t* op, const tofu_split_t* splits, int32_t nsplits,
                                 const tofu_tensor_t* A, const tofu_tensor_t* B, const tofu_tensor_t* C, void* workspace,
                                 size_t workspace_bytes, void* hip_stream) {
  return tofu::shard_matmul(op, splits, nsplits, A, B, C, workspace, workspace_bytes, hip_stream, false);
}

extern "C" int tofu_shard_matmul_accumulate(const tofu_op_desc_t* op, const tofu_split_t* splits, int32_t nsplits,
                                            const tofu_tensor_t* A, const tofu_tensor_t* B, const tofu_tensor_t* C, void* workspace,
                                            size_t workspace_bytes, void* hip_stream) {
  return tofu::shard_matmul(op, splits, nsplits, A, B, C, workspace, workspace_bytes, hip_stream, true);
}

// ---- the same shard for callers that cannot allocate -------------------------------------
// The K slices go to a fixed array in device memory instead of a caller-owned workspace.  In host
// code the array's name is only a handle: its device address is looked up once per device with
// hipGetSymbolAddress and kept; every launch takes that address, never the name.
namespace tofu {

constexpr size_t kStaticScratchBytes = TOFU_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static void* g_scratch_addr[kMaxDevices];   // device address of `scratch` on each device, 0 until looked up
static std::mutex g_scratch_mutex;

// Address of this device's copy of `scratch` (each GPU holds its own copy at its own address).
static int static_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail(TOFU_ERR_HIP, "hipGetDevice failed: %s", hipGetErrorString(e));
  if (dev < 0 || dev >= kMaxDevices) return fail(TOFU_ERR_UNSUPPORTED, "device index %d outside [0,%d)", dev, kMaxDevices);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_addr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) return fail(TOFU_ERR_HIP, "hipGetSymbolAddress(scratch) failed on device %d: %s", dev, hipGetErrorString(e));
    g_scratch_addr[dev] = ptr;
  }
  *out = g_scratch_addr[dev];
  return TOFU_OK;
}

}  // namespace tofu

extern "C" int tofu_shard_matmul_noalloc(const tofu_op_desc_t* op, const tofu_split_t* splits, int32_t nsplits,
                                         const tofu_tensor_t* A, const tofu_tensor_t* B, const tofu_tensor_t* C, void* hip_stream) {
  using namespace tofu;
  if (!op || op->kind != TOFU_OP_MATMUL) return fail(TOFU_ERR_INVALID_ARG, "operator description is not a matmul");
  // size check first, on the host, before anything touches the device (0 also for an invalid plan: the shard call reports that)
  const size_t need = tofu_workspace_bytes(op, splits, nsplits);
  if (need > kStaticScratchBytes)
    return fail(TOFU_ERR_WORKSPACE_TOO_SMALL, "matmul shard needs %zu bytes for its K slices; the built-in scratch array holds %zu: use tofu_shard_matmul with a workspace",
                need, kStaticScratchBytes);
  void* ws = nullptr;
  if (need > 0) {
    int rc = static_scratch(&ws);
    if (rc) return rc;
  }
  return shard_matmul(op, splits, nsplits, A, B, C, ws, need > 0 ? kStaticScratchBytes : 0, hip_stream, false);
}
