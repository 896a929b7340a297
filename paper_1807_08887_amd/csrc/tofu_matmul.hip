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
// Kernel: a 128 x 128 output tile per workgroup, K walked in steps.  Four wavefronts (2 x 2)
// each own a 64 x 64 block of the tile = 2 x 2 MFMA blocks of 32 x 32, so one k pair costs four
// MFMAs against two A and two B operand values per lane.  Each step stages A[128 x BK] and
// B[BK x 128] in LDS through registers, double-buffered so that the global loads of step t+2
// are in flight while the matrix cores work on step t; one barrier per step.  An operand whose
// global vectors run along k is kept row-major with the step's k values permuted so that the
// values a lane feeds to four successive MFMAs are one 16-byte LDS read (two 8-byte writes per
// global vector); an operand whose vectors run along the other index is kept k-major, written
// whole, and the two MFMA blocks of a wavefront take INTERLEAVED rows / columns (block j owns
// columns 2c + j), so that both blocks' values are one 8-byte read and a lane's two results of
// a row are one 8-byte store.
// Few tiles (the M = 128 LSTM gate GEMM has 32 to 256 of them for 256 compute units): the
// reduction is then cut inside the worker -- a partition-n-reduce of its own.  First inside the
// workgroup (KG = 2): eight wavefronts, the second four taking the other half of every K step
// and handing their accumulators over through LDS at the end (no memory traffic); then, if
// there are still fewer workgroups than compute units, into K slices across workgroups, which
// go to the caller's workspace and are summed in fixed order by a second kernel.
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
  int k_slice;      // K elements per slice (multiple of the step); slices = gridDim.y
  int tiles_m, tiles_n;   // number of tiles along m and n
  int accumulate;   // 1: the product is added to what the output box holds (only without K slices; the slice sum adds otherwise)
  int c_vec2;       // 1: two adjacent columns of C may be stored as one 8-byte vector
  uint32_t a_bytes, b_bytes;   // bytes spanned by the two input boxes (buffer bounds, fast path)
};

typedef float v2f32 __attribute__((ext_vector_type(2)));

// KG: wavefront groups of four that share a tile and split every K step between them (1 or 2).
// TA: A is contiguous along m (a transposed view) instead of along k.
// TB: B is contiguous along k (a transposed view) instead of along n.
template <int KG, bool TA, bool TB>
struct MatmulCfg {
  static constexpr int BM = 128, BN = 128, BKG = 32, BK = BKG * KG;
  static constexpr int kThreads = 256 * KG;
  static constexpr int FM = 2, FN = 2;               // 32x32 MFMA blocks per wavefront: a 64 x 64 block of the tile
  // A tile.  TA (vectors along m): k-major As[k][m], written whole; block i of a wavefront owns rows
  // 2r + i, so one 8-byte read serves both blocks.  Otherwise (vectors along k): m-major As[m][slot]
  // with the k values of every group of 32 permuted so that the 16 values one lane feeds to
  // successive MFMAs -- k = half, half + 2, half + 4, ... -- are consecutive:
  // slot(k) = 32 * (k / 32) + (k % 2) * 16 + (k % 32) / 2.  A global vector k0..k0+3 is then two
  // 8-byte writes, and one 16-byte read serves four MFMA steps.  The pitch of BK + 4 floats keeps
  // rows 16-byte aligned and sends the eight lanes of a 128-byte read phase to different banks.
  static constexpr int LDA = TA ? BM + 4 : BK + 4;
  static constexpr int kAStage = TA ? BK * LDA : BM * LDA;     // floats of one A buffer
  // B tile.  Vectors along n: k-major Bs[k][n], written whole, block j owns columns 2c + j.
  // TB (vectors along k): n-major Bs[n][slot] with the same permuted k slots as A.
  static constexpr int LDB = TB ? BK + 4 : BN + 4;
  static constexpr int kBStage = TB ? BN * LDB : BK * LDB;     // floats of one B buffer
  static constexpr int kLdsFloats = 2 * (kAStage + kBStage);
  static constexpr int AV = BM * BK / 4 / kThreads;  // 16-byte vectors of A per thread per step (4)
  static constexpr int BV = BK * BN / 4 / kThreads;
  static_assert(AV == 4 && BV == 4, "staging is four vectors of each operand per thread");
  static_assert(kLdsFloats >= (KG - 1) * BM * BN, "the accumulator hand-over of the second wavefront group reuses the staging buffers");
};

// GUARDED: every step stages with guarded element loads (any strides, any K range); otherwise every step is a
// whole one of 16-byte buffer loads (the host launches the two forms for the two parts of a ragged K range).
template <int KG, bool TA, bool TB, bool GUARDED>
__global__ void __launch_bounds__(256 * KG) matmul_kernel(const MatmulArgs p) {
  using Cfg = MatmulCfg<KG, TA, TB>;
  constexpr int NT = Cfg::kThreads, LDA = Cfg::LDA, LDB = Cfg::LDB, FM = Cfg::FM, FN = Cfg::FN;
  constexpr int BM = Cfg::BM, BN = Cfg::BN, BK = Cfg::BK, BKG = Cfg::BKG;
  __shared__ __attribute__((aligned(16))) float lds[Cfg::kLdsFloats];
  constexpr int AST = Cfg::kAStage, BST = Cfg::kBStage;
  float* As = lds;                      // [2][AST]: [BK][LDA] (TA) or [BM][LDA]
  float* Bs = lds + 2 * AST;            // [2][BST]: [BK][LDB] or (TB) [BN][LDB]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, half = lane >> 5;
  const int kg = wave >> 2, wq = wave & 3, wm = wq >> 1, wn = wq & 1;
  // Workgroups are dealt round robin to the 8 XCDs; renumber them so that every XCD works on a run of
  // consecutive tiles (one or a few tile rows: the A panel stays in that XCD's L2).  A workgroup takes the
  // tiles first, first + G, first + 2 G, ... (G workgroups) and walks them as ONE stream of K steps: the
  // loads of the next tile's first steps are in flight while the last steps of the current tile are
  // multiplied, so only the first tile of a workgroup pays the latency of a cold start.
  const int G = gridDim.x, xcd = blockIdx.x & 7, per = G >> 3, rem = G & 7;
  const int first = xcd * per + min(xcd, rem) + (blockIdx.x >> 3);
  const int n_tiles = p.tiles_m * p.tiles_n;
  const int my_tiles = (n_tiles - first + G - 1) / G;
  const int k_begin = blockIdx.y * p.k_slice;
  const int k_end = min(p.k, k_begin + p.k_slice);
  // Steps per tile.  The vector kernel walks the whole steps of its K range as a pipelined stream and, when the
  // range does not end on a step boundary, finishes every tile with one tail step of guarded loads; each tile
  // is then a stream of its own (nothing of the next tile is in flight while the tail uses the staging buffers).
  const int steps = GUARDED ? (k_end - k_begin + BK - 1) / BK : (k_end - k_begin) / BK;
  const int k_tail = GUARDED ? 0 : (k_end - k_begin) - steps * BK;
  const bool per_tile = k_tail > 0;
  const int total = per_tile ? steps : my_tiles * steps;  // steps of one stream
  // Fast path: per-lane byte offsets are fixed for a tile; a K step only moves a scalar offset.  Vectors
  // that start past m or n read as zero (offset out of range); a vector that straddles the edge
  // may read a neighbouring row's values, which only reach accumulators that are never stored.
  // The offsets belong to the LOAD stream, which runs two steps ahead of the multiplication.
  uint32_t a_voff[Cfg::AV], b_voff[Cfg::BV];
  int ld_m0 = 0, ld_n0 = 0;
  auto set_load_tile = [&](int tile) {
    ld_m0 = (tile / p.tiles_n) * BM;
    ld_n0 = (tile % p.tiles_n) * BN;
#pragma unroll
    for (int i = 0; i < Cfg::AV; ++i) {
      const int idx = tid + i * NT;
      if (TA) {   // vector = rows m..m+3 of one k
        const int kk = idx / (BM / 4), mq = idx % (BM / 4);
        a_voff[i] = ld_m0 + 4 * mq < p.m ? 4u * (uint32_t)((int64_t)kk * p.a_cs + ld_m0 + 4 * mq) : kNoOffset;
      } else {    // vector = columns k..k+3 of one row
        const int row = idx / (BK / 4), q = idx % (BK / 4);
        a_voff[i] = ld_m0 + row < p.m ? 4u * (uint32_t)((int64_t)(ld_m0 + row) * p.a_rs + 4 * q) : kNoOffset;
      }
    }
#pragma unroll
    for (int i = 0; i < Cfg::BV; ++i) {
      const int idx = tid + i * NT;
      if (TB) {   // vector = rows k..k+3 of one column
        const int col = idx / (BK / 4), q = idx % (BK / 4);
        b_voff[i] = ld_n0 + col < p.n ? 4u * (uint32_t)((int64_t)(ld_n0 + col) * p.b_cs + 4 * q) : kNoOffset;
      } else {    // vector = columns n..n+3 of one row
        const int row = idx / (BN / 4), c = idx % (BN / 4);
        b_voff[i] = ld_n0 + 4 * c < p.n ? 4u * (uint32_t)((int64_t)row * p.b_rs + ld_n0 + 4 * c) : kNoOffset;
      }
    }
  };
  // position of the load stream: step ld_t of tile ld_tile; advancing past a tile's last step moves on to
  // the workgroup's next tile, and past the last tile stays on the final step (staged again, never used)
  int ld_tile = first, ld_t = 0, ld_left = total;
  auto advance_load = [&]() {
    if (ld_left <= 1) return;
    --ld_left;
    if (++ld_t == steps) {
      ld_t = 0;
      ld_tile += G;
      set_load_tile(ld_tile);
    }
  };
  const __amdgpu_buffer_rsrc_t a_rsrc = make_rsrc(p.A, p.a_bytes);
  const __amdgpu_buffer_rsrc_t b_rsrc = make_rsrc(p.B, p.b_bytes);

  v4f32 ra[Cfg::AV], rb[Cfg::BV];

  // guarded element loads of the step at (m0, n0, k0) into the staging registers' layout
  auto load_guarded = [&](int m0, int n0, int k0) {
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
  };
  auto load_global = [&]() {          // the step the load stream stands on
    const int k0 = k_begin + ld_t * BK;
    if constexpr (!GUARDED) {
      const uint32_t a_soff = 4u * (uint32_t)((int64_t)k0 * p.a_cs), b_soff = 4u * (uint32_t)((int64_t)k0 * p.b_rs);
#pragma unroll
      for (int i = 0; i < Cfg::AV; ++i) ra[i] = buf_load4(a_rsrc, a_voff[i], a_soff);
#pragma unroll
      for (int i = 0; i < Cfg::BV; ++i) rb[i] = buf_load4(b_rsrc, b_voff[i], b_soff);
    } else {
      load_guarded(ld_m0, ld_n0, k0);
    }
  };
  // vector q of a row holds k = 4q .. 4q+3: the even two go to slots 2 (q % 8), +1 of group q / 8, the odd two 16 further on
  auto store_a = [&](float* as, int i) {
    const int idx = tid + i * NT;
    if (TA) {
      *reinterpret_cast<v4f32*>(as + (idx / (BM / 4)) * LDA + 4 * (idx % (BM / 4))) = ra[i];
    } else {
      const int row = idx / (BK / 4), q = idx % (BK / 4);
      float* dst = as + row * LDA + (q >> 3) * BKG + 2 * (q & 7);
      v2f32 even = {ra[i][0], ra[i][2]}, odd = {ra[i][1], ra[i][3]};
      *reinterpret_cast<v2f32*>(dst) = even;
      *reinterpret_cast<v2f32*>(dst + BKG / 2) = odd;
    }
  };
  auto store_b = [&](float* bs, int i) {
    const int idx = tid + i * NT;
    if (TB) {
      const int col = idx / (BK / 4), q = idx % (BK / 4);
      float* dst = bs + col * LDB + (q >> 3) * BKG + 2 * (q & 7);
      v2f32 even = {rb[i][0], rb[i][2]}, odd = {rb[i][1], rb[i][3]};
      *reinterpret_cast<v2f32*>(dst) = even;
      *reinterpret_cast<v2f32*>(dst + BKG / 2) = odd;
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
  auto start_stream = [&](int tile) {
    ld_tile = tile;
    ld_t = 0;
    ld_left = total;
    set_load_tile(tile);
    if (total > 0) {      // the loads of the first two steps are in flight together
      load_global();
      v4f32 ra0[Cfg::AV], rb0[Cfg::BV];
#pragma unroll
      for (int i = 0; i < Cfg::AV; ++i) ra0[i] = ra[i];
#pragma unroll
      for (int i = 0; i < Cfg::BV; ++i) rb0[i] = rb[i];
      advance_load();
      load_global();
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < Cfg::AV; ++i) { v4f32 t = ra[i]; ra[i] = ra0[i]; ra0[i] = t; }
#pragma unroll
      for (int i = 0; i < Cfg::BV; ++i) { v4f32 t = rb[i]; rb[i] = rb0[i]; rb0[i] = t; }
      store_lds(0);
#pragma unroll
      for (int i = 0; i < Cfg::AV; ++i) ra[i] = ra0[i];
#pragma unroll
      for (int i = 0; i < Cfg::BV; ++i) rb[i] = rb0[i];
    }
    __syncthreads();
  };
  // Staging work of one step = AV tiles of A + BV tiles of B per lane.  In a HOT step each item
  // (write last step's registers to LDS, then reload them for the step after next) is issued
  // between two k pairs of the MFMA stream, so that no MFMA waits behind a block of staging
  // instructions.  Steps whose reload would touch a ragged K tail, and operands that need the
  // guarded element loads, stage in one block instead.
  constexpr int KS = BKG / 2, NI = Cfg::AV + Cfg::BV;   // k pairs of a wavefront per step; staging items
  static_assert(1 + (NI - 1) < KS, "staging items must fit into one step");
  // One step of the stream on buffer `buf`; on entry the load stream stands on the step after next.
  auto run_step = [&](int buf, auto hot_tag) {
    constexpr bool HOT = decltype(hot_tag)::value;
    // this wavefront's operand rows: its group's half of the step (kg), its quarter of the tile (wm, wn)
    const float* as = TA ? As + buf * AST + (kg * BKG + half) * LDA + wm * 64 + 2 * l32
                         : As + buf * AST + (wm * 64 + l32) * LDA + kg * BKG + half * (BKG / 2);
    const float* bs = TB ? Bs + buf * BST + (wn * 64 + l32) * LDB + kg * BKG + half * (BKG / 2)
                         : Bs + buf * BST + (kg * BKG + half) * LDB + wn * 64 + 2 * l32;
    float* as_next = As + (buf ^ 1) * AST;
    float* bs_next = Bs + (buf ^ 1) * BST;
    const int k0 = k_begin + ld_t * BK;
    const uint32_t a_soff = 4u * (uint32_t)((int64_t)k0 * p.a_cs), b_soff = 4u * (uint32_t)((int64_t)k0 * p.b_rs);
    // operands of k pair s+1 are fetched before the MFMAs of k pair s are issued
    v2f32 a2[2], b2[2];                        // k-major tiles: both blocks' values of one k pair per 8-byte read
    v4f32 ag[2][FM], bg[2][FN];                // vectors along k: the values of four k pairs per 16-byte read
    auto fetch = [&](int s) {
      if constexpr (TA) {
        a2[s & 1] = *reinterpret_cast<const v2f32*>(as + 2 * s * LDA);
      } else if (s % 4 == 0) {
#pragma unroll
        for (int i = 0; i < FM; ++i) ag[(s / 4) & 1][i] = *reinterpret_cast<const v4f32*>(as + i * 32 * LDA + s);
      }
      if constexpr (!TB) {
        b2[s & 1] = *reinterpret_cast<const v2f32*>(bs + 2 * s * LDB);
      } else if (s % 4 == 0) {
#pragma unroll
        for (int j = 0; j < FN; ++j) bg[(s / 4) & 1][j] = *reinterpret_cast<const v4f32*>(bs + j * 32 * LDB + s);
      }
    };
    fetch(0);
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      if (s + 1 < KS) fetch(s + 1);
      if (HOT) {
        if (s >= 1 && s - 1 < NI) {
          const int item = s - 1;
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
        load_global();
      }
      __builtin_amdgcn_sched_barrier(0);       // keep fetch and staging ahead of the MFMAs they overlap with
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
          acc[i][j] = mfma_32x32x2(TA ? a2[s & 1][i] : ag[(s / 4) & 1][i][s % 4], TB ? bg[(s / 4) & 1][j][s % 4] : b2[s & 1][j], acc[i][j]);
    }
    __syncthreads();
  };
  auto store_tile = [&](int tile) {
    const int m0 = (tile / p.tiles_n) * BM, n0 = (tile % p.tiles_n) * BN;
    float* C = p.C + (int64_t)blockIdx.y * p.c_slice;
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int r = acc_row(v, half);
        const int row = m0 + wm * 64 + (TA ? 2 * r + i : 32 * i + r);
        if (row >= p.m) continue;
        if (!TB && p.c_vec2) {          // the lane's two columns 2c, 2c+1 of this row are adjacent in memory
          const int col = n0 + wn * 64 + 2 * l32;
          if (col + 1 < p.n) {
            v2f32* c = reinterpret_cast<v2f32*>(C + (int64_t)row * p.c_rs + col);
            v2f32 val = {acc[i][0][v], acc[i][1][v]};
            *c = p.accumulate ? *c + val : val;
            continue;
          }
        }
#pragma unroll
        for (int j = 0; j < FN; ++j) {
          const int col = n0 + wn * 64 + (TB ? 32 * j + l32 : 2 * l32 + j);
          if (col < p.n) {
            float* c = C + (int64_t)row * p.c_rs + (int64_t)col * p.c_cs;
            *c = p.accumulate ? *c + acc[i][j][v] : acc[i][j][v];
          }
        }
      }
  };

  // the end of a tile: hand-over between the wavefront groups (KG = 2), store, clear
  auto finish_tile = [&](int tile) {
    if constexpr (KG == 2) {
      // The second group of wavefronts hands its accumulators over through LDS (one tile per workgroup here, so
      // the staging buffers are idle after the last step's barrier); the first group adds them to its own and
      // stores: result = first + second.
      float* red = lds + (size_t)wq * (FM * FN * 16 * 64) + lane;
      if (kg == 1) {
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
          for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int q = 0; q < 16; ++q) red[((i * FN + j) * 16 + q) * 64] = acc[i][j][q];
      }
      __syncthreads();
      if (kg == 0) {
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
          for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[i][j][q] += red[((i * FN + j) * 16 + q) * 64];
        store_tile(tile);
      }
    } else {
      store_tile(tile);
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) acc[i][j] = acc_zero();
    }
  };

  // The K range's ragged end (vector kernel only): guarded loads, one buffer, a rolled multiplication loop.
  // Runs after the tile's last whole step (whose barrier left both staging buffers idle).
  auto tail_step = [&](int tile) {
    load_guarded((tile / p.tiles_n) * BM, (tile % p.tiles_n) * BN, k_begin + steps * BK);
    store_lds(0);
    __syncthreads();
    const float* as = TA ? As + (kg * BKG + half) * LDA + wm * 64 + 2 * l32 : As + (wm * 64 + l32) * LDA + kg * BKG + half * (BKG / 2);
    const float* bs = TB ? Bs + (wn * 64 + l32) * LDB + kg * BKG + half * (BKG / 2) : Bs + (kg * BKG + half) * LDB + wn * 64 + 2 * l32;
#pragma unroll 1
    for (int s = 0; s < BKG / 2; ++s) {
      float a[FM], b[FN];
#pragma unroll
      for (int i = 0; i < FM; ++i) a[i] = TA ? as[2 * s * LDA + i] : as[i * 32 * LDA + s];
#pragma unroll
      for (int j = 0; j < FN; ++j) b[j] = TB ? bs[j * 32 * LDB + s] : bs[2 * s * LDB + j];
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) acc[i][j] = mfma_32x32x2(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  };

  int tile = first;
  for (int i = 0; i < my_tiles; ++i, tile += G) {
    if (i == 0 || per_tile) start_stream(tile);
    for (int t = 0; t < steps; ++t) {
      advance_load();                   // the load stream now stands on the step after next (or the last one)
      run_step((per_tile ? t : i * steps + t) & 1, std::integral_constant<bool, !GUARDED>());
    }
    if (!GUARDED && k_tail > 0) tail_step(tile);
    finish_tile(tile);
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
constexpr int kBM = 128, kBN = 128, kBKG = 32;
constexpr int kComputeUnits = 256;
constexpr int kMaxSplit = 16;        // K slices across workgroups

// Wavefront groups per workgroup: with more tiles than compute units two independent four-wavefront workgroups
// share a compute unit; with fewer, one workgroup of eight wavefronts splits every K step inside itself.
static int matmul_groups(int64_t tiles) { return tiles > kComputeUnits ? 1 : 2; }

int matmul_split_k(int64_t m, int64_t n, int64_t k) {
  int64_t tiles = ((m + kBM - 1) / kBM) * ((n + kBN - 1) / kBN);
  if (tiles * 2 > kComputeUnits || k < 1024) return 1;
  int64_t s = kComputeUnits / tiles;
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
  p.tiles_m = tiles_m;
  const int64_t a_span = 1 + (m - 1) * as[0] + (k - 1) * as[1], b_span = 1 + (k - 1) * bs[0] + (n - 1) * bs[1];
  // Vector staging needs each operand contiguous along one index with the other stride a whole
  // number of vectors: A along k (plain) or along m (ta), B along n (plain) or along k (tb).
  const bool ta = as[1] != 1 && as[0] == 1, tb = bs[1] != 1 && bs[0] == 1;
  const int64_t a_ld = ta ? as[1] : as[0], b_ld = tb ? bs[1] : bs[0];
  const bool fast = (ta || as[1] == 1) && (tb || bs[1] == 1) && a_ld >= 0 && b_ld >= 0 && a_ld % 4 == 0 && b_ld % 4 == 0 &&
                    (reinterpret_cast<uintptr_t>(p.A) & 15) == 0 && (reinterpret_cast<uintptr_t>(p.B) & 15) == 0 &&
                    a_span < ((int64_t)1 << 29) && b_span < ((int64_t)1 << 29);
  p.a_bytes = fast ? (uint32_t)(4 * a_span) : 0;
  p.b_bytes = fast ? (uint32_t)(4 * b_span) : 0;

  const int kg = matmul_groups((int64_t)tiles_m * p.tiles_n);
  const int bk = kBKG * kg;            // K elements per step
  p.c_vec2 = 0;
  const int split = matmul_split_k(m, n, k);
  if (split > 1) {
    const size_t need = (size_t)split * (size_t)m * (size_t)n * sizeof(float);
    if (!workspace || workspace_bytes < need)
      return fail(TOFU_ERR_WORKSPACE_TOO_SMALL, "matmul shard needs %zu workspace bytes, got %zu", need, workspace ? workspace_bytes : (size_t)0);
    if (reinterpret_cast<uintptr_t>(workspace) & 15) return fail(TOFU_ERR_INVALID_ARG, "workspace must be 16-byte aligned");
    p.C = static_cast<float*>(workspace);
    p.accumulate = 0;
    p.c_rs = n; p.c_cs = 1; p.c_slice = m * n;
    p.c_vec2 = n % 2 == 0;             // the workspace is dense and 16-byte aligned
    p.k_slice = (int)(((k + split - 1) / split + bk - 1) / bk * bk);
  } else {
    p.C = c_out;
    p.accumulate = accumulate ? 1 : 0;
    p.c_rs = cs[0]; p.c_cs = cs[1]; p.c_slice = 0;
    p.c_vec2 = cs[1] == 1 && cs[0] % 2 == 0 && (reinterpret_cast<uintptr_t>(c_out) & 7) == 0;
    p.k_slice = (int)((k + bk - 1) / bk * bk);
  }
  const int slices = (int)((k + p.k_slice - 1) / p.k_slice);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  // KG = 2: one tile per workgroup (its accumulator hand-over uses the staging buffers).  KG = 1: at most two
  // workgroups per compute unit, each walking its tiles as one stream of K steps.
  const int n_tiles = tiles_m * p.tiles_n;
  auto groups_for = [&](int n_slices) {
    const int slots = 2 * kComputeUnits / n_slices > 0 ? 2 * kComputeUnits / n_slices : 1;
    return kg == 2 ? n_tiles : (n_tiles < slots ? n_tiles : slots);
  };
  auto launched = [&](const char* what) {
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? TOFU_OK : fail(TOFU_ERR_HIP, "matmul %s launch failed: %s", what, hipGetErrorString(e));
  };
  const int n_slices = slices > 0 ? slices : 1;
  void (*kern)(const MatmulArgs);
  if (!fast) kern = kg == 2 ? matmul_kernel<2, false, false, true> : matmul_kernel<1, false, false, true>;   // element loads, any strides
  else if (kg == 2) kern = ta ? (tb ? matmul_kernel<2, true, true, false> : matmul_kernel<2, true, false, false>) : (tb ? matmul_kernel<2, false, true, false> : matmul_kernel<2, false, false, false>);
  else kern = ta ? (tb ? matmul_kernel<1, true, true, false> : matmul_kernel<1, true, false, false>) : (tb ? matmul_kernel<1, false, true, false> : matmul_kernel<1, false, false, false>);
  hipLaunchKernelGGL(kern, dim3(groups_for(n_slices), n_slices), dim3(256 * kg), 0, s, p);
  if ((rc = launched(fast ? "(vector loads)" : "(element loads)"))) return rc;
  hipError_t e;
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
