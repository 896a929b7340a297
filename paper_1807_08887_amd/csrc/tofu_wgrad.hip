// Shard of the weight gradient of a 3x3, stride-1 convolution (arXiv 1807.08887 Sec. 4.2).
//   dw[co,ci,kh,kw] = sum_{n,h,w} dy[n,co,h,w] * x[n,ci,h+kh-pad,w+kw-pad],  x = 0 outside the tensor.
// C_out and C_in are output dimensions of this operator (Case-1: shards write disjoint blocks of
// dw); the batch index is a reduction index (Case-2: a batch shard produces a full-size PARTIAL
// dw that tofu_partition_reduce sums with the other workers' partials).
//
// Kernel: GEMM  [co] x [(ci,tap)] over K = (n,h,w) on fp32 MFMA 32x32x2 tiles.
//   * A workgroup owns BM output channels x 32 input channels x all 9 taps; wavefront w owns 32 of
//     the output channels and nine 32x32 accumulator blocks, one per tap (lane = input channel).
//   * One step of the K loop is up to 32 output positions of one image: one output row (or a
//     chunk of at most 32 columns of a wider row), or several whole rows of a narrow image.
//     dy[n, co tile, those positions] is staged k-major (Ds[position][co]) and the x rows they
//     touch, x[n, ci tile, h-pad .. h+R-1-pad+2, :], are staged with their zero border, so the
//     nine taps are nine shifted reads of the same staged rows.  One MFMA contracts two
//     adjacent output columns (lanes 0-31: w, lanes 32-63: w+1).
//   * Load balance: the work is T tiles x (NB images x their row groups) units, one unit being the
//     output rows one step takes (or the chunks of one wide row).  400 tiles cannot fill 512 workgroup
//     slots evenly, so the units are dealt to 512 workgroups as tofu_balance.h describes: a
//     workgroup of its own for the first part of every tile, the tails shared out among the rest,
//     every workgroup the same number of steps to within a few, and the workgroups that run side
//     by side at the same (image, row) at the same time.  Every piece goes tap-major to a workspace
//     slot and a second kernel sums each tile's slots in the order of the units (fixed, no atomics)
//     and restores the [co][ci][kh][kw] layout.  Whole waves of 512 tiles (and every tile of a
//     single-image shard) run one workgroup per tile in a launch of their own and write dw directly.
//   * Tile order: channel tile rows are numbered in panels of kWgradPanel, output channel tile fastest
//     inside a panel, so that the 64 workgroups of one XCD are 4 output x 16 input channel tiles,
//     which share 4 dy rows and 16 x rows per step through that XCD's L2.
#include <hip/hip_runtime.h>

#include "tofu_balance.h"
#include "tofu_internal.h"
#include "tofu_mfma.h"

namespace tofu {

struct WgradArgs {
  const float* x;    // element at the low corner of the (clipped) input box
  const float* dy;   // element (n_lo, co_lo, 0, 0)
  float* out;        // dw element (co_lo, ci_lo, 0, 0)
  int accumulate;    // 1: the shard's sum is added to what the output box holds
  float* slots;      // workspace: partial tiles of kSlotFloats floats (slot numbering: tofu_balance.h)
  int64_t xs[4], ds[4], os[4];   // element strides: x (n,c,h,w), dy (n,co,h,w), out (co,ci,kh,kw)
  uint32_t x_bytes, dy_bytes;    // bytes spanned by the two input boxes (buffer bounds, fast path)
  int NB, CO, CI;    // images, output channels, input channels of the shard
  int HO, WO;        // output rows / columns
  int IH, IW;        // rows / columns of the clipped input box
  int plh, plw;      // zero rows / columns in front of the input box
  int tiles_m, tiles_n;
  int tile0, n_tiles;  // the launch covers the tiles [tile0, tile0 + n_tiles) of the tile order
  Balance bal;       // balanced launches: how the units of those tiles are dealt to bal.groups workgroups
  int CW;            // output columns per K step (<= 32, multiple of 4 unless WO itself is not)
  int chunks;        // column chunks per output row
  int vec;           // 1: rows of dy are contiguous and 16-byte aligned -> vector loads (generic path)
};

// LDS geometry is fixed so that every staging index splits with compile-time divisors.
constexpr int kKR = 32;              // dy positions per K step (a chunk of one output row)
constexpr int kLDW = kKR + 2;        // staged x columns per row: chunk widened by the filter window
constexpr int kPLX = 3 * kLDW + 3;
constexpr int kWgradPanel = 4;       // output-channel tiles per panel of the tile order
constexpr int kSlotFloats = 9 * 128 * 32;   // one partial tile in the workspace: [tap][128 co][32 ci]   // staged floats per input channel; odd -> 32 channels hit 32 banks

// Tile number -> (input-channel tile, output-channel tile): panels of kWgradPanel output-channel tiles,
// the output-channel tile fastest inside a panel.
__host__ __device__ __forceinline__ void wgrad_decode_tile(int tile, int tiles_m, int tiles_n, int& tile_n, int& tile_m) {
  const int panel_tiles = kWgradPanel * tiles_n;
  const int panel = tile / panel_tiles, rem = tile - panel * panel_tiles;
  const int rows = tiles_m - panel * kWgradPanel < kWgradPanel ? tiles_m - panel * kWgradPanel : kWgradPanel;
  tile_n = rem / rows;
  tile_m = panel * kWgradPanel + (rem - tile_n * rows);
}

// FAST: dy rows are whole aligned vectors (or one of the narrow-image forms below applies) and
// every operand offset fits 32 bits.  Then each lane's staging addresses are fixed byte offsets,
// a step only changes a scalar offset, and all padding comes from out-of-range buffer reads
// selected by one comparison per item -- no branches, no per-step index arithmetic.  Rows wider
// than 32 columns are cut into equal chunks, one chunk per step.  Otherwise a generic guarded
// path is used.
// BALANCED: the workgroup walks a range of units and writes every segment to a workspace slot
// (even a whole tile: one simple epilogue keeps the register count down); otherwise a workgroup
// is one whole tile and writes dw directly.
// R, DVEC (with KPT): narrow images put R whole output rows into one step, R * CWE <= 32 positions
// with CWE = 2 * KPT / R columns per row (the width rounded up to even; a spare column is zeros).
// DVEC = 4: the R rows are one contiguous, 16-byte aligned run of dy (CWE == WO, dense rows);
// DVEC = 1: dy is loaded element by element (any width, any alignment).
// CHUNKED: output rows are wider than 32 columns and a step is one chunk of a row; which staged
// columns lie outside the image then depends on the step (else it is folded into the offsets).
template <int BM, int BCI, bool FAST, bool BALANCED, int KPT = 0, int R = 1, int DVEC = 4, bool CHUNKED = false>
__global__ void __launch_bounds__(64 * (BM / 32), FAST ? 2 : 1) wgrad_kernel(const WgradArgs p) {
  static_assert(!CHUNKED || (FAST && R == 1), "chunks are cut from single rows");
  static_assert(KPT == 0 || (FAST && KPT % 2 == 0 && KPT >= 4), "a compile-time column-pair count needs the fast staging maps");
  static_assert(R == 1 || (KPT > 0 && (2 * KPT) % R == 0 && (2 * KPT / R) % 2 == 0), "rows per step need a compile-time even row width");
  constexpr int NW = BM / 32, NT = 64 * NW, LDD = BM + 2;
  constexpr int CWE = R == 1 ? kKR : 2 * KPT / R;   // staged dy columns per row
  constexpr int LDX = R == 1 ? kLDW : CWE + 2;      // staged x columns per row (row widened by the filter window)
  constexpr int XROWS = R + 2;                      // staged x rows per step
  constexpr int D_ITEMS = BM * (kKR / 4), X_ITEMS = BCI * 3 * kLDW;
  constexpr int DJ = (D_ITEMS + NT - 1) / NT, XJ = (X_ITEMS + NT - 1) / NT;
  constexpr int TPC = NT / BCI;                 // threads that stage one input channel (fast path)
  constexpr int XF = (XROWS * LDX + TPC - 1) / TPC;  // elements per such thread
  static_assert(BCI == 32 && NT % BCI == 0 && D_ITEMS % NT == 0, "staging maps assume 32 input channels and whole passes");
  static_assert(XF * TPC <= kPLX, "idle fast-path slots must land in the plane's padding");
  __shared__ float Ds[2][kKR][LDD];        // dy chunk, k-major: Ds[column][co]
  __shared__ float Xs[2][BCI * kPLX];      // x rows h-pad..h-pad+2 of the chunk, zero border included

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, half = lane >> 5;
  // consecutive workgroup numbers (which share operand rows) stay on one XCD
  const int total = BALANCED ? p.bal.groups : p.n_tiles;
  const int per_xcd = (total + 7) / 8;
  const int g = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (g >= total) return;
  const int HG = (p.HO + R - 1) / R;             // row groups (= units) per image: groups of R output rows
  const int UPT = p.NB * HG;                     // units per tile
  const int KP = (p.CW + 1) / 2;             // column pairs contracted per step
  const __amdgpu_buffer_rsrc_t d_rsrc = make_rsrc(p.dy, p.dy_bytes);
  // the x buffer starts plh rows and plw columns before the box, so that staged element (r, c) of a
  // step has the non-negative offset r * xs2 + c * xs3; the border itself is never read (predicated)
  const int64_t x_back = (int64_t)p.plh * p.xs[2] + (int64_t)p.plw * p.xs[3];
  const __amdgpu_buffer_rsrc_t x_rsrc = make_rsrc(p.x - x_back, p.x_bytes + 4u * (uint32_t)x_back);
  const int d_row = tid / (kKR / 4), d_q = tid % (kKR / 4);
  const int x_ci = tid / TPC, x_sub = tid % TPC;

  BalanceWalk walk;
  if (BALANCED) {
    walk = balance_walk(p.bal, UPT, g);
    if (walk.count == 0) return;
  }
  const int n_segments = BALANCED ? walk.count : 1;
  for (int seg_i = 0; seg_i < n_segments; ++seg_i) {
  // ---- one segment: row groups [r_begin, r_end) of one tile, numbered image-major (image n, group h -> n * HG + h) ----
  int tile = p.tile0 + g, r_begin = 0, r_end = UPT, slot = 0;
  if (BALANCED) {
    const BalanceSegment seg = balance_segment(walk, seg_i);
    tile = p.tile0 + seg.tile; r_begin = seg.begin; r_end = seg.end; slot = seg.slot;
  }
  int tile_n, tile_m;
  wgrad_decode_tile(tile, p.tiles_m, p.tiles_n, tile_n, tile_m);
  const int m0 = tile_m * BM, c0 = tile_n * BCI;
  const int steps = (r_end - r_begin) * p.chunks;

  // ---- fast-path staging maps ----
  // dy: thread -> (row = tid/8 + 32*j, columns 4*(tid%8) .. +3); x: thread -> (channel tid/TPC, elements tid%TPC + TPC*j)
  constexpr int DN = DVEC == 4 ? 1 : 4;          // loads per dy item
  uint32_t d_voff[DJ][DN], x_voff[XF];
  const int d_r = (4 * d_q) / CWE;               // staged row of this thread's four dy positions (element loads)
  if (FAST) {
#pragma unroll
    for (int j = 0; j < DJ; ++j) {
      const int row = d_row + j * (NT / (kKR / 4));
      if (DVEC == 4) {
        // positions 4*d_q .. +3 of the step's run of R * CWE contiguous floats (one row when R == 1)
        const bool ok = m0 + row < p.CO && 4 * d_q < (R == 1 ? p.CW : R * CWE);
        d_voff[j][0] = ok ? 4u * (uint32_t)((int64_t)(m0 + row) * p.ds[1] + 4 * d_q) : kNoOffset;
      } else {
#pragma unroll
        for (int jj = 0; jj < DN; ++jj) {
          const int c = (4 * d_q + jj) % CWE;
          const bool ok = m0 + row < p.CO && d_r < R && c < p.WO;
          d_voff[j][jj] = ok ? 4u * (uint32_t)((int64_t)(m0 + row) * p.ds[1] + (int64_t)d_r * p.ds[2] + c) : kNoOffset;
        }
      }
    }
#pragma unroll
    for (int j = 0; j < XF; ++j) {
      const int e = x_sub + TPC * j, r = e / LDX, c = e - r * LDX;
      const bool ok = e < XROWS * LDX && c0 + x_ci < p.CI && (CHUNKED || (unsigned)(c - p.plw) < (unsigned)p.IW);
      // offsets are relative to input row (oh - plh) and input column (chunk start - plw)
      x_voff[j] = ok ? 4u * (uint32_t)((int64_t)(c0 + x_ci) * p.xs[1] + (int64_t)r * p.xs[2] + (int64_t)c * p.xs[3]) : kNoOffset;
    }
  }

  v4f32 rd[DJ];
  float rx[FAST ? XF : XJ];
  // fast-path loads of one staging item for the step whose first output row is oh
  auto load_d = [&](int j, uint32_t d_soff, int oh, int cw0) {
    if (DVEC == 4) {
      const bool col_ok = !CHUNKED || cw0 + 4 * d_q < p.WO;   // the last chunk of a row may be short (whole vectors)
      rd[j] = buf_load4(d_rsrc, col_ok ? d_voff[j][0] : kNoOffset, d_soff);
    } else {
      const bool row_ok = oh + d_r < p.HO;       // the last group of rows of an image may be short
#pragma unroll
      for (int jj = 0; jj < DN; ++jj) rd[j][jj] = buf_load(d_rsrc, row_ok ? d_voff[j][jj] : kNoOffset, d_soff);
    }
  };
  auto load_x = [&](int j, uint32_t x_soff, int oh, int cw0) {
    const int e = x_sub + TPC * j;
    const int r = R == 1 ? (e >= LDX) + (e >= 2 * LDX) : e / LDX;   // staged row of this element
    bool ok = (unsigned)(oh + r - p.plh) < (unsigned)p.IH;
    if (CHUNKED) ok = ok && (unsigned)(cw0 + e - r * LDX - p.plw) < (unsigned)p.IW;
    rx[j] = buf_load(x_rsrc, ok ? x_voff[j] : kNoOffset, x_soff);
  };
  auto load_global = [&](int step) {
    const int sr = step / p.chunks, chunk = step - sr * p.chunks;
    const int row_id = r_begin + sr;
    const int n = row_id / HG, oh = (row_id - n * HG) * R;   // image and first output row of the step
    if (FAST) {
      const int cw0 = chunk * p.CW;
      const uint32_t d_soff = 4u * (uint32_t)((int64_t)n * p.ds[0] + (int64_t)oh * p.ds[2] + cw0);
      const uint32_t x_soff = 4u * (uint32_t)((int64_t)n * p.xs[0] + (int64_t)oh * p.xs[2] + (int64_t)cw0 * p.xs[3]);
#pragma unroll
      for (int j = 0; j < DJ; ++j) load_d(j, d_soff, oh, cw0);
#pragma unroll
      for (int j = 0; j < XF; ++j) load_x(j, x_soff, oh, cw0);
      return;
    }
    const int cw0 = chunk * p.CW;
    const float* db = p.dy + (int64_t)n * p.ds[0] + (int64_t)m0 * p.ds[1] + (int64_t)oh * p.ds[2] + (int64_t)cw0 * p.ds[3];
    const float* xb = p.x + (int64_t)n * p.xs[0] + (int64_t)c0 * p.xs[1];
#pragma unroll
    for (int j = 0; j < DJ; ++j) {
      const int idx = tid + j * NT, row = idx / (kKR / 4), q = idx % (kKR / 4);
      const bool row_ok = m0 + row < p.CO;
      const int col = 4 * q;                   // first of four columns, relative to the chunk
      if (p.vec && row_ok && col + 3 < p.CW && cw0 + col + 3 < p.WO) {
        rd[j] = *reinterpret_cast<const v4f32*>(db + (int64_t)row * p.ds[1] + col);
      } else {
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
          const bool ok = row_ok && col + jj < p.CW && cw0 + col + jj < p.WO;
          rd[j][jj] = ok ? db[(int64_t)row * p.ds[1] + (int64_t)(col + jj) * p.ds[3]] : 0.f;
        }
      }
    }
#pragma unroll
    for (int j = 0; j < (FAST ? 0 : XJ); ++j) {
      const int idx = tid + j * NT, ci_l = idx / (3 * kLDW), rem = idx % (3 * kLDW), r = rem / kLDW, c = rem % kLDW;
      const int ih = oh + r - p.plh, iw = cw0 + c - p.plw;
      const bool ok = idx < X_ITEMS && c0 + ci_l < p.CI && ih >= 0 && ih < p.IH && iw >= 0 && iw < p.IW;
      rx[j] = ok ? xb[(int64_t)ci_l * p.xs[1] + (int64_t)ih * p.xs[2] + (int64_t)iw * p.xs[3]] : 0.f;
    }
  };
  auto store_lds = [&](int buf) {
#pragma unroll
    for (int j = 0; j < DJ; ++j) {
      const int row = d_row + j * (NT / (kKR / 4));
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) Ds[buf][4 * d_q + jj][row] = rd[j][jj];
    }
    if (FAST) {
#pragma unroll
      for (int j = 0; j < XF; ++j) Xs[buf][x_ci * kPLX + x_sub + TPC * j] = rx[j];   // slots past 3*kLDW fall in the plane's padding
    } else {
#pragma unroll
      for (int j = 0; j < (FAST ? 0 : XJ); ++j) {
        const int idx = tid + j * NT, ci_l = idx / (3 * kLDW), rem = idx % (3 * kLDW);
        if (idx < X_ITEMS) Xs[buf][ci_l * kPLX + rem] = rx[j];
      }
    }
  };

  acc16 acc[9];
#pragma unroll
  for (int t = 0; t < 9; ++t) acc[t] = acc_zero();

  if constexpr (KPT > 0) {
    // Column-pair count known at compile time (KPT == (CW + 1) / 2 rounded up to even): the step
    // is fully unrolled and the staging work of a lane (DJ dy items, XF x items) is dealt out
    // over the fetch slots of the step, IPS items per slot, the last two slots left empty.  An
    // item writes the registers loaded for step t+1 to the idle LDS buffer and reloads them for
    // step t+2 at once, so no MFMA waits behind a block of staging instructions and every load
    // has a whole step to land.
    constexpr int NI = DJ + XF, IPS = (NI + KPT - 3) / (KPT - 2);
    load_global(0);
    store_lds(0);
    load_global(min(1, steps - 1));
    __syncthreads();
    for (int t = 0; t < steps; ++t) {
      const int buf = t & 1;
      const int nxt = min(t + 2, steps - 1);
      const int sr = nxt / p.chunks, cw0 = (nxt - sr * p.chunks) * p.CW;
      const int row_id = r_begin + sr;
      const int n = row_id / HG, oh = (row_id - n * HG) * R;
      const uint32_t d_soff = 4u * (uint32_t)((int64_t)n * p.ds[0] + (int64_t)oh * p.ds[2] + cw0);
      const uint32_t x_soff = 4u * (uint32_t)((int64_t)n * p.xs[0] + (int64_t)oh * p.xs[2] + (int64_t)cw0 * p.xs[3]);
      const float* dsm = &Ds[buf][half][wave * 32 + l32];
      const float* xsm = &Xs[buf][l32 * kPLX + half];
      auto fetch = [&](int kp, float& a, float (&b)[9]) {
        a = dsm[2 * kp * LDD];
#pragma unroll
        for (int tap = 0; tap < 9; ++tap) b[tap] = xsm[((2 * kp) / CWE) * LDX + (2 * kp) % CWE + (tap / 3) * LDX + tap % 3];
      };
      auto fma9 = [&](float a, const float (&b)[9]) {
#pragma unroll
        for (int tap = 0; tap < 9; ++tap) acc[tap] = mfma_32x32x2(a, b[tap], acc[tap]);
      };
      auto stage = [&](int slot) {
#pragma unroll
        for (int item = slot * IPS; item < (slot + 1) * IPS && item < NI; ++item) {
          if (item < DJ) {
            const int row = d_row + item * (NT / (kKR / 4));
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) Ds[buf ^ 1][4 * d_q + jj][row] = rd[item][jj];
            load_d(item, d_soff, oh, cw0);
          } else {
            const int j = item - DJ;
            Xs[buf ^ 1][x_ci * kPLX + x_sub + TPC * j] = rx[j];
            load_x(j, x_soff, oh, cw0);
          }
        }
      };
      float a0, a1, b0[9], b1[9];
      fetch(0, a0, b0);
#pragma unroll
      for (int kp = 0; kp < KPT; kp += 2) {
        fetch(kp + 1, a1, b1);
        stage(kp);
        __builtin_amdgcn_sched_barrier(0);         // keep fetch and staging ahead of the MFMAs they overlap with
        fma9(a0, b0);
        fetch(kp + 2 < KPT ? kp + 2 : KPT - 1, a0, b0);   // past the end: a harmless re-read
        stage(kp + 1);
        __builtin_amdgcn_sched_barrier(0);
        fma9(a1, b1);
      }
      __syncthreads();
    }
  } else {
    load_global(0);
    store_lds(0);
    __syncthreads();
    // Column pairs per step, rounded up to even (the staged columns past CW are zeros) so that the
    // two operand register sets below alternate without a remainder case.
    const int KPE = (KP + 1) & ~1;
    const int half_way = (KPE / 2) & ~1;
    for (int t = 0; t < steps; ++t) {
      const int buf = t & 1;
      // Branch-free body (the compiler can then count outstanding LDS operations exactly): the
      // last step stages its own tiles again into the idle buffer.
      load_global(min(t + 1, steps - 1));
      const float* dsm = &Ds[buf][half][wave * 32 + l32];
      const float* xsm = &Xs[buf][l32 * kPLX + half];
      // Two operand register sets alternate: while the nine MFMAs of one column pair run, the
      // operands of the next pair are fetched into the other set (no register copies).
      auto fetch = [&](int kp, float& a, float (&b)[9]) {
        a = dsm[2 * kp * LDD];
  #pragma unroll
        for (int tap = 0; tap < 9; ++tap) b[tap] = xsm[2 * kp + (tap / 3) * kLDW + tap % 3];
      };
      auto fma9 = [&](float a, const float (&b)[9]) {
  #pragma unroll
        for (int tap = 0; tap < 9; ++tap) acc[tap] = mfma_32x32x2(a, b[tap], acc[tap]);
      };
      float a0, a1, b0[9], b1[9];
      fetch(0, a0, b0);
      for (int kp = 0; kp < KPE; kp += 2) {
        // the next step's tiles go to the other LDS buffer half-way through, in the MFMA shadow
        if (kp == half_way) store_lds(buf ^ 1);
        fetch(kp + 1, a1, b1);
        __builtin_amdgcn_sched_barrier(0);           // keep each fetch ahead of the MFMAs it overlaps with
        fma9(a0, b0);
        fetch(min(kp + 2, KPE - 1), a0, b0);         // past the end: a harmless re-read
        __builtin_amdgcn_sched_barrier(0);
        fma9(a1, b1);
      }
      __syncthreads();
    }
  }

  if (BALANCED) {
    // slot [tap][co_local][ci_local]: a lane row of 32 input channels is one 128-byte store
    float* o = p.slots + (int64_t)slot * kSlotFloats + (wave * 32 + 4 * half) * BCI + l32;
#pragma unroll
    for (int tap = 0; tap < 9; ++tap)
#pragma unroll
      for (int v = 0; v < 16; ++v) o[(tap * BM + 8 * (v >> 2) + (v & 3)) * BCI] = acc[tap][v];
  } else {
    const int ci = c0 + l32;
#pragma unroll
    for (int tap = 0; tap < 9; ++tap)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int co = m0 + wave * 32 + acc_row(v, half);
        if (co < p.CO && ci < p.CI) {
          float* o = p.out + (int64_t)co * p.os[0] + (int64_t)ci * p.os[1] + (tap / 3) * p.os[2] + (tap % 3) * p.os[3];
          *o = p.accumulate ? *o + acc[tap][v] : acc[tap][v];
        }
      }
  }
  __syncthreads();   // the next segment's prologue overwrites LDS buffer 0
  }  // segments
}

// Sums every tile's pieces (workspace slots) in the order of their units and writes
// dw[co][ci][kh][kw], or with `accumulate` adds that sum to what dw holds.  One thread per (co, ci): its nine
// reads per slot are coalesced across lanes (ci fastest).  A workgroup handles eight output-channel rows of a
// tile at a time.  DENSE (dw rows of a (co) are contiguous over (ci, kh, kw) and 16-byte aligned): the sums
// go through LDS and leave as 16-byte vectors, 1152 contiguous bytes per row; otherwise every thread writes
// its nine values where the strides put them.
template <bool DENSE>
__global__ void __launch_bounds__(256) wgrad_segment_sum_kernel(float* __restrict__ dw, int64_t s_co, int64_t s_ci, int64_t s_kh, int64_t s_kw,
                                                                 const float* __restrict__ slots, const Balance bal, int UPT, int tile0,
                                                                 int tiles_m, int tiles_n, int CO, int CI, int accumulate) {
  constexpr int BM = 128, BCI = 32, ROWS = 256 / BCI, ROW = BCI * 9;
  __shared__ __align__(16) float tile_s[DENSE ? ROWS * (ROW + 4) : 4];
  const int64_t items = (int64_t)bal.n * BM * BCI;   // the balanced tiles [tile0, tile0 + bal.n): a multiple of the block size
  for (int64_t i0 = (int64_t)blockIdx.x * blockDim.x; i0 < items; i0 += (int64_t)gridDim.x * blockDim.x) {
    const int64_t i = i0 + threadIdx.x;
    const int tile = (int)(i / (BM * BCI)), local = (int)(i % (BM * BCI)), co_l = local / BCI, ci_l = local % BCI;
    int tile_n, tile_m;
    wgrad_decode_tile(tile0 + tile, tiles_m, tiles_n, tile_n, tile_m);
    const int co = tile_m * BM + co_l, ci = tile_n * BCI + ci_l;
    const bool live = co < CO && ci < CI;
    float acc[9];
#pragma unroll
    for (int tap = 0; tap < 9; ++tap) acc[tap] = 0.f;
    if (live)
      balance_for_each_slot(bal, UPT, tile, [&](int slot) {
        const float* sl = slots + (int64_t)slot * kSlotFloats + co_l * BCI + ci_l;
#pragma unroll
        for (int tap = 0; tap < 9; ++tap) acc[tap] += sl[tap * BM * BCI];
      });
    if constexpr (DENSE) {
      const int r = threadIdx.x / BCI;
#pragma unroll
      for (int tap = 0; tap < 9; ++tap) tile_s[r * (ROW + 4) + ci_l * 9 + tap] = acc[tap];
      __syncthreads();
      // the block's eight rows start at output channel co - r; every row holds the tile's input channels x 9 taps
      const int co0 = co - r, c0 = tile_n * BCI;
      const int valid = (CI - c0 < BCI ? CI - c0 : BCI) * 9;            // floats of a row that lie inside the box
      for (int v = threadIdx.x; v < ROWS * (ROW / 4); v += 256) {
        const int row = v / (ROW / 4), q = v - row * (ROW / 4);
        if (co0 + row >= CO || 4 * q >= valid) continue;
        const float* src = &tile_s[row * (ROW + 4) + 4 * q];
        float* o = dw + (int64_t)(co0 + row) * s_co + (int64_t)c0 * 9 + 4 * q;
        if (4 * q + 3 < valid) {
          v4f32 val = *reinterpret_cast<const v4f32*>(src);
          if (accumulate) {
            const v4f32 old = *reinterpret_cast<const v4f32*>(o);
            val = old + val;
          }
          *reinterpret_cast<v4f32*>(o) = val;
        } else {
          for (int e = 0; 4 * q + e < valid; ++e) o[e] = accumulate ? o[e] + src[e] : src[e];
        }
      }
      __syncthreads();
    } else {
      if (!live) continue;
#pragma unroll
      for (int tap = 0; tap < 9; ++tap) {
        float* o = dw + co * s_co + ci * s_ci + (tap / 3) * s_kh + (tap % 3) * s_kw;
        *o = accumulate ? *o + acc[tap] : acc[tap];
      }
    }
  }
}

constexpr int gBM = 128, gBCI = 32;
constexpr int kWgradSlots = 512;       // two resident workgroups on each of the 256 compute units

constexpr int kWgradSegmentCost = 1;   // units a workgroup loses per segment (set-up, pipeline fill, slot write)

// Tiles of a shard that are launched one workgroup each (whole waves of kWgradSlots; all of them for a single
// image or when the last wave is nearly full); the others, the last `tiles - whole`, are balanced.
static int64_t wgrad_whole_tiles(int64_t tiles, int64_t nb) {
  const int64_t rest = tiles % kWgradSlots;
  return (nb < 2 || rest * 32 >= kWgradSlots * 31) ? tiles : tiles - rest;
}

// Rows one step takes for an image of wo columns in the fastest form that may apply (see shard_wgrad).
static int wgrad_max_rows_per_step(int64_t ho, int64_t wo) { return wo == 7 ? 4 : ((wo == 14 || wo == 16) && ho % 2 == 0) ? 2 : 1; }

// Workspace for a shard of co x ci output channels, nb images of ho x wo outputs: enough for whichever
// form of the kernel (rows per step) the operands' strides and alignment allow.
size_t wgrad_workspace_bytes(int64_t co, int64_t ci, int64_t nb, int64_t ho, int64_t wo) {
  const int64_t tiles = ((co + gBM - 1) / gBM) * ((ci + gBCI - 1) / gBCI);
  const int64_t rest = tiles - wgrad_whole_tiles(tiles, nb);
  if (rest == 0) return 0;
  int64_t slots = 0;
  for (int rows = 1; rows <= wgrad_max_rows_per_step(ho, wo); rows *= 2) {
    const int64_t upt = nb * ((ho + rows - 1) / rows);
    const int64_t n = balance_slots(balance_plan(rest, upt, kWgradSlots, kWgradSegmentCost), (int)upt);
    if (n > slots) slots = n;
  }
  return (size_t)slots * kSlotFloats * sizeof(float);
}

static int shard_wgrad(const tofu_op_desc_t* op, const tofu_split_t* splits, int32_t nsplits, const tofu_tensor_t* x,
                       const tofu_tensor_t* dy, const tofu_tensor_t* dw, void* workspace, size_t workspace_bytes, void* hip_stream,
                       bool accumulate) {
  if (!op || op->kind != TOFU_OP_CONV2D_WGRAD) return fail(TOFU_ERR_INVALID_ARG, "operator description is not a conv2d weight gradient");
  tofu_region_t out_box, in_boxes[2];
  int64_t pad_lo[2], pad_hi[2];
  int32_t partial = 0;
  int rc = tofu_op_regions(op, splits, nsplits, &out_box, in_boxes, pad_lo, pad_hi, &partial);
  if (rc) return rc;
  if (op->KH != 3 || op->KW != 3 || op->stride != 1 || op->pad > 1)
    return fail(TOFU_ERR_UNSUPPORTED, "conv2d weight-gradient kernels implement KH = KW = 3, stride 1, pad 0 or 1");
  if ((rc = check_tensor("x", x, 4, &in_boxes[0]))) return rc;
  if ((rc = check_tensor("dy", dy, 4, &in_boxes[1]))) return rc;
  if ((rc = check_tensor("dw", dw, 4, &out_box))) return rc;
  if (volume(&out_box) == 0) return TOFU_OK;

  int64_t xs[4], ds[4], os[4];
  effective_strides(x, xs);
  effective_strides(dy, ds);
  effective_strides(dw, os);
  WgradArgs p;
  p.x = element_ptr(x, xs, in_boxes[0].lo);
  p.dy = element_ptr(dy, ds, in_boxes[1].lo);
  float* dw_out = const_cast<float*>(element_ptr(dw, os, out_box.lo));
  for (int d = 0; d < 4; ++d) { p.xs[d] = xs[d]; p.ds[d] = ds[d]; p.os[d] = os[d]; }
  const int64_t CO = out_box.hi[0] - out_box.lo[0], CI = out_box.hi[1] - out_box.lo[1];
  const int64_t NB = in_boxes[0].hi[0] - in_boxes[0].lo[0];
  const int64_t HO = in_boxes[1].hi[2] - in_boxes[1].lo[2], WO = in_boxes[1].hi[3] - in_boxes[1].lo[3];
  if (CO >= (1 << 30) || CI >= (1 << 30) || NB * HO >= (1 << 30) || WO >= (1 << 20))
    return fail(TOFU_ERR_UNSUPPORTED, "conv2d weight-gradient shard extent too large");
  p.NB = (int)NB; p.CO = (int)CO; p.CI = (int)CI; p.HO = (int)HO; p.WO = (int)WO;
  p.IH = (int)(in_boxes[0].hi[2] - in_boxes[0].lo[2]);
  p.IW = (int)(in_boxes[0].hi[3] - in_boxes[0].lo[3]);
  p.plh = (int)pad_lo[0]; p.plw = (int)pad_lo[1];
  p.tiles_m = (int)((CO + gBM - 1) / gBM);
  p.tiles_n = (int)((CI + gBCI - 1) / gBCI);
  // cut an output row into equal chunks of at most 32 columns, whole 16-byte vectors when possible
  p.chunks = (int)((WO + kKR - 1) / kKR);
  p.CW = (int)((WO + p.chunks - 1) / p.chunks);
  if (p.chunks > 1) p.CW = (p.CW + 3) / 4 * 4;
  p.vec = ds[3] == 1 && ds[1] % 4 == 0 && ds[2] % 4 == 0 && ds[0] % 4 == 0 && (reinterpret_cast<uintptr_t>(p.dy) & 15) == 0;
  const int NT = 64 * (gBM / 32);
  // fast path: buffer loads with 32-bit byte offsets from the boxes' low corners
  int64_t x_span = 1, d_span = 1;
  bool nonneg = true;
  for (int d = 0; d < 4; ++d) {
    nonneg = nonneg && xs[d] >= 0 && ds[d] >= 0;
    x_span += (in_boxes[0].hi[d] - in_boxes[0].lo[d] - 1) * xs[d];
    d_span += (in_boxes[1].hi[d] - in_boxes[1].lo[d] - 1) * ds[d];
  }
  const bool fits = nonneg && x_span + p.plh * xs[2] + p.plw * xs[3] < ((int64_t)1 << 29) && d_span < ((int64_t)1 << 29);
  // one output row (or one chunk of at most 32 columns of it) per step, rows of whole aligned vectors
  const bool fast_row = fits && p.vec && WO % 4 == 0;
  // narrow images: several whole rows per step.  14 or 16 wide: two dense rows are one aligned run of
  // 28 or 32 floats; 7 wide: four rows, element loads (rows padded to 8 positions in LDS)
  const bool two_rows = fits && HO % 2 == 0 && ds[3] == 1 && ds[2] == WO && ds[1] % 4 == 0 && ds[0] % 4 == 0 &&
                        (reinterpret_cast<uintptr_t>(p.dy) & 15) == 0;
  const bool fast_2x14 = two_rows && WO == 14, fast_2x16 = two_rows && WO == 16;
  const bool fast_4x7 = fits && WO == 7 && ds[3] == 1;
  const bool fast = fast_row || fast_2x14 || fast_2x16 || fast_4x7;
  p.x_bytes = fast ? (uint32_t)(4 * x_span) : 0;
  p.dy_bytes = fast ? (uint32_t)(4 * d_span) : 0;
  const int64_t rows_per_step = !fast ? 1 : (fast_2x14 || fast_2x16) ? 2 : fast_4x7 ? 4 : 1;   // the R of the kernel picked below
  const int64_t tiles = (int64_t)p.tiles_m * p.tiles_n, UPT = NB * ((HO + rows_per_step - 1) / rows_per_step);
  const int64_t whole = wgrad_whole_tiles(tiles, NB), rest = tiles - whole;
  p.bal = Balance{0, 0, 0, 0, 0, 0};
  if (rest > 0) p.bal = balance_plan(rest, UPT, kWgradSlots, kWgradSegmentCost);
  p.out = dw_out;
  p.accumulate = accumulate ? 1 : 0;
  p.slots = static_cast<float*>(workspace);
  const size_t need = rest > 0 ? (size_t)balance_slots(p.bal, (int)UPT) * kSlotFloats * sizeof(float) : 0;
  if (need > 0 && (!workspace || workspace_bytes < need))
    return fail(TOFU_ERR_WORKSPACE_TOO_SMALL, "conv2d weight-gradient shard needs %zu workspace bytes, got %zu", need, workspace ? workspace_bytes : (size_t)0);
  // fast shards of the common widths run the fully unrolled step (column pairs rounded up to even)
  const int kpe = ((p.CW + 1) / 2 + 1) & ~1;
  void (*kern_balanced)(const WgradArgs) =
             !fast                 ? wgrad_kernel<gBM, gBCI, false, true>
           : fast_2x14           ? wgrad_kernel<gBM, gBCI, true, true, 14, 2, 4>
           : fast_2x16           ? wgrad_kernel<gBM, gBCI, true, true, 16, 2, 4>
           : fast_4x7            ? wgrad_kernel<gBM, gBCI, true, true, 16, 4, 1>
           : p.chunks > 1        ? (kpe == 14 ? wgrad_kernel<gBM, gBCI, true, true, 14, 1, 4, true> : wgrad_kernel<gBM, gBCI, true, true, 0, 1, 4, true>)
           : kpe == 8            ? wgrad_kernel<gBM, gBCI, true, true, 8>
           : kpe == 14           ? wgrad_kernel<gBM, gBCI, true, true, 14>
           : kpe == 16           ? wgrad_kernel<gBM, gBCI, true, true, 16>
                                 : wgrad_kernel<gBM, gBCI, true, true>;
  void (*kern_whole)(const WgradArgs) =
             !fast                 ? wgrad_kernel<gBM, gBCI, false, false>
           : fast_2x14           ? wgrad_kernel<gBM, gBCI, true, false, 14, 2, 4>
           : fast_2x16           ? wgrad_kernel<gBM, gBCI, true, false, 16, 2, 4>
           : fast_4x7            ? wgrad_kernel<gBM, gBCI, true, false, 16, 4, 1>
           : p.chunks > 1        ? (kpe == 14 ? wgrad_kernel<gBM, gBCI, true, false, 14, 1, 4, true> : wgrad_kernel<gBM, gBCI, true, false, 0, 1, 4, true>)
           : kpe == 8            ? wgrad_kernel<gBM, gBCI, true, false, 8>
           : kpe == 14           ? wgrad_kernel<gBM, gBCI, true, false, 14>
           : kpe == 16           ? wgrad_kernel<gBM, gBCI, true, false, 16>
                                 : wgrad_kernel<gBM, gBCI, true, false>;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  hipError_t e;
  if (whole > 0) {   // whole waves: one workgroup per tile, dw written directly
    p.tile0 = 0; p.n_tiles = (int)whole;
    hipLaunchKernelGGL(kern_whole, dim3((unsigned)((whole + 7) / 8 * 8)), dim3(NT), 0, s, p);
    e = hipGetLastError();
    if (e != hipSuccess) return fail(TOFU_ERR_HIP, "conv2d weight-gradient launch failed: %s", hipGetErrorString(e));
  }
  if (rest > 0) {    // the last, partial wave: balanced over all workgroup slots, pieces summed by a second kernel
    p.tile0 = (int)whole; p.n_tiles = (int)rest;
    hipLaunchKernelGGL(kern_balanced, dim3((p.bal.groups + 7) / 8 * 8), dim3(NT), 0, s, p);
    e = hipGetLastError();
    if (e != hipSuccess) return fail(TOFU_ERR_HIP, "conv2d weight-gradient launch failed: %s", hipGetErrorString(e));
    const int64_t items = rest * gBM * gBCI;
    const int blocks = (int)((items + 255) / 256 < 8192 ? (items + 255) / 256 : 8192);
    const bool dense = os[3] == 1 && os[2] == 3 && os[1] == 9 && os[0] % 4 == 0 && (reinterpret_cast<uintptr_t>(dw_out) & 15) == 0;
    hipLaunchKernelGGL(dense ? wgrad_segment_sum_kernel<true> : wgrad_segment_sum_kernel<false>, dim3(blocks), dim3(256), 0, s, dw_out, os[0], os[1], os[2], os[3],
                       static_cast<const float*>(workspace), p.bal, (int)UPT, (int)whole, p.tiles_m, p.tiles_n,
                       (int)CO, (int)CI, accumulate ? 1 : 0);
    e = hipGetLastError();
    if (e != hipSuccess) return fail(TOFU_ERR_HIP, "conv2d weight-gradient segment sum launch failed: %s", hipGetErrorString(e));
  }
  return TOFU_OK;
}

}  // namespace tofu

extern "C" int tofu_shard_conv2d_wgrad(const tofu_op_desc_t* op, const tofu_split_t* splits, int32_t nsplits,
                                       const tofu_tensor_t* x, const tofu_tensor_t* dy, const tofu_tensor_t* dw, void* workspace,
                                       size_t workspace_bytes, void* hip_stream) {
  return tofu::shard_wgrad(op, splits, nsplits, x, dy, dw, workspace, workspace_bytes, hip_stream, false);
}

extern "C" int tofu_shard_conv2d_wgrad_accumulate(const tofu_op_desc_t* op, const tofu_split_t* splits, int32_t nsplits,
                                                  const tofu_tensor_t* x, const tofu_tensor_t* dy, const tofu_tensor_t* dw,
                                                  void* workspace, size_t workspace_bytes, void* hip_stream) {
  return tofu::shard_wgrad(op, splits, nsplits, x, dy, dw, workspace, workspace_bytes, hip_stream, true);
}
