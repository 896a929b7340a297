// Shard of a 3x3, stride-1 convolution forward pass (arXiv 1807.08887: Fig. 1 loop nest in two
// spatial dimensions; Sec. 4.2 Case-1 for N / C_out / H / W splits -- H and W splits read a
// halo-widened input region -- and Case-2 for a C_in split, which yields a partial output).
//   y[n,co,h,w] = sum_{ci,kh,kw} x[n,ci,h+kh-pad,w+kw-pad] * wt[co,ci,kh,kw],  x = 0 outside the
// GLOBAL tensor.  A shard whose box ends at an interior cut gets real halo rows there instead of
// zeros, so the zero border is asymmetric ("residual padding") and is applied per side.
//
// Kernel: implicit GEMM  [co] x [(n,h,w)] over K = (ci, kh, kw) on fp32 MFMA 32x32x2 tiles.
//   * A workgroup owns BM output channels x BN consecutive output positions (positions are
//     numbered n-major over the shard's output box, so lanes stay dense for 14x14 or 7x14 boxes).
//   * Per step of CK input channels it stages in LDS, through registers and double-buffered,
//       - the weights wt[co, ci0..ci0+CK, :, :] transposed to k-major  Ws[(ci,tap)][co], and
//       - for every input channel the input rows the tile's positions can touch, each row
//         widened by the filter window and with the zero border materialised, so that the nine
//         taps are nine shifted reads of the SAME staged rows (no im2col copy, 9x reuse in LDS).
//     Rows are kept in "virtual row" order: image i, padded row u -> i*(BH+2)+u; a tile stages
//     the virtual rows [T_a, T_b] its positions need.
//   * One MFMA contracts the same tap of two adjacent input channels (lanes 0-31: ci, lanes
//     32-63: ci+1); the B operand of a lane is one LDS read at (its position's row/col) + tap.
//   * Launch: full waves of 512 tiles run one workgroup per tile.  The channel steps of the last,
//     partial wave's tiles are dealt to 512 workgroups as tofu_balance.h describes (the same work
//     for every workgroup, neighbours at the same steps at the same time); every piece of a tile
//     goes to a workspace slot and a second kernel sums each tile's slots in the order of the
//     channel steps (fixed, no atomics).
// The same kernel serves the variant that reads its input region from several blocks (the fetch
// fused into the consumer, Sec. 6) and, on reversed filters, the data gradient.
#include <hip/hip_runtime.h>

#include <string.h>

#include <type_traits>

#include "tofu_balance.h"
#include "tofu_internal.h"
#include "tofu_mfma.h"

namespace tofu {

struct ConvArgs {
  const float* x;   // element at the low corner of the (clipped) input box
  const float* w;   // element (co_lo, ci_lo, 0, 0)
  float* y;         // element at the low corner of the output box
  int accumulate;   // 1: the shard's result is added to what the output box holds
  int64_t xs[4], ws[4], ys[4];   // element strides (n, c, h, w) / (co, ci, kh, kw) / (n, co, h, w)
  uint32_t x_bytes, w_bytes;     // bytes spanned by the input box / the filter box (buffer bounds)
  int NB, CO, CI;   // images, output channels and input channels of the shard
  int BH, BW;       // output box rows / columns
  int IH, IW;       // rows / columns of the clipped input box
  int plh, plw;     // zero rows / columns in front of the input box (residual padding, low side)
  int P;            // NB * BH * BW output positions
  int tiles_m, tiles_n;
  int LDW;          // floats per staged row  (BW + 2)
  int PL;           // floats per staged channel plane
  int E;            // upper bound over all tiles of the staged floats per channel (<= PL)
  int w_fast;       // 1: weights dense over (ci,kh,kw) and 16-byte aligned -> vector loads
  // Balanced launches: the channel steps of the tiles [tile0, tile0 + n_tiles) are dealt to bal.groups
  // workgroups as tofu_balance.h describes; every piece of a tile leaves its accumulators in a slot of
  // `slots`.  Whole-tile launches cover the same tile range with one workgroup per tile.
  int tile0, n_tiles;
  Balance bal;
  float* slots;
};

// Input region held by several blocks (the fetch fused into the consumer, Sec. 6): every block
// spans the region's channels and holds a box of its (image, row, column) coordinates.
constexpr int kMaxConvSources = 16;
struct ConvSrc {
  const float* base;   // address the region's low corner WOULD have inside this block
  int64_t s[4];        // element strides (n, c, h, w) of the block
  int lo[3], hi[3];    // (image, row, column) box held, relative to the region's low corner
};
struct ConvSources {
  int n;
  ConvSrc src[kMaxConvSources];
};
// Lanes with nothing to read (zero border, idle staging slots) load from here in the multi-block kernels.
__device__ float kZeroWords[64];

// Tile number -> (position tile, channel tile row).  Tiles are numbered in panels of kPanelRows channel
// tile rows; inside a panel the channel row runs fastest.  The 64 workgroups that run side by side on one
// XCD are consecutive tiles, i.e. a block of 8 position tiles x 8 channel rows (or all rows, when the shard has
// fewer): per step they share 8 input tiles and 8 filter rows through that XCD's L2, close to the least a
// block of 64 can read.  (Channel row fastest over ALL rows made 64 tiles = 1.6 position tiles x 40 rows
// for a shard of 2560 output channels, which re-read the filters once per 1.6 position tiles.)
constexpr int kPanelRows = 8;
__device__ __forceinline__ void decode_tile(int tile, int tiles_m, int tiles_n, int& tile_n, int& tile_m) {
  const int panel_tiles = kPanelRows * tiles_n;
  const int panel = tile / panel_tiles, rem = tile - panel * panel_tiles;
  const int rows = min(kPanelRows, tiles_m - panel * kPanelRows);
  tile_n = rem / rows;
  tile_m = panel * kPanelRows + (rem - tile_n * rows);
}

template <int BM, int BN, int CK, int WM, int WN, int XJ, int KH = 3, int KW = 3>
struct ConvCfg {
  static constexpr int kThreads = 64 * WM * WN;
  static constexpr int TM = BM / WM, TN = BN / WN, FM = TM / 32, FN = TN / 32;
  static constexpr int T = KH * KW;            // filter taps
  static constexpr int KK = CK * T;            // GEMM-K per step
  static constexpr int LDM = BM + 1;           // Ws[kk][m]; odd pitch keeps the transposing writes spread over the banks
  static constexpr int WV = (BM * KK / 4 + kThreads - 1) / kThreads;   // weight vectors per thread per step
  // each LDS buffer ends with scratch floats that absorb the writes of idle staging slots
  static constexpr int WB = KK * LDM + 3 * LDM + 64;                   // floats per weight buffer
  static int xb(int PL) { return CK * PL + 64; }                       // floats per input buffer
  static_assert(TM % 32 == 0 && TN % 32 == 0 && CK % 4 == 0, "bad tile");   // CK % 4: KK holds whole vectors, channels pair up
  static size_t lds_floats(int PL) { return 2 * ((size_t)WB + (size_t)xb(PL)); }
};

// SRC: where the input region lives.  0: one buffer, addressed with 32-bit buffer offsets.  1: several
// blocks, each staging item keeps a 64-bit address and its own increment per channel step.  2: several
// blocks that share their channel stride and lie within one 2 GiB window of addresses: the window is one
// buffer and an item's offset points into whichever block holds its element, so the step loop is that of
// form 0 (the blocks of a halo exchange are usually allocated alike and close together).
template <int BM, int BN, int CK, int WM, int WN, int XJ, int SRC, bool BALANCED, int KH = 3, int KW = 3>
__device__ __forceinline__ void conv2d_body(const ConvArgs& p, const ConvSources* srcs) {
  constexpr bool MULTI = SRC == 1;
  using Cfg = ConvCfg<BM, BN, CK, WM, WN, XJ, KH, KW>;
  constexpr int NT = Cfg::kThreads, FM = Cfg::FM, FN = Cfg::FN, KK = Cfg::KK, LDM = Cfg::LDM, WV = Cfg::WV, T = Cfg::T;
  constexpr uint32_t kNone = kNoOffset;
  extern __shared__ float lds[];
  const int PL = p.PL, LDW = p.LDW;
  constexpr int WB = Cfg::WB;
  const int XB = CK * PL + 64;
  float* Ws = lds;                           // [2][WB]: KK rows of LDM floats + scratch
  float* Xs = lds + 2 * WB;                  // [2][XB]: CK planes of PL floats + scratch

  // Compute units are handed workgroups round-robin over the 8 XCDs; renumber so that
  // consecutive logical workgroups (which share staged input rows) land on the same XCD's L2.
  const int total = BALANCED ? p.bal.groups : p.n_tiles;
  const int per_xcd = (total + 7) / 8;
  const int lid = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (lid >= total) return;                   // grid is padded to a multiple of 8
  const int steps_all = (p.CI + CK - 1) / CK;
  // balanced: this workgroup's segments (pieces of tiles)
  BalanceWalk walk;
  if (BALANCED) {
    walk = balance_walk(p.bal, steps_all, lid);
    if (walk.count == 0) return;
  }
  int seg_i = 0;
  do {
  // The per-lane staging lists below are rebuilt for every segment.  The thread index is made
  // opaque once per segment so that the parts of them that do not depend on the tile are not
  // kept in registers across the step loop of the previous segment.
  int tid = threadIdx.x;
  if (BALANCED) asm volatile("" : "+v"(tid));
  const int lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, half = lane >> 5;
  const int wm = wave / WN, wn = wave % WN;
  int tile = p.tile0 + lid, s_begin = 0, s_end = steps_all, slot = 0;
  if (BALANCED) {
    const BalanceSegment seg = balance_segment(walk, seg_i);
    tile = p.tile0 + seg.tile; s_begin = seg.begin; s_end = seg.end; slot = seg.slot;
  }
  int tile_n, tile_m;
  decode_tile(tile, p.tiles_m, p.tiles_n, tile_n, tile_m);
  const int m0 = tile_m * BM;
  const int p_begin = tile_n * BN;
  const int p_end = min(p.P, p_begin + BN);
  const int img_rows = p.BH + KH - 1;         // window-widened rows per image in virtual-row order
  const int plane = p.BH * p.BW;

  // virtual rows staged by this tile
  const int ra = p_begin / p.BW, rb = (p_end - 1) / p.BW;
  const int T_a = (ra / p.BH) * img_rows + ra % p.BH;
  const int T_b = (rb / p.BH) * img_rows + rb % p.BH + KH - 1;
  const int E = (T_b - T_a + 1) * LDW;        // staged floats per channel for this tile

  // ---- per-thread staging lists, fixed for the whole K loop ----
  uint32_t x_voff[MULTI ? 1 : XJ];   // byte offset of the element inside channel step 0, kNone = reads as zero
  const float* x_ptr[MULTI ? XJ : 1];  // multi-block form: address of the element inside channel step 0 ...
  int x_inc[MULTI ? XJ : 1];           // ... and its element increment per channel step (0 for lanes that read zeros)
  int x_loff[XJ];        // LDS float index inside one x buffer (or its scratch tail)
#pragma unroll
  for (int j = 0; j < XJ; ++j) {
    const int idx = tid + j * NT;
    const int ci_l = idx / p.E, rem = idx - ci_l * p.E;
    const int s = rem / LDW, c = rem - s * LDW;
    const int V = T_a + s;
    const int img = V / img_rows, u = V - img * img_rows;
    const int ih = u - p.plh, iw = c - p.plw;
    const bool live = ci_l < CK && rem < E;
    const bool valid = live && img < p.NB && ih >= 0 && ih < p.IH && iw >= 0 && iw < p.IW;
    x_loff[j] = live ? ci_l * PL + rem : CK * PL + lane;
    if constexpr (MULTI) {
      x_ptr[j] = kZeroWords;
      x_inc[j] = 0;
      for (int b = 0; b < srcs->n; ++b) {     // the blocks tile the region: at most one of them holds the coordinate
        const ConvSrc& S = srcs->src[b];
        if (valid && img >= S.lo[0] && img < S.hi[0] && ih >= S.lo[1] && ih < S.hi[1] && iw >= S.lo[2] && iw < S.hi[2]) {
          x_ptr[j] = S.base + ((int64_t)img * S.s[0] + (int64_t)ci_l * S.s[1] + (int64_t)ih * S.s[2] + (int64_t)iw * S.s[3]);
          x_inc[j] = CK * (int)S.s[1];
        }
      }
    } else if constexpr (SRC == 2) {
      x_voff[j] = kNone;
      for (int b = 0; b < srcs->n; ++b) {     // the blocks tile the region: at most one of them holds the coordinate
        const ConvSrc& S = srcs->src[b];
        if (valid && img >= S.lo[0] && img < S.hi[0] && ih >= S.lo[1] && ih < S.hi[1] && iw >= S.lo[2] && iw < S.hi[2])
          x_voff[j] = 4u * (uint32_t)((S.base - p.x) + (int64_t)img * S.s[0] + (int64_t)ci_l * S.s[1] + (int64_t)ih * S.s[2] + (int64_t)iw * S.s[3]);
      }
    } else {
      x_voff[j] = valid ? 4u * (uint32_t)((int64_t)img * p.xs[0] + (int64_t)ci_l * p.xs[1] + (int64_t)ih * p.xs[2] + (int64_t)iw * p.xs[3]) : kNone;
    }
  }
  uint32_t w_voff[WV];
  int w_loff[WV];
#pragma unroll
  for (int i = 0; i < WV; ++i) {
    const int idx = tid + i * NT, row = idx / (KK / 4), q = idx - row * (KK / 4);
    const bool live = idx < BM * KK / 4;
    w_loff[i] = live ? 4 * q * LDM + row : KK * LDM + lane;
    w_voff[i] = (live && m0 + row < p.CO) ? 4u * (uint32_t)((int64_t)(m0 + row) * p.ws[0] + 4 * q) : kNone;
  }
  const __amdgpu_buffer_rsrc_t x_rsrc = make_rsrc(p.x, p.x_bytes);
  const __amdgpu_buffer_rsrc_t w_rsrc = make_rsrc(p.w, p.w_bytes);

  float rx[XJ];
  v4f32 rw[WV];
  auto load_global = [&](int local_step) {
    const int step = s_begin + local_step;      // channel step of the whole reduction
    const int ci0 = step * CK;
    const bool whole = ci0 + CK <= p.CI;        // only the last step can run past the shard's channels
    if constexpr (MULTI) {
#pragma unroll
      for (int j = 0; j < XJ; ++j) {
        const bool ok = whole || ci0 + (tid + j * NT) / p.E < p.CI;
        const float* src = x_ptr[j] + (int64_t)step * x_inc[j];
        rx[j] = *(ok ? src : kZeroWords);
      }
    } else {
      const uint32_t x_soff = 4u * (uint32_t)((int64_t)ci0 * p.xs[1]);
      if (whole) {
#pragma unroll
        for (int j = 0; j < XJ; ++j) rx[j] = buf_load(x_rsrc, x_voff[j], x_soff);
      } else {
#pragma unroll
        for (int j = 0; j < XJ; ++j) {
          const bool ok = ci0 + (tid + j * NT) / p.E < p.CI;
          rx[j] = buf_load(x_rsrc, ok ? x_voff[j] : kNone, x_soff);
        }
      }
    }
    if (p.w_fast && whole) {
      const uint32_t w_soff = 4u * T * (uint32_t)ci0;
#pragma unroll
      for (int i = 0; i < WV; ++i) rw[i] = buf_load4(w_rsrc, w_voff[i], w_soff);
    } else {
#pragma unroll
      for (int i = 0; i < WV; ++i) {
        const int idx = tid + i * NT, row = idx / (KK / 4), q = idx - row * (KK / 4);
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
          const int kk = 4 * q + jj, ci_l = kk / T, tap = kk - ci_l * T, kh = tap / KW, kw = tap - kh * KW;
          const bool ok = idx < BM * KK / 4 && m0 + row < p.CO && ci0 + ci_l < p.CI;
          rw[i][jj] = ok ? p.w[(int64_t)(m0 + row) * p.ws[0] + (int64_t)(ci0 + ci_l) * p.ws[1] + kh * p.ws[2] + kw * p.ws[3]] : 0.f;
        }
      }
    }
  };
  auto store_lds = [&](int buf) {
    float* xs = Xs + buf * XB;
    float* wsm = Ws + buf * WB;
#pragma unroll
    for (int j = 0; j < XJ; ++j) xs[x_loff[j]] = rx[j];
#pragma unroll
    for (int i = 0; i < WV; ++i)
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) wsm[w_loff[i] + jj * LDM] = rw[i][jj];
  };

  // ---- per-lane position of each N block: LDS offset of tap (0,0) and output offset ----
  int pos_l[FN];
  int64_t y_off[FN];
  bool pos_ok[FN];
#pragma unroll
  for (int j = 0; j < FN; ++j) {
    int pp = p_begin + wn * Cfg::TN + j * 32 + l32;
    pos_ok[j] = pp < p_end;
    if (!pos_ok[j]) pp = p_end - 1;          // keep the address inside the staged rows
    const int img = pp / plane, q = pp - img * plane, oh = q / p.BW, ow = q - oh * p.BW;
    pos_l[j] = (img * img_rows + oh - T_a) * LDW + ow + half * PL;
    y_off[j] = (int64_t)img * p.ys[0] + (int64_t)oh * p.ys[2] + (int64_t)ow * p.ys[3];
  }

  acc16 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j) acc[i][j] = acc_zero();

  const int steps = s_end - s_begin;
  constexpr int KS = (CK / 2) * T;            // MFMA k-steps per step: (channel pair, tap)
  // Staging work of one step = XJ input items + WV weight items.  In a HOT step each item (write
  // last step's registers to LDS, then reload them for the step after next) is issued between
  // two k-steps of the MFMA stream, one item every STRIDE k-steps, so that no MFMA waits behind
  // a block of staging instructions.  Steps whose reload would touch the ragged last channel
  // step (or weights that are not dense) use the guarded loads in one block instead.
  constexpr int NI = XJ + WV, STRIDE = (KS - 2) / NI > 0 ? (KS - 2) / NI : 1;
  static_assert(1 + (NI - 1) * STRIDE < KS, "staging items must fit into one step");
  const int n_hot = !p.w_fast ? 0 : (p.CI % CK == 0 || s_end < steps_all) ? steps : max(0, steps - 3);

  // Pipeline: the tiles of step t+1 are written to LDS during step t, and right after each write
  // the global load of step t+2 is issued into the same register, so every load has a whole step
  // to land.  The body is branch-free (the compiler can then count outstanding LDS operations
  // exactly): the last steps simply stage the final tiles again into the idle buffer.
  load_global(0);
  store_lds(0);
  load_global(min(1, steps - 1));
  __syncthreads();

  auto run_step = [&](int t, auto hot_tag) {
    constexpr bool HOT = decltype(hot_tag)::value;
    const int buf = t & 1;
    const float* wsm = Ws + buf * WB + wm * Cfg::TM + l32 + half * T * LDM;
    const float* xs = Xs + buf * XB;
    float* xs_next = Xs + (buf ^ 1) * XB;
    float* ws_next = Ws + (buf ^ 1) * WB;
    const int nxt = min(t + 2, steps - 1), nxt_abs = s_begin + nxt;
    const uint32_t x_soff = MULTI ? 0u : 4u * (uint32_t)((int64_t)nxt_abs * CK * p.xs[1]), w_soff = 4u * T * (uint32_t)(nxt_abs * CK);
    // operands of k-step s+1 are fetched before the MFMAs of k-step s are issued
    float a[2][FM], b[2][FN];
    auto fetch = [&](int s, float (&av)[FM], float (&bv)[FN]) {
      const int cp = s / T, tap = s % T, kh = tap / KW, kw = tap % KW;
#pragma unroll
      for (int i = 0; i < FM; ++i) av[i] = wsm[(cp * 2 * T + tap) * LDM + i * 32];
#pragma unroll
      for (int j = 0; j < FN; ++j) bv[j] = xs[cp * 2 * PL + pos_l[j] + kh * LDW + kw];
    };
    fetch(0, a[0], b[0]);
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      if (s + 1 < KS) fetch(s + 1, a[(s + 1) & 1], b[(s + 1) & 1]);
      if (HOT) {
        if (s >= 1 && (s - 1) % STRIDE == 0 && (s - 1) / STRIDE < NI) {
          const int item = (s - 1) / STRIDE;
          if (item < XJ) {
            xs_next[x_loff[item]] = rx[item];
            if constexpr (MULTI) rx[item] = x_ptr[item][(int64_t)nxt_abs * x_inc[item]];
            else rx[item] = buf_load(x_rsrc, x_voff[item], x_soff);
          } else {
            const int i = item - XJ;
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) ws_next[w_loff[i] + jj * LDM] = rw[i][jj];
            rw[i] = buf_load4(w_rsrc, w_voff[i], w_soff);
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
        for (int j = 0; j < FN; ++j) acc[i][j] = mfma_32x32x2(a[s & 1][i], b[s & 1][j], acc[i][j]);
    }
    __syncthreads();
  };
  for (int t = 0; t < n_hot; ++t) run_step(t, std::true_type());
  for (int t = n_hot; t < steps; ++t) run_step(t, std::false_type());

  if constexpr (BALANCED) {
    // slot [(i, j, v)][thread]: every store instruction of the workgroup writes NT consecutive floats
    float* o = p.slots + (int64_t)slot * (BM * BN) + tid;
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
      for (int j = 0; j < FN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[((i * FN + j) * 16 + v) * NT] = acc[i][j][v];
    __syncthreads();   // the next segment's prologue overwrites LDS buffer 0
  } else {
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
      for (int j = 0; j < FN; ++j) {
        if (!pos_ok[j]) continue;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int co = m0 + wm * Cfg::TM + i * 32 + acc_row(v, half);
          if (co < p.CO) {
            float* o = p.y + y_off[j] + (int64_t)co * p.ys[1];
            *o = p.accumulate ? *o + acc[i][j][v] : acc[i][j][v];
          }
        }
      }
  }
  ++seg_i;
  } while (BALANCED && seg_i < walk.count);
}

// Sums the slots of every balanced tile in the order of its channel steps and writes the output
// box (or adds the sum to it).  One
// workgroup per (tile, 32x32 accumulator block): thread and accumulator index map to (channel,
// position) exactly as in the convolution kernel, so reads are NT consecutive floats and writes
// follow the output rows.
template <int BM, int BN, int WM, int WN>
__global__ void __launch_bounds__(64 * WM * WN) conv2d_segment_sum_kernel(const ConvArgs p, int steps_all) {
  constexpr int NT = 64 * WM * WN, TM = BM / WM, TN = BN / WN, FN = TN / 32;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, half = lane >> 5;
  const int wm = wave / WN, wn = wave % WN;
  const int t_rel = blockIdx.x, blk = blockIdx.y, i = blk / FN, j = blk % FN;
  const int tile = p.tile0 + t_rel;
  int tile_n, tile_m;
  decode_tile(tile, p.tiles_m, p.tiles_n, tile_n, tile_m);
  const int plane = p.BH * p.BW;
  const int pp = tile_n * BN + wn * TN + j * 32 + l32;
  const bool pos_ok = pp < p.P;
  const int img = pp / plane, q = pp - img * plane, oh = q / p.BW, ow = q - oh * p.BW;
  const int64_t y_off = (int64_t)img * p.ys[0] + (int64_t)oh * p.ys[2] + (int64_t)ow * p.ys[3];
  float acc[16];
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.f;
  balance_for_each_slot(p.bal, steps_all, t_rel, [&](int slot) {
    const float* sl = p.slots + (int64_t)slot * (BM * BN) + (i * FN + j) * 16 * NT + tid;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] += sl[v * NT];
  });
  if (!pos_ok) return;
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int co = tile_m * BM + wm * TM + i * 32 + acc_row(v, half);
    if (co < p.CO) {
      float* o = p.y + y_off + (int64_t)co * p.ys[1];
      *o = p.accumulate ? *o + acc[v] : acc[v];
    }
  }
}

// input region in one buffer
template <int BM, int BN, int CK, int WM, int WN, int XJ, bool BALANCED, int KH = 3, int KW = 3>
__global__ void __launch_bounds__(64 * WM * WN, 2) conv2d_kernel(const ConvArgs p) {
  conv2d_body<BM, BN, CK, WM, WN, XJ, 0, BALANCED, KH, KW>(p, nullptr);
}

// input region read from the blocks that hold it
template <int BM, int BN, int CK, int WM, int WN, int XJ, bool BALANCED, bool WINDOW, int KH = 3, int KW = 3>
__global__ void __launch_bounds__(64 * WM * WN, 2) conv2d_multi_kernel(const ConvArgs p, const ConvSources srcs) {
  conv2d_body<BM, BN, CK, WM, WN, XJ, WINDOW ? 2 : 1, BALANCED, KH, KW>(p, &srcs);
}

constexpr size_t kLdsLimit = 64 * 1024;   // dynamic LDS a launch may ask for without raising the kernel's limit; the plans stay below it

// Most floats per channel any tile of BN consecutive positions stages (rows touched + window rows).
static int64_t max_staged(int64_t P, int64_t BH, int64_t BW, int64_t BN, int64_t KH = 3, int64_t KW = 3) {
  int64_t max_slots = 0;
  for (int64_t pb = 0; pb < P; pb += BN) {
    const int64_t pe = pb + BN < P ? pb + BN : P;
    const int64_t ra = pb / BW, rb = (pe - 1) / BW;
    const int64_t slots = ((rb / BH) * (BH + KH - 1) + rb % BH + KH - 1) - ((ra / BH) * (BH + KH - 1) + ra % BH) + 1;
    if (slots > max_slots) max_slots = slots;
  }
  return max_slots * (BW + KW - 1);
}

constexpr int kConvSlots = 512;        // two resident workgroups on each of the 256 compute units (a third one per unit
                                       // fits only with register spills and measured no faster)

// Which kernel shape a shard of P positions in BH x BW boxes uses, and how its tiles are launched:
// the first `whole` tiles one workgroup each (full waves of kConvSlots), the channel steps of the
// remaining `rest` tiles dealt to kConvSlots workgroups (`bal`, see tofu_balance.h).
struct ConvPlan {
  int variant;        // 3x3: 0: 64 x 256 positions, 4 channels per step; 1: 64 x 128, 8 channels; 2: 64 x 128, 4 channels;
                      // 1x3: 10: 64 x 256 positions, 12 channels per step; 11: 64 x 128, 12 channels; -1: none fits
  int64_t E;          // staged floats per channel
  int64_t tiles, whole, rest;
  Balance bal;        // of the `rest` tiles
  int64_t slots;      // accumulator slots the balanced launch writes
  int BM, BN, CK;
};

// Channel steps a workgroup loses per segment (list set-up, filling the pipeline, writing the slot).
constexpr int kSegmentCost = 2;

static ConvPlan conv_plan(int64_t P, int64_t BH, int64_t BW, int64_t CO, int64_t CI, bool multi = false, int KH = 3, int KW = 3, int BM = 64) {
  ConvPlan pl;
  memset(&pl, 0, sizeof(pl));
  const int64_t E256 = max_staged(P, BH, BW, 256, KH, KW), E128 = max_staged(P, BH, BW, 128, KH, KW);
  // 256 positions per workgroup (64 x 64 per wavefront) whenever its staged rows fit and the shard
  // has at least that many positions; else 128 positions, with fewer channels per step when the
  // staged rows are wide.
  (void)multi;   // both forms use the same shapes today; the plan is asked per form so that they may differ
  // a shard of few positions: 128-position tiles when they leave at least a tenth less of the last tile empty
  const bool small_tiles = ((P + 127) / 128 * 128) * 10 <= ((P + 255) / 256 * 256) * 9;
  if (KH == 1 && KW == 3) {
    // a row of three taps: 12 channels per step give the same 36-deep step as 4 channels of 3 x 3
    if (P >= 256 && !small_tiles && 12 * E256 <= 13 * 256) { pl.variant = 10; pl.E = E256; pl.BN = 256; pl.CK = 12; }
    else if (12 * E128 <= 13 * 256) { pl.variant = 11; pl.E = E128; pl.BN = 128; pl.CK = 12; }
    else { pl.variant = -1; pl.E = E128; return pl; }
  } else if (KH != 3 || KW != 3) { pl.variant = -1; return pl; }
  else if (P >= 256 && !small_tiles && 4 * E256 <= 8 * 256) { pl.variant = 0; pl.E = E256; pl.BN = 256; pl.CK = 4; }
  else if (8 * E128 <= 10 * 256) { pl.variant = 1; pl.E = E128; pl.BN = 128; pl.CK = 8; }
  else if (4 * E128 <= 10 * 256) { pl.variant = 2; pl.E = E128; pl.BN = 128; pl.CK = 4; }
  else { pl.variant = -1; pl.E = E128; return pl; }
  pl.BM = BM;
  pl.tiles = ((CO + BM - 1) / BM) * ((P + pl.BN - 1) / pl.BN);
  const int64_t steps = (CI + pl.CK - 1) / pl.CK;
  pl.rest = pl.tiles % kConvSlots;
  // a last wave that is nearly full, or a reduction too short to cut, is launched as whole tiles
  if (pl.rest * 32 >= kConvSlots * 31 || steps < 4) pl.rest = 0;
  pl.whole = pl.tiles - pl.rest;
  if (pl.rest > 0) {
    pl.bal = balance_plan(pl.rest, steps, kConvSlots, kSegmentCost);
    pl.slots = balance_slots(pl.bal, (int)steps);
  }
  return pl;
}

static size_t plan_bytes(const ConvPlan& pl) {
  if (pl.variant < 0 || pl.rest == 0) return 0;
  return (size_t)pl.slots * pl.BM * pl.BN * sizeof(float);
}

// A shard's output channels are computed in tile rows of 64.  When the last row would hold at most 32
// channels it is computed by a launch of its own with 32-row tiles (one MFMA block per wavefront instead of
// two), so that a shard of 160 channels costs 160 rows of work and not 192.  -> channels of the 64-row part
// (a multiple of 64, possibly 0); the rest, if any, is the 32-row part.
static int64_t conv_main_channels(int64_t CO) {
  const int64_t tail = CO % 64;
  return (tail == 0 || tail > 32) ? CO : CO - tail;
}

// enough for either entry point (one input buffer, or the region read from several blocks) and for both channel parts,
// which run one after the other on the stream and use the slots in turn
size_t conv_workspace_bytes(int64_t P, int64_t BH, int64_t BW, int64_t CO, int64_t CI, int KH, int KW) {
  const int64_t co_main = conv_main_channels(CO);
  size_t need = 0;
  for (int part = 0; part < 2; ++part) {
    const int64_t co = part == 0 ? co_main : CO - co_main;
    if (co == 0) continue;
    for (int multi = 0; multi < 2; ++multi) {
      const size_t n = plan_bytes(conv_plan(P, BH, BW, co, CI, multi != 0, KH, KW, part == 0 ? 64 : 32));
      if (n > need) need = n;
    }
  }
  return need;
}

template <int BM, int BN, int CK, int WM, int WN, int XJ, int KH = 3, int KW = 3>
static int launch_conv(ConvArgs p, const ConvSources* srcs, const ConvPlan& pl, hipStream_t stream) {
  using Cfg = ConvCfg<BM, BN, CK, WM, WN, XJ, KH, KW>;
  p.tiles_m = (p.CO + BM - 1) / BM;
  p.tiles_n = (p.P + BN - 1) / BN;
  p.E = (int)pl.E;
  p.PL = (p.E + 63) / 64 * 64 + 32;
  const size_t lds_bytes = sizeof(float) * Cfg::lds_floats(p.PL);
  if (lds_bytes > kLdsLimit) return fail(TOFU_ERR_UNSUPPORTED, "conv2d: staging needs %zu bytes of LDS", lds_bytes);
  auto launch = [&](bool balanced, int wgs) {
    const dim3 grid((wgs + 7) / 8 * 8), block(Cfg::kThreads);
    if (srcs) {
      if constexpr (KH == 3 && KW == 3) {   // the multi-block form exists for the 3 x 3 shapes only (the caller checked)
        const bool window = p.x != nullptr;   // the blocks lie in one window of addresses that starts at p.x
        if (balanced && window) hipLaunchKernelGGL((conv2d_multi_kernel<BM, BN, CK, WM, WN, XJ, true, true>), grid, block, lds_bytes, stream, p, *srcs);
        else if (balanced) hipLaunchKernelGGL((conv2d_multi_kernel<BM, BN, CK, WM, WN, XJ, true, false>), grid, block, lds_bytes, stream, p, *srcs);
        else if (window) hipLaunchKernelGGL((conv2d_multi_kernel<BM, BN, CK, WM, WN, XJ, false, true>), grid, block, lds_bytes, stream, p, *srcs);
        else hipLaunchKernelGGL((conv2d_multi_kernel<BM, BN, CK, WM, WN, XJ, false, false>), grid, block, lds_bytes, stream, p, *srcs);
      }
    } else {
      if (balanced) hipLaunchKernelGGL((conv2d_kernel<BM, BN, CK, WM, WN, XJ, true, KH, KW>), grid, block, lds_bytes, stream, p);
      else hipLaunchKernelGGL((conv2d_kernel<BM, BN, CK, WM, WN, XJ, false, KH, KW>), grid, block, lds_bytes, stream, p);
    }
  };
  if (pl.whole > 0) {
    p.tile0 = 0; p.n_tiles = (int)pl.whole; memset(&p.bal, 0, sizeof(p.bal));
    launch(false, (int)pl.whole);
  }
  if (pl.rest > 0) {
    p.tile0 = (int)pl.whole; p.n_tiles = (int)pl.rest; p.bal = pl.bal;
    launch(true, pl.bal.groups);
    hipLaunchKernelGGL((conv2d_segment_sum_kernel<BM, BN, WM, WN>), dim3((unsigned)pl.rest, Cfg::FM * Cfg::FN), dim3(Cfg::kThreads), 0, stream,
                       p, (p.CI + CK - 1) / CK);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(TOFU_ERR_HIP, "conv2d launch failed: %s", hipGetErrorString(e));
  return TOFU_OK;
}

// One convolution-shaped problem after all region arithmetic: write box `out_box` (n, m, h, w)
// of y from box `in_box` (n, k, rows, columns) of x, where output row h reads input rows
// h - out_box.lo[2] + kh - pad_lo[0] of the box (zeros outside it), likewise for columns.
struct ConvProblem {
  tofu_region_t out_box, in_box;
  int64_t pad_lo[2];
  const float* x;            // element at in_box's low corner in the single input buffer, or NULL ...
  int64_t xs[4];
  const ConvSources* srcs;   // ... when the box is read from several blocks
  int64_t window_bytes = 0;  // > 0: the blocks share their channel stride (xs[1]) and lie in [x, x + window_bytes)
  const float* w;            // element (m_lo, k_lo, 0, 0); strides (m, k, kh, kw)
  int64_t ws[4];
  float* y;                  // element at out_box's low corner
  int64_t ys[4];
  void* workspace;           // piece slots of a balanced launch (conv_workspace_bytes), may be NULL when none are needed
  size_t workspace_bytes;
  bool accumulate;           // add to the output box instead of overwriting it
  int KH = 3, KW = 3;        // filter rows / columns: 3 x 3 or 1 x 3
};

static int conv_core(const ConvProblem& q, hipStream_t stream) {
  ConvArgs p;
  p.x = q.x; p.w = q.w; p.y = q.y;
  p.accumulate = q.accumulate ? 1 : 0;
  const int64_t NB = q.out_box.hi[0] - q.out_box.lo[0], CO = q.out_box.hi[1] - q.out_box.lo[1];
  const int64_t BH = q.out_box.hi[2] - q.out_box.lo[2], BW = q.out_box.hi[3] - q.out_box.lo[3];
  const int64_t CI = q.in_box.hi[1] - q.in_box.lo[1];
  const int64_t P = NB * BH * BW;
  if (P >= (1 << 30) || CO >= (1 << 30) || CI >= (1 << 30)) return fail(TOFU_ERR_UNSUPPORTED, "conv2d shard extent exceeds 2^30");
  for (int d = 0; d < 4; ++d) { p.xs[d] = q.xs[d]; p.ws[d] = q.ws[d]; p.ys[d] = q.ys[d]; }
  // lanes address the filters (and a single input buffer) with 32-bit byte offsets from the boxes' low corners
  int64_t x_span = 1, w_span = 1;
  const int64_t w_ext[4] = {CO, CI, q.KH, q.KW};
  for (int d = 0; d < 4; ++d) {
    if (q.xs[d] < 0 || q.ws[d] < 0) return fail(TOFU_ERR_UNSUPPORTED, "conv2d: negative strides are not supported");
    x_span += (q.in_box.hi[d] - q.in_box.lo[d] - 1) * q.xs[d];
    w_span += (w_ext[d] - 1) * q.ws[d];
  }
  if (x_span >= ((int64_t)1 << 29) || w_span >= ((int64_t)1 << 29))
    return fail(TOFU_ERR_UNSUPPORTED, "conv2d: an operand region spans 2 GiB or more");
  p.x_bytes = q.srcs ? (uint32_t)q.window_bytes : (uint32_t)(4 * x_span);
  p.w_bytes = (uint32_t)(4 * w_span);
  p.NB = (int)NB; p.CO = (int)CO; p.CI = (int)CI; p.BH = (int)BH; p.BW = (int)BW; p.P = (int)P;
  p.IH = (int)(q.in_box.hi[2] - q.in_box.lo[2]);
  p.IW = (int)(q.in_box.hi[3] - q.in_box.lo[3]);
  p.plh = (int)q.pad_lo[0]; p.plw = (int)q.pad_lo[1];
  p.LDW = (int)BW + q.KW - 1;
  p.w_fast = q.ws[3] == 1 && (q.KH == 1 || q.ws[2] == q.KW) && q.ws[1] == q.KH * q.KW && q.ws[0] % 4 == 0 && (reinterpret_cast<uintptr_t>(p.w) & 15) == 0;

  if (q.srcs && (q.KH != 3 || q.KW != 3)) return fail(TOFU_ERR_UNSUPPORTED, "conv2d: only 3 x 3 filters read their region from several blocks");
  if (q.workspace && (reinterpret_cast<uintptr_t>(q.workspace) & 15)) return fail(TOFU_ERR_INVALID_ARG, "workspace must be 16-byte aligned");
  p.slots = static_cast<float*>(q.workspace);
  // the 64-row part of the output channels, then the 32-row part (see conv_main_channels)
  const int64_t co_main = conv_main_channels(CO);
  ConvPlan plans[2];
  for (int part = 0; part < 2; ++part) {
    const int64_t co = part == 0 ? co_main : CO - co_main;
    if (co == 0) continue;
    plans[part] = conv_plan(P, BH, BW, co, CI, q.srcs != nullptr, q.KH, q.KW, part == 0 ? 64 : 32);
    if (plans[part].variant < 0)
      return fail(TOFU_ERR_UNSUPPORTED, "conv2d: output box is too wide for the staging buffers (%lld staged floats per channel)", (long long)plans[part].E);
    const size_t need = plan_bytes(plans[part]);
    if (need > 0 && (!q.workspace || q.workspace_bytes < need))
      return fail(TOFU_ERR_WORKSPACE_TOO_SMALL, "conv2d shard needs %zu workspace bytes, got %zu", need, q.workspace ? q.workspace_bytes : (size_t)0);
  }
  for (int part = 0; part < 2; ++part) {
    const int64_t co0 = part == 0 ? 0 : co_main, co = part == 0 ? co_main : CO - co_main;
    if (co == 0) continue;
    ConvArgs pp = p;
    pp.w = p.w + co0 * q.ws[0];
    pp.y = p.y + co0 * q.ys[1];
    pp.CO = (int)co;
    pp.w_bytes = (uint32_t)(4 * (w_span - (CO - co) * q.ws[0]));
    const ConvPlan& pl = plans[part];
    int rc;
    if (part == 0) {
      rc = pl.variant == 10  ? launch_conv<64, 256, 12, 1, 4, 13, 1, 3>(pp, q.srcs, pl, stream)
           : pl.variant == 11 ? launch_conv<64, 128, 12, 1, 4, 13, 1, 3>(pp, q.srcs, pl, stream)
           : pl.variant == 0  ? launch_conv<64, 256, 4, 1, 4, 8>(pp, q.srcs, pl, stream)
           : pl.variant == 1  ? launch_conv<64, 128, 8, 1, 4, 10>(pp, q.srcs, pl, stream)
                              : launch_conv<64, 128, 4, 1, 4, 10>(pp, q.srcs, pl, stream);
    } else {
      rc = pl.variant == 10  ? launch_conv<32, 256, 12, 1, 4, 13, 1, 3>(pp, q.srcs, pl, stream)
           : pl.variant == 11 ? launch_conv<32, 128, 12, 1, 4, 13, 1, 3>(pp, q.srcs, pl, stream)
           : pl.variant == 0  ? launch_conv<32, 256, 4, 1, 4, 8>(pp, q.srcs, pl, stream)
           : pl.variant == 1  ? launch_conv<32, 128, 8, 1, 4, 10>(pp, q.srcs, pl, stream)
                              : launch_conv<32, 128, 4, 1, 4, 10>(pp, q.srcs, pl, stream);
    }
    if (rc) return rc;
  }
  return TOFU_OK;
}

// Shared by the two forward entry points: `x` is the single buffer that holds the input region,
// or NULL when the region is read from the `nsrc` blocks `x_srcs`.
static int shard_conv2d(const tofu_op_desc_t* op, const tofu_split_t* splits, int32_t nsplits, const tofu_tensor_t* x,
                        const tofu_tensor_t* x_srcs, int32_t nsrc, const tofu_tensor_t* w, const tofu_tensor_t* y, void* workspace,
                        size_t workspace_bytes, void* hip_stream, bool accumulate) {
  if (!op || op->kind != TOFU_OP_CONV2D) return fail(TOFU_ERR_INVALID_ARG, "operator description is not a conv2d");
  ConvProblem q;
  tofu_region_t in_boxes[2];
  int64_t pad_hi[2];
  int32_t partial = 0;
  int rc = tofu_op_regions(op, splits, nsplits, &q.out_box, in_boxes, q.pad_lo, pad_hi, &partial);
  if (rc) return rc;
  q.in_box = in_boxes[0];
  if (op->KH != 3 || op->KW != 3 || op->stride != 1 || op->pad > 1)
    return fail(TOFU_ERR_UNSUPPORTED, "conv2d kernels implement KH = KW = 3, stride 1, pad 0 or 1");
  const bool multi = x == nullptr;
  tofu_region_t inter[kMaxConvSources];
  if (multi) {
    if (nsrc < 1 || nsrc > kMaxConvSources) return fail(TOFU_ERR_INVALID_ARG, "nsrc = %d outside [1,%d]", (int)nsrc, kMaxConvSources);
    if (!x_srcs) return fail(TOFU_ERR_INVALID_ARG, "x_srcs is NULL");
    if ((rc = check_tiling("x_srcs", &in_boxes[0], x_srcs, nsrc, inter))) return rc;
  } else if ((rc = check_tensor("x", x, 4, &in_boxes[0]))) {
    return rc;
  }
  if ((rc = check_tensor("w", w, 4, &in_boxes[1]))) return rc;
  if ((rc = check_tensor("y", y, 4, &q.out_box))) return rc;
  if (volume(&q.out_box) == 0) return TOFU_OK;

  effective_strides(w, q.ws);
  effective_strides(y, q.ys);
  q.w = element_ptr(w, q.ws, in_boxes[1].lo);
  q.y = const_cast<float*>(element_ptr(y, q.ys, q.out_box.lo));
  ConvSources srcs;
  srcs.n = 0;
  q.srcs = nullptr;
  if (multi) {
    q.x = nullptr;
    for (int d = 0; d < 4; ++d) q.xs[d] = 0;
    for (int j = 0; j < nsrc; ++j) {
      if (volume(&inter[j]) == 0) continue;
      if (inter[j].lo[1] != in_boxes[0].lo[1] || inter[j].hi[1] != in_boxes[0].hi[1])
        return fail(TOFU_ERR_UNSUPPORTED, "conv2d: x_srcs[%d] holds only part of the region's channels; assemble the region with tofu_region_fetch", j);
      ConvSrc& S = srcs.src[srcs.n++];
      int64_t st[4];
      effective_strides(&x_srcs[j], st);
      S.base = element_ptr(&x_srcs[j], st, in_boxes[0].lo);
      for (int d = 0; d < 4; ++d) S.s[d] = st[d];
      if (st[1] >= ((int64_t)1 << 27) || st[1] <= -((int64_t)1 << 27))
        return fail(TOFU_ERR_UNSUPPORTED, "conv2d: channel stride of x_srcs[%d] does not fit the kernel's 32-bit step", j);
      const int dims[3] = {0, 2, 3};
      for (int i = 0; i < 3; ++i) {
        S.lo[i] = (int)(inter[j].lo[dims[i]] - in_boxes[0].lo[dims[i]]);
        S.hi[i] = (int)(inter[j].hi[dims[i]] - in_boxes[0].lo[dims[i]]);
      }
    }
    q.srcs = &srcs;
    // Blocks with one channel stride whose held parts lie within 2 GiB of each other are read as one buffer.
    const char* lo = nullptr;
    const char* hi = nullptr;
    bool alike = srcs.n > 0;
    int idx = 0;
    for (int j = 0; j < nsrc && alike; ++j) {
      if (volume(&inter[j]) == 0) continue;
      const ConvSrc& S = srcs.src[idx++];
      for (int d = 0; d < 4; ++d) alike = alike && S.s[d] >= 0;
      alike = alike && S.s[1] == srcs.src[0].s[1];
      int64_t st[4] = {S.s[0], S.s[1], S.s[2], S.s[3]};
      const char *blo, *bhi;
      box_byte_span(&x_srcs[j], st, &inter[j], &blo, &bhi);
      if (!lo || blo < lo) lo = blo;
      if (!hi || bhi > hi) hi = bhi;
    }
    if (alike && hi - lo < ((int64_t)1 << 31)) {
      q.x = reinterpret_cast<const float*>(lo);
      q.xs[1] = srcs.src[0].s[1];
      q.window_bytes = hi - lo;
    }
  } else {
    effective_strides(x, q.xs);
    q.x = element_ptr(x, q.xs, in_boxes[0].lo);
  }
  q.workspace = workspace;
  q.workspace_bytes = workspace_bytes;
  q.accumulate = accumulate;
  return conv_core(q, static_cast<hipStream_t>(hip_stream));
}

// out[(ci * CO + co) * 9 + t] = w[co, ci, 2 - t / 3, 2 - t % 3]: the filters of the data gradient
// seen as a forward convolution of dy.  A workgroup moves a block of kFlipCo x 32 (co, ci) pairs
// through LDS so that both the reads (runs along ci, tap) and the writes (runs along co, tap)
// are contiguous when the filters are dense; small blocks, so that a shard's filters make
// thousands of workgroups.
constexpr int kFlipCo = 8;
__global__ void __launch_bounds__(256) flip_filters_kernel(float* __restrict__ out, const float* __restrict__ w, int64_t s_co,
                                                           int64_t s_ci, int64_t s_kh, int64_t s_kw, int CO, int CI) {
  __shared__ float tile[kFlipCo][32 * 9 + 1];   // [co][ci * 9 + tap]
  const int co0 = blockIdx.x * kFlipCo, ci0 = blockIdx.y * 32;
  for (int i = threadIdx.x; i < kFlipCo * 288; i += 256) {
    const int co = i / 288, r = i - co * 288, ci = r / 9, tap = r - ci * 9;
    float v = 0.f;
    if (co0 + co < CO && ci0 + ci < CI) v = w[(co0 + co) * s_co + (ci0 + ci) * s_ci + (tap / 3) * s_kh + (tap % 3) * s_kw];
    tile[co][r] = v;
  }
  __syncthreads();
  for (int i = threadIdx.x; i < 32 * kFlipCo * 9; i += 256) {
    const int ci = i / (kFlipCo * 9), r = i - ci * (kFlipCo * 9), co = r / 9, t = r - co * 9;
    if (co0 + co < CO && ci0 + ci < CI) out[((int64_t)(ci0 + ci) * CO + co0 + co) * 9 + t] = tile[co][ci * 9 + 8 - t];
  }
}

// out[(m * K + k) * T + t] = w[m * s_m + k * s_k + t * s_t]: filters brought to the dense
// [m][k][taps] order the convolution kernel loads as vectors (conv1d keeps its filters as
// [ci][co][dx], Fig. 1).  A workgroup moves 32 x 32 (m, k) pairs through LDS: it reads runs along
// (m, t) for one k -- contiguous in such a source -- and writes runs along (k, t) for one m.
template <int T>
__global__ void __launch_bounds__(256) repack_filters_kernel(float* __restrict__ out, const float* __restrict__ w, int64_t s_m, int64_t s_k,
                                                             int64_t s_t, int M, int K) {
  __shared__ float tile[32][32 * T + 1];   // [k][m * T + t]
  const int m0 = blockIdx.x * 32, k0 = blockIdx.y * 32;
  for (int i = threadIdx.x; i < 32 * 32 * T; i += 256) {
    const int k = i / (32 * T), r = i - k * (32 * T), m = r / T, t = r - m * T;
    float v = 0.f;
    if (m0 + m < M && k0 + k < K) v = w[(int64_t)(m0 + m) * s_m + (int64_t)(k0 + k) * s_k + t * s_t];
    tile[k][r] = v;
  }
  __syncthreads();
  for (int i = threadIdx.x; i < 32 * 32 * T; i += 256) {
    const int m = i / (32 * T), r = i - m * (32 * T), k = r / T, t = r - k * T;
    if (m0 + m < M && k0 + k < K) out[((int64_t)(m0 + m) * K + k0 + k) * T + t] = tile[k][m * T + t];
  }
}

int64_t conv1d_chunk(int64_t bw) {
  // rows of d columns: a tile of 256 consecutive positions stages every row it touches, d + 2 floats each
  int64_t best = 1, best_score = -1;
  for (int64_t d = 1; d <= bw && d <= 272; ++d) {
    if (bw % d) continue;
    const int64_t rows = 256 % d == 0 ? 256 / d : 255 / d + 2;
    const int64_t score = rows * (d + 2);
    if (best_score < 0 || score <= best_score) { best = d; best_score = score; }
  }
  return best;
}

static int shard_conv1d(const tofu_op_desc_t* op, const tofu_split_t* splits, int32_t nsplits, const tofu_tensor_t* data,
                        const tofu_tensor_t* filters, const tofu_tensor_t* out, void* workspace, size_t workspace_bytes, void* hip_stream,
                        bool accumulate) {
  if (!op || op->kind != TOFU_OP_CONV1D) return fail(TOFU_ERR_INVALID_ARG, "operator description is not a conv1d");
  tofu_region_t out_box, in_boxes[2];
  int32_t partial = 0;
  int rc = tofu_op_regions(op, splits, nsplits, &out_box, in_boxes, nullptr, nullptr, &partial);
  if (rc) return rc;
  if (op->KW != 3) return fail(TOFU_ERR_UNSUPPORTED, "conv1d kernels implement a window of 3");
  if ((rc = check_tensor("data", data, 3, &in_boxes[0]))) return rc;
  if ((rc = check_tensor("filters", filters, 3, &in_boxes[1]))) return rc;
  if ((rc = check_tensor("out", out, 3, &out_box))) return rc;
  if (volume(&out_box) == 0) return TOFU_OK;
  const int64_t NB = out_box.hi[0] - out_box.lo[0], CO = out_box.hi[1] - out_box.lo[1], BW = out_box.hi[2] - out_box.lo[2];
  const int64_t CI = in_boxes[0].hi[1] - in_boxes[0].lo[1];
  if (CO >= (1 << 30) || CI >= (1 << 30)) return fail(TOFU_ERR_UNSUPPORTED, "conv1d shard extent exceeds 2^30");
  int64_t ds[3], fs[3], os[3];
  effective_strides(data, ds);
  effective_strides(filters, fs);
  effective_strides(out, os);

  // An output row of BW columns is handed to the convolution kernel as BW / CW rows of CW columns:
  // row r reads data columns [r * CW, r * CW + CW + 2), so consecutive rows overlap by the window.
  const int64_t CW = conv1d_chunk(BW), rows = BW / CW;
  ConvProblem q;
  q.KH = 1; q.KW = 3;
  q.pad_lo[0] = q.pad_lo[1] = 0;
  const int64_t olo[4] = {0, 0, 0, 0}, ohi[4] = {NB, CO, rows, CW}, ihi[4] = {NB, CI, rows, CW + 2};
  memset(&q.out_box, 0, sizeof(q.out_box));
  memset(&q.in_box, 0, sizeof(q.in_box));
  q.out_box.ndim = q.in_box.ndim = 4;
  for (int d = 0; d < 4; ++d) { q.out_box.lo[d] = q.in_box.lo[d] = olo[d]; q.out_box.hi[d] = ohi[d]; q.in_box.hi[d] = ihi[d]; }
  q.x = element_ptr(data, ds, in_boxes[0].lo);
  q.xs[0] = ds[0]; q.xs[1] = ds[1]; q.xs[2] = CW * ds[2]; q.xs[3] = ds[2];
  q.srcs = nullptr;
  q.y = const_cast<float*>(element_ptr(out, os, out_box.lo));
  q.ys[0] = os[0]; q.ys[1] = os[1]; q.ys[2] = CW * os[2]; q.ys[3] = os[2];
  q.accumulate = accumulate;

  // filters[ci][co][dx] seen as (co, ci, -, dx); a buffer that is physically [co][ci][dx] is used in place
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const float* f = element_ptr(filters, fs, in_boxes[1].lo);
  const bool in_place = fs[2] == 1 && fs[0] == 3 && fs[1] % 4 == 0 && fs[1] >= 3 * CI && (reinterpret_cast<uintptr_t>(f) & 15) == 0;
  const size_t repack_bytes = in_place ? 0 : ((size_t)CO * (size_t)CI * 3 * sizeof(float) + 255) / 256 * 256;
  const size_t need = repack_bytes + conv_workspace_bytes(NB * BW, rows, CW, CO, CI, 1, 3);
  if (need > 0) {
    if (!workspace || workspace_bytes < need)
      return fail(TOFU_ERR_WORKSPACE_TOO_SMALL, "conv1d shard needs %zu workspace bytes, got %zu", need, workspace ? workspace_bytes : (size_t)0);
    if (reinterpret_cast<uintptr_t>(workspace) & 15) return fail(TOFU_ERR_INVALID_ARG, "workspace must be 16-byte aligned");
  }
  if (in_place) {
    q.w = f;
    q.ws[0] = fs[1]; q.ws[1] = fs[0]; q.ws[2] = 0; q.ws[3] = fs[2];
  } else {
    hipLaunchKernelGGL(repack_filters_kernel<3>, dim3((unsigned)((CO + 31) / 32), (unsigned)((CI + 31) / 32)), dim3(256), 0, stream,
                       static_cast<float*>(workspace), f, fs[1], fs[0], fs[2], (int)CO, (int)CI);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(TOFU_ERR_HIP, "conv1d filter launch failed: %s", hipGetErrorString(e));
    q.w = static_cast<const float*>(workspace);
    q.ws[0] = CI * 3; q.ws[1] = 3; q.ws[2] = 0; q.ws[3] = 1;
  }
  q.workspace = workspace ? static_cast<char*>(workspace) + repack_bytes : nullptr;
  q.workspace_bytes = workspace ? workspace_bytes - repack_bytes : 0;
  return conv_core(q, stream);
}

}  // namespace tofu

extern "C" int tofu_shard_conv1d(const tofu_op_desc_t* op, const tofu_split_t* splits, int32_t nsplits,
                                 const tofu_tensor_t* data, const tofu_tensor_t* filters, const tofu_tensor_t* out, void* workspace,
                                 size_t workspace_bytes, void* hip_stream) {
  return tofu::shard_conv1d(op, splits, nsplits, data, filters, out, workspace, workspace_bytes, hip_stream, false);
}

extern "C" int tofu_shard_conv1d_accumulate(const tofu_op_desc_t* op, const tofu_split_t* splits, int32_t nsplits,
                                            const tofu_tensor_t* data, const tofu_tensor_t* filters, const tofu_tensor_t* out,
                                            void* workspace, size_t workspace_bytes, void* hip_stream) {
  return tofu::shard_conv1d(op, splits, nsplits, data, filters, out, workspace, workspace_bytes, hip_stream, true);
}

extern "C" int tofu_shard_conv2d(const tofu_op_desc_t* op, const tofu_split_t* splits, int32_t nsplits,
                                 const tofu_tensor_t* x, const tofu_tensor_t* w, const tofu_tensor_t* y, void* workspace,
                                 size_t workspace_bytes, void* hip_stream) {
  if (!x) return tofu::fail(TOFU_ERR_INVALID_ARG, "x is NULL");
  return tofu::shard_conv2d(op, splits, nsplits, x, nullptr, 0, w, y, workspace, workspace_bytes, hip_stream, false);
}

extern "C" int tofu_shard_conv2d_accumulate(const tofu_op_desc_t* op, const tofu_split_t* splits, int32_t nsplits,
                                            const tofu_tensor_t* x, const tofu_tensor_t* w, const tofu_tensor_t* y, void* workspace,
                                            size_t workspace_bytes, void* hip_stream) {
  if (!x) return tofu::fail(TOFU_ERR_INVALID_ARG, "x is NULL");
  return tofu::shard_conv2d(op, splits, nsplits, x, nullptr, 0, w, y, workspace, workspace_bytes, hip_stream, true);
}

extern "C" int tofu_shard_conv2d_fused(const tofu_op_desc_t* op, const tofu_split_t* splits, int32_t nsplits,
                                       const tofu_tensor_t* x_srcs, int32_t nsrc, const tofu_tensor_t* w, const tofu_tensor_t* y,
                                       void* workspace, size_t workspace_bytes, void* hip_stream) {
  return tofu::shard_conv2d(op, splits, nsplits, nullptr, x_srcs, nsrc, w, y, workspace, workspace_bytes, hip_stream, false);
}

namespace tofu {
static int shard_dgrad(const tofu_op_desc_t* op, const tofu_split_t* splits, int32_t nsplits, const tofu_tensor_t* dy,
                       const tofu_tensor_t* w, const tofu_tensor_t* dx, void* workspace, size_t workspace_bytes, void* hip_stream,
                       bool accumulate) {
  if (!op || op->kind != TOFU_OP_CONV2D_DGRAD) return fail(TOFU_ERR_INVALID_ARG, "operator description is not a conv2d data gradient");
  ConvProblem q;
  tofu_region_t in_boxes[2];
  int64_t pad_hi[2];
  int32_t partial = 0;
  int rc = tofu_op_regions(op, splits, nsplits, &q.out_box, in_boxes, q.pad_lo, pad_hi, &partial);
  if (rc) return rc;
  q.in_box = in_boxes[0];
  if (op->KH != 3 || op->KW != 3 || op->stride != 1 || op->pad != 1)
    return fail(TOFU_ERR_UNSUPPORTED, "conv2d data-gradient kernels implement KH = KW = 3, stride 1, pad 1");
  if ((rc = check_tensor("dy", dy, 4, &in_boxes[0]))) return rc;
  if ((rc = check_tensor("w", w, 4, &in_boxes[1]))) return rc;
  if ((rc = check_tensor("dx", dx, 4, &q.out_box))) return rc;
  if (volume(&q.out_box) == 0) return TOFU_OK;
  const int64_t CO = in_boxes[1].hi[0] - in_boxes[1].lo[0], CI = in_boxes[1].hi[1] - in_boxes[1].lo[1];
  if (CO >= (1 << 30) || CI >= (1 << 30)) return fail(TOFU_ERR_UNSUPPORTED, "conv2d shard extent exceeds 2^30");
  // workspace = reversed filters, then (from the next 256-byte boundary) the convolution's segment slots
  const size_t flip_bytes = ((size_t)CO * (size_t)CI * 9 * sizeof(float) + 255) / 256 * 256;
  const int64_t P = (q.out_box.hi[0] - q.out_box.lo[0]) * (q.out_box.hi[2] - q.out_box.lo[2]) * (q.out_box.hi[3] - q.out_box.lo[3]);
  const size_t need = flip_bytes + conv_workspace_bytes(P, q.out_box.hi[2] - q.out_box.lo[2], q.out_box.hi[3] - q.out_box.lo[3], CI, CO);
  if (!workspace || workspace_bytes < need)
    return fail(TOFU_ERR_WORKSPACE_TOO_SMALL, "conv2d data-gradient shard needs %zu workspace bytes, got %zu", need, workspace ? workspace_bytes : (size_t)0);
  if (reinterpret_cast<uintptr_t>(workspace) & 15) return fail(TOFU_ERR_INVALID_ARG, "workspace must be 16-byte aligned");

  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  int64_t wst[4];
  effective_strides(w, wst);
  hipLaunchKernelGGL(flip_filters_kernel, dim3((unsigned)((CO + kFlipCo - 1) / kFlipCo), (unsigned)((CI + 31) / 32)), dim3(256), 0, stream,
                     static_cast<float*>(workspace), element_ptr(w, wst, in_boxes[1].lo), wst[0], wst[1], wst[2], wst[3], (int)CO, (int)CI);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(TOFU_ERR_HIP, "conv2d data-gradient filter launch failed: %s", hipGetErrorString(e));

  // dx = forward convolution of dy with the reversed filters [ci][co][3][3]
  effective_strides(dy, q.xs);
  effective_strides(dx, q.ys);
  q.x = element_ptr(dy, q.xs, in_boxes[0].lo);
  q.srcs = nullptr;
  q.w = static_cast<const float*>(workspace);
  q.ws[0] = CO * 9; q.ws[1] = 9; q.ws[2] = 3; q.ws[3] = 1;
  q.y = const_cast<float*>(element_ptr(dx, q.ys, q.out_box.lo));
  q.workspace = static_cast<char*>(workspace) + flip_bytes;
  q.workspace_bytes = workspace_bytes - flip_bytes;
  q.accumulate = accumulate;
  return conv_core(q, stream);
}
}  // namespace tofu

extern "C" int tofu_shard_conv2d_dgrad(const tofu_op_desc_t* op, const tofu_split_t* splits, int32_t nsplits,
                                       const tofu_tensor_t* dy, const tofu_tensor_t* w, const tofu_tensor_t* dx, void* workspace,
                                       size_t workspace_bytes, void* hip_stream) {
  return tofu::shard_dgrad(op, splits, nsplits, dy, w, dx, workspace, workspace_bytes, hip_stream, false);
}

extern "C" int tofu_shard_conv2d_dgrad_accumulate(const tofu_op_desc_t* op, const tofu_split_t* splits, int32_t nsplits,
                                                  const tofu_tensor_t* dy, const tofu_tensor_t* w, const tofu_tensor_t* dx,
                                                  void* workspace, size_t workspace_bytes, void* hip_stream) {
  return tofu::shard_dgrad(op, splits, nsplits, dy, w, dx, workspace, workspace_bytes, hip_stream, true);
}
