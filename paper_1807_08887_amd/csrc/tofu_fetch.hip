// Fused region fetch (arXiv 1807.08887 Sec. 6, "MultiFetch"): one launch takes the pointers of
// all blocks that hold parts of a worker's input region and assembles the region in place,
// instead of split -> copy -> concatenate with an intermediate buffer per step.
//
// Host side: intersect every source block with the destination box and prove from the boxes
// alone that the intersections tile the destination exactly.  Dimensions that are contiguous in
// the destination and in every source (and that no source cuts) are merged, so the halo fetch
// of a [N,C,8,14] region from a [N,C,7,14] block and a [N,C,1,14] block becomes
// rows x 112 floats = 98 from one pointer ++ 14 from the other.
// Device side, destination-driven: a lane owns one vector position inside a row (so neighbouring
// lanes write neighbouring bytes and every destination line is written whole, whichever source
// it comes from), looks up the source that holds that position ONCE, and then walks down the
// rows with constant pointer increments: the loop body is UNROLL loads, UNROLL stores and two
// 64-bit adds.  A workgroup owns a short run of consecutive rows (one trip of UNROLL loads per
// lane unless the region has more rows than the grid can number).  When a source cuts the outermost dimension there is a single "row" and the
// kernel degenerates to one lookup + one copy per lane.  Pure HBM stream: 1 read + 1 write per
// element; loads are ordinary, stores carry the streaming (nontemporal) hint, which measured
// fastest of the four combinations on MI355X.
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <string.h>

#include "tofu_internal.h"

namespace tofu {

constexpr int kMaxFetchSources = 16;

// n / d for any 32-bit n via one multiply-high: q = (mulhi(n, m) + n) >> s with the 33-bit
// magic 2^32 + m = ceil(2^(32+s) / d), s = ceil(log2 d)  (Granlund & Montgomery, 1994).
struct FastDiv {
  uint32_t d, m, s;
};
static FastDiv make_fastdiv(uint32_t d) {
  FastDiv f;
  f.d = d;
  uint32_t s = 0;
  while (((uint64_t)1 << s) < d) ++s;
  f.s = s;
  f.m = (uint32_t)(((((uint64_t)1 << s) - d) << 32) / d + 1);
  return f;
}
__device__ __forceinline__ uint32_t fdiv(uint32_t n, const FastDiv& f) {
  return (uint32_t)(((uint64_t)__umulhi(n, f.m) + n) >> f.s);
}

// After merging, dimension 0 is the "row" (outer) index when no source cuts it, and dimensions
// 1..n_inner are the coordinates inside a row; all boxes are relative to the destination box.
// Strides are kept in 32 bits (checked on the host) so that index * stride is one 32x32->64 multiply.
struct FetchSource {
  const float* base;                 // element at (row 0, inner coordinate 0 of the destination box)
  int32_t row_stride;                // elements between rows
  int32_t stride[TOFU_MAX_DIMS];     // element strides of the inner dimensions
  int32_t lo[TOFU_MAX_DIMS];         // inner box held by this source, half-open
  int32_t hi[TOFU_MAX_DIMS];
};

struct FetchPlan {
  float* dst;                        // element at the low corner of the destination box
  int32_t dst_row_stride;
  int32_t dst_stride[TOFU_MAX_DIMS];
  FastDiv size[TOFU_MAX_DIMS];       // inner extents, innermost first; the innermost is in vectors
  int32_t n_inner;
  int32_t vec;                       // floats per vector: 4, 2 or 1
  int32_t n_src;
  uint32_t row_vecs;                 // vectors in one row
  FastDiv row_vecs_div;              // same, for thread -> (row of the workgroup, vector of the row)
  uint32_t rows;                     // number of rows
  uint32_t rows_per_block;           // rows a workgroup covers per trip (row_vecs <= 256), else 1
  uint32_t rows_per_group;           // consecutive rows owned by one workgroup (multiple of rows_per_block)
  FetchSource src[kMaxFetchSources];
};

template <int VEC> struct VecT;
template <> struct VecT<4> { typedef float type __attribute__((ext_vector_type(4))); };
template <> struct VecT<2> { typedef float type __attribute__((ext_vector_type(2))); };
template <> struct VecT<1> { typedef float type; };

// FLAT > 0: a row has a single (merged) inner dimension and at most FLAT sources.  The lane's
// coordinate is then its vector index, and the source table is read with constant indices, so
// all table reads are issued together at the top of the kernel instead of one dependent scalar
// round trip per source (a wavefront only lives for a few microseconds here).
template <int VEC, int UNROLL, int FLAT>
__global__ void __launch_bounds__(256) fetch_kernel(const FetchPlan t) {
  typedef typename VecT<VEC>::type V;
  // Which vector of the row; which rows.  A workgroup owns a run of consecutive rows (its trips
  // then touch neighbouring DRAM pages, which measured ~7 % faster than striding the whole
  // region) and covers rows_per_block of them per trip.
  uint32_t col, row;
  const uint32_t row_step = t.rows_per_block;
  const uint32_t row_end = min(t.rows, (blockIdx.y + 1) * t.rows_per_group);
  if (t.rows_per_block > 1) {
    const uint32_t sub = fdiv(threadIdx.x, t.row_vecs_div);   // small rows: several rows per workgroup
    col = threadIdx.x - sub * t.row_vecs;
    if (sub >= t.rows_per_block) return;
    row = blockIdx.y * t.rows_per_group + sub;
  } else {
    col = blockIdx.x * blockDim.x + threadIdx.x;
    if (col >= t.row_vecs) return;
    row = blockIdx.y * t.rows_per_group;
  }
  if (row >= row_end) return;

  // inner coordinates of this lane's vector (innermost coordinate in floats), once
  int32_t coord[TOFU_MAX_DIMS];
  uint32_t rest = col;
  int64_t d_off = 0;
#pragma unroll
  for (int i = 0; i < (FLAT ? 1 : TOFU_MAX_DIMS); ++i) {      // i = 0 is the innermost dimension
    coord[i] = 0;
    if (FLAT) {
      coord[0] = (int32_t)(col * VEC);
      d_off = (int64_t)coord[0] * t.dst_stride[0];
    } else if (i < t.n_inner) {
      const uint32_t q = fdiv(rest, t.size[i]);
      const uint32_t r = rest - q * t.size[i].d;
      coord[i] = (int32_t)(i == 0 ? r * VEC : r);
      d_off += (int64_t)coord[i] * t.dst_stride[i];           // 32 x 32 -> 64
      rest = q;
    }
  }
  // the source that holds this position: every candidate address is formed from scalar table
  // reads (the loop index is wave-uniform) and the lane keeps the one whose box contains it
  const float* s = nullptr;
  int64_t s_step = 0;
#pragma unroll
  for (int j = 0; j < (FLAT ? FLAT : kMaxFetchSources); ++j) {
    if (!FLAT && j >= t.n_src) break;
    const FetchSource& sc = t.src[j];        // unused slots of a FLAT plan have an empty box
    bool inside = true;
    int64_t off = (int64_t)(int32_t)row * sc.row_stride;
#pragma unroll
    for (int i = 0; i < (FLAT ? 1 : TOFU_MAX_DIMS); ++i) {
      if (FLAT || i < t.n_inner) {                           // uniform; no early exit, so reads stay scalar
        inside = inside & (coord[i] >= sc.lo[i]) & (coord[i] < sc.hi[i]);
        off += (int64_t)coord[i] * sc.stride[i];
      }
    }
    const float* cand = sc.base + off;
    const int64_t cand_step = (int64_t)(int32_t)row_step * sc.row_stride;
    s = inside ? cand : s;
    s_step = inside ? cand_step : s_step;
  }
  float* d = t.dst + d_off + (int64_t)(int32_t)row * t.dst_row_stride;
  const int64_t d_step = (int64_t)(int32_t)row_step * t.dst_row_stride;

  for (; row + (UNROLL - 1) * row_step < row_end; row += UNROLL * row_step) {
    V v[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) v[u] = *reinterpret_cast<const V*>(s + u * s_step);
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) __builtin_nontemporal_store(v[u], reinterpret_cast<V*>(d + u * d_step));
    s += UNROLL * s_step;
    d += UNROLL * d_step;
  }
  for (; row < row_end; row += row_step) {
    __builtin_nontemporal_store(*reinterpret_cast<const V*>(s), reinterpret_cast<V*>(d));
    s += s_step;
    d += d_step;
  }
}

// Lowest and one-past-highest byte address a tensor's extent can touch.
static void byte_span(const tofu_tensor_t* t, const int64_t* stride, const char** lo, const char** hi) {
  box_byte_span(t, stride, &t->extent, lo, hi);
}

}  // namespace tofu

extern "C" int tofu_region_fetch(const tofu_tensor_t* dst, const tofu_tensor_t* srcs, int32_t nsrc, void* hip_stream) {
  using namespace tofu;
  if (!dst) return fail(TOFU_ERR_INVALID_ARG, "dst is NULL");
  const int nd = dst->extent.ndim;
  if (nd < 1 || nd > TOFU_MAX_DIMS) return fail(TOFU_ERR_INVALID_ARG, "dst ndim %d outside [1,%d]", nd, TOFU_MAX_DIMS);
  int rc = check_tensor("dst", dst, nd, nullptr);
  if (rc) return rc;
  if (nsrc < 0 || nsrc > kMaxFetchSources) return fail(TOFU_ERR_INVALID_ARG, "nsrc = %d outside [0,%d]", (int)nsrc, kMaxFetchSources);
  if (nsrc > 0 && !srcs) return fail(TOFU_ERR_INVALID_ARG, "srcs is NULL");
  const int64_t want = volume(&dst->extent);
  if (want == 0) return TOFU_OK;
  if (!dst->data) return fail(TOFU_ERR_INVALID_ARG, "dst has a NULL data pointer");

  int64_t dstr[TOFU_MAX_DIMS];
  effective_strides(dst, dstr);
  const char *dlo, *dhi;
  byte_span(dst, dstr, &dlo, &dhi);

  // ---- intersections and the exact-tiling proof ----
  tofu_region_t inter[kMaxFetchSources];
  if ((rc = check_tiling("srcs", &dst->extent, srcs, nsrc, inter))) return rc;

  // ---- gather the live sources: strides, and their boxes relative to the destination box ----
  struct Live {
    const float* base;
    int64_t stride[TOFU_MAX_DIMS];
    int64_t lo[TOFU_MAX_DIMS], hi[TOFU_MAX_DIMS];
  } live[kMaxFetchSources];
  int n_live = 0;
  for (int j = 0; j < nsrc; ++j) {
    if (volume(&inter[j]) == 0) continue;
    int64_t sstr[TOFU_MAX_DIMS];
    effective_strides(&srcs[j], sstr);
    const char *slo, *shi;
    byte_span(&srcs[j], sstr, &slo, &shi);
    if (slo < dhi && dlo < shi) return fail(TOFU_ERR_INVALID_ARG, "dst overlaps srcs[%d] in memory", j);
    Live& L = live[n_live++];
    L.base = element_ptr(&srcs[j], sstr, dst->extent.lo);   // address the destination's low corner WOULD have in this source
    for (int d = 0; d < nd; ++d) {
      L.stride[d] = sstr[d];
      L.lo[d] = inter[j].lo[d] - dst->extent.lo[d];
      L.hi[d] = inter[j].hi[d] - dst->extent.lo[d];
    }
  }

  // ---- merge neighbouring dimensions that are contiguous everywhere and cut by nobody ----
  int64_t size[TOFU_MAX_DIMS], ds[TOFU_MAX_DIMS];
  int m = 0;
  for (int d = 0; d < nd; ++d) {
    const int64_t e = dst->extent.hi[d] - dst->extent.lo[d];
    bool merge = m > 0 && ds[m - 1] == e * dstr[d];
    for (int j = 0; j < n_live && merge; ++j)
      merge = live[j].lo[d] == 0 && live[j].hi[d] == e && live[j].stride[m - 1] == e * live[j].stride[d];
    // live[j].stride/lo/hi are rewritten in place in merged numbering; index m-1 is already merged, index d is raw
    if (merge) {
      size[m - 1] *= e;
      ds[m - 1] = dstr[d];
      for (int j = 0; j < n_live; ++j) {
        live[j].lo[m - 1] *= e;
        live[j].hi[m - 1] *= e;
        live[j].stride[m - 1] = live[j].stride[d];
      }
    } else {
      size[m] = e;
      ds[m] = dstr[d];
      for (int j = 0; j < n_live; ++j) {
        live[j].lo[m] = live[j].lo[d];
        live[j].hi[m] = live[j].hi[d];
        live[j].stride[m] = live[j].stride[d];
      }
      ++m;
    }
  }
  // dimension 0 becomes the row index when every source spans it; otherwise there is one row
  bool has_rows = m > 1;
  for (int j = 0; j < n_live && has_rows; ++j) has_rows = live[j].lo[0] == 0 && live[j].hi[0] == size[0];
  const int first_inner = has_rows ? 1 : 0;
  const int n_inner = m - first_inner;
  const int last = m - 1;

  // ---- widest vector every address and every source boundary allows ----
  int vec = 1;
  for (int v = 4; v > 1; v /= 2) {
    bool ok = ds[last] == 1 && size[last] % v == 0 &&
              (reinterpret_cast<uintptr_t>(element_ptr(dst, dstr, dst->extent.lo)) % (4 * v)) == 0;
    for (int d = 0; d < last && ok; ++d) ok = ds[d] % v == 0;
    for (int j = 0; j < n_live && ok; ++j) {
      ok = live[j].stride[last] == 1 && live[j].lo[last] % v == 0 && live[j].hi[last] % v == 0 &&
           (reinterpret_cast<uintptr_t>(live[j].base) % (4 * v)) == 0;
      for (int d = 0; d < last && ok; ++d) ok = live[j].stride[d] % v == 0;
    }
    if (ok) { vec = v; break; }
  }

  FetchPlan plan;
  memset(&plan, 0, sizeof(plan));
  plan.dst = const_cast<float*>(element_ptr(dst, dstr, dst->extent.lo));
  plan.vec = vec;
  plan.n_inner = n_inner;
  plan.n_src = n_live;
  plan.rows = has_rows ? (uint32_t)size[0] : 1;
  auto fits32 = [](int64_t v) { return v > -((int64_t)1 << 31) && v < ((int64_t)1 << 31); };
  bool strides_fit = !has_rows || fits32(ds[0]);
  for (int d = 0; d < m; ++d) {
    strides_fit = strides_fit && fits32(ds[d]);
    for (int j = 0; j < n_live; ++j) strides_fit = strides_fit && fits32(live[j].stride[d]);
  }
  if (!strides_fit) return fail(TOFU_ERR_UNSUPPORTED, "fetch: an element stride does not fit 32 bits");
  plan.dst_row_stride = has_rows ? (int32_t)ds[0] : 0;
  int64_t row_vecs = 1;
  for (int i = 0; i < n_inner; ++i) {            // innermost first
    const int d = last - i;
    int64_t e = i == 0 ? size[d] / vec : size[d];
    if (e >= ((int64_t)1 << 31)) return fail(TOFU_ERR_UNSUPPORTED, "fetch: a merged extent exceeds 2^31");
    plan.size[i] = make_fastdiv((uint32_t)e);
    plan.dst_stride[i] = (int32_t)ds[d];
    row_vecs *= e;
  }
  if (row_vecs >= ((int64_t)1 << 31) || (has_rows && size[0] >= ((int64_t)1 << 31)))
    return fail(TOFU_ERR_UNSUPPORTED, "fetch: the region has 2^31 or more vectors per row or rows; split the call");
  plan.row_vecs = (uint32_t)row_vecs;
  plan.row_vecs_div = make_fastdiv((uint32_t)row_vecs);
  for (int j = 0; j < n_live; ++j) {
    FetchSource& sc = plan.src[j];
    sc.base = live[j].base;
    sc.row_stride = has_rows ? (int32_t)live[j].stride[0] : 0;
    for (int i = 0; i < n_inner; ++i) {
      const int d = last - i;
      sc.stride[i] = (int32_t)live[j].stride[d];
      sc.lo[i] = (int32_t)live[j].lo[d];
      sc.hi[i] = (int32_t)live[j].hi[d];
    }
  }

  // ---- launch shape: lanes along a row, workgroups (and trips) down the rows ----
  // A workgroup owns UNROLL trips' worth of consecutive rows, so every lane has all its loads in
  // flight at once and then only stores: many short workgroups measured faster than fewer that
  // loop (48.3 us against 49.5 - 60 us for the 294 MB halo fetch as the rows per workgroup grow).
  constexpr int kUnroll = 4;
  constexpr int64_t kMaxGroups = 65535;          // grid.y limit
  dim3 grid;
  if (row_vecs <= 256) {
    plan.rows_per_block = (uint32_t)(256 / row_vecs);
    grid.x = 1;
  } else {
    plan.rows_per_block = 1;
    grid.x = (unsigned)((row_vecs + 255) / 256);
  }
  // consecutive rows per workgroup: a whole number of trips, at least one
  int64_t per = (int64_t)plan.rows_per_block * kUnroll;
  if ((plan.rows + per - 1) / per > kMaxGroups) per = (plan.rows + kMaxGroups - 1) / kMaxGroups;
  per = (per + plan.rows_per_block - 1) / plan.rows_per_block * plan.rows_per_block;
  plan.rows_per_group = (uint32_t)per;
  grid.y = (unsigned)((plan.rows + per - 1) / per);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const int flat = n_inner != 1 ? 0 : n_live <= 2 ? 2 : n_live <= 4 ? 4 : 0;
  // whole rows per workgroup: no more lanes than rows_per_block rows need (rounded to wavefronts)
  const unsigned threads = row_vecs <= 256 ? (unsigned)((plan.rows_per_block * row_vecs + 63) / 64 * 64) : 256u;
#define TOFU_FETCH_LAUNCH(V)                                                                                   \
  do {                                                                                                         \
    if (flat == 2) hipLaunchKernelGGL((fetch_kernel<V, kUnroll, 2>), grid, dim3(threads), 0, s, plan);         \
    else if (flat == 4) hipLaunchKernelGGL((fetch_kernel<V, kUnroll, 4>), grid, dim3(threads), 0, s, plan);    \
    else hipLaunchKernelGGL((fetch_kernel<V, kUnroll, 0>), grid, dim3(threads), 0, s, plan);                   \
  } while (0)
  if (vec == 4) TOFU_FETCH_LAUNCH(4);
  else if (vec == 2) TOFU_FETCH_LAUNCH(2);
  else TOFU_FETCH_LAUNCH(1);
#undef TOFU_FETCH_LAUNCH
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(TOFU_ERR_HIP, "fetch launch failed: %s", hipGetErrorString(e));
  return TOFU_OK;
}
