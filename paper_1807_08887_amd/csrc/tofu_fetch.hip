// Fused region fetch (arXiv 1807.08887 Sec. 6, "MultiFetch"): one launch takes the pointers of
// all blocks that hold parts of a worker's input region and assembles the region in place,
// instead of split -> copy -> concatenate with an intermediate buffer per step.
//
// Host side: intersect every source block with the destination box, prove from the boxes alone
// that the intersections tile the destination exactly, and turn each intersection into a
// "piece": a strided set of contiguous runs.  Adjacent dimensions that are contiguous in both
// the source and the destination are merged so runs are as long as the layouts allow, and the
// widest vector (16, 8 or 4 bytes) that both sides' alignment permits is chosen per piece.
// Device side: a flat index space over all pieces' vectors; a lane finds its piece from a short
// prefix table kept in kernel arguments, decodes its run with multiply-shift division and moves
// UNROLL independent vectors per trip.  The kernel is a pure HBM stream: 1 read + 1 write per
// element.
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <string.h>

#include "tofu_internal.h"

namespace tofu {

constexpr int kMaxFetchSources = 16;
constexpr int kMaxOuter = TOFU_MAX_DIMS - 1;

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

struct FetchPiece {
  const float* src;            // element at the piece's low corner
  float* dst;
  int64_t sstride[kMaxOuter];  // element strides of the outer (run-index) dimensions
  int64_t dstride[kMaxOuter];
  FastDiv size[kMaxOuter];     // extents of the outer dimensions, innermost outer dim first
  FastDiv vec_per_run;         // vectors in one contiguous run
  int64_t s_inner, d_inner;    // element stride along the run (1 when vectorised)
  int32_t n_outer;
  int32_t vec;                 // floats per vector: 4, 2 or 1
  int64_t item_begin;          // first flat item index of this piece
};

struct FetchTable {
  int32_t n_pieces;
  int64_t n_items;
  FetchPiece piece[kMaxFetchSources];
};

template <int VEC> struct VecT;
template <> struct VecT<4> { typedef float type __attribute__((ext_vector_type(4))); };
template <> struct VecT<2> { typedef float type __attribute__((ext_vector_type(2))); };
template <> struct VecT<1> { typedef float type; };

// Find the piece that owns flat item `item` and the addresses it moves.  The loop index is
// wave-uniform, so every table access is a scalar load from the kernel-argument segment.
__device__ __forceinline__ int locate(const FetchTable& t, int64_t item, const float** s, float** d) {
  int vec = 0;
  for (int p = 0; p < t.n_pieces; ++p) {
    const FetchPiece& pc = t.piece[p];
    const int64_t end = p + 1 < t.n_pieces ? t.piece[p + 1].item_begin : t.n_items;
    if (item < pc.item_begin || item >= end) continue;
    uint32_t local = (uint32_t)(item - pc.item_begin);
    uint32_t run = fdiv(local, pc.vec_per_run);
    uint32_t c = local - run * pc.vec_per_run.d;
    int64_t so = (int64_t)c * pc.vec * pc.s_inner, dofs = (int64_t)c * pc.vec * pc.d_inner;
    for (int i = 0; i < pc.n_outer; ++i) {
      uint32_t q = fdiv(run, pc.size[i]);
      uint32_t r = run - q * pc.size[i].d;
      so += (int64_t)r * pc.sstride[i];
      dofs += (int64_t)r * pc.dstride[i];
      run = q;
    }
    *s = pc.src + so;
    *d = pc.dst + dofs;
    vec = pc.vec;
  }
  return vec;
}

template <int UNROLL>
__global__ void __launch_bounds__(256) fetch_kernel(const FetchTable t) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t base = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; base < t.n_items; base += UNROLL * stride) {
    const float* s[UNROLL];
    float* d[UNROLL];
    int vec[UNROLL];
    VecT<4>::type v4[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      int64_t item = base + u * stride;
      vec[u] = 0;
      if (item < t.n_items) vec[u] = locate(t, item, &s[u], &d[u]);
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      if (vec[u] == 4) {
        v4[u] = __builtin_nontemporal_load(reinterpret_cast<const VecT<4>::type*>(s[u]));
      } else if (vec[u] == 2) {
        VecT<2>::type v = __builtin_nontemporal_load(reinterpret_cast<const VecT<2>::type*>(s[u]));
        v4[u].x = v.x; v4[u].y = v.y;
      } else if (vec[u] == 1) {
        v4[u].x = __builtin_nontemporal_load(s[u]);
      }
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      if (vec[u] == 4) {
        __builtin_nontemporal_store(v4[u], reinterpret_cast<VecT<4>::type*>(d[u]));
      } else if (vec[u] == 2) {
        VecT<2>::type v; v.x = v4[u].x; v.y = v4[u].y;
        __builtin_nontemporal_store(v, reinterpret_cast<VecT<2>::type*>(d[u]));
      } else if (vec[u] == 1) {
        __builtin_nontemporal_store(v4[u].x, d[u]);
      }
    }
  }
}

// Lowest and one-past-highest byte address a tensor's extent can touch.
static void byte_span(const tofu_tensor_t* t, const int64_t* stride, const char** lo, const char** hi) {
  int64_t min_off = 0, max_off = 0;
  for (int d = 0; d < t->extent.ndim; ++d) {
    int64_t e = t->extent.hi[d] - t->extent.lo[d] - 1;
    if (e < 0) e = 0;
    if (stride[d] >= 0) max_off += e * stride[d]; else min_off += e * stride[d];
  }
  *lo = static_cast<const char*>(t->data) + min_off * (int64_t)sizeof(float);
  *hi = static_cast<const char*>(t->data) + (max_off + 1) * (int64_t)sizeof(float);
}

static int build_piece(const tofu_tensor_t* dst, const int64_t* dstr, const tofu_tensor_t* src, const int64_t* sstr,
                       const tofu_region_t* box, FetchPiece* pc) {
  // gather dimensions with extent > 1, outermost first
  int n = 0;
  int64_t size[TOFU_MAX_DIMS], ss[TOFU_MAX_DIMS], ds[TOFU_MAX_DIMS];
  for (int d = 0; d < box->ndim; ++d) {
    int64_t e = box->hi[d] - box->lo[d];
    if (e == 1) continue;
    size[n] = e; ss[n] = sstr[d]; ds[n] = dstr[d]; ++n;
  }
  // merge neighbours that are contiguous on both sides
  int m = 0;
  for (int i = 0; i < n; ++i) {
    if (m > 0 && ss[m - 1] == size[i] * ss[i] && ds[m - 1] == size[i] * ds[i]) {
      size[m - 1] *= size[i]; ss[m - 1] = ss[i]; ds[m - 1] = ds[i];
    } else {
      size[m] = size[i]; ss[m] = ss[i]; ds[m] = ds[i]; ++m;
    }
  }
  if (m == 0) { size[0] = 1; ss[0] = 1; ds[0] = 1; m = 1; }   // a single element
  pc->src = element_ptr(src, sstr, box->lo);
  pc->dst = const_cast<float*>(element_ptr(dst, dstr, box->lo));
  int64_t run = size[m - 1];
  pc->s_inner = ss[m - 1];
  pc->d_inner = ds[m - 1];
  int vec = 1;
  if (pc->s_inner == 1 && pc->d_inner == 1) {
    for (int v = 4; v > 1; v /= 2) {
      bool ok = run % v == 0 && (reinterpret_cast<uintptr_t>(pc->src) % (4 * v)) == 0 &&
                (reinterpret_cast<uintptr_t>(pc->dst) % (4 * v)) == 0;
      for (int i = 0; i + 1 < m; ++i) ok = ok && ss[i] % v == 0 && ds[i] % v == 0;
      if (ok) { vec = v; break; }
    }
  }
  pc->vec = vec;
  int64_t items = run / vec, runs = 1;
  pc->n_outer = m - 1;
  for (int i = 0; i < m - 1; ++i) {          // innermost outer dimension first
    int src_i = m - 2 - i;
    if (size[src_i] >= ((int64_t)1 << 31)) return fail(TOFU_ERR_UNSUPPORTED, "fetch: a merged extent exceeds 2^31");
    pc->size[i] = make_fastdiv((uint32_t)size[src_i]);
    pc->sstride[i] = ss[src_i];
    pc->dstride[i] = ds[src_i];
    runs *= size[src_i];
  }
  if (items >= ((int64_t)1 << 31) || runs * items >= ((int64_t)1 << 31))
    return fail(TOFU_ERR_UNSUPPORTED, "fetch: one source contributes 2^31 or more vectors; split the call");
  pc->vec_per_run = make_fastdiv((uint32_t)items);
  pc->item_begin = runs * items;   // caller turns counts into a prefix
  return TOFU_OK;
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

  tofu_region_t inter[kMaxFetchSources];
  int64_t covered = 0;
  for (int j = 0; j < nsrc; ++j) {
    char name[24];
    snprintf(name, sizeof(name), "srcs[%d]", j);
    rc = check_tensor(name, &srcs[j], nd, nullptr);
    if (rc) return rc;
    inter[j].ndim = nd;
    for (int d = 0; d < nd; ++d) {
      inter[j].lo[d] = srcs[j].extent.lo[d] > dst->extent.lo[d] ? srcs[j].extent.lo[d] : dst->extent.lo[d];
      inter[j].hi[d] = srcs[j].extent.hi[d] < dst->extent.hi[d] ? srcs[j].extent.hi[d] : dst->extent.hi[d];
    }
    int64_t v = volume(&inter[j]);
    if (v == 0) continue;
    if (!srcs[j].data) return fail(TOFU_ERR_INVALID_ARG, "srcs[%d] has a NULL data pointer", j);
    for (int i = 0; i < j; ++i) {
      if (volume(&inter[i]) == 0) continue;
      bool disjoint = false;
      for (int d = 0; d < nd; ++d) disjoint = disjoint || inter[i].hi[d] <= inter[j].lo[d] || inter[j].hi[d] <= inter[i].lo[d];
      if (!disjoint) return fail(TOFU_ERR_OVERLAP, "srcs[%d] and srcs[%d] both hold part of the destination region", i, j);
    }
    covered += v;
  }
  if (covered != want)
    return fail(TOFU_ERR_UNCOVERED, "sources hold %lld of the %lld elements of the destination region", (long long)covered, (long long)want);

  FetchTable table;
  memset(&table, 0, sizeof(table));
  int64_t next = 0;
  for (int j = 0; j < nsrc; ++j) {
    if (volume(&inter[j]) == 0) continue;
    int64_t sstr[TOFU_MAX_DIMS];
    effective_strides(&srcs[j], sstr);
    const char *slo, *shi;
    byte_span(&srcs[j], sstr, &slo, &shi);
    if (slo < dhi && dlo < shi) return fail(TOFU_ERR_INVALID_ARG, "dst overlaps srcs[%d] in memory", j);
    FetchPiece* pc = &table.piece[table.n_pieces];
    rc = build_piece(dst, dstr, &srcs[j], sstr, &inter[j], pc);
    if (rc) return rc;
    int64_t count = pc->item_begin;
    pc->item_begin = next;
    next += count;
    ++table.n_pieces;
  }
  table.n_items = next;
  constexpr int kUnroll = 4;
  int64_t want_blocks = (next + 256 * kUnroll - 1) / (256 * kUnroll);
  int blocks = (int)(want_blocks < 8192 ? want_blocks : 8192);
  hipLaunchKernelGGL((fetch_kernel<kUnroll>), dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(hip_stream), table);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(TOFU_ERR_HIP, "fetch launch failed: %s", hipGetErrorString(e));
  return TOFU_OK;
}
