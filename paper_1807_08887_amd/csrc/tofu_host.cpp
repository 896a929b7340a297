// Host-side integer arithmetic of the shard path: shard ranges, composition of partition steps,
// input regions (arXiv 1807.08887 Sec. 4.2, Sec. 5.2, Appendix A.1) and argument validation.
// Nothing here touches the device.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include "tofu_internal.h"

namespace tofu {

static thread_local char g_error[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_error, sizeof(g_error), fmt, ap);
  va_end(ap);
  return code;
}

int iter_ndim(int32_t kind) {
  switch (kind) {
    case TOFU_OP_MATMUL: return 3;
    case TOFU_OP_CONV2D: return 5;
    case TOFU_OP_CONV2D_WGRAD: return 3;
    case TOFU_OP_CONV2D_DGRAD: return 5;
    case TOFU_OP_LSTM_CELL: return 2;
    case TOFU_OP_CONV1D: return 4;
    default: return 0;
  }
}

int64_t conv_out_extent(int64_t size, int64_t ksize, int64_t stride, int64_t pad) {
  int64_t span = size + 2 * pad - ksize;
  return span < 0 ? 0 : span / stride + 1;
}

int check_op(const tofu_op_desc_t* op) {
  if (!op) return fail(TOFU_ERR_INVALID_ARG, "operator description is NULL");
  if (op->kind == TOFU_OP_LSTM_CELL) {
    if (op->M < 1 || op->N < 1) return fail(TOFU_ERR_INVALID_ARG, "lstm cell needs batch (M) and hidden units (N) >= 1");
    return TOFU_OK;
  }
  if (op->kind == TOFU_OP_MATMUL) {
    if (op->M < 1 || op->N < 1 || op->K < 1)
      return fail(TOFU_ERR_INVALID_ARG, "matmul needs M,N,K >= 1 (got %lld,%lld,%lld)", (long long)op->M,
                  (long long)op->N, (long long)op->K);
    return TOFU_OK;
  }
  if (op->kind == TOFU_OP_CONV2D || op->kind == TOFU_OP_CONV2D_WGRAD || op->kind == TOFU_OP_CONV2D_DGRAD) {
    if (op->batch < 1 || op->c_in < 1 || op->c_out < 1 || op->H < 1 || op->W < 1 || op->KH < 1 || op->KW < 1 ||
        op->stride < 1 || op->pad < 0)
      return fail(TOFU_ERR_INVALID_ARG, "conv needs positive sizes, stride >= 1 and pad >= 0");
    if (conv_out_extent(op->H, op->KH, op->stride, op->pad) < 1 || conv_out_extent(op->W, op->KW, op->stride, op->pad) < 1)
      return fail(TOFU_ERR_INVALID_ARG, "conv output would be empty");
    return TOFU_OK;
  }
  if (op->kind == TOFU_OP_CONV1D) {
    if (op->batch < 1 || op->c_in < 1 || op->c_out < 1 || op->W < 1 || op->KW < 1)
      return fail(TOFU_ERR_INVALID_ARG, "conv1d needs positive batch, c_in, c_out, W and KW");
    if (op->W < op->KW) return fail(TOFU_ERR_INVALID_ARG, "conv1d output would be empty");
    return TOFU_OK;
  }
  return fail(TOFU_ERR_INVALID_ARG, "unknown operator kind %d", (int)op->kind);
}

// Extents of the iteration dimensions, in enumerator order; reduction dimensions come last.
static void iter_extents(const tofu_op_desc_t* op, int64_t* ext, int* first_reduce) {
  switch (op->kind) {
    case TOFU_OP_MATMUL:
      ext[TOFU_MM_DIM_M] = op->M; ext[TOFU_MM_DIM_N] = op->N; ext[TOFU_MM_DIM_K] = op->K;
      *first_reduce = TOFU_MM_DIM_K;
      break;
    case TOFU_OP_CONV2D:
      ext[TOFU_CONV_DIM_N] = op->batch; ext[TOFU_CONV_DIM_CO] = op->c_out;
      ext[TOFU_CONV_DIM_H] = conv_out_extent(op->H, op->KH, op->stride, op->pad);
      ext[TOFU_CONV_DIM_W] = conv_out_extent(op->W, op->KW, op->stride, op->pad);
      ext[TOFU_CONV_DIM_CI] = op->c_in;
      *first_reduce = TOFU_CONV_DIM_CI;
      break;
    case TOFU_OP_LSTM_CELL:
      ext[TOFU_LSTM_DIM_B] = op->M; ext[TOFU_LSTM_DIM_H] = op->N;
      *first_reduce = 2;          // no reduction dimension
      break;
    case TOFU_OP_CONV1D:
      ext[TOFU_CONV1D_DIM_B] = op->batch; ext[TOFU_CONV1D_DIM_CO] = op->c_out;
      ext[TOFU_CONV1D_DIM_X] = op->W - op->KW + 1; ext[TOFU_CONV1D_DIM_CI] = op->c_in;
      *first_reduce = TOFU_CONV1D_DIM_CI;
      break;
    case TOFU_OP_CONV2D_DGRAD:
      ext[TOFU_DGRAD_DIM_N] = op->batch; ext[TOFU_DGRAD_DIM_CI] = op->c_in;
      ext[TOFU_DGRAD_DIM_H] = op->H; ext[TOFU_DGRAD_DIM_W] = op->W;
      ext[TOFU_DGRAD_DIM_CO] = op->c_out;
      *first_reduce = TOFU_DGRAD_DIM_CO;
      break;
    default:
      ext[TOFU_WGRAD_DIM_CO] = op->c_out; ext[TOFU_WGRAD_DIM_CI] = op->c_in; ext[TOFU_WGRAD_DIM_N] = op->batch;
      *first_reduce = TOFU_WGRAD_DIM_N;
      break;
  }
}

static int shard_range_impl(int64_t extent, int32_t k, int32_t shard, int64_t* lo, int64_t* hi) {
  if (extent < 0) return fail(TOFU_ERR_INVALID_ARG, "extent %lld is negative", (long long)extent);
  if (k < 1) return fail(TOFU_ERR_INVALID_ARG, "k = %d, need k >= 1", (int)k);
  if (shard < 0 || shard >= k) return fail(TOFU_ERR_INVALID_ARG, "shard %d outside [0,%d)", (int)shard, (int)k);
  if ((int64_t)k > extent)
    return fail(TOFU_ERR_INVALID_ARG, "cannot cut an extent of %lld into %d non-empty parts", (long long)extent, (int)k);
  // 128-bit products: shard*extent can exceed 63 bits for huge extents.
  *lo = (int64_t)(((__int128)shard * extent) / k);
  *hi = (int64_t)(((__int128)(shard + 1) * extent) / k);
  return TOFU_OK;
}

int apply_splits(const tofu_op_desc_t* op, const tofu_split_t* splits, int32_t nsplits, IterRanges* r,
                 int32_t* is_partial) {
  int rc = check_op(op);
  if (rc) return rc;
  if (nsplits < 0 || (nsplits > 0 && !splits)) return fail(TOFU_ERR_INVALID_ARG, "bad split list");
  int nd = iter_ndim(op->kind), first_reduce = 0;
  int64_t ext[5];
  iter_extents(op, ext, &first_reduce);
  for (int d = 0; d < nd; ++d) { r->lo[d] = 0; r->hi[d] = ext[d]; }
  *is_partial = 0;
  for (int32_t i = 0; i < nsplits; ++i) {
    int d = splits[i].dim;
    if (d < 0 || d >= nd) return fail(TOFU_ERR_INVALID_ARG, "split %d names dimension %d, operator has %d", (int)i, d, nd);
    int64_t a, b;
    rc = shard_range_impl(r->hi[d] - r->lo[d], splits[i].k, splits[i].shard, &a, &b);   // cut the CURRENT range
    if (rc) return rc;
    r->hi[d] = r->lo[d] + b;
    r->lo[d] = r->lo[d] + a;
    if (d >= first_reduce && splits[i].k > 1) *is_partial = 1;
  }
  return TOFU_OK;
}

// Input coordinates read through index o*stride + d - pad for o in [out_lo,out_hi), d in [0,ksize):
// the output range widened by the filter window, clipped to [0,size); the rows cut off are zeros.
static void window(int64_t out_lo, int64_t out_hi, int64_t ksize, int64_t stride, int64_t pad, int64_t size,
                   int64_t* lo, int64_t* hi, int64_t* cut_lo, int64_t* cut_hi) {
  int64_t need_lo = out_lo * stride - pad;
  int64_t need_hi = (out_hi - 1) * stride + ksize - pad;   // exclusive
  *lo = need_lo < 0 ? 0 : need_lo;
  *hi = need_hi > size ? size : need_hi;
  *cut_lo = *lo - need_lo;
  *cut_hi = need_hi - *hi;
}

// Output positions o whose window o*stride + d - pad, d in [0,ksize), reaches an input coordinate
// in [in_lo,in_hi): the dy range a data-gradient shard reads, clipped to [0,out_size); cut_lo and
// cut_hi count the positions of the unclipped range that lie outside dy.
static void window_back(int64_t in_lo, int64_t in_hi, int64_t ksize, int64_t stride, int64_t pad, int64_t out_size,
                        int64_t* lo, int64_t* hi, int64_t* cut_lo, int64_t* cut_hi) {
  const int64_t a = in_lo + pad - (ksize - 1);
  int64_t need_lo = a >= 0 ? (a + stride - 1) / stride : -((-a) / stride);   // ceil(a / stride)
  const int64_t b = in_hi - 1 + pad;
  int64_t need_hi = (b >= 0 ? b / stride : -((-b + stride - 1) / stride)) + 1;  // floor(b / stride) + 1
  *lo = need_lo < 0 ? 0 : need_lo;
  *hi = need_hi > out_size ? out_size : need_hi;
  *cut_lo = *lo - need_lo;
  *cut_hi = need_hi - *hi;
}

static void set_box(tofu_region_t* b, int nd, const int64_t* lo, const int64_t* hi) {
  memset(b, 0, sizeof(*b));
  b->ndim = nd;
  for (int d = 0; d < nd; ++d) { b->lo[d] = lo[d]; b->hi[d] = hi[d]; }
}

void effective_strides(const tofu_tensor_t* t, int64_t* stride) {
  int nd = t->extent.ndim;
  bool all_zero = true;
  for (int d = 0; d < nd; ++d) all_zero = all_zero && t->stride[d] == 0;
  if (!all_zero) {
    for (int d = 0; d < nd; ++d) stride[d] = t->stride[d];
    return;
  }
  int64_t s = 1;
  for (int d = nd - 1; d >= 0; --d) {
    stride[d] = s;
    s *= t->extent.hi[d] - t->extent.lo[d];
  }
}

int64_t volume(const tofu_region_t* r) {
  int64_t v = 1;
  for (int d = 0; d < r->ndim; ++d) {
    int64_t e = r->hi[d] - r->lo[d];
    v *= e > 0 ? e : 0;
  }
  return v;
}

bool contains(const tofu_region_t* outer, const tofu_region_t* inner) {
  if (volume(inner) == 0) return true;
  for (int d = 0; d < inner->ndim; ++d)
    if (inner->lo[d] < outer->lo[d] || inner->hi[d] > outer->hi[d]) return false;
  return true;
}

int check_tensor(const char* name, const tofu_tensor_t* t, int32_t ndim, const tofu_region_t* need) {
  if (!t) return fail(TOFU_ERR_INVALID_ARG, "%s is NULL", name);
  if (t->extent.ndim != ndim) return fail(TOFU_ERR_INVALID_ARG, "%s has ndim %d, expected %d", name, (int)t->extent.ndim, (int)ndim);
  for (int d = 0; d < ndim; ++d)
    if (t->extent.lo[d] > t->extent.hi[d]) return fail(TOFU_ERR_INVALID_ARG, "%s extent has lo > hi in dimension %d", name, d);
  if (need && !contains(&t->extent, need)) {
    char buf[256]; int n = 0;
    for (int d = 0; d < ndim && n < 200; ++d)
      n += snprintf(buf + n, sizeof(buf) - n, " [%lld,%lld) vs held [%lld,%lld)", (long long)need->lo[d], (long long)need->hi[d],
                    (long long)t->extent.lo[d], (long long)t->extent.hi[d]);
    return fail(TOFU_ERR_REGION_MISMATCH, "%s does not hold the region this shard needs:%s", name, buf);
  }
  if (need && volume(need) > 0 && !t->data) return fail(TOFU_ERR_INVALID_ARG, "%s has a NULL data pointer", name);
  return TOFU_OK;
}

int check_tiling(const char* name, const tofu_region_t* want, const tofu_tensor_t* srcs, int32_t nsrc, tofu_region_t* inter) {
  const int nd = want->ndim;
  const int64_t need = volume(want);
  int64_t covered = 0;
  for (int j = 0; j < nsrc; ++j) {
    char item[40];
    snprintf(item, sizeof(item), "%s[%d]", name, j);
    int rc = check_tensor(item, &srcs[j], nd, nullptr);
    if (rc) return rc;
    inter[j].ndim = nd;
    for (int d = 0; d < nd; ++d) {
      inter[j].lo[d] = srcs[j].extent.lo[d] > want->lo[d] ? srcs[j].extent.lo[d] : want->lo[d];
      inter[j].hi[d] = srcs[j].extent.hi[d] < want->hi[d] ? srcs[j].extent.hi[d] : want->hi[d];
    }
    const int64_t v = volume(&inter[j]);
    if (v == 0) continue;
    if (!srcs[j].data) return fail(TOFU_ERR_INVALID_ARG, "%s has a NULL data pointer", item);
    for (int i = 0; i < j; ++i) {
      if (volume(&inter[i]) == 0) continue;
      bool disjoint = false;
      for (int d = 0; d < nd; ++d) disjoint = disjoint || inter[i].hi[d] <= inter[j].lo[d] || inter[j].hi[d] <= inter[i].lo[d];
      if (!disjoint) return fail(TOFU_ERR_OVERLAP, "%s[%d] and %s[%d] both hold part of the wanted region", name, i, name, j);
    }
    covered += v;
  }
  if (covered != need)
    return fail(TOFU_ERR_UNCOVERED, "%s hold %lld of the %lld elements of the wanted region", name, (long long)covered, (long long)need);
  return TOFU_OK;
}

const float* element_ptr(const tofu_tensor_t* t, const int64_t* stride, const int64_t* coord) {
  const float* p = static_cast<const float*>(t->data);
  for (int d = 0; d < t->extent.ndim; ++d) p += (coord[d] - t->extent.lo[d]) * stride[d];
  return p;
}

void box_byte_span(const tofu_tensor_t* t, const int64_t* stride, const tofu_region_t* box, const char** lo, const char** hi) {
  int64_t min_off = 0, max_off = 0;
  for (int d = 0; d < box->ndim; ++d) {
    const int64_t first = box->lo[d] - t->extent.lo[d];
    int64_t last = box->hi[d] - 1 - t->extent.lo[d];
    if (last < first) last = first;               // an empty range touches nothing; keep the span well formed
    const int64_t a = first * stride[d], b = last * stride[d];
    min_off += a < b ? a : b;
    max_off += a < b ? b : a;
  }
  *lo = static_cast<const char*>(t->data) + min_off * (int64_t)sizeof(float);
  *hi = static_cast<const char*>(t->data) + (max_off + 1) * (int64_t)sizeof(float);
}

}  // namespace tofu

using namespace tofu;

extern "C" {

const char* tofu_last_error(void) { return g_error; }

int tofu_shard_range(int64_t extent, int32_t k, int32_t shard, int64_t* lo, int64_t* hi) {
  if (!lo || !hi) return fail(TOFU_ERR_INVALID_ARG, "lo/hi output pointer is NULL");
  return shard_range_impl(extent, k, shard, lo, hi);
}

int tofu_op_regions(const tofu_op_desc_t* op, const tofu_split_t* splits, int32_t nsplits, tofu_region_t* out_box,
                    tofu_region_t* in_boxes, int64_t* pad_lo, int64_t* pad_hi, int32_t* is_partial) {
  IterRanges r;
  int32_t partial = 0;
  int rc = apply_splits(op, splits, nsplits, &r, &partial);
  if (rc) return rc;
  int64_t plo[2] = {0, 0}, phi[2] = {0, 0};
  tofu_region_t ob, ib[2];
  if (op->kind == TOFU_OP_MATMUL) {
    const int M = TOFU_MM_DIM_M, N = TOFU_MM_DIM_N, K = TOFU_MM_DIM_K;
    int64_t lo[2], hi[2];
    lo[0] = r.lo[M]; hi[0] = r.hi[M]; lo[1] = r.lo[N]; hi[1] = r.hi[N]; set_box(&ob, 2, lo, hi);
    lo[0] = r.lo[M]; hi[0] = r.hi[M]; lo[1] = r.lo[K]; hi[1] = r.hi[K]; set_box(&ib[0], 2, lo, hi);
    lo[0] = r.lo[K]; hi[0] = r.hi[K]; lo[1] = r.lo[N]; hi[1] = r.hi[N]; set_box(&ib[1], 2, lo, hi);
  } else if (op->kind == TOFU_OP_CONV2D) {
    const int N = TOFU_CONV_DIM_N, CO = TOFU_CONV_DIM_CO, H = TOFU_CONV_DIM_H, W = TOFU_CONV_DIM_W, CI = TOFU_CONV_DIM_CI;
    int64_t lo[4], hi[4];
    lo[0] = r.lo[N]; hi[0] = r.hi[N]; lo[1] = r.lo[CO]; hi[1] = r.hi[CO];
    lo[2] = r.lo[H]; hi[2] = r.hi[H]; lo[3] = r.lo[W]; hi[3] = r.hi[W];
    set_box(&ob, 4, lo, hi);
    lo[1] = r.lo[CI]; hi[1] = r.hi[CI];
    window(r.lo[H], r.hi[H], op->KH, op->stride, op->pad, op->H, &lo[2], &hi[2], &plo[0], &phi[0]);
    window(r.lo[W], r.hi[W], op->KW, op->stride, op->pad, op->W, &lo[3], &hi[3], &plo[1], &phi[1]);
    set_box(&ib[0], 4, lo, hi);
    lo[0] = r.lo[CO]; hi[0] = r.hi[CO]; lo[1] = r.lo[CI]; hi[1] = r.hi[CI];
    lo[2] = 0; hi[2] = op->KH; lo[3] = 0; hi[3] = op->KW;
    set_box(&ib[1], 4, lo, hi);
  } else if (op->kind == TOFU_OP_CONV1D) {
    const int B = TOFU_CONV1D_DIM_B, CO = TOFU_CONV1D_DIM_CO, X = TOFU_CONV1D_DIM_X, CI = TOFU_CONV1D_DIM_CI;
    int64_t lo[3] = {r.lo[B], r.lo[CO], r.lo[X]}, hi[3] = {r.hi[B], r.hi[CO], r.hi[X]};
    set_box(&ob, 3, lo, hi);
    lo[1] = r.lo[CI]; hi[1] = r.hi[CI];
    hi[2] = r.hi[X] + op->KW - 1;               // data[x + dx]: the output range widened by the window, always inside the tensor
    set_box(&ib[0], 3, lo, hi);
    lo[0] = r.lo[CI]; hi[0] = r.hi[CI]; lo[1] = r.lo[CO]; hi[1] = r.hi[CO]; lo[2] = 0; hi[2] = op->KW;
    set_box(&ib[1], 3, lo, hi);
  } else if (op->kind == TOFU_OP_LSTM_CELL) {   // element-wise: inputs are read where the output is written
    int64_t lo[3] = {r.lo[0], r.lo[1], 0}, hi[3] = {r.hi[0], r.hi[1], 4};
    set_box(&ob, 2, lo, hi);
    set_box(&ib[0], 3, lo, hi);
    set_box(&ib[1], 2, lo, hi);
  } else if (op->kind == TOFU_OP_CONV2D_DGRAD) {
    const int N = TOFU_DGRAD_DIM_N, CI = TOFU_DGRAD_DIM_CI, H = TOFU_DGRAD_DIM_H, W = TOFU_DGRAD_DIM_W, CO = TOFU_DGRAD_DIM_CO;
    const int64_t ho = conv_out_extent(op->H, op->KH, op->stride, op->pad), wo = conv_out_extent(op->W, op->KW, op->stride, op->pad);
    int64_t lo[4], hi[4];
    lo[0] = r.lo[N]; hi[0] = r.hi[N]; lo[1] = r.lo[CI]; hi[1] = r.hi[CI];
    lo[2] = r.lo[H]; hi[2] = r.hi[H]; lo[3] = r.lo[W]; hi[3] = r.hi[W];
    set_box(&ob, 4, lo, hi);
    lo[1] = r.lo[CO]; hi[1] = r.hi[CO];
    window_back(r.lo[H], r.hi[H], op->KH, op->stride, op->pad, ho, &lo[2], &hi[2], &plo[0], &phi[0]);
    window_back(r.lo[W], r.hi[W], op->KW, op->stride, op->pad, wo, &lo[3], &hi[3], &plo[1], &phi[1]);
    set_box(&ib[0], 4, lo, hi);
    lo[0] = r.lo[CO]; hi[0] = r.hi[CO]; lo[1] = r.lo[CI]; hi[1] = r.hi[CI];
    lo[2] = 0; hi[2] = op->KH; lo[3] = 0; hi[3] = op->KW;
    set_box(&ib[1], 4, lo, hi);
  } else {
    const int CO = TOFU_WGRAD_DIM_CO, CI = TOFU_WGRAD_DIM_CI, N = TOFU_WGRAD_DIM_N;
    int64_t ho = conv_out_extent(op->H, op->KH, op->stride, op->pad), wo = conv_out_extent(op->W, op->KW, op->stride, op->pad);
    int64_t lo[4], hi[4];
    lo[0] = r.lo[CO]; hi[0] = r.hi[CO]; lo[1] = r.lo[CI]; hi[1] = r.hi[CI];
    lo[2] = 0; hi[2] = op->KH; lo[3] = 0; hi[3] = op->KW;
    set_box(&ob, 4, lo, hi);
    lo[0] = r.lo[N]; hi[0] = r.hi[N]; lo[1] = r.lo[CI]; hi[1] = r.hi[CI];
    window(0, ho, op->KH, op->stride, op->pad, op->H, &lo[2], &hi[2], &plo[0], &phi[0]);
    window(0, wo, op->KW, op->stride, op->pad, op->W, &lo[3], &hi[3], &plo[1], &phi[1]);
    set_box(&ib[0], 4, lo, hi);
    lo[1] = r.lo[CO]; hi[1] = r.hi[CO]; lo[2] = 0; hi[2] = ho; lo[3] = 0; hi[3] = wo;
    set_box(&ib[1], 4, lo, hi);
  }
  if (out_box) *out_box = ob;
  if (in_boxes) { in_boxes[0] = ib[0]; in_boxes[1] = ib[1]; }
  if (pad_lo) { pad_lo[0] = plo[0]; pad_lo[1] = plo[1]; }
  if (pad_hi) { pad_hi[0] = phi[0]; pad_hi[1] = phi[1]; }
  if (is_partial) *is_partial = partial;
  return TOFU_OK;
}

size_t tofu_workspace_bytes(const tofu_op_desc_t* op, const tofu_split_t* splits, int32_t nsplits) {
  g_error[0] = 0;                      // a 0 with an empty error text means "no workspace needed", with a text "invalid"
  IterRanges r;
  int32_t partial = 0;
  if (apply_splits(op, splits, nsplits, &r, &partial)) return 0;
  if (op->kind == TOFU_OP_MATMUL) {
    int64_t m = r.hi[0] - r.lo[0], n = r.hi[1] - r.lo[1], k = r.hi[2] - r.lo[2];
    int s = matmul_split_k(m, n, k);
    return s > 1 ? (size_t)s * (size_t)m * (size_t)n * sizeof(float) : 0;
  }
  if (op->kind == TOFU_OP_CONV2D_WGRAD) {
    return wgrad_workspace_bytes(r.hi[0] - r.lo[0], r.hi[1] - r.lo[1], r.hi[2] - r.lo[2], conv_out_extent(op->H, op->KH, op->stride, op->pad),
                                 conv_out_extent(op->W, op->KW, op->stride, op->pad));
  }
  if (op->kind == TOFU_OP_CONV2D) {         // segment slots of the balanced last wave
    const int64_t bh = r.hi[TOFU_CONV_DIM_H] - r.lo[TOFU_CONV_DIM_H], bw = r.hi[TOFU_CONV_DIM_W] - r.lo[TOFU_CONV_DIM_W];
    if (op->KH != 3 || op->KW != 3 || op->stride != 1 || op->pad > 1) return 0;
    return conv_workspace_bytes((r.hi[TOFU_CONV_DIM_N] - r.lo[TOFU_CONV_DIM_N]) * bh * bw, bh, bw,
                                r.hi[TOFU_CONV_DIM_CO] - r.lo[TOFU_CONV_DIM_CO], r.hi[TOFU_CONV_DIM_CI] - r.lo[TOFU_CONV_DIM_CI]);
  }
  if (op->kind == TOFU_OP_CONV1D) {         // the shard's filters re-ordered to [co][ci][dx], then the slots
    const int64_t nb = r.hi[TOFU_CONV1D_DIM_B] - r.lo[TOFU_CONV1D_DIM_B], bw = r.hi[TOFU_CONV1D_DIM_X] - r.lo[TOFU_CONV1D_DIM_X];
    const int64_t co = r.hi[TOFU_CONV1D_DIM_CO] - r.lo[TOFU_CONV1D_DIM_CO], ci = r.hi[TOFU_CONV1D_DIM_CI] - r.lo[TOFU_CONV1D_DIM_CI];
    const size_t repack = ((size_t)ci * (size_t)co * (size_t)op->KW * sizeof(float) + 255) / 256 * 256;
    if (op->KW != 3) return repack;
    const int64_t cw = conv1d_chunk(bw);
    return repack + conv_workspace_bytes(nb * bw, bw / cw, cw, co, ci, 1, 3);
  }
  if (op->kind == TOFU_OP_CONV2D_DGRAD) {   // the shard's filters, taps reversed and channels exchanged, then the slots
    const int64_t ci = r.hi[TOFU_DGRAD_DIM_CI] - r.lo[TOFU_DGRAD_DIM_CI], co = r.hi[TOFU_DGRAD_DIM_CO] - r.lo[TOFU_DGRAD_DIM_CO];
    const int64_t bh = r.hi[TOFU_DGRAD_DIM_H] - r.lo[TOFU_DGRAD_DIM_H], bw = r.hi[TOFU_DGRAD_DIM_W] - r.lo[TOFU_DGRAD_DIM_W];
    const size_t flip = ((size_t)ci * (size_t)co * (size_t)(op->KH * op->KW) * sizeof(float) + 255) / 256 * 256;
    if (op->KH != 3 || op->KW != 3 || op->stride != 1) return flip;
    return flip + conv_workspace_bytes((r.hi[TOFU_DGRAD_DIM_N] - r.lo[TOFU_DGRAD_DIM_N]) * bh * bw, bh, bw, ci, co);
  }
  return 0;
}

}  // extern "C"
