// Region analysis for operators in tensor-description form (arXiv 1807.08887 Sec. 4.1-4.2,
// Appendix A.2-A.3): interval arithmetic over affine index expressions, symbolically for the
// basic 2-way strategies and with concrete ranges for any plan.  Host integer arithmetic only.
#include <string.h>

#include "tofu_internal.h"
#include "tofu_tdl.h"

namespace tofu {

static int check_tdl(const tofu_tdl_op_t* op) {
  if (!op) return fail(TOFU_ERR_INVALID_ARG, "operator description is NULL");
  if (op->n_vars < 1 || op->n_vars > TOFU_TDL_MAX_VARS || op->n_out < 0 || op->n_out > op->n_vars || op->n_out > TOFU_MAX_DIMS)
    return fail(TOFU_ERR_INVALID_ARG, "description needs 1..%d variables, the first n_out <= %d of them output indices", TOFU_TDL_MAX_VARS, TOFU_MAX_DIMS);
  if (op->n_inputs < 1 || op->n_inputs > TOFU_TDL_MAX_INPUTS) return fail(TOFU_ERR_INVALID_ARG, "description needs 1..%d inputs", TOFU_TDL_MAX_INPUTS);
  for (int v = 0; v < op->n_vars; ++v)
    if (op->extent[v] < 1) return fail(TOFU_ERR_INVALID_ARG, "variable %d has extent %lld", v, (long long)op->extent[v]);
  for (int i = 0; i < op->n_inputs; ++i) {
    const tofu_tdl_access_t& a = op->input[i];
    if (a.ndim < 1 || a.ndim > TOFU_MAX_DIMS) return fail(TOFU_ERR_INVALID_ARG, "input %d has ndim %d", i, (int)a.ndim);
    for (int d = 0; d < a.ndim; ++d)
      if (a.size[d] < 1) return fail(TOFU_ERR_INVALID_ARG, "input %d dimension %d has size %lld", i, d, (long long)a.size[d]);
  }
  return TOFU_OK;
}

// Range [lo, hi) of an affine index over variable ranges [vlo, vhi): a positive coefficient takes
// the variable's ends in order, a negative one exchanges them.
static void affine_range(const tofu_tdl_index_t& e, int n_vars, const int64_t* vlo, const int64_t* vhi, int64_t* lo, int64_t* hi) {
  int64_t a = e.offset, b = e.offset;
  for (int v = 0; v < n_vars; ++v) {
    const int64_t c = e.coef[v];
    if (c > 0) { a += c * vlo[v]; b += c * (vhi[v] - 1); }
    else if (c < 0) { a += c * (vhi[v] - 1); b += c * vlo[v]; }
  }
  *lo = a;
  *hi = b + 1;
}

static int share_of(const tofu_tdl_op_t* op, const tofu_split_t* splits, int32_t nsplits, int64_t* vlo, int64_t* vhi, int32_t* partial) {
  if (nsplits < 0 || (nsplits > 0 && !splits)) return fail(TOFU_ERR_INVALID_ARG, "bad split list");
  for (int v = 0; v < op->n_vars; ++v) { vlo[v] = 0; vhi[v] = op->extent[v]; }
  *partial = 0;
  for (int32_t i = 0; i < nsplits; ++i) {
    const int v = splits[i].dim;
    if (v < 0 || v >= op->n_vars) return fail(TOFU_ERR_INVALID_ARG, "split %d names variable %d, operator has %d", (int)i, v, (int)op->n_vars);
    int64_t a, b;
    int rc = tofu_shard_range(vhi[v] - vlo[v], splits[i].k, splits[i].shard, &a, &b);
    if (rc) return rc;
    vhi[v] = vlo[v] + b;
    vlo[v] = vlo[v] + a;
    if (v >= op->n_out && splits[i].k > 1) *partial = 1;
  }
  return TOFU_OK;
}

}  // namespace tofu

using namespace tofu;

extern "C" int tofu_tdl_from_op(const tofu_op_desc_t* op, tofu_tdl_op_t* out) {
  int rc = check_op(op);
  if (rc) return rc;
  if (!out) return fail(TOFU_ERR_INVALID_ARG, "out is NULL");
  memset(out, 0, sizeof(*out));
  auto dim = [&](tofu_tdl_access_t& a, int d, int64_t size) -> tofu_tdl_index_t& {
    a.size[d] = size;
    return a.index[d];
  };
  if (op->kind == TOFU_OP_LSTM_CELL) {                   // vars: b, h | gate (the four gates of a unit are all read)
    out->n_vars = 3; out->n_out = 2; out->n_inputs = 2;
    out->extent[0] = op->M; out->extent[1] = op->N; out->extent[2] = 4;
    tofu_tdl_access_t &g = out->input[0], &c = out->input[1];
    g.ndim = 3; c.ndim = 2;
    dim(g, 0, op->M).coef[0] = 1; dim(g, 1, op->N).coef[1] = 1; dim(g, 2, 4).coef[2] = 1;
    dim(c, 0, op->M).coef[0] = 1; dim(c, 1, op->N).coef[1] = 1;
    return TOFU_OK;
  }
  if (op->kind == TOFU_OP_CONV1D) {                      // vars: b, co, x | ci, dx  (Fig. 3)
    out->n_vars = 5; out->n_out = 3; out->n_inputs = 2;
    const int64_t ext[5] = {op->batch, op->c_out, op->W - op->KW + 1, op->c_in, op->KW};
    memcpy(out->extent, ext, sizeof(ext));
    tofu_tdl_access_t &d = out->input[0], &f = out->input[1];
    d.ndim = f.ndim = 3;
    dim(d, 0, op->batch).coef[0] = 1; dim(d, 1, op->c_in).coef[3] = 1;
    tofu_tdl_index_t& dx = dim(d, 2, op->W); dx.coef[2] = 1; dx.coef[4] = 1;
    dim(f, 0, op->c_in).coef[3] = 1; dim(f, 1, op->c_out).coef[1] = 1; dim(f, 2, op->KW).coef[4] = 1;
    return TOFU_OK;
  }
  if (op->kind == TOFU_OP_MATMUL) {                      // vars: m, n | k
    out->n_vars = 3; out->n_out = 2; out->n_inputs = 2;
    out->extent[0] = op->M; out->extent[1] = op->N; out->extent[2] = op->K;
    tofu_tdl_access_t &A = out->input[0], &B = out->input[1];
    A.ndim = B.ndim = 2;
    dim(A, 0, op->M).coef[0] = 1; dim(A, 1, op->K).coef[2] = 1;
    dim(B, 0, op->K).coef[2] = 1; dim(B, 1, op->N).coef[1] = 1;
    return TOFU_OK;
  }
  const int64_t ho = conv_out_extent(op->H, op->KH, op->stride, op->pad), wo = conv_out_extent(op->W, op->KW, op->stride, op->pad);
  if (op->kind == TOFU_OP_CONV2D) {                      // vars: n, co, h, w | ci, kh, kw
    out->n_vars = 7; out->n_out = 4; out->n_inputs = 2;
    const int64_t ext[7] = {op->batch, op->c_out, ho, wo, op->c_in, op->KH, op->KW};
    memcpy(out->extent, ext, sizeof(ext));
    tofu_tdl_access_t &x = out->input[0], &w = out->input[1];
    x.ndim = w.ndim = 4;
    dim(x, 0, op->batch).coef[0] = 1; dim(x, 1, op->c_in).coef[4] = 1;
    tofu_tdl_index_t& xh = dim(x, 2, op->H); xh.coef[2] = op->stride; xh.coef[5] = 1; xh.offset = -op->pad;
    tofu_tdl_index_t& xw = dim(x, 3, op->W); xw.coef[3] = op->stride; xw.coef[6] = 1; xw.offset = -op->pad;
    dim(w, 0, op->c_out).coef[1] = 1; dim(w, 1, op->c_in).coef[4] = 1; dim(w, 2, op->KH).coef[5] = 1; dim(w, 3, op->KW).coef[6] = 1;
    return TOFU_OK;
  }
  if (op->kind == TOFU_OP_CONV2D_WGRAD) {                // vars: co, ci, kh, kw | n, h, w
    out->n_vars = 7; out->n_out = 4; out->n_inputs = 2;
    const int64_t ext[7] = {op->c_out, op->c_in, op->KH, op->KW, op->batch, ho, wo};
    memcpy(out->extent, ext, sizeof(ext));
    tofu_tdl_access_t &x = out->input[0], &dy = out->input[1];
    x.ndim = dy.ndim = 4;
    dim(x, 0, op->batch).coef[4] = 1; dim(x, 1, op->c_in).coef[1] = 1;
    tofu_tdl_index_t& xh = dim(x, 2, op->H); xh.coef[5] = op->stride; xh.coef[2] = 1; xh.offset = -op->pad;
    tofu_tdl_index_t& xw = dim(x, 3, op->W); xw.coef[6] = op->stride; xw.coef[3] = 1; xw.offset = -op->pad;
    dim(dy, 0, op->batch).coef[4] = 1; dim(dy, 1, op->c_out).coef[0] = 1; dim(dy, 2, ho).coef[5] = 1; dim(dy, 3, wo).coef[6] = 1;
    return TOFU_OK;
  }
  // data gradient, stride 1: dx[n, ci, ih, iw] = Sum(co, kh, kw: dy[n, co, ih + pad - kh, iw + pad - kw] * w[co, ci, kh, kw])
  if (op->stride != 1) return fail(TOFU_ERR_UNSUPPORTED, "the data gradient's index is affine only for stride 1");
  out->n_vars = 7; out->n_out = 4; out->n_inputs = 2;    // vars: n, ci, ih, iw | co, kh, kw
  const int64_t ext[7] = {op->batch, op->c_in, op->H, op->W, op->c_out, op->KH, op->KW};
  memcpy(out->extent, ext, sizeof(ext));
  tofu_tdl_access_t &dy = out->input[0], &w = out->input[1];
  dy.ndim = w.ndim = 4;
  dim(dy, 0, op->batch).coef[0] = 1; dim(dy, 1, op->c_out).coef[4] = 1;
  tofu_tdl_index_t& dh = dim(dy, 2, ho); dh.coef[2] = 1; dh.coef[5] = -1; dh.offset = op->pad;
  tofu_tdl_index_t& dw = dim(dy, 3, wo); dw.coef[3] = 1; dw.coef[6] = -1; dw.offset = op->pad;
  dim(w, 0, op->c_out).coef[4] = 1; dim(w, 1, op->c_in).coef[1] = 1; dim(w, 2, op->KH).coef[5] = 1; dim(w, 3, op->KW).coef[6] = 1;
  return TOFU_OK;
}

extern "C" int tofu_tdl_symbolic(const tofu_tdl_op_t* op, int32_t split_var, int32_t half, int32_t input, int32_t dim,
                                 tofu_tdl_interval_t* out) {
  int rc = check_tdl(op);
  if (rc) return rc;
  if (!out) return fail(TOFU_ERR_INVALID_ARG, "out is NULL");
  if (split_var < -1 || split_var >= op->n_vars || (half != 0 && half != 1)) return fail(TOFU_ERR_INVALID_ARG, "bad split variable or half");
  if (input < 0 || input >= op->n_inputs || dim < 0 || dim >= op->input[input].ndim) return fail(TOFU_ERR_INVALID_ARG, "bad input or dimension");
  // Every variable starts as <u_v = 1> (the whole range [0, X_v]); the split variable as
  // <u_v = 1/2> or <l_v = 1/2, u_v = 1>.  Coefficients are kept in halves (den = 2).
  memset(out, 0, sizeof(*out));
  out->den = 2;
  const tofu_tdl_index_t& e = op->input[input].index[dim];
  out->constant = e.offset;
  for (int v = 0; v < op->n_vars; ++v) {
    int64_t l2 = 0, u2 = 2;                       // the variable's interval, in halves
    if (v == split_var) { l2 = half ? 1 : 0; u2 = half ? 2 : 1; }
    const int64_t c = e.coef[v];
    if (c >= 0) { out->lower_num[v] = c * l2; out->upper_num[v] = c * u2; }
    else { out->lower_num[v] = c * u2; out->upper_num[v] = c * l2; }   // negative scale: ends exchanged
  }
  bool even = true;
  for (int v = 0; v < op->n_vars; ++v) even = even && out->lower_num[v] % 2 == 0 && out->upper_num[v] % 2 == 0;
  if (even) {
    out->den = 1;
    for (int v = 0; v < op->n_vars; ++v) { out->lower_num[v] /= 2; out->upper_num[v] /= 2; }
  }
  return TOFU_OK;
}

extern "C" int tofu_tdl_regions(const tofu_tdl_op_t* op, const tofu_split_t* splits, int32_t nsplits, tofu_region_t* out_box,
                                tofu_region_t* in_boxes, int64_t* cut_lo, int64_t* cut_hi, int32_t* is_partial) {
  int rc = check_tdl(op);
  if (rc) return rc;
  int64_t vlo[TOFU_TDL_MAX_VARS], vhi[TOFU_TDL_MAX_VARS];
  int32_t partial = 0;
  if ((rc = share_of(op, splits, nsplits, vlo, vhi, &partial))) return rc;
  if (out_box) {
    memset(out_box, 0, sizeof(*out_box));
    out_box->ndim = op->n_out;
    for (int v = 0; v < op->n_out; ++v) { out_box->lo[v] = vlo[v]; out_box->hi[v] = vhi[v]; }
  }
  for (int i = 0; i < op->n_inputs; ++i) {
    const tofu_tdl_access_t& a = op->input[i];
    tofu_region_t box;
    memset(&box, 0, sizeof(box));
    box.ndim = a.ndim;
    for (int d = 0; d < a.ndim; ++d) {
      int64_t lo, hi;
      affine_range(a.index[d], op->n_vars, vlo, vhi, &lo, &hi);
      box.lo[d] = lo < 0 ? 0 : lo;
      box.hi[d] = hi > a.size[d] ? a.size[d] : hi;
      if (cut_lo) cut_lo[i * TOFU_MAX_DIMS + d] = box.lo[d] - lo;
      if (cut_hi) cut_hi[i * TOFU_MAX_DIMS + d] = hi - box.hi[d];
    }
    if (in_boxes) in_boxes[i] = box;
  }
  if (is_partial) *is_partial = partial;
  return TOFU_OK;
}

extern "C" int tofu_tdl_fetch_elements(const tofu_tdl_op_t* op, int32_t var, int32_t k, int32_t input, int32_t part_dim,
                                       int64_t* elements) {
  int rc = check_tdl(op);
  if (rc) return rc;
  if (!elements) return fail(TOFU_ERR_INVALID_ARG, "elements is NULL");
  if (var < 0 || var >= op->n_vars || input < 0 || input >= op->n_inputs || part_dim < 0 || part_dim >= op->input[input].ndim)
    return fail(TOFU_ERR_INVALID_ARG, "bad variable, input or dimension");
  const tofu_tdl_access_t& a = op->input[input];
  int64_t total = 0;
  for (int32_t w = 0; w < k; ++w) {
    tofu_split_t sp = {var, k, w};
    tofu_region_t boxes[TOFU_TDL_MAX_INPUTS];
    if ((rc = tofu_tdl_regions(op, &sp, 1, nullptr, boxes, nullptr, nullptr, nullptr))) return rc;
    int64_t held_lo, held_hi;
    if ((rc = tofu_shard_range(a.size[part_dim], k, w, &held_lo, &held_hi))) return rc;
    // |need| - |need intersected with the held slab|
    const tofu_region_t& need = boxes[input];
    tofu_region_t both = need;
    both.lo[part_dim] = need.lo[part_dim] > held_lo ? need.lo[part_dim] : held_lo;
    both.hi[part_dim] = need.hi[part_dim] < held_hi ? need.hi[part_dim] : held_hi;
    total += volume(&need) - volume(&both);
  }
  *elements = total;
  return TOFU_OK;
}
