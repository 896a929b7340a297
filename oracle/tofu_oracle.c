/*
 * tofu_oracle.c -- TEST INFRASTRUCTURE, not part of the product.
 *
 * Plain fp64 CPU definitions of what the partition-n-reduce shard path of
 * arXiv 1807.08887 must reproduce.  Partition-n-reduce (Sec. 3.1) reaches
 * exactly the unpartitioned operator's result by a different schedule, so the
 * oracle is the operator's definition written out as a loop nest over the
 * UNPARTITIONED tensors, in the style of the paper's naive conv1d (Fig. 1):
 * every output element is one fixed-order fp64 sum of products of the fp32
 * inputs.  Nothing is blocked, fused or reordered.  The only parallelism is an
 * OpenMP loop over output elements; each element is summed by one thread.
 *
 * Every routine also returns S = sum |a*b| over the same terms; the parity
 * bound of the GPU path is |gpu - value| <= 1e-5 * S per element.
 *
 * An optional reduction range [r0,r1) restricts the sum; it exists so that a
 * single worker's partial output (Sec. 4.2 Case-2) can be checked.  With the
 * full range the routines know nothing about partitions.
 *
 * This file shares no code with the HIP library and must never be linked into
 * or imported by it.  Only tests, the smoke check and the bench's cpu_baseline
 * leg may use it.
 */
#include <math.h>
#include <stdint.h>

typedef int64_t i64;

/* ---- matrix multiplication: C[m,n] = sum_k A[m,k] * B[k,n] ---------------- */
static void mm_elem(const float* A, const float* B, i64 N, i64 K, i64 m, i64 n, i64 k0, i64 k1,
                    double* val, double* absum) {
  double acc = 0.0, as = 0.0;
  for (i64 k = k0; k < k1; ++k) {
    double p = (double)A[m * K + k] * (double)B[k * N + n];
    acc += p;
    as += fabs(p);
  }
  *val = acc;
  *absum = as;
}

/* Dense box [m0,m1) x [n0,n1) of C, row-major into val/absum. */
void oracle_matmul_box(const float* A, const float* B, i64 M, i64 N, i64 K, i64 m0, i64 m1, i64 n0,
                       i64 n1, i64 k0, i64 k1, double* val, double* absum) {
  (void)M;
  i64 nm = m1 - m0, nn = n1 - n0;
#pragma omp parallel for schedule(static)
  for (i64 e = 0; e < nm * nn; ++e) {
    i64 m = m0 + e / nn, n = n0 + e % nn;
    mm_elem(A, B, N, K, m, n, k0, k1, &val[e], &absum[e]);
  }
}

/* Listed output coordinates: pts[i] = (m, n). */
void oracle_matmul_pts(const float* A, const float* B, i64 M, i64 N, i64 K, i64 npts, const i64* pts,
                       i64 k0, i64 k1, double* val, double* absum) {
  (void)M;
#pragma omp parallel for schedule(static)
  for (i64 i = 0; i < npts; ++i) mm_elem(A, B, N, K, pts[2 * i], pts[2 * i + 1], k0, k1, &val[i], &absum[i]);
}

/* ---- 2-D convolution (cross-correlation, zero padding) --------------------
 * y[n,co,h,w] = sum_{ci,kh,kw} x[n,ci,h*s+kh-p,w*s+kw-p] * wt[co,ci,kh,kw],
 * x taken as zero outside [0,H) x [0,W).  Two-dimensional form of Fig. 1. */
typedef struct {
  i64 batch, c_in, c_out, H, W, KH, KW, stride, pad, HO, WO;
} conv_t;

static conv_t conv_make(i64 batch, i64 c_in, i64 c_out, i64 H, i64 W, i64 KH, i64 KW, i64 stride, i64 pad) {
  conv_t c = {batch, c_in, c_out, H, W, KH, KW, stride, pad, 0, 0};
  c.HO = (H + 2 * pad - KH) / stride + 1;
  c.WO = (W + 2 * pad - KW) / stride + 1;
  return c;
}

static void conv_elem(const float* x, const float* wt, const conv_t* c, i64 n, i64 co, i64 h, i64 w, i64 ci0,
                      i64 ci1, double* val, double* absum) {
  double acc = 0.0, as = 0.0;
  for (i64 ci = ci0; ci < ci1; ++ci)
    for (i64 kh = 0; kh < c->KH; ++kh)
      for (i64 kw = 0; kw < c->KW; ++kw) {
        i64 ih = h * c->stride + kh - c->pad, iw = w * c->stride + kw - c->pad;
        if (ih < 0 || ih >= c->H || iw < 0 || iw >= c->W) continue; /* zero padding */
        double p = (double)x[((n * c->c_in + ci) * c->H + ih) * c->W + iw] *
                   (double)wt[((co * c->c_in + ci) * c->KH + kh) * c->KW + kw];
        acc += p;
        as += fabs(p);
      }
  *val = acc;
  *absum = as;
}

/* Dense box lo[4]..hi[4] over (n,co,h,w) of y, row-major into val/absum. */
void oracle_conv2d_box(const float* x, const float* wt, i64 batch, i64 c_in, i64 c_out, i64 H, i64 W, i64 KH,
                       i64 KW, i64 stride, i64 pad, const i64* lo, const i64* hi, i64 ci0, i64 ci1, double* val,
                       double* absum) {
  conv_t c = conv_make(batch, c_in, c_out, H, W, KH, KW, stride, pad);
  i64 d0 = hi[0] - lo[0], d1 = hi[1] - lo[1], d2 = hi[2] - lo[2], d3 = hi[3] - lo[3];
#pragma omp parallel for schedule(static)
  for (i64 e = 0; e < d0 * d1 * d2 * d3; ++e) {
    i64 r = e;
    i64 w = lo[3] + r % d3; r /= d3;
    i64 h = lo[2] + r % d2; r /= d2;
    i64 co = lo[1] + r % d1; r /= d1;
    i64 n = lo[0] + r;
    conv_elem(x, wt, &c, n, co, h, w, ci0, ci1, &val[e], &absum[e]);
  }
}

/* Listed output coordinates: pts[i] = (n, co, h, w). */
void oracle_conv2d_pts(const float* x, const float* wt, i64 batch, i64 c_in, i64 c_out, i64 H, i64 W, i64 KH,
                       i64 KW, i64 stride, i64 pad, i64 npts, const i64* pts, i64 ci0, i64 ci1, double* val,
                       double* absum) {
  conv_t c = conv_make(batch, c_in, c_out, H, W, KH, KW, stride, pad);
#pragma omp parallel for schedule(static)
  for (i64 i = 0; i < npts; ++i)
    conv_elem(x, wt, &c, pts[4 * i], pts[4 * i + 1], pts[4 * i + 2], pts[4 * i + 3], ci0, ci1, &val[i], &absum[i]);
}

/* ---- 1-D convolution, the paper's running example (Fig. 1: the loop nest; Fig. 3: its
 * description): out[b,co,x] = sum_{ci,dx} data[b,ci,x+dx] * filters[ci,co,dx].
 * data is [batch, c_in, X + DX - 1], filters [c_in, c_out, DX], out [batch, c_out, X]: no
 * padding and no stride; filters are indexed (ci, co, dx) as printed there.
 * Box lo[3]..hi[3] over (b,co,x), ci summed over [ci0,ci1). */
void oracle_conv1d_box(const float* data, const float* filters, i64 batch, i64 c_in, i64 c_out, i64 X, i64 DX,
                       const i64* lo, const i64* hi, i64 ci0, i64 ci1, double* val, double* absum) {
  (void)batch;
  i64 L = X + DX - 1;
  i64 d0 = hi[0] - lo[0], d1 = hi[1] - lo[1], d2 = hi[2] - lo[2];
#pragma omp parallel for schedule(static)
  for (i64 e = 0; e < d0 * d1 * d2; ++e) {
    i64 r = e;
    i64 x = lo[2] + r % d2; r /= d2;
    i64 co = lo[1] + r % d1; r /= d1;
    i64 b = lo[0] + r;
    double acc = 0.0, as = 0.0;
    for (i64 ci = ci0; ci < ci1; ++ci)
      for (i64 dx = 0; dx < DX; ++dx) {
        double p = (double)data[(b * c_in + ci) * L + x + dx] * (double)filters[(ci * c_out + co) * DX + dx];
        acc += p;
        as += fabs(p);
      }
    val[e] = acc;
    absum[e] = as;
  }
}

/* ---- weight gradient of that convolution ------------------------------------
 * dw[co,ci,kh,kw] = sum_{n,h,w} dy[n,co,h,w] * x[n,ci,h*s+kh-p,w*s+kw-p],
 * the derivative of sum(dy*y) with respect to wt[co,ci,kh,kw]. */
static void wgrad_elem(const float* x, const float* dy, const conv_t* c, i64 co, i64 ci, i64 kh, i64 kw, i64 n0,
                       i64 n1, double* val, double* absum) {
  double acc = 0.0, as = 0.0;
  for (i64 n = n0; n < n1; ++n)
    for (i64 h = 0; h < c->HO; ++h)
      for (i64 w = 0; w < c->WO; ++w) {
        i64 ih = h * c->stride + kh - c->pad, iw = w * c->stride + kw - c->pad;
        if (ih < 0 || ih >= c->H || iw < 0 || iw >= c->W) continue;
        double p = (double)dy[((n * c->c_out + co) * c->HO + h) * c->WO + w] *
                   (double)x[((n * c->c_in + ci) * c->H + ih) * c->W + iw];
        acc += p;
        as += fabs(p);
      }
  *val = acc;
  *absum = as;
}

/* Dense box lo[4]..hi[4] over (co,ci,kh,kw) of dw. */
void oracle_wgrad_box(const float* x, const float* dy, i64 batch, i64 c_in, i64 c_out, i64 H, i64 W, i64 KH,
                      i64 KW, i64 stride, i64 pad, const i64* lo, const i64* hi, i64 n0, i64 n1, double* val,
                      double* absum) {
  conv_t c = conv_make(batch, c_in, c_out, H, W, KH, KW, stride, pad);
  i64 d0 = hi[0] - lo[0], d1 = hi[1] - lo[1], d2 = hi[2] - lo[2], d3 = hi[3] - lo[3];
#pragma omp parallel for schedule(static)
  for (i64 e = 0; e < d0 * d1 * d2 * d3; ++e) {
    i64 r = e;
    i64 kw = lo[3] + r % d3; r /= d3;
    i64 kh = lo[2] + r % d2; r /= d2;
    i64 ci = lo[1] + r % d1; r /= d1;
    i64 co = lo[0] + r;
    wgrad_elem(x, dy, &c, co, ci, kh, kw, n0, n1, &val[e], &absum[e]);
  }
}

/* Listed output coordinates: pts[i] = (co, ci, kh, kw). */
void oracle_wgrad_pts(const float* x, const float* dy, i64 batch, i64 c_in, i64 c_out, i64 H, i64 W, i64 KH,
                      i64 KW, i64 stride, i64 pad, i64 npts, const i64* pts, i64 n0, i64 n1, double* val,
                      double* absum) {
  conv_t c = conv_make(batch, c_in, c_out, H, W, KH, KW, stride, pad);
#pragma omp parallel for schedule(static)
  for (i64 i = 0; i < npts; ++i)
    wgrad_elem(x, dy, &c, pts[4 * i], pts[4 * i + 1], pts[4 * i + 2], pts[4 * i + 3], n0, n1, &val[i], &absum[i]);
}

/* ---- data gradient of that convolution ---------------------------------------
 * dx[n,ci,ih,iw] = sum_{co} sum_{(h,kh): h*s+kh-p = ih} sum_{(w,kw): w*s+kw-p = iw} dy[n,co,h,w] * wt[co,ci,kh,kw],
 * the derivative of sum(dy*y) with respect to x[n,ci,ih,iw]: every output position whose
 * window covers (ih,iw) contributes through the tap that points at it.  Forward and backward
 * operators of a layer are partitioned as one group (Sec. 5.1); the output channel co is the
 * reduction index here, so a co split is Case-2 (Sec. 4.2) and [co0,co1) restricts the sum. */
static void dgrad_elem(const float* dy, const float* wt, const conv_t* c, i64 n, i64 ci, i64 ih, i64 iw, i64 co0,
                       i64 co1, double* val, double* absum) {
  double acc = 0.0, as = 0.0;
  for (i64 co = co0; co < co1; ++co)
    for (i64 kh = 0; kh < c->KH; ++kh)
      for (i64 kw = 0; kw < c->KW; ++kw) {
        i64 hs = ih + c->pad - kh, ws = iw + c->pad - kw;   /* h*s and w*s of the output position, if any */
        if (hs < 0 || ws < 0 || hs % c->stride || ws % c->stride) continue;
        i64 h = hs / c->stride, w = ws / c->stride;
        if (h >= c->HO || w >= c->WO) continue;
        double p = (double)dy[((n * c->c_out + co) * c->HO + h) * c->WO + w] *
                   (double)wt[((co * c->c_in + ci) * c->KH + kh) * c->KW + kw];
        acc += p;
        as += fabs(p);
      }
  *val = acc;
  *absum = as;
}

/* Dense box lo[4]..hi[4] over (n,ci,ih,iw) of dx. */
void oracle_dgrad_box(const float* dy, const float* wt, i64 batch, i64 c_in, i64 c_out, i64 H, i64 W, i64 KH,
                      i64 KW, i64 stride, i64 pad, const i64* lo, const i64* hi, i64 co0, i64 co1, double* val,
                      double* absum) {
  conv_t c = conv_make(batch, c_in, c_out, H, W, KH, KW, stride, pad);
  i64 d0 = hi[0] - lo[0], d1 = hi[1] - lo[1], d2 = hi[2] - lo[2], d3 = hi[3] - lo[3];
#pragma omp parallel for schedule(static)
  for (i64 e = 0; e < d0 * d1 * d2 * d3; ++e) {
    i64 r = e;
    i64 iw = lo[3] + r % d3; r /= d3;
    i64 ih = lo[2] + r % d2; r /= d2;
    i64 ci = lo[1] + r % d1; r /= d1;
    i64 n = lo[0] + r;
    dgrad_elem(dy, wt, &c, n, ci, ih, iw, co0, co1, &val[e], &absum[e]);
  }
}

/* Listed output coordinates: pts[i] = (n, ci, ih, iw). */
void oracle_dgrad_pts(const float* dy, const float* wt, i64 batch, i64 c_in, i64 c_out, i64 H, i64 W, i64 KH,
                      i64 KW, i64 stride, i64 pad, i64 npts, const i64* pts, i64 co0, i64 co1, double* val,
                      double* absum) {
  conv_t c = conv_make(batch, c_in, c_out, H, W, KH, KW, stride, pad);
#pragma omp parallel for schedule(static)
  for (i64 i = 0; i < npts; ++i)
    dgrad_elem(dy, wt, &c, pts[4 * i], pts[4 * i + 1], pts[4 * i + 2], pts[4 * i + 3], co0, co1, &val[i], &absum[i]);
}

/* ---- output reduction of partition-n-reduce (Sec. 3.1 way 2) ----------------
 * val[i] = sum_j partials[j][i] in fp64, absum[i] = sum_j |partials[j][i]|. */
void oracle_reduce(const float* const* partials, i64 k, i64 count, double* val, double* absum) {
#pragma omp parallel for schedule(static)
  for (i64 i = 0; i < count; ++i) {
    double acc = 0.0, as = 0.0;
    for (i64 j = 0; j < k; ++j) {
      double p = (double)partials[j][i];
      acc += p;
      as += fabs(p);
    }
    val[i] = acc;
    absum[i] = as;
  }
}

/* The other built-in reducers of the operator description language (Sec. 4.1: Sum, Max, Min,
 * Prod): the output reduction of a Case-2 split of an operator that reduces with one of them.
 * op: 1 = Max, 2 = Min, 3 = Prod.  Max / Min are exact (val is one of the inputs; a NaN input is
 * skipped unless all are NaN, the fmax / fmin convention); Prod multiplies in fp64.
 * absum[i] = |val[i]| (the scale the tolerance is measured against). */
void oracle_reduce_op(const float* const* partials, i64 k, i64 count, i64 op, double* val, double* absum) {
#pragma omp parallel for schedule(static)
  for (i64 i = 0; i < count; ++i) {
    double acc = (double)partials[0][i];
    for (i64 j = 1; j < k; ++j) {
      double p = (double)partials[j][i];
      if (op == 1) acc = fmax(acc, p);
      else if (op == 2) acc = fmin(acc, p);
      else acc *= p;
    }
    val[i] = acc;
    absum[i] = fabs(acc);
  }
}

/* ---- LSTM cell update after the gate GEMM --------------------------------------
 * The element-wise stage that consumes the gate pre-activations (Sec. 5.1: consecutive
 * element-wise operators are merged and share their producer's partition).  gates[b][h][4] holds
 * the pre-activations of the input, forget, cell and output gates of hidden unit h:
 *   c_new = sigmoid(f) * c_prev + sigmoid(i) * tanh(g),   h_new = sigmoid(o) * tanh(c_new).
 * scale_c = |sigmoid(f) * c_prev| + |sigmoid(i) * tanh(g)| and scale_h = 1 are the magnitudes
 * the tolerance is measured against. */
void oracle_lstm_cell(const float* gates, const float* c_prev, i64 count, double* c_new, double* h_new, double* scale_c) {
#pragma omp parallel for schedule(static)
  for (i64 e = 0; e < count; ++e) {
    double gi = gates[4 * e], gf = gates[4 * e + 1], gg = gates[4 * e + 2], go = gates[4 * e + 3];
    double si = 1.0 / (1.0 + exp(-gi)), sf = 1.0 / (1.0 + exp(-gf)), so = 1.0 / (1.0 + exp(-go));
    double a = sf * (double)c_prev[e], b = si * tanh(gg);
    c_new[e] = a + b;
    h_new[e] = so * tanh(a + b);
    scale_c[e] = fabs(a) + fabs(b);
  }
}

/* Number of OpenMP threads the loops above will use (reported by the bench). */
#ifdef _OPENMP
#include <omp.h>
int oracle_threads(void) { return omp_get_max_threads(); }
#else
int oracle_threads(void) { return 1; }
#endif
