/*
 * tofu_tdl.h -- host-side region analysis for operators given in tensor-description form
 * (arXiv 1807.08887 Sec. 4.1: an operator is a lambda from output indices to a value, with
 * optional reduction variables; Sec. 4.2: its partition strategies follow from the ranges of
 * the input tensors each worker's share of the indices reaches).
 *
 * The interval arithmetic of Sec. 4.2 only admits affine index expressions (an interval may be
 * shifted, scaled and added to another; a product of two intervals is an error), so an index
 * expression is given here directly in affine form: sum_v coef[v] * var_v + offset.
 *
 * Everything in this header is integer / rational host arithmetic; nothing touches a device.
 * Return values are TOFU_OK or a negative tofu_status_t (tofu.h), text in tofu_last_error().
 */
#ifndef TOFU_TDL_H_
#define TOFU_TDL_H_

#include <stddef.h>
#include <stdint.h>

#include "tofu.h"

#ifdef __cplusplus
extern "C" {
#endif

#define TOFU_TDL_MAX_VARS 8
#define TOFU_TDL_MAX_INPUTS 4

/* Index expression of one tensor dimension. */
typedef struct {
  int64_t coef[TOFU_TDL_MAX_VARS];   /* per index variable; 0 = the variable does not appear */
  int64_t offset;
} tofu_tdl_index_t;

/* How the operator indexes one input tensor. */
typedef struct {
  int32_t ndim;
  int64_t size[TOFU_MAX_DIMS];               /* extents of the global tensor                    */
  tofu_tdl_index_t index[TOFU_MAX_DIMS];     /* coordinate read in each dimension               */
} tofu_tdl_access_t;

/* An operator: output[v_0..v_{n_out-1}] = Reduce(v_{n_out}..v_{n_vars-1} : f(inputs[...])).
 * The output tensor is indexed by the output variables in order (extent[v] each). */
typedef struct {
  int32_t n_vars;                            /* 1..TOFU_TDL_MAX_VARS                             */
  int32_t n_out;                             /* the first n_out variables index the output       */
  int64_t extent[TOFU_TDL_MAX_VARS];         /* variable v ranges over [0, extent[v])            */
  int32_t n_inputs;                          /* 1..TOFU_TDL_MAX_INPUTS                           */
  tofu_tdl_access_t input[TOFU_TDL_MAX_INPUTS];
} tofu_tdl_op_t;

/* The description of one of the built-in operators (tofu_op_kind_t); inputs in the order of
 * tofu_op_regions.  Variables (output indices | reduction variables):
 *   matmul   m, n | k                      conv2d   n, co, h, w | ci, kh, kw
 *   wgrad    co, ci, kh, kw | n, h, w      dgrad    n, ci, ih, iw | co, kh, kw
 *   lstm     b, h | gate                   conv1d   b, co, x | ci, dx
 * so a TOFU_*_DIM_* name is the variable of the same position, except TOFU_WGRAD_DIM_N, which
 * is variable 4.  UNSUPPORTED for a data gradient with stride > 1 (its index is not affine in
 * integers). */
int tofu_tdl_from_op(const tofu_op_desc_t* op, tofu_tdl_op_t* out);

/* Symbolic interval (Eq. 1) of input `input`, dimension `dim`, for the basic 2-way strategy
 * that cuts variable `split_var` in halves and gives this worker half `half` (0 or 1);
 * split_var = -1 analyses the unpartitioned operator.  The interval is
 *   [ sum_v lower[v] * X_v + constant , sum_v upper[v] * X_v + constant ]
 * over the symbolic upper bounds X_v (variable v ranges over [0, X_v]); coefficients are
 * written as numerator / denominator pairs with denominator 1 or 2.
 * Scaling by a negative coefficient exchanges the two ends. */
typedef struct {
  int64_t lower_num[TOFU_TDL_MAX_VARS], upper_num[TOFU_TDL_MAX_VARS];
  int64_t den;                               /* common denominator of all coefficients (1 or 2) */
  int64_t constant;
} tofu_tdl_interval_t;
int tofu_tdl_symbolic(const tofu_tdl_op_t* op, int32_t split_var, int32_t half, int32_t input, int32_t dim,
                      tofu_tdl_interval_t* out);

/* Regions of one shard for concrete extents, any k and nested steps (splits[i].dim names a
 * variable; each step cuts the range left by the earlier ones, as in tofu_op_regions):
 *   out_box        box of the output tensor the shard writes (ndim = n_out),
 *   in_boxes[i]    box of input i it reads, clipped to the tensor (i < n_inputs),
 *   cut_lo/cut_hi  [i * TOFU_MAX_DIMS + d]: how far the unclipped range of input i, dimension d
 *                  reaches outside the tensor on the low / high side (those reads are zeros),
 *   is_partial     1 when a reduction variable was split.
 * Any out pointer may be NULL.  Errors as tofu_op_regions. */
int tofu_tdl_regions(const tofu_tdl_op_t* op, const tofu_split_t* splits, int32_t nsplits, tofu_region_t* out_box,
                     tofu_region_t* in_boxes, int64_t* cut_lo, int64_t* cut_hi, int32_t* is_partial);

/* Communication of one basic strategy for one input (Appendix A.3, first situation): the
 * operator is cut k ways along variable `var`, input `input` is held cut k ways along its
 * dimension `part_dim`; every worker fetches the part of its region it does not hold.
 * Writes the number of elements fetched, summed over the k workers.  For k = 2 this is
 * 2 * (1/2 | 1/4 | 0) of the tensor's size in the three cases of the lemma, and the halo
 * overlap for a strategy that widens its region by a window. */
int tofu_tdl_fetch_elements(const tofu_tdl_op_t* op, int32_t var, int32_t k, int32_t input, int32_t part_dim,
                            int64_t* elements);

#ifdef __cplusplus
}
#endif

#endif /* TOFU_TDL_H_ */
