/*
 * tofu_plan.h -- host-side search for the partition plan of a coarsened dataflow graph
 * (arXiv 1807.08887 Sec. 5: dynamic programming over a linear graph of operator groups with a
 * brute-force search inside each group, Sec. 5.1; recursion over k = k_1 * k_2 * ... workers
 * with one basic plan per step, Sec. 5.2; communication cost of a basic plan, Appendix A.3).
 *
 * A graph is a list of operators in tensor-description form (tofu_tdl.h).  Every operator names
 * the graph tensor behind each of its inputs and behind its output, and the coarsened group it
 * belongs to (Sec. 5.1: a forward operator and its backward operators form one group; merged
 * element-wise operators or unrolled timesteps are given as one operator).  Groups are
 * numbered along the chain; the tensors that are used on both sides of a group boundary are
 * the state of the dynamic programme, so the graph has to be linear in the paper's sense only
 * as far as that state stays small (TOFU_PLAN_MAX_FRONTIER tensors).
 *
 * A BASIC PLAN for k workers gives every tensor one dimension along which it is held cut k
 * ways and every operator one index variable along which its iteration space is cut k ways
 * (an output variable: Case-1, a reduction variable: Case-2, Sec. 4.2).  Its cost is the number
 * of elements moved (Appendix A.3), summed over operators and workers:
 *   first situation   for each input, the part of the region a worker's share of the operator
 *                     reads that lies outside the worker's slab of the tensor;
 *   second situation  the part of the region a worker's share produces (the whole output when
 *                     a reduction variable is cut: a partial sum) that lies outside its slab.
 * Slabs and shares use the balanced ranges of tofu_shard_range.
 *
 * RECURSION (Sec. 5.2).  Step i searches the best basic plan for k_i workers on the graph of ONE
 * worker group of the previous step and applies it to all groups.  Reading used for that graph:
 * every operator keeps its description with the cut variable's extent reduced to group 0's
 * share, and sees as each input tensor the region this share reads (what the group holds plus
 * what it fetched -- the "extra inputs" of the paper's figure) and as its output the region it
 * produces; the next step cuts those regions along the dimension chosen for the tensor.  The
 * cost of step i counts all prod_{j<i} k_j groups: delta_i = (prod_{j<i} k_j) * cost(p_i).
 *
 * Host integer arithmetic only; nothing touches a device.  Return values are TOFU_OK or a
 * negative tofu_status_t (tofu.h) with text in tofu_last_error().
 */
#ifndef TOFU_PLAN_H_
#define TOFU_PLAN_H_

#include <stddef.h>
#include <stdint.h>

#include "tofu.h"
#include "tofu_tdl.h"

#ifdef __cplusplus
extern "C" {
#endif

#define TOFU_PLAN_MAX_FRONTIER 6   /* tensors alive across one group boundary               */
#define TOFU_PLAN_MAX_GROUP 8      /* tensors first used inside one group                   */
#define TOFU_PLAN_MAX_STEPS 16     /* recursion steps                                       */

typedef struct {
  tofu_tdl_op_t desc;                               /* index variables and input accesses             */
  int32_t input_tensor[TOFU_TDL_MAX_INPUTS];        /* graph tensor read by input i (i < n_inputs)    */
  int32_t output_tensor;                            /* graph tensor written (indexed by the output
                                                       variables in order)                            */
  int32_t group;                                    /* coarsened group, non-decreasing over `ops`     */
} tofu_plan_op_t;

typedef struct {
  int32_t n_tensors;                                /* tensors are numbered 0 .. n_tensors-1; their
                                                       shapes are those the operators state, and all
                                                       operators that touch a tensor must agree       */
  int32_t n_ops;
  const tofu_plan_op_t* ops;                        /* HOST array                                     */
} tofu_plan_graph_t;

/* Cost (elements moved, both situations, all k workers) of operator `op` cut along variable
 * `var` when the graph's tensors are held cut along tensor_dim[t] (HOST array of n_tensors
 * entries; only the operator's own tensors are read).  INVALID_ARG for a variable or a
 * dimension that does not exist or is shorter than k. */
int tofu_plan_strategy_cost(const tofu_plan_graph_t* g, int32_t op, int32_t var, int32_t k,
                            const int32_t* tensor_dim, int64_t* elements);

/* Cost of a complete basic plan: sum of tofu_plan_strategy_cost over the operators with
 * op_var[o] as operator o's variable. */
int tofu_plan_cost(const tofu_plan_graph_t* g, int32_t k, const int32_t* tensor_dim,
                   const int32_t* op_var, int64_t* elements);

/* Best basic plan for k workers: dynamic programme over the groups in order, state = the
 * dimensions of the tensors alive across the boundary, exhaustive search over the dimensions
 * of the tensors first used inside the group; given its tensors' dimensions every operator
 * takes its cheapest variable independently (the lowest-numbered one among equals).  Among
 * plans of equal cost the one met first in a fixed enumeration order is returned, so the result
 * is deterministic; which of several equally cheap plans that is, is not part of the contract.
 *   tensor_dim[n_tensors], op_var[n_ops]  the plan (HOST arrays, may be NULL),
 *   elements                               its cost,
 *   configurations                         how many assignments of tensor dimensions were
 *                                          examined (sum over groups of states * assignments of
 *                                          the group's new tensors); may be NULL.
 * Candidates are the dimensions of extent >= k (in every operator's view of the tensor) and the
 * variables of extent >= k; a tensor or operator without candidate -> UNSUPPORTED, a boundary
 * with more than TOFU_PLAN_MAX_FRONTIER tensors or a group that introduces more than
 * TOFU_PLAN_MAX_GROUP -> UNSUPPORTED. */
int tofu_plan_basic(const tofu_plan_graph_t* g, int32_t k, int32_t* tensor_dim, int32_t* op_var,
                    int64_t* elements, int64_t* configurations);

/* Recursive search for k = ks[0] * ks[1] * ... * ks[steps-1] workers (the caller orders the
 * factors; the paper takes them non-increasing).  Outputs (HOST arrays, any may be NULL):
 *   tensor_dim[s * n_tensors + t], op_var[s * n_ops + o]   the basic plan of step s,
 *   step_elements[s]                                       delta_s, all groups of step s counted,
 *   total                                                  sum of the deltas.
 * Worker w's shard of operator o is the split list (op_var[s * n_ops + o], ks[s], digit_s(w)),
 * s = 0 .. steps-1, in the form the shard calls of tofu.h and tofu_tdl_regions take. */
int tofu_plan_recursive(const tofu_plan_graph_t* g, const int32_t* ks, int32_t steps,
                        int32_t* tensor_dim, int32_t* op_var, int64_t* step_elements, int64_t* total);

/* Worker `worker`'s shard of operator `op` under a recursive plan (Appendix A.1: a plan is the
 * sequence of basic plans <p_1, ..., p_m>; Sec. 5.2: step i cuts every group of step i-1 k_i
 * ways).  The k = ks[0] * ... * ks[steps-1] workers are numbered so that the step-1 group is the
 * most significant digit of the worker number in the mixed radix (ks[0], ..., ks[steps-1]):
 * worker = ((d_0 * ks[1] + d_1) * ks[2] + d_2) ..., 0 <= d_s < ks[s].  Writes
 *   splits[s] = (op_var[s * n_ops + op], ks[s], d_s),  s = 0 .. steps-1,
 * the split list the shard calls of tofu.h and tofu_tdl_regions take (`splits` is a HOST array of
 * `steps` entries; op_var as tofu_plan_recursive returns it).  The shards of all k workers tile
 * the operator's iteration space exactly.
 * Errors: INVALID_ARG for NULL arrays, steps outside [1, TOFU_PLAN_MAX_STEPS], a ks[s] < 2,
 * op outside [0, n_ops), worker outside [0, k) or a negative variable. */
int tofu_plan_worker_splits(const int32_t* op_var, int32_t n_ops, const int32_t* ks, int32_t steps,
                            int32_t op, int64_t worker, tofu_split_t* splits);

#ifdef __cplusplus
}
#endif

#endif /* TOFU_PLAN_H_ */
