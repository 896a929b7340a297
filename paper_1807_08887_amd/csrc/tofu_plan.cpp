// Partition-plan search over a coarsened dataflow graph (arXiv 1807.08887 Sec. 5.1: dynamic
// programme over the chain of operator groups, exhaustive inside a group; Sec. 5.2: recursion
// with one basic plan per step; Appendix A.3: cost of a basic plan = elements fetched for the
// inputs plus elements produced for other workers).  Host integer arithmetic only.
#include <string.h>

#include <algorithm>
#include <limits>
#include <vector>

#include "tofu_internal.h"
#include "tofu_plan.h"

namespace tofu {
namespace {

constexpr int64_t kInf = std::numeric_limits<int64_t>::max() / 4;
constexpr int64_t kMaxSearch = 50'000'000;   // (state, assignment) pairs examined per group at most

// One operator's view of a graph tensor: slot -1 = its output, else input `slot`.
struct Use {
  int op, slot;
};

struct Tables {
  // in_cost[o][v][i][d], out_cost[o][v][d]; kInf for a variable or dimension that cannot be cut k ways
  std::vector<int64_t> in_cost, out_cost;
  int n_ops;
  int64_t& in(int o, int v, int i, int d) { return in_cost[((o * TOFU_TDL_MAX_VARS + v) * TOFU_TDL_MAX_INPUTS + i) * TOFU_MAX_DIMS + d]; }
  int64_t& out(int o, int v, int d) { return out_cost[(o * TOFU_TDL_MAX_VARS + v) * TOFU_MAX_DIMS + d]; }
};

struct Graph {
  int n_tensors = 0;
  std::vector<tofu_plan_op_t> ops;
  std::vector<std::vector<Use>> uses;       // per tensor
  std::vector<int> ndim;                    // per tensor
  std::vector<int> group_of;                // per op: index into the sorted list of distinct groups
  int n_groups = 0;
};

int64_t view_size(const Graph& G, const Use& u, int d) {
  const tofu_tdl_op_t& D = G.ops[u.op].desc;
  return u.slot < 0 ? D.extent[d] : D.input[u.slot].size[d];
}

int load_graph(const tofu_plan_graph_t* g, Graph* G, bool check_shapes) {
  if (!g || !g->ops) return fail(TOFU_ERR_INVALID_ARG, "graph or its operator list is NULL");
  if (g->n_ops < 1 || g->n_tensors < 1) return fail(TOFU_ERR_INVALID_ARG, "graph needs at least one operator and one tensor");
  G->n_tensors = g->n_tensors;
  G->ops.assign(g->ops, g->ops + g->n_ops);
  G->uses.assign(g->n_tensors, {});
  G->ndim.assign(g->n_tensors, 0);
  G->group_of.assign(g->n_ops, 0);
  int groups = 0;
  for (int o = 0; o < g->n_ops; ++o) {
    const tofu_plan_op_t& P = G->ops[o];
    // the description is validated by the region analysis itself
    int rc = tofu_tdl_regions(&P.desc, nullptr, 0, nullptr, nullptr, nullptr, nullptr, nullptr);
    if (rc) return rc;
    if (P.desc.n_out < 1) return fail(TOFU_ERR_INVALID_ARG, "operator %d has no output index", o);
    if (o > 0 && P.group < G->ops[o - 1].group) return fail(TOFU_ERR_INVALID_ARG, "operators must be listed in group order (operator %d)", o);
    if (o > 0 && P.group != G->ops[o - 1].group) ++groups;
    G->group_of[o] = groups;
    for (int i = -1; i < P.desc.n_inputs; ++i) {
      const int t = i < 0 ? P.output_tensor : P.input_tensor[i];
      if (t < 0 || t >= g->n_tensors) return fail(TOFU_ERR_INVALID_ARG, "operator %d names tensor %d, graph has %d", o, t, (int)g->n_tensors);
      const int nd = i < 0 ? P.desc.n_out : P.desc.input[i].ndim;
      Use u = {o, i};
      if (!G->uses[t].empty()) {
        if (G->ndim[t] != nd) return fail(TOFU_ERR_INVALID_ARG, "operator %d sees tensor %d with %d dimensions, an earlier operator with %d", o, t, nd, G->ndim[t]);
        if (check_shapes)
          for (int d = 0; d < nd; ++d)
            if (view_size(*G, u, d) != view_size(*G, G->uses[t][0], d))
              return fail(TOFU_ERR_INVALID_ARG, "operator %d states extent %lld for dimension %d of tensor %d, an earlier operator %lld", o,
                          (long long)view_size(*G, u, d), d, t, (long long)view_size(*G, G->uses[t][0], d));
      }
      G->ndim[t] = nd;
      G->uses[t].push_back(u);
    }
  }
  G->n_groups = groups + 1;
  for (int t = 0; t < g->n_tensors; ++t)
    if (G->uses[t].empty()) return fail(TOFU_ERR_INVALID_ARG, "tensor %d is used by no operator", t);
  return TOFU_OK;
}

// Elements a k-way cut of operator o along v produces outside the producing worker's slab
// (dimension d) of the output (Appendix A.3, second situation).
int produced_elsewhere(const tofu_tdl_op_t& D, int v, int k, int d, int64_t* elements) {
  int64_t total = 0;
  for (int w = 0; w < k; ++w) {
    tofu_split_t sp = {v, k, w};
    tofu_region_t box;
    int rc = tofu_tdl_regions(&D, &sp, 1, &box, nullptr, nullptr, nullptr, nullptr);
    if (rc) return rc;
    int64_t lo, hi;
    if ((rc = tofu_shard_range(D.extent[d], k, w, &lo, &hi))) return rc;
    tofu_region_t both = box;
    both.lo[d] = std::max(box.lo[d], lo);
    both.hi[d] = std::min(box.hi[d], hi);
    total += volume(&box) - volume(&both);
  }
  *elements = total;
  return TOFU_OK;
}

int build_tables(const Graph& G, int k, Tables* T) {
  const int n = (int)G.ops.size();
  T->n_ops = n;
  T->in_cost.assign((size_t)n * TOFU_TDL_MAX_VARS * TOFU_TDL_MAX_INPUTS * TOFU_MAX_DIMS, kInf);
  T->out_cost.assign((size_t)n * TOFU_TDL_MAX_VARS * TOFU_MAX_DIMS, kInf);
  for (int o = 0; o < n; ++o) {
    const tofu_tdl_op_t& D = G.ops[o].desc;
    for (int v = 0; v < D.n_vars; ++v) {
      if (D.extent[v] < k) continue;
      for (int i = 0; i < D.n_inputs; ++i)
        for (int d = 0; d < D.input[i].ndim; ++d) {
          if (D.input[i].size[d] < k) continue;
          int rc = tofu_tdl_fetch_elements(&D, v, k, i, d, &T->in(o, v, i, d));
          if (rc) return rc;
        }
      for (int d = 0; d < D.n_out; ++d) {
        if (D.extent[d] < k) continue;
        int rc = produced_elsewhere(D, v, k, d, &T->out(o, v, d));
        if (rc) return rc;
      }
    }
  }
  return TOFU_OK;
}

// Cheapest variable of operator o given the dimensions of its tensors; kInf when none fits.
int64_t best_var(const Graph& G, Tables& T, int o, const int* dim_of, int* var_out) {
  const tofu_plan_op_t& P = G.ops[o];
  int64_t best = kInf;
  int arg = -1;
  for (int v = 0; v < P.desc.n_vars; ++v) {
    int64_t c = T.out(o, v, dim_of[P.output_tensor]);
    for (int i = 0; i < P.desc.n_inputs && c < kInf; ++i) {
      const int64_t x = T.in(o, v, i, dim_of[P.input_tensor[i]]);
      c = x >= kInf ? kInf : c + x;
    }
    if (c < best) { best = c; arg = v; }
  }
  if (var_out) *var_out = arg;
  return best;
}

int strategy_cost(const Graph& G, Tables& T, int o, int v, const int32_t* tensor_dim, int64_t* elements) {
  const tofu_plan_op_t& P = G.ops[o];
  if (v < 0 || v >= P.desc.n_vars) return fail(TOFU_ERR_INVALID_ARG, "operator %d has no variable %d", o, v);
  int64_t c = 0;
  for (int i = -1; i < P.desc.n_inputs; ++i) {
    const int t = i < 0 ? P.output_tensor : P.input_tensor[i];
    const int d = tensor_dim[t];
    if (d < 0 || d >= G.ndim[t]) return fail(TOFU_ERR_INVALID_ARG, "tensor %d has no dimension %d", t, d);
    const int64_t x = i < 0 ? T.out(o, v, d) : T.in(o, v, i, d);
    if (x >= kInf) return fail(TOFU_ERR_INVALID_ARG, "operator %d: variable %d or dimension %d of tensor %d is shorter than the number of workers", o, v, d, t);
    c += x;
  }
  *elements = c;
  return TOFU_OK;
}

struct Step {
  std::vector<int> frontier;                 // tensors alive after this group, ascending
  std::vector<int> intro;                    // tensors first used in this group, ascending
  std::vector<int32_t> back_state, back_assign;   // per state of `frontier`: where its best cost came from
};

int basic_plan(const Graph& G, int k, int32_t* tensor_dim, int32_t* op_var, int64_t* elements, int64_t* configurations) {
  if (k < 1) return fail(TOFU_ERR_INVALID_ARG, "k = %d", k);
  Tables T;
  int rc = build_tables(G, k, &T);
  if (rc) return rc;
  const int nt = G.n_tensors, no = (int)G.ops.size();
  // candidate dimensions of every tensor: long enough in every operator's view of it
  std::vector<std::vector<int>> cand(nt);
  std::vector<int> first(nt, G.n_groups), last(nt, -1);
  for (int t = 0; t < nt; ++t) {
    for (int d = 0; d < G.ndim[t]; ++d) {
      bool ok = true;
      for (const Use& u : G.uses[t]) ok = ok && view_size(G, u, d) >= k;
      if (ok) cand[t].push_back(d);
    }
    if (cand[t].empty()) return fail(TOFU_ERR_UNSUPPORTED, "tensor %d has no dimension of extent >= %d", t, k);
    for (const Use& u : G.uses[t]) {
      first[t] = std::min(first[t], G.group_of[u.op]);
      last[t] = std::max(last[t], G.group_of[u.op]);
    }
  }
  std::vector<Step> steps(G.n_groups);
  for (int j = 0; j < G.n_groups; ++j)
    for (int t = 0; t < nt; ++t) {
      if (first[t] == j) steps[j].intro.push_back(t);
      if (first[t] <= j && last[t] > j) steps[j].frontier.push_back(t);
    }
  auto count = [&](const std::vector<int>& ts) {
    int64_t n = 1;
    for (int t : ts) n *= (int64_t)cand[t].size();
    return n;
  };
  auto decode = [&](const std::vector<int>& ts, int64_t code, int* dim_of) {
    for (int t : ts) {
      dim_of[t] = cand[t][code % (int64_t)cand[t].size()];
      code /= (int64_t)cand[t].size();
    }
  };
  auto encode = [&](const std::vector<int>& ts, const int* dim_of) {
    int64_t code = 0, mul = 1;
    for (int t : ts) {
      const int pos = (int)(std::find(cand[t].begin(), cand[t].end(), dim_of[t]) - cand[t].begin());
      code += mul * pos;
      mul *= (int64_t)cand[t].size();
    }
    return code;
  };

  std::vector<int64_t> cost_prev(1, 0), cost_cur;
  std::vector<int> empty;
  std::vector<int> dim_of(nt, 0);
  int64_t examined = 0;
  for (int j = 0; j < G.n_groups; ++j) {
    Step& S = steps[j];
    if ((int)S.frontier.size() > TOFU_PLAN_MAX_FRONTIER)
      return fail(TOFU_ERR_UNSUPPORTED, "%d tensors are alive after group %d (at most %d)", (int)S.frontier.size(), j, TOFU_PLAN_MAX_FRONTIER);
    if ((int)S.intro.size() > TOFU_PLAN_MAX_GROUP)
      return fail(TOFU_ERR_UNSUPPORTED, "group %d introduces %d tensors (at most %d)", j, (int)S.intro.size(), TOFU_PLAN_MAX_GROUP);
    const std::vector<int>& prev = j > 0 ? steps[j - 1].frontier : empty;
    const int64_t n_prev = count(prev), n_assign = count(S.intro), n_cur = count(S.frontier);
    if (n_prev * n_assign > kMaxSearch) return fail(TOFU_ERR_UNSUPPORTED, "group %d: %lld configurations exceed the search limit", j, (long long)(n_prev * n_assign));
    cost_cur.assign(n_cur, kInf);
    S.back_state.assign(n_cur, -1);
    S.back_assign.assign(n_cur, -1);
    for (int64_t s = 0; s < n_prev; ++s) {
      if (cost_prev[s] >= kInf) continue;
      decode(prev, s, dim_of.data());
      for (int64_t a = 0; a < n_assign; ++a) {
        decode(S.intro, a, dim_of.data());
        ++examined;
        int64_t c = cost_prev[s];
        for (int o = 0; o < no && c < kInf; ++o) {
          if (G.group_of[o] != j) continue;
          const int64_t x = best_var(G, T, o, dim_of.data(), nullptr);
          c = x >= kInf ? kInf : c + x;
        }
        if (c >= kInf) continue;
        const int64_t ns = encode(S.frontier, dim_of.data());
        if (c < cost_cur[ns]) {
          cost_cur[ns] = c;
          S.back_state[ns] = (int32_t)s;
          S.back_assign[ns] = (int32_t)a;
        }
      }
    }
    cost_prev.swap(cost_cur);
  }
  // the last frontier is empty: a single state
  if (cost_prev.empty() || cost_prev[0] >= kInf) return fail(TOFU_ERR_UNSUPPORTED, "no operator variable of extent >= %d fits some operator", k);
  if (elements) *elements = cost_prev[0];
  if (configurations) *configurations = examined;
  // walk back: the state after group j fixes the frontier tensors, its back pointers the rest
  std::vector<int> plan_dim(nt, -1);
  int64_t state = 0;
  for (int j = G.n_groups - 1; j >= 0; --j) {
    const Step& S = steps[j];
    std::vector<int> tmp(nt, 0);
    decode(S.frontier, state, tmp.data());
    for (int t : S.frontier) plan_dim[t] = tmp[t];
    decode(S.intro, S.back_assign[state], tmp.data());
    for (int t : S.intro) plan_dim[t] = tmp[t];
    state = S.back_state[state];
  }
  for (int t = 0; t < nt; ++t)
    if (tensor_dim) tensor_dim[t] = plan_dim[t];
  for (int o = 0; o < no; ++o) {
    int v = -1;
    best_var(G, T, o, plan_dim.data(), &v);
    if (op_var) op_var[o] = v;
  }
  return TOFU_OK;
}

// The graph of worker group 0 after cutting every operator along its chosen variable: the
// variable keeps group 0's share, every input becomes the region that share reads.
int reduce_graph(Graph* G, int k, const int32_t* op_var) {
  for (size_t o = 0; o < G->ops.size(); ++o) {
    tofu_tdl_op_t& D = G->ops[o].desc;
    tofu_split_t sp = {op_var[o], k, 0};
    tofu_region_t boxes[TOFU_TDL_MAX_INPUTS];
    int rc = tofu_tdl_regions(&D, &sp, 1, nullptr, boxes, nullptr, nullptr, nullptr);
    if (rc) return rc;
    int64_t lo, hi;
    if ((rc = tofu_shard_range(D.extent[op_var[o]], k, 0, &lo, &hi))) return rc;
    D.extent[op_var[o]] = hi - lo;
    for (int i = 0; i < D.n_inputs; ++i)
      for (int d = 0; d < D.input[i].ndim; ++d) {
        D.input[i].size[d] = boxes[i].hi[d] - boxes[i].lo[d];
        D.input[i].index[d].offset -= boxes[i].lo[d];
      }
  }
  return TOFU_OK;
}

}  // namespace
}  // namespace tofu

using namespace tofu;

extern "C" int tofu_plan_strategy_cost(const tofu_plan_graph_t* g, int32_t op, int32_t var, int32_t k, const int32_t* tensor_dim,
                                       int64_t* elements) {
  Graph G;
  int rc = load_graph(g, &G, true);
  if (rc) return rc;
  if (!tensor_dim || !elements) return fail(TOFU_ERR_INVALID_ARG, "tensor_dim or elements is NULL");
  if (op < 0 || op >= g->n_ops) return fail(TOFU_ERR_INVALID_ARG, "graph has no operator %d", (int)op);
  if (k < 1) return fail(TOFU_ERR_INVALID_ARG, "k = %d", (int)k);
  Tables T;
  if ((rc = build_tables(G, k, &T))) return rc;
  return strategy_cost(G, T, op, var, tensor_dim, elements);
}

extern "C" int tofu_plan_cost(const tofu_plan_graph_t* g, int32_t k, const int32_t* tensor_dim, const int32_t* op_var, int64_t* elements) {
  Graph G;
  int rc = load_graph(g, &G, true);
  if (rc) return rc;
  if (!tensor_dim || !op_var || !elements) return fail(TOFU_ERR_INVALID_ARG, "tensor_dim, op_var or elements is NULL");
  if (k < 1) return fail(TOFU_ERR_INVALID_ARG, "k = %d", (int)k);
  Tables T;
  if ((rc = build_tables(G, k, &T))) return rc;
  int64_t total = 0;
  for (int o = 0; o < g->n_ops; ++o) {
    int64_t c;
    if ((rc = strategy_cost(G, T, o, op_var[o], tensor_dim, &c))) return rc;
    total += c;
  }
  *elements = total;
  return TOFU_OK;
}

extern "C" int tofu_plan_basic(const tofu_plan_graph_t* g, int32_t k, int32_t* tensor_dim, int32_t* op_var, int64_t* elements,
                               int64_t* configurations) {
  Graph G;
  int rc = load_graph(g, &G, true);
  if (rc) return rc;
  return basic_plan(G, k, tensor_dim, op_var, elements, configurations);
}

extern "C" int tofu_plan_recursive(const tofu_plan_graph_t* g, const int32_t* ks, int32_t steps, int32_t* tensor_dim, int32_t* op_var,
                                   int64_t* step_elements, int64_t* total) {
  Graph G;
  int rc = load_graph(g, &G, true);
  if (rc) return rc;
  if (!ks || steps < 1 || steps > TOFU_PLAN_MAX_STEPS) return fail(TOFU_ERR_INVALID_ARG, "ks is NULL or steps = %d outside [1,%d]", (int)steps, TOFU_PLAN_MAX_STEPS);
  int64_t groups = 1, sum = 0;
  std::vector<int32_t> dims(g->n_tensors), vars(g->n_ops);
  for (int s = 0; s < steps; ++s) {
    if (ks[s] < 2) return fail(TOFU_ERR_INVALID_ARG, "ks[%d] = %d: every step needs at least two workers", s, (int)ks[s]);
    int64_t cost = 0;
    if ((rc = basic_plan(G, ks[s], dims.data(), vars.data(), &cost, nullptr))) return rc;
    if (cost > kInf / groups) return fail(TOFU_ERR_UNSUPPORTED, "cost overflows 64 bits");
    if (tensor_dim) memcpy(tensor_dim + (size_t)s * g->n_tensors, dims.data(), sizeof(int32_t) * g->n_tensors);
    if (op_var) memcpy(op_var + (size_t)s * g->n_ops, vars.data(), sizeof(int32_t) * g->n_ops);
    if (step_elements) step_elements[s] = groups * cost;
    sum += groups * cost;
    groups *= ks[s];
    if (s + 1 < steps && (rc = reduce_graph(&G, ks[s], vars.data()))) return rc;
  }
  if (total) *total = sum;
  return TOFU_OK;
}

extern "C" int tofu_plan_worker_splits(const int32_t* op_var, int32_t n_ops, const int32_t* ks, int32_t steps, int32_t op,
                                       int64_t worker, tofu_split_t* splits) {
  if (!op_var || !ks || !splits) return fail(TOFU_ERR_INVALID_ARG, "op_var, ks or splits is NULL");
  if (steps < 1 || steps > TOFU_PLAN_MAX_STEPS) return fail(TOFU_ERR_INVALID_ARG, "steps = %d outside [1,%d]", (int)steps, TOFU_PLAN_MAX_STEPS);
  if (n_ops < 1 || op < 0 || op >= n_ops) return fail(TOFU_ERR_INVALID_ARG, "operator %d outside [0,%d)", (int)op, (int)n_ops);
  int64_t k = 1;
  for (int s = 0; s < steps; ++s) {
    if (ks[s] < 2) return fail(TOFU_ERR_INVALID_ARG, "ks[%d] = %d: every step needs at least two workers", s, (int)ks[s]);
    if (k > kInf / ks[s]) return fail(TOFU_ERR_UNSUPPORTED, "worker count overflows 64 bits");
    k *= ks[s];
  }
  if (worker < 0 || worker >= k) return fail(TOFU_ERR_INVALID_ARG, "worker %lld outside [0,%lld)", (long long)worker, (long long)k);
  // digits of the worker number, least significant (the last step) first
  int64_t w = worker;
  for (int s = steps - 1; s >= 0; --s) {
    const int32_t var = op_var[(size_t)s * n_ops + op];
    if (var < 0) return fail(TOFU_ERR_INVALID_ARG, "step %d has no variable for operator %d", s, (int)op);
    splits[s].dim = var;
    splits[s].k = ks[s];
    splits[s].shard = (int32_t)(w % ks[s]);
    w /= ks[s];
  }
  return TOFU_OK;
}
