"""Pins of the oracle's plan cost and search (oracle/plan.py) against what the paper and the
arithmetic fix: the fractions of the cost lemma (Appendix A.3), closed forms of well-known plans
(data parallelism = the all-reduce volume of the weights), the paper's example of a matrix
product cut twice (Sec. 5.2), commutativity and the ordering of per-step costs (Appendix A.3),
and the size of the per-step search space (Sec. 5.2).  CPU only."""
import itertools
import os

from oracle import plan as P
from oracle import tdl as O

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _gold(name):
    rows = [l.split() for l in open(os.path.join(GOLD, name)) if l.strip() and not l.startswith("#")]
    return {k: int(v) for k, v in rows}


def test_lemma_fractions_for_a_matrix_product():
    """Cut in halves along m: A (indexed by m) costs 0 held by rows and 2 * S/4 held by columns;
    B (not indexed by m) costs 2 * S/2 whichever way it is held; the output likewise 0 or 2 * S/4.
    Cut along the reduction index k: both inputs 0 when held along their k dimension, and every
    worker sends half of its full-size partial: 2 * S/2."""
    M, N, K = 8, 6, 4
    op = O.matmul(M, N, K)
    SA, SB, SC = M * K, K * N, M * N
    assert P.strategy_cost(op, "m", 2, [0, 0], 0) == 0 + SB + 0
    assert P.strategy_cost(op, "m", 2, [1, 1], 1) == SA // 2 + SB + SC // 2
    assert P.strategy_cost(op, "n", 2, [0, 1], 1) == SA + 0 + 0
    assert P.strategy_cost(op, "k", 2, [1, 0], 0) == 0 + 0 + SC
    assert P.strategy_cost(op, "k", 2, [0, 1], 1) == SA // 2 + SB // 2 + SC
    # k workers: a tensor needed whole costs (k - 1) * S in total, an aligned one nothing
    assert P.strategy_cost(op, "m", 4, [0, 0], 0) == 3 * SB


def test_halo_strategy_costs_the_window_overlap():
    """conv1d of Fig. 1 cut along x with the data held along x: each half reads DX - 1 = 2 extra
    columns of the other half's slab... only the low half does (the high half's window ends with the tensor)."""
    B, CI, CO, X, DX = 2, 3, 2, 8, 3
    op = O.conv1d(B, CI, CO, X, DX)
    # data [B, CI, X + DX - 1 = 10] held in halves [0,5) | [5,10): worker 0 reads [0,6), worker 1 reads [4,10)
    data_fetch = B * CI * (1 + 1)
    filters_whole = CI * CO * DX          # filters are not indexed by x: each worker fetches the half it lacks
    assert P.strategy_cost(op, "x", 2, [2, 0], 2) == data_fetch + filters_whole


def test_cost_is_separable_over_operators():
    g, _ = P.mlp_graph(4, [2, 4, 2])
    assert P.basic_brute(g, 2, separable=True)[0] == P.basic_brute(g, 2, separable=False)[0]


def test_data_parallel_plan_costs_the_all_reduce_volume():
    """Every operator cut along the batch, every tensor held along its first dimension, at every
    step: activations never move; each weight is gathered by every worker once per operator that
    reads it (the forward product and the data gradient: the cost is a sum over operators'
    inputs) and each weight gradient is reduced over all workers, (k - 1) * S elements each."""
    batch, widths = 8, [4, 6, 2]
    g, n_t = P.mlp_graph(batch, widths)
    L = len(widths) - 1
    ks = [2, 2, 2]
    var_of = {("m", "n", "k"): 0, ("m", "j", "n"): 0, ("j", "n", "m"): 2}     # position of the batch variable
    op_var = [var_of[tuple(n for n, _ in node["op"]["vars"])] for node in g]
    deltas, total = P.sequence_cost(g, ks, [[0] * n_t] * 3, [op_var] * 3)
    weights = sum(widths[l - 1] * widths[l] for l in range(1, L + 1))
    assert total == (8 - 1) * 3 * weights
    assert deltas == [3 * weights, 2 * 3 * weights, 4 * 3 * weights]


def test_matrix_product_cut_twice_becomes_a_grid():
    """Sec. 5.2's figure: after a first cut by rows, B is held whole by each group; cutting by rows
    again would fetch it again (cost doubles), cutting by columns does not -- the cheapest second
    step is not the first step's plan, and the per-step costs do not decrease."""
    n = 8
    g = [dict(op=O.matmul(n, n, n), inputs=[0, 1], output=2, group=0)]
    first, _ = P.basic_brute(g, 2)
    assert first == n * n                                      # every strategy of a square product costs one matrix
    assert P.basic_cost(g, 2, {0: 0, 1: 0, 2: 0}, [0]) == n * n
    g2 = P.reduce_graph(g, 2, [0])                             # by rows: variable m
    assert [s for s, _ in g2[0]["op"]["inputs"]] == [(n // 2, n), (n, n)]
    rows_again = P.basic_cost(g2, 2, {0: 0, 1: 0, 2: 0}, [0])
    by_columns = P.basic_cost(g2, 2, {0: 1, 1: 1, 2: 1}, [1])
    assert rows_again == n * n and by_columns == n * n // 2
    second, _ = P.basic_brute(g2, 2)
    assert second == by_columns
    assert 2 * second >= first                                 # delta_2 >= delta_1


def test_two_basic_plans_commute():
    """cost(<p1, p2>) = cost(<p2, p1>) for plans whose cut dimensions scale with one index
    (Appendix A.3, commutativity), on a rectangular product."""
    op = O.matmul(8, 4, 12)
    g = [dict(op=op, inputs=[0, 1], output=2, group=0)]
    plans = {"m": ({0: 0, 1: 0, 2: 0}, [0]), "n": ({0: 1, 1: 1, 2: 1}, [1]), "k": ({0: 1, 1: 0, 2: 0}, [2])}
    for a, b in itertools.combinations(plans, 2):
        ab = P.sequence_cost(g, [2, 2], [plans[a][0], plans[b][0]], [plans[a][1], plans[b][1]])[1]
        ba = P.sequence_cost(g, [2, 2], [plans[b][0], plans[a][0]], [plans[b][1], plans[a][1]])[1]
        assert ab == ba, (a, b)


def test_greedy_steps_have_non_decreasing_costs():
    """Theorem 1: with the cheapest basic plan taken at every step, delta_i <= delta_{i+1}."""
    for batch, widths in [(8, [8, 8, 8]), (16, [4, 4]), (4, [16, 8])]:
        g, _ = P.mlp_graph(batch, widths, backward=False)
        deltas, groups = [], 1
        for _ in range(2):
            dims, vars_ = P.candidates(g, 2)
            ids = sorted(dims)
            best = None
            for choice in itertools.product(*[dims[t] for t in ids]):
                td = dict(zip(ids, choice))
                for ov in itertools.product(*vars_):
                    c = P.basic_cost(g, 2, td, ov)
                    if best is None or c < best[0]:
                        best = (c, td, ov)
            deltas.append(groups * best[0])
            groups *= 2
            g = P.reduce_graph(g, 2, best[2])
        assert deltas[0] <= deltas[1], (batch, widths, deltas)


def conv_group(B=2, C=2, K=2, H=3, KH=2):
    """One 2D-convolution operator group (Sec. 5.1): forward, data gradient and weight gradient over
    the six tensors x, w, y, dx, dw, dy (ids 0..5); no padding, stride 1."""
    ho = H - KH + 1
    x, w, y, dx, dw, dy = range(6)
    fwd = O.conv2d(B, C, K, H, H, KH, KH, 1, 0)
    dgrad = dict(vars=[("n", B), ("ci", C), ("ih", H), ("iw", H), ("co", K), ("kh", KH), ("kw", KH)], n_out=4,
                 inputs=[((B, K, ho, ho), [{"n": 1}, {"co": 1}, {"ih": 1, "kh": -1}, {"iw": 1, "kw": -1}]),
                         ((K, C, KH, KH), [{"co": 1}, {"ci": 1}, {"kh": 1}, {"kw": 1}])])
    wgrad = dict(vars=[("co", K), ("ci", C), ("kh", KH), ("kw", KH), ("n", B), ("h", ho), ("w", ho)], n_out=4,
                 inputs=[((B, C, H, H), [{"n": 1}, {"ci": 1}, {"h": 1, "kh": 1}, {"w": 1, "kw": 1}]),
                         ((B, K, ho, ho), [{"n": 1}, {"co": 1}, {"h": 1}, {"w": 1}])])
    return [dict(op=fwd, inputs=[x, w], output=y, group=0), dict(op=dgrad, inputs=[dy, w], output=dx, group=0),
            dict(op=wgrad, inputs=[x, dy], output=dw, group=0)]


def test_search_space_of_a_convolution_group():
    """Sec. 5.2: a 2D-convolution operator group has six 4-D tensors; one step of the recursion
    enumerates 4^6 assignments of their dimensions."""
    gold = _gold("search_space_counts.txt")
    g = conv_group()
    dims, _ = P.candidates(g, 2)
    assert len(dims) == 6 and all(len(d) == 4 for d in dims.values())
    cost, visited = P.basic_brute(g, 2)
    assert visited == gold["configs_per_step"] and 3 * visited == gold["configs_three_steps"]
    # the cheapest plan is no dearer than cutting everything along the batch
    assert cost <= P.basic_cost(g, 2, {t: 0 for t in range(6)}, [0, 0, 4])
