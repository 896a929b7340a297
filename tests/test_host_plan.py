"""CPU tests of the library's plan search (include/tofu_plan.h) against the oracle's marking-based
cost and exhaustive search (oracle/plan.py).  No device call is made."""
import itertools

import pytest

import paper_1807_08887_amd as tofu
from paper_1807_08887_amd import plan as L
from paper_1807_08887_amd import tdl as T
from oracle import plan as P
from oracle import tdl as O
from test_host_tdl import _to_lib
from test_plan_pins import _gold, conv_group


def to_lib(graph, n_tensors):
    return L.graph(n_tensors, [(_to_lib(n["op"]), n["inputs"], n["output"], n["group"]) for n in graph])


def n_tensors_of(graph):
    return 1 + max(max(n["inputs"] + [n["output"]]) for n in graph)


GRAPHS = {
    "matmul": [dict(op=O.matmul(8, 4, 12), inputs=[0, 1], output=2, group=0)],
    "mlp_fwd": P.mlp_graph(8, [4, 6, 2], backward=False)[0],
    "mlp_train": P.mlp_graph(4, [2, 4, 2])[0],
    "conv1d_chain": [dict(op=O.conv1d(2, 3, 4, 8, 3), inputs=[0, 1], output=2, group=0),
                     dict(op=O.conv1d(2, 4, 2, 6, 3), inputs=[2, 3], output=4, group=1)],
}


@pytest.mark.parametrize("name", sorted(GRAPHS))
def test_strategy_costs_match_marked_coordinates(name):
    graph = GRAPHS[name]
    g = to_lib(graph, n_tensors_of(graph))
    for k in (2, 3):
        dims, vars_ = P.candidates(graph, k)
        for o, node in enumerate(graph):
            tens = node["inputs"] + [node["output"]]
            for v in vars_[o]:
                for choice in itertools.product(*[dims[t] for t in tens]):
                    td = [0] * n_tensors_of(graph)
                    for t, d in zip(tens, choice):
                        td[t] = d
                    want = P.strategy_cost(node["op"], node["op"]["vars"][v][0], k, list(choice[:-1]), choice[-1])
                    assert L.strategy_cost(g, o, v, k, td) == want, (name, k, o, v, choice)


@pytest.mark.parametrize("name", sorted(GRAPHS))
@pytest.mark.parametrize("k", [2, 3])
def test_basic_plan_is_a_minimiser(name, k):
    graph = GRAPHS[name]
    g = to_lib(graph, n_tensors_of(graph))
    res = L.basic(g, k)
    best, _ = P.basic_brute(graph, k)
    assert res["elements"] == best
    # the plan it returns really costs that much, by the oracle's marking and by the library's own sum
    assert P.basic_cost(graph, k, res["tensor_dim"], res["op_var"]) == best
    assert L.cost(g, k, res["tensor_dim"], res["op_var"]) == best


@pytest.mark.parametrize("name,ks", [("matmul", [2, 2]), ("mlp_fwd", [2, 2]), ("mlp_train", [2, 2]), ("matmul", [3, 2]),
                                     ("conv1d_chain", [2, 2])])
def test_recursive_plan_steps_are_minimisers_of_the_group_graphs(name, ks):
    """Every step's plan is the cheapest basic plan of worker group 0's graph, the per-step costs count
    all groups, and (Theorem 1) they do not decrease when the steps have the same number of workers."""
    graph = GRAPHS[name]
    g = to_lib(graph, n_tensors_of(graph))
    res = L.recursive(g, ks)
    groups, cur = 1, graph
    for s, k in enumerate(ks):
        c = P.basic_cost(cur, k, res["tensor_dim"][s], res["op_var"][s])
        assert groups * c == res["step_elements"][s], (name, s)
        assert c == P.basic_brute(cur, k)[0], (name, s)
        cur = P.reduce_graph(cur, k, res["op_var"][s])
        groups *= k
    assert res["total"] == sum(res["step_elements"])
    deltas, total = P.sequence_cost(graph, ks, res["tensor_dim"], res["op_var"])
    assert deltas == res["step_elements"] and total == res["total"]
    if len(set(ks)) == 1 and name != "conv1d_chain":     # halo strategies are outside the theorem's assumptions
        assert all(a <= b for a, b in zip(res["step_elements"], res["step_elements"][1:]))


def test_matrix_product_cut_twice_becomes_a_grid():
    """Sec. 5.2's figure: the second step does not repeat the first step's variable."""
    n = 16
    g = to_lib([dict(op=O.matmul(n, n, n), inputs=[0, 1], output=2, group=0)], 3)
    res = L.recursive(g, [2, 2])
    assert res["step_elements"] == [n * n, n * n]
    assert res["op_var"][0] != res["op_var"][1]
    # worker 3's shard follows from the two steps' variables and its digits (1, 1)
    sp = L.worker_splits(res["op_var"], [2, 2], 0, 3)
    assert sp == [(res["op_var"][0][0], 2, 1), (res["op_var"][1][0], 2, 1)]
    reg = T.regions(_to_lib(O.matmul(n, n, n)), sp)
    assert [hi - lo for lo, hi in reg["out_box"]] in ([n // 2, n // 2], [n // 2, n], [n, n // 2])


def test_search_space_of_a_convolution_group_matches_the_paper():
    gold = _gold("search_space_counts.txt")
    graph = conv_group()
    g = to_lib(graph, 6)
    res = L.basic(g, 2)
    assert res["configurations"] == gold["configs_per_step"]
    assert res["elements"] == P.basic_brute(graph, 2)[0]


def test_large_layers_plan_quickly_and_prefer_what_is_small_to_move():
    """WResNet-like sizes (Sec. 7.4): with big activations and small filters the filters are what moves
    (batch cut); with small activations and big filters the activations move (channel cut)."""
    def layer(batch, c, hw):
        desc = T.from_op(tofu.conv2d_desc(batch, c, c, hw, hw))
        return L.graph(3, [(desc, [0, 1], 2, 0)])
    low = L.basic(layer(128, 64, 56), 8)          # activations 128*64*56*56 = 25.7M elements, filters 36,864
    assert low["op_var"] == [0] and low["tensor_dim"][0] == 0 and low["tensor_dim"][2] == 0
    assert low["elements"] == 7 * 64 * 64 * 9     # every worker gathers the filters
    high = L.basic(layer(8, 2560, 7), 8)          # activations 8*2560*49 = 1.0M elements, filters 59M
    assert high["op_var"][0] in (1, 4)            # an output-channel or input-channel cut: the filters stay put
    assert high["elements"] <= 7 * 8 * 2560 * 49 + 1


def test_error_paths():
    ok = [dict(op=O.matmul(8, 4, 12), inputs=[0, 1], output=2, group=0)]
    with pytest.raises(tofu.TofuError) as e:      # tensor id outside the graph
        L.basic(to_lib(ok, 2), 2)
    assert e.value.status == -1
    with pytest.raises(tofu.TofuError) as e:      # unused tensor
        L.basic(to_lib(ok, 4), 2)
    assert e.value.status == -1 and "tensor 3" in str(e.value)
    two = [dict(op=O.matmul(8, 4, 12), inputs=[0, 1], output=2, group=1), dict(op=O.matmul(8, 6, 4), inputs=[2, 3], output=4, group=0)]
    with pytest.raises(tofu.TofuError) as e:      # groups out of order
        L.basic(to_lib(two, 5), 2)
    assert e.value.status == -1
    bad = [dict(op=O.matmul(8, 4, 12), inputs=[0, 1], output=2, group=0), dict(op=O.matmul(8, 6, 5), inputs=[2, 3], output=4, group=1)]
    with pytest.raises(tofu.TofuError) as e:      # the second operator sees tensor 2 as [8,5], the first wrote [8,4]
        L.basic(to_lib(bad, 5), 2)
    assert e.value.status == -1 and "extent" in str(e.value)
    with pytest.raises(tofu.TofuError) as e:      # nothing is long enough for 16 workers
        L.basic(to_lib(ok, 3), 16)
    assert e.value.status == -6
    g = to_lib(ok, 3)
    with pytest.raises(tofu.TofuError) as e:
        L.strategy_cost(g, 0, 5, 2, [0, 0, 0])
    assert e.value.status == -1
    with pytest.raises(tofu.TofuError) as e:
        L.strategy_cost(g, 0, 0, 2, [0, 2, 0])
    assert e.value.status == -1
    with pytest.raises(tofu.TofuError) as e:
        L.recursive(g, [2, 1])
    assert e.value.status == -1


def test_large_rnn_like_chain_for_eight_workers():
    """Four 8192-wide layers trained with batch 512 (weights 67M elements each, activations 4M): the
    recursive plan for 2*2*2 workers moves far less than data parallelism, whose cost is the closed
    form (k - 1) * 3 * sum of weight sizes, its per-step costs do not decrease, and the search takes
    seconds at most (Table 1 of the paper: seconds with recursion)."""
    import time
    batch, widths = 512, [8192] * 5
    graph, n_t = P.mlp_graph(batch, widths)
    g = to_lib(graph, n_t)
    t0 = time.time()
    res = L.recursive(g, [2, 2, 2])
    assert time.time() - t0 < 20
    weights = 4 * 8192 * 8192
    assert res["total"] < 7 * 3 * weights // 10
    assert all(a <= b for a, b in zip(res["step_elements"], res["step_elements"][1:]))
    # every worker's shard of the first layer's product is a valid plan for the shard calls
    desc = _to_lib(graph[0]["op"])
    seen = set()
    for w in range(8):
        reg = T.regions(desc, L.worker_splits(res["op_var"], [2, 2, 2], 0, w))
        seen.add(tuple(map(tuple, reg["out_box"])) + tuple(map(tuple, reg["in_boxes"][0])))
    assert len(seen) == 8


def test_resnet_like_chain_moves_filters_low_and_activations_high():
    """A chain of 3x3 convolutions shaped like a widened ResNet trunk (feature map halves, channels double;
    Sec. 7.4: lower layers have large feature maps and small filters, higher layers the opposite): searched
    for 8 workers in three recursive steps, the lowest layers keep cutting the batch (filters are what
    moves) and the highest layer ends up cutting channels (activations move), total cost below that of
    cutting the batch everywhere, per-step costs non-decreasing."""
    batch = 32
    layers = [(160, 160, 56, 1), (160, 320, 56, 2), (320, 320, 28, 1), (320, 640, 28, 2), (640, 640, 14, 1), (640, 1280, 14, 2),
              (1280, 1280, 7, 1)]
    ops = []
    for l, (ci, co, hw, stride) in enumerate(layers):
        desc = T.from_op(tofu.conv2d_desc(batch, ci, co, hw, hw, stride=stride))
        ops.append((desc, [2 * l, 2 * l + 1], 2 * l + 2, l))        # activations 0, 2, 4, ...; filters 1, 3, 5, ...
    g = L.graph(2 * len(layers) + 1, ops)
    res = L.recursive(g, [2, 2, 2])
    assert all(a <= b for a, b in zip(res["step_elements"], res["step_elements"][1:]))
    cuts = [[res["op_var"][s][l] for s in range(3)] for l in range(len(layers))]
    assert cuts[0] == [0, 0, 0] and cuts[1] == [0, 0, 0]              # batch, batch, batch
    assert any(v in (1, 4) for v in cuts[-1])                         # output or input channels somewhere in the last layer
    # data parallelism: every worker gathers every filter tensor once per step level -> (k - 1) * sum of filter sizes
    dp = 7 * sum(ci * co * 9 for ci, co, _, _ in layers)
    assert res["total"] < dp
    # a single 8-way step may only cut one dimension per tensor: never cheaper than the recursion's grid
    one = L.basic(g, 8)
    assert one["elements"] >= res["total"]


def test_worker_splits_match_the_oracle_for_every_worker():
    """tofu_plan_worker_splits against oracle.regions.worker_splits: every worker of several mixed-radix
    plans, variables taken per step and operator from a (made-up) recursive plan; and its error paths."""
    from oracle import regions as R
    for ks, op_var in [([2, 2, 2], [[0, 2], [0, 1], [1, 1]]), ([2, 3, 2], [[2, 0], [1, 1], [0, 2]]), ([5], [[1, 0]]), ([4, 2], [[0, 0], [2, 1]])]:
        total = 1
        for k in ks:
            total *= k
        for op in range(2):
            for w in range(total):
                want = R.worker_splits([step[op] for step in op_var], ks, w)
                assert L.worker_splits(op_var, ks, op, w) == [tuple(x) for x in want]
    with pytest.raises(tofu.TofuError):
        L.worker_splits([[0]], [2], 0, 2)            # worker outside [0, k)
    with pytest.raises(tofu.TofuError):
        L.worker_splits([[0]], [2], 1, 0)            # operator outside the plan
    with pytest.raises(tofu.TofuError):
        L.worker_splits([[0]], [1], 0, 0)            # a one-way step
