"""Pins for the CPU oracle: things the paper and the mathematics fix, checked
without the GPU library.  A dropped term, a wrong sign or index, a transposed
operand or a min-instead-of-max level in oracle/asnn_oracle.c fails here."""
import itertools
import math
import os

import numpy as np
import pytest

import oracle
from brute_force import brute_levels, brute_required, brute_values
from workloads import make_config, layered_skip, tiny_neat

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _act(n, edges, input_ids, X, **kw):
    src = np.array([e[0] for e in edges], dtype=np.int32)
    dst = np.array([e[1] for e in edges], dtype=np.int32)
    w = np.array([e[2] for e in edges], dtype=np.float32)
    return oracle.activate(n, src, dst, w, np.array(input_ids, dtype=np.int32), np.asarray(X, dtype=np.float32), **kw)


# ---------------------------------------------------------------- closed forms
def test_sigmoid_rational_points():
    """Introduction, display equation: sigmoid(ln(k)/4.97) = k/(k+1)."""
    rows = [l.split() for l in open(os.path.join(GOLDEN, "sigmoid_rational_points.txt")) if l.strip() and l[0] != "#"]
    ks = [float(r[0]) for r in rows]
    want = np.array([float(r[1]) for r in rows])
    x = np.array([[math.log(k) / 4.97 for k in ks]], dtype=np.float32)   # one raw input, batch = points
    # node 0 = raw input, node 1 = sigmoid(1.0 * x)
    v = _act(2, [(0, 1, 1.0)], [0], x, raw_inputs=True)
    assert np.abs(v[1] - want).max() < 2e-7
    # squashed input: sensor value itself is sigmoid(x)
    v = _act(1, [], [0], x)
    assert np.abs(v[0] - want).max() < 2e-7


def test_empty_sum_is_one_half_exactly():
    """Activation kernel: sum starts at 0, so a non-sensor with no incoming
    connection outputs sigmoid(0) = 0.5 exactly."""
    v = _act(3, [(0, 2, 1.5)], [0], [[0.3, 0.9]])
    assert (v[1] == np.float32(0.5)).all()
    lv, nl = oracle.levels(3, [0], [2])
    assert lv.tolist() == [0, 0, 1] and nl == 2


def test_single_edge_chain_by_hand():
    """x=0 -> sensor 0.5; w = 2 ln(3)/4.97 -> sum = ln(3)/4.97 -> 0.75;
    next edge w = ln(9)/(0.75*4.97) -> 0.9."""
    w1 = 2.0 * math.log(3.0) / 4.97
    w2 = math.log(9.0) / (0.75 * 4.97)
    v = _act(3, [(0, 1, w1), (1, 2, w2)], [0], [[0.0]])
    assert abs(v[0, 0] - 0.5) == 0
    assert abs(v[1, 0] - 0.75) < 2e-7
    assert abs(v[2, 0] - 0.9) < 3e-7


def test_all_zero_weights_give_one_half():
    wl = make_config(3, "small")
    v = oracle.activate(wl.n_nodes, wl.src, wl.dst, np.zeros_like(wl.w), wl.input_ids, wl.X)
    mask = np.ones(wl.n_nodes, dtype=bool)
    mask[wl.input_ids] = False
    assert (v[mask] == np.float32(0.5)).all()


def test_sigmoid_symmetry_and_saturation():
    """sigmoid(x)+sigmoid(-x)=1; e^(-4.97x) overflowing must give exactly 0,
    never NaN; large positive sums give exactly 1."""
    x = np.array([[0.1, 0.7, 2.0, 30.0, 1000.0, 3.0e38]], dtype=np.float32)
    vp = _act(2, [(0, 1, 1.0)], [0], x, raw_inputs=True)[1]
    vn = _act(2, [(0, 1, -1.0)], [0], x, raw_inputs=True)[1]
    assert np.isfinite(vp).all() and np.isfinite(vn).all()
    assert np.abs(vp.astype(np.float64) + vn - 1.0).max() < 1.2e-7
    assert vn[-1] == 0.0 and vn[-2] == 0.0 and vp[-1] == 1.0
    # high in-degree saturation: 4096 parallel edges of weight -1 from a 0.5 sensor
    edges = [(0, 1, -1.0)] * 4096
    v = _act(2, edges, [0], [[0.0]])
    assert v[1, 0] == 0.0


# ------------------------------------------------------------------ brute force
def _all_dags(n):
    pairs = [(i, j) for i in range(n) for j in range(i + 1, n)]
    for mask in range(1 << len(pairs)):
        yield [pairs[k] for k in range(len(pairs)) if (mask >> k) & 1]


@pytest.mark.parametrize("n", [1, 2, 3, 4, 5])
def test_exhaustive_small_dags(n):
    rng = np.random.default_rng(100 + n)
    count = 0
    for edges in _all_dags(n):
        count += 1
        if n == 5 and count % 3:       # a third of the 1024 five-node DAGs
            continue
        ids = rng.permutation(n)       # random labels so id order is not topological
        ew = [(int(ids[a]), int(ids[b]), float(rng.uniform(-2, 2))) for a, b in edges]
        indeg = np.zeros(n, int)
        for _, b, _ in ew:
            indeg[b] += 1
        roots = [v for v in range(n) if indeg[v] == 0]
        inputs = [v for v in roots if rng.random() < 0.7]
        x = rng.uniform(0, 1, size=len(inputs)).astype(np.float32)
        lv, nl = oracle.levels(n, [e[0] for e in ew], [e[1] for e in ew])
        bl = brute_levels(n, ew)
        assert lv.tolist() == bl
        assert nl == max(bl) + 1
        v = _act(n, ew, inputs, x.reshape(-1, 1))[:, 0]
        bv = brute_values(n, ew, inputs, x)
        assert np.abs(v - np.array(bv)).max() < 4e-7, (edges, ids)


def test_random_12_node_dags_with_parallel_edges():
    rng = np.random.default_rng(7)
    for trial in range(40):
        n = int(rng.integers(6, 13))
        order = rng.permutation(n)
        m = int(rng.integers(n, 3 * n))
        ew = []
        for _ in range(m):
            i, j = sorted(rng.choice(n, size=2, replace=False))
            ew.append((int(order[i]), int(order[j]), float(rng.uniform(-2, 2))))
        ew += ew[:3]                                     # parallel edges add
        indeg = np.zeros(n, int)
        for _, b, _ in ew:
            indeg[b] += 1
        inputs = [v for v in range(n) if indeg[v] == 0][: max(1, n // 4)]
        X = rng.uniform(0, 1, size=(len(inputs), 3)).astype(np.float32)
        lv, _ = oracle.levels(n, [e[0] for e in ew], [e[1] for e in ew])
        assert lv.tolist() == brute_levels(n, ew)
        v = _act(n, ew, inputs, X)
        for b in range(3):
            bv = brute_values(n, ew, inputs, X[:, b])
            assert np.abs(v[:, b] - np.array(bv)).max() < 6e-7


def test_config1_levels_by_longest_path_dp():
    """Config 1's own graph: longest path by dynamic programming over a
    topological order recovered from the brute-force side only."""
    wl = tiny_neat(seed=0)
    edges = list(zip(wl.src.tolist(), wl.dst.tolist()))
    incoming = {v: [] for v in range(wl.n_nodes)}
    for a, b in edges:
        incoming[b].append(a)
    memo = {}

    def longest(v):
        if v not in memo:
            memo[v] = max((1 + longest(a) for a in incoming[v]), default=0)
        return memo[v]

    want = [longest(v) for v in range(wl.n_nodes)]
    lv, nl = oracle.levels(wl.n_nodes, wl.src, wl.dst)
    assert lv.tolist() == want and nl == max(want) + 1
    # and its values against the recursive definition (memoised here: 76 nodes)
    vals = {}
    slot = {int(v): k for k, v in enumerate(wl.input_ids)}
    inc = {v: [] for v in range(wl.n_nodes)}
    for a, b, w in zip(wl.src.tolist(), wl.dst.tolist(), wl.w.tolist()):
        inc[b].append((a, w))

    def value(v):
        if v not in vals:
            if v in slot:
                s = float(wl.X[slot[v], 0])
            else:
                s = sum(w * value(a) for a, w in inc[v])
            vals[v] = 1.0 / (1.0 + math.exp(-4.97 * s))
        return vals[v]

    got = oracle.activate(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.X)[:, 0]
    assert np.abs(got - np.array([value(v) for v in range(wl.n_nodes)])).max() < 2e-6


# ---------------------------------------------- the paper's segmentation listing
def test_levels_equal_paper_segmentation():
    """When every node without incoming edges is an input and R = all nodes,
    the layers of the set-based segmentation are the level sets 1, 2, ..."""
    for seed in range(6):
        wl = layered_skip(seed=seed, n_nodes=90, n_inputs=7, n_outputs=5, n_levels=9, B=1, mean_extra_degree=2.0)
        CON = set(zip(wl.src.tolist(), wl.dst.tolist()))
        L = oracle.segment_network(range(wl.n_nodes), wl.input_ids.tolist(), wl.output_ids.tolist(), CON)
        lv, nl = oracle.levels(wl.n_nodes, wl.src, wl.dst)
        assert len(L) == nl - 1
        for k, layer in enumerate(L):
            assert layer == set(np.nonzero(lv == k + 1)[0].tolist())


def test_longest_not_shortest_path():
    """Diamond plus chord: 0->1->2->3 and 0->3; node 3 waits for its whole
    input set, so it sits in layer 3, not 1."""
    lv, nl = oracle.levels(4, [0, 1, 2, 0], [1, 2, 3, 3])
    assert lv.tolist() == [0, 1, 2, 3] and nl == 4
    L = oracle.segment_network(range(4), [0], [3], {(0, 1), (1, 2), (2, 3), (0, 3)})
    assert L == [{1}, {2}, {3}]


# ------------------------------------------------------------ library reduction
def _dense_chain(Ws, X):
    h = 1.0 / (1.0 + np.exp(-4.97 * X.astype(np.float64)))
    hs = [h]
    for W in Ws:
        h = h.astype(np.float32).astype(np.float64)      # stored values are float32
        h = 1.0 / (1.0 + np.exp(-4.97 * (W.astype(np.float64) @ h)))
        hs.append(h)
    return hs


def test_unpruned_layered_net_equals_matmul_chain():
    rng = np.random.default_rng(3)
    sizes = [13, 17, 11, 5]
    B = 9
    Ws = [(rng.standard_normal((sizes[i + 1], sizes[i])) / np.sqrt(sizes[i])).astype(np.float32) for i in range(3)]
    start = np.concatenate([[0], np.cumsum(sizes)])
    src, dst, w = [], [], []
    for li, W in enumerate(Ws):
        for r in range(W.shape[0]):
            for c in range(W.shape[1]):
                src.append(start[li] + c); dst.append(start[li + 1] + r); w.append(W[r, c])
    X = rng.uniform(0, 1, size=(sizes[0], B)).astype(np.float32)
    n = int(start[-1])
    relabel = rng.permutation(n)
    eperm = rng.permutation(len(src))
    src = relabel[np.array(src)][eperm]; dst = relabel[np.array(dst)][eperm]; w = np.array(w, np.float32)[eperm]
    inputs = relabel[np.arange(sizes[0])]
    v = oracle.activate(n, src, dst, w, inputs, X)
    hs = _dense_chain(Ws, X)
    for li in range(4):
        got = v[relabel[np.arange(start[li], start[li + 1])]]
        assert np.abs(got - hs[li]).max() < 2e-7
    lv, nl = oracle.levels(n, src, dst)
    assert nl == 4
    assert (lv[relabel] == np.repeat(np.arange(4), sizes)).all()


def test_pruned_mlp_equals_masked_dense_chain():
    """Config 2 (reduced) as masked dense matrices."""
    wl = make_config(2, "small")
    sizes = wl.meta["layer_sizes"]
    lv = wl.planted_level
    v = oracle.activate(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.X)
    # position of a node inside its layer: inputs by X row, others by id order
    pos = np.full(wl.n_nodes, -1)
    pos[wl.input_ids] = np.arange(len(wl.input_ids))
    for l in range(1, 4):
        ids = np.nonzero(lv == l)[0]
        pos[ids] = np.arange(len(ids))
    Ws = [np.zeros((sizes[l + 1], sizes[l])) for l in range(3)]
    for a, b, w in zip(wl.src, wl.dst, wl.w):
        assert lv[b] == lv[a] + 1
        Ws[lv[a]][pos[b], pos[a]] += float(w)
    hs = _dense_chain(Ws, wl.X)
    for l in range(4):
        ids = wl.input_ids if l == 0 else np.nonzero(lv == l)[0]
        assert np.abs(v[ids] - hs[l]).max() < 3e-7


# ------------------------------------------------------------- level invariants
@pytest.mark.parametrize("idx,scale", [(2, "small"), (3, "small"), (4, "small"), (5, "small"), (2, "full"), (3, "full")])
def test_planted_levels_and_invariants(idx, scale):
    wl = make_config(idx, scale)
    lv, nl = oracle.levels(wl.n_nodes, wl.src, wl.dst)
    assert (lv == wl.planted_level).all()
    assert nl == wl.planted_level.max() + 1
    assert (lv[wl.dst] > lv[wl.src]).all()
    best = np.full(wl.n_nodes, -1)
    np.maximum.at(best, wl.dst, lv[wl.src])
    has_in = np.bincount(wl.dst, minlength=wl.n_nodes) > 0
    assert (lv[has_in] == best[has_in] + 1).all()
    assert (lv[~has_in] == 0).all()


# ------------------------------------------------------------------ metamorphic
def test_relabel_and_shuffle_invariance():
    wl = make_config(3, "small")
    v = oracle.activate(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.X)
    lv, _ = oracle.levels(wl.n_nodes, wl.src, wl.dst)
    rng = np.random.default_rng(11)
    relabel = rng.permutation(wl.n_nodes).astype(np.int32)
    ep = rng.permutation(wl.n_edges)
    v2 = oracle.activate(wl.n_nodes, relabel[wl.src][ep], relabel[wl.dst][ep], wl.w[ep], relabel[wl.input_ids], wl.X)
    lv2, _ = oracle.levels(wl.n_nodes, relabel[wl.src][ep], relabel[wl.dst][ep])
    assert (lv2[relabel] == lv).all()
    assert np.abs(v2[relabel] - v).max() < 5e-7      # only the summation order moved


def test_split_edge_weight():
    wl = make_config(3, "small")
    v = oracle.activate(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.X)
    src = np.concatenate([wl.src, wl.src]); dst = np.concatenate([wl.dst, wl.dst])
    w = np.concatenate([wl.w * np.float32(0.5), wl.w * np.float32(0.5)])
    v2 = oracle.activate(wl.n_nodes, src, dst, w, wl.input_ids, wl.X)
    assert np.abs(v2 - v).max() < 5e-7


def test_batch_columns_independent():
    wl = make_config(4, "small")
    v = oracle.activate(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.X)
    for b in (0, wl.B - 1):
        vb = oracle.activate(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.X[:, b:b + 1])
        assert (vb[:, 0] == v[:, b]).all()


def test_population_equals_per_network_calls():
    wl = make_config(5, "small")
    v = oracle.activate(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.X)
    lv, _ = oracle.levels(wl.n_nodes, wl.src, wl.dst)
    for k in range(wl.n_nets):
        n0, n1 = wl.net_node_ptr[k], wl.net_node_ptr[k + 1]
        e0, e1 = wl.net_edge_ptr[k], wl.net_edge_ptr[k + 1]
        i0, i1 = wl.net_input_ptr[k], wl.net_input_ptr[k + 1]
        vk = oracle.activate(n1 - n0, wl.src[e0:e1] - n0, wl.dst[e0:e1] - n0, wl.w[e0:e1],
                             wl.input_ids[i0:i1] - n0, wl.X[i0:i1])
        assert (vk == v[n0:n1]).all()
        lk, _ = oracle.levels(n1 - n0, wl.src[e0:e1] - n0, wl.dst[e0:e1] - n0)
        assert (lk == lv[n0:n1]).all()


def test_f32_mode_close_to_f64_on_shallow_net():
    wl = make_config(2, "small")
    a = oracle.activate(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.X)
    b = oracle.activate(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.X, mode=oracle.F32)
    assert 0 < np.abs(a - b).max() < 5e-6


# -------------------------------------------------------------------- errors
def test_error_paths():
    with pytest.raises(oracle.OracleError) as e:
        oracle.levels(3, [0, 1, 2], [1, 2, 0])
    assert e.value.code == -2
    with pytest.raises(oracle.OracleError) as e:
        oracle.levels(3, [0], [0])                      # self loop
    assert e.value.code == -2
    with pytest.raises(oracle.OracleError) as e:
        oracle.levels(3, [0], [3])
    assert e.value.code == -1
    with pytest.raises(oracle.OracleError) as e:
        _act(3, [(0, 1, 1.0)], [1], [[0.5]])
    assert e.value.code == -3
    with pytest.raises(oracle.OracleError) as e:
        _act(3, [(0, 1, 1.0)], [0, 0], [[0.5], [0.5]])
    assert e.value.code == -4
    lv, nl = oracle.levels(0, [], [])
    assert nl == 0 and lv.shape[0] == 0


# ---------------------------------------------------------------- required set
def test_required_set_by_brute_force_and_in_the_segmentation():
    """R = nodes from which an output is reachable.  Pinned by forward search
    from every node on small DAGs, and through the paper's segmentation: with
    R given, its layers hold exactly the required nodes, level by level."""
    rng = np.random.default_rng(21)
    for trial in range(30):
        n = int(rng.integers(5, 13))
        order = rng.permutation(n)
        m = int(rng.integers(n // 2, 2 * n))
        edges = []
        for _ in range(m):
            i, j = sorted(rng.choice(n, size=2, replace=False))
            edges.append((int(order[i]), int(order[j])))
        outs = rng.choice(n, size=int(rng.integers(1, 3)), replace=False)
        src = [e[0] for e in edges]; dst = [e[1] for e in edges]
        got = oracle.required(n, src, dst, outs)
        assert got.tolist() == brute_required(n, edges, outs)
        # the kept connections are those that end in R; levels of the kept graph, restricted to R,
        # are the layers the segmentation produces when it is handed R
        keep = got[np.array(dst)] if edges else np.zeros(0, bool)
        ksrc = np.array(src, np.int32)[keep]; kdst = np.array(dst, np.int32)[keep]
        lv, _ = oracle.levels(n, ksrc, kdst)
        indeg = np.bincount(kdst, minlength=n)
        IN = [v for v in range(n) if indeg[v] == 0]          # every root acts as an input layer here
        L = oracle.segment_network(set(np.nonzero(got)[0].tolist()), IN, outs.tolist(), set(zip(ksrc.tolist(), kdst.tolist())))
        for k, layer in enumerate(L):
            assert layer == {v for v in range(n) if got[v] and lv[v] == k + 1}
        assigned = set().union(*L) if L else set()
        assert assigned == {v for v in range(n) if got[v] and lv[v] > 0}


def test_required_set_preserves_outputs():
    wl = make_config(1, "small")
    req = oracle.required(wl.n_nodes, wl.src, wl.dst, wl.output_ids)
    assert req[wl.output_ids].all() and not req.all()          # config 1 has dead-end hidden nodes
    keep = req[wl.dst]
    full = oracle.activate(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.X)
    cut = oracle.activate(wl.n_nodes, wl.src[keep], wl.dst[keep], wl.w[keep], wl.input_ids, wl.X)
    assert (full[req] == cut[req]).all()
