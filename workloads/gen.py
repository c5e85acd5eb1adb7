"""Seeded generators for the five synthetic ASNN workloads.

Every generator returns a :class:`Workload`: a directed acyclic network given
as an edge list ``(src[e] -> dst[e], w[e])`` with *randomly permuted node ids
and shuffled edge order*, the ids of its input and output nodes, one batch of
input vectors ``X[n_inputs, B]`` (row k feeds ``input_ids[k]``), and, where the
construction fixes it, the level the generator planted for every node (the
first source of every non-level-0 node is forced into the level just below, so
the longest path to the node is known by construction).

Only numpy's ``Generator(PCG64(seed))`` is used; the order of the draws is
the order of the statements below and is part of the recipe.  Nothing here
computes a level from the edges or evaluates the network.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

CONFIG_NAMES = {
    1: "tiny_neat",
    2: "pruned_mlp_784_1000_1000_10",
    3: "layered_skip_100k",
    4: "deep_narrow_1M",
    5: "population_1024",
}


@dataclass
class Workload:
    name: str
    n_nodes: int
    src: np.ndarray            # int32 [E]
    dst: np.ndarray            # int32 [E]
    w: np.ndarray              # float32 [E]
    input_ids: np.ndarray      # int32 [n_inputs]
    output_ids: np.ndarray     # int32 [n_outputs]
    X: np.ndarray              # float32 [n_inputs, B], batch contiguous
    planted_level: Optional[np.ndarray] = None   # int32 [N] or None
    # population bookkeeping (None for a single network)
    net_node_ptr: Optional[np.ndarray] = None    # int32 [n_nets+1]
    net_edge_ptr: Optional[np.ndarray] = None    # int64 [n_nets+1]
    net_input_ptr: Optional[np.ndarray] = None   # int32 [n_nets+1] rows of X / input_ids
    net_output_ptr: Optional[np.ndarray] = None  # int32 [n_nets+1] rows of output_ids
    meta: dict = field(default_factory=dict)

    @property
    def n_edges(self) -> int:
        return int(self.src.shape[0])

    @property
    def B(self) -> int:
        return int(self.X.shape[1])

    @property
    def n_nets(self) -> int:
        return 1 if self.net_node_ptr is None else int(self.net_node_ptr.shape[0] - 1)


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed))


def _uniform32(rng, lo, hi, size):
    u = rng.random(size=size, dtype=np.float32)
    return (np.float32(lo) + (np.float32(hi) - np.float32(lo)) * u).astype(np.float32)


def _relabel_and_shuffle(rng, n_nodes, src, dst, w, ids_list, planted):
    """Random node relabelling and edge shuffle, drawn after the structure."""
    relabel = rng.permutation(n_nodes).astype(np.int32)      # old id -> new id
    eperm = rng.permutation(src.shape[0])
    src2 = relabel[src][eperm].astype(np.int32)
    dst2 = relabel[dst][eperm].astype(np.int32)
    w2 = w[eperm].astype(np.float32)
    ids2 = [relabel[i].astype(np.int32) for i in ids_list]
    planted2 = None
    if planted is not None:
        planted2 = np.empty(n_nodes, dtype=np.int32)
        planted2[relabel] = planted
    return src2, dst2, w2, ids2, planted2


def _layered_edges(rng, level_sizes, degree, p_prev):
    """Edges of a layered-skip network in planted (level-contiguous) ids.

    level_sizes[l] nodes sit in level l; ``degree`` holds the in-degree of
    every node of levels >= 1 in id order.  Source k of a node in level l:
    k == 0 -> a node of level l-1 (plants the level); otherwise level l-1 with
    probability p_prev, else a level drawn uniformly from 0..l-1; the node is
    uniform inside the chosen level.  Sources are drawn with replacement, so
    parallel edges occur.
    """
    level_sizes = np.asarray(level_sizes, dtype=np.int64)
    level_start = np.concatenate([[0], np.cumsum(level_sizes)])
    n_nodes = int(level_start[-1])
    node_level = np.repeat(np.arange(level_sizes.shape[0]), level_sizes)
    first_dst = int(level_sizes[0])
    degree = np.asarray(degree, dtype=np.int64)
    assert degree.shape[0] == n_nodes - first_dst
    dst = np.repeat(np.arange(first_dst, n_nodes, dtype=np.int64), degree)
    n_edges = dst.shape[0]
    row_start = np.concatenate([[0], np.cumsum(degree)])[:-1]
    is_first = np.zeros(n_edges, dtype=bool)
    is_first[row_start[degree > 0]] = True
    lvl_dst = node_level[dst]
    u_prev = rng.random(n_edges)
    u_level = rng.random(n_edges)
    u_node = rng.random(n_edges)
    any_lower = np.minimum((u_level * lvl_dst).astype(np.int64), lvl_dst - 1)
    src_level = np.where(is_first | (u_prev < p_prev), lvl_dst - 1, any_lower)
    size = level_sizes[src_level]
    src = level_start[src_level] + np.minimum((u_node * size).astype(np.int64), size - 1)
    return n_nodes, src.astype(np.int32), dst.astype(np.int32), node_level.astype(np.int32)


# --------------------------------------------------------------------------
# config 1
# --------------------------------------------------------------------------
def tiny_neat(seed=0, n_inputs=8, n_outputs=4, n_hidden=64, n_edges=512, B=1):
    """NEAT-style tiny network: ids in a random topological order, distinct
    edges sampled uniformly from (earlier, later) pairs, never into an input.
    ids 0..n_inputs-1 are inputs, the next n_outputs ids are outputs.
    Hidden nodes without any incoming edge are expected."""
    rng = _rng(seed)
    n = n_inputs + n_outputs + n_hidden
    order = rng.permutation(n)                      # order[p] = node at position p
    is_input = np.zeros(n, dtype=bool)
    is_input[:n_inputs] = True
    pi, pj = np.triu_indices(n, k=1)                # positions, pi < pj
    a, b = order[pi], order[pj]
    ok = ~is_input[b]
    a, b = a[ok], b[ok]
    assert a.shape[0] >= n_edges
    pick = rng.choice(a.shape[0], size=n_edges, replace=False)
    src = a[pick].astype(np.int32)
    dst = b[pick].astype(np.int32)
    w = _uniform32(rng, -2.0, 2.0, n_edges)
    X = rng.random(size=(n_inputs, B), dtype=np.float32)
    eperm = rng.permutation(n_edges)
    return Workload(
        name=CONFIG_NAMES[1], n_nodes=n, src=src[eperm], dst=dst[eperm], w=w[eperm],
        input_ids=np.arange(n_inputs, dtype=np.int32),
        output_ids=np.arange(n_inputs, n_inputs + n_outputs, dtype=np.int32),
        X=X, planted_level=None, meta={"seed": seed})


# --------------------------------------------------------------------------
# config 2
# --------------------------------------------------------------------------
def pruned_mlp(seed=0, layers=(784, 1000, 1000, 10), keep_edges=0.10, drop_hidden=0.05, B=256):
    """Fully connected MLP, weights N(0, std=1/sqrt(dense fan_in)); first a
    fraction of every hidden layer's nodes is deleted with all their edges,
    then exactly ``keep_edges`` of the remaining edges are kept, uniformly."""
    rng = _rng(seed)
    layers = list(layers)
    kept = []
    for li, width in enumerate(layers):
        if 0 < li < len(layers) - 1:
            n_drop = int(round(drop_hidden * width))
            gone = rng.choice(width, size=n_drop, replace=False)
            mask = np.ones(width, dtype=bool)
            mask[gone] = False
            kept.append(np.nonzero(mask)[0])
        else:
            kept.append(np.arange(width))
    sizes = [k.shape[0] for k in kept]
    start = np.concatenate([[0], np.cumsum(sizes)])
    n = int(start[-1])
    srcs, dsts, ws = [], [], []
    for li in range(len(layers) - 1):
        fan_in = layers[li]
        a = np.arange(start[li], start[li + 1])
        b = np.arange(start[li + 1], start[li + 2])
        bb, aa = np.meshgrid(b, a, indexing="ij")       # dst-major dense block
        wt = (rng.standard_normal(size=bb.shape) / np.sqrt(fan_in)).astype(np.float32)
        srcs.append(aa.ravel()); dsts.append(bb.ravel()); ws.append(wt.ravel())
    src = np.concatenate(srcs); dst = np.concatenate(dsts); w = np.concatenate(ws)
    n_keep = int(round(keep_edges * src.shape[0]))
    pick = rng.choice(src.shape[0], size=n_keep, replace=False)
    src, dst, w = src[pick], dst[pick], w[pick]
    indeg = np.bincount(dst, minlength=n)
    assert (indeg[start[1]:] > 0).all(), "a hidden/output node lost every in-edge"
    planted = np.repeat(np.arange(len(layers)), sizes).astype(np.int32)
    X = rng.random(size=(sizes[0], B), dtype=np.float32)
    inputs = np.arange(0, start[1], dtype=np.int32)
    outputs = np.arange(start[-2], start[-1], dtype=np.int32)
    src, dst, w, (inputs, outputs), planted = _relabel_and_shuffle(
        rng, n, src, dst, w, [inputs, outputs], planted)
    return Workload(name=CONFIG_NAMES[2], n_nodes=n, src=src, dst=dst, w=w,
                    input_ids=inputs, output_ids=outputs, X=X, planted_level=planted,
                    meta={"seed": seed, "layer_sizes": sizes})


# --------------------------------------------------------------------------
# config 3
# --------------------------------------------------------------------------
def _split_even(total, parts):
    base, extra = divmod(total, parts)
    return [base + (1 if i < extra else 0) for i in range(parts)]


def layered_skip(seed=0, n_nodes=100_000, n_inputs=1000, n_outputs=1000, n_levels=50,
                 mean_extra_degree=10.0, B=1024, w_range=1.0, _rng_obj=None, relabel=True):
    """Level 0 = inputs, last level = outputs, hidden nodes split evenly over
    the levels between; in-degree Poisson(mean)+1; sources from any lower
    level (level uniform, then node uniform), first source in the level below."""
    rng = _rng(seed) if _rng_obj is None else _rng_obj
    hidden = n_nodes - n_inputs - n_outputs
    assert n_levels >= 2 and hidden >= 0
    if n_levels == 2:
        assert hidden == 0
        sizes = [n_inputs, n_outputs]
    else:
        sizes = [n_inputs] + _split_even(hidden, n_levels - 2) + [n_outputs]
    assert min(sizes) > 0
    degree = rng.poisson(mean_extra_degree, size=n_nodes - n_inputs) + 1
    n, src, dst, planted = _layered_edges(rng, sizes, degree, p_prev=0.0)
    w = _uniform32(rng, -w_range, w_range, src.shape[0])
    X = rng.random(size=(n_inputs, B), dtype=np.float32)
    inputs = np.arange(n_inputs, dtype=np.int32)
    outputs = np.arange(n - n_outputs, n, dtype=np.int32)
    if relabel:
        src, dst, w, (inputs, outputs), planted = _relabel_and_shuffle(
            rng, n, src, dst, w, [inputs, outputs], planted)
    return Workload(name=CONFIG_NAMES[3], n_nodes=n, src=src, dst=dst, w=w,
                    input_ids=inputs, output_ids=outputs, X=X, planted_level=planted,
                    meta={"seed": seed, "level_sizes": sizes})


# --------------------------------------------------------------------------
# config 4
# --------------------------------------------------------------------------
def deep_narrow(seed=0, n_levels=1000, width=1000, target_edges=16_000_000, B=64,
                zipf_exponent=2.1, max_degree=4096, p_prev=0.7):
    """n_levels levels of ``width`` nodes (level 0 = inputs, last = outputs).
    In-degree d = clip(floor(c * u**(-1/(a-1))), 1, max_degree), u ~ U(0,1): a
    power law with pdf exponent a, whose scale c is found by bisection on the
    same draws so that the edge total is within 1 % of ``target_edges`` (an
    unscaled Zipf(2.1) clipped to [1, 4096] has a mean near 4 and cannot give
    16 edges per node).  70 % of the sources come from the level just below."""
    rng = _rng(seed)
    sizes = [width] * n_levels
    n_dst = width * (n_levels - 1)
    u = rng.random(n_dst)
    tail = u ** (-1.0 / (zipf_exponent - 1.0))

    def total(c):
        return int(np.clip(np.floor(c * tail), 1, max_degree).sum())

    lo, hi = 1e-3, float(max_degree)
    for _ in range(64):
        mid = 0.5 * (lo + hi)
        if total(mid) < target_edges:
            lo = mid
        else:
            hi = mid
    c = hi
    degree = np.clip(np.floor(c * tail), 1, max_degree).astype(np.int64)
    n, src, dst, planted = _layered_edges(rng, sizes, degree, p_prev=p_prev)
    w = _uniform32(rng, -1.0, 1.0, src.shape[0])
    X = rng.random(size=(width, B), dtype=np.float32)
    inputs = np.arange(width, dtype=np.int32)
    outputs = np.arange(n - width, n, dtype=np.int32)
    src, dst, w, (inputs, outputs), planted = _relabel_and_shuffle(
        rng, n, src, dst, w, [inputs, outputs], planted)
    return Workload(name=CONFIG_NAMES[4], n_nodes=n, src=src, dst=dst, w=w,
                    input_ids=inputs, output_ids=outputs, X=X, planted_level=planted,
                    meta={"seed": seed, "degree_scale_c": c, "max_degree": int(degree.max())})


# --------------------------------------------------------------------------
# config 5
# --------------------------------------------------------------------------
def population(seed=0, n_nets=1024, n_inputs=32, n_outputs=8, hidden_range=(500, 4000),
               depth_range=(5, 40), ratio_range=(8.0, 12.0), B=128):
    """A population of distinct networks packed as a disjoint union: node ids
    of net k are offset by net_node_ptr[k]; edges of net k occupy
    [net_edge_ptr[k], net_edge_ptr[k+1]); X rows / input_ids of net k occupy
    [net_input_ptr[k], net_input_ptr[k+1]).  Ids are permuted and edges
    shuffled inside each net."""
    rng = _rng(seed)
    H = rng.integers(hidden_range[0], hidden_range[1] + 1, size=n_nets)
    D = rng.integers(depth_range[0], depth_range[1] + 1, size=n_nets)
    R = rng.uniform(ratio_range[0], ratio_range[1], size=n_nets)
    srcs, dsts, ws, ins, outs, plants = [], [], [], [], [], []
    node_ptr = [0]; edge_ptr = [0]
    for k in range(n_nets):
        n = n_inputs + n_outputs + int(H[k])
        d = int(min(D[k], int(H[k]) + 2))
        sizes = [n_inputs] + _split_even(int(H[k]), d - 2) + [n_outputs]
        lam = max(R[k] * n / (n - n_inputs) - 1.0, 0.0)
        degree = rng.poisson(lam, size=n - n_inputs) + 1
        _, src, dst, planted = _layered_edges(rng, sizes, degree, p_prev=0.0)
        w = _uniform32(rng, -2.0, 2.0, src.shape[0])
        inputs = np.arange(n_inputs, dtype=np.int32)
        outputs = np.arange(n - n_outputs, n, dtype=np.int32)
        src, dst, w, (inputs, outputs), planted = _relabel_and_shuffle(
            rng, n, src, dst, w, [inputs, outputs], planted)
        off = node_ptr[-1]
        srcs.append(src + off); dsts.append(dst + off); ws.append(w)
        ins.append(inputs + off); outs.append(outputs + off); plants.append(planted)
        node_ptr.append(off + n); edge_ptr.append(edge_ptr[-1] + src.shape[0])
    X = rng.random(size=(n_nets * n_inputs, B), dtype=np.float32)
    return Workload(
        name=CONFIG_NAMES[5], n_nodes=node_ptr[-1],
        src=np.concatenate(srcs).astype(np.int32), dst=np.concatenate(dsts).astype(np.int32),
        w=np.concatenate(ws).astype(np.float32),
        input_ids=np.concatenate(ins).astype(np.int32),
        output_ids=np.concatenate(outs).astype(np.int32),
        X=X, planted_level=np.concatenate(plants).astype(np.int32),
        net_node_ptr=np.asarray(node_ptr, dtype=np.int32),
        net_edge_ptr=np.asarray(edge_ptr, dtype=np.int64),
        net_input_ptr=np.arange(n_nets + 1, dtype=np.int32) * n_inputs,
        net_output_ptr=np.arange(n_nets + 1, dtype=np.int32) * n_outputs,
        meta={"seed": seed, "depths": D.tolist()})


# --------------------------------------------------------------------------
def make_config(index: int, scale: str = "full", seed: int = 0) -> Workload:
    """The five workloads at full size, or a ``small`` variant of the same
    recipe that a CPU finishes in well under a second (several tiles wide,
    ragged sizes on purpose)."""
    if scale not in ("full", "small"):
        raise ValueError(scale)
    full = scale == "full"
    if index == 1:
        return tiny_neat(seed=seed)
    if index == 2:
        return pruned_mlp(seed=seed) if full else pruned_mlp(
            seed=seed, layers=(61, 100, 80, 7), keep_edges=0.3, drop_hidden=0.05, B=37)
    if index == 3:
        return layered_skip(seed=seed) if full else layered_skip(
            seed=seed, n_nodes=3011, n_inputs=50, n_outputs=21, n_levels=12, B=131)
    if index == 4:
        return deep_narrow(seed=seed) if full else deep_narrow(
            seed=seed, n_levels=60, width=53, target_edges=53 * 59 * 16, B=19, max_degree=300)
    if index == 5:
        return population(seed=seed) if full else population(
            seed=seed, n_nets=9, hidden_range=(40, 300), depth_range=(3, 12), B=21)
    raise ValueError(index)
