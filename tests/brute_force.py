"""Brute-force evaluation of tiny ASNNs straight from the definition.

Independent of ``oracle/`` and of the GPU library on purpose: it is what pins
the oracle.  Pure Python, exponential time, for DAGs of a dozen nodes.

value(v): memo-free recursion over incoming edges (Introduction: weighted sum
of incoming node values, then the 4.97-slope sigmoid; sensors squash their
external input; a node with no incoming edge that is no sensor sees an empty
sum).  level(v): length of the longest path ending in v, found by enumerating
every path backwards (the segmentation algorithm admits a node only once its
entire input set is assigned, so its layer is one more than the deepest input).
"""
from __future__ import annotations

import math


def _sig(x: float) -> float:
    t = -4.97 * x
    if t > 700.0:
        return 0.0
    return 1.0 / (1.0 + math.exp(t))


def brute_values(n_nodes, edges, input_ids, x, raw_inputs=False):
    """edges: list of (a, b, w); x: one input vector (list of floats, aligned
    with input_ids).  Returns the list of all node values in exact-ish double
    arithmetic (no float32 rounding of stored values)."""
    slot = {int(v): k for k, v in enumerate(input_ids)}
    incoming = {v: [] for v in range(n_nodes)}
    for (a, b, w) in edges:
        incoming[int(b)].append((int(a), float(w)))

    def value(v):
        if v in slot:
            return float(x[slot[v]]) if raw_inputs else _sig(float(x[slot[v]]))
        total = 0.0
        for (a, w) in incoming[v]:
            total += w * value(a)
        return _sig(total)

    return [value(v) for v in range(n_nodes)]


def brute_levels(n_nodes, edges):
    """Longest path (in edges) ending at each node, by enumerating all paths."""
    incoming = {v: [] for v in range(n_nodes)}
    for e in edges:
        incoming[int(e[1])].append(int(e[0]))

    def longest(v):
        best = 0
        for a in incoming[v]:
            best = max(best, 1 + longest(a))
        return best

    return [longest(v) for v in range(n_nodes)]


def brute_required(n_nodes, edges, output_ids):
    """v is required iff some path leads from v to an output (outputs included), by forward search from each v."""
    outgoing = {v: [] for v in range(n_nodes)}
    for e in edges:
        outgoing[int(e[0])].append(int(e[1]))
    outs = set(int(o) for o in output_ids)

    def reaches(v):
        if v in outs:
            return True
        return any(reaches(b) for b in outgoing[v])

    return [reaches(v) for v in range(n_nodes)]
