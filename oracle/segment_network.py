"""Set-based network segmentation for small networks -- test infrastructure.

What the paper's segmentation step computes (Sec. "Sequential activation", segmentation
algorithm and the paragraph after it), stated from the definition rather than from the listing:
starting from the input nodes, the next layer is made of the required nodes that are not assigned
yet, receive at least one connection from an assigned node, and whose ENTIRE set of incoming
nodes is already assigned; layers are peeled off until none can be formed.  (The listing's line
that tests a candidate is garbled; the comment above it and the prose after the listing both say
"entire input set", which is the reading taken.)

segment_network(R, IN, OP, CON) -> list of layers after the input layer, each a set of nodes.
A predecessor map is built once; every round looks at each unassigned node.  Quadratic in the
worst case, meant for networks of a few dozen nodes.  OP is accepted because the algorithm is
stated with it; the layering does not depend on it.
"""
from __future__ import annotations


def segment_network(R, IN, OP, CON):
    required = set(R)
    assigned = set(IN)
    incoming = {}
    for a, b in CON:
        incoming.setdefault(b, set()).add(a)
    waiting = {n for n in incoming if n in required and n not in assigned}
    layers = []
    while waiting:
        layer = {n for n in waiting if incoming[n] <= assigned}
        if not layer:
            break           # what is left depends on nodes that can never be assigned
        layers.append(layer)
        assigned |= layer
        waiting -= layer
    return layers
