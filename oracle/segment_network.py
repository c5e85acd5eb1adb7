"""The paper's set-based network segmentation, written out for small networks.

Follows the "Network segmentation algorithm" (Sec. "Sequential activation") in
its own notation: R = required nodes, IN = input nodes, OP = output nodes,
CON = set of connections (a, b); s = nodes already assigned; c = candidates of
the next layer; t = candidates whose entire input set lies in s.  The garbled
"all <- (...)" line is read as: all(a in s for every (a, b) in CON with b = n),
which is what the comment above it and the prose after the listing say.

Returns the list of layers *after* the input layer, each a set of nodes, as the
algorithm does (L excludes IN).  Test infrastructure; quadratic, tiny inputs only.
"""
from __future__ import annotations


def segment_network(R, IN, OP, CON):
    R = set(R)
    CON = list(CON)
    L = []
    s = set(IN)
    while True:
        # candidate nodes for the next layer
        c = {b for (a, b) in CON if a in s and b not in s}
        # used nodes whose entire input set is in s
        t = set()
        for n in c:
            entire = all(a in s for (a, b) in CON if b == n)
            if n in R and entire:
                t = t | {n}
        if not t:
            break
        L = L + [t]
        s = s | t
    return L
