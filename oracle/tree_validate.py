"""Structural check of packed draft trees (what the library's calls trust their callers for).

Follows the tree conventions of Section 2.2 as this build fixes them: per sequence, row 0 is the
root with parent -1; every other row's parent is an earlier row of the same sequence (BFS order
implies it); the tokens of one node's children are distinct (they are different Top-k picks); a
node has at most MAX_CHILDREN children (the library's sampling accept rules try the children of a
node one after the other and keep lists of that length; Top-k expansion gives a node k children).
Test infrastructure only.
"""
import numpy as np

MAX_CHILDREN = 256


def tree_validate(parent, token, node_offsets):
    """Returns (number of offending rows, global index of the first one or -1).  A row offends if it is
    a root with parent != -1, a non-root whose parent is not in [0, row), or (token given) a non-root
    that shares parent and token with an earlier non-root row (whatever that row's own state), or a
    non-root with MAX_CHILDREN or more earlier rows of the same parent.  Offsets must not decrease (else
    every row of the batch counts as offending)."""
    parent = np.asarray(parent, np.int64)
    offs = np.asarray(node_offsets, np.int64)
    if np.any(np.diff(offs) < 0) or offs[0] != 0:
        return len(parent), 0 if len(parent) else -1
    bad = []
    for s in range(len(offs) - 1):
        o, n = int(offs[s]), int(offs[s + 1] - offs[s])
        seen = set()
        children = {}
        for i in range(n):
            p = int(parent[o + i])
            wrong = (p != -1) if i == 0 else not (0 <= p < i)
            if i > 0 and token is not None:
                key = (p, int(token[o + i]))
                wrong = wrong or key in seen
                seen.add(key)
            if i > 0:
                wrong = wrong or children.get(p, 0) >= MAX_CHILDREN
                children[p] = children.get(p, 0) + 1
            if wrong:
                bad.append(o + i)
    return len(bad), (bad[0] if bad else -1)
