"""Pins for the checker's structural tree check: hand-made trees with known defects, and agreement
with a reachability test (every row of a valid tree reaches its root by following parents)."""
import numpy as np

from oracle.tree_validate import tree_validate


def test_known_defects():
    good = [-1, 0, 0, 1, 1, 2]
    assert tree_validate(good, None, [0, 6]) == (0, -1)
    assert tree_validate(good, [9, 4, 5, 7, 8, 7], [0, 6]) == (0, -1)          # equal tokens under different parents
    assert tree_validate(good, [9, 4, 5, 7, 7, 7], [0, 6]) == (1, 4)           # siblings 3 and 4 share token 7
    assert tree_validate([0, 0, 0], None, [0, 3]) == (1, 0)                    # root with a parent
    assert tree_validate([-1, 1, 0], None, [0, 3]) == (1, 1)                   # own parent
    assert tree_validate([-1, 2, 1], None, [0, 3]) == (1, 1)                   # parent after the row
    assert tree_validate([-1, -1, 0], None, [0, 3]) == (1, 1)                  # a second root
    assert tree_validate([-1, 0, -1, 0, 5], None, [0, 2, 5]) == (1, 4)         # parent outside the sequence
    assert tree_validate([], None, [0, 0, 0]) == (0, -1)
    assert tree_validate([-1, 0], None, [0, 2, 1])[0] == 2                     # decreasing offsets
    star = [-1] + [0] * 300                                                    # the root has 300 children:
    assert tree_validate(star, None, [0, 301]) == (44, 257)                    # those after the 256th offend
    assert tree_validate([-1] + [0] * 256, None, [0, 257]) == (0, -1)


def test_valid_iff_every_row_reaches_the_root_through_earlier_rows():
    rs = np.random.RandomState(0)
    for _ in range(300):
        n = int(rs.randint(1, 12))
        parent = rs.randint(-2, n, size=n)
        parent[0] = -1 if rs.uniform() < 0.9 else 0
        ok = parent[0] == -1
        for i in range(1, n):
            j, steps = i, 0
            while j > 0 and 0 <= parent[j] < j:
                j, steps = parent[j], steps + 1
            ok = ok and j == 0
        assert (tree_validate(parent, None, [0, n])[0] == 0) == ok
