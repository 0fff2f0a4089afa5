"""Pins for the checker's level-by-level Top-K expansion (Section 2.2, Expansion): a hand-worked
tree, brute-force ranking by path products, structural invariants, and agreement with the
whole-tree builder of the step pipeline (written separately, driven by the same draft rows)."""
import math
import os

import numpy as np
import pytest

from oracle import draft_entropy_topk
from oracle.tree_expand import new_state, tree_expand
from oracle import pipeline as P
from synth import workloads as W


def _golden():
    rows, sets = [], {}
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "expand_hand_tree.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        if "=" in line:
            k, v = line.split("=")
            sets[k.strip()] = [int(t) for t in v.split()]
        else:
            rows.append([float(t) for t in line.split()])
    return np.asarray(rows), sets


def test_hand_worked_two_levels():
    rows, sets = _golden()
    st = new_state()
    tree_expand(st, [[7, 3]], np.log([[0.6, 0.3]]), [0.64], F=2, cap=64)
    assert st["frontier"] == sets["frontier_after_level_1"]
    tree_expand(st, [[5, 9], [8, 1]], np.log([[0.5, 0.4], [0.9, 0.05]]), [0.69, 0.2], F=2, cap=64)
    assert st["frontier"] == sets["frontier_after_level_2"]
    assert st["parent"] == [int(r) for r in rows[:, 1]] and st["token"] == [int(r) for r in rows[:, 2]]
    assert np.allclose(np.exp(np.asarray(st["cum"], np.float64)), rows[:, 4], rtol=1e-6)
    assert np.allclose(np.exp(np.asarray(st["logc"], np.float64)), rows[:, 3], rtol=1e-6)
    assert st["depth"] == [0, 1, 1, 2, 2, 2, 2] and st["level"] == 2
    assert [float(e) for e in st["ent"][:3]] == [np.float32(0.64), np.float32(0.69), np.float32(0.2)]


def _grow(rs, levels, K, F, cap=10 ** 6, limit=None):
    st = new_state()
    for _ in range(levels):
        nf = len(st["frontier"])
        p = rs.dirichlet(np.ones(K + 3), size=max(nf, 1))[:, :K]
        p = -np.sort(-p, axis=1)
        idx = np.stack([rs.permutation(1000)[:K] for _ in range(max(nf, 1))])
        tree_expand(st, idx, np.log(p), rs.uniform(0, 2, size=max(nf, 1)), F, cap, limit)
    return st


def test_frontier_is_the_top_F_by_path_product():
    rs = np.random.RandomState(0)
    for trial in range(100):
        K, F = int(rs.randint(2, 5)), int(rs.randint(1, 4))
        st = _grow(rs, int(rs.randint(1, 5)), K, F)
        n = len(st["parent"])
        value = np.ones(n)
        for i in range(1, n):                               # explicit products in float64
            value[i] = value[st["parent"][i]] * math.exp(float(st["logc"][i]))
        deepest = max(st["depth"])
        level = [i for i in range(n) if st["depth"][i] == deepest]
        want = sorted(sorted(level, key=lambda i: (-value[i], i))[:F])
        assert st["frontier"] == want, trial
        assert np.allclose(np.exp(np.asarray(st["cum"], np.float64)), value, rtol=1e-5)


def test_structure():
    rs = np.random.RandomState(1)
    K, F, levels = 3, 2, 5
    st = _grow(rs, levels, K, F)
    n = len(st["parent"])
    assert n == 1 + K + (levels - 1) * F * K                # root, its K children, then F * K per level
    par = st["parent"]
    assert all(par[i] < i for i in range(1, n)) and all(par[i] <= par[i + 1] for i in range(1, n - 1))   # BFS order
    assert all(st["depth"][i] == st["depth"][par[i]] + 1 for i in range(1, n))
    assert all(st["cum"][i] <= st["cum"][par[i]] for i in range(1, n))                                    # V bounded by ancestors
    expanded = sorted(set(par[1:]))
    assert all(par.count(f) == K for f in expanded)
    assert all(st["ent"][i] == 0 for i in range(n) if i not in expanded)


def test_capacity_and_depth_limit():
    rs = np.random.RandomState(2)
    st = _grow(rs, 4, 3, 2, cap=12)                         # 1 + 3 + 6 = 10 rows; three more would make 13
    assert len(st["parent"]) == 10 and st["frontier"] == []
    st = _grow(rs, 3, 3, 2, cap=13)                         # the first frontier row's children fit, the second's do not
    assert len(st["parent"]) == 13 and st["parent"][10:] == [st["parent"][10]] * 3
    st = _grow(rs, 6, 2, 2, limit=3)
    assert st["level"] == 3 and max(st["depth"]) == 3 and st["frontier"] == []


def test_agrees_with_the_whole_tree_builder():
    """Level by level with the checker's quantification of the same seeded draft rows gives the
    tree that the step pipeline grows in one go."""
    w = W.small(W.WORKLOADS[2], V=600, topk=4, frontier=3, max_depth=4)
    ref = P.expand_tree(w, 0, 0, w.max_depth)
    st = new_state()
    for d in range(w.max_depth):
        x = W.logits_rows(w, 0, "draft", 0, st["frontier"])
        r = draft_entropy_topk(x, w.topk, w.temperature)
        tree_expand(st, r["topk_idx"], r["topk_logp"].astype(np.float32), r["ent_topk"], w.frontier, 10 ** 6)
    assert st["parent"] == list(ref["parent"]) and st["token"] == list(ref["token"])
    assert np.allclose(np.asarray(st["logc"], np.float64), ref["logc"], atol=1e-6)
