"""Pins for the checker's pruning (Section 2.2 reranking, Section 4.3 node budget): a hand-worked
tree, brute-force path products, and the invariants the paper's validity argument rests on."""
import math
import os

import numpy as np
import pytest

from oracle import tree_prune

INT_MAX = 2 ** 31 - 1
NINF = float("-inf")


def _run(parent, logc, d_max=INT_MAX, theta=NINF, max_nodes=0):
    n = len(parent)
    return tree_prune(np.asarray(parent, np.int32), np.asarray(logc, np.float32), [0, n],
                      [d_max], [theta], [max_nodes])


def _hand_tree():
    rows, sets = [], {}
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "prune_hand_tree.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        if "=" in line:
            k, v = line.split("=")
            sets[k.strip()] = [int(t) for t in v.split()]
        else:
            rows.append([float(t) for t in line.split()])
    rows = np.asarray(rows)
    return rows[:, 1].astype(int), rows[:, 2], rows[:, 3], sets


def test_hand_worked_tree():
    parent, c, value, sets = _hand_tree()
    logc = np.log(c)
    r = _run(parent, logc)
    assert np.allclose(np.exp(r["cumlogp"].astype(np.float64)), value, rtol=1e-6)
    assert list(r["depth"]) == [0, 1, 1, 2, 2, 2, 3, 3]
    assert list(np.nonzero(_run(parent, logc, max_nodes=4)["keep"])[0]) == [0] + sets["top4"]
    assert list(np.nonzero(_run(parent, logc, theta=math.log(0.1))["keep"])[0]) == [0] + sets["thr0.1"]
    assert list(np.nonzero(_run(parent, logc, d_max=1)["keep"])[0]) == [0] + sets["depth1"]
    # renumbering: kept 0 1 2 3 5 -> node 5 (child of 2) becomes row 4 with parent 2
    r4 = _run(parent, logc, max_nodes=4)
    assert list(r4["out_src"]) == [0, 1, 2, 3, 5] and list(r4["out_parent"]) == [-1, 0, 0, 1, 2]
    assert list(r4["out_offsets"]) == [0, 5]


def _random_tree(rs, n, maxfan=4):
    parent = [-1]
    for i in range(1, n):
        parent.append(int(rs.randint(max(0, i - 6), i)))
    return np.asarray(parent, np.int32)


def _brute(parent, prob, d_max, vmin, budget):
    """Definition by explicit path enumeration in float64 products."""
    n = len(parent)
    paths = []
    for i in range(n):
        p, j = [], i
        while j > 0:
            p.append(j)
            j = int(parent[j])
        paths.append(p[::-1])
    val = [math.prod(prob[j] for j in p) for p in paths]
    ok = [all(len(paths[j]) <= d_max and val[j] >= vmin for j in p) for p in paths]
    cand = [i for i in range(1, n) if ok[i]]
    if budget > 0 and len(cand) > budget:
        cand = sorted(cand, key=lambda i: (-val[i], i))[:budget]
    return sorted([0] + cand), val


@pytest.mark.parametrize("seed", range(12))
def test_brute_force_small_trees(seed):
    rs = np.random.RandomState(seed)
    n = int(rs.randint(2, 40))
    parent = _random_tree(rs, n)
    prob = rs.uniform(0.05, 1.0, size=n)
    prob[0] = 1.0
    d_max = int(rs.randint(1, 7))
    vmin = float(rs.choice([0.0, 1e-3, 0.02, 0.2]))
    budget = int(rs.choice([0, 1, 3, 8, 20]))
    kept, val = _brute(parent, prob, d_max, vmin, budget)
    r = _run(parent, np.log(prob), d_max, math.log(vmin) if vmin > 0 else NINF, budget)
    # float32 sums vs float64 products agree unless a value sits within rounding of a cut
    near = min([abs(v - vmin) / max(vmin, 1e-30) for v in val[1:]] + [1.0])
    if near > 1e-4:
        assert list(np.nonzero(r["keep"])[0]) == kept
    assert np.allclose(np.exp(r["cumlogp"].astype(np.float64)), val, rtol=1e-5)


@pytest.mark.parametrize("seed", range(8))
def test_invariants(seed):
    rs = np.random.RandomState(100 + seed)
    n = int(rs.randint(5, 200))
    parent = _random_tree(rs, n)
    logc = -rs.exponential(1.0, size=n)
    logc[0] = 0.0
    r = _run(parent, logc, d_max=int(rs.randint(2, 9)), theta=-float(rs.uniform(1, 8)),
             max_nodes=int(rs.randint(1, 60)))
    keep = r["keep"].astype(bool)
    S = r["cumlogp"]
    assert keep[0]
    for i in range(1, n):
        assert S[i] <= S[parent[i]]                       # value bounded by the ancestors'
        if keep[i]:
            assert keep[parent[i]]                        # kept set is ancestor-closed
    src, par = r["out_src"], r["out_parent"]
    assert list(src) == list(np.nonzero(keep)[0])
    assert par[0] == -1 and all(0 <= par[j] < j for j in range(1, len(par)))
    for j in range(1, len(par)):
        assert src[par[j]] == parent[src[j]]              # renumbered parent is the same node
    assert r["out_offsets"][1] == keep.sum()


def test_filters_off_is_identity_and_threshold_extremes():
    rs = np.random.RandomState(7)
    parent = _random_tree(rs, 50)
    logc = -rs.exponential(0.5, size=50)
    r = _run(parent, logc)
    assert r["keep"].all() and list(r["out_parent"]) == list(parent)
    r = _run(parent, logc, theta=1e-30)                    # nothing but the root has S >= 0+
    assert list(np.nonzero(r["keep"])[0]) == [0]
    chain = np.arange(-1, 19)
    r = _run(chain, np.zeros(20), theta=0.0, d_max=19, max_nodes=19)   # all c = 1
    assert r["keep"].all()
    r = _run(chain, np.zeros(20), d_max=5)
    assert list(np.nonzero(r["keep"])[0]) == list(range(6))
    r = _run(chain, np.full(20, 1e-6))                      # log c slightly above 0 is clamped
    assert np.all(r["cumlogp"] == 0.0)


def test_lower_threshold_never_removes_a_node():
    rs = np.random.RandomState(9)
    parent = _random_tree(rs, 129)
    logc = -rs.exponential(1.2, size=129)
    kept = [set(np.nonzero(_run(parent, logc, theta=t)["keep"])[0]) for t in (-2.0, -4.0, -8.0)]
    assert kept[0] <= kept[1] <= kept[2] and len(kept[0]) < len(kept[2])


def test_budget_ties_stay_ancestor_closed():
    # every confidence is 1/2: many equal values; the cut must still take parents before children
    parent = np.asarray([-1, 0, 0, 1, 1, 2, 2, 3, 3, 4], np.int32)
    logc = np.full(10, math.log(0.5))
    for budget in range(1, 9):
        keep = _run(parent, logc, max_nodes=budget)["keep"].astype(bool)
        assert keep.sum() == budget + 1
        assert list(np.nonzero(keep)[0]) == list(range(budget + 1))     # BFS order == (value, index) order
        assert all(keep[parent[i]] for i in range(1, 10) if keep[i])


def test_batch_of_ragged_sequences():
    rs = np.random.RandomState(21)
    sizes = [1, 17, 0, 40, 3]
    parents, logcs = [], []
    for n in sizes:
        if n:
            parents.append(_random_tree(rs, n))
            c = -rs.exponential(1.0, size=n)
            c[0] = 0
            logcs.append(c)
    offs = np.concatenate([[0], np.cumsum(sizes)])
    B = len(sizes)
    r = tree_prune(np.concatenate(parents), np.concatenate(logcs).astype(np.float32), offs,
                   [4] * B, [-3.0] * B, [6] * B)
    k = 0
    for s, n in enumerate(sizes):
        if n == 0:
            assert r["out_offsets"][s + 1] == r["out_offsets"][s]
            continue
        one = _run(parents[k], logcs[k], 4, -3.0, 6)
        k += 1
        a, b = r["out_offsets"][s], r["out_offsets"][s + 1]
        assert np.array_equal(r["out_src"][a:b], one["out_src"])
        assert np.array_equal(r["out_parent"][a:b], one["out_parent"])
        assert np.array_equal(r["keep"][offs[s]:offs[s + 1]], one["keep"])
