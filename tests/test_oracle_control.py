"""Pins for the checker's complexity quantification and adaptive decision (Sections 4.1 - 4.3):
hand-worked values of the Section 4.3 formulas, closed forms of Eq. 1 on uniform rows, brute-force
enumeration of the deepest paths, and a library routine for the bin lookup."""
import math
import os

import numpy as np
import pytest

from oracle import adaptive_control, draft_entropy_topk

GAMMA = [0.3, 0.6, 1.0]
EDGES8 = [0.5, 1.0, 1.5, 2.5, 4.0, 6.0, 9.0]          # synthetic: the paper prints no boundaries


def _run(parent, logc, ent, edges=EDGES8, gamma=GAMMA, alpha=3, d_base=5, n_default=20, mode=0):
    n = len(parent)
    return adaptive_control(np.asarray(parent, np.int32), np.asarray(logc, np.float32),
                            np.asarray(ent, np.float32), [0, n], edges, gamma, alpha, d_base, n_default, mode)


def _golden():
    rows = []
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "control_figure_example.txt")):
        line = line.strip()
        if line and not line.startswith("#"):
            rows.append([int(t) for t in line.split()])
    return rows


def test_section_4_3_formulas_on_the_figure_example():
    """A two-node tree whose single path entropy is placed in each bin in turn."""
    mids = [0.25, 0.75, 1.25, 2.0, 3.0, 5.0, 7.0, 20.0]
    for (b, delta, dp, npr), phi in zip(_golden(), mids):
        r = _run([-1, 0], [0.0, -0.1], [phi, 99.0])
        assert int(r["bin"][0]) == b and abs(r["phi"][0] - np.float32(phi)) < 1e-6
        assert int(r["d_prime"][0]) == dp and int(r["n_prime"][0]) == npr, (b, r)


def test_chain_path_entropy_excludes_the_last_nodes_own_row():
    """A chain of T tokens has T terms: the rows of the root and of the first T - 1 tokens."""
    rs = np.random.RandomState(0)
    n = 9
    ent = rs.uniform(0.0, 2.0, size=n).astype(np.float32)
    ent[-1] = 1000.0                                     # the leaf was never expanded: must not count
    r = _run(list(range(-1, n - 1)), [0.0] + [-0.3] * (n - 1), ent)
    assert int(r["pstar"][0]) == n - 1
    assert abs(r["phi"][0] - math.fsum(float(x) for x in ent[:-1])) < 1e-12


def test_uniform_rows_give_T_log_K():
    """Eq. 1 on rows that are uniform over their Top-K: every term is ln K."""
    K, V, T = 4, 32, 5
    rows = np.full((T, V), -50.0, np.float32)
    rows[:, :K] = 0.0
    e = draft_entropy_topk(rows, K, 1.0)["ent_topk"]
    assert np.allclose(e, math.log(K), atol=1e-12)
    ent = list(e) + [7.0]
    r = _run(list(range(-1, T)), [0.0] + [math.log(1.0 / K)] * T, ent)
    assert abs(r["phi"][0] - T * math.log(K)) < 1e-5


def _brute(parent, prob, ent, mode):
    """All root-to-deepest-level paths, explicit products in float64."""
    n = len(parent)
    children = {i: [j for j in range(n) if parent[j] == i] for i in range(n)}
    paths = []

    def walk(i, path, value):
        if not children[i]:
            paths.append((path, value))
        for c in children[i]:
            walk(c, path + [c], value * prob[c])
    walk(0, [0], 1.0)
    D = max(len(p) for p, _ in paths)
    deep = [(p, v) for p, v in paths if len(p) == D]
    if mode == 0:
        p, _ = max(deep, key=lambda t: (t[1], -t[0][-1]))
    else:
        p, _ = max(deep, key=lambda t: (prob[t[0][-1]], -t[0][-1]))
    return p[-1], math.fsum(float(ent[a]) for a in p[:-1])


@pytest.mark.parametrize("mode", [0, 1])
def test_operational_path_against_brute_force(mode):
    rs = np.random.RandomState(3 + mode)
    for trial in range(200):
        n = int(rs.randint(2, 14))
        parent = [-1] + [int(rs.randint(max(0, i - 4), i)) for i in range(1, n)]
        prob = np.concatenate([[1.0], rs.uniform(0.05, 0.95, size=n - 1)])
        ent = rs.uniform(0.0, 2.3, size=n).astype(np.float32)
        want_node, want_phi = _brute(parent, prob, ent, mode)
        r = _run(parent, np.log(prob), ent, mode=mode)
        assert int(r["pstar"][0]) == want_node and abs(r["phi"][0] - want_phi) < 1e-9, trial


def test_bin_lookup_is_searchsorted():
    rs = np.random.RandomState(5)
    edges = np.sort(rs.uniform(0.0, 5.0, size=7)).astype(np.float32)
    for _ in range(300):
        phi = np.float32(rs.uniform(-0.5, 6.0))
        r = _run([-1, 0], [0.0, -1.0], [phi, 0.0], edges=edges)
        assert int(r["bin"][0]) == int(np.searchsorted(edges, phi, side="right"))
    for j, e in enumerate(edges):                        # a value on a boundary belongs to the upper bin
        assert int(_run([-1, 0], [0.0, -1.0], [e, 0.0], edges=edges)["bin"][0]) == j + 1


def test_root_only_tree_empty_sequence_and_batches():
    r = _run([-1], [0.0], [3.0])
    assert int(r["pstar"][0]) == 0 and r["phi"][0] == 0.0 and int(r["bin"][0]) == 0
    assert int(r["d_prime"][0]) == 8 and int(r["n_prime"][0]) == 9
    parent = np.asarray([-1, 0, 0, -1, 0, 1], np.int32)
    logc = np.asarray([0, -0.2, -0.1, 0, -0.5, -0.5], np.float32)
    ent = np.asarray([0.7, 0, 0, 2.0, 3.0, 0], np.float32)
    r = adaptive_control(parent, logc, ent, [0, 3, 3, 6], EDGES8, GAMMA, 3, 5, 20)
    assert list(r["pstar"]) == [2, -1, 2] and list(r["bin"][[0, 2]]) == [1, 5]
    assert abs(r["phi"][2] - 5.0) < 1e-12 and list(r["d_prime"]) == [7, 5, 5] and list(r["n_prime"]) == [14, 20, 20]


def test_rounding_and_clamping_of_the_budget():
    # gamma * N_default + 0.5 is floored: 0.3 * 55 = 16.5 in exact arithmetic, but gamma is the
    # float32 nearest to 0.3 (slightly above), so the product is just above 16.5 -> 17
    r = _run([-1, 0], [0.0, -1.0], [0.1, 0.0], n_default=55)
    assert int(r["n_prime"][0]) == 17 + 3
    # alpha below the bin number: no negative extension
    r = _run([-1, 0], [0.0, -1.0], [1.2, 0.0], alpha=1)
    assert int(r["bin"][0]) == 2 and int(r["d_prime"][0]) == 5 and int(r["n_prime"][0]) == 20


def test_more_entropy_never_lowers_the_bin():
    rs = np.random.RandomState(9)
    parent = [-1, 0, 1, 2, 3]
    ent = rs.uniform(0, 1, size=5).astype(np.float32)
    last = -1
    for bump in np.linspace(0, 6, 25):
        e = ent.copy()
        e[1] += np.float32(bump)
        b = int(_run(parent, [0, -1, -1, -1, -1], e)["bin"][0])
        assert b >= last
        last = b
