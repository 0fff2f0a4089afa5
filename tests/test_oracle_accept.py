"""Pins for the checker's accept walk (Section 2.1 rule; Section 2.2 tree verification): brute-force
path enumeration, planted paths, textbook chain speculative sampling, and the exact output
distribution on tiny vocabularies."""
import itertools
import math

import numpy as np
import pytest

from oracle import verify_accept
from oracle.verify_accept import GREEDY, STOCHASTIC, STOCHASTIC_POINTMASS


def _random_tree(rs, n):
    return np.asarray([-1] + [int(rs.randint(max(0, i - 5), i)) for i in range(1, n)], np.int32)


def _distinct_sibling_tokens(rs, parent, V):
    token = np.full(len(parent), -1, np.int32)
    for p in range(len(parent)):
        kids = [c for c in range(1, len(parent)) if parent[c] == p]
        token[kids] = rs.choice(V, size=len(kids), replace=False)
    return token


def _depths(parent):
    d = [0] * len(parent)
    for i in range(1, len(parent)):
        d[i] = d[parent[i]] + 1
    return d


@pytest.mark.parametrize("seed", range(10))
def test_greedy_is_longest_confirmed_path_brute_force(seed):
    rs = np.random.RandomState(seed)
    n, V = int(rs.randint(2, 30)), 6                     # tiny vocabulary -> matches are common
    parent = _random_tree(rs, n)
    token = _distinct_sibling_tokens(rs, parent, V)
    tl = rs.randn(n, V).astype(np.float32)
    am = tl.argmax(axis=1)
    # enumerate every root-to-node path; a path is confirmed if each token is the argmax at its parent
    best = []
    for i in range(n):
        path, j = [], i
        while j > 0:
            path.append(j)
            j = int(parent[j])
        path = path[::-1]
        if all(token[c] == am[parent[c]] for c in path) and len(path) > len(best):
            best = path
    D = max(1, max(_depths(parent)))
    r = verify_accept(tl, None, token, parent, [0, n], GREEDY, 1.0, None, D)
    assert r["accept_len"][0] == len(best)
    assert list(r["accept_path"][0, :len(best)]) == best
    assert all(r["accept_path"][0, len(best):] == -1)
    stop = best[-1] if best else 0
    assert r["bonus_token"][0] == am[stop]


def test_planted_path_and_batch():
    rs = np.random.RandomState(42)
    V = 50
    trees = []
    for n in (12, 1, 25):
        parent = _random_tree(rs, n)
        token = _distinct_sibling_tokens(rs, parent, V)
        tl = rs.randn(n, V).astype(np.float32)
        tl[np.arange(n), rs.randint(0, V, size=n)] += 0.0
        # make the target confirm a chosen root-to-leaf path and nothing beyond it
        leaf = n - 1
        path, j = [], leaf
        while j > 0:
            path.append(j)
            j = int(parent[j])
        path = path[::-1]
        for c in path:
            tl[parent[c], token[c]] = 30.0
        kids_of_leaf = [c for c in range(1, n) if parent[c] == leaf]
        assert not kids_of_leaf
        trees.append((parent, token, tl, path))
    offs = np.concatenate([[0], np.cumsum([len(t[0]) for t in trees])])
    r = verify_accept(np.concatenate([t[2] for t in trees]), None, np.concatenate([t[1] for t in trees]),
                      np.concatenate([t[0] for t in trees]), offs, GREEDY, 1.0, None, 25)
    for s, (parent, token, tl, path) in enumerate(trees):
        assert r["accept_len"][s] == len(path)
        assert list(r["accept_path"][s, :len(path)]) == path
        assert r["bonus_token"][s] == tl[path[-1] if path else 0].argmax()


def _textbook_chain(p_rows, q_rows, tokens, u_nodes, u_bonus):
    """Speculative sampling on a chain of drafts, as in Section 2.1."""
    n_acc = 0
    for i, x in enumerate(tokens):
        p, q = p_rows[i], q_rows[i]
        if u_nodes[i] < min(1.0, p[x] / q[x]):
            n_acc += 1
            continue
        res = np.maximum(p - q, 0)
        res /= res.sum()
        return n_acc, int(np.searchsorted(np.cumsum(res), u_bonus, side="right"))
    p = p_rows[len(tokens)]
    return n_acc, int(np.searchsorted(np.cumsum(p), u_bonus, side="right"))


@pytest.mark.parametrize("seed", range(20))
def test_chain_tree_is_textbook_speculative_sampling(seed):
    rs = np.random.RandomState(seed)
    k, V = 5, 12
    tl = (rs.randn(k + 1, V) * 1.5).astype(np.float32)
    dl = (tl + rs.randn(k + 1, V) * 0.7).astype(np.float32)
    sm = lambda x: np.exp(x.astype(np.float64) - x.max()) / np.exp(x.astype(np.float64) - x.max()).sum()
    P = [sm(r) for r in tl]
    Q = [sm(r) for r in dl]
    tokens = [int(rs.choice(V, p=Q[i])) for i in range(k)]            # drafts sampled from q
    parent = np.arange(-1, k)
    token = np.asarray([-1] + tokens, np.int32)
    u = rs.uniform(size=k + 2).astype(np.float32)
    r = verify_accept(tl, dl, token, parent, [0, k + 1], STOCHASTIC, 1.0, u, k)
    n_acc, bonus = _textbook_chain(P, Q, tokens, u[1:k + 1], float(u[k + 1]))
    assert r["accept_len"][0] == n_acc and r["bonus_token"][0] == bonus
    assert list(r["accept_path"][0, :n_acc]) == list(range(1, n_acc + 1))


def _first_token_distribution(tl, dl, kids_tokens, mode, V):
    """Exact law of the first emitted token for a root with the given children, found from the
    checker as a black box: each accept test is a threshold in its own uniform (bisection), and
    the bonus draw is a step function of its uniform (bisection on each step)."""
    k = len(kids_tokens)
    n = k + 1
    parent = np.asarray([-1] + [0] * k, np.int32)
    token = np.asarray([-1] + list(kids_tokens), np.int32)
    TL = np.zeros((n, V), np.float32)
    DL = np.zeros((n, V), np.float32)
    TL[0], DL[0] = tl, dl

    def run(u_nodes, u_bonus):
        u = np.asarray([0.0] + list(u_nodes) + [u_bonus], np.float64)
        r = verify_accept(TL, DL, token, parent, [0, n], mode, 1.0, u, 1)
        return (int(r["accept_path"][0, 0]), int(r["bonus_token"][0]))

    dist = np.zeros(V)
    reach = 1.0
    u_nodes = [1.0 - 1e-16] * k                      # everything rejected unless lowered
    for j in range(k):
        lo, hi = 0.0, 1.0                            # accept iff u_j < t_j
        probe = list(u_nodes)
        for _ in range(60):
            mid = 0.5 * (lo + hi)
            probe[j] = mid
            if run(probe, 0.5)[0] == j + 1:
                lo = mid
            else:
                hi = mid
        t = 1.0 if hi >= 1.0 - 1e-12 else 0.5 * (lo + hi)
        dist[kids_tokens[j]] += reach * t
        reach *= 1.0 - t
        if reach <= 0:
            break
    if reach > 0:
        # bonus token as a function of its uniform: find every step
        edges = [0.0]
        cur = run(u_nodes, 0.0)[1]
        seq = [cur]
        while True:
            if run(u_nodes, 1.0 - 1e-15)[1] == cur:
                break
            lo, hi = edges[-1], 1.0
            for _ in range(60):
                mid = 0.5 * (lo + hi)
                if run(u_nodes, mid)[1] == cur:
                    lo = mid
                else:
                    hi = mid
            edges.append(0.5 * (lo + hi))
            cur = run(u_nodes, hi + 1e-15)[1]
            seq.append(cur)
        edges.append(1.0)
        for tkn, a, b in zip(seq, edges[:-1], edges[1:]):
            dist[tkn] += reach * (b - a)
    return dist


@pytest.mark.parametrize("seed", range(4))
def test_pointmass_mode_reproduces_target_exactly(seed):
    # whatever the (deterministic) candidate set, the first emitted token follows p
    rs = np.random.RandomState(seed)
    V = 6
    tl = (rs.randn(V) * 1.2).astype(np.float32)
    dl = (rs.randn(V) * 1.2).astype(np.float32)
    p = np.exp(tl.astype(np.float64)) / np.exp(tl.astype(np.float64)).sum()
    kids = list(rs.choice(V, size=3, replace=False))
    dist = _first_token_distribution(tl, dl, kids, STOCHASTIC_POINTMASS, V)
    assert np.allclose(dist, p, atol=1e-9)


@pytest.mark.parametrize("seed", range(3))
def test_ratio_mode_reproduces_target_when_children_are_drawn_from_the_draft(seed):
    # two children drawn from q without replacement: averaged over the draws, the first
    # emitted token follows p exactly (the guarantee of Section 2.1 carried to several candidates)
    rs = np.random.RandomState(10 + seed)
    V = 4
    tl = (rs.randn(V) * 1.0).astype(np.float32)
    dl = (rs.randn(V) * 1.0).astype(np.float32)
    p = np.exp(tl.astype(np.float64)) / np.exp(tl.astype(np.float64)).sum()
    q = np.exp(dl.astype(np.float64)) / np.exp(dl.astype(np.float64)).sum()
    total = np.zeros(V)
    for x1, x2 in itertools.permutations(range(V), 2):
        pr = q[x1] * q[x2] / (1.0 - q[x1])
        total += pr * _first_token_distribution(tl, dl, [x1, x2], STOCHASTIC, V)
    assert np.allclose(total, p, atol=1e-8)


def test_one_hot_target_makes_stochastic_walk_greedy():
    rs = np.random.RandomState(77)
    n, V = 20, 9
    parent = _random_tree(rs, n)
    token = _distinct_sibling_tokens(rs, parent, V)
    tl = rs.randn(n, V).astype(np.float32)
    tl[np.arange(n), rs.randint(0, V, size=n)] += 80.0               # p is one-hot to 1e-30
    dl = rs.randn(n, V).astype(np.float32)
    D = max(_depths(parent))
    g = verify_accept(tl, None, token, parent, [0, n], GREEDY, 1.0, None, D)
    for mode in (STOCHASTIC, STOCHASTIC_POINTMASS):
        for rep in range(5):
            u = rs.uniform(0.0, 0.999, size=n + 1).astype(np.float32)
            s = verify_accept(tl, dl, token, parent, [0, n], mode, 1.0, u, D)
            assert all(np.array_equal(s[k], g[k]) for k in g)
    # and so does a low temperature on an ordinary target
    tl2 = rs.randn(n, V).astype(np.float32)
    g = verify_accept(tl2, None, token, parent, [0, n], GREEDY, 1.0, None, D)
    u = rs.uniform(0.0, 0.999, size=n + 1).astype(np.float32)
    s = verify_accept(tl2, dl, token, parent, [0, n], STOCHASTIC_POINTMASS, 1e-3, u, D)
    assert all(np.array_equal(s[k], g[k]) for k in g)


def test_walk_outputs_are_well_formed():
    rs = np.random.RandomState(5)
    n, V = 40, 5
    parent = _random_tree(rs, n)
    token = _distinct_sibling_tokens(rs, parent, V)
    D = max(_depths(parent))
    for mode in (GREEDY, STOCHASTIC, STOCHASTIC_POINTMASS):
        for rep in range(10):
            tl = rs.randn(n, V).astype(np.float32)
            dl = rs.randn(n, V).astype(np.float32)
            u = rs.uniform(size=n + 1).astype(np.float32)
            r = verify_accept(tl, dl, token, parent, [0, n], mode, 1.0, u, D)
            k = int(r["accept_len"][0])
            path = list(r["accept_path"][0, :k])
            assert 0 <= k <= D and all(r["accept_path"][0, k:] == -1)
            prev = 0
            for c in path:
                assert parent[c] == prev
                prev = c
            assert 0 <= r["bonus_token"][0] < V
