"""Pins for the checker's draft quantification (Section 4.1, Eq. 1): closed forms, hand sums,
invariances and library routines.  None of these re-use the checker's own formula."""
import math

import numpy as np
import pytest
import scipy.special
import scipy.stats

from oracle import draft_entropy_topk


def test_uniform_logits_closed_form():
    V, K = 1000, 10
    r = draft_entropy_topk(np.full((2, V), 3.25, np.float32), K)
    assert np.allclose(r["ent_full"], math.log(V), rtol=0, atol=1e-12)
    assert np.allclose(r["ent_topk"], math.log(K), rtol=0, atol=1e-12)
    assert np.array_equal(r["topk_idx"], np.tile(np.arange(K), (2, 1)))      # ties -> lower index
    assert np.allclose(r["topk_logp"], -math.log(V), atol=1e-12)
    assert np.allclose(r["lse"], 3.25 + math.log(V), atol=1e-12)


def test_one_hot_is_zero_entropy():
    V = 512
    x = np.zeros((1, V), np.float32)
    x[0, 77] = 60.0
    r = draft_entropy_topk(x, 5)
    # the other V-1 tokens hold about V * e^-60 of the mass: entropy ~ V * 60 * e^-60 ~ 3e-22
    assert r["ent_full"][0] < 1e-20 and r["ent_topk"][0] < 1e-20
    assert r["topk_idx"][0, 0] == 77 and list(r["topk_idx"][0, 1:]) == [0, 1, 2, 3]
    y = np.full((1, V), -np.inf, np.float32)
    y[0, 3] = 1.5
    r = draft_entropy_topk(y, 1)
    assert r["ent_full"][0] == 0.0 and r["ent_topk"][0] == 0.0 and r["topk_logp"][0, 0] == 0.0


@pytest.mark.parametrize("a", [0.5, 0.75, 0.9, 0.999])
def test_two_point_binary_entropy(a):
    # two live tokens with probabilities (a, 1-a); the rest are masked out
    x = np.full((1, 64), -np.inf, np.float32)
    x[0, 10], x[0, 40] = math.log(a), math.log(1 - a)
    r = draft_entropy_topk(x, 2)
    h = -a * math.log(a) - (1 - a) * math.log(1 - a)
    assert abs(r["ent_full"][0] - h) < 1e-7          # float32 storage of the logits
    assert abs(r["ent_topk"][0] - h) < 1e-7
    assert list(r["topk_idx"][0]) == ([10, 40] if a >= 0.5 else [40, 10])


def test_eq1_worked_two_token_example():
    # golden/eq1_two_token.txt: Top-K = 2 with renormalised probabilities (0.75, 0.25)
    import os
    vals = {}
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "eq1_two_token.txt")):
        if line.strip() and not line.startswith("#"):
            k, v = line.split("=")
            vals[k.strip()] = float(v)
    # a third, less likely token must not change the Top-2 entropy (renormalisation over the K)
    p = np.array([0.6, 0.2, 0.2 - 1e-3, 1e-3])
    x = np.log(p)[None].astype(np.float32)
    r = draft_entropy_topk(x, 2)
    assert abs(r["ent_topk"][0] - vals["I_t"]) < 1e-6
    assert abs(r["ent_full"][0] - scipy.stats.entropy(p)) < 1e-6


def _geometric_entropy(lam, n):
    """Entropy (nats) of p_v proportional to exp(-lam v), v = 0..n-1, in closed form."""
    r = math.exp(-lam)
    norm = (1 - r) / (1 - r ** n)
    mean = r / (1 - r) - n * r ** n / (1 - r ** n)
    return -math.log(norm) + lam * mean


@pytest.mark.parametrize("lam,V,K", [(0.3, 200, 10), (1.0, 50, 4), (0.05, 3000, 32)])
def test_geometric_distribution_closed_form(lam, V, K):
    x = (-lam * np.arange(V))[None].astype(np.float64)
    r = draft_entropy_topk(x, K)
    assert abs(r["ent_full"][0] - _geometric_entropy(lam, V)) < 1e-10
    assert abs(r["ent_topk"][0] - _geometric_entropy(lam, K)) < 1e-10       # Top-K renormalised
    assert np.array_equal(r["topk_idx"][0], np.arange(K))
    norm = (1 - math.exp(-lam)) / (1 - math.exp(-lam * V))
    assert np.allclose(r["topk_logp"][0], math.log(norm) - lam * np.arange(K), atol=1e-10)


def test_tiny_vocab_by_hand_fsum():
    rs = np.random.RandomState(5)
    for V in (2, 3, 7, 16):
        x = rs.randn(V).astype(np.float32) * 3
        e = [math.exp(float(v)) for v in x]
        z = math.fsum(e)
        p = [v / z for v in e]
        h = -math.fsum(v * math.log(v) for v in p)
        K = min(3, V)
        top = sorted(range(V), key=lambda i: (-float(x[i]), i))[:K]
        zk = math.fsum(p[i] for i in top)
        hk = -math.fsum(p[i] / zk * math.log(p[i] / zk) for i in top)
        r = draft_entropy_topk(x[None], K)
        assert list(r["topk_idx"][0]) == top
        assert abs(r["ent_full"][0] - h) < 1e-12 and abs(r["ent_topk"][0] - hk) < 1e-12
        assert np.allclose(r["topk_logp"][0], [math.log(p[i]) for i in top], atol=1e-12)
        assert abs(r["lse"][0] - math.log(z)) < 1e-12


def test_against_library_routines():
    rs = np.random.RandomState(11)
    x = (rs.randn(4, 777) * rs.uniform(0.3, 8, size=(4, 1))).astype(np.float32)
    for T in (1.0, 0.7, 2.5):
        r = draft_entropy_topk(x, 9, temperature=T)
        ls = scipy.special.log_softmax(x.astype(np.float64) / T, axis=1)
        assert np.allclose(r["ent_full"], scipy.stats.entropy(np.exp(ls), axis=1), atol=1e-12)
        assert np.allclose(r["lse"], scipy.special.logsumexp(x.astype(np.float64) / T, axis=1), atol=1e-12)
        for i in range(4):
            idx = r["topk_idx"][i]
            assert np.allclose(r["topk_logp"][i], ls[i, idx], atol=1e-12)
            assert np.all(np.diff(x[i, idx]) <= 0)                    # descending
            assert x[i, idx[-1]] >= np.delete(x[i], idx).max()        # nothing better left out
            pk = np.exp(ls[i, idx])
            assert abs(r["ent_topk"][i] - scipy.stats.entropy(pk / pk.sum())) < 1e-12


def test_invariances():
    rs = np.random.RandomState(3)
    x = (rs.randn(3, 300) * 4).astype(np.float32)
    base = draft_entropy_topk(x, 8)
    # K = V: the Top-K entropy is the full entropy
    full = draft_entropy_topk(x, 300)
    assert np.allclose(full["ent_topk"], full["ent_full"], atol=1e-12)
    # a common shift changes nothing but lse (shift exactly representable)
    sh = draft_entropy_topk(x + np.float32(8.0), 8)
    x8 = (x + np.float32(8.0)).astype(np.float32)
    ref = draft_entropy_topk(x8, 8)
    assert np.array_equal(sh["topk_idx"], ref["topk_idx"])
    assert np.allclose(draft_entropy_topk(x.astype(np.float64) + 8.0, 8)["ent_full"], base["ent_full"], atol=1e-12)
    # permuting the vocabulary permutes the indices and leaves the entropies alone
    perm = rs.permutation(300)
    pr = draft_entropy_topk(x[:, perm], 8)
    assert np.allclose(pr["ent_full"], base["ent_full"], atol=1e-12)
    assert np.allclose(pr["ent_topk"], base["ent_topk"], atol=1e-12)
    assert np.array_equal(perm[pr["topk_idx"]], base["topk_idx"])
    # temperature: logits * T at temperature T is the same distribution
    t = draft_entropy_topk(x.astype(np.float64) * 2.0, 8, temperature=2.0)
    assert np.allclose(t["ent_topk"], base["ent_topk"], atol=1e-12)
    assert np.allclose(t["topk_logp"], base["topk_logp"], atol=1e-12)


def test_tie_rule_lower_index_first():
    x = np.array([[1.0, 5.0, 5.0, 0.0, 5.0, 2.0]], np.float32)
    r = draft_entropy_topk(x, 4)
    assert list(r["topk_idx"][0]) == [1, 2, 4, 5]
