"""Pins for the checker's tree-masked attention (Section 2.2: tree-mask attention): reductions to
ordinary causal attention, to independent single-query attention, a pure-Python brute force, and
properties that hold for any mask."""
import math

import numpy as np
import pytest
import scipy.special
import torch

from oracle import tree_attention
from oracle.tree_attention import ancestor_mask


def _rand(rs, L, M, Hq, Hkv, D, scale_k=1.0):
    q = rs.randn(M, Hq, D).astype(np.float32)
    kp = (rs.randn(L, Hkv, D) * scale_k).astype(np.float32)
    vp = rs.randn(L, Hkv, D).astype(np.float32)
    kt = (rs.randn(M, Hkv, D) * scale_k).astype(np.float32)
    vt = rs.randn(M, Hkv, D).astype(np.float32)
    return q, kp, vp, kt, vt


def _call(t, parent, L, scale):
    M = len(parent)
    return tree_attention(*t, np.asarray(parent, np.int32), [0, M], [0, L], scale)


def test_chain_tree_is_causal_attention():
    rs = np.random.RandomState(0)
    L, M, Hq, Hkv, D = 37, 9, 4, 2, 16
    t = _rand(rs, L, M, Hq, Hkv, D)
    o, lse = _call(t, np.arange(-1, M - 1), L, 0.25)
    # independent dense causal attention over the L+M positions, last M queries, via torch
    q, kp, vp, kt, vt = (torch.from_numpy(x).double() for x in t)
    K = torch.cat([kp, kt]).repeat_interleave(Hq // Hkv, dim=1)      # [L+M, Hq, D]
    Vv = torch.cat([vp, vt]).repeat_interleave(Hq // Hkv, dim=1)
    causal = torch.ones(L + M, L + M).tril().bool()[L:]               # rows of the last M positions
    ref = torch.nn.functional.scaled_dot_product_attention(
        q.permute(1, 0, 2), K.permute(1, 0, 2), Vv.permute(1, 0, 2), attn_mask=causal, scale=0.25)
    assert np.allclose(o, ref.permute(1, 0, 2).numpy(), atol=1e-12)


def test_star_tree_is_independent_single_queries():
    rs = np.random.RandomState(1)
    L, M, Hq, Hkv, D = 20, 6, 2, 2, 8
    q, kp, vp, kt, vt = _rand(rs, L, M, Hq, Hkv, D)
    parent = [-1] + [0] * (M - 1)
    o, _ = _call((q, kp, vp, kt, vt), parent, L, 0.3)
    for i in range(M):
        rows = [0] if i == 0 else [0, i]                              # prefix + root + itself
        for h in range(Hq):
            keys = np.concatenate([kp[:, h], kt[rows, h]]).astype(np.float64)
            vals = np.concatenate([vp[:, h], vt[rows, h]]).astype(np.float64)
            w = scipy.special.softmax(0.3 * keys @ q[i, h].astype(np.float64))
            assert np.allclose(o[i, h], w @ vals, atol=1e-12)


def test_pure_python_brute_force_with_dense_mask():
    rs = np.random.RandomState(2)
    L, Hq, Hkv, D = 5, 4, 2, 4
    parent = [-1, 0, 0, 1, 1, 2, 4]
    M = len(parent)
    q, kp, vp, kt, vt = _rand(rs, L, M, Hq, Hkv, D)
    o, lse = _call((q, kp, vp, kt, vt), parent, L, 0.5)
    anc = {0: {0}, 1: {0, 1}, 2: {0, 2}, 3: {0, 1, 3}, 4: {0, 1, 4}, 5: {0, 2, 5}, 6: {0, 1, 4, 6}}
    assert all(set(np.nonzero(ancestor_mask(parent)[i])[0]) == anc[i] for i in range(M))
    for i in range(M):
        for h in range(Hq):
            g = h // (Hq // Hkv)
            keys = [(kp[j, g], vp[j, g]) for j in range(L)] + [(kt[j, g], vt[j, g]) for j in sorted(anc[i])]
            sc = [0.5 * math.fsum(float(a) * float(b) for a, b in zip(q[i, h], k)) for k, _ in keys]
            z = math.fsum(math.exp(s) for s in sc)
            for d in range(D):
                want = math.fsum(math.exp(s) / z * float(v[d]) for s, (_, v) in zip(sc, keys))
                assert abs(o[i, h, d] - want) < 1e-12
            assert abs(lse[i, h] - math.log(z)) < 1e-12


def test_constant_values_and_sibling_independence_and_gqa():
    rs = np.random.RandomState(3)
    L, M, Hq, Hkv, D = 11, 8, 4, 2, 8
    parent = [-1, 0, 0, 1, 1, 2, 3, 3]
    q, kp, vp, kt, vt = _rand(rs, L, M, Hq, Hkv, D, scale_k=3.0)
    # all value rows equal -> that row comes out whatever the mask and weights are
    row = rs.randn(D).astype(np.float32)
    o, _ = _call((q, kp, np.broadcast_to(row, vp.shape), kt, np.broadcast_to(row, vt.shape)), parent, L, 1.0)
    assert np.allclose(o, row.astype(np.float64), atol=1e-12)
    # a row never sees a node off its root path: change node 2, rows 1, 3, 4, 6, 7 are bit-identical
    base, _ = _call((q, kp, vp, kt, vt), parent, L, 1.0)
    kt2, vt2 = kt.copy(), vt.copy()
    kt2[2] += 5.0
    vt2[2] -= 3.0
    alt, _ = _call((q, kp, vp, kt2, vt2), parent, L, 1.0)
    for i in (0, 1, 3, 4, 6, 7):
        assert np.array_equal(base[i], alt[i])
    for i in (2, 5):
        assert not np.allclose(base[i], alt[i])
    # grouped-query heads: replicating each KV head G times and using Hkv = Hq is the same thing
    rep = lambda x: np.repeat(x, Hq // Hkv, axis=1)
    full, _ = _call((q, rep(kp), rep(vp), rep(kt), rep(vt)), parent, L, 1.0)
    assert np.array_equal(base, full)


def test_no_prefix_and_ragged_batch_and_bf16_storage():
    rs = np.random.RandomState(4)
    Hq, Hkv, D = 2, 1, 8
    # L = 0: the root attends to itself only -> its output is its own value row
    q, kp, vp, kt, vt = _rand(rs, 0, 3, Hq, Hkv, D)
    o, lse = _call((q, kp, vp, kt, vt), [-1, 0, 1], 0, 0.7)
    assert np.allclose(o[0], np.broadcast_to(vt[0, 0], (Hq, D)), atol=1e-15)
    assert np.allclose(lse[0], 0.7 * (q[0].astype(np.float64) @ kt[0, 0].astype(np.float64)), atol=1e-12)
    # two sequences packed with offsets == each one on its own
    a = _rand(rs, 6, 4, Hq, Hkv, D)
    b = _rand(rs, 9, 2, Hq, Hkv, D)
    pa, pb = [-1, 0, 0, 2], [-1, 0]
    packed = [np.concatenate([x, y]) for x, y in zip(a, b)]
    o, _ = tree_attention(packed[0], packed[1], packed[2], packed[3], packed[4],
                          np.asarray(pa + pb, np.int32), [0, 4, 6], [0, 6, 15], 0.4)
    oa, _ = _call(a, pa, 6, 0.4)
    ob, _ = _call(b, pb, 9, 0.4)
    assert np.array_equal(o[:4], oa) and np.array_equal(o[4:], ob)
    # bfloat16 bit patterns are widened exactly as torch widens them
    bits = rs.randint(0, 1 << 16, size=(6, 1, 8)).astype(np.uint16)
    bits = np.where((bits & 0x7F80) == 0x7F80, np.uint16(0x3F80), bits)      # no inf / nan
    ref = torch.from_numpy(bits.astype(np.int32)).to(torch.int16).view(torch.bfloat16).double().numpy()
    from oracle.tree_attention import _widen
    assert np.array_equal(_widen(bits), ref)


def test_split_invariance_of_the_definition():
    # attention over the prefix may be evaluated in pieces and merged by log-sum-exp weights
    rs = np.random.RandomState(5)
    L, M, Hq, Hkv, D = 64, 3, 2, 2, 8
    t = _rand(rs, L, M, Hq, Hkv, D)
    parent = [-1, 0, 1]
    o, lse = _call(t, parent, L, 0.35)
    q, kp, vp, kt, vt = t
    # piece A: first 40 prefix tokens only (through a no-op tree of the same rows is not possible,
    # so evaluate the pieces directly with scipy)
    for i in range(M):
        for h in range(Hq):
            rows = [j for j in range(M) if ancestor_mask(parent)[i, j]]
            pieces = [(kp[:40, h], vp[:40, h]), (kp[40:, h], vp[40:, h]), (kt[rows, h], vt[rows, h])]
            ls, outs = [], []
            for k, v in pieces:
                s = 0.35 * k.astype(np.float64) @ q[i, h].astype(np.float64)
                ls.append(scipy.special.logsumexp(s))
                outs.append(scipy.special.softmax(s) @ v.astype(np.float64))
            wts = scipy.special.softmax(np.asarray(ls))
            assert np.allclose(o[i, h], sum(w * x for w, x in zip(wts, outs)), atol=1e-12)
            assert abs(lse[i, h] - scipy.special.logsumexp(ls)) < 1e-12
