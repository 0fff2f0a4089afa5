"""Pins for the checker's commit of the accepted path into the KV cache (Section 2.1: accepted
tokens join the context, later drafts are discarded): the cache after commits equals the plain
concatenation of the accepted tokens' rows, and attention over a cache grown by commits equals
ordinary causal attention over the whole sequence."""
import numpy as np
import torch

from oracle import tree_attention
from oracle.kv_commit import kv_commit


def _setup(rs, B, Hkv, D, cap, sizes, lens):
    NN = sum(sizes)
    kt = rs.randn(NN, Hkv, D).astype(np.float32)
    vt = rs.randn(NN, Hkv, D).astype(np.float32)
    kc = rs.randn(B * cap, Hkv, D).astype(np.float32)
    vc = rs.randn(B * cap, Hkv, D).astype(np.float32)
    no = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    co = (np.arange(B + 1) * cap).astype(np.int64)
    return kt, vt, kc, vc, no, co, np.asarray(lens, np.int64)


def test_commit_is_concatenation_of_root_and_accepted_rows():
    rs = np.random.RandomState(0)
    sizes, lens = [7, 0, 12, 3], [5, 2, 0, 9]
    kt, vt, kc, vc, no, co, ln = _setup(rs, 4, 2, 8, 16, sizes, lens)
    path = np.full((4, 5), -1, np.int32)
    path[0, :3] = [2, 4, 6]
    path[2, :5] = [1, 3, 7, 8, 11]
    alen = np.asarray([3, 0, 5, 0], np.int32)
    k2, v2, l2 = kv_commit(kt, vt, no, path, alen, kc, vc, co, ln)
    assert list(l2) == [5 + 4, 2, 0 + 6, 9 + 1]
    for s, rows in enumerate(([0, 2, 4, 6], [], [0, 1, 3, 7, 8, 11], [0])):
        a = int(co[s])
        want_k = np.concatenate([kc[a:a + lens[s]], kt[no[s] + np.asarray(rows, int)]]) if rows else kc[a:a + lens[s]]
        assert np.array_equal(k2[a:a + l2[s]], want_k)
        want_v = np.concatenate([vc[a:a + lens[s]], vt[no[s] + np.asarray(rows, int)]]) if rows else vc[a:a + lens[s]]
        assert np.array_equal(v2[a:a + l2[s]], want_v)
        assert np.array_equal(k2[a + l2[s]:a + 16], kc[a + l2[s]:a + 16])      # the spare capacity is untouched
    assert np.array_equal(kc, _setup(np.random.RandomState(0), 4, 2, 8, 16, sizes, lens)[2])   # input not modified


def test_capacity_takes_the_leading_rows():
    rs = np.random.RandomState(1)
    kt, vt, kc, vc, no, co, ln = _setup(rs, 1, 1, 4, 6, [5], [4])
    path = np.asarray([[1, 2, 4]], np.int32)
    k2, v2, l2 = kv_commit(kt, vt, no, path, [3], kc, vc, co, ln)
    assert int(l2[0]) == 6 and np.array_equal(k2[4:6], kt[[0, 1]])


def test_decoding_through_commits_is_causal_attention():
    """A chain of tokens verified in several steps with different accepted lengths: the cache that
    the commits build makes the last step's attention equal to dense causal attention over the
    whole token sequence (computed with a library routine)."""
    rs = np.random.RandomState(2)
    Hq = Hkv = 2
    D, T = 8, 23
    K = rs.randn(T, Hkv, D).astype(np.float32)            # K/V of the true token sequence
    V = rs.randn(T, Hkv, D).astype(np.float32)
    Q = rs.randn(T, Hq, D).astype(np.float32)
    cap = 40
    kc, vc = np.zeros((cap, Hkv, D), np.float32), np.zeros((cap, Hkv, D), np.float32)
    lens = np.asarray([0], np.int64)
    pos = 0                                               # the root of the next step is token `pos`
    for accepted, drafted in ((2, 4), (0, 3), (4, 4), (1, 5)):
        m = drafted + 1                                   # chain tree: root + drafted tokens
        kt = rs.randn(m, Hkv, D).astype(np.float32)       # rejected drafts carry unrelated K/V
        vt = rs.randn(m, Hkv, D).astype(np.float32)
        kt[:accepted + 1], vt[:accepted + 1] = K[pos:pos + accepted + 1], V[pos:pos + accepted + 1]
        path = np.full((1, drafted), -1, np.int32)
        path[0, :accepted] = np.arange(1, accepted + 1)
        kc, vc, lens = kv_commit(kt, vt, [0, m], path, [accepted], kc, vc, [0, cap], lens)
        pos += accepted + 1
    assert int(lens[0]) == pos == 11
    # the next step: a chain of the remaining tokens over the committed cache
    m = T - pos
    o, _ = tree_attention(Q[pos:], kc[:pos], vc[:pos], K[pos:], V[pos:], np.arange(-1, m - 1), [0, m], [0, pos], 0.3)
    q, k, v = (torch.from_numpy(x).double().permute(1, 0, 2) for x in (Q, K, V))
    ref = torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=True, scale=0.3).permute(1, 0, 2).numpy()
    assert np.allclose(o, ref[pos:], atol=1e-12)


def test_paged_cache_is_the_dense_cache_in_other_places():
    """Scattering a dense cache into pages under a random block table and gathering it back is the
    identity, and a paged commit followed by the gather equals the dense commit."""
    from oracle.kv_commit import gather_pages, kv_commit_paged
    rs = np.random.RandomState(3)
    B, pt, max_blocks, Hkv, D = 3, 4, 5, 2, 8
    lens = np.asarray([7, 0, 13], np.int64)
    table = rs.permutation(B * max_blocks + 3)[:B * max_blocks].reshape(B, max_blocks)
    dense_k = rs.randn(int(lens.sum()), Hkv, D).astype(np.float32)
    dense_v = rs.randn(int(lens.sum()), Hkv, D).astype(np.float32)
    pages_k = rs.randn(B * max_blocks + 3, pt, Hkv, D).astype(np.float32)
    pages_v = rs.randn(B * max_blocks + 3, pt, Hkv, D).astype(np.float32)
    row = 0
    for s in range(B):
        for t in range(int(lens[s])):
            pages_k[table[s, t // pt], t % pt] = dense_k[row]
            pages_v[table[s, t // pt], t % pt] = dense_v[row]
            row += 1
    gk, offs = gather_pages(pages_k, table, lens)
    assert np.array_equal(gk, dense_k) and list(offs) == [0, 7, 7, 20]
    sizes = [5, 2, 6]
    no = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    kt = rs.randn(int(no[-1]), Hkv, D).astype(np.float32)
    vt = rs.randn(int(no[-1]), Hkv, D).astype(np.float32)
    path = np.asarray([[1, 3, 4], [-1, -1, -1], [2, 5, -1]], np.int32)
    alen = np.asarray([3, 0, 2], np.int32)
    pk, pv, pl = kv_commit_paged(kt, vt, no, path, alen, pages_k, pages_v, table, lens)
    # the dense commit on regions with spare capacity, for comparison
    cap = max_blocks * pt
    ck = np.zeros((B * cap, Hkv, D), np.float32)
    cv = np.zeros((B * cap, Hkv, D), np.float32)
    for s in range(B):
        ck[s * cap:s * cap + lens[s]] = dense_k[offs[s]:offs[s + 1]]
        cv[s * cap:s * cap + lens[s]] = dense_v[offs[s]:offs[s + 1]]
    dk, dv, dl = kv_commit(kt, vt, no, path, alen, ck, cv, np.arange(B + 1) * cap, lens)
    assert np.array_equal(pl, dl)
    gk2, o2 = gather_pages(pk, table, pl)
    gv2, _ = gather_pages(pv, table, pl)
    for s in range(B):
        assert np.array_equal(gk2[o2[s]:o2[s + 1]], dk[s * cap:s * cap + dl[s]])
        assert np.array_equal(gv2[o2[s]:o2[s + 1]], dv[s * cap:s * cap + dl[s]])
