"""GPU parity of hs_kv_commit (bit-exact) and of hs_tree_attention_lens on caches with spare
capacity, alone and in a decoding loop of several verify / commit steps."""
import numpy as np
import pytest

from oracle import tree_attention
from oracle.kv_commit import kv_commit
from synth import workloads as W

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def G():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import gpu_util
    return gpu_util


def _bits(t):
    torch.cuda.synchronize()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def _random_parents(rs, n, back=5):
    return [-1] + [int(rs.randint(max(0, i - back), i)) for i in range(1, n)]


def _random_path(rs, parent, max_depth):
    """A root path of random length (what an accept walk could return)."""
    n = len(parent)
    if n == 0:
        return [], 0
    children = {i: [j for j in range(n) if parent[j] == i] for i in range(n)}
    path, cur = [], 0
    while children[cur] and len(path) < max_depth and rs.uniform() < 0.75:
        cur = children[cur][int(rs.randint(len(children[cur])))]
        path.append(cur)
    return path, len(path)


@pytest.mark.parametrize("wid", [1, 2])
def test_commit_matches_the_checker(G, wid):
    import paper_2505_13254_amd as hs
    w = W.WORKLOADS[wid]
    rs = np.random.RandomState(wid)
    sizes = [9, 0, 33, 1, 17]
    caps = [20, 8, 40, 3, 10]
    lens = [4, 2, 0, 3, 7]                                # sequence 3 is full, sequence 4 overflows
    B, max_depth = len(sizes), 6
    parents = [_random_parents(rs, n) if n else [] for n in sizes]
    parts = [W.attention_inputs(w, 0, s, caps[s], sizes[s], "unit", parent=np.asarray(parents[s])) for s in range(B)]
    kc, vc, kt, vt = (np.concatenate([p[i] for p in parts], axis=0) for i in (1, 2, 3, 4))
    no = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    co = np.concatenate([[0], np.cumsum(caps)]).astype(np.int64)
    path = np.full((B, max_depth), -1, np.int32)
    alen = np.zeros(B, np.int32)
    for s in range(B):
        p, n = _random_path(rs, parents[s], max_depth)
        path[s, :n], alen[s] = p, n
    alen[4] = max(alen[4], 3)                             # make sure the overflow case overflows
    path[4, :3] = np.where(path[4, :3] < 0, 1, path[4, :3])
    want_k, want_v, want_l = kv_commit(kt, vt, no, path, alen, kc, vc, co, np.asarray(lens, np.int64))
    dk, dv, dl = G.dev_store(kc), G.dev_store(vc), G.dev(np.asarray(lens, np.int64))
    hs.hs_kv_commit(G.dev_store(kt), G.dev_store(vt), G.dev(no), G.dev(path), G.dev(alen), dk, dv, G.dev(co), dl)
    assert np.array_equal(_bits(dl), want_l)
    assert np.array_equal(_bits(dk), want_k) and np.array_equal(_bits(dv), want_v)
    assert int(want_l[4]) == caps[4] and int(want_l[3]) == 3


@pytest.mark.parametrize("wid,B", [(1, 3), (2, 4), (5, 100)])
def test_decoding_loop_on_caches_with_spare_capacity(G, wid, B):
    """Three verify / commit rounds: attention over the used part of each cache region, a random
    accepted path, commit; the checker follows with its own commit and attention."""
    import paper_2505_13254_amd as hs
    w = W.small(W.WORKLOADS[wid], B=B)
    rs = np.random.RandomState(10 + wid)
    tol = 1e-4 if w.dtype == "f32" else 2e-2
    max_depth = 5
    caps = [int(x) for x in rs.randint(40, 400 if B < 50 else 90, size=B)]
    lens = np.asarray([int(rs.randint(0, c - 30)) for c in caps], np.int64)
    if B == 4:
        caps[1], lens[1] = 3000, 2700                      # long enough to be cut into key splits
    co = np.concatenate([[0], np.cumsum(caps)]).astype(np.int64)
    fill = [W.attention_inputs(w, 1, s, caps[s], 1, "unit") for s in range(B)]
    kc, vc = (np.concatenate([p[i] for p in fill], axis=0) for i in (1, 2))
    dk, dv, dl, dco = G.dev_store(kc), G.dev_store(vc), G.dev(lens), G.dev(co)
    for step in range(3):
        sizes = [int(x) for x in rs.randint(0 if step else 1, 12, size=B)]
        parents = [_random_parents(rs, n) if n else [] for n in sizes]
        parts = [W.attention_inputs(w, 2 + step, s, 0, sizes[s], "unit", parent=np.asarray(parents[s])) for s in range(B)]
        q, kt, vt = (np.concatenate([p[i] for p in parts], axis=0) for i in (0, 3, 4))
        par = np.concatenate([np.asarray(p, np.int32) for p in parents]).astype(np.int32)
        no = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
        # the checker: packed prefix = the used part of every region
        used_k = np.concatenate([kc[co[s]:co[s] + lens[s]] for s in range(B)], axis=0)
        used_v = np.concatenate([vc[co[s]:co[s] + lens[s]] for s in range(B)], axis=0)
        po = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
        want_o, _ = tree_attention(q, used_k, used_v, kt, vt, par, no, po, 1.0 / np.sqrt(w.D))
        dkt, dvt = G.dev_store(kt), G.dev_store(vt)
        o, _ = hs.hs_tree_attention(G.dev_store(q), dk, dv, dkt, dvt, G.dev(par), G.dev(no), dco,
                                    torch.from_numpy(no), torch.from_numpy(co), 1.0 / float(np.sqrt(w.D)),
                                    prefix_lens=dl, host_prefix_lens=torch.from_numpy(lens.copy()))
        assert np.abs(G.host(o).astype(np.float64) - want_o).max() <= tol, step
        path = np.full((B, max_depth), -1, np.int32)
        alen = np.zeros(B, np.int32)
        for s in range(B):
            p, n = _random_path(rs, parents[s], max_depth)
            path[s, :n], alen[s] = p, n
        kc, vc, lens = kv_commit(kt, vt, no, path, alen, kc, vc, co, lens)
        hs.hs_kv_commit(dkt, dvt, G.dev(no), G.dev(path), G.dev(alen), dk, dv, dco, dl)
        assert np.array_equal(_bits(dl), lens) and np.array_equal(_bits(dk), kc) and np.array_equal(_bits(dv), vc)


def test_equal_lengths_in_regions_at_different_offsets(G):
    """Two cache layouts with the same tree sizes and the same used lengths, whose regions start at different
    offsets, called in turns: a call's plan (the library remembers its last few) holds each region's own
    offset, so every call must read its own keys."""
    import paper_2505_13254_amd as hs
    B = 3
    w = W.small(W.WORKLOADS[2], B=B)
    rs = np.random.RandomState(77)
    sizes, lens = [9, 20, 5], np.asarray([700, 130, 64], np.int64)
    parents = [_random_parents(rs, n) for n in sizes]
    par = np.concatenate([np.asarray(p, np.int32) for p in parents]).astype(np.int32)
    no = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    po = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    parts = [W.attention_inputs(w, 3, s, 0, sizes[s], "unit", parent=np.asarray(parents[s])) for s in range(B)]
    q, kt, vt = (np.concatenate([p[i] for p in parts], axis=0) for i in (0, 3, 4))
    dq, dkt, dvt, dpar, dno, dl = G.dev_store(q), G.dev_store(kt), G.dev_store(vt), G.dev(par), G.dev(no), G.dev(lens)
    layouts = []
    for k, caps in enumerate(([800, 200, 64], [1500, 130, 900])):
        co = np.concatenate([[0], np.cumsum(caps)]).astype(np.int64)
        fill = [W.attention_inputs(w, 10 + k, s, caps[s], 1, "unit") for s in range(B)]
        kc, vc = (np.concatenate([p[i] for p in fill], axis=0) for i in (1, 2))
        used_k = np.concatenate([kc[co[s]:co[s] + lens[s]] for s in range(B)], axis=0)
        used_v = np.concatenate([vc[co[s]:co[s] + lens[s]] for s in range(B)], axis=0)
        want, _ = tree_attention(q, used_k, used_v, kt, vt, par, no, po, 1.0 / np.sqrt(w.D))
        layouts.append((G.dev_store(kc), G.dev_store(vc), G.dev(co), co, want))
    assert np.abs(layouts[0][4] - layouts[1][4]).max() > 0.05     # (the two layouts hold different keys)
    for turn in range(4):
        dk, dv, dco, co, want = layouts[turn % 2]
        o, _ = hs.hs_tree_attention(dq, dk, dv, dkt, dvt, dpar, dno, dco, torch.from_numpy(no), torch.from_numpy(co),
                                    1.0 / float(np.sqrt(w.D)), prefix_lens=dl, host_prefix_lens=torch.from_numpy(lens.copy()))
        assert np.abs(G.host(o).astype(np.float64) - want).max() <= 2e-2, turn


def test_verify_commit_loop_over_layers(G):
    """Three decoding steps of a two-layer model slice, each: tree attention of every layer over its
    own cache, greedy accept walk on target logits, commit of the accepted path into every layer's
    cache with the path the accept kernel left on the device.  The checker runs the same loop."""
    import paper_2505_13254_amd as hs
    from oracle import verify_accept
    w = W.small(W.WORKLOADS[2], V=3000)
    rs = np.random.RandomState(77)
    layers, B, cap, max_depth = 2, 3, 200, 4
    scale = 1.0 / float(np.sqrt(w.D))
    co = (np.arange(B + 1) * cap).astype(np.int64)
    lens = np.asarray([60, 0, 131], np.int64)
    kc, vc = [], []
    for l in range(layers):
        fill = [W.attention_inputs(w, 40 + l, s, cap, 1, "unit") for s in range(B)]
        kc.append(np.concatenate([p[1] for p in fill], axis=0))
        vc.append(np.concatenate([p[2] for p in fill], axis=0))
    dk, dv = [G.dev_store(x) for x in kc], [G.dev_store(x) for x in vc]
    dl, dco = [G.dev(lens.copy()) for _ in range(layers)], G.dev(co)
    for step in range(3):
        sizes = [int(x) for x in rs.randint(2, 14, size=B)]
        parents = [_random_parents(rs, n, back=3) for n in sizes]
        par = np.concatenate([np.asarray(p, np.int32) for p in parents])
        no = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
        NN = int(no[-1])
        token = rs.randint(0, w.V, size=NN).astype(np.int32)
        for s in range(B):                                  # distinct tokens among siblings
            seen = set()
            for i in range(1, sizes[s]):
                while (parents[s][i], int(token[no[s] + i])) in seen:
                    token[no[s] + i] = rs.randint(0, w.V)
                seen.add((parents[s][i], int(token[no[s] + i])))
        tgt = rs.randn(NN, w.V).astype(np.float32)
        for s in range(B):                                  # plant a path of random length
            cur = 0
            for _ in range(int(rs.randint(0, max_depth + 1))):
                kids = [i for i in range(sizes[s]) if parents[s][i] == cur]
                if not kids:
                    break
                nxt = kids[int(rs.randint(len(kids)))]
                tgt[no[s] + cur, token[no[s] + nxt]] = 50.0
                cur = nxt
        want_acc = verify_accept(tgt, None, token, par, no, 0, 1.0, None, max_depth)
        acc = hs.hs_verify_accept(G.dev(tgt), None, G.dev(token), G.dev(par), G.dev(no), 0, 1.0, None, max_depth)
        for k in want_acc:
            assert np.array_equal(G.host(acc[k]), want_acc[k]), (step, k)
        po = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
        for l in range(layers):
            parts = [W.attention_inputs(w, 100 + 10 * step + l, s, 0, sizes[s], "unit", parent=np.asarray(parents[s]))
                     for s in range(B)]
            q, kt, vt = (np.concatenate([p[i] for p in parts], axis=0) for i in (0, 3, 4))
            used_k = np.concatenate([kc[l][co[s]:co[s] + lens[s]] for s in range(B)], axis=0)
            used_v = np.concatenate([vc[l][co[s]:co[s] + lens[s]] for s in range(B)], axis=0)
            want_o, _ = tree_attention(q, used_k, used_v, kt, vt, par, no, po, scale)
            dkt, dvt = G.dev_store(kt), G.dev_store(vt)
            o, _ = hs.hs_tree_attention(G.dev_store(q), dk[l], dv[l], dkt, dvt, G.dev(par), G.dev(no), dco,
                                        torch.from_numpy(no), torch.from_numpy(co), scale,
                                        prefix_lens=dl[l], host_prefix_lens=torch.from_numpy(lens.copy()))
            assert np.abs(G.host(o).astype(np.float64) - want_o).max() <= 2e-2, (step, l)
            # the path goes from the accept kernel to the commit kernel without leaving the device
            hs.hs_kv_commit(dkt, dvt, G.dev(no), acc["accept_path"], acc["accept_len"], dk[l], dv[l], dco, dl[l])
            kc[l], vc[l], new_lens = kv_commit(kt, vt, no, want_acc["accept_path"], want_acc["accept_len"], kc[l], vc[l],
                                               co, lens)
            assert np.array_equal(_bits(dl[l]), new_lens) and np.array_equal(_bits(dk[l]), kc[l])
            assert np.array_equal(_bits(dv[l]), vc[l])
        lens = new_lens
        assert np.array_equal(lens - (po[1:] - po[:-1]), want_acc["accept_len"] + 1)


def _paginate(rs, dense, offs, lens, max_blocks, n_spare=5, pt=64):
    """Scatters a packed dense cache into a page pool under a random block table."""
    B = len(lens)
    n_pages = B * max_blocks + n_spare
    table = rs.permutation(n_pages)[:B * max_blocks].reshape(B, max_blocks).astype(np.int32)
    pool = np.zeros((n_pages, pt) + dense.shape[1:], dense.dtype)
    if dense.dtype == np.uint16:
        pool[:] = 0x7fc0                                             # NaN in unused slots: must never be read
    else:
        pool[:] = np.nan
    for s in range(B):
        for t in range(int(lens[s])):
            pool[table[s, t // pt], t % pt] = dense[offs[s] + t]
    return pool, table


@pytest.mark.parametrize("wid,B", [(1, 3), (2, 4), (5, 100)])
def test_paged_attention_and_commit(G, wid, B):
    """Attention over paged caches equals the checker's attention over the gathered dense cache; the
    paged commit equals the checker's; two rounds."""
    import paper_2505_13254_amd as hs
    from oracle.kv_commit import gather_pages, kv_commit_paged
    w = W.small(W.WORKLOADS[wid], B=B)
    rs = np.random.RandomState(20 + wid)
    tol = 1e-4 if w.dtype == "f32" else 2e-2
    max_depth = 5
    lens = np.asarray([int(x) for x in rs.randint(0, 300 if B < 50 else 80, size=B)], np.int64)
    if B == 4:
        lens[1] = 2700                                               # long enough to be cut into key splits
    max_blocks = int((lens.max() + 2 * (max_depth + 1) + 63) // 64)
    offs = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    fill = [W.attention_inputs(w, 1, s, int(lens[s]), 1, "unit") for s in range(B)]
    dense_k, dense_v = (np.concatenate([p[i] for p in fill], axis=0) for i in (1, 2))
    state = np.random.RandomState(5)
    pool_k, table = _paginate(state, dense_k, offs, lens, max_blocks)
    pool_v, _ = _paginate(np.random.RandomState(5), dense_v, offs, lens, max_blocks)
    dk, dv, dt_, dl = G.dev_store(pool_k), G.dev_store(pool_v), G.dev(table), G.dev(lens)
    for step in range(2):
        sizes = [int(x) for x in rs.randint(0 if step else 1, 12, size=B)]
        parents = [_random_parents(rs, n) if n else [] for n in sizes]
        parts = [W.attention_inputs(w, 2 + step, s, 0, sizes[s], "unit", parent=np.asarray(parents[s])) for s in range(B)]
        q, kt, vt = (np.concatenate([p[i] for p in parts], axis=0) for i in (0, 3, 4))
        par = np.concatenate([np.asarray(p, np.int32) for p in parents]).astype(np.int32)
        no = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
        gk, po = gather_pages(pool_k, table, lens)
        gv, _ = gather_pages(pool_v, table, lens)
        want_o, _ = tree_attention(q, gk, gv, kt, vt, par, no, po, 1.0 / np.sqrt(w.D))
        dkt, dvt = G.dev_store(kt), G.dev_store(vt)
        o, _ = hs.hs_tree_attention_paged(G.dev_store(q), dk, dv, dkt, dvt, G.dev(par), G.dev(no), torch.from_numpy(no),
                                          dt_, dl, torch.from_numpy(lens.copy()), 1.0 / float(np.sqrt(w.D)))
        assert np.abs(G.host(o).astype(np.float64) - want_o).max() <= tol, step
        path = np.full((B, max_depth), -1, np.int32)
        alen = np.zeros(B, np.int32)
        for s in range(B):
            p, n = _random_path(rs, parents[s], max_depth)
            path[s, :n], alen[s] = p, n
        pool_k, pool_v, lens = kv_commit_paged(kt, vt, no, path, alen, pool_k, pool_v, table, lens)
        hs.hs_kv_commit_paged(dkt, dvt, G.dev(no), G.dev(path), G.dev(alen), dk, dv, dt_, dl)
        assert np.array_equal(_bits(dl), lens)
        raw = lambda x: x.view(np.uint32) if x.dtype == np.float32 else x       # (unused slots hold NaN)
        assert np.array_equal(raw(_bits(dk)), raw(pool_k)) and np.array_equal(raw(_bits(dv)), raw(pool_v))


@pytest.mark.parametrize("D,sizes", [(128, [100, 129, 7]), (64, [100, 129, 7]), (128, [100, 300, 7]), (64, [9, 700, 61])])
def test_paged_attention_with_several_row_groups(G, D, sizes):
    """Trees of more than 64 rows on the 8B shape (4 query heads per KV head: more than 256 rows per
    KV head, i.e. several row groups that read the same pages), next to small trees, over paged caches
    with a shuffled page order; one sequence long enough to be cut into key splits.  Also with head
    dimension 64 (KV heads taken in pairs by the matrix-core kernel) and with trees past 256 rows (ancestor
    table from its own launch)."""
    import paper_2505_13254_amd as hs
    from oracle.kv_commit import gather_pages
    w = W.small(W.WORKLOADS[2], B=3, D=D)
    rs = np.random.RandomState(77)
    B = 3
    lens = np.asarray([300, 2700, 65], np.int64)
    max_blocks = int((lens.max() + 63) // 64)
    offs = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    fill = [W.attention_inputs(w, 1, s, int(lens[s]), 1, "unit") for s in range(B)]
    dense_k, dense_v = (np.concatenate([p[i] for p in fill], axis=0) for i in (1, 2))
    pool_k, table = _paginate(np.random.RandomState(5), dense_k, offs, lens, max_blocks)
    pool_v, _ = _paginate(np.random.RandomState(5), dense_v, offs, lens, max_blocks)
    parents = [_random_parents(rs, n) for n in sizes]
    parts = [W.attention_inputs(w, 2, s, 0, sizes[s], "unit", parent=np.asarray(parents[s])) for s in range(B)]
    q, kt, vt = (np.concatenate([p[i] for p in parts], axis=0) for i in (0, 3, 4))
    par = np.concatenate([np.asarray(p, np.int32) for p in parents]).astype(np.int32)
    no = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    gk, po = gather_pages(pool_k, table, lens)
    gv, _ = gather_pages(pool_v, table, lens)
    want_o, _ = tree_attention(q, gk, gv, kt, vt, par, no, po, 1.0 / np.sqrt(w.D))
    o, _ = hs.hs_tree_attention_paged(G.dev_store(q), G.dev_store(pool_k), G.dev_store(pool_v), G.dev_store(kt),
                                      G.dev_store(vt), G.dev(par), G.dev(no), torch.from_numpy(no), G.dev(table),
                                      G.dev(lens), torch.from_numpy(lens.copy()), 1.0 / float(np.sqrt(w.D)))
    assert np.abs(G.host(o).astype(np.float64) - want_o).max() <= 2e-2
    assert hs.hs_tree_attention_last_kernel() == 1
