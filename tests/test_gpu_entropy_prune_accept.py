"""GPU parity of hs_draft_entropy_topk, hs_tree_prune and hs_verify_accept against the CPU checker:
bit-exact indices / kept sets / paths, entropies within 1e-5 relative."""
import math

import numpy as np
import pytest

from synth import workloads as W
from oracle import draft_entropy_topk, tree_prune, verify_accept, pipeline as P

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def G():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import gpu_util
    return gpu_util


def _check_entropy(G, rows, K, T=1.0, logp_tol=2e-5):
    want = draft_entropy_topk(rows, K, T)
    got = G.run_entropy(rows, K, T)
    assert np.array_equal(got["topk_idx"], want["topk_idx"])
    fin = np.isfinite(want["topk_logp"])
    worst = float(np.max(np.abs(got["topk_logp"][fin] - want["topk_logp"][fin]) / np.maximum(1, np.abs(want["topk_logp"][fin]))))
    assert worst <= logp_tol, worst
    assert np.array_equal(np.isfinite(got["topk_logp"]), fin)
    assert G.entropy_err(got["ent_topk"], want["ent_topk"]) <= 1.0
    assert G.entropy_err(got["ent_full"], want["ent_full"]) <= 1.0
    worst = float(np.max(np.abs(got["lse"] - want["lse"]) / np.maximum(1, np.abs(want["lse"]))))
    assert worst <= 2e-6, worst
    return got, want


def test_entropy_workload1_rows(G):
    w = W.WORKLOADS[1]
    rows = W.logits_rows(w, 0, "draft", 0, range(17))
    _check_entropy(G, rows, 10)
    _check_entropy(G, rows, 10, T=0.7)


@pytest.mark.parametrize("R,V,K", [(1, 5, 5), (3, 64, 1), (2, 1000, 64), (5, 4097, 7), (1, 131, 3), (7, 20000, 10),
                                   (300, 777, 4), (2, 262147, 10), (1200, 20000, 10), (700, 40000, 1)])
def test_entropy_shapes_spanning_tiles_and_tails(G, R, V, K):
    rs = np.random.RandomState(R * 1000 + V)
    rows = (rs.randn(R, V) * rs.uniform(0.3, 10, size=(R, 1))).astype(np.float32)
    _check_entropy(G, rows, K)


def test_entropy_edge_rows(G):
    V, K = 9000, 10
    rs = np.random.RandomState(1)
    rows = np.zeros((8, V), np.float32)
    rows[0] = 2.5                                            # all equal: indices 0..K-1, ln V, ln K
    rows[1, 4321] = 60.0                                     # one-hot
    rows[2] = np.sort(rs.randn(V)).astype(np.float32)        # ascending: every tile raises the threshold
    rows[3] = -np.sort(rs.randn(V)).astype(np.float32)       # descending
    rows[4] = -np.inf
    rows[4, [5, 77, 8000]] = [0.0, 1.0, -1.0]                # masked vocabulary, fewer live tokens than K
    rows[5] = np.round(rs.randn(V) * 2).astype(np.float32)   # heavy ties
    rows[6] = rs.randn(V).astype(np.float32) * 30            # nearly one-hot
    rows[7] = rs.randn(V).astype(np.float32) * 1e-3          # nearly uniform
    got, want = _check_entropy(G, rows, K)
    assert list(got["topk_idx"][0]) == list(range(K))
    assert abs(got["ent_full"][0] - math.log(V)) < 1e-4 and abs(got["ent_topk"][0] - math.log(K)) < 1e-5
    assert got["ent_full"][1] < 1e-8 and got["ent_topk"][1] < 1e-8


@pytest.mark.parametrize("R,K", [(3, 1), (3, 10), (40, 1), (40, 10)])
def test_entropy_ties_across_tiles_and_slices(G, R, K):
    """Rows of equal or heavily tied logits over the full vocabulary: the lowest indices must win in
    every workgroup size and slicing, and nearly every element ties with the threshold."""
    V = 128256
    rs = np.random.RandomState(R + K)
    rows = np.round(rs.randn(R, V)).astype(np.float32)       # a handful of distinct values
    rows[0] = 0.0                                            # all equal
    rows[1] = -np.inf
    rows[1, 100000:] = 1.5                                   # equal, and only late in the row
    _check_entropy(G, rows, K)


def test_entropy_row_stride_and_unaligned_rows(G):
    import torch
    import paper_2505_13254_amd as hs
    rs = np.random.RandomState(2)
    big = rs.randn(6, 5003).astype(np.float32) * 3
    t = G.dev(big)
    view = t[:, 1:4998]                                      # stride 5003, V = 4997, misaligned start
    out = hs.hs_draft_entropy_topk(view, 8)
    want = draft_entropy_topk(big[:, 1:4998], 8)
    assert np.array_equal(G.host(out["topk_idx"]), want["topk_idx"])
    assert G.entropy_err(G.host(out["ent_full"]), want["ent_full"]) <= 1.0


def test_entropy_is_deterministic(G):
    rs = np.random.RandomState(3)
    rows = (rs.randn(40, 30011) * 4).astype(np.float32)
    a, b = G.run_entropy(rows, 10), G.run_entropy(rows, 10)
    for k in a:
        assert np.array_equal(a[k], b[k])


# ------------------------------------------------------------------------------------------ prune
@pytest.mark.parametrize("R,V,K", [(1, 128256, 10), (10, 128256, 10), (51, 128256, 10), (61, 32000, 1), (7, 5000, 64),
                                   (40, 100003, 13), (300, 4099, 5)])
def test_entropy_in_one_launch_on_a_prepared_workspace(G, R, V, K):
    """hs_draft_entropy_topk_fused: the rows' last slices merge (one counter per row in a prepared
    workspace, left at zero): against the checker, bit-identical to the two-launch call, on calls in a row
    on one workspace (larger shape first, then smaller ones, then with a row index list)."""
    import paper_2505_13254_amd as hs
    rs = np.random.RandomState(R + V + K)
    tau = np.exp(rs.uniform(np.log(0.3), np.log(8.0), size=(R, 1)))
    x = (rs.normal(size=(R, V)) * tau).astype(np.float32)
    x[0, : min(V, 3 * K)] = x[0, 0]                                   # ties across slices
    xd = G.dev(x)
    sizes = sorted({1, max(1, R // 3), R})
    # (fewer rows are cut into more slices each: the workspace is sized for the largest need)
    ws = hs.workspace(max(hs.lib().hs_draft_entropy_topk_workspace(r, V, K) for r in sizes + [4]), G.DEV)
    ws.fill_(0x5A)                                                    # unknown content first ...
    hs.hs_workspace_prepare(ws)                                       # ... then prepared, once
    want = draft_entropy_topk(x, K, 1.0)
    plain = {k: G.host(v) for k, v in hs.hs_draft_entropy_topk(xd, K, 1.0).items()}
    for rep in range(3):
        got = {k: G.host(v) for k, v in hs.hs_draft_entropy_topk(xd, K, 1.0, ws=ws, fused=True).items()}
        assert np.array_equal(got["topk_idx"], want["topk_idx"])
        for k in ("ent_topk", "ent_full"):
            assert G.entropy_err(got[k], want[k]) <= 1.0, k
        for k in plain:
            assert got[k].tobytes() == plain[k].tobytes(), k          # same merge arithmetic: same bits
    # fewer rows on the same workspace (other slice counts, other counters), then rows by index
    for R2 in sizes:
        got = {k: G.host(v) for k, v in hs.hs_draft_entropy_topk(xd[:R2], K, 1.0, ws=ws, fused=True).items()}
        ref = {k: G.host(v) for k, v in hs.hs_draft_entropy_topk(xd[:R2], K, 1.0).items()}
        for k in ref:
            assert got[k].tobytes() == ref[k].tobytes(), (R2, k)
    idx = np.asarray([R - 1, 0, -1, R // 2][: max(1, min(4, R))], np.int32)
    out = {k: torch.full_like(v[: len(idx)], -3) for k, v in hs.hs_draft_entropy_topk(xd, K, 1.0).items()}
    ref = {k: v.clone() for k, v in out.items()}
    hs.hs_draft_entropy_topk(xd, K, 1.0, out=out, ws=ws, row_index=G.dev(idx, torch.int32), fused=True)
    hs.hs_draft_entropy_topk(xd, K, 1.0, out=ref, row_index=G.dev(idx, torch.int32))
    for k in ref:
        assert G.host(out[k]).tobytes() == G.host(ref[k]).tobytes(), k


def _prune_equal(got, want):
    for k in ("depth", "keep", "out_offsets", "out_src", "out_parent"):
        assert np.array_equal(got[k], want[k]), k
    assert np.array_equal(got["cumlogp"].view(np.uint32), want["cumlogp"].view(np.uint32))   # bit for bit
    assert got["tail_is_padded"], "out_src / out_parent past the surviving rows must be zero"


def test_prune_workload1_and_sweeps(G):
    st = P.build_step(W.WORKLOADS[1], 0, with_attention=False)
    _prune_equal(G.run_prune(st["prune_in"]), st["prune_out"])
    w3 = W.small(W.WORKLOADS[3], V=4096)
    for th in w3.theta:
        st = P.build_step(w3, 0, theta=th, with_attention=False)
        _prune_equal(G.run_prune(st["prune_in"]), st["prune_out"])


@pytest.mark.parametrize("seed", range(6))
def test_prune_random_ragged_batches(G, seed):
    rs = np.random.RandomState(seed)
    sizes = [int(x) for x in rs.choice([0, 1, 2, 17, 64, 257, 511, 1000], size=rs.randint(1, 9))]
    if sum(sizes) == 0:
        sizes.append(5)
    parents, logcs = [], []
    for n in sizes:
        if n:
            parents.append(np.asarray([-1] + [rs.randint(max(0, i - 12), i) for i in range(1, n)], np.int32))
            c = -rs.exponential(0.7, size=n)
            c[rs.rand(n) < 0.1] = 1e-7                      # slightly positive: clamped
            c = np.round(c * 4) / 4 if seed % 2 else c      # many equal sums on odd seeds
            c[0] = 0
            logcs.append(c)
    B = len(sizes)
    pin = dict(parent=np.concatenate(parents), logc=np.concatenate(logcs).astype(np.float32),
               node_offsets=np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32),
               d_max=rs.choice([2, 5, 9, 2 ** 31 - 1], size=B).astype(np.int32),
               theta=rs.choice([-np.inf, -8.0, -3.0, -0.5], size=B).astype(np.float32),
               max_nodes=rs.choice([0, 1, 7, 60, 128], size=B).astype(np.int32))
    want = tree_prune(pin["parent"], pin["logc"], pin["node_offsets"], pin["d_max"], pin["theta"], pin["max_nodes"])
    _prune_equal(G.run_prune(pin), want)


def test_prune_tree_larger_than_lds(G):
    rs = np.random.RandomState(11)
    n = 6000
    parent = np.asarray([-1] + [rs.randint(max(0, i - 40), i) for i in range(1, n)], np.int32)
    logc = (-rs.exponential(0.05, size=n)).astype(np.float32)
    pin = dict(parent=parent, logc=logc, node_offsets=np.asarray([0, n], np.int32),
               d_max=np.asarray([2 ** 31 - 1], np.int32), theta=np.asarray([-6.0], np.float32),
               max_nodes=np.asarray([900], np.int32))
    want = tree_prune(parent, logc, pin["node_offsets"], pin["d_max"], pin["theta"], pin["max_nodes"])
    _prune_equal(G.run_prune(pin), want)


# ------------------------------------------------------------------------------------------ accept
def _accept_equal(got, want):
    for k in ("accept_len", "accept_path", "bonus_token"):
        assert np.array_equal(got[k], want[k]), (k, got[k], want[k])


def _planted(step, rs):
    """Make the target confirm a random root-to-leaf path of every sequence (known answer)."""
    no = step["node_offsets"]
    for s in range(len(no) - 1):
        o, n = int(no[s]), int(no[s + 1] - no[s])
        if n < 2:
            continue
        c = o + int(rs.randint(1, n))
        while step["parent"][c] >= 0:
            p = o + int(step["parent"][c])
            step["target_logits"][p, step["token"][c]] = step["target_logits"][p].max() + 2.0
            c = p


@pytest.mark.parametrize("wid,small", [(1, {}), (3, dict(V=4096)), (2, dict(V=8192)), (5, dict(V=2048, B=6))])
def test_accept_greedy(G, wid, small):
    w = W.small(W.WORKLOADS[wid], **small)
    rs = np.random.RandomState(wid)
    for planted in (False, True):
        st = P.build_step(w, 0, theta=w.theta[-1], with_attention=False)   # the loosest threshold
        if planted:
            _planted(st, rs)
        D = max(1, int(P.tree_depth(st["parent"], st["node_offsets"]).max()))
        want = P.accept_out(st, P.GREEDY, None, D)
        _accept_equal(G.run_accept(st, 0, None, D), want)
        if planted:
            assert want["accept_len"].max() >= 1
    # a walk cut short by max_depth
    want = P.accept_out(st, P.GREEDY, None, 1)
    _accept_equal(G.run_accept(st, 0, None, 1), want)


@pytest.mark.parametrize("mode", [1, 2])
@pytest.mark.parametrize("wid,small", [(1, {}), (2, dict(V=8192)), (2, dict(V=12292)), (4, dict(V=4099)),
                                       (5, dict(V=2048, B=5)), (5, dict(V=20480, B=3))])
def test_accept_stochastic(G, mode, wid, small):
    w = W.small(W.WORKLOADS[wid], **small)
    lens = []
    for seed in range(3):
        st = P.build_step(w, seed, with_attention=False)
        u, want = P.safe_uniforms(st, mode)
        D = max(1, int(P.tree_depth(st["parent"], st["node_offsets"]).max()))
        _accept_equal(G.run_accept(st, mode, u, D), want)
        lens += list(want["accept_len"])
    if wid != 1:                                             # (the tiny workload keeps 3 unlikely nodes)
        assert max(lens) >= 1                                # some walk went below the root


@pytest.mark.parametrize("V,pad", [(12290, 2), (8193, 3), (8190, 1)])
def test_accept_stochastic_padded_rows(G, V, pad):
    """Rows with a stride above V: 16-byte aligned rows whose length is no multiple of four (the
    rejection chains' lists of live tokens take the last V % 4 tokens separately) and unaligned rows."""
    import paper_2505_13254_amd as hs
    w = W.small(W.WORKLOADS[2], V=V)
    for seed in range(2):
        st = P.build_step(w, seed, with_attention=False)
        u, want = P.safe_uniforms(st, 1)
        D = max(1, int(P.tree_depth(st["parent"], st["node_offsets"]).max()))
        NN = st["target_logits"].shape[0]
        bufs = []
        for name in ("target_logits", "draft_logits"):
            b = torch.full((NN, V + pad), float("nan"), dtype=torch.float32, device="cuda:0")
            b[:, :V] = torch.from_numpy(st[name]).to("cuda:0")
            bufs.append(b[:, :V])
        out = hs.hs_verify_accept(bufs[0], bufs[1], G.dev(st["token"], torch.int32), G.dev(st["parent"], torch.int32),
                                  G.dev(st["node_offsets"], torch.int32), 1, w.temperature,
                                  G.dev(u, torch.float32), D)
        _accept_equal({k: G.host(v) for k, v in out.items()}, want)


def test_accept_stochastic_is_deterministic(G):
    w = W.small(W.WORKLOADS[2], V=16384)
    st = P.build_step(w, 3, with_attention=False)
    u, want = P.safe_uniforms(st, 1)
    D = max(1, int(P.tree_depth(st["parent"], st["node_offsets"]).max()))
    first = G.run_accept(st, 1, u, D)
    _accept_equal(first, want)
    for _ in range(3):
        _accept_equal(G.run_accept(st, 1, u, D), first)


@pytest.mark.parametrize("V,n_kids,T", [(16384, 14, 1.0), (40000, 9, 1.0), (6000, 24, 1.0), (12288, 12, 0.7),
                                        (9000, 10, 1.6)])
def test_accept_long_rejection_chains(G, V, n_kids, T):
    """A root whose many children are (nearly) all rejected, so that the bonus token depends on every
    pass of the root's chain: the list of live tokens is built, compacted in memory, and ends in LDS."""
    import paper_2505_13254_amd as hs
    rs = np.random.RandomState(V + n_kids)
    done, rejected_all = 0, 0
    for attempt in range(40):
        draft = (rs.normal(size=(1 + n_kids, V)) * 2.5).astype(np.float32)
        target = (0.8 * draft + rs.normal(size=draft.shape) * 1.5).astype(np.float32)
        parent = np.asarray([-1] + [0] * n_kids, np.int32)
        token = np.zeros(1 + n_kids, np.int32)
        token[1:] = np.argsort(-draft[0], kind="stable")[:n_kids]          # the draft's best tokens, distinct
        offs = np.asarray([0, 1 + n_kids], np.int32)
        u = np.concatenate([0.9 + 0.0999 * rs.rand(1 + n_kids), rs.rand(1)]).astype(np.float32)
        from oracle import verify_accept
        base = verify_accept(target, draft, token, parent, offs, 1, T, u, 1)
        ok = True
        for sgn in (-1.0, 1.0):
            un = u.astype(np.float64).copy()
            un[:1 + n_kids] *= 1.0 + sgn * 1e-4
            un[1 + n_kids:] = np.clip(un[1 + n_kids:] + sgn * 1e-5, 0.0, 1.0 - 1e-12)
            alt = verify_accept(target, draft, token, parent, offs, 1, T, un, 1)
            ok = ok and all(np.array_equal(alt[k], base[k]) for k in base)
        if not ok:
            continue
        out = hs.hs_verify_accept(G.dev(target), G.dev(draft), G.dev(token, torch.int32), G.dev(parent, torch.int32),
                                  G.dev(offs, torch.int32), 1, T, G.dev(u, torch.float32), 1)
        _accept_equal({k: G.host(v) for k, v in out.items()}, base)
        done += 1
        rejected_all += int(base["accept_len"][0] == 0)
        if done >= 6 and rejected_all >= 2:
            break
    assert done >= 6 and rejected_all >= 2, (done, rejected_all)


@pytest.mark.parametrize("mode", [1, 2])
def test_accept_more_children_than_the_lists_hold(G, mode):
    """A root with 300 children: the sampling rules try the 256 lowest rows (the documented limit), the
    same ones on every run.  With an accepting draw placed on child 200 the walk is the checker's;
    with every draw rejecting, the result is that of the tree cut to its first 256 children."""
    import paper_2505_13254_amd as hs
    from oracle import verify_accept
    rs = np.random.RandomState(5 + mode)
    V, n_kids = 4096, 300
    draft = (rs.normal(size=(1 + n_kids, V)) * 1.5).astype(np.float32)
    target = (0.8 * draft + rs.normal(size=draft.shape)).astype(np.float32)
    parent = np.asarray([-1] + [0] * n_kids, np.int32)
    token = np.zeros(1 + n_kids, np.int32)
    token[1:] = np.argsort(-draft[0], kind="stable")[:n_kids]
    offs = np.asarray([0, 1 + n_kids], np.int32)

    def gpu(u, par=parent, tok=token, off=offs, tl=target, dl=draft):
        out = hs.hs_verify_accept(G.dev(tl), G.dev(dl), G.dev(tok, torch.int32), G.dev(par, torch.int32),
                                  G.dev(off, torch.int32), mode, 1.0, G.dev(u, torch.float32), 1)
        return {k: G.host(v) for k, v in out.items()}
    # (a) child 200 accepts for sure (u = 0; the target favours its token far more than the draft does, so
    # that its residual probability survives the rejections before it), the others reject (u close to 1)
    target[0, token[200]] += 12.0
    u = np.concatenate([np.full(1 + n_kids, 0.9999), [0.37]]).astype(np.float32)
    u[200] = 0.0
    want = verify_accept(target, draft, token, parent, offs, mode, 1.0, u, 1)
    assert want["accept_len"][0] == 1 and want["accept_path"][0, 0] == 200
    _accept_equal(gpu(u), want)
    target[0, token[200]] -= 12.0
    # (b) nothing accepts: the first 256 children are tried, twice with the same bits
    u = np.concatenate([np.full(1 + n_kids, 0.99999), [0.61]]).astype(np.float32)
    cut = 257
    uc = np.concatenate([u[:cut], u[-1:]])
    want = verify_accept(target[:cut], draft[:cut], token[:cut], parent[:cut], np.asarray([0, cut], np.int32), mode, 1.0, uc, 1)
    if want["accept_len"][0] == 0:        # (with 256 rejections in a row nearly all mass is gone; any outcome must agree)
        first, second = gpu(u), gpu(u)
        _accept_equal(first, want)
        _accept_equal(second, first)


def test_accept_draft_rows_of_leaves_are_not_read(G):
    """Only rows that have children carry a draft distribution: the others may hold anything."""
    w = W.small(W.WORKLOADS[2], V=8192)
    st = P.build_step(w, 1, with_attention=False)
    u, want = P.safe_uniforms(st, 1)
    D = max(1, int(P.tree_depth(st["parent"], st["node_offsets"]).max()))
    has_child = np.zeros(len(st["parent"]), bool)
    no = st["node_offsets"]
    for s in range(len(no) - 1):
        o, n = int(no[s]), int(no[s + 1] - no[s])
        for i in range(1, n):
            has_child[o + int(st["parent"][o + i])] = True
    assert has_child.any() and not has_child.all()
    st2 = dict(st)
    st2["draft_logits"] = st["draft_logits"].copy()
    st2["draft_logits"][~has_child] = np.nan
    _accept_equal(G.run_accept(st2, 1, u, D), want)


def test_entropy_rows_picked_by_index(G):
    """hs_draft_entropy_topk_rows: result rows come from the rows an index list names (repeats
    allowed); a negative entry leaves its result row untouched."""
    import paper_2505_13254_amd as hs
    rs = np.random.RandomState(77)
    N, V, K = 40, 6000, 10
    x = (rs.normal(size=(N, V)) * 3).astype(np.float32)
    pick = np.asarray([7, 0, 39, 7, -1, 12, 39, 3, -5, 21, 1], np.int32)
    R = len(pick)
    out = dict(topk_idx=torch.full((R, K), -7, dtype=torch.int32, device="cuda:0"),
               topk_logp=torch.full((R, K), 5.0, dtype=torch.float32, device="cuda:0"),
               ent_topk=torch.full((R,), 5.0, dtype=torch.float32, device="cuda:0"),
               ent_full=torch.full((R,), 5.0, dtype=torch.float32, device="cuda:0"),
               lse=torch.full((R,), 5.0, dtype=torch.float32, device="cuda:0"))
    hs.hs_draft_entropy_topk(G.dev(x), K, 0.8, out=out, row_index=G.dev(pick))
    got = {k: G.host(v) for k, v in out.items()}
    live = pick >= 0
    want = draft_entropy_topk(x[pick[live]], K, 0.8)
    assert np.array_equal(got["topk_idx"][live], want["topk_idx"])
    assert G.entropy_err(got["ent_topk"][live], want["ent_topk"]) <= 1.0
    assert G.entropy_err(got["ent_full"][live], want["ent_full"]) <= 1.0
    assert np.all(np.abs(got["topk_logp"][live] - want["topk_logp"]) <= 2e-5 * np.abs(want["topk_logp"]) + 1e-6)
    assert np.all(got["topk_idx"][~live] == -7) and np.all(got["ent_topk"][~live] == 5.0)   # untouched
    # one picked row by itself (few rows: the short-slice plan)
    one = hs.hs_draft_entropy_topk(G.dev(x), K, 0.8, row_index=G.dev(np.asarray([33], np.int32)))
    assert np.array_equal(G.host(one["topk_idx"]), draft_entropy_topk(x[33:34], K, 0.8)["topk_idx"])


def _random_accept_case(rs, sizes, V, mode, T, D):
    """Random trees (a row's parent is one of the five rows before it, siblings carry the draft's best
    tokens), correlated draft and target rows, uniforms with a margin to every decision.  Returns the
    arrays and the checker's result, or None when a decision is too close to call."""
    B, NN = len(sizes), sum(sizes)
    draft = (rs.normal(size=(NN, V)) * 2.5).astype(np.float32)
    corr = rs.choice([0.5, 0.8, 0.95])
    target = (corr * draft + rs.normal(size=draft.shape) * (1.5 * (1 - corr) + 0.3)).astype(np.float32)
    parent, token, offs, o = np.zeros(NN, np.int32), np.zeros(NN, np.int32), [0], 0
    for n in sizes:
        parent[o] = -1
        kids = {}
        for i in range(1, n):
            p = int(rs.randint(max(0, i - 5), i))
            parent[o + i] = p
            kids.setdefault(p, []).append(i)
        for p, ks in kids.items():       # siblings carry the draft's best tokens, distinct
            for c, tk in zip(ks, np.argsort(-draft[o + p], kind="stable")[:len(ks)]):
                token[o + c] = tk
        o += n
        offs.append(o)
    offs = np.asarray(offs, np.int32)
    u = np.concatenate([0.3 + 0.6999 * rs.rand(NN), rs.rand(B)]).astype(np.float32)
    base = verify_accept(target, draft, token, parent, offs, mode, T, u, D)
    for sgn in (-1.0, 1.0):
        un = u.astype(np.float64).copy()
        un[:NN] *= 1.0 + sgn * 1e-4
        un[NN:] = np.clip(un[NN:] + sgn * 1e-5, 0.0, 1.0 - 1e-12)
        alt = verify_accept(target, draft, token, parent, offs, mode, T, un, D)
        if not all(np.array_equal(alt[k], base[k]) for k in base):
            return None
    return target, draft, token, parent, offs, u, base


@pytest.mark.parametrize("seed", [1, 2])
def test_accept_random_trees(G, seed):
    """Forty random cases per seed: both sampling rules, 1 to 3 sequences of up to 25 rows, vocabularies
    on both sides of the sorted residual's conditions (size, alignment), three temperatures, walks cut
    by max_depth; uniforms with a margin to every decision."""
    import paper_2505_13254_amd as hs
    rs = np.random.RandomState(seed)
    done, lens = 0, []
    for attempt in range(200):
        mode = int(rs.choice([1, 1, 2]))
        V = int(rs.choice([4096, 4100, 5000, 8192, 12290, 20000]))
        B = int(rs.randint(1, 4))
        T = float(rs.choice([0.7, 1.0, 1.3]))
        sizes = [int(rs.randint(1, 26)) for _ in range(B)]
        D = int(rs.randint(1, 7))
        case = _random_accept_case(rs, sizes, V, mode, T, D)
        if case is None:
            continue
        target, draft, token, parent, offs, u, base = case
        out = hs.hs_verify_accept(G.dev(target), G.dev(draft) if mode == 1 else None, G.dev(token, torch.int32),
                                  G.dev(parent, torch.int32), G.dev(offs, torch.int32), mode, T,
                                  G.dev(u, torch.float32), D)
        _accept_equal({k: G.host(v) for k, v in out.items()}, base)
        lens += list(base["accept_len"])
        done += 1
        if done == 40:
            break
    assert done == 40 and max(lens) >= 2


def test_accept_ratio_rule_with_more_rows_than_the_tables_cover(G):
    """Beyond 4096 tree rows a call has neither the sorted residual nor the row sums prepared ahead of
    the walk: the chains take plain passes and the walk sums the rows of its stop node itself.  A batch
    of 4104 rows in 216 sequences; the sequences whose decisions are all clear of their uniforms are
    compared (a close call in one sequence does not touch the others)."""
    import paper_2505_13254_amd as hs
    rs = np.random.RandomState(11)
    sizes = [19] * 216
    V, T, D = 4096, 1.0, 4
    NN = sum(sizes)
    assert NN > 4096
    B = len(sizes)
    draft = (rs.normal(size=(NN, V)) * 2.5).astype(np.float32)
    target = (0.8 * draft + rs.normal(size=draft.shape) * 0.6).astype(np.float32)
    parent, token, offs, o = np.zeros(NN, np.int32), np.zeros(NN, np.int32), [0], 0
    for n in sizes:
        parent[o] = -1
        kids = {}
        for i in range(1, n):
            p = int(rs.randint(max(0, i - 5), i))
            parent[o + i] = p
            kids.setdefault(p, []).append(i)
        for p, ks in kids.items():
            for c, tk in zip(ks, np.argsort(-draft[o + p], kind="stable")[:len(ks)]):
                token[o + c] = tk
        o += n
        offs.append(o)
    offs = np.asarray(offs, np.int32)
    u = np.concatenate([0.3 + 0.6999 * rs.rand(NN), rs.rand(B)]).astype(np.float32)
    base = verify_accept(target, draft, token, parent, offs, 1, T, u, D)
    safe = np.ones(B, bool)
    for sgn in (-1.0, 1.0):
        un = u.astype(np.float64).copy()
        un[:NN] *= 1.0 + sgn * 1e-4
        un[NN:] = np.clip(un[NN:] + sgn * 1e-5, 0.0, 1.0 - 1e-12)
        alt = verify_accept(target, draft, token, parent, offs, 1, T, un, D)
        safe &= (alt["accept_len"] == base["accept_len"]) & (alt["bonus_token"] == base["bonus_token"])
        safe &= np.all(alt["accept_path"] == base["accept_path"], axis=1)
    assert safe.sum() > 150
    out = hs.hs_verify_accept(G.dev(target), G.dev(draft), G.dev(token, torch.int32), G.dev(parent, torch.int32),
                              G.dev(offs, torch.int32), 1, T, G.dev(u, torch.float32), D)
    got = {k: G.host(v) for k, v in out.items()}
    assert np.array_equal(got["accept_len"][safe], base["accept_len"][safe])
    assert np.array_equal(got["bonus_token"][safe], base["bonus_token"][safe])
    assert np.array_equal(got["accept_path"][safe], base["accept_path"][safe])
    assert base["accept_len"].max() >= 2
