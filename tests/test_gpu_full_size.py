"""Parity at the workloads' full sizes, in the launch configuration bench.py times: the step is built
and run by the GPU harness, then every stage's device inputs are pulled back and checked against the
CPU checker: whole outputs where that is cheap, sampled rows / heads where it is not."""
import numpy as np
import pytest

from synth import workloads as W
from oracle import draft_entropy_topk, tree_prune, tree_attention, verify_accept

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def H():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2505_13254_amd import harness
    return harness


@pytest.fixture(scope="module")
def G():
    import gpu_util
    return gpu_util


def _np(t):
    torch.cuda.synchronize()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def _check_step(st, rs, n_rows=6, n_heads=3, accept_mode=0):
    w, t, h = st.w, st.t, st.host
    st.run()
    torch.cuda.synchronize()
    # ---- stage 1 on sampled rows: indices bit-exact, entropies 1e-5
    R = t["draft_rows"].shape[0]
    rows = sorted(set(int(x) for x in rs.randint(0, R, size=n_rows)) | {0, R - 1})
    want = draft_entropy_topk(_np(t["draft_rows"][rows]), w.topk, w.temperature)
    got = {k: _np(v)[rows] for k, v in t["s1_out"].items()}
    assert np.array_equal(got["topk_idx"], want["topk_idx"])
    for k in ("ent_topk", "ent_full"):
        assert np.all(np.abs(got[k] - want[k]) <= 1e-5 * np.maximum(np.abs(want[k]), 1e-3)), k
    # ---- stage 2, whole: same float32 confidences on both sides
    pr = tree_prune(_np(t["cand_parent"]), _np(t["cand_logc"]), _np(t["cand_offsets"]), _np(t["d_max"]),
                    _np(t["theta"]), _np(t["max_nodes"]))
    s2 = {k: _np(v) for k, v in t["s2_out"].items()}
    n = int(pr["out_offsets"][-1])
    assert np.array_equal(s2["keep"], pr["keep"]) and np.array_equal(s2["out_offsets"], pr["out_offsets"])
    assert np.array_equal(s2["out_src"][:n], pr["out_src"]) and np.array_equal(s2["out_parent"][:n], pr["out_parent"])
    assert np.array_equal(s2["cumlogp"].view(np.uint32), pr["cumlogp"].view(np.uint32))
    # ---- stage 3 on sampled (batch entry, query head): all rows of that head
    no, po = h["attn_node_offsets"].numpy(), h["attn_prefix_offsets"].numpy()
    parent = _np(t["attn_parent"])
    o = t["o"].float().cpu().numpy()
    G = w.Hq // w.Hkv
    for _ in range(n_heads):
        b = int(rs.randint(0, len(no) - 1))
        hq = int(rs.randint(0, w.Hq))
        g = hq // G
        n0, n1, p0, p1 = int(no[b]), int(no[b + 1]), int(po[b]), int(po[b + 1])
        if n1 == n0:
            continue
        wo, _ = tree_attention(_np(t["q"][n0:n1, hq:hq + 1]), _np(t["k_prefix"][p0:p1, g:g + 1]),
                               _np(t["v_prefix"][p0:p1, g:g + 1]), _np(t["k_tree"][n0:n1, g:g + 1]),
                               _np(t["v_tree"][n0:n1, g:g + 1]), parent[n0:n1], [0, n1 - n0], [0, p1 - p0], h["scale"])
        err = np.abs(o[n0:n1, hq] - wo[:, 0]).max()
        assert err <= (2e-2 if w.dtype == "bf16" else 1e-4), (b, hq, err)
        assert err <= 1e-2 * np.abs(wo).max() + 1e-6, (b, hq, err, np.abs(wo).max())
    # ---- stage 4, whole walk (argmax rows are cheap; the stochastic modes read only visited rows)
    tl = _np(t["target_logits"])
    # (the point-mass rule never uses the draft rows; the checker still wants an array there)
    dl = _np(t["draft_logits"]) if accept_mode == 1 else (tl if accept_mode == 2 else None)
    wa = verify_accept(tl, dl, _np(t["token"]), s2["out_parent"][:n], s2["out_offsets"], accept_mode, w.temperature,
                       _np(t["uniforms"]) if accept_mode else None, h["max_depth"])
    ga = {k: _np(v) for k, v in t["s4_out"].items()}
    for k in wa:
        assert np.array_equal(ga[k], wa[k]), (k, ga[k], wa[k])
    return wa


def test_workload2_bench_configuration(H):
    w = W.WORKLOADS[2]
    st = H.build_step(w, 0, layers=w.layers, accept_mode=0)
    assert st.host["NNp"] == 61 and st.host["cand_nodes"] == 511 and st.t["q"].shape[0] == 61 * 32
    _check_step(st, np.random.RandomState(0), n_heads=6)


def test_workload3_threshold_sweep(H):
    w = W.WORKLOADS[3]
    kept = []
    for th in w.theta:
        st = H.build_step(w, 0, layers=1, accept_mode=0, theta=th)
        _check_step(st, np.random.RandomState(1), n_rows=3, n_heads=2)
        kept.append(set(st.host["out_src"].tolist()))
    assert kept[0] <= kept[1] <= kept[2]


def test_workload4_single_layer(H):
    w = W.WORKLOADS[4]
    st = H.build_step(w, 0, layers=1, accept_mode=0)
    assert st.host["NNp"] == 97
    _check_step(st, np.random.RandomState(2), n_rows=3, n_heads=3)


def test_workload5_ragged_batch(H):
    w = W.WORKLOADS[5]
    st = H.build_step(w, 0, layers=1, accept_mode=0)
    sizes = np.diff(st.host["out_offsets"])
    assert len(sizes) == 16 and sizes.min() >= 2 and sizes.max() <= 129
    res = _check_step(st, np.random.RandomState(3), n_rows=4, n_heads=5)
    assert res["accept_len"].shape == (16,)


@pytest.mark.parametrize("variant", ["peaky", "unit"])
def test_workload5_ragged_launch_with_sharp_scores(H, G, variant):
    """The batched workload's own launch (16 sequences, prefixes of 512 .. 16384 tokens, ragged trees, key
    splits merged by the combine kernel, row groups beyond 256 rows) on inputs whose softmax is far from
    uniform: scores of order one, and planted keys near the end of the prefix and among the ancestors.
    Every head of three sequences is compared: the longest prefix, the shortest, the largest tree."""
    w = W.WORKLOADS[5]
    st = H.build_step(w, 0, layers=1, accept_mode=0)
    t, h = st.t, st.host
    no, po = h["attn_node_offsets"].numpy(), h["attn_prefix_offsets"].numpy()
    par = h["out_parent"]
    B = len(no) - 1
    parts = [W.attention_inputs(w, 1, s, int(po[s + 1] - po[s]), int(no[s + 1] - no[s]), variant,
                                parent=par[no[s]:no[s + 1]]) for s in range(B)]
    for i, name in enumerate(("q", "k_prefix", "v_prefix", "k_tree", "v_tree")):
        t[name].copy_(G.dev_store(np.concatenate([p[i] for p in parts], axis=0)))
    t["o"].zero_()
    st.stage3()
    o = G.host(t["o"])
    Ls, Ms = np.diff(po), np.diff(no)
    assert Ms.max() * (w.Hq // w.Hkv) > 256 and Ls.max() > 8 * 1024     # several row groups, several key splits
    for s in sorted({int(np.argmax(Ls)), int(np.argmin(Ls)), int(np.argmax(Ms))}):
        q, kp, vp, kt, vt = parts[s]
        sub = dict(q=q, k_prefix=kp, v_prefix=vp, k_tree=kt, v_tree=vt, parent=par[no[s]:no[s + 1]],
                   node_offsets=np.asarray([0, Ms[s]]), prefix_offsets=np.asarray([0, Ls[s]]), scale=h["scale"])
        want, _ = tree_attention(q, kp, vp, kt, vt, sub["parent"], sub["node_offsets"], sub["prefix_offsets"], h["scale"])
        diff = np.abs(o[no[s]:no[s + 1]].astype(np.float64) - want)
        assert diff.max() <= 2e-2, (s, diff.max())
        assert diff.max() <= 1e-2 * np.abs(want).max(), (s, diff.max(), np.abs(want).max())
        assert (diff / G.attention_error_bound(sub, want)).max() <= 1.0, s


@pytest.mark.parametrize("wid,mode", [(2, 1), (2, 2), (4, 1)])
def test_stochastic_accept_at_full_vocabulary(H, wid, mode):
    """The sampling modes on the 128256-token vocabulary (workload 2: ratio rule and point-mass rule;
    workload 4 is specified with the ratio rule), one attention layer."""
    w = W.WORKLOADS[wid]
    st = H.build_step(w, 0, layers=1, accept_mode=mode)
    res = _check_step(st, np.random.RandomState(10 + wid + mode), n_rows=2, n_heads=1, accept_mode=mode)
    assert res["bonus_token"].min() >= 0


@pytest.mark.parametrize("name,D,sizes,Ls,variant", [
    ("a tree of 1024 rows on the 8B shape", 128, [1024], [4096], "peaky"),
    ("large and small trees, long and short prefixes", 128, [700, 61, 300], [9000, 100, 3000], "unit"),
    ("head dimension 64 on the 8B head layout", 64, [61, 129], [8192, 2048], "unit_v"),
])
def test_large_trees_and_head_dimension_64_at_full_head_count(G, name, D, sizes, Ls, variant):
    """32 query heads on 8 KV heads as in the 8B workload, with what the matrix-core kernel takes beyond that
    workload's own shape: trees past 256 rows (the ancestor table comes from its own launch) and head
    dimension 64 (KV heads in pairs).  The launch covers all heads; two KV heads' query heads are compared
    with the checker, which gets those heads alone."""
    import paper_2505_13254_amd as hs
    w = W.small(W.WORKLOADS[2], D=D)
    rs = np.random.RandomState(len(name))
    parents = [[-1] + [int(rs.randint(max(0, i - 9), i)) for i in range(1, n)] for n in sizes]
    parts = [W.attention_inputs(w, 51, s, int(L), len(p), variant, parent=np.asarray(p))
             for s, (p, L) in enumerate(zip(parents, Ls))]
    q, kp, vp, kt, vt = (np.concatenate([x[i] for x in parts], axis=0) for i in range(5))
    no = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    po = np.concatenate([[0], np.cumsum(Ls)]).astype(np.int64)
    par = np.concatenate([np.asarray(p, np.int32) for p in parents])
    scale = 1.0 / np.sqrt(D)
    st = dict(w=w, q=q, k_prefix=kp, v_prefix=vp, k_tree=kt, v_tree=vt, parent=par, node_offsets=no,
              prefix_offsets=po, scale=scale)
    got, _ = G.run_attention(st)
    assert hs.hs_tree_attention_last_kernel() == 1
    grp = w.Hq // w.Hkv
    for g in (1, 6):
        hq = slice(g * grp, (g + 1) * grp)
        sub = dict(st, q=q[:, hq], k_prefix=kp[:, g:g + 1], v_prefix=vp[:, g:g + 1], k_tree=kt[:, g:g + 1],
                   v_tree=vt[:, g:g + 1])
        want, _ = tree_attention(sub["q"], sub["k_prefix"], sub["v_prefix"], sub["k_tree"], sub["v_tree"], par, no, po, scale)
        diff = np.abs(got[:, hq].astype(np.float64) - want)
        assert diff.max() <= 2e-2, (g, diff.max())
        assert (diff / G.attention_error_bound(sub, want)).max() <= 1.0, g
