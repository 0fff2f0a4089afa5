"""GPU parity of the device-side pieces of the adaptive step against the CPU checker:
hs_tree_expand (bit-exact trees and frontiers), hs_adaptive_control (bit-exact decisions, phi to
1e-5) and hs_tree_prune_counted (bit-exact)."""
import numpy as np
import pytest

from oracle import adaptive_control, draft_entropy_topk, tree_prune
from oracle.tree_expand import new_state, tree_expand
from oracle import pipeline as P
from synth import workloads as W

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

GAMMA = [0.3, 0.6, 1.0]
EDGES8 = [0.5, 1.0, 1.5, 2.5, 4.0, 6.0, 9.0]
INT_MAX = 2 ** 31 - 1


@pytest.fixture(scope="module")
def G():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import gpu_util
    return gpu_util


def _random_results(rs, n_slots, K, V=50000):
    p = rs.dirichlet(np.ones(K + 4), size=n_slots)[:, :K]
    p = -np.sort(-p, axis=1)
    idx = np.stack([rs.permutation(V)[:K] for _ in range(n_slots)]).astype(np.int32)
    return idx, np.log(p).astype(np.float32), rs.uniform(0, 2.3, size=n_slots).astype(np.float32)


def _host_state(hs_state, B, cap, F):
    torch.cuda.synchronize()
    return {k: v.cpu().numpy() for k, v in hs_state.items()}


@pytest.mark.parametrize("B,K,F,cap,levels,limits", [
    (1, 10, 10, 511, 6, None),                 # the 8B workload's candidate tree
    (5, 4, 3, 64, 7, [7, 2, 0, 5, 7]),         # per-sequence depth limits, one sequence never grows
    (3, 3, 2, 14, 5, None),                    # capacity runs out in the middle of a level
    (2, 64, 64, 1 + 64 + 64 * 64, 2, None),    # the largest level the call takes
])
def test_expand_levels_match_the_checker(G, B, K, F, cap, levels, limits):
    import paper_2505_13254_amd as hs
    rs = np.random.RandomState(B * 100 + K)
    state = hs.new_tree_state(B, cap, F, G.DEV)
    dl = None if limits is None else G.dev(np.asarray(limits, np.int32))
    ref = [new_state() for _ in range(B)]
    for lvl in range(levels):
        idx, lp, ent = _random_results(rs, B * F, K)
        hs.hs_tree_expand(state, G.dev(idx), G.dev(lp), G.dev(ent), dl, B, cap, F, K, first=(lvl == 0))
        got = _host_state(state, B, cap, F)
        for s in range(B):
            tree_expand(ref[s], idx[s * F:(s + 1) * F], lp[s * F:(s + 1) * F], ent[s * F:(s + 1) * F], F, cap,
                        None if limits is None else limits[s])
            r, n = ref[s], len(ref[s]["parent"])
            assert int(got["n_nodes"][s]) == n and int(got["level"][s]) == r["level"], (lvl, s)
            sl = slice(s * cap, s * cap + n)
            assert np.array_equal(got["parent"][sl], r["parent"]) and np.array_equal(got["token"][sl], r["token"])
            assert np.array_equal(got["depth"][sl], r["depth"])
            for k, name in (("logc", "logc"), ("cumlogp", "cum"), ("ent", "ent")):
                assert np.array_equal(got[k][sl].view(np.uint32), np.asarray(r[name], np.float32).view(np.uint32)), (lvl, s, k)
            nf = int(got["n_frontier"][s])
            assert nf == len(r["frontier"])
            assert list(got["frontier"][s * F:s * F + nf]) == r["frontier"]
            rows = got["frontier_rows"][s * F:(s + 1) * F]
            want_rows = [s * cap + f for f in r["frontier"]]
            want_rows += [want_rows[-1] if want_rows else s * cap] * (F - nf)
            assert list(rows) == want_rows, (lvl, s)


def _random_forest(rs, B, max_n):
    parents, logcs, ents = [], [], []
    for s in range(B):
        n = int(rs.randint(0, max_n + 1)) if s != 1 else 0          # one empty sequence
        par = [-1] + [int(rs.randint(max(0, i - 7), i)) for i in range(1, n)]
        parents.append(np.asarray(par[:n], np.int32))
        logcs.append(np.concatenate([[0.0], np.log(rs.uniform(0.02, 1.0, size=max(n - 1, 0)))])[:n].astype(np.float32))
        # per-sequence entropy scale, so that the path sums spread over all bins
        ents.append((rs.uniform(0.0, 2.3, size=n) * 10.0 ** rs.uniform(-2.5, 0.0)).astype(np.float32))
    return parents, logcs, ents


@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("spare", [False, True])
def test_adaptive_control_matches_the_checker(G, mode, spare):
    import paper_2505_13254_amd as hs
    rs = np.random.RandomState(10 + mode)
    B = 40
    parents, logcs, ents = _random_forest(rs, B, 300)
    counts = np.asarray([len(p) for p in parents], np.int32)
    packed_off = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    want = adaptive_control(np.concatenate(parents), np.concatenate(logcs), np.concatenate(ents), packed_off,
                            EDGES8, GAMMA, 3, 6, 60, mode)
    if spare:
        cap = 320
        off = (np.arange(B + 1) * cap).astype(np.int32)
        pad = lambda xs, fill, dt: np.concatenate([np.concatenate([x, np.full(cap - len(x), fill, dt)]) for x in xs])
        par, lc, en = pad(parents, 12345, np.int32), pad(logcs, np.nan, np.float32), pad(ents, np.nan, np.float32)
        nc = G.dev(counts)
    else:
        off, par, lc, en, nc = packed_off, np.concatenate(parents), np.concatenate(logcs), np.concatenate(ents), None
    out = hs.hs_adaptive_control(G.dev(par), G.dev(lc), G.dev(en), G.dev(off), nc, EDGES8, GAMMA, 3, 6, 60, mode)
    got = {k: G.host(v) for k, v in out.items()}
    for k in ("pstar", "bin", "d_prime", "n_prime"):
        assert np.array_equal(got[k], want[k]), k
    assert np.all(np.abs(got["phi"] - want["phi"]) <= 1e-5 * np.maximum(np.abs(want["phi"]), 1e-3))
    assert len(set(want["bin"].tolist())) >= 4                       # the case spreads over the bins


def test_adaptive_control_on_a_bin_boundary_and_with_one_bin(G):
    import paper_2505_13254_amd as hs
    par, lc = np.asarray([-1, 0], np.int32), np.asarray([0, -1], np.float32)
    off = np.asarray([0, 2], np.int32)
    for j, e in enumerate(EDGES8):                                   # a value on a boundary belongs to the upper bin
        out = hs.hs_adaptive_control(G.dev(par), G.dev(lc), G.dev(np.asarray([e, 0], np.float32)), G.dev(off), None,
                                     EDGES8, GAMMA, 3, 5, 20)
        assert int(G.host(out["bin"])[0]) == j + 1
    out = hs.hs_adaptive_control(G.dev(par), G.dev(lc), G.dev(np.asarray([5, 0], np.float32)), G.dev(off), None,
                                 [], [0.5], 2, 5, 20)
    assert int(G.host(out["bin"])[0]) == 0 and int(G.host(out["d_prime"])[0]) == 7 and int(G.host(out["n_prime"])[0]) == 12


def test_prune_counted_matches_the_checker(G):
    import paper_2505_13254_amd as hs
    rs = np.random.RandomState(21)
    B, cap = 9, 200
    parents, logcs, _ = _random_forest(rs, B, cap)
    counts = np.asarray([len(p) for p in parents], np.int32)
    packed_off = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    d_max = rs.randint(2, 12, size=B).astype(np.int32)
    theta = np.where(rs.uniform(size=B) < 0.5, -np.inf, -6.0).astype(np.float32)
    budget = rs.randint(0, 60, size=B).astype(np.int32)
    want = tree_prune(np.concatenate(parents), np.concatenate(logcs), packed_off, d_max, theta, budget)
    pad = lambda xs, fill, dt: np.concatenate([np.concatenate([x, np.full(cap - len(x), fill, dt)]) for x in xs])
    out = hs.hs_tree_prune(G.dev(pad(parents, 777, np.int32)), G.dev(pad(logcs, np.nan, np.float32)),
                           G.dev((np.arange(B + 1) * cap).astype(np.int32)), G.dev(d_max), G.dev(theta), G.dev(budget),
                           node_counts=G.dev(counts))
    got = {k: G.host(v) for k, v in out.items()}
    n = int(want["out_offsets"][-1])
    assert np.array_equal(got["out_offsets"], want["out_offsets"])
    assert np.array_equal(got["out_src"][:n], want["out_src"]) and np.array_equal(got["out_parent"][:n], want["out_parent"])
    for s in range(B):
        a, b = s * cap, packed_off[s]
        c = int(counts[s])
        assert np.array_equal(got["keep"][a:a + c], want["keep"][b:b + c])
        assert np.array_equal(got["cumlogp"][a:a + c].view(np.uint32), want["cumlogp"][b:b + c].view(np.uint32))
        assert np.array_equal(got["depth"][a:a + c], want["depth"][b:b + c])


def test_device_loop_grows_the_pipelines_tree(G):
    """Expansion driven entirely on the device (gather of the frontier's draft rows, quantification,
    growth) reproduces the candidate tree that the checker's pipeline builds on the host."""
    import paper_2505_13254_amd as hs
    w = W.small(W.WORKLOADS[2], V=4000, topk=5, frontier=4, max_depth=4)
    K, F, depth = w.topk, w.frontier, w.max_depth
    ref = P.expand_tree(w, 0, 0, depth)
    cap = len(ref["parent"])
    rows_all = G.dev(W.logits_rows(w, 0, "draft", 0, range(cap)))     # the draft row of every candidate
    state = hs.new_tree_state(1, cap, F, G.DEV)
    x = rows_all[:1].repeat(F, 1).contiguous()                        # level 0: the root's row in slot 0
    for lvl in range(depth):
        r = hs.hs_draft_entropy_topk(x, K, w.temperature, want_full=False)
        hs.hs_tree_expand(state, r["topk_idx"], r["topk_logp"], r["ent_topk"], None, 1, cap, F, K, first=(lvl == 0))
        x = rows_all.index_select(0, state["frontier_rows"].long())   # stands in for the draft model's next pass
    got = _host_state(state, 1, cap, F)
    assert int(got["n_nodes"][0]) == cap
    assert np.array_equal(got["parent"], ref["parent"]) and np.array_equal(got["token"], ref["token"])
    assert np.allclose(got["logc"], ref["logc"], rtol=2e-5, atol=2e-6)
    ent_ref = np.zeros(cap)
    ent_ref[ref["draft_ids"]] = ref["stage1"]["ent_topk"]
    assert np.all(np.abs(got["ent"] - ent_ref) <= 1e-5 * np.maximum(np.abs(ent_ref), 1e-3))


def test_tree_validate_matches_the_checker(G):
    import paper_2505_13254_amd as hs
    from oracle.tree_validate import tree_validate
    rs = np.random.RandomState(33)
    cases = [([-1, 0, 0, 1, 1, 2], [9, 4, 5, 7, 7, 7], [0, 6]),
             ([-1, 0, -1, 0, 5], None, [0, 2, 5]),
             ([0, 0, 0], None, [0, 3]),
             ([-1, 0], None, [0, 2, 1]),
             ([-1, 0, 1, -1, 0, 0], [1, 2, 3, 4, 5, 6], [0, 3, 3, 6]),
             ([-1] + [0] * 300 + [1] * 256, None, [0, 557]),          # a node with more than 256 children
             ([-1, 0] + [1] * 257, list(range(259)), [0, 259])]
    for _ in range(40):                                            # random forests, some rows damaged
        sizes = [int(x) for x in rs.randint(0, 40, size=int(rs.randint(1, 6)))]
        par, tok = [], []
        for n in sizes:
            par += [-1] + [int(rs.randint(0, i)) for i in range(1, n)] if n else []
            tok += [int(x) for x in rs.randint(0, 6, size=n)]
        par = np.asarray(par, np.int32)
        for k in rs.randint(0, max(len(par), 1), size=int(rs.randint(0, 3))):
            if len(par):
                par[k] = int(rs.randint(-2, len(par)))
        cases.append((par, tok if rs.uniform() < 0.5 else None, np.concatenate([[0], np.cumsum(sizes)])))
    for par, tok, off in cases:
        want = tree_validate(par, tok, off)
        rep = hs.hs_tree_validate(G.dev(np.asarray(par, np.int32)), None if tok is None else G.dev(np.asarray(tok, np.int32)),
                                  G.dev(np.asarray(off, np.int32)))
        assert tuple(int(x) for x in G.host(rep)) == want, (list(par), tok, list(off))
