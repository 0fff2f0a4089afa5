"""The device-driven adaptive step (level-by-level expansion, complexity decision, extended
drafting, pruning, attention, accept) against the CPU checker's pipeline, eager and as cached HIP
graphs (one per entropy bin), with several replays of each graph."""
import numpy as np
import pytest

from oracle import pipeline as P, tree_attention
from synth import workloads as W

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def H():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2505_13254_amd import harness
    return harness


def _np(t):
    torch.cuda.synchronize()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def _check(st, b, want, layers, heads=((-1, 5),)):
    d_prime, n_prime = st.decision(b)
    assert b == int(want["control"]["bin"][0]) and d_prime == int(want["control"]["d_prime"][0])
    assert n_prime == int(want["control"]["n_prime"][0])
    t = st.t
    # the decision the device took (what the prune call and the extra levels were given)
    for k in ("bin", "d_prime", "n_prime"):
        assert int(_np(t["ctl"][k])[0]) == int(want["control"][k][0]), k
    p_gpu, p_want = int(_np(t["ctl"]["pstar"])[0]), int(want["control"]["pstar"][0])
    if p_gpu != p_want:
        # Nearly one-hot draft rows: several final tokens carry a confidence of 1 up to rounding, and
        # float32 and float64 log-probabilities order them differently.  What is unique then is the
        # decision (checked above); the path itself must be one of the tied best of the same level.
        sw = want["state"]
        par, lc = np.asarray(sw["parent"]), np.minimum(np.asarray(sw["logc"], np.float64), 0.0)
        depth = lambda i: 0 if i == 0 else 1 + depth(int(par[i]))
        assert st.pstar_mode == 1 and depth(p_gpu) == depth(p_want) and abs(lc[p_gpu] - lc[p_want]) <= 1e-6
    n = len(want["state"]["parent"])
    assert int(_np(t["state"]["n_nodes"])[0]) == n
    assert np.array_equal(_np(t["state"]["parent"])[:n], want["state"]["parent"])
    assert np.array_equal(_np(t["state"]["token"])[:n], want["state"]["token"])
    M = n_prime + 1
    assert np.array_equal(_np(t["s2_out"]["out_src"])[:M], want["prune"]["out_src"])
    assert np.array_equal(_np(t["s2_out"]["out_parent"])[:M], want["prune"]["out_parent"])
    a = t["attn"][M]
    for k in ("accept_len", "bonus_token"):
        assert np.array_equal(_np(a["s4_out"][k]), want["accept"][k]), k
    L = int(st.host["prefix_offsets"][1])
    # attention of sampled (layer, query head) pairs against the checker
    for l, hq in heads:
        l = l % layers
        g = hq // (st.w.Hq // st.w.Hkv)
        wo, _ = tree_attention(_np(a["q"][l * M:(l + 1) * M, hq:hq + 1]), _np(t["k_prefix"][l * L:(l + 1) * L, g:g + 1]),
                               _np(t["v_prefix"][l * L:(l + 1) * L, g:g + 1]), _np(a["k_tree"][l * M:(l + 1) * M, g:g + 1]),
                               _np(a["v_tree"][l * M:(l + 1) * M, g:g + 1]), want["prune"]["out_parent"], [0, M], [0, L],
                               st.host["scale"])
        o = a["o"].float().cpu().numpy()[l * M:(l + 1) * M, hq]
        assert np.abs(o - wo[:, 0]).max() <= 2e-2
        assert np.abs(o - wo[:, 0]).max() <= 1e-2 * np.abs(wo).max()


def _clear(st):
    """Eager work of the program's own between replays; stale outputs cannot pass for fresh ones."""
    for a in st.t["attn"].values():
        a["o"].zero_()
        a["s4_out"]["accept_len"].fill_(-7)
    st.t["state"]["n_nodes"].fill_(0)
    st.t["ctl"]["bin"].fill_(-3)
    torch.cuda.synchronize()


def _alternating_steps(H, w, layers, base, temps, order, heads, pstar_mode=0):
    """One AdaptiveStep, every per-bin graph captured once, then a sequence of steps whose draft rows,
    and with them the entropy bin and the graph to replay, change from step to step.  `base`: the
    seven (synthetic) bin boundaries, placed so that the draft temperatures fall into different bins."""
    st = H.build_adaptive(w, 0, layers=layers, edges=base, pstar_mode=pstar_mode)
    want = {T: P.adaptive_step(W.small(w, temperature=T), 0, base, st.gamma, st.alpha, pstar_mode=pstar_mode)
            for T in temps}
    shapes = {T: (int(x["control"]["d_prime"][0]), int(x["control"]["n_prime"][0])) for T, x in want.items()}
    assert len(set(shapes.values())) >= 3, shapes          # at least three different graphs get used
    st.capture()                                           # the drafting graph and one graph per distinct (d', N')
    assert len({id(g) for k, g in st.graphs.items() if k != "draft"}) == len({st.decision(b) for b in range(8)})
    prev = None
    for T in order:
        st.set_temperature(T)
        _clear(st)
        b = st.step_graph()
        assert b == int(want[T]["control"]["bin"][0])
        assert prev is None or shapes[T] != prev, "the sequence is meant to switch graphs at every step"
        prev = shapes[T]
        _check(st, b, want[T], layers, heads)
    return st


@pytest.mark.parametrize("pstar_mode", [0, 1])
def test_adaptive_steps_switch_between_cached_graphs(H, pstar_mode):
    w = W.small(W.WORKLOADS[2], V=6000, prefix_len=(300, 300), topk=5, frontier=4, max_depth=4, max_nodes=20)
    if pstar_mode == 0:
        edges = [0.4, 1.0, 2.5, 4.5, 5.8, 6.3, 6.4]   # Phi is 0.18 / 0.66 / 1.64 / 3.68 / 5.51 at the temperatures below
        temps = [0.0625, 0.125, 0.25, 0.5, 1.0]
    else:                                             # the other reading of P*: other paths, other sums
        edges = [0.2, 1.0, 2.5, 4.5, 5.8, 6.3, 6.4]   # Phi is 0.0002 / 0.79 / 2.37 / 3.68 / 5.51
        temps = [0.015625, 0.0625, 0.25, 0.5, 1.0]
    a, b, c, d, e = temps
    order = [e, a, b, c, a, d, b, e, a, c, b, d]
    _alternating_steps(H, w, 2, edges, temps, order, ((-1, 5), (0, 0)), pstar_mode)


def test_adaptive_steps_at_the_full_8b_size(H):
    """Sections 4.1 - 4.3 end to end at V = 128256, L = 2048, 32 layers: alternating bins, sampled heads."""
    w = W.WORKLOADS[2]
    edges = [1.0, 3.0, 8.0, 11.0, 12.0, 13.0, 14.0]   # Phi is 0.57 / 2.38 / 7.13 / 10.2 at the temperatures below
    temps = [0.125, 0.25, 0.5, 1.0]
    order = [1.0, 0.125, 0.5, 0.25, 1.0, 0.125, 0.25, 0.5, 0.125, 1.0]
    _alternating_steps(H, w, w.layers, edges, temps, order, ((0, 0), (13, 17), (31, 31)))


@pytest.mark.parametrize("scale,want_bin", [(1.0, None), (1e-3, 7), (1e3, 0)])
def test_adaptive_step_eager_and_graphs(H, scale, want_bin):
    w = W.small(W.WORKLOADS[2], V=6000, prefix_len=(300, 300), topk=5, frontier=4, max_depth=4, max_nodes=20)
    layers = 2
    base = [0.5 * w.max_depth * x for x in (0.2, 0.4, 0.6, 0.8, 1.0, 1.3, 1.7)]
    edges = [e * scale for e in base]
    st = H.build_adaptive(w, 0, layers=layers, edges=edges)
    want = P.adaptive_step(w, 0, edges, st.gamma, st.alpha)
    if want_bin is not None:
        assert int(want["control"]["bin"][0]) == want_bin
    b = st.step_eager()
    _check(st, b, want, layers)
    st.capture(bins=[b])
    for rep in range(3):
        _clear(st)
        assert st.step_graph() == b
        _check(st, b, want, layers)
