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


def _check(st, b, want, layers):
    d_prime, n_prime = st.decision(b)
    assert b == int(want["control"]["bin"][0]) and d_prime == int(want["control"]["d_prime"][0])
    assert n_prime == int(want["control"]["n_prime"][0])
    t = st.t
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
    # attention of the last layer, one query head, against the checker
    l, hq = layers - 1, 5
    g = hq // (st.w.Hq // st.w.Hkv)
    wo, _ = tree_attention(_np(a["q"][l * M:(l + 1) * M, hq:hq + 1]), _np(t["k_prefix"][l * L:(l + 1) * L, g:g + 1]),
                           _np(t["v_prefix"][l * L:(l + 1) * L, g:g + 1]), _np(a["k_tree"][l * M:(l + 1) * M, g:g + 1]),
                           _np(a["v_tree"][l * M:(l + 1) * M, g:g + 1]), want["prune"]["out_parent"], [0, M], [0, L],
                           st.host["scale"])
    o = a["o"].float().cpu().numpy()[l * M:(l + 1) * M, hq]
    assert np.abs(o - wo[:, 0]).max() <= 2e-2


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
        # eager work of the program's own between the replays, and outputs cleared
        for a in st.t["attn"].values():
            a["o"].zero_()
            a["s4_out"]["accept_len"].fill_(-7)
        st.t["state"]["n_nodes"].fill_(0)
        torch.cuda.synchronize()
        assert st.step_graph() == b
        _check(st, b, want, layers)
