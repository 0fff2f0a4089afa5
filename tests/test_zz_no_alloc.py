"""hs_tree_prune_static (the entry point that allocates nothing: its scratch is a static device array of the
library) against hs_tree_prune on a caller's workspace: identical outputs, bit for bit, on two calls in
a row of which the second is the smaller one (the scratch keeps the first call's contents)."""
import ctypes

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
KEYS = ("depth", "cumlogp", "keep", "out_offsets", "out_src", "out_parent")


def _trees(seed, B, n_lo, n_hi):
    rs = np.random.RandomState(seed)
    sizes = rs.randint(n_lo, n_hi + 1, size=B)
    sizes[rs.randint(B)] = 0 if B > 2 else sizes[0]          # an empty sequence among several
    off = np.zeros(B + 1, np.int32)
    off[1:] = np.cumsum(sizes)
    NN = int(off[-1])
    parent = np.full(NN, -1, np.int32)
    for s in range(B):
        for i in range(1, int(sizes[s])):
            parent[off[s] + i] = rs.randint(max(0, i - 9), i)
    logc = (-rs.exponential(0.7, size=NN)).astype(np.float32)
    d_max = rs.randint(2, 12, size=B).astype(np.int32)
    theta = rs.uniform(-9.0, -2.0, size=B).astype(np.float32)
    budget = rs.randint(0, 60, size=B).astype(np.int32)      # 0 switches the budget off
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    return dict(parent=t(parent), logc=t(logc), node_offsets=t(off), d_max=t(d_max), theta=t(theta), max_nodes=t(budget),
                NN=NN, B=B)


def _outputs(NN, B, fill):
    o = dict(depth=torch.full((NN,), fill, dtype=torch.int32, device=DEV),
             cumlogp=torch.full((NN,), float(fill), dtype=torch.float32, device=DEV),
             keep=torch.full((NN,), 7, dtype=torch.uint8, device=DEV),
             out_offsets=torch.full((B + 1,), fill, dtype=torch.int32, device=DEV),
             out_src=torch.full((max(NN, 1),), fill, dtype=torch.int32, device=DEV),
             out_parent=torch.full((max(NN, 1),), fill, dtype=torch.int32, device=DEV))
    return o


def _both(hs, c):
    args = (c["parent"], c["logc"], c["node_offsets"], c["d_max"], c["theta"], c["max_nodes"])
    want = hs.hs_tree_prune(*args, out=_outputs(c["NN"], c["B"], -5))
    got = _outputs(c["NN"], c["B"], -9)
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    hs.hs_tree_prune_static(*args, out=got)
    torch.cuda.synchronize()
    free_after = torch.cuda.mem_get_info()[0]
    for k in KEYS:
        a, b = want[k].cpu().numpy(), got[k].cpu().numpy()
        assert a.tobytes() == b.tobytes(), k
    return free_before, free_after


def test_static_scratch_matches_workspace_call_twice_in_a_row():
    import paper_2505_13254_amd as hs
    big = _trees(3, 23, 200, 5000)        # several trees beyond the LDS-resident size, ragged, one empty (~60 k nodes)
    small = _trees(4, 5, 1, 300)          # the smaller call afterwards: stale scratch must not leak into it
    one = _trees(5, 1, 511, 511)          # single sequence (the selecting workgroup emits by itself)
    _both(hs, big)                        # (the first call on the device resolves the array's address)
    f0, f1 = _both(hs, small)
    assert f0 == f1, "the call changed the amount of free device memory"
    f0, f1 = _both(hs, one)
    assert f0 == f1
    _both(hs, big)


def test_static_scratch_limits_are_refused_before_any_launch():
    import paper_2505_13254_amd as hs
    lib = hs.lib()
    c = _trees(6, 2, 3, 9)
    o = _outputs(c["NN"], c["B"], 0)
    p = lambda t: ctypes.c_void_p(t.data_ptr())
    tail = (p(c["d_max"]), p(c["theta"]), p(c["max_nodes"]), p(o["depth"]), p(o["cumlogp"]), p(o["keep"]),
            p(o["out_offsets"]), p(o["out_src"]), p(o["out_parent"]), None)
    # more nodes / sequences than the static scratch holds: HS_ERR_UNSUPPORTED (3), nothing launched
    assert lib.hs_tree_prune_static(p(c["parent"]), p(c["logc"]), p(c["node_offsets"]), 2, 65537, *tail) == 3
    assert b"static scratch" in lib.hs_last_error()
    assert lib.hs_tree_prune_static(p(c["parent"]), p(c["logc"]), p(c["node_offsets"]), 4097, 10, *tail) == 3
    assert lib.hs_tree_prune_static(None, p(c["logc"]), p(c["node_offsets"]), 2, c["NN"], *tail) == 1   # HS_ERR_NULL
    torch.cuda.synchronize()
    assert int(o["out_offsets"].abs().sum()) == 0     # untouched
