"""Input generators are reproducible (checksums), and the step builder yields the workloads'
stated shapes."""
import importlib.util
import os

import numpy as np
import pytest

from synth import workloads as W
from oracle import pipeline as P

HERE = os.path.dirname(os.path.abspath(__file__))


def _load(name):
    spec = importlib.util.spec_from_file_location(name, os.path.join(HERE, "golden", name + ".py"))
    m = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(m)
    return m


def test_input_checksums_match_golden():
    import zlib
    want = {}
    for line in open(os.path.join(HERE, "golden", "input_checksums.txt")):
        if not line.startswith("#"):
            name, dt, shape, crc = line.split()
            want[name] = (dt, shape, crc)
    got = {}
    for name, t in _load("make_input_checksums").entries():
        t = np.ascontiguousarray(t)
        got[name] = (str(t.dtype), "x".join(map(str, t.shape)), "%08x" % zlib.crc32(t.tobytes()))
    assert got == want


def test_oracle_config1_matches_golden():
    want = {}
    for line in open(os.path.join(HERE, "golden", "oracle_config1.txt")):
        if not line.startswith("#"):
            k, v = line.split("=")
            want[k.strip()] = np.asarray([float(x) for x in v.split()])
    got = _load("make_oracle_config1").compute()
    assert set(got) == set(want)
    for k in want:
        assert np.allclose(np.asarray(got[k], np.float64).ravel(), want[k], rtol=1e-10, atol=1e-12), k


def test_bf16_rounding_is_nearest_even():
    import torch
    x = np.concatenate([np.random.RandomState(0).randn(4096).astype(np.float32) * 3,
                        np.asarray([1.00390625, 1.01171875, -1.00390625, 0.0, 65504.0], np.float32)])
    bits = W.rng.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().astype(np.uint16)
    assert np.array_equal(bits, ref)


def test_tree_shapes():
    w = W.WORKLOADS
    for wid, n in ((1, 16), (3, 128), (4, 96)):
        p = W.tree_parents(w[wid], 0)
        assert len(p) == n + 1 and p[0] == -1 and all(0 <= p[i] < i for i in range(1, len(p)))
        d = P.tree_depth(p, [0, len(p)])
        assert d.max() <= w[wid].max_depth and np.all(np.diff(d) >= 0)        # BFS order
        fan = np.bincount(p[1:])
        assert fan.max() <= w[wid].topk
    L = W.prefix_lengths(w[5], 0)
    assert len(L) == 16 and L.min() >= 512 and L.max() <= 16384


def test_step_of_the_8b_workload_has_61_rows():
    w = W.small(W.WORKLOADS[2], V=8192, prefix_len=(64, 64))       # reduced vocabulary and prefix
    st = P.build_step(w, 0, with_attention=False)
    assert st["prune_in"]["node_offsets"][-1] == 1 + 10 + 5 * 100   # candidates of a top-10 expansion
    assert st["node_offsets"][-1] == 61
    par = st["parent"]
    assert par[0] == -1 and all(0 <= par[i] < i for i in range(1, 61))
    for p in range(61):                                              # siblings carry distinct tokens
        kids = st["token"][[c for c in range(1, 61) if par[c] == p]]
        assert len(set(kids)) == len(kids)
    g = P.accept_out(st, P.GREEDY)
    assert 0 <= g["accept_len"][0] <= 6


def test_batched_workload_is_ragged():
    w = W.small(W.WORKLOADS[5], V=2048, B=8, prefix_len=(16, 64))
    st = P.build_step(w, 1, with_attention=True)
    sizes = np.diff(st["node_offsets"])
    assert sizes.min() >= 2 and sizes.max() <= 129 and len(set(sizes)) > 3
    assert st["q"].shape[0] == st["node_offsets"][-1]
    assert st["k_prefix"].shape[0] == st["prefix_offsets"][-1]
