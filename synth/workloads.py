"""Seeded synthetic inputs for the five verification workloads.

Only raw inputs are made here: prefix lengths, random tree shapes, logits rows,
Q/K/V tensors and uniforms.  Anything that needs the method's own arithmetic
(top-k expansion, confidences, pruning) is done by whoever consumes these
inputs, so the CPU checker and the GPU library can both be fed from this module
without sharing any of their code.

Streams are keyed by (workload id, seed, tensor tag, sequence, row), so a row
can be regenerated on its own, in any order.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Tuple

import numpy as np

from . import rng

# tensor tags
_T_LEN, _T_TREE, _T_PERM, _T_TAU, _T_DRAFT, _T_TARGET, _T_Q, _T_KP, _T_VP, _T_KT, _T_VT, _T_U, _T_PLANT = range(13)


@dataclass(frozen=True)
class Workload:
    wid: int
    name: str
    dtype: str                    # "f32" or "bf16": storage type of Q/K/V/O
    B: int
    Hq: int
    Hkv: int
    D: int
    V: int
    prefix_len: Tuple[int, int]   # inclusive range the prefix length is drawn from
    logits: str                   # "gauss" (tau * N(0,1)) or "zipf"
    tau: Tuple[float, float] = (1.0, 1.0)
    rho: float = 0.9              # draft/target correlation of the gaussian rows
    zipf_s: float = 1.1
    zipf_noise: float = 0.5
    tree: str = "random"          # "levels", "grow" or "expand"
    levels: Tuple[int, ...] = ()  # tree == "levels": nodes per depth
    n_nodes: int = 0              # tree == "grow": draft nodes
    max_depth: int = 0
    fanout: Tuple[int, int] = (1, 1)
    topk: int = 10                # K of the draft top-k
    frontier: int = 10            # tree == "expand": nodes expanded per depth
    theta: Tuple[float, ...] = (float("-inf"),)
    max_nodes: int = 0
    accept: Tuple[str, ...] = ("greedy",)
    temperature: float = 1.0
    margin: float = 0.0           # forced top-1/top-2 logit gap
    layers: int = 1               # decoder layers of the model this layer is shaped after


WORKLOADS = {
    1: Workload(1, "tiny", "f32", 1, 8, 8, 64, 1024, (128, 128), "gauss", tau=(0.5, 8.0),
                tree="levels", levels=(3, 4, 5, 4), max_depth=4, theta=(-4.0,), margin=1e-3, layers=1),
    2: Workload(2, "llama3-8b", "bf16", 1, 32, 8, 128, 128256, (2048, 2048), "zipf",
                tree="expand", max_depth=6, max_nodes=60, accept=("greedy", "stochastic"), layers=32),
    3: Workload(3, "llama2-13b", "bf16", 1, 40, 40, 128, 32000, (4096, 4096), "gauss", tau=(0.3, 10.0),
                tree="grow", n_nodes=128, max_depth=8, fanout=(1, 4), theta=(-2.0, -4.0, -8.0), layers=40),
    4: Workload(4, "llama3-70b", "bf16", 1, 64, 8, 128, 128256, (8192, 8192), "zipf",
                tree="grow", n_nodes=96, max_depth=10, fanout=(1, 3), accept=("stochastic",), layers=80),
    5: Workload(5, "batched-8b", "bf16", 16, 32, 8, 128, 128256, (512, 16384), "gauss", tau=(0.3, 10.0),
                tree="expand", max_depth=10, max_nodes=128, layers=32),
}


def small(w: Workload, **kw) -> Workload:
    """A reduced copy of a workload (for CPU-sized tests); fields overridden by keyword."""
    return replace(w, **kw)


def _key(w: Workload, seed: int, tag: int, s: int = 0, row: int = 0, extra: int = 0):
    return rng.make_key(w.wid, seed, tag, s, row, extra)


# ----------------------------------------------------------------------------- shapes
def prefix_lengths(w: Workload, seed: int) -> np.ndarray:
    lo, hi = w.prefix_len
    if lo == hi:
        return np.full(w.B, lo, dtype=np.int64)
    return rng.randint(_key(w, seed, _T_LEN), w.B, lo, hi)


def tree_parents(w: Workload, seed: int, s: int = 0) -> np.ndarray:
    """Parent pointers (int32, root first, BFS order, parent[0] = -1) of a random tree.

    "levels": fixed node count per depth, each node's parent uniform over the previous depth.
    "grow":   breadth-first growth, fan-out uniform in `fanout`, at most
              ceil(1.5 * n_nodes / max_depth) nodes per depth, until n_nodes or max_depth.
    """
    key = _key(w, seed, _T_TREE, s)
    if w.tree == "levels":
        parent = [-1]
        prev = [0]
        ctr = 0
        for cnt in w.levels:
            draws = rng.randint(rng.make_key(int(key), ctr), cnt, 0, len(prev) - 1)
            ctr += 1
            ps = np.sort(np.asarray(prev)[draws])          # siblings contiguous, BFS order
            cur = list(range(len(parent), len(parent) + cnt))
            parent.extend(int(p) for p in ps)
            prev = cur
        return np.asarray(parent, dtype=np.int32)
    if w.tree == "grow":
        cap = -(-3 * w.n_nodes // (2 * w.max_depth))
        fo = rng.randint(key, 4 * w.n_nodes + 16, w.fanout[0], w.fanout[1])
        parent, depth = [-1], [0]
        level_count = {}
        head, draw = 0, 0
        while head < len(parent) and len(parent) < w.n_nodes + 1:
            d = depth[head] + 1
            if d <= w.max_depth:
                k = int(fo[draw]); draw += 1
                for _ in range(k):
                    if len(parent) >= w.n_nodes + 1 or level_count.get(d, 0) >= cap:
                        break
                    parent.append(head); depth.append(d)
                    level_count[d] = level_count.get(d, 0) + 1
            head += 1
        return np.asarray(parent, dtype=np.int32)
    raise ValueError("tree_parents: workload %r builds its tree by top-k expansion" % w.name)


# ----------------------------------------------------------------------------- logits
def _top2_gap(x: np.ndarray) -> float:
    p = np.partition(x, x.size - 2)
    return float(p[-1] - p[-2])


def _gauss_pair(w: Workload, seed: int, s: int, row: int, extra: int):
    u = rng.uniform(_key(w, seed, _T_TAU, s, row), 1)[0]
    tau = float(np.exp(np.log(w.tau[0]) + u * (np.log(w.tau[1]) - np.log(w.tau[0]))))
    zd = rng.normal(_key(w, seed, _T_DRAFT, s, row, extra), w.V)
    zn = rng.normal(_key(w, seed, _T_TARGET, s, row, extra), w.V)
    return tau, zd, zn


def _row(w: Workload, seed: int, kind: str, s: int, row: int, extra: int) -> np.ndarray:
    if w.logits == "gauss":
        tau, zd, zn = _gauss_pair(w, seed, s, row, extra)
        z = zd if kind == "draft" else w.rho * zd + np.sqrt(1.0 - w.rho * w.rho) * zn
        return (tau * z).astype(np.float32)
    if w.logits == "zipf":
        perm = rng.permutation(_key(w, seed, _T_PERM, s, row), w.V)
        tag = _T_DRAFT if kind == "draft" else _T_TARGET
        noise = rng.normal(_key(w, seed, tag, s, row, extra), w.V)
        x = np.empty(w.V, dtype=np.float32)
        x[perm] = (-w.zipf_s * np.log(np.arange(1, w.V + 1, dtype=np.float64))
                   + w.zipf_noise * noise).astype(np.float32)
        return x
    raise ValueError(w.logits)


def logits_row(w: Workload, seed: int, kind: str, s: int, row: int) -> np.ndarray:
    """One float32 row of draft ("draft") or target ("target") logits over the vocabulary.

    `row` identifies the tree node the row belongs to; a node's draft and target
    rows share what the recipe says they share (tau and the correlated part for
    "gauss", the rank permutation for "zipf").  With w.margin > 0 the node's two rows
    are redrawn together until the two largest logits of each differ by the margin.
    """
    assert kind in ("draft", "target")
    if w.margin <= 0.0:
        return _row(w, seed, kind, s, row, 0)
    for extra in range(64):
        xd = _row(w, seed, "draft", s, row, extra)
        xt = _row(w, seed, "target", s, row, extra)
        if _top2_gap(xd) >= w.margin and _top2_gap(xt) >= w.margin:
            return xd if kind == "draft" else xt
    raise RuntimeError("no draw met the argmax margin")


def logits_rows(w: Workload, seed: int, kind: str, s: int, rows) -> np.ndarray:
    rows = list(rows)
    out = np.empty((len(rows), w.V), dtype=np.float32)
    for i, r in enumerate(rows):
        out[i] = logits_row(w, seed, kind, s, int(r))
    return out


# ----------------------------------------------------------------------------- attention tensors
def _quantise(w: Workload, x: np.ndarray) -> np.ndarray:
    """Storage form: float32 as is; bf16 as uint16 bit patterns (rounded once, here)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return x if w.dtype == "f32" else rng.f32_to_bf16_bits(x)


def attention_inputs(w: Workload, seed: int, s: int, L: int, M: int, variant: str = "config",
                     parent: np.ndarray | None = None):
    """q [M,Hq,D], k_prefix/v_prefix [L,Hkv,D], k_tree/v_tree [M,Hkv,D] in storage form.

    variant "config": every element N(0,1)/sqrt(D), as the workloads state.
    variant "unit":   Q and K are N(0,1) (scores of order one after the 1/sqrt(D) scale).
    variant "peaky":  "unit", plus a few keys made to point along chosen queries so that a
                      handful of scores stand far above the rest; some planted keys are in
                      the last part of the prefix and some are tree rows (needs `parent`).
    variant "hot":    "peaky" with planted scores of 120, 135, 150, ... instead of 8: exp() of the
                      gap to the other scores overflows float32, so an implementation must track
                      the running maximum to get these rows right.
    variant "cold":   "unit", with the first keys of the prefix (up to 64) pointing away from two chosen
                      queries: scores of -150 there, so a running maximum that starts from those keys
                      starts hugely negative and every later score towers above it.
    variants "unit_v", "peaky_v": "unit" / "peaky" with V drawn N(0,1) as well, so that outputs are
                      of order one and an absolute tolerance of a few hundredths means something.
    """
    D = w.D
    v_unit = variant.endswith("_v")
    if v_unit:
        variant = variant[:-2]
    sc = 1.0 / np.sqrt(D) if variant == "config" else 1.0
    sv = 1.0 if v_unit else 1.0 / np.sqrt(D)
    q = rng.normal(_key(w, seed, _T_Q, s), M * w.Hq * D).reshape(M, w.Hq, D) * sc
    kp = rng.normal(_key(w, seed, _T_KP, s), L * w.Hkv * D).reshape(L, w.Hkv, D) * sc
    vp = rng.normal(_key(w, seed, _T_VP, s), L * w.Hkv * D).reshape(L, w.Hkv, D) * sv
    kt = rng.normal(_key(w, seed, _T_KT, s), M * w.Hkv * D).reshape(M, w.Hkv, D) * sc
    vt = rng.normal(_key(w, seed, _T_VT, s), M * w.Hkv * D).reshape(M, w.Hkv, D) * sv
    if variant in ("peaky", "hot") and M > 0:
        G = w.Hq // w.Hkv
        picks = rng.randint(_key(w, seed, _T_PLANT, s), 4 * 8, 0, 1 << 30).reshape(8, 4)
        for n, (a, b, c, d) in enumerate(picks):
            i, h = int(a) % M, int(b) % w.Hq
            g = h // G
            unit = q[i, h] / np.linalg.norm(q[i, h])
            score = 8.0 if variant == "peaky" else 120.0 + 15.0 * n
            amp = score * np.sqrt(D) / np.linalg.norm(q[i, h])  # score = |q| amp / sqrt(D)
            if int(c) % 2 == 0 and L > 0:
                j = L - 1 - (int(d) % max(1, min(L, 40)))          # near the end of the prefix
                kp[j, g] = unit * amp
            else:
                j = i
                steps = int(d) % 4
                while parent is not None and steps > 0 and parent[j] >= 0:
                    j = int(parent[j]); steps -= 1
                kt[j, g] = unit * amp                               # an ancestor (or the row itself)
    elif variant == "cold" and M > 0 and L > 0:
        G = w.Hq // w.Hkv
        picks = rng.randint(_key(w, seed, _T_PLANT, s), 2 * 2, 0, 1 << 30).reshape(2, 2)
        for a, b in picks:
            i, h = int(a) % M, int(b) % w.Hq
            unit = q[i, h] / np.linalg.norm(q[i, h])
            amp = 150.0 * np.sqrt(D) / np.linalg.norm(q[i, h])
            kp[:min(L, 64), h // G] = -unit * amp
    elif variant not in ("config", "unit", "peaky", "hot", "cold"):
        raise ValueError(variant)
    return tuple(_quantise(w, t) for t in (q, kp, vp, kt, vt))


# ----------------------------------------------------------------------------- tree recipes
def label_children(parent: np.ndarray, topk_idx: np.ndarray, topk_logp: np.ndarray, topk: int):
    """Tokens and log-confidences of a random-shape tree (workloads 1, 3, 4): child number r of a node (in
    row order) carries that node's r-th most likely draft token and its log-probability, as the Top-K
    results of every node's draft row list them.  Returns (token int32 [M], logc [M] in topk_logp's dtype)."""
    M = len(parent)
    token = np.full(M, -1, np.int32)
    logc = np.zeros(M, np.asarray(topk_logp).dtype)
    rank = {}
    for i in range(1, M):
        p = int(parent[i])
        k = rank.get(p, 0)
        rank[p] = k + 1
        assert k < topk, "fan-out exceeds K"
        token[i] = topk_idx[p, k]
        logc[i] = topk_logp[p, k]
    return token, logc


def batch_budgets(w: Workload, root_entropy):
    """(depth, node budget) per sequence of the batched workload from the Top-K entropies of the root
    rows: sequences are ranked by entropy (ties: lower sequence first); the lower the entropy, the deeper
    the draft and the smaller the verified set, in eight equal-count bins."""
    B = len(root_entropy)
    order = sorted(range(B), key=lambda s: (float(root_entropy[s]), s))
    depth, budget = [0] * B, [0] * B
    for rank, s in enumerate(order):
        b = rank * 8 // B
        depth[s] = max(2, w.max_depth - b)
        budget[s] = int(round(8 + (w.max_nodes - 8) * b / 7.0))
    return depth, budget


# ----------------------------------------------------------------------------- uniforms
def uniforms(w: Workload, seed: int, n: int, redraw: int = 0) -> np.ndarray:
    """n float32 uniforms in [0, 1) for the stochastic accept rule (node draws, then one per sequence)."""
    u = rng.uniform(_key(w, seed, _T_U, 0, 0, redraw), n).astype(np.float32)
    return np.minimum(u, np.float32(1.0 - 2.0 ** -24))
