"""One verification step of a synthetic workload on the GPU library.

Host-side glue only: it grows the draft tree by Top-K expansion (Section 2.2, Expansion) with
hs_draft_entropy_topk, keeps every input resident in device memory, and issues the four calls of
a step on the current stream.  All arithmetic of the step runs in libheterospec.so.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np
import torch

from synth import workloads as W
from . import binding as hs

INT_MAX = 2 ** 31 - 1


def _dev(x, dtype=None, device="cuda:0"):
    t = torch.from_numpy(np.ascontiguousarray(x))
    if dtype is not None:
        t = t.to(dtype)
    return t.to(device)


def _store(x, device):
    x = np.ascontiguousarray(x)
    if x.dtype == np.uint16:                           # bfloat16 bit patterns
        return torch.from_numpy(x.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(x).to(device)


def _in_parallel(fn, items, workers: int = 16):
    """The seeded input generators are pure functions of their key, and numpy releases the interpreter
    lock inside its array operations: the layers' / sequences' tensors are generated side by side."""
    from concurrent.futures import ThreadPoolExecutor
    items = list(items)
    if len(items) <= 1:
        return [fn(x) for x in items]
    with ThreadPoolExecutor(max_workers=min(workers, len(items))) as ex:
        return list(ex.map(fn, items))


def expand_tree(w: W.Workload, seed: int, s: int, depth: int, device="cuda:0"):
    """Top-K expansion with the library's own calls: per level the frontier's draft rows are quantified
    (hs_draft_entropy_topk) and the tree grows on the device (hs_tree_expand: children of the frontier,
    next frontier = the `frontier` new rows with the largest cumulative confidence).  The host only
    fetches the rows the next level asks for.  Returns the candidate tree (host arrays) and the expanded
    rows' logits (device, in expansion order)."""
    K, F = w.topk, w.frontier
    cap = 1 + K + max(0, depth - 1) * F * K
    state = hs.new_tree_state(1, cap, F, device)
    idx = torch.zeros((F, K), dtype=torch.int32, device=device)
    lp = torch.zeros((F, K), dtype=torch.float32, device=device)
    ent = torch.zeros(F, dtype=torch.float32, device=device)
    draft_ids: List[int] = []
    rows = []
    chosen = [0]
    for d in range(depth):
        x = _dev(W.logits_rows(w, seed, "draft", s, chosen), device=device)
        r = hs.hs_draft_entropy_topk(x, K, w.temperature, want_full=False)
        n = len(chosen)                       # the frontier's slots, in row order; the rest is unused
        idx[:n], lp[:n], ent[:n] = r["topk_idx"], r["topk_logp"], r["ent_topk"]
        hs.hs_tree_expand(state, idx, lp, ent, None, 1, cap, F, K, first=(d == 0))
        draft_ids += chosen
        rows.append(x)
        chosen = state["frontier"][:int(state["n_frontier"][0])].cpu().tolist()
    n = int(state["n_nodes"][0])
    return dict(parent=state["parent"][:n].cpu().numpy(), token=state["token"][:n].cpu().numpy(),
                logc=state["logc"][:n].cpu().numpy(), draft_ids=np.asarray(draft_ids, np.int64),
                rows=torch.cat(rows, dim=0))


def fixed_tree(w: W.Workload, seed: int, s: int, device="cuda:0"):
    """Random-shape tree: every node's draft row is quantified; the workload's recipe labels the nodes
    with their parents' Top-K tokens."""
    parent = W.tree_parents(w, seed, s)
    M = len(parent)
    x = _dev(W.logits_rows(w, seed, "draft", s, range(M)), device=device)
    r = hs.hs_draft_entropy_topk(x, w.topk, w.temperature, want_full=False)
    token, logc = W.label_children(parent, r["topk_idx"].cpu().numpy(), r["topk_logp"].cpu().numpy(), w.topk)
    return dict(parent=parent, token=token, logc=logc, draft_ids=np.arange(M), rows=x)


def sequence_budget(w: W.Workload, seed: int, device="cuda:0"):
    """(depth, node budget) per sequence of the batched workload, by the workload's recipe from the Top-K
    entropy of each root row (first term of Eq. 1)."""
    x = _dev(np.concatenate([W.logits_rows(w, seed, "draft", s, [0]) for s in range(w.B)]), device=device)
    ent = hs.hs_draft_entropy_topk(x, w.topk, w.temperature, want_full=False)["ent_topk"].cpu().numpy()
    return W.batch_budgets(w, ent)


@dataclass
class Step:
    """Device-resident inputs, outputs and workspaces of one verification step."""
    w: W.Workload
    layers: int
    accept_mode: int
    t: Dict[str, torch.Tensor] = field(default_factory=dict)
    host: Dict[str, object] = field(default_factory=dict)
    sets: List[Dict[str, torch.Tensor]] = field(default_factory=list)   # rotating copies of the logits (see rotate_logits)
    k: int = 0                                                          # steps run so far

    def rotate_logits(self, min_bytes: float = 320e6) -> int:
        """Makes enough copies of the step's logits arrays (draft rows, target rows, draft rows of the kept
        nodes) that a run of steps, each reading the next copy, streams them from HBM instead of finding
        the previous step's rows in the 256 MB last-level cache.  Returns the number of copies in use."""
        names = [n for n in ("draft_rows", "target_logits", "draft_logits") if n in self.t]
        per_set = sum(self.t[n].numel() * 4 for n in names)
        n_sets = max(1, min(8, int(-(-min_bytes // per_set))))
        self.sets = [{n: self.t[n] for n in names}] + [{n: self.t[n].clone() for n in names} for _ in range(n_sets - 1)]
        return n_sets

    def _logits(self, name):
        return self.sets[self.k % len(self.sets)][name] if self.sets else self.t[name]

    # ---- the four stages, each one C call
    def stage1(self):
        # (one launch: the workspace was prepared when the step was built and only this call uses it)
        return hs.hs_draft_entropy_topk(self._logits("draft_rows"), self.w.topk, self.w.temperature,
                                        out=self.t["s1_out"], ws=self.t["s1_ws"], fused=True)

    def stage2(self):
        return hs.hs_tree_prune(self.t["cand_parent"], self.t["cand_logc"], self.t["cand_offsets"],
                                self.t["d_max"], self.t["theta"], self.t["max_nodes"],
                                out=self.t["s2_out"], ws=self.t["s2_ws"])

    def stage3(self):
        t, h = self.t, self.host
        if self.layers > 1:
            # every layer verifies the tree that stage 2 has just left on the device
            return hs.hs_tree_attention(t["q"], t["k_prefix"], t["v_prefix"], t["k_tree"], t["v_tree"],
                                        t["s2_out"]["out_parent"], t["attn_node_offsets"], t["attn_prefix_offsets"],
                                        h["attn_node_offsets"], h["attn_prefix_offsets"], h["scale"],
                                        out=t["o"], ws=t["s3_ws"], shared_tree=True)
        return hs.hs_tree_attention(t["q"], t["k_prefix"], t["v_prefix"], t["k_tree"], t["v_tree"],
                                    t["attn_parent"], t["attn_node_offsets"], t["attn_prefix_offsets"],
                                    h["attn_node_offsets"], h["attn_prefix_offsets"], h["scale"],
                                    out=t["o"], ws=t["s3_ws"])

    def stage4(self):
        t, h = self.t, self.host
        r = hs.hs_verify_accept(self._logits("target_logits"),
                                self._logits("draft_logits") if self.accept_mode == 1 else None,
                                t["token"], t["s2_out"]["out_parent"], t["s2_out"]["out_offsets"],
                                self.accept_mode, self.w.temperature,
                                t["uniforms"] if self.accept_mode != 0 else None, h["max_depth"],
                                out=t["s4_out"], ws=t["s4_ws"])
        self.k += 1          # the step is complete: the next one reads the next copy of the logits
        return r

    def run(self):
        self.stage1()
        self.stage2()
        self.stage3()
        self.stage4()

    # ---- algorithmic bytes (what the step has to move at least once)
    def bytes_stage1(self) -> int:
        return int(self.t["draft_rows"].numel()) * 4

    def bytes_stage3(self) -> int:
        h, w = self.host, self.w
        es = 4 if w.dtype == "f32" else 2
        total = 0
        for s in range(len(h["attn_node_offsets"]) - 1):
            M = int(h["attn_node_offsets"][s + 1] - h["attn_node_offsets"][s])
            L = int(h["attn_prefix_offsets"][s + 1] - h["attn_prefix_offsets"][s])
            total += (2 * (L + M) * w.Hkv * w.D + 2 * M * w.Hq * w.D) * es
        return total

    def flops_stage3(self) -> int:
        """Multiply-adds of both products times two: every row meets its prefix and its root path."""
        h, w = self.host, self.w
        no, po = h["attn_node_offsets"].numpy(), h["attn_prefix_offsets"].numpy()
        par = self.t["attn_parent"].cpu().numpy()
        total = 0
        for s in range(len(no) - 1):
            n0, M, L = int(no[s]), int(no[s + 1] - no[s]), int(po[s + 1] - po[s])
            depth = np.zeros(M, np.int64)
            for i in range(1, M):
                depth[i] = depth[par[n0 + i]] + 1
            total += 4 * w.Hq * w.D * int((L + depth + 1).sum())
        return total

    def bytes_stage4(self) -> int:
        n = int(self.t["target_logits"].numel()) * 4
        return n * (2 if self.accept_mode == 1 else 1)


def build_step(w: W.Workload, seed: int = 0, layers: Optional[int] = None, accept_mode: int = 0,
               theta: Optional[float] = None, device="cuda:0") -> Step:
    """Generates the workload's inputs, grows and prunes its trees with the library, and lays out
    everything a timed step needs in device memory.  With layers > 1 (single-sequence workloads) the
    attention stage covers that many decoder layers at once: each layer has its own Q and K/V cache
    and is passed as one entry of the batch, all sharing the step's pruned tree."""
    layers = layers or 1
    if layers > 1 and w.B != 1:
        raise ValueError("layer replication is for single-sequence workloads")
    B = w.B
    theta = w.theta[0] if theta is None else theta
    budget = sequence_budget(w, seed, device) if (w.tree == "expand" and B > 1) else None
    trees = []
    for s in range(B):
        if w.tree == "expand":
            trees.append(expand_tree(w, seed, s, budget[0][s] if budget else w.max_depth, device))
        else:
            trees.append(fixed_tree(w, seed, s, device))
    st = Step(w=w, layers=layers, accept_mode=accept_mode)
    t, h = st.t, st.host
    # stage 1: every expanded row of the step in one call
    t["draft_rows"] = torch.cat([tr["rows"] for tr in trees], dim=0).contiguous()
    R = t["draft_rows"].shape[0]
    t["s1_out"] = dict(topk_idx=torch.empty((R, w.topk), dtype=torch.int32, device=device),
                       topk_logp=torch.empty((R, w.topk), dtype=torch.float32, device=device),
                       ent_topk=torch.empty(R, dtype=torch.float32, device=device),
                       ent_full=torch.empty(R, dtype=torch.float32, device=device),
                       lse=torch.empty(R, dtype=torch.float32, device=device))
    t["s1_ws"] = hs.workspace(hs.lib().hs_draft_entropy_topk_workspace(R, w.V, w.topk), device)
    hs.hs_workspace_prepare(t["s1_ws"])
    # stage 2
    cand_off = np.zeros(B + 1, np.int32)
    cand_off[1:] = np.cumsum([len(tr["parent"]) for tr in trees])
    NNc = int(cand_off[-1])
    t["cand_parent"] = _dev(np.concatenate([tr["parent"] for tr in trees]), torch.int32, device)
    t["cand_logc"] = _dev(np.concatenate([tr["logc"] for tr in trees]), torch.float32, device)
    t["cand_offsets"] = _dev(cand_off, torch.int32, device)
    t["d_max"] = _dev(np.asarray([(budget[0][s] if budget else w.max_depth) for s in range(B)]), torch.int32, device)
    t["theta"] = _dev(np.full(B, theta), torch.float32, device)
    t["max_nodes"] = _dev(np.asarray([(budget[1][s] if budget else w.max_nodes) for s in range(B)]), torch.int32, device)
    t["s2_out"] = dict(depth=torch.empty(NNc, dtype=torch.int32, device=device),
                       cumlogp=torch.empty(NNc, dtype=torch.float32, device=device),
                       keep=torch.empty(NNc, dtype=torch.uint8, device=device),
                       out_offsets=torch.empty(B + 1, dtype=torch.int32, device=device),
                       out_src=torch.empty(NNc, dtype=torch.int32, device=device),
                       out_parent=torch.empty(NNc, dtype=torch.int32, device=device))
    t["s2_ws"] = hs.workspace(hs.lib().hs_tree_prune_workspace(B, NNc), device)
    st.stage2()
    torch.cuda.synchronize()
    oo = t["s2_out"]["out_offsets"].cpu().numpy()
    NNp = int(oo[-1])
    src = t["s2_out"]["out_src"][:NNp].cpu().numpy()
    par = t["s2_out"]["out_parent"][:NNp].cpu().numpy()
    h.update(NNp=NNp, cand_nodes=NNc, out_offsets=oo, out_src=src, out_parent=par,
             kept_draft_nodes=NNp - int((np.diff(oo) > 0).sum()))
    depth = np.zeros(NNp, np.int32)
    for s in range(B):
        for i in range(int(oo[s]) + 1, int(oo[s + 1])):
            depth[i] = depth[int(oo[s]) + par[i]] + 1
    h["max_depth"] = max(1, int(depth.max()) if NNp else 1)
    # stage 4 inputs: target rows of the kept nodes, draft rows where the node was expanded
    token = np.concatenate([trees[s]["token"][src[oo[s]:oo[s + 1]]] for s in range(B)]).astype(np.int32)
    t["token"] = _dev(token, torch.int32, device)
    t["target_logits"] = torch.empty((NNp, w.V), dtype=torch.float32, device=device)
    for s in range(B):
        for i0 in range(int(oo[s]), int(oo[s + 1]), 64):
            i1 = min(i0 + 64, int(oo[s + 1]))
            t["target_logits"][i0:i1] = _dev(W.logits_rows(w, seed, "target", s, src[i0:i1]), device=device)
    if accept_mode == 1:
        t["draft_logits"] = torch.zeros((NNp, w.V), dtype=torch.float32, device=device)
        row0 = 0
        for s in range(B):
            pos = {int(c): j for j, c in enumerate(trees[s]["draft_ids"])}
            for j, c in enumerate(src[oo[s]:oo[s + 1]]):
                if int(c) in pos:
                    t["draft_logits"][int(oo[s]) + j] = t["draft_rows"][row0 + pos[int(c)]]
            row0 += len(trees[s]["draft_ids"])
    t["uniforms"] = _dev(W.uniforms(w, seed, NNp + B), torch.float32, device)
    t["s4_out"] = dict(accept_len=torch.empty(B, dtype=torch.int32, device=device),
                       accept_path=torch.empty((B, h["max_depth"]), dtype=torch.int32, device=device),
                       bonus_token=torch.empty(B, dtype=torch.int32, device=device))
    t["s4_ws"] = hs.workspace(hs.lib().hs_verify_accept_workspace_mode(B, NNp, w.V, accept_mode), device)
    # stage 3 inputs
    L = W.prefix_lengths(w, seed)
    if layers > 1:
        M = NNp
        parts = _in_parallel(lambda l: W.attention_inputs(w, seed, 1000 + l, int(L[0]), M, "config", parent=par),
                             range(layers))
        no = (np.arange(layers + 1) * M).astype(np.int32)
        po = (np.arange(layers + 1) * int(L[0])).astype(np.int64)
        t["attn_parent"] = _dev(np.tile(par, layers), torch.int32, device)
    else:
        parts = _in_parallel(lambda s: W.attention_inputs(w, seed, s, int(L[s]), int(oo[s + 1] - oo[s]), "config",
                                                          parent=par[oo[s]:oo[s + 1]]), range(B))
        no = oo.astype(np.int32)
        po = np.zeros(B + 1, np.int64)
        po[1:] = np.cumsum(L)
        t["attn_parent"] = t["s2_out"]["out_parent"]
    for i, name in enumerate(("q", "k_prefix", "v_prefix", "k_tree", "v_tree")):
        t[name] = torch.cat([_store(p[i], device) for p in parts], dim=0).contiguous()
    t["attn_node_offsets"] = _dev(no, torch.int32, device) if layers > 1 else t["s2_out"]["out_offsets"]
    t["attn_prefix_offsets"] = _dev(po, torch.int64, device)
    h.update(attn_node_offsets=torch.from_numpy(no.copy()), attn_prefix_offsets=torch.from_numpy(po.copy()),
             scale=1.0 / float(np.sqrt(w.D)))
    t["o"] = torch.empty_like(t["q"])
    nb = len(no) - 1
    t["s3_ws"] = hs.workspace(hs.lib().hs_tree_attention_workspace(
        nb, int(no[-1]), int(po[-1]), w.Hq, w.Hkv, w.D, hs.HS_F32 if w.dtype == "f32" else hs.HS_BF16), device)
    return st


# ------------------------------------------------------------------------------------------------
# The adaptive step, device-driven: Top-K growth level by level (hs_tree_expand), complexity
# quantification and decision (hs_adaptive_control), extended drafting, pruning to the decided
# budget, verification.  The host reads one number per step, the entropy bin, and replays the HIP
# graph specialised for that bin (Section 4.3, Dynamic Computational Adaptation: one cached
# computation graph per complexity region).
@dataclass
class AdaptiveStep:
    w: W.Workload
    layers: int
    d_base: int
    alpha: int
    n_default: int
    edges: List[float]
    gamma: List[float]
    pstar_mode: int = 0
    t: Dict[str, object] = field(default_factory=dict)
    host: Dict[str, object] = field(default_factory=dict)
    graphs: Dict[object, object] = field(default_factory=dict)

    # ---- what a bin means (Section 4.3): asked of the library, which holds the formula
    def decision(self, b: int):
        return hs.hs_adaptive_policy(b, self.gamma, self.alpha, self.d_base, self.n_default)

    def set_temperature(self, T: float):
        """Swaps the draft model's output rows for those of draft temperature T (a power of two, so that
        the scaling is exact): softmax(x / T) of the stored rows is what the drafting calls then see,
        with their own temperature argument, which a captured graph has baked in, left at the
        workload's.  Stands in for the next step's draft distributions."""
        m, e = np.frexp(T)
        if m != 0.5 or T <= 0:
            raise ValueError("T must be a power of two")
        t = self.t
        torch.mul(t["draft_base"], 1.0 / T, out=t["draft_all"])
        t["x_root"].copy_(t["draft_all"][:1].expand_as(t["x_root"]))

    # ---- pieces, each a few library calls on device-resident data
    def _level(self, first: bool):
        t, w, h = self.t, self.w, self.host
        # The draft model's pass over the frontier is not part of this build: its logits rows exist for
        # all candidates beforehand, and the scan reads the frontier's rows where they lie.
        if first:
            r = hs.hs_draft_entropy_topk(t["x_root"], w.topk, w.temperature, out=t["s1_out"], ws=t["s1_ws"], fused=True)
        else:
            r = hs.hs_draft_entropy_topk(t["draft_all"], w.topk, w.temperature, out=t["s1_out"], ws=t["s1_ws"],
                                         row_index=t["state"]["frontier_rows"], fused=True)
        hs.hs_tree_expand(t["state"], r["topk_idx"], r["topk_logp"], r["ent_topk"], None, 1, h["cap"], w.frontier,
                          w.topk, first=first)

    def run_draft(self):
        """Base drafting to d_base levels, then the complexity decision (device only)."""
        t, h = self.t, self.host
        for lvl in range(self.d_base):
            self._level(lvl == 0)
        st = t["state"]
        hs.hs_adaptive_control(st["parent"], st["logc"], st["ent"], st["node_offsets"], st["n_nodes"], self.edges,
                               self.gamma, self.alpha, self.d_base, self.n_default, self.pstar_mode, out=t["ctl"])

    def run_verify(self, b: int):
        """Extended drafting for bin b, pruning to the decided budget, attention on all layers, accept."""
        t, h, w = self.t, self.host, self.w
        d_prime, n_prime = self.decision(b)
        for _ in range(d_prime - self.d_base):
            self._level(False)
        st, ctl = t["state"], t["ctl"]
        hs.hs_tree_prune(st["parent"], st["logc"], st["node_offsets"], ctl["d_prime"], t["theta"], ctl["n_prime"],
                         node_counts=st["n_nodes"], out=t["s2_out"], ws=t["s2_ws"])
        M = n_prime + 1
        a = t["attn"][M]
        src = t["s2_out"]["out_src"][:M]
        par = t["s2_out"]["out_parent"][:M]
        hs.hs_tree_attention(a["q"], t["k_prefix"], t["v_prefix"], a["k_tree"], a["v_tree"], par,
                             a["node_offsets"], t["prefix_offsets"], a["host_node_offsets"], h["prefix_offsets"],
                             h["scale"], out=a["o"], ws=a["ws"], shared_tree=True)
        # stands in for the target model's output rows of the kept nodes
        torch.index_select(st["token"], 0, src, out=a["token"])
        torch.index_select(t["target_all"], 0, src, out=a["target"])
        hs.hs_verify_accept(a["target"], None, a["token"], par, t["s2_out"]["out_offsets"], 0, w.temperature, None,
                            d_prime, out=a["s4_out"], ws=a["s4_ws"])

    def read_bin(self) -> int:
        return int(self.t["ctl"]["bin"].cpu()[0])

    # ---- HIP graphs: one for the drafting part, one per bin for the rest
    def capture(self, bins=None):
        pool = None
        self.run_draft()
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            self.run_draft()
        self.graphs["draft"] = g
        for b in (bins if bins is not None else range(len(self.edges) + 1)):
            key = self.decision(b)
            if key in self.graphs:
                self.graphs[b] = self.graphs[key]
                continue
            self.run_draft()
            self.run_verify(b)
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                self.run_verify(b)
            self.graphs[key] = self.graphs[b] = g

    def step_eager(self) -> int:
        self.run_draft()
        b = self.read_bin()
        self.run_verify(b)
        return b

    def step_graph(self) -> int:
        self.graphs["draft"].replay()
        b = self.read_bin()
        self.graphs[b].replay()
        return b

    def result(self, b: int):
        torch.cuda.synchronize()
        ctl = self.t["ctl"]
        d_prime, n_prime = int(ctl["d_prime"].cpu()[0]), int(ctl["n_prime"].cpu()[0])   # the device's decision
        a = self.t["attn"][n_prime + 1]
        return dict(bin=b, d_prime=d_prime, n_prime=n_prime,
                    accept_len=int(a["s4_out"]["accept_len"].cpu()[0]),
                    bonus_token=int(a["s4_out"]["bonus_token"].cpu()[0]))


def build_adaptive(w: W.Workload, seed: int = 0, layers: Optional[int] = None, edges=None, gamma=(0.3, 0.6, 1.0),
                   alpha: Optional[int] = None, device="cuda:0", pstar_mode: int = 0) -> AdaptiveStep:
    """Single-sequence workloads grown by Top-K expansion (the 8B shape).  edges: the seven bin
    boundaries of the eight entropy bins (synthetic: the paper prints none)."""
    if w.B != 1 or w.tree != "expand":
        raise ValueError("the adaptive step is built for single-sequence Top-K expansion workloads")
    layers = layers or 1
    d_base, K, F = w.max_depth, w.topk, w.frontier
    alpha = alpha if alpha is not None else -(-d_base // 2)          # ceil(depth / 2), Section 5
    edges = list(edges) if edges is not None else [0.5 * d_base * x for x in (0.2, 0.4, 0.6, 0.8, 1.0, 1.3, 1.7)]
    st = AdaptiveStep(w=w, layers=layers, d_base=d_base, alpha=alpha, n_default=w.max_nodes, edges=edges,
                      gamma=list(gamma), pstar_mode=pstar_mode)
    t, h = st.t, st.host
    cap = 1 + K + (d_base + alpha - 1) * F * K
    h.update(cap=cap, scale=1.0 / float(np.sqrt(w.D)))
    i32 = dict(dtype=torch.int32, device=device)
    # the draft and target rows of every possible candidate (row = candidate index)
    t["draft_all"] = torch.empty((cap, w.V), dtype=torch.float32, device=device)
    t["target_all"] = torch.empty((cap, w.V), dtype=torch.float32, device=device)
    for i0 in range(0, cap, 64):
        ids = range(i0, min(i0 + 64, cap))
        t["draft_all"][i0:i0 + len(ids)] = _dev(W.logits_rows(w, seed, "draft", 0, ids), device=device)
        t["target_all"][i0:i0 + len(ids)] = _dev(W.logits_rows(w, seed, "target", 0, ids), device=device)
    t["draft_base"] = t["draft_all"].clone()          # the rows as generated (set_temperature rescales from them)
    t["x_root"] = t["draft_all"][:1].repeat(F, 1).contiguous()
    t["s1_out"] = dict(topk_idx=torch.empty((F, K), **i32),
                       topk_logp=torch.empty((F, K), dtype=torch.float32, device=device),
                       ent_topk=torch.empty(F, dtype=torch.float32, device=device))
    t["s1_ws"] = hs.workspace(hs.lib().hs_draft_entropy_topk_workspace(F, w.V, K), device)
    hs.hs_workspace_prepare(t["s1_ws"])          # (the level loop's scans run in one launch each from here on)
    t["state"] = hs.new_tree_state(1, cap, F, device)
    t["ctl"] = dict(phi=torch.empty(1, dtype=torch.float32, device=device))
    for k in ("pstar", "bin", "d_prime", "n_prime"):
        t["ctl"][k] = torch.empty(1, **i32)
    t["theta"] = _dev(np.full(1, w.theta[0]), torch.float32, device)
    t["s2_out"] = dict(depth=torch.empty(cap, **i32), cumlogp=torch.empty(cap, dtype=torch.float32, device=device),
                       keep=torch.empty(cap, dtype=torch.uint8, device=device), out_offsets=torch.empty(2, **i32),
                       out_src=torch.empty(cap, **i32), out_parent=torch.empty(cap, **i32))
    t["s2_ws"] = hs.workspace(hs.lib().hs_tree_prune_workspace(1, cap), device)
    # attention: the prefix caches of all layers are shared by the bins; Q and the tree K/V depend
    # on the number of verified rows
    L = int(W.prefix_lengths(w, seed)[0])
    sizes = sorted({st.decision(b)[1] + 1 for b in range(len(edges) + 1)})
    kp, vp = [], []
    for l in range(layers):
        _, a, b_, _, _ = W.attention_inputs(w, seed, 1000 + l, L, 1, "config")
        kp.append(_store(a, device))
        vp.append(_store(b_, device))
    t["k_prefix"], t["v_prefix"] = torch.cat(kp, dim=0).contiguous(), torch.cat(vp, dim=0).contiguous()
    po = (np.arange(layers + 1) * L).astype(np.int64)
    t["prefix_offsets"] = _dev(po, torch.int64, device)
    h["prefix_offsets"] = torch.from_numpy(po.copy())
    dt = hs.HS_F32 if w.dtype == "f32" else hs.HS_BF16
    t["attn"] = {}
    for M in sizes:
        parts = [W.attention_inputs(w, seed, 2000 + l, 0, M, "config") for l in range(layers)]
        no = (np.arange(layers + 1) * M).astype(np.int32)
        a = dict(q=torch.cat([_store(p[0], device) for p in parts], dim=0).contiguous(),
                 k_tree=torch.cat([_store(p[3], device) for p in parts], dim=0).contiguous(),
                 v_tree=torch.cat([_store(p[4], device) for p in parts], dim=0).contiguous(),
                 node_offsets=_dev(no, torch.int32, device),
                 host_node_offsets=torch.from_numpy(no.copy()), token=torch.empty(M, **i32),
                 target=torch.empty((M, w.V), dtype=torch.float32, device=device))
        a["o"] = torch.empty_like(a["q"])
        a["ws"] = hs.workspace(hs.lib().hs_tree_attention_workspace(layers, layers * M, int(po[-1]), w.Hq, w.Hkv, w.D,
                                                                   dt), device)
        a["s4_out"] = dict(accept_len=torch.empty(1, **i32), bonus_token=torch.empty(1, **i32),
                           accept_path=torch.empty((1, d_base + alpha), **i32))
        a["s4_ws"] = hs.workspace(hs.lib().hs_verify_accept_workspace_mode(1, M, w.V, 0), device)
        t["attn"][M] = a
    h["sizes"] = sizes
    return st
