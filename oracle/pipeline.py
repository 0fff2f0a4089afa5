"""One verification step of a synthetic workload, stage by stage, with the CPU checker.

Builds the inputs of each of the four stages from the seeded raw inputs and the
checker's own results for the stage before, and keeps both, so a test can feed
any stage of the GPU library the same bytes and compare.  The tree of an
"expand" workload is grown as Section 2.2 (Expansion) describes: every depth,
the most promising nodes by cumulative confidence are expanded with their
Top-K draft tokens.  Test infrastructure only.
"""
from __future__ import annotations

import numpy as np

from synth import workloads as W
from . import draft_entropy_topk, tree_prune, tree_attention, verify_accept
from .verify_accept import GREEDY, STOCHASTIC, STOCHASTIC_POINTMASS

NEG_INF = float("-inf")
INT_MAX = 2 ** 31 - 1


def expand_tree(w, seed, s, depth, frontier=None, K=None, quantify=draft_entropy_topk):
    """Top-K expansion to `depth` levels.  Returns dict(parent, token, logc (f64), ent_topk per
    expanded row, draft_ids (candidate id of each expanded row, in order), rows (float32 logits
    of those rows), stage1 (the checker's outputs for `rows`))."""
    K = K or w.topk
    frontier = frontier or w.frontier
    parent, token, logc, cum, dep = [-1], [-1], [0.0], [0.0], [0]
    draft_ids, rows, res = [], [], []
    level = [0]
    for d in range(depth):
        # the nodes of this depth with the largest cumulative confidence are expanded
        chosen = sorted(level, key=lambda i: (-cum[i], i))[:frontier]
        chosen.sort()
        x = W.logits_rows(w, seed, "draft", s, chosen)
        r = quantify(x, K, w.temperature)
        nxt = []
        for j, i in enumerate(chosen):
            draft_ids.append(i)
            for k in range(K):
                parent.append(i)
                token.append(int(r["topk_idx"][j, k]))
                logc.append(float(r["topk_logp"][j, k]))
                cum.append(cum[i] + min(float(r["topk_logp"][j, k]), 0.0))
                dep.append(d + 1)
                nxt.append(len(parent) - 1)
        rows.append(x)
        res.append(r)
        level = nxt
    stage1 = {k: np.concatenate([r[k] for r in res], axis=0) for k in res[0]}
    return dict(parent=np.asarray(parent, np.int32), token=np.asarray(token, np.int32),
                logc=np.asarray(logc, np.float64), draft_ids=np.asarray(draft_ids, np.int64),
                rows=np.concatenate(rows, axis=0), stage1=stage1)


def fixed_tree(w, seed, s, quantify=draft_entropy_topk):
    """A random-shape tree: every node's draft row is quantified at once; child number r of a
    node carries that node's r-th most likely draft token and its log-probability."""
    parent = W.tree_parents(w, seed, s)
    M = len(parent)
    x = W.logits_rows(w, seed, "draft", s, range(M))
    r = quantify(x, w.topk, w.temperature)
    token, logc = W.label_children(parent, r["topk_idx"], np.asarray(r["topk_logp"], np.float64), w.topk)
    return dict(parent=parent, token=token, logc=logc, draft_ids=np.arange(M), rows=x, stage1=r)


def sequence_budget(w, seed, B):
    """Per-sequence (depth, node budget) of the batched workload: sequences are ranked by the
    Top-K entropy of their root row (the first term of Eq. 1); the lower the entropy, the deeper
    the draft and the smaller the verified set, in eight equal-count bins."""
    ent = []
    for s in range(B):
        x = W.logits_rows(w, seed, "draft", s, [0])
        ent.append(float(draft_entropy_topk(x, w.topk, w.temperature)["ent_topk"][0]))
    return W.batch_budgets(w, ent)


def build_step(w, seed, theta=None, with_attention=True, variant="config", depth_budget=None):
    """All four stages' inputs and the checker's outputs for one step of workload w."""
    B = w.B
    theta = w.theta[0] if theta is None else theta
    if w.tree == "expand" and B > 1 and depth_budget is None:
        depth_budget = sequence_budget(w, seed, B)
    trees = []
    for s in range(B):
        if w.tree == "expand":
            d = depth_budget[0][s] if depth_budget else w.max_depth
            trees.append(expand_tree(w, seed, s, d))
        else:
            trees.append(fixed_tree(w, seed, s))
    # ---- stage 2 inputs: packed candidate trees
    node_offsets = np.zeros(B + 1, np.int32)
    node_offsets[1:] = np.cumsum([len(t["parent"]) for t in trees])
    parent = np.concatenate([t["parent"] for t in trees])
    logc = np.concatenate([t["logc"] for t in trees]).astype(np.float32)
    token = np.concatenate([t["token"] for t in trees])
    d_max = np.asarray([(depth_budget[0][s] if depth_budget else w.max_depth) for s in range(B)], np.int32)
    thetas = np.full(B, theta, np.float32)
    budget = np.asarray([(depth_budget[1][s] if depth_budget else w.max_nodes) for s in range(B)], np.int32)
    pr = tree_prune(parent, logc, node_offsets, d_max, thetas, budget)
    step = dict(w=w, seed=seed, trees=trees,
                prune_in=dict(parent=parent, logc=logc, node_offsets=node_offsets, d_max=d_max,
                              theta=thetas, max_nodes=budget),
                prune_out=pr, cand_token=token)
    # ---- pruned tree
    oo = pr["out_offsets"]
    ptoken = np.concatenate([token[node_offsets[s]:node_offsets[s + 1]][pr["out_src"][oo[s]:oo[s + 1]]]
                             for s in range(B)])
    step.update(node_offsets=oo.copy(), parent=pr["out_parent"].copy(), token=ptoken.astype(np.int32))
    NN = int(oo[-1])
    # ---- stage 4 inputs: logits rows of the kept nodes
    tgt = np.empty((NN, w.V), np.float32)
    drf = np.zeros((NN, w.V), np.float32)
    for s in range(B):
        src = pr["out_src"][oo[s]:oo[s + 1]]
        tgt[oo[s]:oo[s + 1]] = W.logits_rows(w, seed, "target", s, src)
        t = trees[s]
        pos = {int(c): j for j, c in enumerate(t["draft_ids"])}
        for j, c in enumerate(src):
            if int(c) in pos:
                drf[oo[s] + j] = t["rows"][pos[int(c)]]
    step.update(target_logits=tgt, draft_logits=drf)
    # ---- stage 3 inputs
    if with_attention:
        L = W.prefix_lengths(w, seed)
        prefix_offsets = np.zeros(B + 1, np.int64)
        prefix_offsets[1:] = np.cumsum(L)
        parts = [W.attention_inputs(w, seed, s, int(L[s]), int(oo[s + 1] - oo[s]), variant,
                                    parent=step["parent"][oo[s]:oo[s + 1]]) for s in range(B)]
        q, kp, vp, kt, vt = (np.concatenate([p[i] for p in parts], axis=0) for i in range(5))
        step.update(q=q, k_prefix=kp, v_prefix=vp, k_tree=kt, v_tree=vt, prefix_offsets=prefix_offsets,
                    scale=1.0 / np.sqrt(w.D))
    return step


def attention_out(step):
    return tree_attention(step["q"], step["k_prefix"], step["v_prefix"], step["k_tree"], step["v_tree"],
                          step["parent"], step["node_offsets"], step["prefix_offsets"], step["scale"])


def tree_depth(parent, node_offsets):
    d = np.zeros(len(parent), np.int32)
    for s in range(len(node_offsets) - 1):
        o = int(node_offsets[s])
        for i in range(1, int(node_offsets[s + 1]) - o):
            d[o + i] = d[o + int(parent[o + i])] + 1
    return d


def accept_out(step, mode, uniforms=None, max_depth=None):
    w = step["w"]
    max_depth = max_depth or max(1, int(tree_depth(step["parent"], step["node_offsets"]).max()))
    return verify_accept(step["target_logits"], step["draft_logits"], step["token"], step["parent"],
                         step["node_offsets"], mode, w.temperature, uniforms, max_depth)


# ----------------------------------------------------------------------------- margins
def prune_margin(step):
    """Smallest distance of any candidate's cumulative log-probability to its threshold, and the
    smallest gap across the node-budget cut; float32 and float64 confidences then give the same
    kept set as long as their cumulative difference stays below this."""
    pin, po = step["prune_in"], step["prune_out"]
    gap = np.inf
    offs = pin["node_offsets"]
    for s in range(len(offs) - 1):
        S = po["cumlogp"][offs[s]:offs[s + 1]].astype(np.float64)
        keep = po["keep"][offs[s]:offs[s + 1]].astype(bool)
        th = float(pin["theta"][s])
        if np.isfinite(th):
            gap = min(gap, float(np.abs(S[1:] - th).min()) if len(S) > 1 else np.inf)
        if pin["max_nodes"][s] > 0 and keep[1:].sum() == pin["max_nodes"][s] and (~keep[1:]).any():
            lo = S[1:][keep[1:]].min()
            dropped = S[1:][~keep[1:]]
            dropped = dropped[dropped <= lo]
            if len(dropped):
                gap = min(gap, float(lo - dropped.max()))
    return gap


def safe_uniforms(step, mode, rel=1e-4, cdf_abs=1e-5, tries=64):
    """Uniforms for which every accept test on the walked path is at least `rel` (relative) away
    from its threshold and the bonus draw at least `cdf_abs` from a step of the distribution
    function, so float32 and float64 arithmetic take the same decisions.  Returns (uniforms,
    result of the walk)."""
    w = step["w"]
    NN, B = int(step["node_offsets"][-1]), len(step["node_offsets"]) - 1
    for redraw in range(tries):
        u = W.uniforms(w, step["seed"], NN + B, redraw)
        base = accept_out(step, mode, u)
        ok = True
        for sgn in (-1.0, 1.0):
            un = u.astype(np.float64).copy()
            un[:NN] = un[:NN] * (1.0 + sgn * rel)
            un[NN:] = np.clip(un[NN:] + sgn * cdf_abs, 0.0, 1.0 - 1e-12)
            alt = accept_out(step, mode, un)
            ok = ok and all(np.array_equal(alt[k], base[k]) for k in base)
        if ok:
            return u, base
    raise RuntimeError("no margin-safe uniforms found")


# ----------------------------------------------------------------------------- the adaptive step
def adaptive_step(w, seed, edges, gamma, alpha, logp_dtype=np.float32, pstar_mode=0):
    """The whole adaptive step of a single-sequence expansion workload with the checker: base
    drafting to w.max_depth levels, complexity decision, extended drafting, pruning to the decided
    budget, greedy accept walk (Sections 4.1 - 4.3 around the Section 2.2 tree).  Confidences are
    rounded to `logp_dtype` before they enter the tree, as the library's are."""
    from .tree_expand import new_state, tree_expand
    from .adaptive_control import adaptive_control
    K, F, d_base = w.topk, w.frontier, w.max_depth
    cap = 1 + K + (d_base + alpha - 1) * F * K
    st = new_state()

    def level():
        x = W.logits_rows(w, seed, "draft", 0, st["frontier"])
        r = draft_entropy_topk(x, K, w.temperature)
        tree_expand(st, r["topk_idx"], r["topk_logp"].astype(logp_dtype), r["ent_topk"].astype(np.float32), F, cap)

    for _ in range(d_base):
        level()
    n = len(st["parent"])
    ctl = adaptive_control(st["parent"], st["logc"], st["ent"], [0, n], edges, gamma, alpha, d_base, w.max_nodes, pstar_mode)
    d_prime, n_prime = int(ctl["d_prime"][0]), int(ctl["n_prime"][0])
    for _ in range(d_prime - d_base):
        level()
    n = len(st["parent"])
    pr = tree_prune(np.asarray(st["parent"], np.int32), np.asarray(st["logc"], np.float32), [0, n], [d_prime],
                    [w.theta[0]], [n_prime])
    src = pr["out_src"]
    token = np.asarray(st["token"], np.int32)[src]
    tgt = W.logits_rows(w, seed, "target", 0, src)
    acc = verify_accept(tgt, None, token, pr["out_parent"], pr["out_offsets"], GREEDY, w.temperature, None, d_prime)
    return dict(state=st, control=ctl, prune=pr, token=token, accept=acc)
