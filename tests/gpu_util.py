"""Helpers for the GPU parity tests: numpy <-> device tensors and the four calls on a step."""
import numpy as np
import torch

import paper_2505_13254_amd as hs

DEV = "cuda:0"


def dev(x, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(x))
    if dtype is not None:
        t = t.to(dtype)
    return t.to(DEV)


def dev_store(x):
    """A stored attention tensor (float32, or uint16 bfloat16 bit patterns) as a device tensor."""
    x = np.ascontiguousarray(x)
    if x.dtype == np.uint16:
        return torch.from_numpy(x.view(np.int16)).to(DEV).view(torch.bfloat16)
    return torch.from_numpy(x).to(DEV)


def host(t):
    torch.cuda.synchronize()
    if t.dtype == torch.bfloat16:
        return t.float().cpu().numpy()
    return t.cpu().numpy()


def run_entropy(rows, K, T=1.0):
    out = hs.hs_draft_entropy_topk(dev(rows), K, T)
    return {k: host(v) for k, v in out.items()}


def run_prune(pin):
    out = hs.hs_tree_prune(dev(pin["parent"], torch.int32), dev(pin["logc"], torch.float32),
                           dev(pin["node_offsets"], torch.int32), dev(pin["d_max"], torch.int32),
                           dev(pin["theta"], torch.float32), dev(pin["max_nodes"], torch.int32))
    r = {k: host(v) for k, v in out.items()}
    n = int(r["out_offsets"][-1])
    # past the surviving rows the two arrays are padded with rows that hang off a root and repeat it
    r["tail_is_padded"] = bool((r["out_src"][n:] == 0).all() and (r["out_parent"][n:] == 0).all())
    r["out_src"], r["out_parent"] = r["out_src"][:n], r["out_parent"][:n]
    return r


def run_attention(step, want_lse=True):
    no = np.asarray(step["node_offsets"], np.int32)
    po = np.asarray(step["prefix_offsets"], np.int64)
    o, lse = hs.hs_tree_attention(dev_store(step["q"]), dev_store(step["k_prefix"]), dev_store(step["v_prefix"]),
                                  dev_store(step["k_tree"]), dev_store(step["v_tree"]),
                                  dev(step["parent"], torch.int32), dev(no), dev(po),
                                  torch.from_numpy(no), torch.from_numpy(po), float(step["scale"]), want_lse=want_lse)
    return host(o), (host(lse) if lse is not None else None)


def run_accept(step, mode, uniforms, max_depth, temperature=None):
    w = step["w"]
    out = hs.hs_verify_accept(dev(step["target_logits"]), dev(step["draft_logits"]) if mode != 0 else None,
                              dev(step["token"], torch.int32), dev(step["parent"], torch.int32),
                              dev(step["node_offsets"], torch.int32), mode,
                              w.temperature if temperature is None else temperature,
                              dev(uniforms, torch.float32) if uniforms is not None else None, max_depth)
    return {k: host(v) for k, v in out.items()}


def entropy_err(got, want):
    """Worst |dH| in units of the tolerance 1e-5 * max(|H|, 1e-3) (the stated float32 entropy
    tolerance with an absolute floor); a value <= 1 passes."""
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    return float(np.max(np.abs(got - want) / (1e-5 * np.maximum(np.abs(want), 1e-3))))


BF16_U = 2.0 ** -8      # unit roundoff of bfloat16 (8 significant bits, round to nearest)


def attention_error_bound(step, want_o):
    """Element-wise bound on |kernel output - exact output| of the bfloat16 attention kernel, derived from
    its arithmetic (what is rounded where), with u = 2^-8:

      * Q is multiplied by scale * log2(e) and rounded to bfloat16 once more, so a score moves by at most
        delta = u * scale * max_j sum_d |q_d k_jd| (natural-log units, over the keys the row sees), and every
        softmax weight by a factor within exp(+-2 delta);
      * a weight is rounded to bfloat16 for the second product (relative u) while the denominator sums
        the unrounded weights;
      * the result is rounded to bfloat16 once (relative u);
      * float32 accumulation of up to a few 10^4 terms: relative 5e-5 (generous).

    With o the exact output and A = sum_j w_j |v_j| (the exact weights on |V|):
        |error| <= u |o| + ((1 + u) exp(2 delta) - 1 + 5e-5) A
    A comes from the checker run on |V|; delta from |Q| |K|^T over the visible keys."""
    from oracle import tree_attention
    from oracle.tree_attention import _widen, ancestor_mask
    q, kp, kt = _widen(step["q"]), _widen(step["k_prefix"]), _widen(step["k_tree"])
    absv_p, absv_t = np.abs(_widen(step["v_prefix"])), np.abs(_widen(step["v_tree"]))
    A, _ = tree_attention(step["q"], step["k_prefix"], absv_p, step["k_tree"], absv_t, step["parent"],
                          step["node_offsets"], step["prefix_offsets"], step["scale"])
    NN, Hq, D = q.shape
    G = Hq // kt.shape[1]
    no, po = step["node_offsets"], step["prefix_offsets"]
    delta = np.zeros((NN, Hq))
    for s in range(len(no) - 1):
        n0, n1, p0, p1 = int(no[s]), int(no[s + 1]), int(po[s]), int(po[s + 1])
        if n1 == n0:
            continue
        anc = ancestor_mask(np.asarray(step["parent"][n0:n1]))
        for h in range(Hq):
            g = h // G
            aq = np.abs(q[n0:n1, h])
            d = np.where(anc, aq @ np.abs(kt[n0:n1, g]).T, 0.0).max(axis=1)
            if p1 > p0:
                d = np.maximum(d, (aq @ np.abs(kp[p0:p1, g]).T).max(axis=1))
            delta[n0:n1, h] = BF16_U * float(step["scale"]) * d
    grow = (1.0 + BF16_U) * np.exp(2.0 * delta) - 1.0 + 5e-5
    return BF16_U * np.abs(want_o) + grow[:, :, None] * A + 1e-7
