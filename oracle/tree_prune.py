"""Reranking / pruning of the draft tree by cumulative confidence.

Follows Section 2.2: the global acceptance value of node i is the product of the
confidences on the path root -> i (kept here as a sum of logs), and the pruned
subtree keeps the best nodes by that value; Section 4.3 (Top-N pruning) makes the
node budget N' a per-sequence number.  The workloads also filter by depth and by a
threshold on the cumulative log-probability, so all three filters are arguments.
Test infrastructure only.

Definition used on both sides (so the kept set can be compared bit for bit):
  depth[0] = 0, depth[i] = depth[parent[i]] + 1
  S[0] = 0,     S[i] = fl32(S[parent[i]] + min(logc[i], 0))      one float32 add per node
  pass[i]  = depth[i] <= d_max and S[i] >= theta
  cand     = { i >= 1 : pass holds for i and for every ancestor of i }
  if max_nodes > 0 and |cand| > max_nodes: keep the first max_nodes of cand under
      (S descending, index ascending); the root is always kept.
  Kept nodes are emitted in ascending original index with parents renumbered.
"""
import numpy as np


def tree_prune(parent, logc, node_offsets, d_max, theta, max_nodes):
    """parent int32 [NN] (local indices, -1 at each root), logc float32 [NN], node_offsets [B+1];
    d_max int [B], theta float32 [B], max_nodes int [B].
    Returns dict(depth i32 [NN], cumlogp f32 [NN], keep u8 [NN], out_offsets i32 [B+1],
                 out_src i32 [NN'], out_parent i32 [NN'])."""
    parent = np.asarray(parent, np.int32)
    logc = np.asarray(logc, np.float32)
    offs = np.asarray(node_offsets, np.int64)
    B = len(offs) - 1
    NN = int(offs[-1])
    depth = np.zeros(NN, np.int32)
    S = np.zeros(NN, np.float32)
    keep = np.zeros(NN, np.uint8)
    out_offsets = np.zeros(B + 1, np.int32)
    out_src, out_parent = [], []
    for s in range(B):
        o, n = int(offs[s]), int(offs[s + 1] - offs[s])
        if n == 0:
            out_offsets[s + 1] = out_offsets[s]
            continue
        par = parent[o:o + n]
        ok = np.zeros(n, bool)
        ok[0] = True
        th = np.float32(theta[s])
        for i in range(1, n):
            p = int(par[i])
            assert 0 <= p < i
            depth[o + i] = depth[o + p] + 1
            S[o + i] = np.float32(S[o + p] + min(logc[o + i], np.float32(0.0)))
            ok[i] = ok[p] and depth[o + i] <= int(d_max[s]) and S[o + i] >= th
        cand = [i for i in range(1, n) if ok[i]]
        if int(max_nodes[s]) > 0 and len(cand) > int(max_nodes[s]):
            cand.sort(key=lambda i: (-float(S[o + i]), i))
            cand = cand[:int(max_nodes[s])]
        kept = [0] + sorted(cand)
        new_index = {old: new for new, old in enumerate(kept)}
        for old in kept:
            keep[o + old] = 1
            out_src.append(old)
            out_parent.append(-1 if old == 0 else new_index[int(par[old])])
        out_offsets[s + 1] = out_offsets[s] + len(kept)
    return dict(depth=depth, cumlogp=S, keep=keep, out_offsets=out_offsets,
                out_src=np.asarray(out_src, np.int32), out_parent=np.asarray(out_parent, np.int32))
