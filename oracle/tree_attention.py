"""Tree-masked attention of the draft tree's rows over the prefix KV cache.

Follows Section 2.2 (Reranking: the pruned tree is verified in one pass with
tree-mask attention): row i of a sequence attends to every prefix token and to
the tree rows on its own root path (the root, its ancestors and itself), with
ordinary scaled-dot-product softmax attention.  Float64 throughout over the
stored (float32 or bfloat16) inputs.  Test infrastructure only.
"""
import numpy as np


def _widen(x):
    """Stored tensor -> float64.  uint16 arrays hold bfloat16 bit patterns."""
    x = np.asarray(x)
    if x.dtype == np.uint16:
        return (x.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return x.astype(np.float64)


def ancestor_mask(parent):
    """mask[i, j] = True iff tree row j is i itself or an ancestor of i."""
    M = len(parent)
    mask = np.zeros((M, M), bool)
    for i in range(M):
        j = i
        while j >= 0:
            mask[i, j] = True
            j = int(parent[j])
    return mask


def tree_attention(q, k_prefix, v_prefix, k_tree, v_tree, parent, node_offsets, prefix_offsets,
                   scale):
    """q [NN,Hq,D]; k_prefix, v_prefix [sum L,Hkv,D]; k_tree, v_tree [NN,Hkv,D];
    parent int32 [NN] local indices; node_offsets [B+1]; prefix_offsets [B+1].
    Returns (o float64 [NN,Hq,D], lse float64 [NN,Hq]); lse = ln of the softmax denominator
    of the scaled scores."""
    q, kp, vp, kt, vt = (_widen(t) for t in (q, k_prefix, v_prefix, k_tree, v_tree))
    NN, Hq, D = q.shape
    Hkv = kt.shape[1]
    G = Hq // Hkv
    o = np.zeros((NN, Hq, D))
    lse = np.zeros((NN, Hq))
    B = len(node_offsets) - 1
    for s in range(B):
        n0, n1 = int(node_offsets[s]), int(node_offsets[s + 1])
        p0, p1 = int(prefix_offsets[s]), int(prefix_offsets[s + 1])
        M, L = n1 - n0, p1 - p0
        if M == 0:
            continue
        allowed = np.concatenate([np.ones((M, L), bool), ancestor_mask(parent[n0:n1])], axis=1)
        for h in range(Hq):
            g = h // G
            keys = np.concatenate([kp[p0:p1, g], kt[n0:n1, g]], axis=0)        # [L+M, D]
            vals = np.concatenate([vp[p0:p1, g], vt[n0:n1, g]], axis=0)
            sc = scale * (q[n0:n1, h] @ keys.T)                                  # [M, L+M]
            sc = np.where(allowed, sc, -np.inf)
            mx = sc.max(axis=1, keepdims=True)
            e = np.exp(sc - mx)
            den = e.sum(axis=1, keepdims=True)
            o[n0:n1, h] = (e / den) @ vals
            lse[n0:n1, h] = (mx + np.log(den))[:, 0]
    return o, lse
