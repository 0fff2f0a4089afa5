"""Complexity quantification and the adaptive decision that follows it.

Follows Section 4.1 (Eq. 1: cumulative meta-path Top-K entropy Phi of the operational path P*),
Section 4.2 (the decision tree's leaves are non-overlapping entropy bins B_0 .. B_{n-1}, lowest
entropy first; only their boundaries are needed at run time) and Section 4.3 (Dynamic Extended
Drafting: d' = d_base + Delta; Top-N pruning: N' = gamma * N_default + Delta; Delta = alpha - i
for the low-entropy bin B_i, no change for the other bins).  Test infrastructure only.

Per sequence, with the tree as parent pointers in BFS order (row 0 = root):
  depth, S    as in the reranking step: S[i] = fl32(S[parent] + min(logc[i], 0))
  D           the deepest level present
  P*          the node of level D with the best final confidence:
                mode 0: largest cumulative value S (ties: lower row)
                mode 1: largest own confidence min(logc, 0) (ties: lower row)
  Phi         sum of ent[a] over the strict ancestors a of P*, root first: ent[a] is the Top-K
              entropy of the draft distribution at a, the one that a's child on the path was
              drawn from, so a path of T tokens has T terms (Eq. 1)
  bin         number of bin boundaries that Phi (summed in float32, root first: the precision in
              which the decision is taken on both sides) has reached
  Delta       max(alpha - bin, 0) for bin < len(gamma), else 0
  d'          d_base + Delta
  N'          floor(float64(gamma[bin]) * N_default + 0.5) + Delta for bin < len(gamma), else N_default
"""
import numpy as np


def adaptive_control(parent, logc, ent, node_offsets, bin_edges, gamma, alpha, d_base, n_default, mode=0):
    """parent int32 [NN] (local, -1 at roots), logc float32 [NN], ent float32 [NN], node_offsets [B+1];
    bin_edges float32 ascending [n_bins - 1]; gamma float32 [n_low]; alpha, d_base, n_default ints.
    Returns dict(phi f64 [B], pstar i32 [B], bin i32 [B], d_prime i32 [B], n_prime i32 [B])."""
    parent = np.asarray(parent, np.int32)
    logc = np.asarray(logc, np.float32)
    ent = np.asarray(ent, np.float32)
    offs = np.asarray(node_offsets, np.int64)
    edges = np.asarray(bin_edges, np.float32)
    gamma = np.asarray(gamma, np.float32)
    assert np.all(np.diff(edges) >= 0)
    B = len(offs) - 1
    phi = np.zeros(B, np.float64)
    pstar = np.zeros(B, np.int32)
    bins = np.zeros(B, np.int32)
    d_prime = np.zeros(B, np.int32)
    n_prime = np.zeros(B, np.int32)
    for s in range(B):
        o, n = int(offs[s]), int(offs[s + 1] - offs[s])
        if n == 0:
            pstar[s] = -1
            d_prime[s], n_prime[s] = d_base, n_default
            continue
        par = parent[o:o + n]
        depth = np.zeros(n, np.int64)
        S = np.zeros(n, np.float32)
        for i in range(1, n):
            p = int(par[i])
            assert 0 <= p < i
            depth[i] = depth[p] + 1
            S[i] = np.float32(S[p] + min(logc[o + i], np.float32(0.0)))
        D = int(depth.max())
        level = [i for i in range(n) if depth[i] == D]
        if mode == 0:
            best = min(level, key=lambda i: (-float(S[i]), i))
        else:
            best = min(level, key=lambda i: (-float(min(logc[o + i], np.float32(0.0))), i))
        path = []
        a = int(par[best])
        while a >= 0:
            path.append(a)
            a = int(par[a])
        path.reverse()                                   # root first
        acc32 = np.float32(0.0)
        acc64 = 0.0
        for a in path:
            acc32 = np.float32(acc32 + ent[o + a])
            acc64 += float(ent[o + a])
        b = int(np.sum(acc32 >= edges))
        low = b < len(gamma)
        delta = max(int(alpha) - b, 0) if low else 0
        phi[s], pstar[s], bins[s] = acc64, best, b
        d_prime[s] = int(d_base) + delta
        n_prime[s] = (int(np.floor(np.float64(gamma[b]) * float(n_default) + 0.5)) + delta) if low else int(n_default)
    return dict(phi=phi, pstar=pstar, bin=bins, d_prime=d_prime, n_prime=n_prime)
