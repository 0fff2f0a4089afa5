"""Draft-side quantification: softmax over the vocabulary, Top-K, and the Top-K entropy.

Follows Section 4.1, Eq. 1 (the per-position term I_t: entropy of the Top-K
probabilities after renormalising them to sum to one) and Section 2.2
(Expansion: a node's confidence c_j is the draft model's probability of its token).
Natural logarithm; ties between equal logits go to the lower vocabulary index.
Test infrastructure only.
"""
import numpy as np


def _entropy(p):
    """-sum p ln p with 0 ln 0 := 0."""
    nz = p > 0.0
    return float(-(p[nz] * np.log(p[nz])).sum())


def draft_entropy_topk(logits, K, temperature=1.0):
    """logits float32 [R, V].  Returns a dict of
        topk_idx  int32 [R, K]  the K largest logits' indices, largest first
        topk_logp f64   [R, K]  log softmax(logits / temperature) at those indices
        ent_topk  f64   [R]     Eq. 1 inner sum: entropy of the renormalised Top-K probabilities
        ent_full  f64   [R]     entropy of the whole softmax
        lse       f64   [R]     ln sum_v exp(logits_v / temperature)
    """
    logits = np.asarray(logits)
    R, V = logits.shape
    assert 1 <= K <= V and temperature > 0
    out = dict(topk_idx=np.zeros((R, K), np.int32), topk_logp=np.zeros((R, K)),
               ent_topk=np.zeros(R), ent_full=np.zeros(R), lse=np.zeros(R))
    for r in range(R):
        raw = logits[r].astype(np.float64)
        x = raw / float(temperature)
        m = x.max()
        Z = np.exp(x - m).sum()
        logp = x - m - np.log(Z)
        p = np.exp(logp)
        # order by (logit descending, index ascending): stable sort of the negated raw logits
        order = np.argsort(-raw, kind="stable")[:K]
        pk = p[order]
        pt = pk / pk.sum()                       # "normalized probabilities of the Top-K tokens"
        out["topk_idx"][r] = order
        out["topk_logp"][r] = logp[order]
        out["ent_topk"][r] = _entropy(pt)
        out["ent_full"][r] = _entropy(p)
        out["lse"][r] = m + np.log(Z)
    return out
