"""The accept walk over a verified draft tree.

Follows Section 2.1: a drafted token x is accepted with probability
min(1, p(x) / p_hat(x)) (p target, p_hat draft); on rejection the next token is
drawn from the residual of p after removing p_hat, later drafts are dropped and
decoding resumes there.  The tree form (several candidate children per node,
tried one after another, most confident first) is the multi-candidate extension
of that rule used by tree-based verification (Section 2.2, Section 6); with
temperature 0 (the paper's default setting, Section 5) it is the longest
root-to-leaf path whose every token is the target's argmax at its parent.
Uniform numbers are inputs: u[node] decides the test of that node, u[NN + s]
draws the bonus token of sequence s.  Float64.  Test infrastructure only.
"""
import numpy as np

GREEDY, STOCHASTIC, STOCHASTIC_POINTMASS = 0, 1, 2


def _softmax(x):
    x = x.astype(np.float64)
    e = np.exp(x - x.max())
    return e / e.sum()


def _inverse_cdf(p, u):
    """First index whose running sum of p exceeds u (ascending index); last positive entry if none."""
    c = np.cumsum(p)
    hit = np.nonzero(c > u)[0]
    if len(hit):
        return int(hit[0])
    return int(np.nonzero(p > 0)[0][-1])


def verify_accept(target_logits, draft_logits, token, parent, node_offsets, mode, temperature,
                  uniforms, max_depth):
    """Returns dict(accept_len i32 [B], accept_path i32 [B, max_depth] (local indices, -1 padded),
    bonus_token i32 [B]).  draft_logits[n] is the draft distribution the children of node n were
    proposed from; it and `uniforms` may be None in greedy mode."""
    offs = np.asarray(node_offsets, np.int64)
    B, NN = len(offs) - 1, int(offs[-1])
    accept_len = np.zeros(B, np.int32)
    accept_path = np.full((B, max_depth), -1, np.int32)
    bonus = np.zeros(B, np.int32)
    for s in range(B):
        o, n = int(offs[s]), int(offs[s + 1] - offs[s])
        if n == 0:
            bonus[s] = -1
            continue
        par = np.asarray(parent[o:o + n])
        cur, path = 0, []
        while True:
            children = [c for c in range(1, n) if par[c] == cur]
            if len(path) >= max_depth:
                children = []                       # no room to record a longer path: stop here
            nxt = None
            if mode == GREEDY:
                best = int(np.argmax(target_logits[o + cur]))        # first maximum = lower index
                for c in children:
                    if int(token[o + c]) == best:
                        nxt = c
                        break
                if nxt is None:
                    bonus[s] = best
            else:
                p = _softmax(target_logits[o + cur] / np.float64(temperature))
                q = _softmax(draft_logits[o + cur] / np.float64(temperature)) if children else None
                for c in children:
                    x = int(token[o + c])
                    u = float(uniforms[o + c])
                    if mode == STOCHASTIC:
                        if p[x] >= q[x] or u * q[x] < p[x]:          # u < min(1, p/q)
                            nxt = c
                            break
                        r = np.maximum(p - q, 0.0)                    # residual of p after q
                        p = r / r.sum()
                        q = q.copy()
                        q[x] = 0.0                                    # x cannot be proposed again
                        q = q / q.sum()
                    else:                                             # proposal is a point mass at x
                        if u < p[x]:
                            nxt = c
                            break
                        p = p.copy()
                        p[x] = 0.0
                        p = p / p.sum()
                if nxt is None:
                    bonus[s] = _inverse_cdf(p, float(uniforms[NN + s]))
            if nxt is None:
                break
            path.append(nxt)
            cur = nxt
        accept_len[s] = len(path)
        accept_path[s, :len(path)] = path
    return dict(accept_len=accept_len, accept_path=accept_path, bonus_token=bonus)
