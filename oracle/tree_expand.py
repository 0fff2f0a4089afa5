"""One level of draft-tree growth by Top-K expansion.

Follows Section 2.2 (Expansion): the tree grows one depth at a time; the nodes of the newest
depth with the largest global acceptance value V (product of the confidences on the root path,
kept as a sum of logs) are expanded, each with the K most likely tokens of its draft
distribution, the confidence of a child being that token's draft probability.  Section 4.3
(Dynamic Extended Drafting) lets the number of levels differ per sequence, so a per-sequence
depth limit stops a sequence's growth.  Test infrastructure only.

State of one sequence (lists, row 0 = root): parent, token, logc, cum (float32, the reranking
step's definition: cum[child] = fl32(cum[parent] + min(logc[child], 0))), depth, ent (Top-K
entropy of a row's draft distribution, 0 until the row is expanded), `frontier` (rows to expand
now, ascending) and `level` (levels grown so far).

One step: every frontier row f_j (j-th in ascending order) receives K children in rank order from
result row j of the quantification of its draft distribution; ent[f_j] is set; the new frontier
is the F best rows of the new level under (cum descending, row ascending), listed ascending.
Rows beyond the capacity are not created (a frontier row's children are created all or not at
all).  A sequence at its depth limit, or with an empty frontier, is left alone and its frontier
is emptied.
"""
import numpy as np


def new_state():
    return dict(parent=[-1], token=[-1], logc=[np.float32(0.0)], cum=[np.float32(0.0)], depth=[0],
                ent=[np.float32(0.0)], frontier=[0], level=0)


def tree_expand(state, topk_idx, topk_logp, ent_topk, F, cap, d_limit=None):
    """state: dict as new_state() (modified in place and returned); topk_idx int [>= len(frontier), K],
    topk_logp float32 [same, K], ent_topk float32 [same]: results for the frontier rows in order."""
    st = state
    if (d_limit is not None and st["level"] >= d_limit) or not st["frontier"]:
        st["frontier"] = []
        return st
    K = np.asarray(topk_idx).shape[1]
    new = []
    for j, f in enumerate(st["frontier"]):
        st["ent"][f] = np.float32(ent_topk[j])
        if len(st["parent"]) + K > cap:
            continue
        for k in range(K):
            lc = np.float32(topk_logp[j][k])
            st["parent"].append(int(f))
            st["token"].append(int(topk_idx[j][k]))
            st["logc"].append(lc)
            st["cum"].append(np.float32(st["cum"][f] + min(lc, np.float32(0.0))))
            st["depth"].append(st["depth"][f] + 1)
            st["ent"].append(np.float32(0.0))
            new.append(len(st["parent"]) - 1)
    best = sorted(new, key=lambda i: (-float(st["cum"][i]), i))[:F]
    st["frontier"] = sorted(best)
    st["level"] += 1
    return st
