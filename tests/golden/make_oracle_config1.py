"""Writes tests/golden/oracle_config1.txt: the CPU checker's results for the tiny workload
(seed 0), as a regression anchor.  Calls only the input generators and oracle/.
Run from the repository root:  python tests/golden/make_oracle_config1.py"""
import os
import sys

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__)))))
from synth import workloads as W  # noqa: E402
from oracle import pipeline as P  # noqa: E402


def compute():
    st = P.build_step(W.WORKLOADS[1], 0)
    s1 = st["trees"][0]["stage1"]
    o, lse = P.attention_out(st)
    acc = P.accept_out(st, 0)
    return {
        "topk_idx_row0": s1["topk_idx"][0], "ent_topk": s1["ent_topk"], "ent_full": s1["ent_full"],
        "cumlogp": st["prune_out"]["cumlogp"], "keep": st["prune_out"]["keep"],
        "out_parent": st["prune_out"]["out_parent"], "attn_o_row0_head0": o[0, 0, :8], "attn_lse": lse[:, 0],
        "accept_len": acc["accept_len"], "bonus_token": acc["bonus_token"],
    }


def main():
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_config1.txt")
    with open(out, "w") as f:
        f.write("# CPU checker results, workload 1 (tiny), seed 0; written by make_oracle_config1.py\n")
        for k, v in compute().items():
            v = np.asarray(v)
            fmt = "%d" if v.dtype.kind in "iu" else "%.12e"
            f.write(k + " = " + " ".join(fmt % x for x in v.ravel()) + "\n")


if __name__ == "__main__":
    main()
