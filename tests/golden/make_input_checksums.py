"""Writes tests/golden/input_checksums.txt: CRC32 of seeded synthetic input tensors, so the
generators cannot drift unnoticed.  Calls only the input generators.
Run from the repository root:  python tests/golden/make_input_checksums.py"""
import os
import sys
import zlib

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__)))))
from synth import workloads as W  # noqa: E402


def entries():
    w = W.WORKLOADS
    yield "w1.parents", W.tree_parents(w[1], 0)
    yield "w3.parents", W.tree_parents(w[3], 0)
    yield "w4.parents", W.tree_parents(w[4], 0)
    yield "w5.prefix_lengths", W.prefix_lengths(w[5], 0)
    yield "w1.draft.row0", W.logits_row(w[1], 0, "draft", 0, 0)
    yield "w1.target.row3", W.logits_row(w[1], 0, "target", 0, 3)
    yield "w2.draft.row0", W.logits_row(w[2], 0, "draft", 0, 0)
    yield "w2.target.row7", W.logits_row(w[2], 0, "target", 0, 7)
    yield "w3.draft.row5", W.logits_row(w[3], 0, "draft", 0, 5)
    yield "w5.target.s3.row2", W.logits_row(w[5], 0, "target", 3, 2)
    for name, t in zip("q kp vp kt vt".split(), W.attention_inputs(w[1], 0, 0, 128, 17)):
        yield "w1.attn." + name, t
    for name, t in zip("q kp vp kt vt".split(), W.attention_inputs(w[2], 0, 0, 256, 9, "peaky",
                                                                  parent=np.arange(-1, 8))):
        yield "w2.attn.peaky." + name, t
    yield "w2.uniforms", W.uniforms(w[2], 0, 62)


def main():
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "input_checksums.txt")
    with open(out, "w") as f:
        f.write("# CRC32 of seeded synthetic inputs (seed 0); written by make_input_checksums.py\n")
        for name, t in entries():
            t = np.ascontiguousarray(t)
            f.write("%s %s %s %08x\n" % (name, t.dtype, "x".join(map(str, t.shape)), zlib.crc32(t.tobytes())))


if __name__ == "__main__":
    main()
