"""Writes tests/golden/tiny_fp32_greedy.txt from the CPU oracle alone.

The paper prints no numeric example for the stage's forward pass, so this fixture is not a
published value: it freezes what the pinned oracle computes for benchmark config 1 (tiny
fp32 decoder, seed 0, prompt of 32 ids, 8 greedy decode steps) so that a later change to
the oracle's arithmetic or to the seeded generator shows up as a diff.  Run from the repo
root:  python tests/golden/make_tiny_fp32_golden.py
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import synth  # noqa: E402
from oracle.stage_oracle import OracleStage  # noqa: E402


def compute():
    s = synth.CONFIGS["tiny_f32"]
    st = OracleStage(s, 0, s.n_layers_total, 1, 40)
    st.load_tensors(-1, synth.embed_tensors(s, 0))
    st.load_tensors(s.n_layers_total, synth.head_tensors(s, 0))
    for l in range(s.n_layers_total):
        st.load_tensors(l, synth.layer_tensors(s, 0, l))
    tok = synth.token_ids(1, 32, s.vocab)
    nt, lg = st.prefill(tok, [32])
    toks, tops = [int(nt[0])], [float(lg[0].max())]
    for _ in range(8):
        nt, lg = st.decode(nt)
        toks.append(int(nt[0]))
        tops.append(float(lg[0].max()))
    return tok.tolist(), toks, tops


if __name__ == "__main__":
    prompt, toks, tops = compute()
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_fp32_greedy.txt")
    with open(path, "w") as f:
        f.write("# oracle output for benchmark config 1 (written by make_tiny_fp32_golden.py; not a published value)\n")
        f.write("prompt " + " ".join(map(str, prompt)) + "\n")
        f.write("greedy " + " ".join(map(str, toks)) + "\n")
        f.write("top_logit " + " ".join("%.12f" % t for t in tops) + "\n")
    print("wrote", path)
