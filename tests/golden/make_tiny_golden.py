"""Writes tests/golden/tiny_b1_seed0.txt: the oracle's own result on the tiny
configuration (seed 0), kept so that a later change to the oracle's arithmetic
or to the input generator cannot pass unnoticed.  Calls only the oracle and the
input generator; never the HIP path.

    python tests/golden/make_tiny_golden.py
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import spec_oracle as O                      # noqa: E402
from paper_2404_19124_amd import workloads as W          # noqa: E402


def compute():
    wl = W.WORKLOADS["tiny_b1"]
    gen = W.make_generator(wl.seed)
    w = W.make_speculator(wl, gen)
    state, last = W.make_draft_inputs(wl, gen)
    d = O.draft(W.weights_to_numpy(w), W.to_numpy_f32(state), last.numpy(), wl.top_k, wl.B,
                state_dtype=wl.weight_dtype)
    import torch
    logits = W.make_base_logits(wl, torch.from_numpy(d.cand_tokens), gen)
    v = O.verify(W.to_numpy_f32(logits), d.cand_tokens)
    return wl, last, d, v


def main():
    wl, last, d, v = compute()
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_b1_seed0.txt")
    with open(path, "w") as f:
        f.write("# oracle result, tiny configuration (E=D=256, V=1024, n=3, top_k 4/3/2, all 24 leaves kept), seed 0\n")
        f.write("# written by tests/golden/make_tiny_golden.py from oracle/ only\n")
        f.write("last_tok = %d\n" % int(last[0]))
        f.write("cand_leaf = %s\n" % " ".join(str(int(x)) for x in d.cand_leaf[0]))
        f.write("cand_tokens = %s\n" % " ".join(str(int(x)) for x in d.cand_tokens[0].reshape(-1)))
        f.write("cand_scores = %s\n" % " ".join("%.6f" % float(x) for x in d.cand_scores[0]))
        f.write("accept_all = %s\n" % " ".join(str(int(x)) for x in v.accept_all[0]))
        f.write("best_cand = %d\n" % int(v.best_cand[0]))
        f.write("accept_len = %d\n" % int(v.accept_len[0]))
        f.write("out_tokens = %s\n" % " ".join(str(int(x)) for x in v.out_tokens[0]))
    print("wrote", path)


if __name__ == "__main__":
    main()
