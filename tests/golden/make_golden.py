"""Writes tests/golden/tiny_oracle.txt: the oracle's out/lse for the 'tiny'
workload (seed 1001).  Calls only oracle/ and the input generator.  The file is
a regression guard for the oracle itself (its values are pinned by
tests/test_oracle_pins.py, not by this file); the paper prints no numbers for
this computation, so no fixture here is the paper's.

Run from the repo root:  python tests/golden/make_golden.py
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import ref  # noqa: E402
from paper_2512_21450_amd import workloads as wl  # noqa: E402

w = wl.WORKLOADS["tiny"]
x = wl.make_inputs(w)
out, lse = ref.decode_attn_ref(x["q"], x["k_prefix"], x["v_prefix"], x["prefix_lens"],
                               x["k_suffix"], x["v_suffix"], x["suffix_lens"], w.scale, w.G)
path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_oracle.txt")
with open(path, "w") as f:
    f.write("# oracle output for workload 'tiny' (seed 1001); written by tests/golden/make_golden.py\n")
    f.write("# suffix_lens " + " ".join(map(str, x["suffix_lens"])) + "\n")
    f.write("# columns: b h lse out[0] out[21] out[42] out[63]\n")
    for b in range(w.B):
        for h in range(w.Hq):
            f.write(f"{b} {h} {lse[b, h]:.17g} " + " ".join(f"{out[b, h, c]:.17g}" for c in (0, 21, 42, 63)) + "\n")
print("wrote", path)
