"""Writes tests/golden/mask_seed0_round1_c100_N100000.txt from the CPU oracle alone.

Run from the repository root:  python tests/golden/make_mask_pin.py
The stored values are a regression pin of the build-defined mask rule (Eq. (3) with the
Philox4x32-10 keying); tests re-derive them with the independent pure-Python statement.
"""
import os
import sys

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__)))))
from oracle import saps_oracle as O  # noqa: E402

keep = O.mask(100_000, seed=0, rnd=1, seg_c=100.0)
idx = np.flatnonzero(keep)
out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "mask_seed0_round1_c100_N100000.txt")
with open(out, "w") as f:
    f.write("# Eq. (3) mask, seed=0 round=1 c=100 N=100000: K, then every kept coordinate.\n")
    f.write("# Written by tests/golden/make_mask_pin.py (CPU oracle only).\n")
    f.write(f"K {len(idx)}\n")
    f.write(" ".join(str(int(j)) for j in idx) + "\n")
print(out, len(idx))
