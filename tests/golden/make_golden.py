"""Writes tests/golden/mask_vectors.txt from the CPU oracle alone (run from the repo root:
`python tests/golden/make_golden.py`). The paper prints no worked example of its random choice, so
these vectors pin this repository's written mask rule, not a value from the paper."""
import os
import sys

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__)))))
from oracle import mask as omask  # noqa: E402

CASES = []
for key in (0x240617611, 1):
    for step, layer in ((0, 0), (7, 2), (2**40 + 3, 1)):
        for gid, width, k in ((0, 16, 4), (1, 100, 13), (169342, 128, 8), (2449028, 256, 32), (12345, 512, 16),
                              (99, 100, 100)):
            CASES.append((key, step, layer, gid, width, k))

out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "mask_vectors.txt")
with open(out, "w") as f:
    f.write("# key step layer gid width k  kept positions pi_v(0..k-1)\n")
    f.write("# source: oracle.mask.kept_columns (this repository's mask rule; the paper fixes no generator)\n")
    for key, step, layer, gid, width, k in CASES:
        cols = omask.kept_columns(np.array([gid]), width, k, key, step, layer)[0]
        f.write(f"{key:#x} {step} {layer} {gid} {width} {k} " + " ".join(map(str, cols.tolist())) + "\n")
print("wrote", out, len(CASES), "vectors")
