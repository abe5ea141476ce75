"""Writes tests/golden/quantize_2x4.txt from the CPU oracle (and only from it).

The stored values are re-derived in tests/test_oracle_pipeline.py with exact
fractions from the recipe "amax -> scale = amax/448 -> e4m3 RNE cast" of the
problem statement, so the file pins the oracle's behaviour over time and the test
pins the file to the definition.

Run:  python tests/golden/make_golden.py
"""
import os
import sys

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__)))))
import oracle  # noqa: E402

# bf16 bit patterns of a hand-picked 2x4 matrix:
#   row 0:  1.0, -3.0, 0.3984375, 100.0      row 1: -0.001953125, 7.5, 0.0, -0.0625
X = np.array([[0x3F80, 0xC040, 0x3ECC, 0x42C8],
              [0xBB00, 0x40F0, 0x0000, 0xBD80]], dtype=np.uint16)

out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "quantize_2x4.txt")
with open(out, "w") as f:
    f.write("# rowwise / per-tensor / per-column e4m3 quantization of a 2x4 bf16 matrix, written by\n")
    f.write("# tests/golden/make_golden.py from the CPU oracle.  Recipe (problem statement: amax, then scale,\n")
    f.write("# then an OCP e4m3 cast, RNE, saturating at 448): scale = amax/448 (fp32), code = e4m3(x * (448/amax)).\n")
    f.write("# line format: mode | x bits (hex, row-major) | codes (hex, row-major) | scales (fp32 bits, hex)\n")
    for mode, name in ((oracle.SCALE_ROW, "row"), (oracle.SCALE_TENSOR, "tensor"), (oracle.SCALE_COL, "col")):
        q, s = oracle.quantize(X, mode, threads=1)
        f.write("%s | %s | %s | %s\n" % (
            name,
            " ".join("%04x" % v for v in X.ravel()),
            " ".join("%02x" % v for v in q.ravel()),
            " ".join("%08x" % v for v in s.view(np.uint32))))
print("wrote", out)
