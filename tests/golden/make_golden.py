"""Writes tests/golden/config0_oracle.txt from the CPU oracle alone.

The paper prints no worked numeric example for the layer, so the stored values are
the oracle's own outputs on the smallest workload (one 64x64x64->64 masked-binary
layer, seed 0), kept as a regression pin: a later change to the oracle's arithmetic
or to the input recipe shows up as a diff of this file.  Calls only oracle/ and the
seeded input module - never the HIP path.
"""
import hashlib
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import oracle as O                     # noqa: E402
from paper_2601_11660_amd import synth             # noqa: E402


def config0_summary():
    c = synth.conv_case(0, 0, 1, 64, 64, 64, 64, keep=0.6, theta_bound=8)
    acc, out = O.masked_binary_layer(c.a, c.w, c.theta)
    lines = [
        "# one masked-binary 3x3 layer, N=1 H=W=64 Cin=Cout=64, keep 0.6, theta in [-8,8], seed 0",
        "# layer definition: Sec. 3.1.1; accumulator R and threshold step: Algorithm 1",
        f"acc_sha256 {hashlib.sha256(acc.tobytes()).hexdigest()}",
        f"out_sha256 {hashlib.sha256(out.tobytes()).hexdigest()}",
        f"acc_sum {int(acc.astype(np.int64).sum())}",
        f"acc_min {int(acc.min())}",
        f"acc_max {int(acc.max())}",
        f"out_plus_count {int((out == 1).sum())}",
        "acc_0_0_0_first8 " + " ".join(str(int(v)) for v in acc[0, 0, 0, :8]),
        "acc_0_31_17_first8 " + " ".join(str(int(v)) for v in acc[0, 31, 17, :8]),
        "theta_first8 " + " ".join(str(int(v)) for v in c.theta[:8]),
    ]
    return lines


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "config0_oracle.txt")
    with open(path, "w") as f:
        f.write("\n".join(config0_summary()) + "\n")
    print(path)
