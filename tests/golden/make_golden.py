"""Writes tests/golden/tiny_w8a8_4x8x8.txt and tiny_w4a8_3x16x5.txt from the CPU oracle alone.

The paper prints no worked numeric example of the rotated linear (Sec. 3.2 gives
Eq. 9/10 only), so these fixtures are the oracle's own output on two tiny seeded
cases, frozen once its pins passed: a guard against later drift of the oracle, not
an independent pin.  Run:  python tests/golden/make_golden.py
"""
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

from oracle import trdq_oracle as o                      # noqa: E402
from paper_2503_06564_amd import workloads as wl         # noqa: E402

CASES = {
    "tiny_w8a8_4x8x8.txt": dict(seed=0, M=4, K=8, N=8, B=8, wbits=8),
    "tiny_w4a8_3x16x5.txt": dict(seed=11, M=3, K=16, N=5, B=8, wbits=4),
}


def compute(c):
    Xb, W, d, bias = wl.small_case(c["seed"], c["M"], c["K"], c["N"], n_outliers=1, outlier=20.0)
    return o.linear(Xb, W, d, bias, B=c["B"], wbits=c["wbits"])


def main():
    for name, c in CASES.items():
        out = compute(c)
        with open(os.path.join(HERE, name), "w") as f:
            f.write(f"# oracle output, small_case{tuple(c.values())}; written by make_golden.py\n")
            f.write("Xq " + " ".join(map(str, out["Xq"].reshape(-1).tolist())) + "\n")
            f.write("Wq " + " ".join(map(str, out["Wq"].reshape(-1).tolist())) + "\n")
            f.write("acc " + " ".join(map(str, out["acc"].reshape(-1).tolist())) + "\n")
            f.write("Y " + " ".join(f"{v:04x}" for v in out["Y"].reshape(-1).tolist()) + "\n")


if __name__ == "__main__":
    main()
