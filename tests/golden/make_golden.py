"""Writes tests/golden/c1_oracle_rows.txt: a few output values of the CPU oracle on
configuration c1 (fp32 tiny layer, seed 0).  Calls only oracle/ and the input generator.
The paper prints no worked numeric example of a layer, so this fixture is a regression
guard for the oracle and the input recipe, not a paper value.

    python tests/golden/make_golden.py
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import oracle as orc  # noqa: E402
from workloads import gen  # noqa: E402


def main():
    w = gen.config("c1")
    y, _, _ = orc.forward(w, gen.generate(w))
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c1_oracle_rows.txt")
    with open(path, "w") as f:
        f.write("# oracle output y[row, col] of configuration c1 (seed 0); columns 0,1,2,127,255 and the row sum\n")
        for t in range(y.shape[0]):
            vals = [y[t, c] for c in (0, 1, 2, 127, 255)] + [y[t].sum()]
            f.write(" ".join("%.12e" % v for v in vals) + "\n")
    print("wrote", path)


if __name__ == "__main__":
    main()
