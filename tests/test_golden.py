"""The stored c1 oracle rows (written by tests/golden/make_golden.py from the oracle
alone) still come out of the oracle and the seeded input recipe."""
import os

import numpy as np

from oracle import oracle as orc
from workloads import gen


def test_c1_oracle_rows_reproduce():
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "c1_oracle_rows.txt")
    want = np.loadtxt(path, comments="#")
    w = gen.config("c1")
    y, _, _ = orc.forward(w, gen.generate(w))
    got = np.stack([np.concatenate([y[t, [0, 1, 2, 127, 255]], [y[t].sum()]]) for t in range(y.shape[0])])
    assert np.allclose(got, want, rtol=1e-9, atol=1e-10)
