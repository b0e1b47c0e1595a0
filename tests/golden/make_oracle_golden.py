"""Writes tests/golden/oracle_tiny.txt: the oracle's outputs on one tiny seeded
case, as a tripwire against accidental edits of the oracle's arithmetic.

The values come from `oracle/` alone (never from the GPU path).  They are not
paper values: the paper prints no worked example for this operator.  Run from
the repository root:  python tests/golden/make_oracle_golden.py
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import fdl_oracle as O  # noqa: E402


def case():
    # exactly representable inputs so the file does not depend on a generator
    M, K, N = 3, 2, 4
    X = np.array([[0.5, -1.25], [2.0, 0.75], [-0.5, 0.25]])
    W = np.array([[1.0, -0.5], [0.25, 0.75], [-1.5, 0.5], [0.125, 2.0]])
    b = np.array([0.125, -0.25, 0.5, 0.0])
    gamma = np.array([1.0, 1.5, 0.5, -0.75])
    beta = np.array([0.0, 0.25, -0.5, 1.0])
    dY = np.array([[1.0, -2.0, 0.5, 0.25], [0.0, 1.0, -1.0, 2.0], [-0.5, 0.75, 1.5, -1.0]])
    return dict(X=X, W=W, b=b, gamma=gamma, beta=beta, dY=dY, eps=1e-5)


def main():
    c = case()
    r = O.forward_backward(**c)
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_tiny.txt")
    with open(path, "w") as f:
        f.write("# oracle outputs for the fixed 3x2x4 case in make_oracle_golden.py (fp64, repr round-trip)\n")
        for k in ("Y", "mean", "rstd", "dX", "dW", "db", "dgamma", "dbeta"):
            v = np.asarray(r[k]).ravel()
            f.write(k + " " + " ".join(repr(float(x)) for x in v) + "\n")
    print("wrote", path)


if __name__ == "__main__":
    main()
