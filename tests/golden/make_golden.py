"""Writes tests/golden/tiny_chain.txt from the CPU oracle only (no GPU code is involved).

The paper prints no worked numeric example of this operator chain, so there is no
"paper value" to store; this file freezes the oracle's own output on a tiny fixed
case, after the oracle was pinned by tests/oracle_pins.py.  It guards against
accidental changes of the oracle's arithmetic: a deliberate change must regenerate it
and say why in the commit message.

    python tests/golden/make_golden.py
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import oracle  # noqa: E402

M, K, N = 3, 4, 5
# exactly representable inputs (multiples of 1/8), written out rather than drawn
X = np.array([[0.5, -1.25, 2.0, 0.125], [1.0, 0.0, -0.5, 3.0], [-2.0, 0.75, 0.25, -1.0]], dtype=np.float32)
W = np.array([[0.25, 0.5, -0.125, 1.0], [-1.0, 0.125, 0.375, 0.0], [0.5, 0.5, 0.5, 0.5],
              [2.0, -0.75, 0.0, 0.25], [0.0, 1.5, -1.0, -0.5]], dtype=np.float32)
b = np.array([0.125, -0.25, 0.0, 0.5, 1.0], dtype=np.float32)
gamma = np.array([1.0, 0.5, 2.0, 1.25, 0.75], dtype=np.float32)
beta = np.array([0.0, 0.25, -0.5, 1.0, 0.125], dtype=np.float32)
EPS = 1e-5


def main():
    out = oracle.fused_linear_gelu_ln(X, W, b, gamma, beta, EPS, stages=True)
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_chain.txt")
    with open(path, "w") as f:
        f.write("# oracle output for the fixed 3x4x5 case in make_golden.py (no paper value exists; see that file)\n")
        for name in ("Z", "G", "Y"):
            for m in range(M):
                f.write(name + " " + " ".join(repr(float(v)) for v in out[name][m]) + "\n")
        f.write("mu " + " ".join(repr(float(v)) for v in out["mu"]) + "\n")
        f.write("var " + " ".join(repr(float(v)) for v in out["var"]) + "\n")
    print("wrote", path)


if __name__ == "__main__":
    main()
