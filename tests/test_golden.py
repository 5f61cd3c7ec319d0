"""The oracle still reproduces its frozen tiny case (tests/golden/tiny_chain.txt, written by
tests/golden/make_golden.py from the oracle alone), and the hand-checkable first stage of that
case equals sums written out here."""
import importlib.util
import os

import numpy as np

import oracle

HERE = os.path.dirname(os.path.abspath(__file__))


def _load_case():
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(HERE, "golden", "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def _read_golden():
    rows = {}
    for line in open(os.path.join(HERE, "golden", "tiny_chain.txt")):
        if line.startswith("#"):
            continue
        name, *vals = line.split()
        rows.setdefault(name, []).append([float(v) for v in vals])
    return {k: np.array(v) for k, v in rows.items()}


def test_oracle_reproduces_frozen_case():
    c = _load_case()
    out = oracle.fused_linear_gelu_ln(c.X, c.W, c.b, c.gamma, c.beta, c.EPS, stages=True)
    g = _read_golden()
    for name in ("Z", "G", "Y"):
        assert np.max(np.abs(out[name] - g[name])) <= 1e-15, name
    assert np.max(np.abs(out["mu"] - g["mu"][0])) <= 1e-15
    assert np.max(np.abs(out["var"] - g["var"][0])) <= 1e-15


def test_frozen_case_first_stage_by_hand():
    """Z[0][0] and Z[2][4] of the stored case, expanded by hand (all terms exact)."""
    g = _read_golden()
    z00 = 0.125 + (0.5 * 0.25 + -1.25 * 0.5 + 2.0 * -0.125 + 0.125 * 1.0)
    z24 = 1.0 + (-2.0 * 0.0 + 0.75 * 1.5 + 0.25 * -1.0 + -1.0 * -0.5)
    assert g["Z"][0][0] == z00 == -0.5
    assert g["Z"][2][4] == z24 == 2.375
