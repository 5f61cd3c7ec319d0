"""Metric selection (Sec. 2.3 Steps 2-3, Alg. 2): the library against the oracle.  The host-only part
runs without a GPU; the device correlations are GPU tests."""
import math

import numpy as np
import pytest
import torch

from oracle import metric_selection as oracle_ms
from paper_2511_01884_amd import binding as B
from paper_2511_01884_amd.inputs import make_metric_inputs

GAP = 1e-9   # |r| values closer than this may legitimately order differently between two fp64 evaluations


def _compare(got, ref, k):
    r_ref = ref["r"]
    assert np.allclose(got["r"], r_ref, rtol=0, atol=1e-10, equal_nan=True)
    assert np.array_equal(np.isnan(got["r"]), np.isnan(r_ref))
    assert np.allclose(got["score"], ref["score"], rtol=0, atol=1e-10)
    if math.isnan(ref["threshold"]):
        assert math.isnan(got["threshold"])
    else:
        assert abs(got["threshold"] - ref["threshold"]) <= 1e-10
    for i, (tg, tr) in enumerate(zip(got["top"], ref["top"])):
        assert len(tg) == len(tr)
        a = [abs(r_ref[i, m]) for m in tr]
        for p in range(len(tr)):
            lone = (p == 0 or a[p - 1] - a[p] > GAP) and (p + 1 == len(tr) or a[p] - a[p + 1] > GAP)
            if lone:
                assert tg[p] == tr[p], (i, p)
        assert sorted(abs(r_ref[i, m]) for m in tg) == pytest.approx(sorted(a), abs=GAP)
    # the cut decides membership only where a score is clear of it
    clear = [m for m in ref["candidates"] if abs(ref["score"][m] - ref["threshold"]) > GAP]
    assert [m for m in got["selected"] if m in clear] == [m for m in ref["selected"] if m in clear]


# ------------------------------------------------------------------ host part, no GPU
@pytest.mark.parametrize("n,V,J,k,q,min_tasks", [(6, 10, 120, 20, 75.0, 2), (3, 10, 15, 20, 75.0, 2),
                                                 (1, 10, 40, 5, 50.0, 1), (8, 4, 300, 20, 90.0, 3)])
def test_host_selection_matches_oracle(n, V, J, k, q, min_tasks):
    values, runtime = make_metric_inputs(n, V, J, seed=21)
    ref = oracle_ms.select(values.numpy(), runtime.numpy(), k=k, q=q, min_tasks=min_tasks)
    got = B.ff_metric_select_host(ref["r"], None, top_k=k, percentile=q, min_tasks=min_tasks)
    _compare(got, ref, k)


def test_host_selection_with_keep_mask_and_edge_cases():
    values, runtime = make_metric_inputs(4, 10, 60, seed=22)
    v = values.numpy()
    ref = oracle_ms.select(v, runtime.numpy(), k=10, tau=0.999)
    keep = np.array([oracle_ms.collinear_keep(v[i], 0.999) for i in range(4)], dtype=np.uint8)
    assert keep.sum() < keep.size            # the generator plants aliases
    got = B.ff_metric_select_host(ref["r"], keep, top_k=10)
    _compare(got, ref, 10)
    # nothing defined: no candidates, NaN threshold, nothing selected
    out = B.ff_metric_select_host(np.full((2, 5), np.nan))
    assert out["top"] == [[], []] and out["selected"] == [] and math.isnan(out["threshold"])
    # prescribed correlations with every rule deciding something (the case the oracle is pinned on)
    r = np.array([[1.0, -0.9, 0.95, 0.5, 0.1, 0.2], [1.0, -0.9, 0.30, 0.8, 0.1, 0.2]])
    out = B.ff_metric_select_host(r, top_k=3, percentile=25.0)
    assert out["top"] == [[0, 2, 1], [0, 1, 3]] and out["selected"] == [0, 1]
    assert abs(out["threshold"] - 0.64375) < 1e-12
    assert B.ff_metric_select_host(r, top_k=3, percentile=25.0, min_tasks=1)["selected"] == [0, 1, 3]
    r[1, 0] = -1.0                             # sign flips between the tasks
    assert B.ff_metric_select_host(r, top_k=3, percentile=25.0)["selected"] == [1]
    with pytest.raises(B.FFError):
        B.ff_metric_select_host(r, top_k=0)
    with pytest.raises(B.FFError):
        B.ff_metric_select_host(r, percentile=101.0)


# ---------------------------------------------------------------------- device part
GPU_CASES = [(8, 10, 300, 20, 75.0, 0.0), (8, 10, 300, 20, 75.0, 0.999), (5, 10, 2000, 20, 75.0, 0.0),
             (3, 2, 50, 20, 75.0, 0.0), (2, 1, 30, 20, 75.0, 0.0), (4, 37, 257, 7, 60.0, 0.95),
             (1, 10, 64, 20, 75.0, 0.0)]


@pytest.mark.gpu
@pytest.mark.parametrize("n,V,J,k,q,tau", GPU_CASES)
def test_device_selection_matches_oracle(n, V, J, k, q, tau):
    print("[case] metric selection", n, V, J, k, q, tau, flush=True)
    values, runtime = make_metric_inputs(n, V, J, seed=23)
    ref = oracle_ms.select(values.numpy(), runtime.numpy(), k=k, q=q, tau=tau if tau > 0 else None)
    got = B.ff_metric_selection(values.cuda(), runtime.cuda(), top_k=k, percentile=q, collinear_tau=tau)
    # the correlations agree to rounding; metrics that are affine images of one another then tie to
    # within rounding, and which of them takes the last Top-k seat may differ between two fp64
    # evaluations.  So: the decisions must be exactly the oracle's decisions on the library's r ...
    assert np.allclose(got["r"], ref["r"], rtol=0, atol=1e-10, equal_nan=True)
    assert np.array_equal(np.isnan(got["r"]), np.isnan(ref["r"]))
    same = oracle_ms.select_from_r(got["r"], ref["keep"], k=k, q=q)
    assert got["top"] == same["top"] and got["selected"] == same["selected"]
    assert np.allclose(got["score"], same["score"], rtol=0, atol=1e-14)
    assert abs(got["threshold"] - same["threshold"]) <= 1e-14 or (math.isnan(got["threshold"]) and math.isnan(same["threshold"]))
    # ... and the oracle's own wherever no such near-tie sits on a boundary
    boundary_tie = False
    for i, t in enumerate(ref["top"]):
        if len(t) == k:
            rest = [abs(ref["r"][i, m]) for m in range(J) if ref["keep"][i][m] and m not in t and not math.isnan(ref["r"][i, m])]
            if rest and abs(ref["r"][i, t[-1]]) - max(rest) <= GAP:
                boundary_tie = True
    print("  boundary tie:", boundary_tie, flush=True)
    if not boundary_tie:
        _compare(got, ref, k)
    again = B.ff_metric_selection(values.cuda(), runtime.cuda(), top_k=k, percentile=q, collinear_tau=tau)
    assert np.array_equal(again["r"], got["r"], equal_nan=True) and again["selected"] == got["selected"]


@pytest.mark.gpu
def test_device_selection_constant_runtime_and_errors():
    values, runtime = make_metric_inputs(3, 10, 40, seed=24)
    runtime[1] = 2.5                           # one task whose kernels all take the same time
    ref = oracle_ms.select(values.numpy(), runtime.numpy())
    got = B.ff_metric_selection(values.cuda(), runtime.cuda())
    assert np.all(np.isnan(got["r"][1])) and got["top"][1] == []
    _compare(got, ref, 20)
    with pytest.raises(TypeError):
        B.ff_metric_selection(values.float().cuda(), runtime.float().cuda())
    with pytest.raises(ValueError):
        B.ff_metric_selection(values.cuda(), runtime[:2].cuda())
    lib = B.load()
    assert lib.ff_metric_selection(None, None, 1, 1, 1, 20, 75.0, 0.0, 2, None, None, None, None, None, None) == 1
