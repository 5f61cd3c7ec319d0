"""Pins for the metric-selection oracle (Sec. 2.3 Steps 2-3, Alg. 2): facts it must reproduce that do
not come from itself, and planted mistakes that the pins must catch."""
import math
import os
import types

import numpy as np
import pytest
import scipy.stats

from oracle import metric_selection as ms

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "top20_correlations.txt")


def _tables():
    out = {}
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        name, *vals = line.split()
        out[name] = [float(v) for v in vals]
    return out


# ------------------------------------------------------------------------- pins
def pin_pearson_textbook(m):
    # x = 1..5, y = (2, 4, 5, 4, 5): sums of squares 10 and 6, cross sum 6 -> r = 6 / sqrt(60)
    assert abs(m.pearson([1, 2, 3, 4, 5], [2, 4, 5, 4, 5]) - 6 / math.sqrt(60)) < 1e-15
    assert abs(m.pearson([0, 1, 2, 3], [5, 3, 1, -1]) + 1.0) < 1e-15          # exact line, negative slope
    assert abs(m.pearson([0, 1, 2, 3], [1, 1.5, 2, 2.5]) - 1.0) < 1e-15
    assert math.isnan(m.pearson([2, 2, 2], [1, 2, 3])) and math.isnan(m.pearson([1, 2, 3], [7, 7, 7]))
    # ten equal values whose mean does not round back to the value: still a constant column
    for n_, const in ((3, 763774.6425991522), (6, 721540.0601867794), (7, 228762.29839423054),
                      (10, 945270.7010268527)):
        assert math.fsum([const] * n_) / n_ != const          # why the variance is no test for constancy
        assert math.isnan(m.pearson([const] * n_, list(range(n_)))), const
        assert math.isnan(m.pearson(list(range(n_)), [const] * n_)), const
    rng = np.random.default_rng(3)
    for _ in range(20):
        x, y = rng.normal(size=10) * 1e3 + 5e4, rng.normal(size=10)
        want = scipy.stats.pearsonr(x, y)[0]
        assert abs(m.pearson(x, y) - want) < 1e-12
        assert abs(m.pearson(y, x) - want) < 1e-12                             # symmetric
        assert abs(m.pearson(3 * x - 7, 0.5 * y + 2) - want) < 1e-12           # affine maps with positive slopes
        assert abs(m.pearson(-x, y) + want) < 1e-12


def pin_top_k_printed_tables(m):
    """The paper's printed Top-20 tables are ordered by |r|, largest first, signs mixed."""
    rng = np.random.default_rng(4)
    for name, printed in _tables().items():
        assert len(printed) == 20
        extra = list(rng.uniform(-0.6, 0.6, size=30)) + [float("nan")] * 3       # weaker metrics and undefined ones
        pool = printed + extra
        perm = rng.permutation(len(pool))
        shuffled = [pool[j] for j in perm]
        top = m.top_k(shuffled, [True] * len(pool), 20)
        got = [shuffled[j] for j in top]
        assert sorted(map(abs, got), reverse=True) == [abs(v) for v in got], name
        assert sorted(got) == sorted(printed), name
        # in printed order as input, ties keep the printed (index) order
        assert m.top_k(pool, [True] * len(pool), 20) == list(range(20)), name
        # a dropped metric makes room for the next one
        keep = [True] * len(pool)
        keep[0] = False
        t2 = m.top_k(pool, keep, 20)
        assert 0 not in t2 and t2[:19] == list(range(1, 20)) and len(t2) == 20


def pin_percentile(m):
    assert m.percentile([1, 2, 3, 4], 75) == 3.25
    assert m.percentile([4, 1, 3, 2, 5], 75) == 4.0
    assert m.percentile([7.0], 75) == 7.0
    assert m.percentile([0, 10], 75) == 7.5
    v = np.random.default_rng(5).normal(size=37)
    assert abs(m.percentile(v, 75) - np.percentile(v, 75)) < 1e-15
    assert abs(m.percentile(v, 50) - np.median(v)) < 1e-15


def _constructed(n=4, V=10, J=40, seed=6):
    """Tasks whose answer is known by construction.  Metric 0 = runtime (r = +1 everywhere), metric 1 =
    -2 * runtime + 3 (r = -1 everywhere), metric 2 = +runtime in even tasks and -runtime in odd ones,
    metric 3 = runtime in task 0 only and a constant elsewhere, metric 4 = constant; the rest noise."""
    rng = np.random.default_rng(seed)
    runtime = rng.uniform(1.0, 9.0, size=(n, V))
    values = rng.normal(size=(n, V, J))
    for i in range(n):
        values[i, :, 0] = runtime[i]
        values[i, :, 1] = -2.0 * runtime[i] + 3.0
        values[i, :, 2] = runtime[i] if i % 2 == 0 else -runtime[i]
        values[i, :, 3] = runtime[i] if i == 0 else 5.0
        values[i, :, 4] = 1.25
    return values, runtime


def pin_constructed_selection(m):
    values, runtime = _constructed()
    out = m.select(values, runtime, k=20, q=75.0)
    r = out["r"]
    assert np.allclose(r[:, 0], 1.0, atol=1e-12) and np.allclose(r[:, 1], -1.0, atol=1e-12)
    assert np.all(np.isnan(r[:, 4])) and np.all(np.isnan(r[1:, 3])) and abs(r[0, 3] - 1.0) < 1e-12
    for t in out["top"]:
        assert len(t) == 20 and set(t[:3]) == {0, 1, 2} and 4 not in t
    assert 3 in out["top"][0] and all(3 not in t for t in out["top"][1:])
    assert abs(out["score"][0] - 1.0) < 1e-12 and abs(out["score"][2] - 1.0) < 1e-12
    assert abs(out["score"][3] - 0.25) < 1e-12 and out["score"][4] == 0.0                # undefined counts as 0, mean over all n
    sel = out["selected"]
    assert 0 in sel and 1 in sel          # same sign everywhere, in every Top-20, top scores
    assert 2 not in sel                   # sign flips between tasks
    assert 3 not in sel and 4 not in sel  # in one Top-20 only / never defined
    cand_scores = [out["score"][j] for j in out["candidates"]]
    assert abs(out["threshold"] - np.percentile(cand_scores, 75)) < 1e-15
    for j in sel:
        assert out["score"][j] > out["threshold"]
        assert sum(j in t for t in out["top"]) >= 2
    # every candidate above the cut that was left out has a reason
    for j in out["candidates"]:
        if j not in sel and out["score"][j] > out["threshold"]:
            where = [i for i in range(len(out["top"])) if j in out["top"][i]]
            assert len(where) < 2 or len({np.sign(r[i, j]) for i in where}) > 1


def pin_collinear_filter(m):
    values, runtime = _constructed(J=12)
    values[:, :, 5] = 4.0 * values[:, :, 0] - 1.0        # an alias of metric 0
    values[:, :, 6] = -values[:, :, 7]                   # metric 7 mirrors metric 6: the later one goes
    keep = m.collinear_keep(values[0], 0.999)
    assert keep[0] and not keep[1] and not keep[5] and keep[6] and not keep[7] and keep[4]   # 1 is -2*rt+3
    assert all(m.collinear_keep(values[0], None))
    out = m.select(values, runtime, k=3, tau=0.999)
    assert all(5 not in t and 1 not in t and 7 not in t for t in out["top"])
    assert all(t[0] == 0 for t in out["top"])
    # a chain A - B - C with |r(A,B)| = |r(B,C)| = 0.85 but |r(A,C)| = 0.45: B goes, C stays,
    # because C is compared with the metrics that were kept, not with the ones already dropped
    rng = np.random.default_rng(12)
    a = rng.normal(size=(9, 3))
    a -= a.mean(axis=0)
    u, _ = np.linalg.qr(a)
    A = u[:, 0]
    Bm = 0.85 * u[:, 0] + math.sqrt(1 - 0.85 ** 2) * u[:, 1]
    b2 = (0.85 - 0.85 * 0.45) / math.sqrt(1 - 0.85 ** 2)
    C = 0.45 * u[:, 0] + b2 * u[:, 1] + math.sqrt(1 - 0.45 ** 2 - b2 ** 2) * u[:, 2]
    chain = np.stack([A, Bm, C], axis=1)
    assert abs(m.pearson(A, Bm) - 0.85) < 1e-12 and abs(m.pearson(Bm, C) - 0.85) < 1e-12
    assert m.collinear_keep(chain, 0.8) == [True, False, True]


def _with_correlations(rho_rows, V=8, seed=9):
    """values[i][:, m] with Pearson correlation rho_rows[i][m] to runtime[i], by construction:
    rho * u0 + sqrt(1 - rho^2) * u_(m+1) for orthonormal zero-mean vectors u."""
    rng = np.random.default_rng(seed)
    n, J = len(rho_rows), len(rho_rows[0])
    assert J + 1 <= V - 1
    values = np.empty((n, V, J))
    runtime = np.empty((n, V))
    for i in range(n):
        a = rng.normal(size=(V, J + 1))
        a -= a.mean(axis=0)
        u, _ = np.linalg.qr(a)
        runtime[i] = 3.0 + 2.0 * u[:, 0]
        for m_, rho in enumerate(rho_rows[i]):
            values[i, :, m_] = 10.0 * (rho * u[:, 0] + math.sqrt(1 - rho * rho) * u[:, m_ + 1]) - 4.0
    return values, runtime


def pin_prescribed_correlations(m):
    """Correlations fixed by construction; k = 3 and the 25th percentile so that every rule decides
    something: metric 3 scores above the cut but sits in one Top-3 only."""
    rho = [[1.0, -0.9, 0.95, 0.5, 0.1, 0.2],
           [1.0, -0.9, 0.30, 0.8, 0.1, 0.2]]
    values, runtime = _with_correlations(rho)
    out = m.select(values, runtime, k=3, q=25.0)
    assert np.allclose(out["r"], np.array(rho), atol=1e-12)
    assert out["top"] == [[0, 2, 1], [0, 1, 3]]
    assert out["candidates"] == [0, 1, 2, 3]
    assert np.allclose(out["score"], [1.0, 0.9, 0.625, 0.65, 0.1, 0.2], atol=1e-12)
    assert abs(out["threshold"] - 0.64375) < 1e-12          # sorted .625 .65 .9 1.0, position 0.75
    assert out["selected"] == [0, 1]
    assert m.select(values, runtime, k=3, q=25.0, min_tasks=1)["selected"] == [0, 1, 3]
    assert m.select(values, runtime, k=3, q=75.0)["selected"] == [0]     # cut at 0.925


PINS = [pin_prescribed_correlations, pin_pearson_textbook, pin_top_k_printed_tables, pin_percentile, pin_constructed_selection,
        pin_collinear_filter]


@pytest.mark.parametrize("pin", PINS, ids=[p.__name__ for p in PINS])
def test_pin(pin):
    pin(ms)


# --------------------------------------------------------------------- mutants
MUTANTS = [
    ("covariance_not_centred", "sxy = math.fsum((a - mx) * (b - my) for a, b in zip(x, y))",
     "sxy = math.fsum(a * b for a, b in zip(x, y))"),
    ("constant_by_variance", "    if min(x) == max(x) or min(y) == max(y):\n        return float(\"nan\")\n", ""),
    ("no_square_root", "return sxy / math.sqrt(sxx * syy)", "return sxy / (sxx * syy)"),
    ("divides_by_sxx_only", "return sxy / math.sqrt(sxx * syy)", "return sxy / sxx"),
    ("top_by_signed_r", "cand.sort(key=lambda m: (-abs(r_task[m]), m))", "cand.sort(key=lambda m: (-r_task[m], m))"),
    ("top_smallest_first", "cand.sort(key=lambda m: (-abs(r_task[m]), m))", "cand.sort(key=lambda m: (abs(r_task[m]), m))"),
    ("ties_to_higher_index", "cand.sort(key=lambda m: (-abs(r_task[m]), m))", "cand.sort(key=lambda m: (-abs(r_task[m]), -m))"),
    ("nan_enters_top", "if keep[m] and not math.isnan(r_task[m])]", "if keep[m]]"),
    ("percentile_nearest_rank", "return s[lo] + (pos - lo) * (s[hi] - s[lo])", "return s[lo]"),
    ("percentile_of_len", "pos = (len(s) - 1) * q / 100.0", "pos = min(len(s) * q / 100.0, len(s) - 1)"),
    ("score_over_defined_only", "for i in range(n)) / n",
     "for i in range(n)) / max(1, sum(0 if math.isnan(r[i, m]) else 1 for i in range(n)))"),
    ("score_signed", "0.0 if math.isnan(r[i, m]) else abs(r[i, m])", "0.0 if math.isnan(r[i, m]) else r[i, m]"),
    ("sign_rule_dropped", "len(signs) == 1 and ", ""),
    ("single_task_enough", "len(where) >= min_tasks and ", ""),
    ("cut_not_applied", " and score[m] > threshold", ""),
    ("threshold_over_all_metrics", "threshold = percentile([score[m] for m in candidates], q)",
     "threshold = percentile(list(score), q)"),
    ("collinear_signed", "abs(c) >= tau", "c >= tau"),
    ("collinear_against_dropped", "        if keep[m]:\n            kept.append(m)", "        kept.append(m)"),
]


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_mutant_is_caught(name, old, new):
    src = open(ms.__file__).read()
    assert src.count(old) == 1, "mutation site not found or not unique: update this test"
    mod = types.ModuleType("metric_selection_mutant")
    exec(compile(src.replace(old, new), "mutant_" + name, "exec"), mod.__dict__)
    caught = []
    for pin in PINS:
        try:
            pin(mod)
        except AssertionError:
            caught.append(pin.__name__)
    assert caught, "no pin noticed mutant %s" % name
