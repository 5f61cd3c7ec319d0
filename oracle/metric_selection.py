"""CPU oracle for the paper's profiling-metric selection (Sec. 2.3, Steps 2 and 3; Alg. 2).

THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  Plain float64 Python/numpy, the steps in the paper's
order and notation, written to be checked by eye; it shares nothing with the GPU library.

Input: n tasks; for task i a set K_i* of V kernels, each with a runtime and the same J metrics:
    values[i][v][m]   metric m of kernel v of task i        runtime[i][v]

Step 2 (per task).  r_{m,i} = Pearson correlation, over the task's V kernels, between metric m and
the runtime.  Optionally metrics that duplicate an earlier one are dropped first (the paper removes
"aliases and strongly collinear indicators" without giving a rule; the reading taken here: walking
the metrics in index order, a metric is dropped for this task when its |Pearson correlation| with a
metric already kept is >= tau).  Top20_i = the k = 20 kept metrics with the largest |r_{m,i}|.

Step 3 (across tasks).  M* = union of the Top20_i.  Global score S_m = (1/n) sum_i |r_{m,i}| over all
n tasks.  Final = { m in M* : m is in the Top-20 of at least two tasks, r_{m,i} has one sign over
the tasks whose Top-20 contain m, and S_m > P75 of { S_m : m in M* } }.

Readings where the paper is silent: a correlation with a constant column (or constant runtime; all
values equal) is undefined: it is NaN here, never enters a Top-20, and counts as 0 in S_m.  Ties in |r| go to the
lower metric index.  The percentile interpolates linearly between order statistics (position
(len - 1) * q / 100 in the sorted list).
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Sequence

import numpy as np


def pearson(x: Sequence[float], y: Sequence[float]) -> float:
    """r = sum (x - mean x)(y - mean y) / sqrt( sum (x - mean x)^2 * sum (y - mean y)^2 ).
    Undefined (NaN) when either sample is constant, i.e. all its values are equal: decided by comparing
    the values, not by the rounded variance (the mean of equal values need not round to that value)."""
    x = [float(v) for v in x]
    y = [float(v) for v in y]
    n = len(x)
    if n != len(y) or n == 0:
        raise ValueError("two samples of the same positive length")
    if min(x) == max(x) or min(y) == max(y):
        return float("nan")
    mx = math.fsum(x) / n
    my = math.fsum(y) / n
    sxy = math.fsum((a - mx) * (b - my) for a, b in zip(x, y))
    sxx = math.fsum((a - mx) ** 2 for a in x)
    syy = math.fsum((b - my) ** 2 for b in y)
    if not (sxx > 0.0 and syy > 0.0):
        return float("nan")
    return sxy / math.sqrt(sxx * syy)


def correlations(values: np.ndarray, runtime: np.ndarray) -> np.ndarray:
    """r[i][m] for every task and metric."""
    values = np.asarray(values, dtype=np.float64)
    runtime = np.asarray(runtime, dtype=np.float64)
    n, V, J = values.shape
    if runtime.shape != (n, V):
        raise ValueError("runtime must be [n][V]")
    r = np.empty((n, J), dtype=np.float64)
    for i in range(n):
        for m in range(J):
            r[i, m] = pearson(values[i, :, m], runtime[i])
    return r


def collinear_keep(task_values: np.ndarray, tau: Optional[float]) -> List[bool]:
    """keep[m] for one task: metric m survives unless |r(m, m')| >= tau for an earlier kept m'."""
    V, J = task_values.shape
    keep = [True] * J
    if tau is None:
        return keep
    kept: List[int] = []
    for m in range(J):
        for m2 in kept:
            c = pearson(task_values[:, m], task_values[:, m2])
            if not math.isnan(c) and abs(c) >= tau:
                keep[m] = False
                break
        if keep[m]:
            kept.append(m)
    return keep


def top_k(r_task: Sequence[float], keep: Sequence[bool], k: int) -> List[int]:
    """Indices of the k kept metrics with the largest |r| (defined r only), largest first,
    ties to the lower index."""
    cand = [m for m in range(len(r_task)) if keep[m] and not math.isnan(r_task[m])]
    cand.sort(key=lambda m: (-abs(r_task[m]), m))
    return cand[:k]


def percentile(vals: Sequence[float], q: float) -> float:
    s = sorted(float(v) for v in vals)
    if not s:
        return float("nan")
    pos = (len(s) - 1) * q / 100.0
    lo = int(math.floor(pos))
    hi = min(lo + 1, len(s) - 1)
    return s[lo] + (pos - lo) * (s[hi] - s[lo])


def select_from_r(r, keeps, k: int = 20, q: float = 75.0, min_tasks: int = 2) -> Dict[str, object]:
    """Steps after the correlations: r [n][J]; keeps[i][m] says whether metric m survived the
    duplicate filter in task i."""
    r = np.asarray(r, dtype=np.float64)
    n, J = r.shape
    tops = [top_k(list(r[i]), keeps[i], k) for i in range(n)]
    candidates = sorted(set(m for t in tops for m in t))          # M*
    score = np.zeros(J, dtype=np.float64)                         # S_m, over all n tasks
    for m in range(J):
        score[m] = math.fsum(0.0 if math.isnan(r[i, m]) else abs(r[i, m]) for i in range(n)) / n
    threshold = percentile([score[m] for m in candidates], q)
    selected = []
    for m in candidates:
        where = [i for i in range(n) if m in tops[i]]
        signs = set(1 if r[i, m] > 0 else (-1 if r[i, m] < 0 else 0) for i in where)
        if len(where) >= min_tasks and len(signs) == 1 and score[m] > threshold:
            selected.append(m)
    return {"r": r, "top": tops, "candidates": candidates, "score": score, "threshold": threshold,
            "selected": selected}


def select(values, runtime, k: int = 20, q: float = 75.0, tau: Optional[float] = None,
           min_tasks: int = 2) -> Dict[str, object]:
    values = np.asarray(values, dtype=np.float64)
    n, V, J = values.shape
    r = correlations(values, runtime)
    keeps = [collinear_keep(values[i], tau) for i in range(n)]
    out = select_from_r(r, keeps, k, q, min_tasks)
    out["keep"] = keeps
    return out
