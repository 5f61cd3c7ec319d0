"""Builds the (task, kernel, metric) table from the dumps `collect` wrote, runs the library's metric
selection on it (device correlations, host selection) and writes a markdown report.

    python -m paper_2511_01884_amd.metric_study.analyse OUT_DIR REPORT.md
"""
import csv
import glob
import os
import sys
from collections import defaultdict

import torch

from .. import binding as B
from .passes import PASSES
from .variants import KERNEL_TAG, REPEATS, SECOND_PASS_TAG, SIZING_LAUNCHES, TASKS, VARIANTS

LAUNCH_COLUMNS = ["LDS_Block_Size", "VGPR_Count", "Accum_VGPR_Count", "SGPR_Count", "Grid_Size_X"]


def _one(pattern):
    found = glob.glob(pattern, recursive=True)
    if len(found) != 1:
        raise RuntimeError("expected one file for %s, found %d" % (pattern, len(found)))
    return found[0]


def _variant_slices(dispatch_ids, variants=VARIANTS):
    """Dispatches of one kernel in launch order: the sizing launches, then REPEATS per variant; the
    first launch of each variant is a warm-up."""
    ids = sorted(dispatch_ids)
    if len(ids) != SIZING_LAUNCHES + REPEATS * len(variants):
        raise RuntimeError("expected %d dispatches, found %d" % (SIZING_LAUNCHES + REPEATS * len(variants), len(ids)))
    ids = ids[SIZING_LAUNCHES:]
    return [ids[v * REPEATS + 1:(v + 1) * REPEATS] for v in range(len(variants))]


def _mean_us(by_id, ids):
    return sum(int(by_id[i]["End_Timestamp"]) - int(by_id[i]["Start_Timestamp"]) for i in ids) / len(ids) / 1e3


def read_task(task_dir):
    """runtime_us[V] of the tile kernel, runtime_us[V] of the second pass (0 for fused variants) and
    {metric: [V]} for one task."""
    trace = list(csv.DictReader(open(_one(os.path.join(task_dir, "trace", "**", "*kernel_trace.csv")))))
    by_id = {int(r["Dispatch_Id"]): r for r in trace if KERNEL_TAG in r["Kernel_Name"]}
    slices = _variant_slices(by_id.keys())
    runtime = [_mean_us(by_id, s) for s in slices]
    second = {int(r["Dispatch_Id"]): r for r in trace if SECOND_PASS_TAG in r["Kernel_Name"]}
    two_pass = [v for v in VARIANTS if v[4] == B.FF_VARIANT_TILED_TWOPASS]
    second_us = dict(zip((v[0] for v in two_pass),
                         (_mean_us(second, s) for s in _variant_slices(second.keys(), two_pass))))
    second_pass = [second_us.get(v[0], 0.0) for v in VARIANTS]
    metrics = {}
    for col in LAUNCH_COLUMNS:
        metrics["launch_" + col] = [sum(float(by_id[i][col]) for i in s) / len(s) for s in slices]
    for p in range(len(PASSES)):
        acc = defaultdict(lambda: defaultdict(float))     # dispatch -> counter -> summed value
        for r in csv.DictReader(open(_one(os.path.join(task_dir, "pmc%d" % p, "**", "*counter_collection.csv")))):
            if KERNEL_TAG in r["Kernel_Name"]:
                acc[int(r["Dispatch_Id"])][r["Counter_Name"]] += float(r["Counter_Value"])
        pslices = _variant_slices(acc.keys())
        for name in PASSES[p]:
            metrics[name] = [sum(acc[i][name] for i in s) / len(s) for s in pslices]
    return runtime, second_pass, metrics


def _planned_variant(M, K, N):
    """Label of the variant the automatic plan takes for a bf16 problem (ff_plan_query).  The 256 x 128
    tile has one label whatever the number of workgroups per compute unit the grid comes to."""
    d = B.ff_plan_query(M, K, N, B.FF_BF16)
    for label, tile, per_cu, waves, variant in VARIANTS:
        half_height = (tile, per_cu) == (256, 2)
        if d["variant"] != variant or (d["tile_n"], d["tile_m"]) != ((256, 128) if half_height else (tile, tile)):
            continue
        if half_height or (d["workgroups_per_cu"] == per_cu and (waves == 0 or d["waves"] == waves)):
            return label
    return None


def main(argv) -> int:
    out_dir, report = argv[1], argv[2]
    tasks = [t for t in TASKS if os.path.isdir(os.path.join(out_dir, t))]
    if len(tasks) < 2:
        raise RuntimeError("need the dumps of at least two tasks under " + out_dir)
    runtimes, seconds, tables = [], [], []
    for t in tasks:
        rt, sp, m = read_task(os.path.join(out_dir, t))
        runtimes.append(rt)
        seconds.append(sp)
        tables.append(m)
    names = sorted(tables[0])
    values = torch.tensor([[[tab[nm][v] for nm in names] for v in range(len(VARIANTS))] for tab in tables],
                          dtype=torch.float64)
    runtime = torch.tensor(runtimes, dtype=torch.float64)
    lines = ["# Profiling-metric selection on MI355X: this library's tile-kernel variants", "",
             "Procedure: the paper's Sec. 2.3 Steps 2-3 / Alg. 2 (Pearson correlation of every metric with the",
             "kernel runtime per task, Top-20 per task, global score = mean |r| over tasks, keep metrics that are",
             "in several Top-20 lists with one sign and score above the 75th percentile), computed by",
             "`ff_metric_selection`.  Metrics: %d rocprofv3 hardware counters (7 passes) plus launch" % (len(names) - len(LAUNCH_COLUMNS)),
             "parameters.  Tasks: %d shapes of the fused operator (bf16); kernels per task: the %d tile-kernel" % (len(tasks), len(VARIANTS)),
             "variants below (the paper keeps 10 of 100 generated kernels per task; here every variant there is).",
             "Commands: `python -m paper_2511_01884_amd.metric_study.collect DIR` then",
             "`python -m paper_2511_01884_amd.metric_study.analyse DIR REPORT.md`.", "",
             "## Runtime of the tile kernel per variant (microseconds, mean of %d launches)" % (REPEATS - 1), "",
             "| task (M x K x N) | " + " | ".join(v[0] for v in VARIANTS) + " |",
             "|---|" + "---|" * len(VARIANTS)]
    for t, rt in zip(tasks, runtimes):
        lines.append("| %s (%d x %d x %d) | " % ((t,) + TASKS[t]) + " | ".join("%.1f" % x for x in rt) + " |")
    lines += ["", "## Runtime of the whole call per variant: tile kernel plus, for the two-pass variants, the",
              "## normalisation kernel that follows it (microseconds; * marks the fastest of a task, P the",
              "## automatic plan's choice)", "",
              "| task (M x K x N) | " + " | ".join(v[0] for v in VARIANTS) + " |",
              "|---|" + "---|" * len(VARIANTS)]
    for t, rt, sp in zip(tasks, runtimes, seconds):
        whole = [a + b for a, b in zip(rt, sp)]
        M, K, N = TASKS[t]
        planned = _planned_variant(M, K, N)
        cells = ["%.1f%s%s" % (x, "*" if x == min(whole) else "", " P" if v[0] == planned else "")
                 for x, v in zip(whole, VARIANTS)]
        lines.append("| %s (%d x %d x %d) | " % (t, M, K, N) + " | ".join(cells) + " |")
    for title, tau in (("without the duplicate filter", 0.0), ("duplicates dropped at |r| >= 0.999", 0.999)):
        res = B.ff_metric_selection(values.cuda(), runtime.cuda(), top_k=20, percentile=75.0, collinear_tau=tau,
                                    min_tasks=2)
        lines += ["", "## Selection, " + title, "",
                  "Score cut (P75 of the candidates' scores): %.4f.  Selected key subset (%d metrics):" %
                  (res["threshold"], len(res["selected"])), "",
                  "| metric | score | r per task (" + ", ".join(tasks) + ") | Top-20 of |", "|---|---|---|---|"]
        for m in sorted(res["selected"], key=lambda j: -res["score"][j]):
            rs = ", ".join("%+.3f" % res["r"][i][m] for i in range(len(tasks)))
            where = ", ".join(tasks[i] for i in range(len(tasks)) if m in res["top"][i])
            lines.append("| %s | %.4f | %s | %s |" % (names[m], res["score"][m], rs, where))
        if tau == 0.0:
            for i, t in enumerate(tasks):
                lines += ["", "### Top-20 of task %s" % t, "", "| metric | r |", "|---|---|"]
                lines += ["| %s | %+.6f |" % (names[m], res["r"][i][m]) for m in res["top"][i]]
    with open(report, "w") as f:
        f.write("\n".join(lines) + "\n")
    print("[analyse] wrote %s: %d tasks, %d metrics" % (report, len(tasks), len(names)), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv))
