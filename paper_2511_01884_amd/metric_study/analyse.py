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
from .variants import KERNEL_TAG, REPEATS, TASKS, VARIANTS

LAUNCH_COLUMNS = ["LDS_Block_Size", "VGPR_Count", "Accum_VGPR_Count", "SGPR_Count", "Grid_Size_X"]


def _one(pattern):
    found = glob.glob(pattern, recursive=True)
    if len(found) != 1:
        raise RuntimeError("expected one file for %s, found %d" % (pattern, len(found)))
    return found[0]


def _variant_slices(dispatch_ids):
    """Dispatches of the tagged kernel in launch order: one sizing launch, then REPEATS per variant;
    the first launch of each variant is a warm-up."""
    ids = sorted(dispatch_ids)
    if len(ids) != 1 + REPEATS * len(VARIANTS):
        raise RuntimeError("expected %d dispatches of %s, found %d" % (1 + REPEATS * len(VARIANTS), KERNEL_TAG, len(ids)))
    ids = ids[1:]
    return [ids[v * REPEATS + 1:(v + 1) * REPEATS] for v in range(len(VARIANTS))]


def read_task(task_dir):
    """runtime_us[V], {metric: [V]} for one task."""
    rows = [r for r in csv.DictReader(open(_one(os.path.join(task_dir, "trace", "**", "*kernel_trace.csv"))))
            if KERNEL_TAG in r["Kernel_Name"]]
    by_id = {int(r["Dispatch_Id"]): r for r in rows}
    slices = _variant_slices(by_id.keys())
    runtime = [sum(int(by_id[i]["End_Timestamp"]) - int(by_id[i]["Start_Timestamp"]) for i in s) / len(s) / 1e3
               for s in slices]
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
    return runtime, metrics


def main(argv) -> int:
    out_dir, report = argv[1], argv[2]
    tasks = [t for t in TASKS if os.path.isdir(os.path.join(out_dir, t))]
    if len(tasks) < 2:
        raise RuntimeError("need the dumps of at least two tasks under " + out_dir)
    runtimes, tables = [], []
    for t in tasks:
        rt, m = read_task(os.path.join(out_dir, t))
        runtimes.append(rt)
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
