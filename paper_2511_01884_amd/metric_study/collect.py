"""Collects, for every task, one kernel trace (runtimes) and one rocprofv3 counter dump per counter
pass of all kernel variants.  This process never touches the GPU itself; each profiler run is a child
process with its own time limit, and the first failure ends the collection.

    python -m paper_2511_01884_amd.metric_study.collect OUT_DIR [TASK ...]
"""
import os
import subprocess
import sys
import time

from .passes import PASSES

REPO = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
TASK_NAMES = ["sq4096", "tall", "wide", "deepk", "mid", "flat"]   # keys of variants.TASKS
RUN_LIMIT_S = 150


def run(cmd, log):
    env = dict(os.environ, TMPDIR="/tmp", PYTHONPATH=REPO + os.pathsep + os.environ.get("PYTHONPATH", ""))
    t0 = time.time()
    with open(log, "w") as f:
        rc = subprocess.call(["timeout", "-s", "KILL", str(RUN_LIMIT_S)] + cmd, cwd="/tmp", env=env,
                             stdout=f, stderr=subprocess.STDOUT)
    print("[collect] rc=%d %.1fs %s" % (rc, time.time() - t0, " ".join(cmd[:12])), flush=True)
    return rc


def main(argv) -> int:
    out = os.path.abspath(argv[1])
    tasks = argv[2:] or TASK_NAMES
    prog = ["python3", "-m", "paper_2511_01884_amd.metric_study.variants"]
    for task in tasks:
        d = os.path.join(out, task)
        os.makedirs(d, exist_ok=True)
        rc = run(["rocprofv3", "--kernel-trace", "--output-format", "csv", "-d", os.path.join(d, "trace"),
                  "-o", "trace", "--"] + prog + [task], os.path.join(d, "trace.log"))
        if rc != 0:
            return rc
        for i, counters in enumerate(PASSES):
            rc = run(["rocprofv3", "--pmc"] + counters + ["--output-format", "csv", "-d",
                      os.path.join(d, "pmc%d" % i), "-o", "pmc", "--"] + prog + [task],
                     os.path.join(d, "pmc%d.log" % i))
            if rc != 0:
                return rc
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv))
