#!/usr/bin/env python3
"""Benchmark of the fused linear + erf-GELU + LayerNorm library on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg1]

One step = one call of ff_fused_linear_gelu_ln (the whole hot path) on one
synthetic batch already resident in HBM.  Successive steps rotate through
distinct (X, W, Y) buffer sets whose total size exceeds the 256 MB Infinity
Cache, so rates are HBM rates, not cache rates.  Before the warm-up steps the
same step runs untimed for --preheat-ms (default 300 ms): the chip reaches its
steady clock only after some tens of milliseconds of load, which a handful of
warm-up launches does not provide.  Prints ONE JSON line; --timeline adds the
kernels' own per-phase durations to it (and prints them to stderr).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# MI355X published peaks: 256 CUs x 4096 bf16 flop/clk x 2.4 GHz; HBM3E 8 TB/s.
PEAK_BF16_TFLOPS = 2516.6
PEAK_F32_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0
INFINITY_CACHE_BYTES = 256 << 20

# HBM traffic per launch of the dominant kernel, from two `rocprofv3 --pmc` runs (FETCH_SIZE, then
# WRITE_SIZE, KiB per dispatch), each scaled by what the same counter reads for the library's plain
# copy kernel on 256 MiB (`--workload copy`): FETCH_SIZE reads 131080 for 262144 KiB -> factor 2.0;
# WRITE_SIZE 262140 -> 1.0.  An entry is valid only for the device sources of its kernel (its .hip file
# and the shared device helpers) as they were when the counters were taken: `traffic` is null once
# their hash differs.
COMMON_SOURCES = ["ff_device.hpp"]   # device helpers every kernel includes
TRAFFIC = {
    "cfg1": {"sources": ["ff_tile.hip"], "sha256": "977a752d225258d91e2df06011e8c348b6938f706ae84c6743deef9000958301",
             "bytes": int((99551.0 * 2.0 + 33322.0 * 1.0) * 1024)},
    "cfg3": {"sources": ["ff_smallm.hip"], "sha256": "3d3b0c0d2dcbef9f914cc9f692bb843590916bdc620aa9ab6f9bbc9756d5264a",
             "bytes": int((66914.0 * 2.0 + 339.0 * 1.0) * 1024)},
    "xent": {"sources": ["ff_xent.hip"], "sha256": "6f6d24291f7ea6e33d3e4afae0ad2c30eade991481a459c8c95966b01b5506d1",
             "bytes": int((262700.0 * 2.0 + 32.1 * 1.0) * 1024)},
    "rowmean": {"sources": ["ff_rowmean.hip"], "sha256": "e5e79e742f35d38f9b13b80e0d38b9794bfaf330a93e1664410356d6bbd9ac6d",
             "bytes": int((33203.0 * 2.0 + 32882.0 * 1.0) * 1024)},
}


def kernel_source_hash(workload: str) -> str:
    import hashlib
    h = hashlib.sha256()
    for name in sorted(TRAFFIC[workload]["sources"] + COMMON_SOURCES):
        h.update(name.encode())
        h.update(open(os.path.join(ROOT, "paper_2511_01884_amd", "csrc", name), "rb").read())
    return h.hexdigest()


def measured_traffic(workload: str):
    t = TRAFFIC.get(workload)
    if t is None or not t["sha256"] or t["sha256"] != kernel_source_hash(workload):
        return None
    return t["bytes"]


def sustained_ceiling(torch, B, bound: str):
    """What the chip sustains at all, from the library's two do-nothing-else kernels: an MFMA-only loop
    (bf16) or a streaming read of 1 GiB.  Reported beside the published peak, never instead of it."""
    ev0 = torch.cuda.Event(enable_timing=True)
    ev1 = torch.cuda.Event(enable_timing=True)
    if bound == "mfma":
        B.ff_debug_mfma_loop(2000)
        torch.cuda.synchronize()
        ev0.record()
        flops = B.ff_debug_mfma_loop(40000)          # about 10 ms
        ev1.record()
        torch.cuda.synchronize()
        return {"value": flops / (ev0.elapsed_time(ev1) * 1e-3) / 1e12, "unit": "TFLOP/s",
                "what": "register-resident loop of bf16 32x32x16 MFMAs, four wavefronts per compute unit"}
    buf = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").random_(0, 255)
    B.ff_debug_stream_read(buf)
    torch.cuda.synchronize()
    ev0.record()
    n = 0
    for _ in range(10):
        n += B.ff_debug_stream_read(buf)
    ev1.record()
    torch.cuda.synchronize()
    return {"value": n / (ev0.elapsed_time(ev1) * 1e-3) / 1e9, "unit": "GB/s",
            "what": "streaming read of 1 GiB, 16-byte loads, eight in flight per thread"}


def batch_median_ms(torch, step, launches: int = 100, batches: int = 5) -> float:
    """Median over batches of the mean launch time between two events (the protocol's second figure)."""
    out = []
    for _ in range(batches):
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(launches):
            step(i)
        e1.record()
        torch.cuda.synchronize()
        out.append(e0.elapsed_time(e1) / launches)
    return sorted(out)[len(out) // 2]


def preheat(torch, step, ms: float) -> int:
    """Untimed launches of the step for about `ms` of wall time, ahead of the warm-up steps: the chip leaves
    its idle clock state only after some tens of milliseconds of load, far more than five warm-up launches."""
    n = 0
    t_end = time.perf_counter() + ms * 1e-3
    while time.perf_counter() < t_end:
        for _ in range(20):
            step(n)
            n += 1
        torch.cuda.synchronize()
    return n


TILE_STAMPS = ["tile start", "first K slab in LDS", "K loop done", "GELU done, row statistics published",
               "other tiles of the rows arrived", "statistics merged", "stores issued"]
SMALLM_STAMPS = ["workgroup start", "first wavefront's K slice done", "all wavefronts done", "row statistics published",
                 "other workgroups arrived", "statistics merged", "stores issued"]


def phase_timeline(torch, B, step, small_m: bool, launches: int = 3, grid: int = 0):
    """Per-phase durations of one launch from the kernels' own timestamps (ff_debug_set_timeline): the mean,
    minimum and maximum over the workgroups' tiles of the last of `launches` launches."""
    slots, max_tiles = 16, 16 * 512
    buf = torch.zeros(max_tiles * slots, dtype=torch.int64, device="cuda")
    B.ff_debug_set_timeline(buf)
    try:
        for i in range(launches):
            step(i)
        torch.cuda.synchronize()
    finally:
        B.ff_debug_set_timeline(None)
    B.ff_check_device()
    rec = buf.cpu().double().view(-1, slots)
    rec = rec[rec[:, 0] > 0]
    if len(rec) == 0:
        return None
    names = SMALLM_STAMPS if small_m else TILE_STAMPS
    rel = (rec[:, :7] - rec[:, 0].min()) / 100.0          # 100 MHz wall clock -> microseconds
    dur = rel[:, 1:] - rel[:, :-1]
    out = {"tiles": int(len(rec)), "last_stamp_us": float(rel[:, 6].max()), "phases": []}
    if not small_m:
        k_us = (rec[:, 2] - rec[:, 1]) / 100.0
        mhz = (rec[:, 9] - rec[:, 8]) / k_us
        out["k_loop_shader_clock_mhz"] = float(mhz.mean())
        if grid:
            # workgroup w runs on XCD w % 8; records are stored at [round * grid + w]
            live = (buf.cpu().view(-1, slots)[:, 0] > 0).nonzero().flatten()
            xcd = (live % grid) % 8
            out["k_loop_by_xcd"] = [{"xcd": x, "mean_us": float(k_us[xcd == x].mean()),
                                     "spread_us": float(k_us[xcd == x].max() - k_us[xcd == x].min()),
                                     "shader_clock_mhz": float(mhz[xcd == x].mean()),
                                     "kilocycles": float((rec[:, 9] - rec[:, 8])[xcd == x].mean() / 1e3)}
                                    for x in range(8) if bool((xcd == x).any())]
    for k in range(6):
        out["phases"].append({"from": names[k], "to": names[k + 1], "mean_us": float(dur[:, k].mean()),
                              "min_us": float(dur[:, k].min()), "max_us": float(dur[:, k].max())})
    print("phase timeline (%d tiles, last stamp %.1f us after the first):" % (out["tiles"], out["last_stamp_us"]),
          file=sys.stderr)
    for ph in out["phases"]:
        print("  %-38s -> %-38s mean %6.1f  min %6.1f  max %6.1f us" %
              (ph["from"], ph["to"], ph["mean_us"], ph["min_us"], ph["max_us"]), file=sys.stderr)
    for x in out.get("k_loop_by_xcd", []):
        print("  K loop on XCD %d: mean %6.1f us (max - min %4.1f), shader clock %4.0f MHz, %5.1f thousand cycles" %
              (x["xcd"], x["mean_us"], x["spread_us"], x["shader_clock_mhz"], x["kilocycles"]), file=sys.stderr)
    return out


def algorithmic_bytes(M, K, N, esize):
    """Each of X, W, b, gamma, beta read once and Y written once."""
    return (M * K + N * K + M * N + 3 * N) * esize


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--workload", default="cfg1",
                    help="cfg0..cfg4 (default: cfg1, the metric's workload), f32_4096, copy (counter calibration), rowmean "
                         "(second fused chain: Linear, subtract, row-mean, GELU, residual add; bf16 4096^3), or xent "
                         "(row-wise cross-entropy with mean, fp32 32768 x 4096)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-eager", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="target CPU time of the oracle sample")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the batch-median and sustained-ceiling figures")
    ap.add_argument("--cache-warm", action="store_true",
                    help="also time launches on a single buffer set (not in the default run, so that every "
                         "launch of the default command has the rotating-buffer duration)")
    ap.add_argument("--preheat-ms", type=float, default=300.0,
                    help="untimed launches of the step for this long before the warm-up steps (0: none)")
    ap.add_argument("--timeline", action="store_true",
                    help="after the timed region, run three launches with the kernels' phase timestamps switched on "
                         "and report the per-phase durations (cfg0..cfg4 and f32_4096 only)")
    ap.add_argument("--print-source-hash", action="store_true", help="print the kernel source hash and exit")
    args = ap.parse_args()
    if args.print_source_hash:
        for w in TRAFFIC:
            print(w, kernel_source_hash(w))
        return 0

    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU; the path shards by rows with no exchange "
              "(rows are independent: replicate W, split M), and no multi-GPU figure is produced. Re-run with --gpus 1.",
              file=sys.stderr)
        return 2

    import torch
    from paper_2511_01884_amd import binding as B
    from paper_2511_01884_amd.inputs import CONFIGS, make_inputs

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 1
    B.load()  # fails loudly if the HIP library is not built
    torch.cuda.set_device(0)
    if args.workload == "rowmean":
        return bench_rowmean(args, torch, B)
    if args.workload == "xent":
        return bench_xent(args, torch, B)
    if args.workload == "copy":
        return bench_copy(args, torch, B)
    wl = CONFIGS[args.workload]
    M, K, N = wl.M, wl.K, wl.N
    esize = 4 if wl.dtype == "f32" else 2
    flops = 2.0 * M * K * N
    abytes = algorithmic_bytes(M, K, N, esize)

    d = make_inputs(M, K, N, wl.dtype, seed=0)
    set_bytes = (M * K + N * K + M * N) * esize
    n_sets = max(2, -(-int(1.5 * INFINITY_CACHE_BYTES) // set_bytes))
    n_sets = min(n_sets, 16)
    b, gamma, beta = d["b"].cuda(), d["gamma"].cuda(), d["beta"].cuda()
    sets = []
    X0, W0 = d["X"].cuda(), d["W"].cuda()
    for i in range(n_sets):
        X = X0 if i == 0 else X0.clone()
        W = W0 if i == 0 else W0.clone()
        sets.append((X, W, torch.empty((M, N), dtype=X0.dtype, device="cuda")))
    eps = d["eps"]

    def step(i):
        X, W, Y = sets[i % n_sets]
        B.ff_fused_linear_gelu_ln(X, W, b, gamma, beta, eps, Y=Y)

    n_pre = preheat(torch, step, args.preheat_ms)
    for i in range(args.warmup):
        step(i)
    B.ff_check_device()
    torch.cuda.synchronize()
    ev0 = torch.cuda.Event(enable_timing=True)
    ev1 = torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for i in range(args.steps):
        step(i)
    ev1.record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    B.ff_check_device()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    ms_kernel = ev0.elapsed_time(ev1) / args.steps
    variant = B.ff_last_variant()

    # the kernels' own phase timestamps, taken straight after the timed region: the sustained-ceiling
    # kernels further down leave the chip at a lower clock for a while
    timeline = None
    if args.timeline:
        grid = B.ff_plan_query(M, K, N, B.FF_F32 if wl.dtype == "f32" else B.FF_BF16)["grid"]
        timeline = phase_timeline(torch, B, step, small_m=(variant == B.FF_VARIANT_SMALL_M), grid=grid)

    hbm_bound = args.workload == "cfg3"
    if hbm_bound:
        value = abytes / (ms_per_step * 1e-3) / 1e9
        unit = "GB/s"
        roof = {"bound": "hbm", "achieved": abytes / (ms_kernel * 1e-3) / 1e9, "peak": PEAK_HBM_GBS,
                "unit": "GB/s"}
    else:
        value = flops / (ms_per_step * 1e-3) / 1e12
        unit = "TFLOP/s"
        peak = PEAK_F32_TFLOPS if wl.dtype == "f32" else PEAK_BF16_TFLOPS
        roof = {"bound": "mfma", "achieved": flops / (ms_kernel * 1e-3) / 1e12, "peak": peak,
                "unit": "TFLOP/s"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    roof["traffic"] = measured_traffic(args.workload)
    roof["kernel_ms"] = ms_kernel
    if not args.no_extras:
        launches = 100 if ms_kernel < 0.5 else 20
        roof["batch_median_ms"] = batch_median_ms(torch, step, launches)
        if args.cache_warm:   # one buffer set only: inputs stay in the Infinity Cache
            roof["cache_warm_ms"] = batch_median_ms(torch, lambda i: step(0), launches, 3)
        if wl.dtype == "bf16" or hbm_bound:
            roof["sustained"] = sustained_ceiling(torch, B, roof["bound"])
            roof["frac_of_sustained"] = roof["achieved"] / roof["sustained"]["value"]

    out = {
        "metric": "TFLOP/s and % of bf16 MFMA peak (GB/s for small-M) for fused linear+GELU+LN",
        "value": value, "unit": unit, "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if wl.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": "%s: %s fused linear+GELU+LayerNorm M=%d K=%d N=%d" % (wl.name, wl.dtype, M, K, N),
                   "variant": variant, "buffer_sets": n_sets, "preheat_launches": n_pre,
                   "gflop_per_step": flops / 1e9, "algorithmic_mb_per_step": abytes / 1e6},
        "roofline": roof,
    }

    if timeline is not None:
        out["timeline"] = timeline

    if not args.no_eager:
        import torch.nn.functional as F

        def eager(i):
            X, W, _ = sets[i % n_sets]
            return F.layer_norm(F.gelu(F.linear(X, W, b)), (N,), gamma, beta, eps)

        n_e = max(5, args.steps // 4)
        for i in range(5):
            eager(i)
        torch.cuda.synchronize()
        e0 = time.perf_counter()
        for i in range(n_e):
            eager(i)
        torch.cuda.synchronize()
        e_ms = (time.perf_counter() - e0) * 1e3 / n_e
        out["pytorch_eager"] = {"ms_per_step": e_ms, "speedup_of_fused": e_ms / ms_per_step,
                                "note": "unfused layer_norm(gelu(linear())) in the same dtype on the same GPU"}

    if not args.no_cpu_baseline:
        import numpy as np
        import oracle
        arrs = [d[k].float().numpy() for k in ("X", "W", "b", "gamma", "beta")]
        threads = oracle.num_threads()
        probe = min(M, threads)
        c0 = time.perf_counter()
        oracle.fused_linear_gelu_ln(*arrs, eps, rows=list(range(probe)))
        rows_per_s = probe / max(time.perf_counter() - c0, 1e-9)
        n_rows = max(1, min(M, max(probe, int(args.cpu_seconds * rows_per_s))))
        rows = np.linspace(0, M - 1, n_rows).astype(np.int64)
        c0 = time.perf_counter()
        oracle.fused_linear_gelu_ln(*arrs, eps, rows=rows)
        c_s = time.perf_counter() - c0
        frac = n_rows / M
        if hbm_bound:
            c_val, c_unit = abytes * frac / c_s / 1e9, "GB/s"
        else:
            c_val, c_unit = flops * frac / c_s / 1e12, "TFLOP/s"
        out["cpu_baseline"] = {"value": c_val, "unit": c_unit, "cores": threads, "kind": "oracle",
                               "sample": "%d of %d rows (complete rows, all N columns) in %.1f s; rate scaled to the full matrix"
                                         % (n_rows, M, c_s)}
    print(json.dumps(out))
    return 0


def bench_rowmean(args, torch, B) -> int:
    """Second fused chain on bf16 M = K = N = 4096: HBM-bound (W and X read once, Out written once)."""
    import numpy as np
    import torch.nn.functional as F
    import oracle
    from paper_2511_01884_amd.inputs import make_inputs

    M = K = N = 4096
    d = make_inputs(M, K, N, "bf16", seed=0)
    g = torch.Generator(device="cpu").manual_seed(777)
    s_vec = (torch.rand(N, generator=g) * 0.2 - 0.1).to(torch.bfloat16)
    abytes = (N * K + 2 * M * K + 2 * N) * 2
    n_sets = 5
    b, sv = d["b"].cuda(), s_vec.cuda()
    X0, W0 = d["X"].cuda(), d["W"].cuda()
    sets = [(X0 if i == 0 else X0.clone(), W0 if i == 0 else W0.clone(), torch.empty_like(X0)) for i in range(n_sets)]

    def step(i):
        X, W, Out = sets[i % n_sets]
        B.ff_fused_linear_sub_rowmean_gelu_residual(X, W, b, sv, Out=Out)

    preheat(torch, step, args.preheat_ms)
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    ev0 = torch.cuda.Event(enable_timing=True)
    ev1 = torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for i in range(args.steps):
        step(i)
    ev1.record()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    ms_kernel = ev0.elapsed_time(ev1) / args.steps
    out = {
        "metric": "TFLOP/s and % of bf16 MFMA peak (GB/s for small-M) for fused linear+GELU+LN",
        "value": abytes / (ms_per_step * 1e-3) / 1e9, "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "rowmean: bf16 Linear -> subtract -> row-mean -> GELU -> residual add, M=K=N=4096",
                   "buffer_sets": n_sets, "algorithmic_mb_per_step": abytes / 1e6,
                   "note": "one launch per step"},
        "roofline": {"bound": "hbm", "achieved": abytes / (ms_kernel * 1e-3) / 1e9, "peak": PEAK_HBM_GBS,
                     "unit": "GB/s", "frac": abytes / (ms_kernel * 1e-3) / 1e9 / PEAK_HBM_GBS,
                     "traffic": measured_traffic("rowmean"), "kernel_ms": ms_kernel},
    }
    if not args.no_extras:
        out["roofline"]["batch_median_ms"] = batch_median_ms(torch, step)
        out["roofline"]["sustained"] = sustained_ceiling(torch, B, "hbm")
        out["roofline"]["frac_of_sustained"] = out["roofline"]["achieved"] / out["roofline"]["sustained"]["value"]
    if not args.no_eager:
        def eager(i):
            X, W, _ = sets[i % n_sets]
            return X + F.gelu((F.linear(X, W, b) - sv).mean(dim=1, keepdim=True))
        for i in range(5):
            eager(i)
        torch.cuda.synchronize()
        e0 = time.perf_counter()
        n_e = max(5, args.steps // 4)
        for i in range(n_e):
            eager(i)
        torch.cuda.synchronize()
        e_ms = (time.perf_counter() - e0) * 1e3 / n_e
        out["pytorch_eager"] = {"ms_per_step": e_ms, "speedup_of_fused": e_ms / ms_per_step,
                                "note": "unfused composition in bf16 on the same GPU (runs the full GEMM)"}
    if not args.no_cpu_baseline:
        arrs = [d["X"].float().numpy(), d["W"].float().numpy(), d["b"].float().numpy(), s_vec.float().numpy()]
        threads = oracle.num_threads()
        c0 = time.perf_counter()
        oracle.linear_sub_rowmean_gelu_residual(*arrs, rows=list(range(threads)))
        rows_per_s = threads / max(time.perf_counter() - c0, 1e-9)
        n_rows = max(1, min(M, int(args.cpu_seconds * rows_per_s)))
        rows = np.linspace(0, M - 1, n_rows).astype(np.int64)
        c0 = time.perf_counter()
        oracle.linear_sub_rowmean_gelu_residual(*arrs, rows=rows)
        c_s = time.perf_counter() - c0
        out["cpu_baseline"] = {"value": abytes * (n_rows / M) / c_s / 1e9, "unit": "GB/s", "cores": threads,
                               "kind": "oracle",
                               "sample": "%d of %d rows in %.1f s (the oracle evaluates the full linear layer per row); "
                                         "rate scaled to the full matrix" % (n_rows, M, c_s)}
    print(json.dumps(out))
    return 0


def bench_copy(args, torch, B) -> int:
    """The library's plain copy kernel on 256 MiB: the kernel of known traffic that scales the byte counters."""
    nbytes = 256 << 20
    src = torch.empty(nbytes, dtype=torch.uint8, device="cuda").random_(0, 255)
    dst = torch.empty_like(src)
    for _ in range(args.warmup):
        B.ff_debug_copy(src, dst)
    torch.cuda.synchronize()
    ev0 = torch.cuda.Event(enable_timing=True)
    ev1 = torch.cuda.Event(enable_timing=True)
    ev0.record()
    for _ in range(args.steps):
        B.ff_debug_copy(src, dst)
    ev1.record()
    torch.cuda.synchronize()
    assert torch.equal(src, dst)
    ms = ev0.elapsed_time(ev1) / args.steps
    print(json.dumps({"metric": "copy kernel, bytes read + written per second", "value": 2 * nbytes / (ms * 1e-3) / 1e9,
                      "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
                      "higher_is_better": True, "dtype": "u8", "data": "synthetic",
                      "config": {"workload": "copy: 256 MiB device-to-device, counter calibration"}}))
    return 0


def bench_xent(args, torch, B) -> int:
    """Row-wise cross-entropy with mean on fp32 logits [32768, 4096]: HBM-bound, the logits are read once."""
    import torch.nn.functional as F
    import oracle
    from paper_2511_01884_amd.inputs import make_xent_inputs

    Bn, C = 32768, 4096
    logits, targets = make_xent_inputs(Bn, C, "f32", seed=0)
    abytes = Bn * C * 4 + Bn * 8 + 4  # logits and targets read once, the mean written
    n_sets = 2
    sets = [(logits.cuda(), targets.cuda(), torch.empty(1, device="cuda")) for _ in range(n_sets)]

    def step(i):
        L, t, out = sets[i % n_sets]
        B.ff_cross_entropy_mean(L, t, mean_loss=out)

    preheat(torch, step, args.preheat_ms)
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    ev0 = torch.cuda.Event(enable_timing=True)
    ev1 = torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for i in range(args.steps):
        step(i)
    ev1.record()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    ms_kernel = ev0.elapsed_time(ev1) / args.steps
    out = {
        "metric": "TFLOP/s and % of bf16 MFMA peak (GB/s for small-M) for fused linear+GELU+LN",
        "value": abytes / (ms_per_step * 1e-3) / 1e9, "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "xent: row-wise cross-entropy with mean, fp32 logits [32768, 4096], int64 targets",
                   "buffer_sets": n_sets, "algorithmic_mb_per_step": abytes / 1e6},
        "roofline": {"bound": "hbm", "achieved": abytes / (ms_kernel * 1e-3) / 1e9, "peak": PEAK_HBM_GBS,
                     "unit": "GB/s", "frac": abytes / (ms_kernel * 1e-3) / 1e9 / PEAK_HBM_GBS,
                     "traffic": measured_traffic("xent"), "kernel_ms": ms_kernel},
    }
    if not args.no_extras:
        out["roofline"]["batch_median_ms"] = batch_median_ms(torch, step)
        out["roofline"]["sustained"] = sustained_ceiling(torch, B, "hbm")
        out["roofline"]["frac_of_sustained"] = out["roofline"]["achieved"] / out["roofline"]["sustained"]["value"]
    if not args.no_eager:
        def eager(i):
            L, t, _ = sets[i % n_sets]
            return F.cross_entropy(L, t)
        for i in range(5):
            eager(i)
        torch.cuda.synchronize()
        e0 = time.perf_counter()
        n_e = max(5, args.steps // 4)
        for i in range(n_e):
            eager(i)
        torch.cuda.synchronize()
        e_ms = (time.perf_counter() - e0) * 1e3 / n_e
        out["pytorch_eager"] = {"ms_per_step": e_ms, "speedup_of_fused": e_ms / ms_per_step,
                                "note": "torch.nn.functional.cross_entropy on the same GPU"}
    if not args.no_cpu_baseline:
        threads = oracle.num_threads()
        Ln, tn = logits.numpy(), targets.numpy()
        c0 = time.perf_counter()
        oracle.cross_entropy(Ln[:1024], tn[:1024])
        rows_per_s = 1024 / max(time.perf_counter() - c0, 1e-9)
        n_rows = max(1024, min(Bn, int(args.cpu_seconds * rows_per_s)))
        c0 = time.perf_counter()
        oracle.cross_entropy(Ln[:n_rows], tn[:n_rows])
        c_s = time.perf_counter() - c0
        out["cpu_baseline"] = {"value": abytes * (n_rows / Bn) / c_s / 1e9, "unit": "GB/s", "cores": threads,
                               "kind": "oracle", "sample": "first %d of %d rows in %.2f s" % (n_rows, Bn, c_s)}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
