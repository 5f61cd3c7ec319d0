"""Shared pieces of the GPU parity tests: run the library and the oracle on the
same seeded inputs and apply the tolerance gates.

Gates (written here so every test uses the same reading):
  fp32:  max |Y_gpu - Y_oracle| <= 1e-4 (the paper's correctness tolerance, Sec. 2.2).
  bf16:  mean |err| <= 2e-3; max |err| <= 2e-2 on elements with |Y_oracle| < 8.
         A bf16 output cannot meet 2e-2 where |y| >= 8 (half an ulp there is
         3.1e-2), so on those elements the gate is half a bf16 ulp of the exact
         value plus 4e-3, and their count is reported.  In addition the result
         must be within one bf16 ulp (plus 5e-5 of fp32 compute error, which
         dominates the ulp for outputs near zero) of the correctly rounded
         oracle value.
"""
from __future__ import annotations

import numpy as np
import torch

import oracle
from paper_2511_01884_amd import binding as B

F32_MAX_ABS = 1e-4
BF16_MAX_ABS = 2e-2
BF16_MEAN_ABS = 2e-3


def to_np32(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy()


def oracle_on(d, rows=None, stages=False):
    return oracle.fused_linear_gelu_ln(
        to_np32(d["X"]), to_np32(d["W"]),
        None if d.get("b") is None else to_np32(d["b"]),
        None if d.get("gamma") is None else to_np32(d["gamma"]),
        None if d.get("beta") is None else to_np32(d["beta"]),
        d["eps"], rows=rows, stages=stages)


def gpu_run(d, variant=B.FF_VARIANT_AUTO, check=True):
    dev = {k: (v.cuda() if isinstance(v, torch.Tensor) else v) for k, v in d.items()}
    B.ff_debug_force_variant(variant)
    try:
        Y = B.ff_fused_linear_gelu_ln(dev["X"], dev["W"], dev.get("b"), dev.get("gamma"),
                                      dev.get("beta"), d["eps"])
        used = B.ff_last_variant()
    finally:
        B.ff_debug_force_variant(B.FF_VARIANT_AUTO)
    if check:
        B.ff_check_device()
    torch.cuda.synchronize()
    return Y, used


def bf16_ulp(x: np.ndarray) -> np.ndarray:
    """Spacing of bf16 values at |x| (8 significant bits)."""
    ax = np.maximum(np.abs(x), 2.0 ** -126)
    return 2.0 ** (np.floor(np.log2(ax)) - 7)


def check_against_oracle(Y_gpu: torch.Tensor, Y64: np.ndarray, dtype: str, label: str = ""):
    """Applies the gates; returns a dict of the error figures."""
    got = Y_gpu.detach().float().cpu().numpy().astype(np.float64)
    assert got.shape == Y64.shape, (got.shape, Y64.shape)
    assert np.all(np.isfinite(got)), label + ": non-finite output"
    err = np.abs(got - Y64)
    stats = {"max_abs": float(err.max()), "mean_abs": float(err.mean())}
    if dtype == "f32":
        assert stats["max_abs"] <= F32_MAX_ABS, (label, stats)
        return stats
    big = np.abs(Y64) >= 8.0
    stats["n_big"] = int(big.sum())
    small_max = float(err[~big].max()) if (~big).any() else 0.0
    stats["max_abs_below8"] = small_max
    assert stats["mean_abs"] <= BF16_MEAN_ABS, (label, stats)
    assert small_max <= BF16_MAX_ABS, (label, stats)
    if big.any():
        bound = 0.5 * bf16_ulp(Y64[big]) + 4e-3
        assert np.all(err[big] <= bound), (label, stats, float((err[big] - bound).max()))
    Yq = oracle.round_bf16(Y64)
    excess = np.maximum(np.abs(got - Yq) - 5e-5, 0.0) / bf16_ulp(Y64)
    stats["max_ulp_vs_rounded"] = float(excess.max())
    assert stats["max_ulp_vs_rounded"] <= 1.0 + 1e-9, (label, stats)
    return stats
