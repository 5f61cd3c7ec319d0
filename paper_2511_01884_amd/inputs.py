"""Seeded synthetic inputs for the fused linear + GELU + LayerNorm operator.

This module draws random tensors and nothing else: it holds none of the
operator's arithmetic, so both the GPU library's tests and the CPU oracle's
tests may use it.  The tensors stand in for the multi-step operator tasks the
paper evaluates on (Sec. 3.1), whose task files are not reproduced here.

Recipe (host generator, one stream per call, draw order X, W, b, gamma, beta,
all drawn in float32, then rounded to nearest-even to the storage dtype; the
rounded values are what every consumer sees):
    X     ~ N(0, 1)                      [M, K]
    W     ~ N(0, variance 1/K)           [N, K]   (so X W^T has unit variance)
    b     ~ U(-0.1, 0.1)                 [N]
    gamma = 1 + 0.1 * N(0, 1)            [N]      (all ones in the plain variant)
    beta  = 0.1 * N(0, 1)                [N]      (all zeros in the plain variant)
    eps   = 1e-5
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict

import torch

EPS = 1e-5


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str  # "f32" or "bf16"
    M: int
    K: int
    N: int
    note: str


# The synthetic workloads the build is measured on: five for the main metric, then the
# fp32 path at a large shape.
CONFIGS: Dict[str, Workload] = {
    "cfg0": Workload("cfg0", "f32", 256, 512, 512, "fp32 parity case"),
    "cfg1": Workload("cfg1", "bf16", 4096, 4096, 4096, "compute-bound square case"),
    "cfg2": Workload("cfg2", "bf16", 65536, 1024, 1024, "tall-skinny, epilogue-heavy"),
    "cfg3": Workload("cfg3", "bf16", 16, 8192, 8192, "small-M, streams W"),
    "cfg4": Workload("cfg4", "bf16", 8192, 4096, 16384, "wide rows, many N tiles"),
    "f32_4096": Workload("f32_4096", "f32", 4096, 4096, 4096, "fp32 inputs and outputs at the square shape"),
}


def torch_dtype(dtype: str) -> torch.dtype:
    if dtype == "f32":
        return torch.float32
    if dtype == "bf16":
        return torch.bfloat16
    raise ValueError("dtype must be 'f32' or 'bf16'")


def make_inputs(M: int, K: int, N: int, dtype: str = "bf16", seed: int = 0,
                plain_affine: bool = False) -> Dict[str, torch.Tensor]:
    """CPU tensors X, W, b, gamma, beta in the storage dtype, plus eps."""
    td = torch_dtype(dtype)
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    X = torch.randn(M, K, generator=g, dtype=torch.float32)
    W = torch.randn(N, K, generator=g, dtype=torch.float32) * (float(K) ** -0.5)
    b = torch.rand(N, generator=g, dtype=torch.float32) * 0.2 - 0.1
    gamma = 1.0 + 0.1 * torch.randn(N, generator=g, dtype=torch.float32)
    beta = 0.1 * torch.randn(N, generator=g, dtype=torch.float32)
    if plain_affine:
        gamma = torch.ones(N, dtype=torch.float32)
        beta = torch.zeros(N, dtype=torch.float32)
    return {
        "X": X.to(td).contiguous(),
        "W": W.to(td).contiguous(),
        "b": b.to(td).contiguous(),
        "gamma": gamma.to(td).contiguous(),
        "beta": beta.to(td).contiguous(),
        "eps": EPS,
    }


def make_integer_inputs(M: int, K: int, N: int, dtype: str = "bf16", seed: int = 0,
                        lo: int = -4, hi: int = 4) -> Dict[str, torch.Tensor]:
    """Integer-valued X, W, b in [lo, hi]: every product and partial sum of the
    linear stage is an exactly representable integer for K * hi * hi < 2**24."""
    td = torch_dtype(dtype)
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    X = torch.randint(lo, hi + 1, (M, K), generator=g).to(td)
    W = torch.randint(lo, hi + 1, (N, K), generator=g).to(td)
    b = torch.randint(lo, hi + 1, (N,), generator=g).to(td)
    return {"X": X.contiguous(), "W": W.contiguous(), "b": b.contiguous()}


def make_xent_inputs(B: int, C: int, dtype: str = "f32", seed: int = 0, scale: float = 1.0):
    """Logits ~ scale * N(0, 1) [B, C] rounded to the storage dtype, targets uniform in [0, C)
    (int64), drawn in that order from one host stream: the shape of input the paper's row-reduction
    case study (Sec. 4) runs on, a batch of score rows and one class index per row."""
    g = torch.Generator(device="cpu").manual_seed(seed)
    logits = (torch.randn(B, C, generator=g, dtype=torch.float32) * scale).to(torch_dtype(dtype))
    targets = torch.randint(0, C, (B,), generator=g, dtype=torch.int64)
    return logits, targets


def make_metric_inputs(n: int, V: int, J: int, seed: int = 0):
    """Synthetic profile dumps for the metric-selection procedure (Sec. 2.3): n tasks, V kernels per
    task, J metrics.  runtime[i][v] is log-normal; metric m follows the runtime with a per-metric
    strength in [-1, 1] (jittered per task, so some metrics flip sign or fade between tasks) plus
    noise, at counter-like magnitudes from 1 to 1e9; every 17th metric is constant, every 19th is an
    exact copy of its left neighbour, every 23rd an affine image of it.  float64 tensors
    values [n,V,J], runtime [n,V]."""
    g = torch.Generator(device="cpu").manual_seed(seed)
    runtime = torch.exp(0.5 * torch.randn(n, V, generator=g, dtype=torch.float64))
    z = (runtime - runtime.mean(dim=1, keepdim=True)) / runtime.std(dim=1, keepdim=True, unbiased=False).clamp_min(1e-30)
    strength = torch.rand(J, generator=g, dtype=torch.float64) * 2 - 1
    jitter = 0.5 * torch.randn(n, J, generator=g, dtype=torch.float64)
    a = (strength[None, :] + jitter).clamp(-1, 1)
    noise = torch.randn(n, V, J, generator=g, dtype=torch.float64)
    scale = torch.pow(10.0, torch.rand(J, generator=g, dtype=torch.float64) * 9)
    offset = scale * (torch.rand(J, generator=g, dtype=torch.float64) * 4)
    values = scale * (a[:, None, :] * z[:, :, None] + torch.sqrt(1 - a * a)[:, None, :] * noise) + offset
    for m in range(J):
        if m % 17 == 16:
            values[:, :, m] = offset[m]
        elif m % 19 == 18 and m > 0:
            values[:, :, m] = values[:, :, m - 1]
        elif m % 23 == 22 and m > 0:
            values[:, :, m] = 3.0 * values[:, :, m - 1] + 1.0
    return values.contiguous(), runtime.contiguous()


def sample_rows(M: int, n: int, tile: int = 256, seed: int = 0):
    """Row indices for sampled checks at full size: the rows next to tile
    boundaries plus seeded random rows, sorted and unique."""
    fixed = {0, M - 1}
    for r in (tile - 1, tile, M - tile - 1, M - tile):
        if 0 <= r < M:
            fixed.add(r)
    g = torch.Generator(device="cpu")
    g.manual_seed(seed + 12345)
    extra = torch.randint(0, M, (max(0, n - len(fixed)),), generator=g).tolist()
    return sorted(fixed.union(extra))
