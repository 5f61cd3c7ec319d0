"""GPU parity of the row-wise cross-entropy (the row reduction of the paper's case study:
row maximum, sum of exponentials, target pick, mean over rows) against the fp64 oracle."""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2511_01884_amd import binding as B
from paper_2511_01884_amd.inputs import make_xent_inputs

pytestmark = pytest.mark.gpu

# fp32 arithmetic gate of the correctness tests (Sec. 2.2 of the paper: 1e-4); bf16 logits are
# widened exactly and the arithmetic is fp32 either way, so the same gate applies
GATE = 1e-4


def _run(logits, targets):
    mean, rows = B.ff_cross_entropy_mean(logits.cuda(), targets.cuda(), with_rows=True)
    torch.cuda.synchronize()
    return float(mean.cpu()[0]), rows.cpu().double().numpy()


def _check(logits, targets, what):
    mean, rows = _run(logits, targets)
    ref_rows, ref_mean = oracle.cross_entropy(logits.float().numpy(), targets.numpy())
    err = np.abs(rows - ref_rows)
    print("[xent] %s: max_abs_row=%.3e mean_abs_row=%.3e mean_err=%.3e" %
          (what, err.max(), err.mean(), abs(mean - ref_mean)), flush=True)
    assert err.max() <= GATE, what
    assert abs(mean - ref_mean) <= GATE, what
    return rows, mean


# (B, C, dtype, scale): rows that are not a multiple of 16 bytes (element loads), a wavefront per row
# (B >= 4096 with short rows) and a workgroup per row, ragged tails of the 8-deep load batches,
# one row, one class
CASES = [(64, 10, "f32", 1.0), (33, 1000, "f32", 1.0), (129, 4096, "f32", 4.0), (7, 50257, "f32", 1.0),
         (5000, 512, "bf16", 1.0), (4100, 36, "f32", 8.0), (3, 131072, "bf16", 2.0), (1, 1, "f32", 1.0),
         (4097, 7, "bf16", 1.0), (4200, 2052, "f32", 1.0), (2, 8200, "bf16", 1.0), (4096, 8, "bf16", 1.0)]


@pytest.mark.parametrize("Bn,C,dtype,scale", CASES)
def test_xent_parity(Bn, C, dtype, scale):
    print("[case] xent", Bn, C, dtype, scale, flush=True)
    logits, targets = make_xent_inputs(Bn, C, dtype, seed=5, scale=scale)
    _check(logits, targets, "%dx%d %s" % (Bn, C, dtype))


def test_xent_full_size_and_repeatable():
    """The benchmark's shape, every row against the oracle; two runs give the same bits; the mean is
    the mean of the per-row losses."""
    Bn, C = 32768, 4096
    logits, targets = make_xent_inputs(Bn, C, "f32", seed=0)
    print("[case] xent full size", Bn, C, flush=True)
    rows, mean = _check(logits, targets, "32768x4096 f32")
    Ld, td = logits.cuda(), targets.cuda()
    m1, r1 = B.ff_cross_entropy_mean(Ld, td, with_rows=True)
    m2, r2 = B.ff_cross_entropy_mean(Ld, td, with_rows=True)
    m3 = B.ff_cross_entropy_mean(Ld, td)  # without the per-row output
    torch.cuda.synchronize()
    assert torch.equal(m1, m2) and torch.equal(r1, r2) and torch.equal(m1, m3)
    assert abs(float(m1.cpu()[0]) - rows.mean()) <= 1e-5
    assert abs(mean - (math.log(C) + 0.5)) < 0.05  # E[loss] for unit-normal scores is about log C + 1/2


def test_xent_extreme_values():
    """Large offsets (exp overflows unless the running maximum is removed), -inf entries (masked
    classes), the maximum in any lane and any position, equal rows."""
    C = 1000
    logits, targets = make_xent_inputs(300, C, "f32", seed=6)
    logits[:100] += 1000.0
    logits[100:200] -= 30000.0
    logits[200:250, ::3] = -float("inf")
    targets[200:250] = torch.clamp((targets[200:250] // 3) * 3 + 1, max=C - 3)  # a class that is not masked
    for r in range(250, 300):
        logits[r, (r * 37) % C] = 80.0 + r
    _check(logits, targets, "extreme")
    # equal logits: log C exactly up to fp32 rounding, for lengths around the load batch sizes
    for C in (1, 3, 64, 255, 256, 257, 2048, 2049, 16384 + 4):
        L = torch.full((5, C), -7.25)
        t = torch.arange(5) % C
        mean, rows = _run(L, t)
        assert np.abs(rows - math.log(C)).max() <= 2e-6 * max(1.0, math.log(C)), (C, rows)


def test_xent_bad_target_gives_nan_row_only():
    logits, targets = make_xent_inputs(4200, 64, "f32", seed=7)
    ref_rows, _ = oracle.cross_entropy(logits.numpy(), targets.numpy())
    targets[17] = 64
    targets[4000] = -100
    mean, rows = _run(logits, targets)
    assert math.isnan(mean) and math.isnan(rows[17]) and math.isnan(rows[4000])
    ok = np.ones(4200, bool)
    ok[[17, 4000]] = False
    assert np.abs(rows[ok] - ref_rows[ok]).max() <= GATE
    # the next call is unaffected
    targets[17] = 0
    targets[4000] = 1
    _check(logits, targets, "after bad targets")


def test_xent_argument_errors():
    L = torch.zeros(4, 8, device="cuda")
    t = torch.zeros(4, dtype=torch.int64, device="cuda")
    with pytest.raises(ValueError):
        B.ff_cross_entropy_mean(L, t.int())
    with pytest.raises(ValueError):
        B.ff_cross_entropy_mean(L, t[:3])
    with pytest.raises(TypeError):
        B.ff_cross_entropy_mean(L.half(), t)
    lib = B.load()
    assert lib.ff_cross_entropy_mean(None, None, 4, 8, 0, None, None, None) == 1      # FF_ERR_NULL
    assert lib.ff_cross_entropy_mean(None, None, 0, 8, 0, None, None, None) == 2      # FF_ERR_SHAPE
    assert lib.ff_cross_entropy_mean(None, None, 4, 8, 7, None, None, None) == 3      # FF_ERR_DTYPE
    assert B.ff_cross_entropy_workspace_bytes(4, 8, 0) > 0 and B.ff_cross_entropy_workspace_bytes(0, 8, 0) == 0


def test_xent_graph_replay_matches_eager():
    """Capturable (no allocation or memset once the workspace exists; the arrival counter is back at zero
    after every launch): every replay, with fresh logits and eager work in between, equals the eager result."""
    Bn, C = 6000, 1500
    logits, targets = make_xent_inputs(Bn, C, "f32", seed=8)
    Ld, td = logits.cuda(), targets.cuda()
    mean_s = torch.empty(1, device="cuda")
    rows_s = torch.empty(Bn, device="cuda")
    B.ff_cross_entropy_mean(Ld, td, row_loss=rows_s, mean_loss=mean_s)   # warm-up: workspace exists
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        with torch.cuda.graph(g, stream=st):
            B.ff_cross_entropy_mean(Ld, td, row_loss=rows_s, mean_loss=mean_s)
    torch.cuda.synchronize()
    for rep in range(4):
        l2, t2 = make_xent_inputs(Bn, C, "f32", seed=300 + rep)
        Ld.copy_(l2.cuda())
        td.copy_(t2.cuda())
        torch.cuda.synchronize()
        m_e, r_e = B.ff_cross_entropy_mean(Ld, td, with_rows=True)
        torch.cuda.synchronize()
        mean_s.zero_()
        rows_s.zero_()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(mean_s, m_e) and torch.equal(rows_s, r_e), "replay %d differs from eager" % rep
    ref_rows, ref_mean = oracle.cross_entropy(Ld.cpu().numpy(), td.cpu().numpy())
    assert np.abs(rows_s.cpu().double().numpy() - ref_rows).max() <= GATE
    assert abs(float(mean_s.cpu()[0]) - ref_mean) <= GATE


def test_xent_full_size_bf16_sampled_against_oracle():
    """bf16 logits at a large size: rows checked one by one on a sample, the mean through the library's rows."""
    Bn, C = 16384, 8192
    logits, targets = make_xent_inputs(Bn, C, "bf16", seed=9, scale=3.0)
    mean, rows = B.ff_cross_entropy_mean(logits.cuda(), targets.cuda(), with_rows=True)
    torch.cuda.synchronize()
    idx = np.unique(np.concatenate([[0, 1, Bn - 1], np.random.default_rng(0).integers(0, Bn, 200)]))
    ref_rows, _ = oracle.cross_entropy(logits[idx].float().numpy(), targets[idx].numpy())
    assert np.abs(rows.cpu().double().numpy()[idx] - ref_rows).max() <= GATE
    assert abs(float(mean.cpu()[0]) - rows.cpu().double().numpy().mean()) <= 1e-5
