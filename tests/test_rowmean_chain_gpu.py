"""GPU parity of the second fused chain (Linear -> subtract -> row-mean -> GELU -> residual add,
the paper's fused-epilogue case study) against the fp64 oracle, which evaluates the chain the
long way (full linear layer, then the mean)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2511_01884_amd import binding as B
from paper_2511_01884_amd.inputs import make_inputs, sample_rows
from parity_util import check_against_oracle, to_np32

pytestmark = pytest.mark.gpu


def _inputs(M, K, N, dtype, seed):
    d = make_inputs(M, K, N, dtype, seed=seed)
    # the subtract vector: the same recipe as the bias, from the next draws of the stream
    g = torch.Generator(device="cpu").manual_seed(seed + 777)
    s = (torch.rand(N, generator=g) * 0.2 - 0.1).to(d["X"].dtype)
    return d["X"], d["W"], d["b"], s


CASES = [(37, 72, 40, "bf16"), (300, 200, 520, "f32"), (5, 8, 8, "bf16"), (1, 8, 8, "f32"),
         (1030, 1024, 2048, "bf16"), (9, 16896, 24, "bf16"), (6, 8448, 16, "f32"),
         (3, 32768, 40, "bf16"), (2, 32768, 8, "f32"),     # the longest supported rows (128 KiB of LDS)
         (5000, 72, 1000, "bf16")]                         # several rows per wavefront, short rows


@pytest.mark.parametrize("M,K,N,dtype", CASES)
def test_rowmean_chain_parity(M, K, N, dtype):
    print("[case] rowmean", M, K, N, dtype, flush=True)
    X, W, b, s = _inputs(M, K, N, dtype, seed=31)
    Out = B.ff_fused_linear_sub_rowmean_gelu_residual(X.cuda(), W.cuda(), b.cuda(), s.cuda())
    torch.cuda.synchronize()
    ref = oracle.linear_sub_rowmean_gelu_residual(to_np32(X), to_np32(W), to_np32(b), to_np32(s))
    print(check_against_oracle(Out, ref, dtype, "rowmean %dx%dx%d" % (M, K, N)))


def test_rowmean_chain_full_size_sampled_rows_and_in_place():
    M = K = N = 4096
    X, W, b, s = _inputs(M, K, N, "bf16", seed=0)
    Xd = X.cuda()
    Out = B.ff_fused_linear_sub_rowmean_gelu_residual(Xd, W.cuda(), b.cuda(), s.cuda())
    torch.cuda.synchronize()
    rows = sample_rows(M, 48)
    ref = oracle.linear_sub_rowmean_gelu_residual(to_np32(X), to_np32(W), to_np32(b), to_np32(s), rows=rows)
    print(check_against_oracle(Out[torch.tensor(rows)], ref, "bf16", "rowmean 4096^3"))
    # in place (Out aliases X) gives the same bits, and so does a second run
    again = B.ff_fused_linear_sub_rowmean_gelu_residual(Xd, W.cuda(), b.cuda(), s.cuda())
    inplace = B.ff_fused_linear_sub_rowmean_gelu_residual(Xd, W.cuda(), b.cuda(), s.cuda(), Out=Xd)
    torch.cuda.synchronize()
    assert torch.equal(again, Out) and torch.equal(inplace, Out)


def test_rowmean_chain_optional_vectors_and_errors():
    X, W, b, s = _inputs(64, 64, 128, "bf16", seed=32)
    Out = B.ff_fused_linear_sub_rowmean_gelu_residual(X.cuda(), W.cuda(), None, None)
    ref = oracle.linear_sub_rowmean_gelu_residual(to_np32(X), to_np32(W))
    check_against_oracle(Out, ref, "bf16")
    with pytest.raises(B.FFError) as e:
        B.ff_fused_linear_sub_rowmean_gelu_residual(torch.zeros(4, 12, device="cuda", dtype=torch.bfloat16),
                                                    torch.zeros(8, 12, device="cuda", dtype=torch.bfloat16),
                                                    None, None)
    assert e.value.status == 5


def test_rowmean_chain_rows_too_long_are_refused():
    X = torch.zeros(2, 32776, device="cuda", dtype=torch.bfloat16)
    W = torch.zeros(8, 32776, device="cuda", dtype=torch.bfloat16)
    with pytest.raises(B.FFError) as e:
        B.ff_fused_linear_sub_rowmean_gelu_residual(X, W, None, None)
    assert e.value.status == 5


def test_rowmean_chain_expired_wait_is_reported_not_hung():
    """Forced from the host: the grid-wide arrival waits for one workgroup more than exists, with a
    3 ms limit.  The kernel must finish, flag the device error once, and the next call must be right."""
    X, W, b, s = _inputs(700, 520, 264, "bf16", seed=33)
    B.ff_debug_set_wait_limit_us(3000)
    B.ff_debug_expect_extra_arrivals(1)
    try:
        B.ff_fused_linear_sub_rowmean_gelu_residual(X.cuda(), W.cuda(), b.cuda(), s.cuda())
        with pytest.raises(B.FFError) as e:
            B.ff_check_device()
        assert e.value.status == 8
    finally:
        B.ff_debug_expect_extra_arrivals(0)
        B.ff_debug_set_wait_limit_us(2000000)
    B.ff_check_device()
    Out = B.ff_fused_linear_sub_rowmean_gelu_residual(X.cuda(), W.cuda(), b.cuda(), s.cuda())
    B.ff_check_device()
    ref = oracle.linear_sub_rowmean_gelu_residual(to_np32(X), to_np32(W), to_np32(b), to_np32(s))
    check_against_oracle(Out, ref, "bf16")


def test_rowmean_chain_graph_replay_matches_eager():
    """Capturable (no allocation or memset once the workspace exists; the counters re-arm themselves):
    every replay, with fresh inputs and eager work in between, equals the eager result bit for bit."""
    M, K, N = 2500, 1032, 776
    X, W, b, s = _inputs(M, K, N, "bf16", seed=34)
    Xd, Wd, bd, sd = X.cuda(), W.cuda(), b.cuda(), s.cuda()
    out_static = torch.empty_like(Xd)
    B.ff_fused_linear_sub_rowmean_gelu_residual(Xd, Wd, bd, sd, Out=out_static)   # warm-up: workspace exists
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        with torch.cuda.graph(g, stream=st):
            B.ff_fused_linear_sub_rowmean_gelu_residual(Xd, Wd, bd, sd, Out=out_static)
    torch.cuda.synchronize()
    for rep in range(4):
        X2, W2, _, _ = _inputs(M, K, N, "bf16", seed=200 + rep)
        Xd.copy_(X2.cuda())
        Wd.copy_(W2.cuda())
        torch.cuda.synchronize()
        eager = B.ff_fused_linear_sub_rowmean_gelu_residual(Xd, Wd, bd, sd).clone()
        torch.cuda.synchronize()
        out_static.zero_()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out_static, eager), "replay %d differs from eager" % rep
    B.ff_check_device()
    ref = oracle.linear_sub_rowmean_gelu_residual(to_np32(Xd.cpu()), to_np32(Wd.cpu()), to_np32(b), to_np32(s),
                                                  rows=list(range(0, M, 97)))
    check_against_oracle(out_static[torch.arange(0, M, 97)], ref, "bf16")
