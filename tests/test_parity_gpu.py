"""GPU parity tests: the HIP library against the fp64 CPU oracle on the same
seeded inputs, element by element (small and ragged shapes), on sampled rows at
the full benchmark sizes, plus the edge cases and invariants of the method."""
import numpy as np
import pytest
import torch

import oracle
from paper_2511_01884_amd import binding as B
from paper_2511_01884_amd.inputs import (CONFIGS, make_inputs, make_integer_inputs, sample_rows)
from parity_util import check_against_oracle, gpu_run, oracle_on, to_np32

pytestmark = pytest.mark.gpu

AUTO, FUSED, TWOPASS, SMALLM = (B.FF_VARIANT_AUTO, B.FF_VARIANT_TILED_FUSED,
                                B.FF_VARIANT_TILED_TWOPASS, B.FF_VARIANT_SMALL_M)


def _announce(*a):
    print("[case]", *a, flush=True)


# ------------------------------------------------------------ element by element
SMALL_CASES = [
    # (M, K, N, dtype, variant, expected variant)
    (256, 512, 512, "f32", AUTO, FUSED),        # the fp32 parity workload
    (256, 512, 512, "f32", TWOPASS, TWOPASS),
    (77, 36, 132, "f32", AUTO, FUSED),          # ragged M, K, N; 128-tiles
    (300, 200, 520, "bf16", AUTO, FUSED),       # ragged everything, K tail of 8
    (300, 200, 520, "bf16", TWOPASS, TWOPASS),
    (129, 64, 8, "bf16", AUTO, FUSED),          # one 8-column tile
    (1, 8, 8, "bf16", FUSED, FUSED),            # smallest legal shape, tiled path
    (2085, 264, 4088, "bf16", AUTO, FUSED),     # 256-tiles, 9 x 16 tiles, ragged
    (2085, 264, 4088, "bf16", TWOPASS, TWOPASS),
    (2100, 96, 2048, "f32", AUTO, FUSED),       # fp32 on 256-tiles
    (40, 128, 1024, "bf16", AUTO, FUSED),       # just above the small-M limit
    (1000, 520, 5004, "f32", AUTO, FUSED),      # fp32, N neither a power of two nor a tile multiple
    (513, 1028, 1284, "f32", TWOPASS, TWOPASS), # fp32, K with a 4-element tail, two-pass
]


@pytest.mark.parametrize("M,K,N,dtype,variant,expect", SMALL_CASES)
def test_full_matrix_parity(M, K, N, dtype, variant, expect):
    _announce("full", M, K, N, dtype, variant)
    d = make_inputs(M, K, N, dtype, seed=11)
    Y, used = gpu_run(d, variant)
    assert used == expect
    stats = check_against_oracle(Y, oracle_on(d), dtype, "%dx%dx%d" % (M, K, N))
    print(stats)


@pytest.mark.parametrize("tile,per_cu", [(64, 1), (64, 2), (128, 1), (128, 2), (256, 1), (256, 2)])
@pytest.mark.parametrize("variant", [FUSED, TWOPASS])
def test_forced_tile_shapes_parity(tile, per_cu, variant):
    """The tile shapes the automatic plan does not pick for this size are kernels of the same
    operator (used as distinct variants by the profiling-metric study): same gates."""
    _announce("forced tile", tile, per_cu, variant)
    d = make_inputs(1300, 520, 2056, "bf16", seed=14)
    B.ff_debug_force_tile(tile, per_cu)
    try:
        Y, used = gpu_run(d, variant)
    finally:
        B.ff_debug_force_tile(0, 0)
    assert used == variant
    print(check_against_oracle(Y, oracle_on(d), "bf16", "tile %d x%d" % (tile, per_cu)))
    with pytest.raises(B.FFError):
        B.ff_debug_force_tile(256, 3)
    with pytest.raises(B.FFError):
        B.ff_debug_force_tile(32, 1)


@pytest.mark.parametrize("M,K,N,dtype", [(256, 512, 512, "f32"), (77, 36, 132, "f32"), (129, 64, 8, "bf16"),
                                         (1, 8, 8, "bf16"), (200, 1000, 72, "bf16")])
def test_64_tiles_small_shapes(M, K, N, dtype):
    """The smallest tile shape on small and ragged problems, fused and two-pass."""
    _announce("tile 64", M, K, N, dtype)
    d = make_inputs(M, K, N, dtype, seed=15)
    ref = oracle_on(d)
    for variant in (FUSED, TWOPASS):
        B.ff_debug_force_tile(64, 0)
        try:
            Y, used = gpu_run(d, variant)
        finally:
            B.ff_debug_force_tile(0, 0)
        assert used == variant
        print(check_against_oracle(Y, ref, dtype, "tile 64 %dx%dx%d" % (M, K, N)))


SMALLM_CASES = [(16, 8192, 8192), (16, 1024, 1024), (5, 520, 1000), (32, 1024, 2048),
                (17, 72, 40), (1, 8, 8), (16, 4096, 32768), (9, 256, 16384 + 64)]


@pytest.mark.parametrize("M,K,N", SMALLM_CASES)
def test_small_m_streamer_parity(M, K, N):
    _announce("small-m", M, K, N)
    d = make_inputs(M, K, N, "bf16", seed=12)
    Y, used = gpu_run(d, AUTO)
    assert used == SMALLM
    stats = check_against_oracle(Y, oracle_on(d), "bf16", "smallm %dx%dx%d" % (M, K, N))
    print(stats)


def test_small_m_shape_through_tiled_path_agrees():
    """The same small-M problem through the tiled kernels must meet the same gates."""
    d = make_inputs(16, 1024, 1024, "bf16", seed=12)
    Y, used = gpu_run(d, FUSED)
    assert used == FUSED
    check_against_oracle(Y, oracle_on(d), "bf16")


# ------------------------------------------------------------- exact GEMM stage
@pytest.mark.parametrize("M,K,N,dtype", [(300, 200, 520, "bf16"), (2085, 264, 4088, "bf16"),
                                         (512, 4096, 256, "bf16"), (77, 36, 132, "f32"),
                                         (2100, 96, 2048, "f32")])
def test_linear_stage_exact_on_integers(M, K, N, dtype):
    """Integer-valued inputs: every partial sum is an exact integer below 2^24, so the
    MFMA core must reproduce the oracle's Z bit for bit (any summation order)."""
    _announce("exact", M, K, N, dtype)
    d = make_integer_inputs(M, K, N, dtype, seed=13)
    Z = B.ff_debug_linear(d["X"].cuda(), d["W"].cuda(), d["b"].cuda())
    torch.cuda.synchronize()
    ref = oracle.fused_linear_gelu_ln(to_np32(d["X"]), to_np32(d["W"]), to_np32(d["b"]),
                                      None, None, 1e-5, stages=True)["Z"]
    assert np.array_equal(Z.cpu().numpy().astype(np.float64), ref)


# ------------------------------------------------- full sizes, sampled rows
@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg3", "cfg4", "f32_4096"])
def test_benchmark_sizes_sampled_rows(name):
    """The launch configuration the benchmark times, checked on complete sampled
    rows (LayerNorm needs whole rows): tile-boundary rows plus seeded random rows."""
    wl = CONFIGS[name]
    _announce("sampled", name)
    d = make_inputs(wl.M, wl.K, wl.N, wl.dtype, seed=0)
    Y, used = gpu_run(d, AUTO)
    assert used == (SMALLM if name == "cfg3" else FUSED)
    rows = list(range(wl.M)) if wl.M <= 64 else sample_rows(wl.M, 48)
    ref = oracle_on(d, rows=rows)
    stats = check_against_oracle(Y[torch.tensor(rows)], ref, wl.dtype, name)
    print(name, stats)
    # property that holds at any size: per-row moments of (Y - beta) / gamma
    g = d["gamma"].float().cuda()
    bta = d["beta"].float().cuda()
    T = (Y.float() - bta) / g
    assert float(T.mean(dim=1).abs().max()) < 2e-2
    assert float((T.var(dim=1, unbiased=False) - 1).abs().max()) < 2e-2


def test_rows_wider_than_the_grid_take_the_two_pass_path_by_themselves():
    """N = 258 tiles of 256 columns: more tiles per row than co-resident workgroups, so the automatic
    plan must pick the two-pass variant (and a forced single-pass must refuse); maximum-width coverage."""
    M, K, N = 40, 64, 258 * 256
    _announce("wide", M, K, N)
    d = make_inputs(M, K, N, "bf16", seed=17)
    Y, used = gpu_run(d, AUTO)
    assert used == TWOPASS
    print(check_against_oracle(Y, oracle_on(d), "bf16", "40x64x66048"))
    with pytest.raises(B.FFError) as e:
        gpu_run(d, FUSED)
    assert e.value.status == 5


@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg4"])
def test_benchmark_sizes_full_matrix(name):
    """Every element of the three large benchmark shapes (the oracle takes seconds to tens of seconds on
    the host's threads), in the launch configuration the benchmark times; a second run must give the
    same bits."""
    wl = CONFIGS[name]
    _announce("full matrix", name)
    d = make_inputs(wl.M, wl.K, wl.N, wl.dtype, seed=0)
    Y, used = gpu_run(d, AUTO)
    assert used == FUSED
    stats = check_against_oracle(Y, oracle_on(d), wl.dtype, name + " full")
    print(name, stats)
    Y2, _ = gpu_run(d, AUTO)
    assert torch.equal(Y, Y2)


def test_wide_rows_plain_affine_moments():
    """gamma = 1, beta = 0 on the wide-row workload: every output row has mean 0 and
    biased variance var/(var+eps) ~ 1, up to bf16 output rounding."""
    wl = CONFIGS["cfg4"]
    d = make_inputs(wl.M, wl.K, wl.N, wl.dtype, seed=0, plain_affine=True)
    Y, used = gpu_run(d, AUTO)
    assert used == FUSED
    Yf = Y.float()
    assert float(Yf.mean(dim=1).abs().max()) < 2e-3
    assert float((Yf.var(dim=1, unbiased=False) - 1).abs().max()) < 5e-3
    rows = sample_rows(wl.M, 16)
    check_against_oracle(Y[torch.tensor(rows)], oracle_on(d, rows=rows), "bf16", "cfg4 plain")


# ------------------------------------------------------------------ edge cases
def test_optional_vectors_default_to_0_1_0():
    d = make_inputs(200, 64, 264, "bf16", seed=14)
    d2 = dict(d, b=None, gamma=None, beta=None)
    Y, _ = gpu_run(d2, AUTO)
    check_against_oracle(Y, oracle_on(d2), "bf16")
    d3 = dict(make_inputs(16, 64, 264, "bf16", seed=14), b=None, gamma=None, beta=None)
    Y, used = gpu_run(d3, AUTO)
    assert used == SMALLM
    check_against_oracle(Y, oracle_on(d3), "bf16")


@pytest.mark.parametrize("M,variant", [(200, AUTO), (16, AUTO)])
def test_constant_rows_give_beta(M, variant):
    """W = 0, constant bias: G is constant along each row, so Y = beta (the
    variance is zero; eps keeps the division finite)."""
    d = make_inputs(M, 64, 512, "bf16", seed=15)
    d["W"] = torch.zeros_like(d["W"])
    d["b"] = torch.full_like(d["b"], 0.75)
    Y, _ = gpu_run(d, variant)
    ref = np.broadcast_to(to_np32(d["beta"]).astype(np.float64), (M, 512))
    assert np.max(np.abs(to_np32(Y).astype(np.float64) - ref)) <= 1e-3


def test_identity_x_transposes_w():
    K = 256
    d = make_inputs(K, K, 512, "f32", seed=16)
    d["X"] = torch.eye(K, dtype=torch.float32)
    Z = B.ff_debug_linear(d["X"].cuda(), d["W"].cuda(), d["b"].cuda())
    want = d["W"].t().double() + d["b"].double()[None, :]
    assert torch.equal(Z.cpu().double(), want.float().double()) or \
        float((Z.cpu().double() - want).abs().max()) < 1e-6


def test_bitwise_deterministic_run_to_run():
    for (M, K, N, dt) in ((2085, 264, 4088, "bf16"), (16, 1024, 4096, "bf16"), (256, 512, 512, "f32")):
        d = make_inputs(M, K, N, dt, seed=17)
        dev = {k: (v.cuda() if isinstance(v, torch.Tensor) else v) for k, v in d.items()}
        outs = []
        for _ in range(3):
            outs.append(B.ff_fused_linear_gelu_ln(dev["X"], dev["W"], dev["b"], dev["gamma"],
                                                  dev["beta"], d["eps"]).clone())
        torch.cuda.synchronize()
        assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])
    B.ff_check_device()


def test_poisoned_caller_workspace():
    """A caller-owned workspace full of NaN bit patterns: nothing may be read before it is written."""
    M, K, N = 600, 128, 1032
    need = B.ff_workspace_bytes(M, K, N, B.FF_BF16)
    assert need > 0
    ws = torch.full((need // 4 + 64,), float("nan"), dtype=torch.float32, device="cuda")
    B.ff_set_workspace(ws)
    try:
        d = make_inputs(M, K, N, "bf16", seed=18)
        Y, _ = gpu_run(d, AUTO)
        check_against_oracle(Y, oracle_on(d), "bf16")
        B.ff_debug_force_variant(TWOPASS)
        assert B.ff_workspace_bytes(M, K, N, B.FF_BF16) > need
        B.ff_debug_force_variant(AUTO)
        with pytest.raises(B.FFError) as e:
            gpu_run(d, TWOPASS)           # bound workspace is too small for the fp32 G
        assert e.value.status == 6
    finally:
        B.ff_debug_force_variant(AUTO)
        B.ff_set_workspace(None)
    Y, _ = gpu_run(d, TWOPASS)             # library-owned workspace again
    check_against_oracle(Y, oracle_on(d), "bf16")


def test_forced_variant_never_substitutes():
    d = make_inputs(64, 64, 64, "bf16", seed=19)
    with pytest.raises(B.FFError) as e:
        gpu_run(d, SMALLM)
    assert e.value.status == 5
    d = make_inputs(8, 64, 64, "f32", seed=19)
    with pytest.raises(B.FFError):
        gpu_run(d, SMALLM)


def test_nonzero_stream():
    d = make_inputs(300, 128, 520, "bf16", seed=20)
    dev = {k: (v.cuda() if isinstance(v, torch.Tensor) else v) for k, v in d.items()}
    s = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        Y = B.ff_fused_linear_gelu_ln(dev["X"], dev["W"], dev["b"], dev["gamma"], dev["beta"], d["eps"])
    s.synchronize()
    check_against_oracle(Y, oracle_on(d), "bf16")


# ------------------------------------------------------- failure path and graphs
@pytest.mark.parametrize("M,K,N", [(600, 128, 1032), (16, 256, 2048)])
def test_expired_wait_is_reported_not_hung(M, K, N):
    """Forced from the host: the kernels wait for one arrival more than will ever
    come, with a 3 ms limit.  They must still finish, flag FF_ERR_DEVICE once, and
    the next ordinary call must be correct again."""
    d = make_inputs(M, K, N, "bf16", seed=21)
    dev = {k: (v.cuda() if isinstance(v, torch.Tensor) else v) for k, v in d.items()}
    B.ff_debug_set_wait_limit_us(3000)
    B.ff_debug_expect_extra_arrivals(1)
    try:
        B.ff_fused_linear_gelu_ln(dev["X"], dev["W"], dev["b"], dev["gamma"], dev["beta"], d["eps"])
        with pytest.raises(B.FFError) as e:
            B.ff_check_device()
        assert e.value.status == 8
    finally:
        B.ff_debug_expect_extra_arrivals(0)
        B.ff_debug_set_wait_limit_us(2000000)
    B.ff_check_device()                      # state was cleared by the failed check
    Y, _ = gpu_run(d, AUTO)
    check_against_oracle(Y, oracle_on(d), "bf16")


@pytest.mark.parametrize("M,K,N", [(2085, 264, 4088), (16, 1024, 4096)])
def test_graph_replay_matches_eager(M, K, N):
    """The call is capturable (no allocation, no memset, counters re-arm themselves):
    every replay, with fresh inputs copied in between, equals the eager result bit for bit."""
    d = make_inputs(M, K, N, "bf16", seed=22)
    dev = {k: (v.cuda() if isinstance(v, torch.Tensor) else v) for k, v in d.items()}
    Y_static = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    args = (dev["X"], dev["W"], dev["b"], dev["gamma"], dev["beta"], d["eps"])
    B.ff_fused_linear_gelu_ln(*args, Y=Y_static)          # warm-up: workspace exists and is clean
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        with torch.cuda.graph(g, stream=s):
            B.ff_fused_linear_gelu_ln(*args, Y=Y_static)
    torch.cuda.synchronize()
    for rep in range(4):
        fresh = make_inputs(M, K, N, "bf16", seed=100 + rep)
        dev["X"].copy_(fresh["X"].cuda())
        dev["W"].copy_(fresh["W"].cuda())
        torch.cuda.synchronize()
        Y_eager = B.ff_fused_linear_gelu_ln(*args).clone()
        torch.cuda.synchronize()
        Y_static.zero_()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(Y_static, Y_eager), "replay %d differs from eager" % rep
    B.ff_check_device()
    ref_in = dict(d, X=dev["X"].cpu(), W=dev["W"].cpu())
    check_against_oracle(Y_static, oracle_on(ref_in), "bf16")


def test_first_call_on_a_fresh_workspace_can_be_captured():
    """The first call after binding a caller-owned workspace (full of NaN patterns) is recorded into a
    graph without any eager call before it: binding cleared the control region itself, the call issues
    nothing but its kernel.  Every replay must equal the oracle's result."""
    M, K, N = 1300, 264, 2056
    d = make_inputs(M, K, N, "bf16", seed=24)
    dev = {k: (v.cuda() if isinstance(v, torch.Tensor) else v) for k, v in d.items()}
    need = B.ff_workspace_bytes(M, K, N, B.FF_BF16)
    ws = torch.full((need // 4 + 64,), float("nan"), dtype=torch.float32, device="cuda")
    Y = torch.zeros((M, N), dtype=torch.bfloat16, device="cuda")
    torch.cuda.synchronize()
    B.ff_set_workspace(ws)
    try:
        g = torch.cuda.CUDAGraph()
        s = torch.cuda.Stream()
        with torch.cuda.stream(s):
            with torch.cuda.graph(g, stream=s):
                B.ff_fused_linear_gelu_ln(dev["X"], dev["W"], dev["b"], dev["gamma"], dev["beta"], d["eps"], Y=Y)
        torch.cuda.synchronize()
        ref = oracle_on(d)
        for rep in range(3):
            Y.zero_()
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            check_against_oracle(Y, ref, "bf16", "captured first call, replay %d" % rep)
        B.ff_check_device()
    finally:
        B.ff_set_workspace(None)


def test_growing_the_own_workspace_during_capture_is_refused():
    """With no caller workspace bound, a call that needs more scratch than the library holds cannot
    allocate while its stream is being captured: it must say so (FF_ERR_WORKSPACE) and leave the
    capture valid; outside the capture the same call allocates and works."""
    M, K, N = 4100, 64, 8200          # forced two-pass: fp32 G of 134 MB, larger than any earlier need
    d = make_inputs(M, K, N, "bf16", seed=25)
    dev = {k: (v.cuda() if isinstance(v, torch.Tensor) else v) for k, v in d.items()}
    small = make_inputs(64, 64, 64, "bf16", seed=25)
    sdev = {k: (v.cuda() if isinstance(v, torch.Tensor) else v) for k, v in small.items()}
    Y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    Ys = torch.empty((64, 64), dtype=torch.bfloat16, device="cuda")
    B.ff_set_workspace(ws := torch.zeros(1 << 18, dtype=torch.float32, device="cuda"))  # drop a large own one
    B.ff_set_workspace(None)
    del ws
    B.ff_fused_linear_gelu_ln(sdev["X"], sdev["W"], sdev["b"], sdev["gamma"], sdev["beta"], small["eps"], Y=Ys)
    torch.cuda.synchronize()
    B.ff_debug_force_variant(TWOPASS)
    status = None
    try:
        g = torch.cuda.CUDAGraph()
        s = torch.cuda.Stream()
        with torch.cuda.stream(s):
            with torch.cuda.graph(g, stream=s):
                try:
                    B.ff_fused_linear_gelu_ln(dev["X"], dev["W"], dev["b"], dev["gamma"], dev["beta"], d["eps"], Y=Y)
                except B.FFError as e:
                    status = e.status
                B.ff_debug_force_variant(AUTO)
                B.ff_fused_linear_gelu_ln(sdev["X"], sdev["W"], sdev["b"], sdev["gamma"], sdev["beta"],
                                          small["eps"], Y=Ys)
        torch.cuda.synchronize()
        assert status == 6
        Ys.zero_()
        g.replay()                       # the capture survived the refused call
        torch.cuda.synchronize()
        check_against_oracle(Ys, oracle_on(small), "bf16", "small call captured after the refusal")
        Y2, used = gpu_run(d, TWOPASS)   # eager: allocates and works
        assert used == TWOPASS
        rows = sample_rows(M, 24)
        check_against_oracle(Y2[torch.tensor(rows)], oracle_on(d, rows=rows), "bf16", "two-pass after growing")
    finally:
        B.ff_debug_force_variant(AUTO)


def test_two_workgroups_per_compute_unit_wait_for_each_other():
    """128-tiles with more workgroups than compute units (two per unit, all of which must be resident
    because they wait for one another inside the launch)."""
    M, K, N = 1024, 256, 8192
    _announce("two per unit", M, K, N)
    d = make_inputs(M, K, N, "bf16", seed=26)
    try:
        B.ff_debug_force_tile(128, 2)
        plan = B.ff_plan_query(M, K, N, B.FF_BF16)
        assert (plan["tile_m"], plan["tile_n"], plan["workgroups_per_cu"]) == (128, 128, 2)
        Y, used = gpu_run(d, AUTO)
        Y2, _ = gpu_run(d, AUTO)
    finally:
        B.ff_debug_force_tile(0, 0)
    assert used == FUSED
    print(check_against_oracle(Y, oracle_on(d), "bf16", "1024x256x8192"))
    assert torch.equal(Y, Y2)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_one_round_of_half_height_tiles(dtype):
    """A shape whose 256 x 256 tiles would leave half the compute units idle: in bf16 the automatic plan
    takes 256-column x 128-row tiles, one per unit.  Cut last tile column and row block."""
    M, K, N = 1000, 320, 8136
    _announce("half-height tiles", M, K, N)
    plan = B.ff_plan_query(M, K, N, B.FF_BF16 if dtype == "bf16" else B.FF_F32)
    want = (FUSED, 128, 256, 1) if dtype == "bf16" else (FUSED, 128, 128, 2)   # fp32 stays with 128 x 128 tiles
    assert (plan["variant"], plan["tile_m"], plan["tile_n"], plan["workgroups_per_cu"]) == want
    d = make_inputs(M, K, N, dtype, seed=33)
    Y, used = gpu_run(d, AUTO)
    assert used == FUSED
    print(check_against_oracle(Y, oracle_on(d), dtype, "half-height tiles"))
    Y2, _ = gpu_run(d, AUTO)
    assert torch.equal(Y, Y2)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("forced", [None, (256, 8), (256, 4)], ids=["auto", "t256w8", "t256w4"])
def test_rows_of_more_than_sixteen_tiles(forced, dtype):
    """Rows wider than 16 tiles: where a workgroup has two threads per row, each merges half of the row's
    partial statistics.  Odd tile counts, a cut last tile (8 columns) and a cut last row block, with a
    bias that moves the row mean far from zero."""
    M, K, N = 700, 192, 5128       # 21 tiles of 256 columns, 41 of 128
    _announce("wide rows %s" % (forced,), M, K, N)
    d = make_inputs(M, K, N, dtype, seed=31)
    d["b"] = (d["b"].float() + 3.0).to(d["b"].dtype)
    try:
        if forced:
            B.ff_debug_force_tile(forced[0], 1)
            B.ff_debug_force_waves(forced[1])
        plan = B.ff_plan_query(M, K, N, B.FF_BF16 if dtype == "bf16" else B.FF_F32)
        assert plan["variant"] == FUSED and -(-N // plan["tile_n"]) > 16
        Y, used = gpu_run(d, AUTO)
        Y2, _ = gpu_run(d, AUTO)
    finally:
        B.ff_debug_force_tile(0, 0)
        B.ff_debug_force_waves(0)
    assert used == FUSED
    print(check_against_oracle(Y, oracle_on(d), dtype, "wide rows"))
    assert torch.equal(Y, Y2)


def test_workspace_grows_between_shapes():
    """Library-owned workspace: a larger shape after a smaller one reallocates and still works."""
    for (M, K, N) in ((64, 64, 64), (1500, 128, 3080), (300, 64, 520)):
        d = make_inputs(M, K, N, "bf16", seed=23)
        Y, _ = gpu_run(d, TWOPASS)
        check_against_oracle(Y, oracle_on(d), "bf16")


# ------------------------------------------------------------ more edge cases
def test_many_rounds_and_a_row_tail():
    """A tall problem: 1172 row-blocks over a grid of one workgroup per compute unit (five rounds), the
    last row-block with 61 rows; checked on sampled complete rows including the last ones."""
    M, K, N = 300_093, 64, 256
    _announce("tall", M, K, N)
    d = make_inputs(M, K, N, "bf16", seed=18)
    Y, used = gpu_run(d, AUTO)
    assert used == FUSED
    rows = sorted(set(sample_rows(M, 40) + [M - 1, M - 61, M - 62, 255, 256]))
    print(check_against_oracle(Y[torch.tensor(rows)], oracle_on(d, rows=rows), "bf16", "tall"))


@pytest.mark.parametrize("M,K,N", [(300, 128, 520), (16, 512, 1024)])
def test_nan_and_inf_stay_in_their_rows(M, K, N):
    """No checking on the device: a NaN or an infinity in a row of X poisons that row of Y and nothing
    else (rows are independent; the statistics of the other rows never see it)."""
    d = make_inputs(M, K, N, "bf16", seed=19)
    ref = oracle_on(d)
    X = d["X"].clone()
    X[3, 5] = float("nan")
    X[7, 0] = float("inf")
    Y, _ = gpu_run(dict(d, X=X), AUTO)
    Yc = Y.float().cpu()
    assert bool(torch.isnan(Yc[3]).all()) and bool(torch.isnan(Yc[7]).all())
    ok = [m for m in range(M) if m not in (3, 7)]
    check_against_oracle(Y[torch.tensor(ok)], ref[ok], "bf16")


@pytest.mark.parametrize("eps", [0.0, 1e-12, 0.25])
def test_eps_values(eps):
    d = make_inputs(130, 96, 264, "f32", seed=20)
    d = dict(d, eps=eps)
    Y, _ = gpu_run(d, AUTO)
    print(check_against_oracle(Y, oracle_on(d), "f32", "eps %g" % eps))


# ------------------------------------------------------------ seeded random shapes
def _random_case(rng, large):
    dtype = rng.choice(["bf16", "bf16", "f32"])
    q = 8 if dtype == "bf16" else 4
    if large:
        M = rng.randint(900, 5000)
        K = q * rng.randint(1, 384 // q)
        N = q * rng.randint(2048 // q, 10000 // q)
    else:
        M = rng.choice([rng.randint(1, 40), rng.randint(1, 600), rng.randint(600, 2500)])
        K = q * rng.randint(1, 768 // q)
        N = q * rng.choice([rng.randint(1, 64), rng.randint(64, 1200), rng.randint(256, 6000 // q)])
    return dtype, M, K, N


@pytest.mark.parametrize("seed,large,cases", [(11, False, 24), (12, False, 24), (13, True, 10)])
def test_random_shapes_against_the_oracle(seed, large, cases):
    """Seeded random shapes through the automatic plan (every tile shape, the small-M kernel, cut tiles in
    every dimension), a third of them with a bias that moves the row mean away from zero; full matrix
    against the oracle, and a second run for bit equality."""
    import random
    rng = random.Random(seed)
    for it in range(cases):
        dtype, M, K, N = _random_case(rng, large)
        d = make_inputs(M, K, N, dtype, seed=1000 * seed + it)
        if rng.random() < 0.3:
            d["b"] = (d["b"].float() + rng.choice([-2.0, 3.0])).to(d["b"].dtype)
        _announce("random %d/%d" % (seed, it), M, K, N)
        Y, _ = gpu_run(d, AUTO)
        Y2, _ = gpu_run(d, AUTO)
        check_against_oracle(Y, oracle_on(d), dtype, "random %dx%dx%d %s" % (M, K, N, dtype))
        assert torch.equal(Y, Y2)
