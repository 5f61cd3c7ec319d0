"""The pins that tie the CPU oracle to facts outside itself.

Each pin is a function of an `oracle.Oracle` instance, so the same list runs
against the real build (tests/test_oracle_pins.py) and against builds with a
planted mistake (tests/test_oracle_mutants.py), where at least one must fail.

Nothing here calls the oracle to produce an expected value: expectations are
closed forms, a 60-digit series, hand-expanded sums, integer arithmetic, or an
independent float64 library composition.
"""
from __future__ import annotations

import math
from decimal import Decimal, getcontext

import numpy as np
import torch

from paper_2511_01884_amd.inputs import make_inputs, make_integer_inputs


# ----------------------------------------------------------------- helpers
def _erf_series(x: Decimal) -> Decimal:
    """erf(x) = 2/sqrt(pi) * sum_n (-1)^n x^(2n+1) / (n! (2n+1)), 80-digit arithmetic."""
    getcontext().prec = 80
    term = x  # x^(2n+1)/n!
    total = x
    n = 0
    x2 = x * x
    while True:
        n += 1
        term = -term * x2 / n
        add = term / (2 * n + 1)
        total += add
        if abs(add) < Decimal(10) ** -75:
            break
    pi = Decimal("3.14159265358979323846264338327950288419716939937510582097494459230781640628620899")
    return 2 * total / pi.sqrt()


def _gelu_exact(z: float) -> float:
    """z * Phi(z) from the series, rounded once to float64."""
    getcontext().prec = 80
    zd = Decimal(z)
    phi = (1 + _erf_series(zd / Decimal(2).sqrt())) / 2
    return float(zd * phi)


# -------------------------------------------------------------------- pins
def pin_gelu_fixed_points(orc):
    """P1: GELU at fixed points against the high-precision series (erf form)."""
    for z in (0.0, 0.5, -0.5, 1.0, -1.0, 2.0, -2.0, 3.0, -3.0, 4.0, -4.0, 6.0, -6.0,
              0.125, -0.125, 1.5, -2.75, 5.25, -5.25):
        want = _gelu_exact(z)
        got = orc.gelu(z)
        # libm erfc is good to about an ulp, and rounding z/sqrt(2) moves erfc by a
        # relative 2x^2 * 2^-53 in the tail (x = 4.24 at z = -6): 1e-14 covers both.
        assert (got == 0.0) if want == 0.0 else abs(got - want) <= 1e-14 * abs(want), (z, got, want)
    # far tails: GELU(10) is 10 to fp64; GELU(-10) is tiny and negative
    assert orc.gelu(10.0) == 10.0
    assert abs(orc.gelu(-10.0) - (-7.619853024160527e-23)) <= 1e-36
    # spot values with textbook Phi: Phi(1) = 0.8413447460685429...
    assert abs(orc.gelu(1.0) - 0.8413447460685429) < 1e-15
    assert abs(orc.gelu(-1.0) + 0.15865525393145707) < 1e-15


def pin_gelu_odd_part(orc):
    """P2: GELU(z) - GELU(-z) = z, since Phi(z) + Phi(-z) = 1."""
    for z in np.linspace(-8.0, 8.0, 1601):
        d = orc.gelu(float(z)) - orc.gelu(float(-z))
        assert abs(d - z) <= 5e-16 * max(1.0, abs(z)), (z, d)


def pin_layernorm_moments(orc):
    """P3: gamma=1, beta=0 -> row mean 0 and biased row variance var/(var+eps);
    gamma=1, beta!=0 -> row mean equals mean(beta)."""
    rng = np.random.default_rng(1)
    for N in (7, 64, 1000):
        g = rng.standard_normal(N) * 0.6 + 0.3
        for eps in (0.0, 1e-5, 0.5):
            y, mu, var = orc.layernorm_row(g, None, None, eps)
            want_mu = math.fsum(g) / N
            want_var = math.fsum((g - want_mu) ** 2) / N
            assert abs(mu - want_mu) < 1e-14 and abs(var - want_var) < 1e-14
            assert abs(math.fsum(y) / N) < 1e-13
            vy = math.fsum((y - math.fsum(y) / N) ** 2) / N
            assert abs(vy - want_var / (want_var + eps)) < 1e-12, (N, eps, vy)
        beta = rng.standard_normal(N).astype(np.float32)
        y, _, _ = orc.layernorm_row(g, None, beta, 1e-5)
        assert abs(math.fsum(y) / N - math.fsum(beta.astype(np.float64)) / N) < 1e-13


def pin_layernorm_biased_variance(orc):
    """Two-element row: g = (0, 2) -> mu = 1, biased var = 1 (unbiased would be 2),
    eps inside the square root: y = -/+ 1/sqrt(1 + eps)."""
    y, mu, var = orc.layernorm_row(np.array([0.0, 2.0]), None, None, 3.0)
    assert mu == 1.0 and var == 1.0
    assert np.allclose(y, [-0.5, 0.5], rtol=0, atol=1e-16)  # 1/sqrt(1+3) = 0.5
    # affine: y*gamma + beta, element by element
    y, _, _ = orc.layernorm_row(np.array([0.0, 2.0]), np.array([2.0, 4.0]), np.array([10.0, 20.0]), 3.0)
    assert np.allclose(y, [-1.0 + 10.0, 2.0 + 20.0], rtol=0, atol=1e-15)


def pin_layernorm_scale_shift(orc):
    """P4: G -> a*G + c leaves Y unchanged at eps = 0 and rescales the centred
    output by sqrt((var+eps)/(var+eps/a^2)) otherwise."""
    rng = np.random.default_rng(2)
    g = rng.standard_normal(257)
    y0, _, var = orc.layernorm_row(g, None, None, 0.0)
    for a, c in ((2.0, 0.0), (0.25, 3.0), (8.0, -1.5)):
        y1, _, _ = orc.layernorm_row(a * g + c, None, None, 0.0)
        assert np.max(np.abs(y1 - y0)) < 1e-12
        eps = 0.01
        ye, _, _ = orc.layernorm_row(g, None, None, eps)
        ys, _, _ = orc.layernorm_row(a * g + c, None, None, eps)
        factor = math.sqrt((var + eps) / (var + eps / a ** 2))
        assert np.max(np.abs(ys - ye * factor)) < 1e-12


def pin_constant_rows(orc):
    """P5: W = 0 and constant bias -> every row of G is constant -> Y = beta exactly."""
    M, K, N = 3, 8, 6
    X = np.arange(M * K, dtype=np.float32).reshape(M, K)
    W = np.zeros((N, K), dtype=np.float32)
    b = np.full(N, 0.75, dtype=np.float32)
    gamma = np.linspace(0.5, 1.5, N).astype(np.float32)
    beta = np.linspace(-1, 1, N).astype(np.float32)
    Y = orc.fused_linear_gelu_ln(X, W, b, gamma, beta, 1e-5)
    assert np.array_equal(Y, np.broadcast_to(beta.astype(np.float64), (M, N)))


def pin_tiny_gemm_by_hand(orc):
    """P6: non-square tiny cases against sums expanded by hand below; a transposed
    W, swapped M/N or dropped bias changes the numbers."""
    # M=2, K=3, N=4
    X = np.array([[1.0, 2.0, -1.0],
                  [0.5, -3.0, 2.0]], dtype=np.float32)
    W = np.array([[1.0, 0.0, 2.0],
                  [-1.0, 1.0, 0.5],
                  [2.0, 2.0, 2.0],
                  [0.0, -0.5, 4.0]], dtype=np.float32)
    b = np.array([0.5, -1.0, 0.25, 2.0], dtype=np.float32)
    Z_hand = np.array([
        # row 0: x = (1, 2, -1)
        [0.5 + (1 * 1 + 2 * 0 + -1 * 2),        # -0.5
         -1.0 + (1 * -1 + 2 * 1 + -1 * 0.5),    # -0.5
         0.25 + (1 * 2 + 2 * 2 + -1 * 2),       # 4.25
         2.0 + (1 * 0 + 2 * -0.5 + -1 * 4)],    # -3.0
        # row 1: x = (0.5, -3, 2)
        [0.5 + (0.5 * 1 + -3 * 0 + 2 * 2),      # 5.0
         -1.0 + (0.5 * -1 + -3 * 1 + 2 * 0.5),  # -3.5
         0.25 + (0.5 * 2 + -3 * 2 + 2 * 2),     # -0.75
         2.0 + (0.5 * 0 + -3 * -0.5 + 2 * 4)],  # 11.5
    ])
    assert np.array_equal(Z_hand, np.array([[-0.5, -0.5, 4.25, -3.0], [5.0, -3.5, -0.75, 11.5]]))
    out = orc.fused_linear_gelu_ln(X, W, b, None, None, 1e-5, stages=True)
    assert np.array_equal(out["Z"], Z_hand)
    for m in range(2):
        assert np.array_equal(orc.linear_row(X[m], W, b), Z_hand[m])
    # downstream stages from the hand values, with the series GELU
    G = np.array([[_gelu_exact(float(z)) for z in row] for row in Z_hand])
    assert np.max(np.abs(out["G"] - G)) < 1e-15
    eps64 = float(np.float32(1e-5))
    for m in range(2):
        mu = math.fsum(G[m]) / 4
        var = math.fsum((G[m] - mu) ** 2) / 4
        y = (G[m] - mu) / math.sqrt(var + eps64)
        assert np.max(np.abs(out["Y"][m] - y)) < 1e-14
        assert abs(out["mu"][m] - mu) < 1e-15 and abs(out["var"][m] - var) < 1e-15
    # M=3, K=5, N=2, no bias: z = X W^T by einsum of integers (exact)
    X2 = np.array([[1, 2, 3, 4, 5], [-1, 0, 1, 0, -1], [2, -2, 2, -2, 2]], dtype=np.float32)
    W2 = np.array([[1, 1, 1, 1, 1], [1, -1, 2, -2, 3]], dtype=np.float32)
    Z2 = np.array([[15.0, 1 - 2 + 6 - 8 + 15], [-1.0, -1 + 2 - 3], [2.0, 2 + 2 + 4 + 4 + 6]])
    out2 = orc.fused_linear_gelu_ln(X2, W2, None, None, None, 1e-5, stages=True)
    assert np.array_equal(out2["Z"], Z2)


def pin_integer_exact_gemm(orc):
    """P7: integer-valued inputs make the linear stage exact; compare with int64 arithmetic."""
    for (M, K, N) in ((5, 64, 9), (17, 1000, 33)):
        d = make_integer_inputs(M, K, N, "bf16", seed=3)
        X = d["X"].float().numpy(); W = d["W"].float().numpy(); b = d["b"].float().numpy()
        Zi = X.astype(np.int64) @ W.astype(np.int64).T + b.astype(np.int64)[None, :]
        out = orc.fused_linear_gelu_ln(X, W, b, None, None, 1e-5, stages=True)
        assert np.array_equal(out["Z"], Zi.astype(np.float64))


def pin_identity_x(orc):
    """P8: X = I gives Z = W^T + b, so Y = LN(GELU(W^T + b)) row by row; K = 1 is an outer product."""
    rng = np.random.default_rng(4)
    K = 6; N = 4
    W = rng.standard_normal((N, K)).astype(np.float32)
    b = rng.standard_normal(N).astype(np.float32)
    out = orc.fused_linear_gelu_ln(np.eye(K, dtype=np.float32), W, b, None, None, 1e-5, stages=True)
    assert np.array_equal(out["Z"], W.T.astype(np.float64) + b.astype(np.float64)[None, :])
    x = rng.standard_normal((5, 1)).astype(np.float32)
    w = rng.standard_normal((3, 1)).astype(np.float32)
    out = orc.fused_linear_gelu_ln(x, w, None, None, None, 1e-5, stages=True)
    assert np.array_equal(out["Z"], x.astype(np.float64) @ w.astype(np.float64).T)


def pin_library_composition(orc):
    """P9: an independent float64 composition of the three public operators
    (torch CPU) on the fp32 parity workload and on ragged shapes."""
    import torch.nn.functional as F
    for (M, K, N, dt, seed) in ((256, 512, 512, "f32", 0), (13, 40, 24, "bf16", 5), (3, 8, 1000, "f32", 6)):
        d = make_inputs(M, K, N, dt, seed=seed)
        t = {k: v.double() for k, v in d.items() if k != "eps"}
        eps64 = float(np.float32(d["eps"]))
        ref = F.layer_norm(F.gelu(F.linear(t["X"], t["W"], t["b"]), approximate="none"),
                           (N,), t["gamma"], t["beta"], eps64).numpy()
        Y = orc.fused_linear_gelu_ln(d["X"].float().numpy(), d["W"].float().numpy(),
                                     d["b"].float().numpy(), d["gamma"].float().numpy(),
                                     d["beta"].float().numpy(), d["eps"])
        assert np.max(np.abs(Y - ref)) < 1e-12, np.max(np.abs(Y - ref))


def pin_row_subset(orc):
    """Rows are independent: a listed subset equals the same rows of the full result, bit for bit."""
    d = make_inputs(37, 48, 40, "bf16", seed=7)
    a = [d[k].float().numpy() for k in ("X", "W", "b", "gamma", "beta")]
    full = orc.fused_linear_gelu_ln(*a, d["eps"])
    rows = [36, 0, 5, 5, 17]
    sub = orc.fused_linear_gelu_ln(*a, d["eps"], rows=rows)
    assert np.array_equal(sub, full[rows])


def pin_gelu_moments(orc):
    """P10 (sanity): for z ~ N(0,1), E[GELU] = 1/(2 sqrt(pi)) and E[GELU^2] = 0.42522148
    (closed form / quadrature); checked by Gauss-Hermite quadrature through the oracle's GELU."""
    x, w = np.polynomial.hermite_e.hermegauss(120)
    g = np.array([orc.gelu(float(v)) for v in x])
    norm = math.sqrt(2 * math.pi)
    m1 = float(np.sum(w * g) / norm)
    assert abs(m1 - 1 / (2 * math.sqrt(math.pi))) < 1e-9
    # E[z*Phi(z)] = E[phi(z)] * ... closed form 1/(2 sqrt(pi)) = 0.28209479177387814
    assert abs(m1 - 0.28209479177387814) < 1e-9


def pin_round_bf16(orc):
    """The bf16 rounding helper: ties to even by hand, and agreement with the
    float32 -> bfloat16 conversion of an independent library on float32-exact values."""
    cases = {1.0: 1.0, 1.00390625: 1.0, 1.01171875: 1.015625, 1.0078125: 1.0078125,
             -1.00390625: -1.0, 3.0: 3.0, 257.0: 256.0, 259.0: 260.0, 0.0: 0.0}
    got = orc.round_bf16(list(cases.keys()))
    assert np.array_equal(got, np.array(list(cases.values())))
    assert orc.round_bf16([3.4e38])[0] == np.inf
    g = torch.Generator().manual_seed(8)
    v = torch.randn(20000, generator=g) * torch.exp(4 * torch.randn(20000, generator=g))
    want = v.to(torch.bfloat16).double().numpy()
    assert np.array_equal(orc.round_bf16(v.double().numpy()), want)
    # a value below a tie in fp64 that fp32 would first round onto the tie
    x = 1.00390625 + 2.0 ** -40  # just above the tie -> must round up
    assert orc.round_bf16([x])[0] == 1.0078125


ALL_PINS = [
    pin_gelu_fixed_points,
    pin_gelu_odd_part,
    pin_layernorm_moments,
    pin_layernorm_biased_variance,
    pin_layernorm_scale_shift,
    pin_constant_rows,
    pin_tiny_gemm_by_hand,
    pin_integer_exact_gemm,
    pin_identity_x,
    pin_library_composition,
    pin_row_subset,
    pin_gelu_moments,
    pin_round_bf16,
]


# ---------------------------------------------- second chain (row-mean epilogue)
def pin_rowmean_chain_collapse(orc):
    """The mean over n of a linear layer is one dot product: mean_n(x.W[n] + b[n] - s[n])
    = x . mean_n(W[n]) + mean(b - s).  Evaluated here with float64 library sums and the
    series GELU, independently of the oracle's long-way loops."""
    rng = np.random.default_rng(9)
    for (M, K, N) in ((4, 7, 5), (9, 64, 33)):
        X = rng.standard_normal((M, K)).astype(np.float32)
        W = (rng.standard_normal((N, K)) / math.sqrt(K)).astype(np.float32)
        b = rng.uniform(-0.5, 0.5, N).astype(np.float32)
        s = rng.uniform(-0.5, 0.5, N).astype(np.float32)
        out, rv = orc.linear_sub_rowmean_gelu_residual(X, W, b, s, with_rowval=True)
        t = X.astype(np.float64) @ W.astype(np.float64).mean(axis=0) + (b.astype(np.float64) - s).mean()
        g = np.array([_gelu_exact(float(v)) for v in t])
        assert np.max(np.abs(rv - g)) < 1e-14
        assert np.max(np.abs(out - (X.astype(np.float64) + g[:, None]))) < 1e-14


def pin_rowmean_chain_by_hand(orc):
    """M=2, K=2, N=3, every number written out."""
    X = np.array([[1.0, 2.0], [-1.0, 0.5]], dtype=np.float32)
    W = np.array([[1.0, 0.0], [0.0, 1.0], [2.0, -1.0]], dtype=np.float32)
    b = np.array([0.5, 0.0, -0.5], dtype=np.float32)
    s = np.array([0.0, 1.0, 0.5], dtype=np.float32)
    # row 0: z = (1.5, 2, -0.5); z - s = (1.5, 1, -1); mean = 0.5
    # row 1: z = (-0.5, 0.5, -3); z - s = (-0.5, -0.5, -3.5); mean = -1.5
    means = [0.5, -1.5]
    out, rv = orc.linear_sub_rowmean_gelu_residual(X, W, b, s, with_rowval=True)
    for m in range(2):
        g = _gelu_exact(means[m])
        assert abs(rv[m] - g) < 1e-15
        assert np.max(np.abs(out[m] - (X[m].astype(np.float64) + g))) < 1e-15
    # optional vectors default to zero; W = 0 leaves only the bias/subtract mean
    out0 = orc.linear_sub_rowmean_gelu_residual(X, np.zeros_like(W), b, s)
    g0 = _gelu_exact(float((b.astype(np.float64) - s).mean()))
    assert np.max(np.abs(out0 - (X.astype(np.float64) + g0))) < 1e-15
    out1 = orc.linear_sub_rowmean_gelu_residual(X, W, None, None)
    out2 = orc.linear_sub_rowmean_gelu_residual(X, W, np.zeros(3, np.float32), np.zeros(3, np.float32))
    assert np.array_equal(out1, out2)


def pin_rowmean_chain_library(orc):
    """float64 library composition of the chain as stated, including a row subset."""
    import torch.nn.functional as F
    g = torch.Generator().manual_seed(10)
    M, K, N = 11, 24, 40
    X = torch.randn(M, K, generator=g); W = torch.randn(N, K, generator=g) / math.sqrt(K)
    b = torch.rand(N, generator=g) - 0.5; s = torch.rand(N, generator=g) - 0.5
    z = F.linear(X.double(), W.double(), b.double()) - s.double()
    ref = (X.double() + F.gelu(z.mean(dim=1, keepdim=True), approximate="none")).numpy()
    out = orc.linear_sub_rowmean_gelu_residual(X.numpy(), W.numpy(), b.numpy(), s.numpy())
    assert np.max(np.abs(out - ref)) < 1e-13
    sub = orc.linear_sub_rowmean_gelu_residual(X.numpy(), W.numpy(), b.numpy(), s.numpy(), rows=[10, 3, 3])
    assert np.array_equal(sub, out[[10, 3, 3]])


ALL_PINS += [pin_rowmean_chain_collapse, pin_rowmean_chain_by_hand, pin_rowmean_chain_library]


# ------------------------------------------------- row-wise cross-entropy
def pin_xent_closed_forms(orc):
    """Equal logits give log C whatever the target; logits that are logs of 1..C give
    log(C(C+1)/2) - log(t+1); two classes give softplus of the logit difference."""
    for C in (1, 2, 7, 64):
        for v in (0.0, -3.5, 1000.0):  # 1000: exp overflows unless the maximum is removed first
            L = np.full((3, C), v, dtype=np.float32)
            t = np.array([0, C - 1, C // 2])
            rl, mean = orc.cross_entropy(L, t)
            assert np.allclose(rl, math.log(C), rtol=0, atol=1e-12), (C, v, rl)
            assert abs(mean - math.log(C)) < 1e-12
    C = 9
    row = np.log(np.arange(1, C + 1, dtype=np.float64)).astype(np.float32)  # rounded once; use the rounded values
    L = np.tile(row, (C, 1))
    t = np.arange(C)
    rl, mean = orc.cross_entropy(L, t)
    tot = math.fsum(math.exp(float(x)) for x in row)
    want = np.array([math.log(tot) - float(row[c]) for c in range(C)])
    assert np.allclose(rl, want, rtol=0, atol=1e-12)
    assert abs(tot - 45.0) < 1e-5  # 1 + 2 + ... + 9, up to the float32 rounding of the logs
    assert abs(mean - math.fsum(want) / C) < 1e-12
    # two classes: loss = log(1 + exp(-(L_t - L_other)))
    d = np.array([-30.0, -2.0, -0.25, 0.0, 0.5, 3.0, 40.0], dtype=np.float32)
    L = np.stack([d, np.zeros_like(d)], axis=1)
    rl, _ = orc.cross_entropy(L, np.zeros(len(d), dtype=np.int64))
    want = np.array([math.log1p(math.exp(-float(x))) if x > -20 else -float(x) + math.log1p(math.exp(float(x)))
                     for x in d])
    assert np.allclose(rl, want, rtol=1e-13, atol=1e-15), (rl, want)
    rl1, _ = orc.cross_entropy(L, np.ones(len(d), dtype=np.int64))
    assert np.allclose(rl1 - rl, d.astype(np.float64), rtol=0, atol=1e-12)  # the two losses differ by the logit gap


def pin_xent_by_hand(orc):
    """Non-square hand case: distinct targets per row, mean over rows (not classes)."""
    L = np.array([[1.0, 2.0, 0.5, -1.0, 0.0],
                  [-2.0, 0.25, 0.25, 3.0, 1.5]], dtype=np.float32)
    t = np.array([3, 1])
    r0 = math.log(math.exp(1.0) + math.exp(2.0) + math.exp(0.5) + math.exp(-1.0) + math.exp(0.0)) - (-1.0)
    r1 = math.log(math.exp(-2.0) + 2 * math.exp(0.25) + math.exp(3.0) + math.exp(1.5)) - 0.25
    rl, mean = orc.cross_entropy(L, t)
    assert abs(rl[0] - r0) < 1e-13 and abs(rl[1] - r1) < 1e-13, (rl, r0, r1)
    assert abs(mean - (r0 + r1) / 2) < 1e-13
    # a target outside [0, C) poisons its row and the mean, nothing else
    rl, mean = orc.cross_entropy(L, np.array([5, 1]))
    assert math.isnan(rl[0]) and abs(rl[1] - r1) < 1e-13 and math.isnan(mean)
    rl, _ = orc.cross_entropy(L, np.array([-1, 1]))
    assert math.isnan(rl[0])


def pin_xent_shift_and_library(orc):
    """Adding a constant to a row changes nothing; the maximum may sit anywhere in the row;
    agreement with an independent float64 library composition on random inputs."""
    g = torch.Generator(device="cpu").manual_seed(11)
    B, C = 37, 203
    L = torch.round(torch.randn(B, C, generator=g) * 3.0 * 1024.0) / 1024.0  # multiples of 2^-10
    t = torch.randint(0, C, (B,), generator=g)
    rl, mean = orc.cross_entropy(L.numpy(), t.numpy())
    # the shifted logits are exact in float32, so the shifted problem is the same problem
    Ls = (L.double() + 64.0).float()
    assert bool((Ls.double() - 64.0 == L.double()).all())
    rls, _ = orc.cross_entropy(Ls.numpy(), t.numpy())
    assert np.allclose(rls, rl, rtol=0, atol=1e-11)
    want = torch.nn.functional.cross_entropy(L.double(), t, reduction="none").numpy()
    assert np.allclose(rl, want, rtol=0, atol=1e-12)
    assert abs(mean - float(torch.nn.functional.cross_entropy(L.double(), t))) < 1e-12
    lse = torch.logsumexp(L.double(), dim=1).numpy()
    assert np.allclose(rl, lse - L.double().numpy()[np.arange(B), t.numpy()], rtol=0, atol=1e-12)
    # one logit so large that exp overflows unless exactly that maximum is removed, at either end and inside
    for pos in (0, 3, 6):
        Lh = np.zeros((2, 7), dtype=np.float32)
        Lh[:, pos] = 1000.0
        rlh, _ = orc.cross_entropy(Lh, np.array([pos, (pos + 1) % 7]))
        assert rlh[0] == 0.0 and rlh[1] == 1000.0, (pos, rlh)
    # maximum in the first, a middle and the last position
    for pos in (0, C // 2, C - 1):
        L2 = L.clone()
        L2[:, pos] = 50.0
        rl2, _ = orc.cross_entropy(L2.numpy(), np.full(B, pos))
        assert np.all(rl2 >= 0) and np.all(rl2 < 1e-15 + C * math.exp(-35.0)), rl2.max()


ALL_PINS += [pin_xent_closed_forms, pin_xent_by_hand, pin_xent_shift_and_library]
