"""The entry point that allocates nothing, through the C ABI, against the ordinary entry point (same
kernels, so the results must agree bit for bit) and against the oracle: two calls in a row, the second
on a smaller input; the size limit; and the small-M and tiled variants."""
import pytest
import torch

from paper_2511_01884_amd import binding as B
from paper_2511_01884_amd.inputs import make_inputs
from parity_util import check_against_oracle, oracle_on

pytestmark = pytest.mark.gpu


def _both(M, K, N, dtype, seed):
    d = make_inputs(M, K, N, dtype, seed=seed)
    dev = [d[k].cuda() for k in ("X", "W", "b", "gamma", "beta")]
    Y_ref = B.ff_fused_linear_gelu_ln(*dev, d["eps"])
    used = B.ff_last_variant()
    Y = torch.full_like(Y_ref, float("nan"))
    B.ff_fused_linear_gelu_ln_noalloc(*dev, d["eps"], Y=Y)
    assert B.ff_last_variant() == used
    B.ff_check_device()
    torch.cuda.synchronize()
    return d, Y, Y_ref


@pytest.mark.parametrize("shapes,dtype", [(((2085, 264, 4088), (300, 200, 520)), "bf16"),
                                          (((16, 1024, 4096), (5, 520, 1000)), "bf16"),
                                          (((600, 128, 1032), (77, 36, 132)), "f32")])
def test_no_alloc_matches_the_ordinary_entry_point_twice_in_a_row(shapes, dtype):
    for seed, (M, K, N) in enumerate(shapes):
        print("[case] no-alloc", M, K, N, dtype, flush=True)
        d, Y, Y_ref = _both(M, K, N, dtype, seed=31 + seed)
        assert torch.equal(Y, Y_ref), "no-alloc result differs from the ordinary entry point"
        check_against_oracle(Y, oracle_on(d), dtype, "no-alloc %dx%dx%d" % (M, K, N))


def test_no_alloc_rejects_what_does_not_fit():
    limit = B.ff_noalloc_max_bytes()
    assert limit == 8 << 20
    # rows wider than the grid need the two-pass variant's fp32 copy of G: far beyond the array
    M, K, N = 40, 64, 258 * 256
    assert B.ff_workspace_bytes(M, K, N, B.FF_BF16) > limit
    d = make_inputs(M, K, N, "bf16", seed=33)
    dev = [d[k].cuda() for k in ("X", "W", "b", "gamma", "beta")]
    Y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(B.FFError) as e:
        B.ff_fused_linear_gelu_ln_noalloc(*dev, d["eps"], Y=Y)
    assert e.value.status == 6
    # and the next call that fits is fine
    d, Y, Y_ref = _both(300, 200, 520, "bf16", seed=34)
    assert torch.equal(Y, Y_ref)
