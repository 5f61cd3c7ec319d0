"""Runs every kernel variant of one task a fixed number of times, in a fixed order, so that the
dispatches of a rocprofv3 dump can be attributed by position.  Run under rocprofv3 as
`python3 -m paper_2511_01884_amd.metric_study.variants TASK`."""
import sys

import torch

from .. import binding as B

# task name -> (M, K, N), all bf16
TASKS = {
    "sq4096": (4096, 4096, 4096),
    "tall": (65536, 1024, 1024),
    "wide": (8192, 4096, 16384),
    "deepk": (2048, 8192, 2048),
    "mid": (8192, 2048, 8192),
    "flat": (1024, 4096, 8192),
}
# (label, tile, workgroups per compute unit, wavefronts per workgroup of the 256 x 256 tile or 0, variant);
# tile 256 with two workgroups per unit is the 256-column x 128-row tile (one per unit where the grid is small)
VARIANTS = [
    ("t256w8_fused", 256, 1, 8, B.FF_VARIANT_TILED_FUSED),
    ("t256w8_twopass", 256, 1, 8, B.FF_VARIANT_TILED_TWOPASS),
    ("t256w4_fused", 256, 1, 4, B.FF_VARIANT_TILED_FUSED),
    ("t256w4_twopass", 256, 1, 4, B.FF_VARIANT_TILED_TWOPASS),
    ("t256x128_fused", 256, 2, 0, B.FF_VARIANT_TILED_FUSED),
    ("t128x1_fused", 128, 1, 0, B.FF_VARIANT_TILED_FUSED),
    ("t128x2_fused", 128, 2, 0, B.FF_VARIANT_TILED_FUSED),
    ("t128x1_twopass", 128, 1, 0, B.FF_VARIANT_TILED_TWOPASS),
    ("t128x2_twopass", 128, 2, 0, B.FF_VARIANT_TILED_TWOPASS),
]
REPEATS = 4          # launches per variant; the first is a warm-up and is not used
KERNEL_TAG = "tile_kernel"
SECOND_PASS_TAG = "finalize_kernel"   # one dispatch after every two-pass launch of the tile kernel
SIZING_LAUNCHES = 40 # two-pass launches ahead of the variants: they size the workspace and load the chip


def main(task: str) -> int:
    M, K, N = TASKS[task]
    g = torch.Generator(device="cpu").manual_seed(0)
    dt = torch.bfloat16
    X = torch.randn(M, K, generator=g).to(dt).cuda()
    W = (torch.randn(N, K, generator=g) * K ** -0.5).to(dt).cuda()
    b = (torch.rand(N, generator=g) * 0.2 - 0.1).to(dt).cuda()
    gamma = (1 + 0.1 * torch.randn(N, generator=g)).to(dt).cuda()
    beta = (0.1 * torch.randn(N, generator=g)).to(dt).cuda()
    Y = torch.empty(M, N, dtype=dt, device="cuda")
    # size the workspace for the largest variant first so that no launch reallocates it
    B.ff_debug_force_variant(B.FF_VARIANT_TILED_TWOPASS)
    B.ff_debug_force_tile(128, 1)
    for _ in range(SIZING_LAUNCHES):
        B.ff_fused_linear_gelu_ln(X, W, b, gamma, beta, 1e-5, Y=Y)
    torch.cuda.synchronize()
    print("[variants] task %s: %d x %d x %d; dispatch order of %s:" % (task, M, K, N, KERNEL_TAG), flush=True)
    print("[variants] %d sizing launches, then %d launches each of: %s" %
          (SIZING_LAUNCHES, REPEATS, ", ".join(v[0] for v in VARIANTS)), flush=True)
    try:
        for label, tile, per_cu, waves, variant in VARIANTS:
            B.ff_debug_force_tile(tile, per_cu)
            B.ff_debug_force_waves(waves)
            B.ff_debug_force_variant(variant)
            for _ in range(REPEATS):
                B.ff_fused_linear_gelu_ln(X, W, b, gamma, beta, 1e-5, Y=Y)
            torch.cuda.synchronize()
            B.ff_check_device()
    finally:
        B.ff_debug_force_tile(0, 0)
        B.ff_debug_force_waves(0)
        B.ff_debug_force_variant(B.FF_VARIANT_AUTO)
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1]))
