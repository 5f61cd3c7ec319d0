"""CPU oracle (test infrastructure only): see oracle/oracle.c for what it computes.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import
this package.  It shares nothing with the GPU library.
"""
from .oracle import (  # noqa: F401
    CFLAGS,
    Oracle,
    SOURCE,
    build,
    cross_entropy,
    fused_linear_gelu_ln,
    gelu,
    layernorm_row,
    linear_row,
    linear_sub_rowmean_gelu_residual,
    num_threads,
    round_bf16,
)
