"""CPU-only checks of the C-ABI library: it loads, exports every symbol the
header declares, and its host-side validation returns error codes (no kernel is
launched and no GPU is needed for any call made here)."""
import ctypes
import os
import re
import subprocess

import pytest

from paper_2511_01884_amd import binding as B
from paper_2511_01884_amd.build import LIB_PATH

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "ff.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ff_[a-z_0-9]+)\s*\(", text)))


def test_header_and_binding_agree():
    names = declared_functions()
    assert "ff_fused_linear_gelu_ln" in names
    assert sorted(B.EXPORTS) == names


def test_library_exports_every_declared_symbol():
    lib = B.load()
    for name in declared_functions():
        assert getattr(lib, name) is not None, name


def test_no_library_gemm_dependency():
    """The library must not link any BLAS / DNN library: there is no fallback path."""
    out = subprocess.check_output(["readelf", "-d", LIB_PATH], text=True).lower()
    for forbidden in ("blas", "miopen", "torch", "rocsolver", "hipdnn"):
        assert forbidden not in out, forbidden


def test_version_and_strings():
    assert B.ff_version() >= 100
    assert B.ff_status_string(0) == "FF_OK"
    for code in range(1, 9):
        assert B.ff_status_string(code).startswith("FF_ERR_")
    assert "unknown" in B.ff_status_string(99)


def test_argument_validation_without_gpu():
    lib = B.load()
    buf = (ctypes.c_char * 4096)()
    base = ctypes.addressof(buf)
    p = ctypes.c_void_p((base + 15) & ~15)
    mis = ctypes.c_void_p(((base + 15) & ~15) + 4)

    def call(X=p, W=p, M=8, K=8, N=8, dtype=B.FF_BF16, Y=p):
        return lib.ff_fused_linear_gelu_ln(X, W, None, None, None, 1e-5, M, K, N, dtype, Y, None)

    assert call(dtype=7) == 3            # FF_ERR_DTYPE
    assert call(M=0) == 2                # FF_ERR_SHAPE
    assert call(K=-8) == 2
    assert call(K=12) == 5               # bf16 needs K % 8 == 0
    assert call(N=12) == 5
    assert call(K=6, dtype=B.FF_F32) == 5  # fp32 needs K % 4 == 0
    assert call(X=None) == 1             # FF_ERR_NULL
    assert call(Y=None) == 1
    assert call(X=mis) == 4              # FF_ERR_ALIGN
    assert lib.ff_debug_linear(p, p, None, 8, 8, 8, B.FF_BF16, None, None) == 1


def test_workspace_bytes_is_host_arithmetic():
    assert B.ff_workspace_bytes(0, 8, 8, B.FF_BF16) == 0
    assert B.ff_workspace_bytes(8, 12, 8, B.FF_BF16) == 0
    small = B.ff_workspace_bytes(256, 512, 512, B.FF_F32)
    big = B.ff_workspace_bytes(8192, 4096, 16384, B.FF_BF16)
    assert 0 < small < big
    # control region + 8 bytes per row per N-tile
    assert big >= (1 << 20) + 8192 * 64 * 8


def test_force_variant_rejects_unknown():
    lib = B.load()
    assert lib.ff_debug_force_variant(9) == 5
    assert lib.ff_debug_force_variant(0) == 0
    assert lib.ff_debug_set_wait_limit_us(0) == 2
    assert lib.ff_debug_set_wait_limit_us(2000000) == 0
