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


def test_plan_query_is_host_arithmetic():
    """The automatic plan: one workgroup owns whole M for M <= 32 (bf16), else MFMA tiles whose size
    follows from how many of them there are per compute unit (256 units assumed without a GPU)."""
    q = lambda M, K, N, dt=B.FF_BF16: B.ff_plan_query(M, K, N, dt)
    big = q(4096, 4096, 4096)
    assert (big["variant"], big["tile_m"], big["tile_n"], big["waves"]) == (B.FF_VARIANT_TILED_FUSED, 256, 256, 8)
    assert (big["grid"], big["rounds"], big["workgroups_per_cu"], big["xcd_order"]) == (256, 1, 1, 1)
    assert q(65536, 1024, 1024)["rounds"] == 4 and q(8192, 4096, 16384)["rounds"] == 8
    small = q(16, 8192, 8192)
    assert small["variant"] == B.FF_VARIANT_SMALL_M and small["grid"] == 256
    assert q(16, 8192, 8192, B.FF_F32)["variant"] == B.FF_VARIANT_TILED_FUSED   # the small-M kernel is bf16 only
    assert q(33, 8192, 8192)["variant"] == B.FF_VARIANT_TILED_FUSED
    flat = q(1024, 4096, 8192)      # 128 tiles of 256 x 256 would leave half the units idle
    assert (flat["tile_m"], flat["tile_n"], flat["grid"], flat["workgroups_per_cu"]) == (128, 256, 256, 1)
    flat32 = q(1024, 4096, 8192, B.FF_F32)
    assert (flat32["tile_m"], flat32["tile_n"], flat32["grid"], flat32["workgroups_per_cu"]) == (128, 128, 512, 2)
    deep = q(2048, 8192, 2048)      # 256 tiles of 128 x 128: one per unit
    assert (deep["tile_m"], deep["tile_n"], deep["grid"]) == (128, 128, 256)
    tiny = q(256, 512, 512)
    assert (tiny["tile_m"], tiny["grid"]) == (64, 32)
    # a row of tiles wider than the launch cannot exchange statistics inside it: two passes
    assert q(256, 512, 64 * 1024 * 2)["variant"] == B.FF_VARIANT_TILED_TWOPASS
    with pytest.raises(B.FFError):
        q(0, 8, 8)
    with pytest.raises(B.FFError):
        q(8, 12, 8)
    lib = B.load()
    assert lib.ff_plan_query(8, 8, 8, B.FF_BF16, None) == 1
