"""ctypes binding of libff.so: the same entry points as include/ff.h, taking
torch tensors.  Argument marshalling only — every step of the operator runs in
the HIP kernels.  There is no CPU or library fallback: if the extension is not
built, loading raises."""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

from .build import LIB_PATH

FF_F32, FF_BF16 = 0, 1
FF_OK = 0
FF_VARIANT_AUTO, FF_VARIANT_TILED_FUSED, FF_VARIANT_TILED_TWOPASS, FF_VARIANT_SMALL_M = 0, 1, 2, 3

EXPORTS = [
    "ff_fused_linear_gelu_ln", "ff_fused_linear_gelu_ln_noalloc", "ff_noalloc_max_bytes",
    "ff_fused_linear_sub_rowmean_gelu_residual", "ff_rowmean_workspace_bytes",
    "ff_cross_entropy_mean", "ff_cross_entropy_workspace_bytes",
    "ff_metric_selection", "ff_metric_select_host",
    "ff_workspace_bytes", "ff_plan_query", "ff_set_workspace", "ff_check_device",
    "ff_status_string", "ff_version", "ff_last_variant", "ff_debug_linear",
    "ff_debug_force_variant", "ff_debug_force_tile", "ff_debug_force_waves", "ff_debug_set_stagger_us", "ff_debug_set_timeline", "ff_debug_copy", "ff_debug_mfma_loop", "ff_debug_stream_read", "ff_debug_set_wait_limit_us", "ff_debug_expect_extra_arrivals",
]

_lib = None


class FFError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(ff_status_string(status))


def load() -> ctypes.CDLL:
    """Load libff.so (built beforehand by build.build_library / __graft_entry__.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                "%s is missing: build it with `python -m paper_2511_01884_amd.build`; "
                "there is no fallback path" % LIB_PATH)
        lib = ctypes.CDLL(LIB_PATH)
        vp, i64, ci = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
        lib.ff_fused_linear_gelu_ln.restype = ci
        lib.ff_fused_linear_gelu_ln.argtypes = [vp, vp, vp, vp, vp, ctypes.c_float, i64, i64, i64, ci, vp, vp]
        lib.ff_fused_linear_gelu_ln_noalloc.restype = ci
        lib.ff_fused_linear_gelu_ln_noalloc.argtypes = [vp, vp, vp, vp, vp, ctypes.c_float, i64, i64, i64, ci, vp, vp]
        lib.ff_noalloc_max_bytes.restype = ctypes.c_size_t
        lib.ff_noalloc_max_bytes.argtypes = []
        lib.ff_fused_linear_sub_rowmean_gelu_residual.restype = ci
        lib.ff_fused_linear_sub_rowmean_gelu_residual.argtypes = [vp, vp, vp, vp, i64, i64, i64, ci, vp, vp]
        lib.ff_rowmean_workspace_bytes.restype = ctypes.c_size_t
        lib.ff_rowmean_workspace_bytes.argtypes = [i64, i64, i64, ci]
        lib.ff_cross_entropy_mean.restype = ci
        lib.ff_cross_entropy_mean.argtypes = [vp, vp, i64, i64, ci, vp, vp, vp]
        lib.ff_metric_selection.restype = ci
        lib.ff_metric_selection.argtypes = [vp, vp, i64, i64, i64, ci, ctypes.c_double, ctypes.c_double, ci,
                                            vp, vp, vp, vp, vp, vp]
        lib.ff_metric_select_host.restype = ci
        lib.ff_metric_select_host.argtypes = [vp, vp, i64, i64, ci, ctypes.c_double, ci, vp, vp, vp, vp]
        lib.ff_cross_entropy_workspace_bytes.restype = ctypes.c_size_t
        lib.ff_cross_entropy_workspace_bytes.argtypes = [i64, i64, ci]
        lib.ff_workspace_bytes.restype = ctypes.c_size_t
        lib.ff_workspace_bytes.argtypes = [i64, i64, i64, ci]
        lib.ff_set_workspace.restype = ci
        lib.ff_set_workspace.argtypes = [vp, ctypes.c_size_t]
        lib.ff_check_device.restype = ci
        lib.ff_check_device.argtypes = [vp]
        lib.ff_status_string.restype = ctypes.c_char_p
        lib.ff_status_string.argtypes = [ci]
        lib.ff_version.restype = ci
        lib.ff_last_variant.restype = ci
        lib.ff_debug_linear.restype = ci
        lib.ff_debug_linear.argtypes = [vp, vp, vp, i64, i64, i64, ci, vp, vp]
        lib.ff_debug_force_variant.restype = ci
        lib.ff_debug_force_variant.argtypes = [ci]
        lib.ff_debug_copy.restype = ci
        lib.ff_debug_copy.argtypes = [vp, vp, ctypes.c_size_t, vp]
        lib.ff_debug_mfma_loop.restype = ci
        lib.ff_debug_mfma_loop.argtypes = [i64, ctypes.POINTER(ctypes.c_double)]
        lib.ff_debug_stream_read.restype = ci
        lib.ff_debug_stream_read.argtypes = [vp, ctypes.c_size_t]
        lib.ff_debug_force_tile.restype = ci
        lib.ff_debug_force_tile.argtypes = [ci, ci]
        lib.ff_debug_force_waves.restype = ci
        lib.ff_debug_force_waves.argtypes = [ci]
        lib.ff_debug_set_stagger_us.restype = ci
        lib.ff_debug_set_stagger_us.argtypes = [ci]
        lib.ff_plan_query.restype = ci
        lib.ff_plan_query.argtypes = [i64, i64, i64, ci, ctypes.POINTER(ctypes.c_int)]
        lib.ff_debug_set_timeline.restype = ci
        lib.ff_debug_set_timeline.argtypes = [vp, ctypes.c_size_t]
        lib.ff_debug_set_wait_limit_us.restype = ci
        lib.ff_debug_set_wait_limit_us.argtypes = [i64]
        lib.ff_debug_expect_extra_arrivals.restype = ci
        lib.ff_debug_expect_extra_arrivals.argtypes = [ci]
        _lib = lib
    return _lib


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return FF_F32
    if t.dtype == torch.bfloat16:
        return FF_BF16
    raise TypeError("tensors must be float32 or bfloat16")


def _ptr(t: Optional[torch.Tensor], like: Optional[torch.Tensor] = None):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("tensors must be contiguous device tensors")
    if like is not None and (t.dtype != like.dtype or t.device != like.device):
        raise ValueError("all tensors must share dtype and device")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def ff_status_string(status: int) -> str:
    return load().ff_status_string(int(status)).decode()


def ff_version() -> int:
    return int(load().ff_version())


def ff_last_variant() -> int:
    return int(load().ff_last_variant())


def ff_plan_query(M: int, K: int, N: int, dtype: int) -> dict:
    """The launch plan a call with this shape would take (no launch)."""
    out = (ctypes.c_int * 8)()
    rc = load().ff_plan_query(M, K, N, dtype, out)
    if rc != FF_OK:
        raise FFError(rc)
    keys = ("variant", "tile_m", "tile_n", "waves", "grid", "rounds", "workgroups_per_cu", "xcd_order")
    return dict(zip(keys, (int(v) for v in out)))


def ff_workspace_bytes(M: int, K: int, N: int, dtype: int) -> int:
    return int(load().ff_workspace_bytes(M, K, N, dtype))


def ff_set_workspace(buf: Optional[torch.Tensor]) -> None:
    if buf is None:
        rc = load().ff_set_workspace(None, 0)
    else:
        rc = load().ff_set_workspace(ctypes.c_void_p(buf.data_ptr()), buf.numel() * buf.element_size())
    if rc != FF_OK:
        raise FFError(rc)


def ff_check_device(stream=None) -> None:
    rc = load().ff_check_device(_stream(stream))
    if rc != FF_OK:
        raise FFError(rc)


def ff_debug_force_variant(variant: int) -> None:
    rc = load().ff_debug_force_variant(int(variant))
    if rc != FF_OK:
        raise FFError(rc)


def ff_debug_copy(src: torch.Tensor, dst: torch.Tensor, stream=None) -> None:
    """dst <- src with the library's plain copy kernel (counter calibration)."""
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes:
        raise ValueError("src and dst must have the same size in bytes")
    with torch.cuda.device(src.device):
        rc = load().ff_debug_copy(_ptr(src), _ptr(dst), nbytes, _stream(stream))
    if rc != FF_OK:
        raise FFError(rc)


def ff_debug_mfma_loop(iters: int) -> float:
    """Launches the MFMA-only loop on the null stream of the current device; returns its flop count."""
    flops = ctypes.c_double(0.0)
    rc = load().ff_debug_mfma_loop(int(iters), ctypes.byref(flops))
    if rc != FF_OK:
        raise FFError(rc)
    return float(flops.value)


def ff_debug_stream_read(src: torch.Tensor) -> int:
    """Launches the streaming-read kernel over src on the null stream; returns the bytes read."""
    nbytes = src.numel() * src.element_size()
    with torch.cuda.device(src.device):
        rc = load().ff_debug_stream_read(_ptr(src), nbytes)
    if rc != FF_OK:
        raise FFError(rc)
    return nbytes


def ff_debug_force_tile(tile: int, wg_per_cu: int = 0) -> None:
    rc = load().ff_debug_force_tile(int(tile), int(wg_per_cu))
    if rc != FF_OK:
        raise FFError(rc)


def ff_debug_force_waves(waves: int) -> None:
    rc = load().ff_debug_force_waves(int(waves))
    if rc != FF_OK:
        raise FFError(rc)


def ff_debug_set_stagger_us(us: int) -> None:
    rc = load().ff_debug_set_stagger_us(int(us))
    if rc != FF_OK:
        raise FFError(rc)


def ff_debug_set_timeline(buf: Optional[torch.Tensor]) -> None:
    """Binds a device tensor (any 8-byte dtype) for the tiled kernels' phase timestamps; None unbinds."""
    if buf is None:
        rc = load().ff_debug_set_timeline(None, 0)
    else:
        with torch.cuda.device(buf.device):
            rc = load().ff_debug_set_timeline(ctypes.c_void_p(buf.data_ptr()), buf.numel() * buf.element_size())
    if rc != FF_OK:
        raise FFError(rc)


def ff_debug_set_wait_limit_us(us: int) -> None:
    rc = load().ff_debug_set_wait_limit_us(int(us))
    if rc != FF_OK:
        raise FFError(rc)


def ff_debug_expect_extra_arrivals(count: int) -> None:
    rc = load().ff_debug_expect_extra_arrivals(int(count))
    if rc != FF_OK:
        raise FFError(rc)


def ff_noalloc_max_bytes() -> int:
    return int(load().ff_noalloc_max_bytes())


def ff_fused_linear_gelu_ln_noalloc(X: torch.Tensor, W: torch.Tensor, b: Optional[torch.Tensor],
                                    gamma: Optional[torch.Tensor], beta: Optional[torch.Tensor],
                                    eps: float, Y: torch.Tensor, stream=None) -> torch.Tensor:
    """The entry point that allocates nothing: the caller passes every tensor, Y included."""
    return ff_fused_linear_gelu_ln(X, W, b, gamma, beta, eps, Y=Y, stream=stream, _entry="ff_fused_linear_gelu_ln_noalloc")


def ff_fused_linear_gelu_ln(X: torch.Tensor, W: torch.Tensor, b: Optional[torch.Tensor],
                            gamma: Optional[torch.Tensor], beta: Optional[torch.Tensor],
                            eps: float, Y: Optional[torch.Tensor] = None, stream=None,
                            _entry: str = "ff_fused_linear_gelu_ln") -> torch.Tensor:
    """Y = LayerNorm_N(GELU(X W^T + b)) * gamma + beta on the device of X.
    Allocates Y with torch if not given; everything else happens in libff.so."""
    if X.dim() != 2 or W.dim() != 2 or X.shape[1] != W.shape[1]:
        raise ValueError("X must be [M,K] and W [N,K]")
    M, K = X.shape
    N = W.shape[0]
    for v in (b, gamma, beta):
        if v is not None and tuple(v.shape) != (N,):
            raise ValueError("b, gamma, beta must have shape [N]")
    if Y is None:
        Y = torch.empty((M, N), dtype=X.dtype, device=X.device)
    elif tuple(Y.shape) != (M, N):
        raise ValueError("Y must be [M,N]")
    with torch.cuda.device(X.device):
        rc = getattr(load(), _entry)(_ptr(X), _ptr(W, X), _ptr(b, X), _ptr(gamma, X),
                                     _ptr(beta, X), float(eps), M, K, N, _dtype_code(X),
                                     _ptr(Y, X), _stream(stream))
    if rc != FF_OK:
        raise FFError(rc)
    return Y


def ff_fused_linear_sub_rowmean_gelu_residual(X: torch.Tensor, W: torch.Tensor, b: Optional[torch.Tensor],
                                              s: Optional[torch.Tensor], Out: Optional[torch.Tensor] = None,
                                              stream=None) -> torch.Tensor:
    """Out = X + GELU(mean_n(X W^T + b - s)) on the device of X (allocates Out if not given)."""
    if X.dim() != 2 or W.dim() != 2 or X.shape[1] != W.shape[1]:
        raise ValueError("X must be [M,K] and W [N,K]")
    M, K = X.shape
    N = W.shape[0]
    for v in (b, s):
        if v is not None and tuple(v.shape) != (N,):
            raise ValueError("b and s must have shape [N]")
    if Out is None:
        Out = torch.empty_like(X)
    elif tuple(Out.shape) != (M, K):
        raise ValueError("Out must be [M,K]")
    with torch.cuda.device(X.device):
        rc = load().ff_fused_linear_sub_rowmean_gelu_residual(
            _ptr(X), _ptr(W, X), _ptr(b, X), _ptr(s, X), M, K, N, _dtype_code(X), _ptr(Out, X),
            _stream(stream))
    if rc != FF_OK:
        raise FFError(rc)
    return Out


def ff_rowmean_workspace_bytes(M: int, K: int, N: int, dtype: int) -> int:
    return int(load().ff_rowmean_workspace_bytes(M, K, N, dtype))


def ff_cross_entropy_mean(logits: torch.Tensor, targets: torch.Tensor, row_loss: Optional[torch.Tensor] = None,
                          mean_loss: Optional[torch.Tensor] = None, with_rows: bool = False, stream=None):
    """Mean over rows of log(sum_c exp(L[r][c])) - L[r][t[r]]; returns the one-element fp32 tensor,
    or (mean, row_loss) when per-row losses are asked for.  Output tensors are allocated if not given."""
    if logits.dim() != 2 or targets.dim() != 1 or targets.shape[0] != logits.shape[0]:
        raise ValueError("logits must be [B,C] and targets [B]")
    if targets.dtype != torch.int64 or not targets.is_cuda or not targets.is_contiguous() \
            or targets.device != logits.device:
        raise ValueError("targets must be a contiguous int64 tensor on the device of logits")
    B, C = logits.shape
    if mean_loss is None:
        mean_loss = torch.empty(1, dtype=torch.float32, device=logits.device)
    if row_loss is None and with_rows:
        row_loss = torch.empty(B, dtype=torch.float32, device=logits.device)
    for v, n in ((mean_loss, 1), (row_loss, B)):
        if v is not None and (v.dtype != torch.float32 or v.numel() != n or v.device != logits.device
                              or not v.is_contiguous()):
            raise ValueError("loss outputs must be contiguous float32 tensors of 1 and B elements")
    with torch.cuda.device(logits.device):
        rc = load().ff_cross_entropy_mean(
            _ptr(logits), ctypes.c_void_p(targets.data_ptr()), B, C, _dtype_code(logits),
            None if row_loss is None else ctypes.c_void_p(row_loss.data_ptr()),
            ctypes.c_void_p(mean_loss.data_ptr()), _stream(stream))
    if rc != FF_OK:
        raise FFError(rc)
    return (mean_loss, row_loss) if row_loss is not None else mean_loss


def ff_cross_entropy_workspace_bytes(B: int, C: int, dtype: int) -> int:
    return int(load().ff_cross_entropy_workspace_bytes(B, C, dtype))


def _selection_outputs(n: int, J: int, k: int):
    import numpy as np
    return (np.empty((n, J), dtype=np.float64), np.empty(J, dtype=np.float64),
            np.empty((n, k), dtype=np.int32), np.empty(J, dtype=np.uint8), np.empty(1, dtype=np.float64))


def _selection_result(r, score, top, selected, threshold):
    return {"r": r, "score": score, "top": [[int(m) for m in row if m >= 0] for row in top],
            "selected": [int(m) for m in selected.nonzero()[0]], "threshold": float(threshold[0])}


def ff_metric_selection(values: torch.Tensor, runtime: torch.Tensor, top_k: int = 20, percentile: float = 75.0,
                        collinear_tau: float = 0.0, min_tasks: int = 2, stream=None):
    """Metric selection on device arrays values [n,V,J] and runtime [n,V] (float64); returns a dict of
    host results: r, score, top (lists of metric indices), selected (indices), threshold."""
    if values.dim() != 3 or runtime.dim() != 2 or tuple(runtime.shape) != tuple(values.shape[:2]):
        raise ValueError("values must be [n,V,J] and runtime [n,V]")
    if values.dtype != torch.float64 or runtime.dtype != torch.float64:
        raise TypeError("values and runtime must be float64")
    for t in (values, runtime):
        if not t.is_cuda or not t.is_contiguous() or t.device != values.device:
            raise ValueError("values and runtime must be contiguous tensors on one device")
    n, V, J = values.shape
    r, score, top, selected, threshold = _selection_outputs(n, J, int(top_k))
    with torch.cuda.device(values.device):
        rc = load().ff_metric_selection(
            ctypes.c_void_p(values.data_ptr()), ctypes.c_void_p(runtime.data_ptr()), n, V, J, int(top_k),
            float(percentile), float(collinear_tau), int(min_tasks), r.ctypes.data, score.ctypes.data,
            top.ctypes.data, selected.ctypes.data, threshold.ctypes.data, _stream(stream))
    if rc != FF_OK:
        raise FFError(rc)
    return _selection_result(r, score, top, selected, threshold)


def ff_metric_select_host(r, keep=None, top_k: int = 20, percentile: float = 75.0, min_tasks: int = 2):
    """The host part alone: r [n,J] float64 numpy, keep [n,J] uint8 numpy or None."""
    import numpy as np
    r = np.ascontiguousarray(r, dtype=np.float64)
    n, J = r.shape
    if keep is not None:
        keep = np.ascontiguousarray(keep, dtype=np.uint8)
        if keep.shape != r.shape:
            raise ValueError("keep must have the shape of r")
    _, score, top, selected, threshold = _selection_outputs(n, J, int(top_k))
    rc = load().ff_metric_select_host(r.ctypes.data, None if keep is None else keep.ctypes.data, n, J, int(top_k),
                                      float(percentile), int(min_tasks), top.ctypes.data, score.ctypes.data,
                                      selected.ctypes.data, threshold.ctypes.data)
    if rc != FF_OK:
        raise FFError(rc)
    return _selection_result(r, score, top, selected, threshold)


def ff_debug_linear(X: torch.Tensor, W: torch.Tensor, b: Optional[torch.Tensor],
                    Z: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """fp32 Z = X W^T + b through the tiled MFMA core (test hook)."""
    M, K = X.shape
    N = W.shape[0]
    if Z is None:
        Z = torch.empty((M, N), dtype=torch.float32, device=X.device)
    with torch.cuda.device(X.device):
        rc = load().ff_debug_linear(_ptr(X), _ptr(W, X), _ptr(b, X), M, K, N, _dtype_code(X),
                                    ctypes.c_void_p(Z.data_ptr()), _stream(stream))
    if rc != FF_OK:
        raise FFError(rc)
    return Z
