"""ctypes front end of the fp64 CPU oracle in oracle.c (test infrastructure only).

The arithmetic lives in oracle.c; this file only marshals numpy arrays.  Inputs
are float32 arrays holding the exact values given to the GPU (a bfloat16 value
widened to float32 is exact), outputs are float64.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
SOURCE = os.path.join(_HERE, "oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

CFLAGS = ["-O2", "-fno-fast-math", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC"]


def build(force: bool = False) -> str:
    """Compile oracle.c with gcc.  Returns the path of the shared library."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(SOURCE):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", *CFLAGS, "-o", tmp, SOURCE, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _bind(path: str):
    lib = ctypes.CDLL(path)
    dp = ctypes.POINTER(ctypes.c_double)
    fp = ctypes.POINTER(ctypes.c_float)
    ip = ctypes.POINTER(ctypes.c_int64)
    i64 = ctypes.c_int64
    lib.oracle_num_threads.restype = ctypes.c_int
    lib.oracle_gelu.restype = ctypes.c_double
    lib.oracle_gelu.argtypes = [ctypes.c_double]
    lib.oracle_linear_row.restype = None
    lib.oracle_linear_row.argtypes = [fp, fp, fp, i64, i64, dp]
    lib.oracle_layernorm_row.restype = None
    lib.oracle_layernorm_row.argtypes = [dp, i64, fp, fp, ctypes.c_double, dp, dp, dp]
    lib.oracle_fused_linear_gelu_ln.restype = ctypes.c_int
    lib.oracle_fused_linear_gelu_ln.argtypes = [
        fp, fp, fp, fp, fp, ctypes.c_float, i64, i64, i64, ip, i64, dp, dp, dp, dp, dp]
    lib.oracle_round_bf16.restype = None
    lib.oracle_round_bf16.argtypes = [dp, i64, dp]
    lib.oracle_linear_sub_rowmean_gelu_residual.restype = ctypes.c_int
    lib.oracle_linear_sub_rowmean_gelu_residual.argtypes = [fp, fp, fp, fp, i64, i64, i64, ip, i64, dp, dp]
    lib.oracle_cross_entropy.restype = ctypes.c_int
    lib.oracle_cross_entropy.argtypes = [fp, ip, i64, i64, dp, dp]
    return lib


def _f32(a, shape=None) -> Optional[np.ndarray]:
    if a is None:
        return None
    a = np.ascontiguousarray(a, dtype=np.float32)
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise ValueError("expected shape %s, got %s" % (shape, a.shape))
    return a


def _ptr(a, ctype):
    if a is None:
        return None
    return a.ctypes.data_as(ctypes.POINTER(ctype))


class Oracle:
    """One loaded build of oracle.c.  The module-level functions use the default
    build; tests that plant mistakes load altered builds through this class."""

    def __init__(self, lib_path: Optional[str] = None):
        self._lib = _bind(lib_path if lib_path is not None else build())

    def num_threads(self) -> int:
        return int(self._lib.oracle_num_threads())


    def gelu(self, z: float) -> float:
        return float(self._lib.oracle_gelu(float(z)))


    def linear_row(self, x, W, b=None) -> np.ndarray:
        W = _f32(W)
        N, K = W.shape
        x = _f32(x, (K,))
        b = _f32(b, (N,))
        z = np.empty(N, dtype=np.float64)
        self._lib.oracle_linear_row(_ptr(x, ctypes.c_float), _ptr(W, ctypes.c_float),
                                  _ptr(b, ctypes.c_float), K, N, _ptr(z, ctypes.c_double))
        return z


    def layernorm_row(self, g, gamma=None, beta=None, eps: float = 0.0):
        """Returns (y, mu, var) for one row; eps is used as given (fp64)."""
        g = np.ascontiguousarray(g, dtype=np.float64)
        N = g.shape[0]
        gamma = _f32(gamma, (N,))
        beta = _f32(beta, (N,))
        y = np.empty(N, dtype=np.float64)
        mu = ctypes.c_double()
        var = ctypes.c_double()
        self._lib.oracle_layernorm_row(_ptr(g, ctypes.c_double), N, _ptr(gamma, ctypes.c_float),
                                     _ptr(beta, ctypes.c_float), float(eps),
                                     _ptr(y, ctypes.c_double), ctypes.byref(mu), ctypes.byref(var))
        return y, mu.value, var.value


    def fused_linear_gelu_ln(self, X, W, b=None, gamma=None, beta=None, eps: float = 1e-5,
                             rows: Optional[Sequence[int]] = None, stages: bool = False):
        """Y (float64, [R,N]) for all rows of X, or for the listed rows only.

        With stages=True returns a dict with Y, Z, G, mu, var.
        eps is rounded to float32 first, as the GPU entry point receives a float.
        """
        X = _f32(X)
        W = _f32(W)
        M, K = X.shape
        N, K2 = W.shape
        if K2 != K:
            raise ValueError("X is [M,K], W must be [N,K]")
        b = _f32(b, (N,))
        gamma = _f32(gamma, (N,))
        beta = _f32(beta, (N,))
        if rows is not None:
            rows_a = np.ascontiguousarray(rows, dtype=np.int64)
            R = int(rows_a.shape[0])
        else:
            rows_a = None
            R = M
        Y = np.empty((R, N), dtype=np.float64)
        Z = np.empty((R, N), dtype=np.float64) if stages else None
        G = np.empty((R, N), dtype=np.float64) if stages else None
        mu = np.empty(R, dtype=np.float64) if stages else None
        var = np.empty(R, dtype=np.float64) if stages else None
        rc = self._lib.oracle_fused_linear_gelu_ln(
            _ptr(X, ctypes.c_float), _ptr(W, ctypes.c_float), _ptr(b, ctypes.c_float),
            _ptr(gamma, ctypes.c_float), _ptr(beta, ctypes.c_float), float(np.float32(eps)),
            M, K, N, _ptr(rows_a, ctypes.c_int64), R,
            _ptr(Y, ctypes.c_double), _ptr(Z, ctypes.c_double), _ptr(G, ctypes.c_double),
            _ptr(mu, ctypes.c_double), _ptr(var, ctypes.c_double))
        if rc != 0:
            raise RuntimeError("oracle_fused_linear_gelu_ln failed (rc=%d)" % rc)
        if stages:
            return {"Y": Y, "Z": Z, "G": G, "mu": mu, "var": var}
        return Y


    def linear_sub_rowmean_gelu_residual(self, X, W, b=None, s=None,
                                         rows: Optional[Sequence[int]] = None, with_rowval: bool = False):
        """Out (float64, [R,K]) = X + GELU(mean_n(X W^T + b - s)), for all or the listed rows."""
        X = _f32(X)
        W = _f32(W)
        M, K = X.shape
        N, K2 = W.shape
        if K2 != K:
            raise ValueError("X is [M,K], W must be [N,K]")
        b = _f32(b, (N,))
        s = _f32(s, (N,))
        if rows is not None:
            rows_a = np.ascontiguousarray(rows, dtype=np.int64)
            R = int(rows_a.shape[0])
        else:
            rows_a = None
            R = M
        Out = np.empty((R, K), dtype=np.float64)
        rv = np.empty(R, dtype=np.float64)
        rc = self._lib.oracle_linear_sub_rowmean_gelu_residual(
            _ptr(X, ctypes.c_float), _ptr(W, ctypes.c_float), _ptr(b, ctypes.c_float),
            _ptr(s, ctypes.c_float), M, K, N, _ptr(rows_a, ctypes.c_int64), R,
            _ptr(Out, ctypes.c_double), _ptr(rv, ctypes.c_double))
        if rc != 0:
            raise RuntimeError("oracle_linear_sub_rowmean_gelu_residual failed (rc=%d)" % rc)
        return (Out, rv) if with_rowval else Out

    def cross_entropy(self, logits, targets):
        """(row_loss float64 [B], mean float) of the row-wise cross-entropy of logits [B,C], targets [B]."""
        L = _f32(logits)
        B, C = L.shape
        t = np.ascontiguousarray(targets, dtype=np.int64)
        if t.shape != (B,):
            raise ValueError("targets must be [B]")
        rl = np.empty(B, dtype=np.float64)
        mean = ctypes.c_double(0.0)
        rc = self._lib.oracle_cross_entropy(_ptr(L, ctypes.c_float), _ptr(t, ctypes.c_int64), B, C,
                                            _ptr(rl, ctypes.c_double), ctypes.byref(mean))
        if rc != 0:
            raise RuntimeError("oracle_cross_entropy failed (rc=%d)" % rc)
        return rl, float(mean.value)

    def round_bf16(self, a) -> np.ndarray:
        """Nearest bfloat16 value (ties to even) of each fp64 element, as float64."""
        a = np.ascontiguousarray(a, dtype=np.float64)
        out = np.empty_like(a)
        self._lib.oracle_round_bf16(_ptr(a, ctypes.c_double), a.size, _ptr(out, ctypes.c_double))
        return out


_default: Optional[Oracle] = None


def _get() -> Oracle:
    global _default
    if _default is None:
        _default = Oracle()
    return _default


def num_threads() -> int:
    return _get().num_threads()


def gelu(z: float) -> float:
    return _get().gelu(z)


def linear_row(x, W, b=None):
    return _get().linear_row(x, W, b)


def layernorm_row(g, gamma=None, beta=None, eps: float = 0.0):
    return _get().layernorm_row(g, gamma, beta, eps)


def fused_linear_gelu_ln(X, W, b=None, gamma=None, beta=None, eps: float = 1e-5,
                         rows=None, stages: bool = False):
    return _get().fused_linear_gelu_ln(X, W, b, gamma, beta, eps, rows, stages)


def linear_sub_rowmean_gelu_residual(X, W, b=None, s=None, rows=None, with_rowval: bool = False):
    return _get().linear_sub_rowmean_gelu_residual(X, W, b, s, rows, with_rowval)


def cross_entropy(logits, targets):
    return _get().cross_entropy(logits, targets)


def round_bf16(a):
    return _get().round_bf16(a)
