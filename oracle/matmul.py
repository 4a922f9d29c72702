"""The three plain products of the linear layer, in fp64 (oracle; tests only).

Section 3.1.2, first differentiation formula: ``C = AB``, ``dA = dC B^T``,
``dB = A^T dC``; here ``Y = X W``, ``dX = dY W^T``, ``dW = X^T dY`` with
``X [M,K]``, ``W [K,N]``, ``Y [M,N]`` row-major.  The loops live in
``cube3d_oracle.c``; this file only marshals numpy arrays.
"""
import ctypes

import numpy as np

from . import build as _build

_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(_build.build())
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int64)
        i64 = ctypes.c_int64
        for name in ("oracle_matmul_nn", "oracle_matmul_nt", "oracle_matmul_tn"):
            f = getattr(lib, name)
            f.argtypes = [dp, dp, dp, i64, i64, i64, ctypes.c_int]
            f.restype = ctypes.c_int
        for name in ("oracle_matmul_nn_at", "oracle_matmul_nt_at", "oracle_matmul_tn_at"):
            f = getattr(lib, name)
            f.argtypes = [dp, dp, dp, i64, i64, i64, ip, ip, i64]
            f.restype = ctypes.c_int
        lib.oracle_max_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _f64(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    if a.ndim != 2:
        raise ValueError("expected a matrix")
    return a


def _dp(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def max_threads() -> int:
    return int(_load().oracle_max_threads())


def forward(X, W, threads: int = 1):
    """``Y = X W``."""
    X, W = _f64(X), _f64(W)
    M, K = X.shape
    K2, N = W.shape
    if K != K2:
        raise ValueError("inner dimensions differ")
    Y = np.empty((M, N), dtype=np.float64)
    rc = _load().oracle_matmul_nn(_dp(X), _dp(W), _dp(Y), M, K, N, threads)
    assert rc == 0
    return Y


def backward_dx(dY, W, threads: int = 1):
    """``dX = dY W^T``."""
    dY, W = _f64(dY), _f64(W)
    M, N = dY.shape
    K, N2 = W.shape
    if N != N2:
        raise ValueError("dY and W differ in N")
    dX = np.empty((M, K), dtype=np.float64)
    rc = _load().oracle_matmul_nt(_dp(dY), _dp(W), _dp(dX), M, K, N, threads)
    assert rc == 0
    return dX


def backward_dw(X, dY, threads: int = 1):
    """``dW = X^T dY``."""
    X, dY = _f64(X), _f64(dY)
    M, K = X.shape
    M2, N = dY.shape
    if M != M2:
        raise ValueError("X and dY differ in M")
    dW = np.empty((K, N), dtype=np.float64)
    rc = _load().oracle_matmul_tn(_dp(X), _dp(dY), _dp(dW), M, K, N, threads)
    assert rc == 0
    return dW


def _at(fn, A, B, dims, rows, cols):
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    cols = np.ascontiguousarray(cols, dtype=np.int64)
    if rows.shape != cols.shape or rows.ndim != 1:
        raise ValueError("rows/cols must be equal-length vectors")
    out = np.empty(rows.shape[0], dtype=np.float64)
    ip = ctypes.POINTER(ctypes.c_int64)
    rc = fn(_dp(A), _dp(B), _dp(out), *dims,
            rows.ctypes.data_as(ip), cols.ctypes.data_as(ip), rows.shape[0])
    if rc != 0:
        raise IndexError("sample position outside the output")
    return out


def forward_at(X, W, rows, cols):
    """Entries ``Y[rows[s], cols[s]]`` of ``Y = X W``."""
    X, W = _f64(X), _f64(W)
    return _at(_load().oracle_matmul_nn_at, X, W,
               (X.shape[0], X.shape[1], W.shape[1]), rows, cols)


def backward_dx_at(dY, W, rows, cols):
    """Entries ``dX[rows[s], cols[s]]`` of ``dX = dY W^T``."""
    dY, W = _f64(dY), _f64(W)
    return _at(_load().oracle_matmul_nt_at, dY, W,
               (dY.shape[0], W.shape[0], dY.shape[1]), rows, cols)


def backward_dw_at(X, dY, rows, cols):
    """Entries ``dW[rows[s], cols[s]]`` of ``dW = X^T dY``."""
    X, dY = _f64(X), _f64(dY)
    return _at(_load().oracle_matmul_tn_at, X, dY,
               (X.shape[0], X.shape[1], dY.shape[1]), rows, cols)
