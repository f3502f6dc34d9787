"""ctypes access to the fp64 CPU oracle (``attnw_oracle.c``).

TEST INFRASTRUCTURE.  Only the tests, the smoke check and the bench's
``cpu_baseline`` leg may import this package; the product package never does.
It shares nothing with the HIP library.

Arrays: fp32 inputs are ``numpy.float32``, bf16 inputs are ``numpy.uint16`` bit
patterns, fp64 inputs are ``numpy.float64``.  Outputs are always fp64.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "attnw_oracle.c")
_LIB = os.path.join(_HERE, "libattnw_oracle.so")

_DT = {"f32": 0, "bf16": 1, "f64": 2}
_NP = {"f32": np.float32, "bf16": np.uint16, "f64": np.float64}

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, no fast-math, OpenMP for row parallelism)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               _SRC, "-o", _LIB, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i64, vp, ci, cf = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int, ctypes.c_float
        lib.oracle_scores.argtypes = [vp, vp, ci, i64, i64, cf, i64, i64, vp, ci]
        lib.oracle_attention_weights.argtypes = [vp, vp, ci, i64, i64, cf, i64, i64, vp, ci]
        lib.oracle_softmax.argtypes = [vp, ci, i64, i64, i64, i64, vp, ci]
        lib.oracle_attention_output.argtypes = [vp, vp, vp, ci, i64, i64, i64, cf, i64, i64, vp, vp, ci]
        lib.oracle_softmax_plain.argtypes = [vp, ci, i64, i64, vp]
        lib.oracle_scale.argtypes = [vp, ci, i64, cf, vp]
        lib.oracle_threads_used.restype = ci
        _lib = lib
    return _lib


def _as(a: np.ndarray, dtype: str) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype != _NP[dtype]:
        raise TypeError(f"dtype {dtype} wants {_NP[dtype].__name__} storage, got {a.dtype}")
    return a


def threads_used() -> int:
    return int(_load().oracle_threads_used())


def scores(Q: np.ndarray, K: np.ndarray, dtype: str, scale, rows: Optional[tuple] = None,
           threads: int = 0) -> np.ndarray:
    """Scaled scores of ONE head: Q, K are [N, d]; returns fp64 [r1-r0, N]."""
    Q, K = _as(Q, dtype), _as(K, dtype)
    N, d = Q.shape
    assert K.shape == (N, d)
    r0, r1 = (0, N) if rows is None else rows
    out = np.empty((r1 - r0, N), dtype=np.float64)
    rc = _load().oracle_scores(Q.ctypes.data, K.ctypes.data, _DT[dtype], N, d, float(np.float32(scale)),
                               r0, r1, out.ctypes.data, threads)
    if rc:
        raise ValueError("oracle_scores: bad arguments")
    return out


def attention_weights(Q: np.ndarray, K: np.ndarray, dtype: str, scale, rows: Optional[tuple] = None,
                      threads: int = 0) -> np.ndarray:
    """Attention weights of ONE head: Q, K are [N, d]; returns fp64 [r1-r0, N]."""
    Q, K = _as(Q, dtype), _as(K, dtype)
    N, d = Q.shape
    assert K.shape == (N, d)
    r0, r1 = (0, N) if rows is None else rows
    out = np.empty((r1 - r0, N), dtype=np.float64)
    rc = _load().oracle_attention_weights(Q.ctypes.data, K.ctypes.data, _DT[dtype], N, d,
                                          float(np.float32(scale)), r0, r1, out.ctypes.data, threads)
    if rc:
        raise ValueError("oracle_attention_weights: bad arguments")
    return out


def attention_weights_bh(Q: np.ndarray, K: np.ndarray, dtype: str, scale, threads: int = 0) -> np.ndarray:
    """All heads: Q, K are [B, H, N, d]; returns fp64 [B, H, N, N] (small cases only)."""
    B, H, N, d = Q.shape
    out = np.empty((B, H, N, N), dtype=np.float64)
    for b in range(B):
        for h in range(H):
            out[b, h] = attention_weights(Q[b, h], K[b, h], dtype, scale, threads=threads)
    return out


def attention_output(Q: np.ndarray, K: np.ndarray, V: np.ndarray, dtype: str, scale, rows: Optional[tuple] = None,
                     threads: int = 0, return_weights: bool = False):
    """Attention output of ONE head: Q, K are [N, d], V is [N, dv]; returns fp64 [r1-r0, dv]
    (and the fp64 weights [r1-r0, N] it was formed from, on request)."""
    Q, K, V = _as(Q, dtype), _as(K, dtype), _as(V, dtype)
    N, d = Q.shape
    assert K.shape == (N, d) and V.shape[0] == N
    dv = V.shape[1]
    r0, r1 = (0, N) if rows is None else rows
    out = np.empty((r1 - r0, dv), dtype=np.float64)
    P = np.empty((r1 - r0, N), dtype=np.float64)
    rc = _load().oracle_attention_output(Q.ctypes.data, K.ctypes.data, V.ctypes.data, _DT[dtype], N, d, dv,
                                         float(np.float32(scale)), r0, r1, out.ctypes.data, P.ctypes.data, threads)
    if rc:
        raise ValueError("oracle_attention_output: bad arguments")
    return (out, P) if return_weights else out


def softmax(S: np.ndarray, dtype: str, rows: Optional[tuple] = None, threads: int = 0) -> np.ndarray:
    """Row softmax (max-subtracted form) of a [rows, cols] matrix; returns fp64."""
    S = _as(S, dtype)
    R, C = S.shape
    r0, r1 = (0, R) if rows is None else rows
    out = np.empty((r1 - r0, C), dtype=np.float64)
    rc = _load().oracle_softmax(S.ctypes.data, _DT[dtype], R, C, r0, r1, out.ctypes.data, threads)
    if rc:
        raise ValueError("oracle_softmax: bad arguments")
    return out


def softmax_plain(S: np.ndarray, dtype: str) -> np.ndarray:
    """The literal definition without max subtraction (small-magnitude inputs only)."""
    S = _as(S, dtype)
    R, C = S.shape
    out = np.empty((R, C), dtype=np.float64)
    rc = _load().oracle_softmax_plain(S.ctypes.data, _DT[dtype], R, C, out.ctypes.data)
    if rc:
        raise ValueError("oracle_softmax_plain: bad arguments")
    return out


def scale(X: np.ndarray, dtype: str, scale) -> np.ndarray:
    """The scaling step alone: fp64 ``scale * X`` (exact), same shape as X."""
    X = _as(X, dtype)
    out = np.empty(X.shape, dtype=np.float64)
    if X.size and _load().oracle_scale(X.ctypes.data, _DT[dtype], X.size, float(np.float32(scale)), out.ctypes.data):
        raise ValueError("oracle_scale: bad arguments")
    return out
