"""Seeded synthetic inputs for the attention-weight workloads.

This module only *draws numbers*: it holds none of the method's arithmetic
(no dot products, no exponentials of scores, no normalisation).  Both the CPU
oracle's tests and the GPU harness feed on the arrays it returns, so that the
two sides always see bit-identical inputs.

The paper measures on synthetic matrices of a given size (Table I: square
n x n score matrices, n = 1024 ... 16384; fused kernel section: Q and K of
shape n x d_k with d_k = 128) and does not say how the entries were drawn.
The five workloads below take those shapes and fix the distribution.

Generator (id ``splitmix64-boxmuller-v1``):
  * a counter-based stream: word(seed, stream, i) is the splitmix64 output
    function applied to ``key(seed, stream) + (i + 1) * GOLDEN``;
  * uniforms ``u = (word >> 11 + 0.5) * 2**-53`` in the open interval (0, 1);
  * standard normals by Box-Muller in fp64 from words 2i and 2i+1;
  * one rounding fp64 -> fp32 (nearest-even); bf16 storage takes the fp32
    value and rounds it nearest-even to the upper 16 bits.
Streams: 0 = Q, 1 = K, 2 = S, 3 = peak mask, 4 / 5 = per-row factors of Q / K.

bf16 arrays are returned as ``numpy.uint16`` bit patterns.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np

GENERATOR_ID = "splitmix64-boxmuller-v1"

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_STREAM_MUL = np.uint64(0xD1B54A32D192ED03)
_CHUNK = 1 << 22

STREAM_Q, STREAM_K, STREAM_S, STREAM_MASK, STREAM_QROW, STREAM_KROW, STREAM_V = range(7)


def _mix(x: np.ndarray) -> np.ndarray:
    """splitmix64 output function on a uint64 array (wraps modulo 2**64)."""
    x = x.copy()
    x ^= x >> np.uint64(30)
    x *= _M1
    x ^= x >> np.uint64(27)
    x *= _M2
    x ^= x >> np.uint64(31)
    return x


def _key(seed: int, stream: int) -> np.uint64:
    with np.errstate(over="ignore"):
        a = _mix(np.array([np.uint64(seed) * _GOLDEN + np.uint64(1)], dtype=np.uint64))[0]
        b = _mix(np.array([np.uint64(stream) * _STREAM_MUL + np.uint64(2)], dtype=np.uint64))[0]
    return a ^ b


def words(seed: int, stream: int, start: int, count: int) -> np.ndarray:
    """``count`` 64-bit words of stream (seed, stream), counters start..start+count-1."""
    key = _key(seed, stream)
    idx = np.arange(start + 1, start + count + 1, dtype=np.uint64)
    with np.errstate(over="ignore"):
        return _mix(key + idx * _GOLDEN)


def uniform01(seed: int, stream: int, count: int, start: int = 0) -> np.ndarray:
    """fp64 uniforms in the open interval (0, 1)."""
    out = np.empty(count, dtype=np.float64)
    for lo in range(0, count, _CHUNK):
        n = min(_CHUNK, count - lo)
        w = words(seed, stream, start + lo, n)
        out[lo:lo + n] = ((w >> np.uint64(11)).astype(np.float64) + 0.5) * 2.0 ** -53
    return out


def standard_normal(seed: int, stream: int, count: int) -> np.ndarray:
    """fp64 N(0,1) draws; draw i uses words 2i and 2i+1 of the stream."""
    out = np.empty(count, dtype=np.float64)
    for lo in range(0, count, _CHUNK):
        n = min(_CHUNK, count - lo)
        w = words(seed, stream, 2 * lo, 2 * n)
        u = ((w >> np.uint64(11)).astype(np.float64) + 0.5) * 2.0 ** -53
        u1, u2 = u[0::2], u[1::2]
        out[lo:lo + n] = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    return out


# --------------------------------------------------------------------------
# storage formats
# --------------------------------------------------------------------------

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even); returns uint16 bit patterns.

    Finite inputs only (the workloads never produce inf/nan)."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((b >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((b + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to fp32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def store(x64: np.ndarray, dtype: str) -> np.ndarray:
    """fp64 draws -> storage array of ``dtype`` ('f32' -> float32, 'bf16' -> uint16 bits)."""
    x32 = x64.astype(np.float32)
    if dtype == "f32":
        return x32
    if dtype == "bf16":
        return f32_to_bf16_bits(x32)
    raise ValueError(f"unknown dtype {dtype!r}")


def widen(a: np.ndarray, dtype: str) -> np.ndarray:
    """Storage array -> exact fp64 values."""
    if dtype == "f32":
        return np.asarray(a, dtype=np.float32).astype(np.float64)
    if dtype == "bf16":
        return bf16_bits_to_f32(a).astype(np.float64)
    raise ValueError(f"unknown dtype {dtype!r}")


# --------------------------------------------------------------------------
# workloads
# --------------------------------------------------------------------------

@dataclass
class FusedInputs:
    name: str
    dtype: str          # 'f32' | 'bf16'
    B: int
    H: int
    N: int
    d: int
    scale: np.float32   # the fp32 value handed to the library
    Q: np.ndarray       # [B, H, N, d] storage array
    K: np.ndarray       # [B, H, N, d]

    @property
    def elements(self) -> int:
        return self.B * self.H * self.N * self.N

    @property
    def itemsize(self) -> int:
        return 4 if self.dtype == "f32" else 2

    @property
    def algorithmic_bytes(self) -> int:
        """P written once + Q and K read once."""
        return self.itemsize * (self.elements + 2 * self.B * self.H * self.N * self.d)


@dataclass
class SoftmaxInputs:
    name: str
    dtype: str
    rows: int
    cols: int
    S: np.ndarray       # [rows, cols] storage array

    @property
    def elements(self) -> int:
        return self.rows * self.cols

    @property
    def itemsize(self) -> int:
        return 4 if self.dtype == "f32" else 2

    @property
    def algorithmic_bytes(self) -> int:
        """S read once + P written once."""
        return 2 * self.itemsize * self.elements


def fused_inputs(name: str, dtype: str, B: int, H: int, N: int, d: int, seed: int,
                 row_factor: Optional[tuple] = None, scale: Optional[float] = None) -> FusedInputs:
    """Q, K ~ N(0,1) i.i.d.; with ``row_factor=(lo, hi)`` every row of Q and of K
    is multiplied by its own factor drawn uniformly from [lo, hi]."""
    n = B * H * N * d
    q = standard_normal(seed, STREAM_Q, n).reshape(B, H, N, d)
    k = standard_normal(seed, STREAM_K, n).reshape(B, H, N, d)
    if row_factor is not None:
        lo, hi = row_factor
        fq = lo + (hi - lo) * uniform01(seed, STREAM_QROW, B * H * N).reshape(B, H, N, 1)
        fk = lo + (hi - lo) * uniform01(seed, STREAM_KROW, B * H * N).reshape(B, H, N, 1)
        q = q * fq
        k = k * fk
    if scale is None:
        scale = 1.0 / np.sqrt(np.float64(d))
    return FusedInputs(name, dtype, B, H, N, d, np.float32(scale), store(q, dtype), store(k, dtype))


def value_inputs(x: FusedInputs, seed: int) -> np.ndarray:
    """V ~ N(0,1) i.i.d., [B, H, N, d] in the storage type of ``x`` (stream of its own: Q and K of the
    same seed are unchanged)."""
    n = x.B * x.H * x.N * x.d
    return store(standard_normal(seed, STREAM_V, n).reshape(x.B, x.H, x.N, x.d), x.dtype)


def softmax_inputs(name: str, dtype: str, rows: int, cols: int, seed: int, sigma: float = 1.0,
                   peak_fraction: float = 0.0, peak_value: float = 8.0) -> SoftmaxInputs:
    """S ~ N(0, sigma^2) i.i.d.; independently a Bernoulli(peak_fraction) subset of
    the entries is overwritten with exactly ``peak_value``."""
    n = rows * cols
    s = standard_normal(seed, STREAM_S, n) * sigma
    if peak_fraction > 0.0:
        mask = uniform01(seed, STREAM_MASK, n) < peak_fraction
        s[mask] = peak_value
    return SoftmaxInputs(name, dtype, rows, cols, store(s.reshape(rows, cols), dtype))


# The five configurations (name -> constructor).  "c1" .. "c5" follow the order
# of the configuration list this build is measured on.

def c1() -> FusedInputs:
    """Single head, fp32, N = 128, d = 64, seed 0."""
    return fused_inputs("c1", "f32", 1, 1, 128, 64, seed=0)


def c2(rows: Optional[int] = None) -> SoftmaxInputs:
    """Row softmax, bf16, [12*2048, 2048], N(0, 2^2) with 1 % of entries = +8, seed 1.

    ``rows`` (optional) returns only the first ``rows`` rows' worth of draws of a
    matrix with that many rows - a smaller matrix of the same recipe, for tests."""
    r = 12 * 2048 if rows is None else rows
    return softmax_inputs("c2", "bf16", r, 2048, seed=1, sigma=2.0, peak_fraction=0.01, peak_value=8.0)


def c3() -> FusedInputs:
    """B = 4, H = 12, N = 1024, d = 64, bf16, seed 2."""
    return fused_inputs("c3", "bf16", 4, 12, 1024, 64, seed=2)


def c4() -> FusedInputs:
    """B = 1, H = 16, N = 4096, d = 128, bf16, seed 3 (the paper's d_k and largest fused n)."""
    return fused_inputs("c4", "bf16", 1, 16, 4096, 128, seed=3)


def c5() -> FusedInputs:
    """B = 1, H = 8, N = 16384, d = 64, bf16, rows scaled by U[0.5, 3], seed 4."""
    return fused_inputs("c5", "bf16", 1, 8, 16384, 64, seed=4, row_factor=(0.5, 3.0))


CONFIGS = {"c1": c1, "c2": c2, "c3": c3, "c4": c4, "c5": c5}
