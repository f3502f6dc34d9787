"""GPU parity of attnw_attention on the element types and head sizes that the tiled bf16 kernel does not
take -- fp32 (d a multiple of 4 up to 256) and bf16 with 128 < d <= 256 -- against the fp64 oracle.

bf16: the bar of test_gpu_attention.py (weights rounded to bf16 before they multiply V, the output once more).

fp32: both contractions run on the fp32 matrix instruction and nothing is rounded but in fp32.  With
B_i = |scale| max_j sum_t |q_it| |k_jt| (what the rounding errors of one score are relative to),
A_it = sum_j P_ij |V_jt| and u = 2^-24:
  * a score is a sum of d fp32 products: |scale| |s^ - s| <= d u B_i, which moves every weight by that
    relative amount (numerator), and the normaliser by at most as much;
  * the exponent argument c s - ref is formed with one rounding and c itself is rounded (2 u |c s|, counted
    with the first item since |c s| <= 1.45 B_i), the exponential is good to a few u, the running sum and
    the rescalings by powers of two add N u at worst;
  * the output is a sum of N fp32 products: N u A_it at worst.
Bar: |O - O_ref| <= ((2 d + 4) u B_i + 2^-20 + 2 N u) (A_it + |O_ref|).  (At d = 64, N = 600 and rows
of spread 2 that is about 2e-4 relative -- twenty times tighter than one bf16 rounding.)"""
import math

import numpy as np
import pytest
import torch

import oracle
import paper_2407_13885_amd as attnw
from paper_2407_13885_amd import workloads as wl

import gpu_util as gu

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    gu.require_gpu()


def _run(x, V, guard=4096):
    Q, K, Vd = gu.to_dev(x.Q, x.dtype), gu.to_dev(x.K, x.dtype), gu.to_dev(V, x.dtype)
    O, canary = gu.empty_like_out((x.B, x.H, x.N, x.d), x.dtype, guard)
    attnw.attnw_attention(Q, K, Vd, O, x.B, x.H, x.N, x.d, float(x.scale), gu.DT[x.dtype])
    torch.cuda.synchronize()
    assert gu.guards_intact(canary), "attention kernel wrote outside O"
    return O


def _check(got, x, V, b, h, rows, what):
    r0, r1 = rows
    ref, P = oracle.attention_output(x.Q[b, h], x.K[b, h], V[b, h], x.dtype, x.scale, rows=rows, return_weights=True)
    A = P @ np.abs(wl.widen(V[b, h], x.dtype))
    if x.dtype == "bf16":
        tol = 2.0 ** -8 * (A + np.abs(ref)) * 1.02 + 1e-6 * A
    else:
        u = 2.0 ** -24
        Bi = abs(float(np.float32(x.scale))) * (np.abs(wl.widen(x.Q[b, h, r0:r1], "f32")) @ np.abs(wl.widen(x.K[b, h], "f32")).T).max(axis=1)
        tol = ((2 * x.d + 4) * u * Bi[:, None] + 2.0 ** -20 + 2 * x.N * u) * (A + np.abs(ref))
    err = np.abs(got[r0:r1] - ref)
    assert np.isfinite(got[r0:r1]).all(), f"{what}: non-finite output"
    if (err > tol).any():
        i = np.unravel_index(np.argmax(err / tol), err.shape)
        raise AssertionError(f"{what} rows {r0}..{r1}: {int((err > tol).sum())} elements beyond the bound; worst at {i}: "
                             f"got {got[r0:r1][i]:.8e} ref {ref[i]:.8e} err {err[i]:.3e} tol {tol[i]:.3e}")


@pytest.mark.parametrize("d", [4, 8, 12, 20, 32, 36, 64, 100, 128, 132, 200, 256])
@pytest.mark.parametrize("N", [1, 31, 32, 33, 100, 257, 600])
def test_attention_f32(N, d):
    x = wl.fused_inputs("t", "f32", 1, 2, N, d, seed=3100 + N + d, row_factor=(0.5, 2.0))
    V = wl.value_inputs(x, seed=3101 + N)
    O = gu.to_f64(_run(x, V))
    for h in range(2):
        _check(O[0, h], x, V, 0, h, (0, N), f"fp32 attention N={N} d={d} head {h}")


@pytest.mark.parametrize("d", [144, 160, 192, 208, 256])
@pytest.mark.parametrize("N", [1, 33, 128, 257, 600])
def test_attention_bf16_large_heads(N, d):
    x = wl.fused_inputs("t", "bf16", 1, 2, N, d, seed=3300 + N + d, row_factor=(0.5, 2.0))
    V = wl.value_inputs(x, seed=3301 + N)
    O = gu.to_f64(_run(x, V))
    for h in range(2):
        _check(O[0, h], x, V, 0, h, (0, N), f"bf16 attention N={N} d={d} head {h}")


@pytest.mark.parametrize("dtype,B,H,N,d", [("f32", 2, 3, 2048, 64), ("f32", 1, 2, 1500, 128), ("f32", 1, 1, 1024, 256),
                                           ("bf16", 2, 2, 2048, 256), ("bf16", 1, 3, 1500, 160)])
def test_attention_general_long(dtype, B, H, N, d):
    """Many sub-tiles per wave, several heads and batches (addressing of the heads), sampled row ranges."""
    x = wl.fused_inputs("t", dtype, B, H, N, d, seed=3500 + H + N + d, row_factor=(0.5, 2.0))
    V = wl.value_inputs(x, seed=3501 + N)
    O = gu.to_f64(_run(x, V))
    assert np.isfinite(O).all()
    for b in range(B):
        for h in range(H):
            for rows in [(0, 40), (N // 2 - 3, N // 2 + 30), (N - 40, N)]:
                _check(O[b, h], x, V, b, h, rows, f"{dtype} attention {B}x{H}x{N}x{d} head ({b},{h})")


@pytest.mark.parametrize("dtype,d", [("f32", 64), ("f32", 20), ("bf16", 192)])
def test_attention_general_negative_and_zero_scale_constant_values(dtype, d):
    N = 333
    x = wl.fused_inputs("t", dtype, 1, 2, N, d, seed=3700 + d, scale=-1.0 / math.sqrt(d), row_factor=(0.5, 3.0))
    V = wl.value_inputs(x, seed=3701 + d)
    O = gu.to_f64(_run(x, V))
    for h in range(2):
        _check(O[0, h], x, V, 0, h, (0, N), f"{dtype} negative scale d={d} head {h}")
    Vw = wl.widen(V[0, 0], dtype)
    one = 2.0 ** -8 if dtype == "bf16" else 2.0 ** -20
    # scale 0: uniform weights, every output row is the column mean of V
    x0 = wl.fused_inputs("t", dtype, 1, 2, N, d, seed=3700 + d, scale=0.0)
    O0 = gu.to_f64(_run(x0, V))
    assert np.abs(O0[0, 0] - Vw.mean(axis=0)).max() <= one * np.abs(Vw).mean(axis=0).max() + 1e-7
    # constant V rows: every output row equals that row (weights sum to 1, up to their rounding)
    Vc = np.broadcast_to(V[:, :, :1, :], V.shape).copy()
    Oc = gu.to_f64(_run(x, Vc))
    v = wl.widen(Vc[0, 1, 0], dtype)
    assert np.abs(Oc[0, 1] - v).max() <= 2 * one * np.abs(v).max()


def test_attention_f32_scores_climbing_along_the_keys():
    """Every sub-tile brings a new row maximum: the reference exponent moves and the accumulators are rescaled."""
    N, d = 1024, 32
    x = wl.fused_inputs("t", "f32", 1, 2, N, d, seed=97)
    a = 4.0
    for step in (0.02, 0.4):
        Kw = wl.widen(x.K, "f32") * 0.05
        Kw[..., 0] = (np.arange(N, dtype=np.float64) * step / (a * float(x.scale)))[None, None, :]
        Qw = wl.widen(x.Q, "f32") * 0.05
        Qw[..., 0] = a
        Qw[0, 1, ::2, 0] = -a
        x.Q[...] = wl.store(Qw, "f32")
        x.K[...] = wl.store(Kw, "f32")
        V = wl.value_inputs(x, seed=98)
        O = gu.to_f64(_run(x, V))
        for h in range(2):
            _check(O[0, h], x, V, 0, h, (0, N), f"fp32 climbing scores step={step} head {h}")


def test_attention_general_is_deterministic():
    x = wl.fused_inputs("t", "f32", 1, 2, 300, 36, seed=6)
    V = wl.value_inputs(x, seed=7)
    a, b = _run(x, V, guard=64), _run(x, V, guard=64)
    assert torch.equal(a.view(torch.int32), b.view(torch.int32))
