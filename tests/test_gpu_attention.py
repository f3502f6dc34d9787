"""GPU parity of attnw_attention (O = softmax(scale Q K^T) V with the weights kept on chip) against the
fp64 oracle.

Tolerance, from the arithmetic of the kernel: the weights are rounded to bf16 (8-bit significand:
relative 2^-8 each at worst) before they multiply V, everything else up to the store is fp32, and
the result is rounded to bf16 once more (2^-8 |O|).  Hence
|O - O_ref| <= 2^-8 (sum_j P_ij |V_jt| + |O_ref|)  up to fp32 effects, for which 2 % of that bound
plus 1e-6 of the first sum is allowed on top.  (Rows with one dominant key come close to the bound;
flat rows stay far below it because the rounding errors of many weights average out.)"""
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
    Q, K, Vd = gu.to_dev(x.Q, "bf16"), gu.to_dev(x.K, "bf16"), gu.to_dev(V, "bf16")
    O, canary = gu.empty_like_out((x.B, x.H, x.N, x.d), "bf16", guard)
    attnw.attnw_attention(Q, K, Vd, O, x.B, x.H, x.N, x.d, float(x.scale), attnw.ATTNW_BF16)
    torch.cuda.synchronize()
    assert gu.guards_intact(canary), "attention kernel wrote outside O"
    return O


def _check_rows(got, x, V, b, h, rows, what):
    """rows: (r0, r1) range or list of single rows and / or ranges."""
    Vw = np.abs(wl.widen(V[b, h], "bf16"))
    spans = [rows] if isinstance(rows, tuple) else [r if isinstance(r, tuple) else (r, r + 1) for r in rows]
    for r0, r1 in spans:
        ref, P = oracle.attention_output(x.Q[b, h], x.K[b, h], V[b, h], "bf16", x.scale, rows=(r0, r1), return_weights=True)
        A = P @ Vw
        tol = 2.0 ** -8 * (A + np.abs(ref)) * 1.02 + 1e-6 * A
        err = np.abs(got[r0:r1] - ref)
        assert np.isfinite(got[r0:r1]).all(), f"{what}: non-finite output"
        if (err > tol).any():
            i = np.unravel_index(np.argmax(err / tol), err.shape)
            raise AssertionError(f"{what} rows {r0}..{r1}: {int((err > tol).sum())} elements beyond the bound; worst at {i}: "
                                 f"got {got[r0:r1][i]:.6e} ref {ref[i]:.6e} err {err[i]:.3e} tol {tol[i]:.3e}")


@pytest.mark.parametrize("B,H,N,d", [(1, 2, 256, 64), (1, 3, 512, 64), (2, 2, 512, 128), (1, 1, 1024, 128),
                                     (1, 100, 1024, 64), (1, 3, 512, 32), (1, 100, 2048, 32)])
def test_attention_bf16_small(B, H, N, d):
    x = wl.fused_inputs("t", "bf16", B, H, N, d, seed=800 + H + N + d)
    V = wl.value_inputs(x, seed=801 + N)
    O = gu.to_f64(_run(x, V))
    for b in range(B):
        for h in range(H if H <= 4 else 3):          # every head of the small cases, three of the many-head case
            hh = h if H <= 4 else (0, H // 2, H - 1)[h]
            _check_rows(O[b, hh], x, V, b, hh, (0, N), f"attention {B}x{H}x{N}x{d} head ({b},{hh})")


@pytest.mark.parametrize("d", [32, 64, 128])
@pytest.mark.parametrize("N", [1, 2, 3, 31, 33, 100, 127, 128, 129, 255, 257, 320, 600, 1000])
def test_attention_any_length(N, d):
    """Lengths that are not whole tiles or strips: rows past the end are clamped on the way in, their
    weights forced to zero, their queries not stored (the guard band around O stays untouched)."""
    x = wl.fused_inputs("t", "bf16", 1, 2, N, d, seed=1500 + N + d, row_factor=(0.5, 2.0))
    V = wl.value_inputs(x, seed=1501 + N)
    O = gu.to_f64(_run(x, V))
    for h in range(2):
        _check_rows(O[0, h], x, V, 0, h, (0, N), f"attention N={N} d={d} head {h}")


@pytest.mark.parametrize("d", [16, 48, 80, 96, 112])
@pytest.mark.parametrize("N", [1, 33, 128, 257, 512, 1000, 1024])
def test_attention_head_sizes_between_the_powers_of_two(N, d):
    """Rows of Q, K, V and O that are not 64, 128 or 256 bytes long are padded on chip: zero Q fragments and V
    columns past the end, output columns past the end not stored (the guard band around O stays untouched)."""
    x = wl.fused_inputs("t", "bf16", 2, 2, N, d, seed=1900 + N + d, row_factor=(0.5, 2.0))
    V = wl.value_inputs(x, seed=1901 + N)
    O = gu.to_f64(_run(x, V))
    for b in range(2):
        for h in range(2):
            _check_rows(O[b, h], x, V, b, h, (0, N), f"attention N={N} d={d} head ({b},{h})")


@pytest.mark.parametrize("d", [32, 48, 64, 80, 112, 128])
@pytest.mark.parametrize("N", [1, 33, 129, 257, 600])
def test_attention_many_heads_take_the_wide_strips(N, d):
    """Few heads run on 64-query strips whose keys are spread over four waves (the tests above); with more than two
    such strips per compute unit the library takes 256-query strips, every wave walking all keys.  Enough heads for
    that, first, middle and last head checked."""
    H = 512 // ((N + 63) // 64) + 1
    x = wl.fused_inputs("t", "bf16", 1, H, N, d, seed=2300 + N + d, row_factor=(0.5, 2.0))
    V = wl.value_inputs(x, seed=2301 + N)
    O = gu.to_f64(_run(x, V))
    assert np.isfinite(O).all()
    for h in (0, H // 2, H - 1):
        _check_rows(O[0, h], x, V, 0, h, (0, N), f"attention wide strips N={N} d={d} head {h} of {H}")


@pytest.mark.parametrize("B,H,N,d", [(1, 1, 4096, 128), (1, 4, 4096, 128), (2, 4, 4096, 64), (1, 1, 16384, 128), (1, 2, 16384, 32)])
def test_attention_few_heads_of_many_keys(B, H, N, d):
    """The sizes the paper measures are single heads: the four partial results of a query block (one per key range,
    each with its own reference exponent and sum) are merged at the end.  Sampled rows of every head."""
    x = wl.fused_inputs("t", "bf16", B, H, N, d, seed=2500 + H + N + d, row_factor=(0.5, 2.0))
    V = wl.value_inputs(x, seed=2501 + N)
    O = gu.to_f64(_run(x, V))
    assert np.isfinite(O).all()
    for b in range(B):
        for h in range(H):
            _check_rows(O[b, h], x, V, b, h, [(0, 40), (N // 2 - 3, N // 2 + 30), (N - 65, N)],
                        f"attention {B}x{H}x{N}x{d} head ({b},{h})")


@pytest.mark.parametrize("B,H,N,d", [(1, 40, 2100, 64), (1, 3, 2100, 64), (1, 3, 2300, 128), (1, 40, 2100, 32)])
def test_attention_any_length_long(B, H, N, d):
    """Ragged lengths of many tiles: only the last tile is compiled with key masks and clamped loads.  40 heads
    of 2100 queries take the instantiation with two query blocks per wave (512-query strips)."""
    x = wl.fused_inputs("t", "bf16", B, H, N, d, seed=1900 + H + N + d, row_factor=(0.5, 2.0))
    V = wl.value_inputs(x, seed=1901 + N)
    O = gu.to_f64(_run(x, V))
    assert np.isfinite(O).all()
    for hh in sorted({0, H // 2, H - 1}):
        _check_rows(O[0, hh], x, V, 0, hh, [(0, 70), (500, 530), (2040, N)], f"attention {B}x{H}x{N}x{d} head {hh}")


# A last strip of at most 64 queries that would start another round of workgroups is left out of the launch and
# follows as a second one with its keys spread over four waves: 256-query strips at d = 32 / 64 / 128, 512-query strips
# (two query blocks per wave); a tail of 1, 33 and 64 rows; next to it a length whose tail is too long for the rule.
@pytest.mark.parametrize("B,H,N,d", [(1, 64, 1025, 64), (1, 128, 545, 32), (1, 32, 2081, 128), (1, 64, 2049, 64),
                                     (1, 128, 2112, 32), (1, 64, 1100, 64)])
def test_attention_last_strip_as_a_launch_of_its_own(B, H, N, d):
    x = wl.fused_inputs("t", "bf16", B, H, N, d, seed=2000 + H + N + d, row_factor=(0.5, 2.0))
    V = wl.value_inputs(x, seed=2001 + N)
    O = gu.to_f64(_run(x, V))
    assert np.isfinite(O).all()
    first_tail = N // 256 * 256 if N % 256 <= 64 else N - 8
    for hh in sorted({0, H // 2, H - 1}):
        _check_rows(O[0, hh], x, V, 0, hh, [(0, 40), (first_tail - 20, N)], f"attention {B}x{H}x{N}x{d} head {hh}")


def test_attention_any_length_scale_zero_is_the_column_mean():
    x = wl.fused_inputs("t", "bf16", 1, 1, 333, 64, seed=21, scale=0.0)
    V = wl.value_inputs(x, seed=22)
    O = gu.to_f64(_run(x, V))
    mean = wl.widen(V[0, 0], "bf16").mean(axis=0)
    assert np.abs(O[0, 0] - mean).max() <= 2.0 ** -8 * np.abs(wl.widen(V[0, 0], "bf16")).mean(axis=0).max()


@pytest.mark.parametrize("d", [64, 128])
def test_attention_negative_scale_sharp_rows_and_special_values(d):
    x = wl.fused_inputs("t", "bf16", 1, 2, 768, d, seed=41 + d, scale=-1.0 / math.sqrt(d), row_factor=(0.5, 3.0))
    V = wl.value_inputs(x, seed=42 + d)
    O = gu.to_f64(_run(x, V))
    for h in range(2):
        _check_rows(O[0, h], x, V, 0, h, (0, 768), f"negative scale d={d} head {h}")
    # Q = 0: uniform weights, the output is the column mean of V for every query
    x.Q[...] = 0
    O0 = gu.to_f64(_run(x, V))
    mean = wl.widen(V[0, 0], "bf16").mean(axis=0)
    assert np.abs(O0[0, 0] - mean).max() <= 2.0 ** -8 * np.abs(wl.widen(V[0, 0], "bf16")).mean(axis=0).max()
    # constant V rows: every output row equals that row exactly (weights sum to 1, up to their rounding)
    Vc = np.broadcast_to(V[:, :, :1, :], V.shape).copy()
    Oc = gu.to_f64(_run(x, Vc))
    v = wl.widen(Vc[0, 1, 0], "bf16")
    assert np.abs(Oc[0, 1] - v).max() <= 2.0 ** -7 * np.abs(v).max()


@pytest.mark.parametrize("name", ["c4", "c5"])
def test_attention_full_size_sampled_rows(name):
    x = wl.CONFIGS[name]()
    V = wl.value_inputs(x, seed=77)
    O = gu.to_f64(_run(x, V))
    assert np.isfinite(O).all()
    rng = np.random.default_rng(9)
    for h in range(x.H):
        rows = sorted({0, 31, 32, 255, 256, x.N // 2, x.N - 257, x.N - 1} | set(rng.integers(0, x.N, size=8).tolist()))
        _check_rows(O[0, h], x, V, 0, h, rows, f"{name} attention head {h}")


@pytest.mark.parametrize("H", [2, 40])          # key ranges over waves / wide strips
@pytest.mark.parametrize("d,step", [(64, 0.02), (128, 0.02), (64, 0.4), (128, 0.25)])
def test_attention_scores_climbing_along_the_keys(d, step, H):
    """Scores that grow with the key index: every sub-tile brings a new row maximum.  Small steps stay
    inside the window in which the kernel keeps its reference exponent (weights above 1 appear), large
    steps (8 and more nats per 32 keys) force the reference to move at every sub-tile; the last keys
    carry all the weight.  Scores stay within a few hundred: the fp32 score arithmetic resolves
    differences of scores only to 2^-24 of their magnitude."""
    N = 1024
    x = wl.fused_inputs("t", "bf16", 1, H, N, d, seed=90 + d)
    # q = e_0 * a (plus noise in the other coordinates), k_j[0] = j * step / (a * scale): score ~ j * step
    a = 4.0
    ramp = (np.arange(N, dtype=np.float64) * step / (a * float(x.scale)))
    Kw = wl.widen(x.K, "bf16") * 0.05
    Kw[..., 0] = ramp[None, None, :]
    Qw = wl.widen(x.Q, "bf16") * 0.05
    Qw[..., 0] = a
    Qw[0, 1, ::2, 0] = -a            # every other query of head 1 sees the scores fall instead
    x.Q[...] = wl.store(Qw, "bf16")
    x.K[...] = wl.store(Kw, "bf16")
    V = wl.value_inputs(x, seed=91 + d)
    O = gu.to_f64(_run(x, V))
    for h in range(2):
        _check_rows(O[0, h], x, V, 0, h, (0, N), f"climbing scores d={d} step={step} head {h}")


def test_attention_is_deterministic():
    x = wl.fused_inputs("t", "bf16", 1, 2, 512, 64, seed=6)
    V = wl.value_inputs(x, seed=7)
    a, b = _run(x, V, guard=0 + 64), _run(x, V, guard=0 + 64)
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))
