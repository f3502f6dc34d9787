"""GPU parity of attnw_attention on many short sequences (bf16, d = 64 with N <= 128, d = 32 with N <= 224: the kernel in
which a wave works alone on a (head, 32 queries) pair) against the fp64 oracle, at the bar of test_gpu_attention.py:
the weights are rounded to bf16 before they multiply V and the output once more, so with A_it = sum_j P_ij |V_jt|
the bound is 2^-8 (A_it + |O_it|) (two roundings of 2^-9 each) plus the fp32 accumulation."""
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
    attnw.attnw_attention(Q, K, Vd, O, x.B, x.H, x.N, x.d, float(x.scale), gu.DT["bf16"])
    torch.cuda.synchronize()
    assert gu.guards_intact(canary), "attention kernel wrote outside O"
    return O


def _check_head(got, x, V, bh, what):
    B, H, N, d = x.B, x.H, x.N, x.d
    b, h = divmod(bh, H)
    ref, P = oracle.attention_output(x.Q[b, h], x.K[b, h], V[b, h], "bf16", x.scale, rows=(0, N), return_weights=True)
    A = P @ np.abs(wl.widen(V[b, h], "bf16"))
    tol = 2.0 ** -8 * (A + np.abs(ref)) * 1.02 + 1e-6 * A
    err = np.abs(got[b, h] - ref)
    assert np.isfinite(got[b, h]).all(), f"{what}: non-finite output"
    if (err > tol).any():
        i = np.unravel_index(np.argmax(err / tol), err.shape)
        raise AssertionError(f"{what} head {bh}: {int((err > tol).sum())} elements beyond the bound; worst at {i}: "
                             f"got {got[b, h][i]:.6e} ref {ref[i]:.6e} err {err[i]:.3e} tol {tol[i]:.3e}")


def _check(B, H, N, d, scale=None, seed=0, row_factor=(0.5, 2.0)):
    x = wl.fused_inputs("t", "bf16", B, H, N, d, seed=6100 + N + d + seed, scale=scale, row_factor=row_factor)
    V = wl.value_inputs(x, seed=6101 + N + seed)
    O = gu.to_f64(_run(x, V))
    assert np.isfinite(O).all()
    BH = B * H
    for bh in sorted({0, 1 % BH, BH // 3, BH // 2, BH - 1}):
        _check_head(O, x, V, bh, f"attention of short sequences {B}x{H}x{N}x{d}")
    return x, V, O


# one to four blocks of keys and queries, last blocks of 1 and of 31 keys, lengths below a block
@pytest.mark.parametrize("N,d", [(1, 32), (2, 64), (7, 32), (31, 64), (32, 32), (33, 64), (49, 32), (49, 64), (63, 32), (64, 64),
                                 (64, 32), (65, 32), (96, 32), (97, 32), (100, 32), (127, 32), (128, 32),
                                 (65, 64), (96, 64), (97, 64), (100, 64), (127, 64), (128, 64),
                                 (129, 32), (144, 32), (160, 32), (161, 32), (192, 32), (197, 32), (223, 32), (224, 32)])
def test_any_length(N, d, monkeypatch):
    monkeypatch.setenv("ATTNW_ATTENTION_KERNEL", "tiny")
    _check(1, 5, N, d)


@pytest.mark.parametrize("B,H,N,d", [(100, 7, 49, 32), (4096, 3, 49, 32), (300, 4, 64, 64), (500, 3, 100, 32), (90, 12, 33, 64),
                                     (2000, 1, 20, 32), (64, 12, 128, 64), (100, 8, 100, 64), (256, 12, 144, 32), (64, 16, 160, 32)])
def test_many_heads_by_default(B, H, N, d):
    """The shapes that take this kernel without being asked; more (head, 32 queries) units than resident waves: unit
    ranges that cross head boundaries."""
    assert B * H * ((N + 31) // 32) >= 256
    _check(B, H, N, d, seed=2)


@pytest.mark.parametrize("N,d", [(49, 32), (64, 64), (100, 32)])
def test_scale_values_and_constant_values(N, d, monkeypatch):
    monkeypatch.setenv("ATTNW_ATTENTION_KERNEL", "tiny")
    x, V, _ = _check(1, 3, N, d, scale=-1.0 / np.sqrt(d), seed=7, row_factor=(0.5, 3.0))
    Vw = wl.widen(V[0, 0], "bf16")
    # scale 0: uniform weights, every output row is the column mean of V
    x0 = wl.fused_inputs("t", "bf16", 1, 3, N, d, seed=6100 + N + d + 7, scale=0.0)
    O0 = gu.to_f64(_run(x0, V))
    assert np.abs(O0[0, 0] - Vw.mean(axis=0)).max() <= 2.0 ** -8 * np.abs(Vw).mean(axis=0).max() + 1e-7
    # constant V rows: every output row equals that row (weights sum to 1, up to their rounding)
    Vc = np.broadcast_to(V[:, :, :1, :], V.shape).copy()
    Oc = gu.to_f64(_run(x, Vc))
    v = wl.widen(Vc[0, 1, 0], "bf16")
    assert np.abs(Oc[0, 1] - v).max() <= 2 * 2.0 ** -8 * np.abs(v).max()


def test_agrees_with_the_tiled_kernel_and_is_deterministic(monkeypatch):
    x = wl.fused_inputs("t", "bf16", 2, 40, 49, 32, seed=5)
    V = wl.value_inputs(x, seed=6)
    monkeypatch.setenv("ATTNW_ATTENTION_KERNEL", "tiny")
    a, b = _run(x, V, guard=64), _run(x, V, guard=64)
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    monkeypatch.setenv("ATTNW_ATTENTION_KERNEL", "tiled")
    t = gu.to_f64(_run(x, V, guard=64))
    # two roundings each, of values that agree to fp32 rounding of the sums
    assert np.abs(gu.to_f64(a) - t).max() <= 2.0 ** -7 * np.abs(t).max()
