"""GPU parity of attnw_fused / attnw_gemm_scores on many short sequences (bf16, N <= 128 with d a multiple of 16 up to
128, N <= 256 with d <= 64: the kernel in which a wave works alone on a (head, 32 queries) pair) against the fp64 oracle: every element of
sampled heads at the bf16 bar, every row sum, the guard bands around the output, the scores bit for bit against the
general kernel."""
import numpy as np
import pytest
import torch

import oracle
from paper_2407_13885_amd import workloads as wl

import gpu_util as gu

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    gu.require_gpu()


def _heads(BH):
    return sorted({0, 1 % BH, BH // 3, BH // 2, BH - 1})


def _check_fused(B, H, N, d, scale=None, row_factor=(0.5, 2.0), seed=0):
    x = wl.fused_inputs("t", "bf16", B, H, N, d, seed=5100 + N + d + seed, scale=scale, row_factor=row_factor)
    got = gu.to_f64(gu.run_fused(x, guard=8192)).reshape(B * H, N, N)
    Qf, Kf = x.Q.reshape(B * H, N, d), x.K.reshape(B * H, N, d)
    for bh in _heads(B * H):
        ref = oracle.attention_weights(Qf[bh], Kf[bh], "bf16", x.scale)
        gu.check_weights(got[bh], ref, "bf16", f"short sequences {B}x{H}x{N}x{d} head {bh}")
    assert np.isfinite(got).all()
    assert np.abs(got.sum(-1) - 1.0).max() <= gu.ROWSUM_BF16


def _check_scores(B, H, N, d, scale=None, seed=0):
    x = wl.fused_inputs("t", "bf16", B, H, N, d, seed=5300 + N + d + seed, scale=scale, row_factor=(0.5, 2.0))
    S = gu.run_scores(x, guard=8192)
    got = gu.to_f64(S).reshape(B * H, N, N)
    Qf, Kf = x.Q.reshape(B * H, N, d), x.K.reshape(B * H, N, d)
    assert np.isfinite(got).all()
    for bh in _heads(B * H):
        ref = oracle.scores(Qf[bh], Kf[bh], "bf16", x.scale)
        acc = d * 2.0 ** -24 * abs(float(x.scale)) * (np.abs(wl.widen(Qf[bh], "bf16")) @ np.abs(wl.widen(Kf[bh], "bf16")).T)
        assert (np.abs(got[bh] - ref) <= acc + 2.0 ** -8 * np.abs(ref) + 1e-30).all(), f"scores {B}x{H}x{N}x{d} head {bh}"
    return x, S


# every way a length meets the 32-key blocks, the 16-byte chunks and the staging writes: multiples of 8 (rows on
# 16-byte boundaries; of 16: padded staging rows), of 4 and not 8 (8-byte staging writes), even (4-byte), odd
# (2-byte); one to four blocks of keys and queries, last blocks of 1 and of 31; lengths of one block under the
# two-block kernel
@pytest.mark.parametrize("N", [1, 2, 3, 7, 8, 9, 16, 24, 31, 32, 33, 40, 48, 49, 52, 56, 63, 64,
                               65, 66, 72, 80, 95, 96, 97, 100, 104, 112, 120, 127, 128])
@pytest.mark.parametrize("d", [32, 64])
def test_any_length_up_to_128(N, d, monkeypatch):
    monkeypatch.setenv("ATTNW_FUSED_KERNEL", "tiny")
    _check_fused(1, 5, N, d)


@pytest.mark.parametrize("d", [16, 48, 80, 96, 112, 128])
@pytest.mark.parametrize("N", [49, 64, 100, 128])
def test_every_head_size(N, d, monkeypatch):
    monkeypatch.setenv("ATTNW_FUSED_KERNEL", "tiny")
    _check_fused(1, 6, N, d, seed=1)


# five to eight blocks of keys (the operands of the next unit are requested later in a unit): every way a length meets
# blocks, chunks and staging writes again; d = 64 up to 224 keys, d <= 48 up to 256
@pytest.mark.parametrize("N,d", [(129, 64), (136, 64), (144, 32), (150, 64), (159, 16), (160, 64), (161, 32), (176, 48), (191, 64),
                                 (192, 64), (193, 32), (197, 64), (200, 32), (223, 64), (224, 64), (225, 32), (250, 48), (255, 32),
                                 (256, 32), (256, 16)])
def test_lengths_up_to_256(N, d, monkeypatch):
    monkeypatch.setenv("ATTNW_FUSED_KERNEL", "tiny")
    _check_fused(1, 5, N, d, seed=3)
    if N in (144, 160, 197, 256):
        _check_fused(2, 300, N, d, seed=4)        # more units than resident waves


@pytest.mark.parametrize("N,d", [(129, 64), (145, 32), (160, 64), (197, 64), (256, 32)])
def test_scaled_scores_up_to_256(N, d, monkeypatch):
    monkeypatch.setenv("ATTNW_FUSED_KERNEL", "tiny")
    x, S = _check_scores(2, 40, N, d, seed=5)
    monkeypatch.setenv("ATTNW_FUSED_KERNEL", "twopass")
    S2 = gu.run_scores(x, guard=8192)
    assert torch.equal(S.view(torch.int16), S2.view(torch.int16))


@pytest.mark.parametrize("B,H,N,d", [(100, 7, 49, 32), (1000, 3, 49, 32), (4096, 3, 49, 32), (500, 4, 100, 64), (64, 16, 128, 64),
                                     (300, 3, 64, 32), (40, 16, 128, 128), (2000, 1, 33, 16), (90, 12, 77, 64), (30, 12, 160, 64), (64, 12, 144, 32)])
def test_many_heads_by_default(B, H, N, d):
    """The shapes that take this kernel without being asked: at least 512 (head, 32-query) units.  More units than
    resident waves: unit ranges that cross head boundaries (the K operands of the next head replace the ones in
    registers in the middle of a range)."""
    assert B * H * ((N + 31) // 32) >= 512
    _check_fused(B, H, N, d, seed=2)


@pytest.mark.parametrize("N,d", [(49, 32), (128, 64), (100, 128)])
@pytest.mark.parametrize("scale", [0.0, -0.125, 0.5])
def test_scale_values(N, d, scale, monkeypatch):
    monkeypatch.setenv("ATTNW_FUSED_KERNEL", "tiny")
    _check_fused(1, 3, N, d, scale=scale, row_factor=(0.5, 3.0), seed=7)


@pytest.mark.parametrize("B,H,N,d,scale", [(1, 3, 1, 64, None), (1, 5, 33, 32, None), (300, 4, 49, 32, None), (1, 3, 64, 64, -0.37),
                                           (70, 8, 100, 64, None), (1, 3, 127, 128, 1.0), (40, 16, 128, 64, None),
                                           (1, 4, 98, 16, 0.0), (2, 3, 52, 80, None)])
def test_scaled_scores(B, H, N, d, scale, monkeypatch):
    """attnw_gemm_scores through the same kernel without the statistics: against the oracle, and bit for bit against
    the general kernel (same order of accumulation, one rounding)."""
    monkeypatch.setenv("ATTNW_FUSED_KERNEL", "tiny")
    x, S = _check_scores(B, H, N, d, scale=scale)
    monkeypatch.setenv("ATTNW_FUSED_KERNEL", "twopass")
    S2 = gu.run_scores(x, guard=8192)
    assert torch.equal(S.view(torch.int16), S2.view(torch.int16))


def test_is_deterministic_and_heads_are_independent(monkeypatch):
    monkeypatch.setenv("ATTNW_FUSED_KERNEL", "tiny")
    x = wl.fused_inputs("t", "bf16", 1, 40, 49, 32, seed=5)
    a, b = gu.run_fused(x, guard=64), gu.run_fused(x, guard=64)
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    y = wl.fused_inputs("t", "bf16", 1, 40, 49, 32, seed=5)
    y.K[0, 17] = wl.fused_inputs("t", "bf16", 1, 1, 49, 32, seed=6).K[0, 0]
    cmp = gu.run_fused(y, guard=64)
    same = (a.view(torch.int16) == cmp.view(torch.int16)).reshape(40, -1).all(dim=1).cpu().numpy()
    assert same[:17].all() and same[18:].all() and not same[17]
