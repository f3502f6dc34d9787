"""GPU parity of attnw_fused on short sequences of any length (bf16, d = 64, N <= 608: the kernel that stages a strip
of 32 queries as the contiguous block of P that it is) against the fp64 oracle: every element of sampled heads at the
bf16 bar, every row sum, the guard bands around P."""
import os

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


def _check(B, H, N, scale=None, row_factor=(0.5, 2.0), seed=0, d=64):
    x = wl.fused_inputs("t", "bf16", B, H, N, d, seed=4100 + N + seed, scale=scale, row_factor=row_factor)
    got = gu.to_f64(gu.run_fused(x, guard=8192)).reshape(B * H, N, N)
    Qf, Kf = x.Q.reshape(B * H, N, d), x.K.reshape(B * H, N, d)
    for bh in sorted({0, 1 % (B * H), B * H // 2, B * H - 1}):
        ref = oracle.attention_weights(Qf[bh], Kf[bh], "bf16", x.scale)
        gu.check_weights(got[bh], ref, "bf16", f"short sequence {B}x{H}x{N} head {bh}")
    assert np.isfinite(got).all()
    assert np.abs(got.sum(-1) - 1.0).max() <= gu.ROWSUM_BF16


# odd lengths (2-byte staging writes), even (4-byte), multiples of 4 (8-byte); one to four pieces of keys per wave;
# lengths with waves that own no key (197: the eighth), with a last strip of one query (33, 65, 257, 577), of 31 (607)
@pytest.mark.parametrize("N", [1, 2, 3, 31, 33, 65, 100, 197, 198, 200, 255, 257, 258, 260, 333, 511, 513, 577, 578, 580,
                               601, 607])
def test_short_sequences_any_length(N):
    _check(1, 3, N)


@pytest.mark.parametrize("N", [129, 144, 197, 255, 257, 333, 510, 577, 607])
def test_short_sequences_of_32_element_heads(N):
    """d = 32: rows of 64 bytes, four K rows per 256-byte line of LDS."""
    _check(1, 3, N, d=32, seed=3)
    if N in (144, 197):
        _check(2, 150, N, d=32, seed=4)


@pytest.mark.parametrize("B,H,N", [(4, 70, 197), (2, 150, 257), (1, 300, 65), (3, 40, 577), (1, 9, 601)])
def test_short_sequences_many_heads(B, H, N):
    """More (head, strip) pairs than workgroups: strip lists that cross head boundaries (the K of the next head
    replaces the one in LDS in the middle of a list); few heads: several workgroups share a head."""
    _check(B, H, N)


@pytest.mark.parametrize("N", [197, 577])
@pytest.mark.parametrize("scale", [0.0, -0.125, 0.5])
def test_short_sequences_scale_values(N, scale):
    _check(1, 2, N, scale=scale, row_factor=(0.5, 3.0), seed=7)


@pytest.mark.parametrize("N", [33, 197, 333, 577])
def test_the_general_kernel_still_serves_these_lengths(N, monkeypatch):
    """ATTNW_FUSED_KERNEL=twopass keeps the same problems on the two-pass kernel (its ragged paths at d = 64 would
    otherwise only be reached by the score GEMM)."""
    monkeypatch.setenv("ATTNW_FUSED_KERNEL", "twopass")
    _check(1, 3, N, seed=11)


def _check_scores(x, S, what):
    d = x.Q.shape[-1]
    got = gu.to_f64(S)
    Qa, Ka = np.abs(wl.widen(x.Q, "bf16")), np.abs(wl.widen(x.K, "bf16"))
    B, H = x.Q.shape[:2]
    for b in range(B):
        for h in range(H):
            ref = oracle.scores(x.Q[b, h], x.K[b, h], "bf16", x.scale)
            acc_bound = d * 2.0 ** -24 * abs(float(x.scale)) * (Qa[b, h] @ Ka[b, h].T)
            assert (np.abs(got[b, h] - ref) <= acc_bound + 2.0 ** -8 * np.abs(ref) + 1e-30).all(), f"{what} head {b},{h}"


@pytest.mark.parametrize("B,H,N,scale", [(1, 3, 1, None), (1, 3, 33, None), (2, 70, 197, None), (1, 3, 198, -0.37),
                                         (1, 2, 200, 1.0), (1, 150, 257, None), (1, 3, 333, 0.0), (2, 20, 577, None),
                                         (1, 3, 578, None), (1, 3, 607, -1.0)])
def test_scaled_scores_of_short_sequences(B, H, N, scale, monkeypatch, d=64):
    """attnw_gemm_scores on the same lengths: the same kernel without the statistics.  Against the oracle, the
    guard bands around S, and bit for bit against the general kernel (same order of accumulation, one rounding)."""
    x = wl.fused_inputs("t", "bf16", B, H, N, d, seed=4300 + N, scale=scale, row_factor=(0.5, 2.0))
    S = gu.run_scores(x, guard=8192)
    _check_scores(x, S, f"scores of short sequences {B}x{H}x{N}")
    monkeypatch.setenv("ATTNW_FUSED_KERNEL", "twopass")
    S2 = gu.run_scores(x, guard=8192)
    assert torch.equal(S.view(torch.int16), S2.view(torch.int16))


@pytest.mark.parametrize("N", [145, 333, 577])
def test_scaled_scores_of_32_element_heads(N, monkeypatch):
    test_scaled_scores_of_short_sequences(1, 3, N, None, monkeypatch, d=32)
