"""Randomised differential test of attnw_fused, attnw_gemm_scores and attnw_attention against the oracle: shapes
drawn from a seeded generator over everything the dispatch distinguishes (short and long sequences, lengths on and off
the tilings, one head to thousands, every head size, fp32), rows sampled for the element-by-element comparison and
EVERY row sum checked.  A run of this kind found the exchange race of the kernel that keeps the scores resident
across compute units (whole strips with wrong sums, in some calls only): every case therefore runs twice."""
import math

import numpy as np
import pytest
import torch

import oracle
import paper_2407_13885_amd as attnw
from paper_2407_13885_amd import workloads as wl

import gpu_util as gu

pytestmark = pytest.mark.gpu

CASES_PER_SEED = 10
MAX_ELEMENTS = 1.5e8          # of P per case: bounds the host side of the check


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    gu.require_gpu()


def _draw(rng, kind):
    if kind == "aligned":     # few heads, lengths on the tilings: the kernels that spread a strip's keys over workgroups
        dtype, d = "bf16", int(rng.choice([64, 128]))
        N = int(256 * rng.integers(2, 33))
        BH = int(rng.choice([1, 2, 3, 4, 5, 6, 7, 8, 12, 16, 24]))
    else:
        dtype = "bf16" if (kind == "attention" or rng.random() < 0.75) else "f32"
        d = int(rng.choice([32, 32, 64, 64, 128, 128, 48, 80, 16, 192, 256])) if kind == "attention" else \
            int(rng.choice([16, 32, 64, 64, 96, 128, 128, 256]))
        N = int(rng.choice([rng.integers(1, 300), rng.integers(300, 1100), 256 * rng.integers(1, 17), 128 * rng.integers(1, 33),
                            rng.integers(1100, 4200), 2 * rng.integers(500, 2100), 4 * rng.integers(250, 1050)]))
        BH = int(rng.choice([1, 1, 2, 3, 8, 33])) if N > 600 else int(rng.choice([1, 2, 9, 70, 300, 2000]))
    if BH * N * N > MAX_ELEMENTS:
        BH = max(1, int(MAX_ELEMENTS // (N * N)))
    scale = float(rng.choice([1 / math.sqrt(d), -1 / math.sqrt(d), 0.05]))
    return dtype, BH, N, d, scale


def _check_fused(x, dtype, BH, N, d, scale, rows, heads, tag):
    tol = gu.ROWSUM_BF16 if dtype == "bf16" else gu.ROWSUM_F32
    for call in range(2):
        P = gu.to_f64(gu.run_fused(x, guard=4096))
        dev = np.abs(P.sum(-1) - 1)
        assert dev.max() <= tol, f"{tag} call {call}: row sums off by {dev.max():.3e} at {np.argwhere(dev > tol)[:4].tolist()}"
        for h in heads:
            ref = np.concatenate([oracle.attention_weights(x.Q[0, h], x.K[0, h], dtype, x.scale, rows=(r, r + 1)) for r in rows])
            gu.check_weights(P[0, h][rows], ref, dtype, f"{tag} call {call} head {h}",
                             abs_f32=gu.ABS_F32 * max(1.0, abs(scale) * math.sqrt(d)))
    S = gu.to_f64(gu.run_scores(x, guard=4096))
    for h in heads:
        ref = np.concatenate([oracle.scores(x.Q[0, h], x.K[0, h], dtype, x.scale, rows=(r, r + 1)) for r in rows])
        qa, ka = np.abs(wl.widen(x.Q[0, h], dtype))[rows], np.abs(wl.widen(x.K[0, h], dtype))
        bound = d * 2.0 ** -24 * abs(scale) * (qa @ ka.T) + (2.0 ** -8 if dtype == "bf16" else 2.0 ** -24) * np.abs(ref) + 1e-30
        assert (np.abs(S[0, h][rows] - ref) <= bound).all(), f"{tag}: scores of head {h}"


def _check_attention(x, BH, N, d, rng, rows, heads, tag):
    V = wl.value_inputs(x, seed=int(rng.integers(1 << 30)))
    Q, K, Vd = gu.to_dev(x.Q, "bf16"), gu.to_dev(x.K, "bf16"), gu.to_dev(V, "bf16")
    O, canary = gu.empty_like_out((1, BH, N, d), "bf16", 4096)
    attnw.attnw_attention(Q, K, Vd, O, 1, BH, N, d, float(x.scale), attnw.ATTNW_BF16)
    torch.cuda.synchronize()
    assert gu.guards_intact(canary), f"{tag}: wrote outside O"
    Of = gu.to_f64(O)
    for h in heads:
        Vw = np.abs(wl.widen(V[0, h], "bf16"))
        for r in rows:
            ref, Pr = oracle.attention_output(x.Q[0, h], x.K[0, h], V[0, h], "bf16", x.scale, rows=(r, r + 1), return_weights=True)
            A = Pr @ Vw
            tol = 2.0 ** -8 * (A + np.abs(ref)) * 1.02 + 1e-6 * A
            assert (np.abs(Of[0, h][r:r + 1] - ref) <= tol).all(), f"{tag}: head {h} row {r}"


@pytest.mark.parametrize("seed", range(8))
def test_random_shapes_against_the_oracle(seed):
    rng = np.random.default_rng(5000 + seed)
    for n in range(CASES_PER_SEED):
        kind = str(rng.choice(["fused", "fused", "attention", "aligned", "aligned"]))
        dtype, BH, N, d, scale = _draw(rng, kind)
        x = wl.fused_inputs("t", dtype, 1, BH, N, d, seed=int(rng.integers(1 << 30)), scale=scale,
                            row_factor=(0.5, 2.5) if dtype == "bf16" else None)
        rows = sorted(set(rng.integers(0, N, size=min(N, 8)).tolist()) | {0, N - 1})
        heads = sorted({0, BH // 2, BH - 1})
        tag = f"[seed {seed} case {n}] {kind} {dtype} BH{BH} N{N} d{d} scale {scale:.3g}"
        print(tag, flush=True)
        if kind == "attention":
            _check_attention(x, BH, N, d, rng, rows, heads, tag)
        else:
            _check_fused(x, dtype, BH, N, d, scale, rows, heads, tag)
