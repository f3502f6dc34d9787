"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times.

Every configuration is compared with the oracle on every element (c4 and c5 in blocks of
512 query rows, which the oracle computes on all host cores), and on a property that
holds at any size and needs no oracle: every row of P sums to 1."""
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


def _row_sums_ok(P, tol):
    worst = 0.0
    for b in range(P.shape[0]):
        for h in range(P.shape[1]):
            worst = max(worst, float((P[b, h].float().sum(-1) - 1.0).abs().max().item()))
    assert worst <= tol, f"row sum off by {worst:.3e}"


def _sample_rows(N, seed, n_random=24):
    fixed = [0, 1, 31, 32, 63, 64, 127, 128, 255, 256, N // 2 - 1, N // 2, N - 257, N - 256, N - 2, N - 1]
    rnd = np.random.default_rng(seed).integers(0, N, size=n_random).tolist()
    return sorted({r for r in fixed + rnd if 0 <= r < N})


def test_c2_full_softmax_bf16():
    s = wl.c2()
    P = gu.run_softmax(gu.to_dev(s.S, "bf16"), s.rows, s.cols, "bf16", guard=4096)
    for r0 in range(0, s.rows, 4096):           # the oracle's fp64 output, 64 MiB at a time
        r1 = min(r0 + 4096, s.rows)
        gu.check_weights(gu.to_f64(P[r0:r1]), oracle.softmax(s.S, "bf16", rows=(r0, r1)), "bf16", f"c2 rows {r0}..{r1}")


def test_c3_full_fused_bf16():
    x = wl.c3()
    P = gu.run_fused(x, guard=8192)
    for b in range(x.B):
        for h in range(x.H):
            ref = oracle.attention_weights(x.Q[b, h], x.K[b, h], "bf16", x.scale)
            gu.check_weights(gu.to_f64(P[b, h]), ref, "bf16", f"c3 head ({b},{h})")


@pytest.mark.parametrize("name", ["c4", "c5"])
def test_large_fused_every_element_and_row_sums(name):
    """Every element of c4 (2.7e8) and c5 (2.1e9) against the oracle, 512 query rows at a time.  On a 16-thread
    host the oracle takes about 2 s for c4 and 15 s for c5; with the comparison the test runs about 10 s / 80 s."""
    import sys
    x = wl.CONFIGS[name]()
    P = gu.run_fused(x, guard=8192)
    _row_sums_ok(P, gu.ROWSUM_BF16)
    step = 512
    for b in range(x.B):
        for h in range(x.H):
            for r0 in range(0, x.N, step):
                r1 = min(r0 + step, x.N)
                ref = oracle.attention_weights(x.Q[b, h], x.K[b, h], "bf16", x.scale, rows=(r0, r1))
                gu.check_weights(gu.to_f64(P[b, h, r0:r1]), ref, "bf16", f"{name} head ({b},{h}) rows {r0}..{r1}")
            print(f"  {name} head ({b},{h}) ok", file=sys.stderr, flush=True)


def test_c4_unfused_pair_full_size():
    """The unfused pair at the paper's fused size: score GEMM checked on sampled rows,
    softmax checked against the oracle softmax of the scores actually produced."""
    x = wl.c4()
    S = gu.run_scores(x)
    Sv = S.view(x.H * x.N, x.N)
    Pm = gu.run_softmax(Sv, x.H * x.N, x.N, "bf16")
    _row_sums_ok(Pm.view(1, x.H, x.N, x.N), gu.ROWSUM_BF16)
    for h in (0, 7, 15):
        rows = _sample_rows(x.N, seed=77 + h, n_random=8)
        ref_s = np.concatenate([oracle.scores(x.Q[0, h], x.K[0, h], "bf16", x.scale, rows=(r, r + 1)) for r in rows])
        got_s = gu.to_f64(S[0, h][rows])
        assert (np.abs(got_s - ref_s) <= 2.0 ** -8 * np.abs(ref_s) + 1e-4).all(), f"scores head {h}"
        s_bits = S[0, h][rows].cpu().view(torch.int16).numpy().view(np.uint16)
        gu.check_weights(gu.to_f64(Pm.view(x.H, x.N, x.N)[h][rows]), oracle.softmax(s_bits, "bf16"), "bf16",
                         f"unfused softmax head {h}")


@pytest.mark.parametrize("name", ["c3", "c4"])
def test_three_kernel_pipeline_full_size(name):
    """Multiply (scale 1), scaling in place, softmax at benchmark sizes: the scaling stage bit for bit on
    sampled rows (first, last and interior blocks of the flat array included), the softmax against the
    oracle softmax of the scaled scores actually produced."""
    import paper_2407_13885_amd as attnw
    x = wl.CONFIGS[name]()
    scale = float(x.scale)
    Q, K = gu.to_dev(x.Q, "bf16"), gu.to_dev(x.K, "bf16")
    S = torch.empty((x.B, x.H, x.N, x.N), dtype=torch.bfloat16, device="cuda")
    attnw.attnw_gemm_scores(Q, K, S, x.B, x.H, x.N, x.d, 1.0, attnw.ATTNW_BF16)
    torch.cuda.synchronize()
    Sv = S.view(x.B * x.H * x.N, x.N)
    picks = []
    for bh in (0, x.B * x.H // 2, x.B * x.H - 1):
        picks += [bh * x.N + r for r in _sample_rows(x.N, seed=90 + bh, n_random=6)]
    picks = sorted(set(picks))
    before = Sv[picks].cpu().view(torch.int16).numpy().view(np.uint16)
    attnw.attnw_scale(S, S, S.numel(), scale, attnw.ATTNW_BF16)
    torch.cuda.synchronize()
    after = Sv[picks].cpu().view(torch.int16).numpy().view(np.uint16)
    exact = oracle.scale(before, "bf16", scale)
    # one rounding to nearest even of the exact product (fp64 -> bf16, normal range)
    u = exact.view(np.uint64)
    r = ((u + ((u >> np.uint64(45)) & np.uint64(1)) + np.uint64((1 << 44) - 1)) >> np.uint64(45)) << np.uint64(45)
    want = (r.view(np.float64).astype(np.float32).view(np.uint32) >> np.uint32(16)).astype(np.uint16)
    assert np.array_equal(after, want), "scaling stage differs from the exact product rounded once"
    Pm = gu.run_softmax(Sv, x.B * x.H * x.N, x.N, "bf16")
    _row_sums_ok(Pm.view(x.B, x.H, x.N, x.N), gu.ROWSUM_BF16)
    gu.check_weights(gu.to_f64(Pm[picks]), oracle.softmax(after, "bf16"), "bf16", f"{name} three-kernel softmax")


def test_long_rows_have_no_systematic_error():
    """One rounding to bf16 hides errors of a few 1e-4 in a row's normaliser from the element-wise
    bound most of the time.  The mean signed relative error of a row does not: rounding errors of
    16384 elements average out to ~1e-5, a normaliser that is off shifts every element the same way.
    Long, sharp rows (the long-row configuration's recipe) through the round-based kernel."""
    x = wl.fused_inputs("t", "bf16", 1, 2, 16384, 64, seed=4, row_factor=(0.5, 3.0))
    P = gu.run_fused(x)
    rows = _sample_rows(x.N, seed=5, n_random=48)
    for h in range(x.H):
        got = gu.to_f64(P[0, h][rows])
        ref = np.concatenate([oracle.attention_weights(x.Q[0, h], x.K[0, h], "bf16", x.scale, rows=(r, r + 1))
                              for r in rows])
        gu.check_weights(got, ref, "bf16", f"long rows head {h}")
        mean_rel = ((got - ref) / ref).mean(-1)
        worst = float(np.abs(mean_rel).max())
        assert worst <= 6e-5, f"head {h}: mean signed relative error of a row {worst:.2e} (row {rows[int(np.abs(mean_rel).argmax())]})"


def test_fused_and_attention_at_the_longest_supported_row():
    """N = 32768 is the longest sequence the round-based kernel takes (one head: P is 2 GiB); sampled rows
    against the oracle, every row sum, and the attention output of the same inputs on sampled rows."""
    import paper_2407_13885_amd as attnw
    x = wl.fused_inputs("t", "bf16", 1, 1, 32768, 64, seed=32, row_factor=(0.5, 2.0))
    P = gu.run_fused(x)
    _row_sums_ok(P, gu.ROWSUM_BF16)
    rows = _sample_rows(x.N, seed=33, n_random=16)
    got = gu.to_f64(P[0, 0][rows])
    ref = np.concatenate([oracle.attention_weights(x.Q[0, 0], x.K[0, 0], "bf16", x.scale, rows=(r, r + 1)) for r in rows])
    gu.check_weights(got, ref, "bf16", "N = 32768 sampled rows")
    del P
    torch.cuda.empty_cache()
    V = wl.value_inputs(x, seed=34)
    Q, K, Vd = gu.to_dev(x.Q, "bf16"), gu.to_dev(x.K, "bf16"), gu.to_dev(V, "bf16")
    O = torch.empty((1, 1, x.N, x.d), dtype=torch.bfloat16, device="cuda")
    attnw.attnw_attention(Q, K, Vd, O, 1, 1, x.N, x.d, float(x.scale), attnw.ATTNW_BF16)
    torch.cuda.synchronize()
    Of = gu.to_f64(O)[0, 0]
    Vw = np.abs(wl.widen(V[0, 0], "bf16"))
    for r in rows[::3]:
        ref_o, Pr = oracle.attention_output(x.Q[0, 0], x.K[0, 0], V[0, 0], "bf16", x.scale, rows=(r, r + 1),
                                            return_weights=True)
        A = Pr @ Vw
        tol = 2.0 ** -8 * (A + np.abs(ref_o)) * 1.02 + 1e-6 * A
        assert (np.abs(Of[r:r + 1] - ref_o) <= tol).all(), f"attention output row {r} at N = 32768"


@pytest.mark.parametrize("N", [65536, 40000])
def test_fused_beyond_the_round_kernel_lengths(N):
    """Sequences longer than the round-based kernel takes (N = 65536: P is 8 GiB) and a long ragged one run on
    the general two-pass kernel: 64-bit row offsets, sampled rows against the oracle, every row sum, and no
    systematic error of the normaliser over rows of that length."""
    x = wl.fused_inputs("t", "bf16", 1, 1, N, 64, seed=64 + N % 7, row_factor=(0.5, 2.0))
    P = gu.run_fused(x)
    _row_sums_ok(P, gu.ROWSUM_BF16)
    rows = _sample_rows(x.N, seed=65, n_random=12)
    got = gu.to_f64(P[0, 0][rows])
    ref = np.concatenate([oracle.attention_weights(x.Q[0, 0], x.K[0, 0], "bf16", x.scale, rows=(r, r + 1)) for r in rows])
    gu.check_weights(got, ref, "bf16", f"N = {N} sampled rows")
    mean_rel = ((got - ref) / np.maximum(ref, 1e-300)).mean(-1)
    assert float(np.abs(mean_rel).max()) <= 6e-5, f"mean signed relative error of a row {np.abs(mean_rel).max():.2e}"


def _bits(t):
    """bf16 device tensor -> host array of its bit patterns (the oracle's storage type)."""
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def test_more_than_two_to_the_31_elements_of_short_sequences_and_rows():
    """600000 windows of 64 tokens (2.46e9 weights, 4.9 GB) and 5e7 softmax rows of 49 columns (2.45e9 elements):
    element indices beyond 32 bits in the kernels that pack many heads / rows into a wave.  Inputs are drawn on the
    device (seeded); every row sum on the device, the first, middle and last heads / row blocks against the oracle."""
    import paper_2407_13885_amd as attnw
    torch.manual_seed(77)
    BH, N, d = 600000, 64, 32
    Q = torch.randn(1, BH, N, d, device="cuda", dtype=torch.bfloat16)
    K = torch.randn_like(Q)
    P = torch.empty(1, BH, N, N, device="cuda", dtype=torch.bfloat16)
    scale = d ** -0.5
    attnw.attnw_fused(Q, K, P, 1, BH, N, d, scale, attnw.ATTNW_BF16)
    torch.cuda.synchronize()
    flat = P.view(-1, N)
    step = 1 << 22
    worst = max(float((flat[i:i + step].float().sum(-1) - 1).abs().max().item()) for i in range(0, flat.shape[0], step))
    assert worst <= gu.ROWSUM_BF16, f"row sum off by {worst:.3e}"
    for h in (0, 1, BH // 2, 524288, 524289, BH - 2, BH - 1):      # (524288 * 64 * 64 = 2^31 elements)
        ref = oracle.attention_weights(_bits(Q[0, h]), _bits(K[0, h]), "bf16", np.float32(scale))
        gu.check_weights(gu.to_f64(P[0, h]), ref, "bf16", f"head {h} of {BH}")
    del P, Q, K, flat
    torch.cuda.empty_cache()

    rows, cols = 50_000_000, 49
    S = torch.empty(rows, cols, device="cuda", dtype=torch.bfloat16)
    for i in range(0, rows, step):
        S[i:i + step] = (torch.randn(min(step, rows - i), cols, device="cuda") * 2).to(torch.bfloat16)
    W = torch.empty_like(S)
    attnw.attnw_softmax(S, W, rows, cols, attnw.ATTNW_BF16)
    torch.cuda.synchronize()
    worst = max(float((W[i:i + step].float().sum(-1) - 1).abs().max().item()) for i in range(0, rows, step))
    assert worst <= gu.ROWSUM_BF16, f"softmax row sum off by {worst:.3e}"
    for r0 in (0, rows // 2, 43826196 - 500, rows - 1000):         # (43826196 * 49 crosses 2^31 elements)
        ref = oracle.softmax(_bits(S[r0:r0 + 1000]), "bf16")
        gu.check_weights(gu.to_f64(W[r0:r0 + 1000]), ref, "bf16", f"softmax rows {r0}..")
