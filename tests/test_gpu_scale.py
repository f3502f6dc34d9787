"""GPU parity of the scaling kernel and of the three-kernel pipeline (matrix multiply, scaling,
softmax as separate kernels: what the paper's fused kernel replaces).

The scaling step has exactly one correct result per element - the exact product rounded once to
the storage type - so it is compared bit for bit with the oracle's fp64 product rounded here."""
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


def round_once(y64: np.ndarray, dtype: str) -> np.ndarray:
    """fp64 -> storage bits with ONE rounding to nearest even (normal-range values)."""
    if dtype == "f32":
        return y64.astype(np.float32).view(np.uint32)
    u = np.ascontiguousarray(y64, dtype=np.float64).view(np.uint64)
    drop = np.uint64(45)                                   # 52 stored significand bits -> 7
    bias = ((u >> drop) & np.uint64(1)) + np.uint64((1 << 44) - 1)
    r = ((u + bias) >> drop) << drop
    return (r.view(np.float64).astype(np.float32).view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def bits_of(t: torch.Tensor, dtype: str) -> np.ndarray:
    if dtype == "f32":
        return t.cpu().numpy().view(np.uint32)
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def run_scale(x_store: np.ndarray, dtype: str, scale: float, inplace: bool = False, guard: int = 1024):
    X = gu.to_dev(x_store.reshape(-1), dtype)
    n = X.numel()
    if inplace:
        attnw.attnw_scale(X, X, n, scale, gu.DT[dtype])
        torch.cuda.synchronize()
        return X
    Y, canary = gu.empty_like_out((n,), dtype, guard)
    attnw.attnw_scale(X, Y, n, scale, gu.DT[dtype])
    torch.cuda.synchronize()
    assert gu.guards_intact(canary), "scale kernel wrote outside Y"
    assert np.array_equal(bits_of(X, dtype), x_store.reshape(-1).view(bits_of(X, dtype).dtype)), "input modified"
    return Y


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("count", [1, 7, 8, 9, 1023, 4096, 1000003, 1 << 22])
def test_scale_bit_exact_any_count(dtype, count):
    x = wl.store(wl.standard_normal(900 + count % 97, 2, count) * 3.0, dtype)
    scale = float(np.float32(1.0 / math.sqrt(128.0)))
    ref = round_once(oracle.scale(x, dtype, scale), dtype)
    assert np.array_equal(bits_of(run_scale(x, dtype, scale), dtype), ref)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("scale", [0.125, -0.37, 3.0, 1.0, 0.0])
def test_scale_values_and_in_place(dtype, scale):
    x = wl.store(wl.standard_normal(41, 2, 70001) * 5.0, dtype)
    ref = round_once(oracle.scale(x, dtype, scale), dtype)
    got = bits_of(run_scale(x, dtype, scale), dtype)
    got_in_place = bits_of(run_scale(x, dtype, scale, inplace=True), dtype)
    assert np.array_equal(got, ref)
    assert np.array_equal(got_in_place, ref)


def test_scale_bf16_products_that_round_to_a_tie_in_fp32():
    """Products whose fp32 rounding lands exactly half way between two bf16 values although the
    exact product does not: rounding twice would go to the even neighbour, the exact product
    decides otherwise in half of the cases."""
    r = np.random.default_rng(12345)
    scales = (r.uniform(0.05, 4.0, 4096)).astype(np.float32)
    xs = wl.store(r.uniform(0.5, 8.0, 512) * r.choice([-1.0, 1.0], 512), "bf16")
    xw = wl.widen(xs, "bf16")
    exact = scales.astype(np.float64)[:, None] * xw[None, :]
    f32 = exact.astype(np.float32)
    tie = ((f32.view(np.uint32) & np.uint32(0xFFFF)) == np.uint32(0x8000)) & (f32.astype(np.float64) != exact)
    si, xi = np.nonzero(tie)
    assert len(si) >= 8, "search found too few cases"
    differs = 0
    for a, b in list(zip(si, xi))[:24]:
        x1 = xs[b:b + 1]
        ref = round_once(oracle.scale(x1, "bf16", float(scales[a])), "bf16")
        twice = wl.f32_to_bf16_bits(f32[a, b:b + 1])
        differs += int(ref[0] != twice[0])
        got = bits_of(run_scale(x1, "bf16", float(scales[a]), guard=64), "bf16")
        assert got[0] == ref[0], (float(scales[a]), float(xw[b]), hex(int(got[0])), hex(int(ref[0])))
    assert differs >= 1, "none of the cases tells single from double rounding"


@pytest.mark.parametrize("dtype,N,d", [("bf16", 512, 64), ("bf16", 320, 128), ("f32", 200, 64)])
def test_three_kernel_pipeline_stage_by_stage(dtype, N, d):
    """gemm_scores at scale 1, attnw_scale in place, attnw_softmax: each stage against the oracle on
    the input that stage actually received."""
    H = 2
    scale = float(np.float32(1.0 / math.sqrt(d)))
    x = wl.fused_inputs("t", dtype, 1, H, N, d, seed=1200 + N, scale=1.0)
    S = gu.run_scores(x, guard=4096)
    got = gu.to_f64(S)
    Qa, Ka = np.abs(wl.widen(x.Q, dtype)), np.abs(wl.widen(x.K, dtype))
    for h in range(H):
        ref = oracle.scores(x.Q[0, h], x.K[0, h], dtype, 1.0)
        acc_bound = d * 2.0 ** -24 * (Qa[0, h] @ Ka[0, h].T)
        store = (2.0 ** -8 if dtype == "bf16" else 2.0 ** -24) * np.abs(ref)
        assert (np.abs(got[0, h] - ref) <= acc_bound + store + 1e-30).all(), f"unscaled scores {dtype} head {h}"
    s_store = bits_of(S.reshape(-1), dtype)
    s_store = s_store.view(np.float32) if dtype == "f32" else s_store
    attnw.attnw_scale(S, S, S.numel(), scale, gu.DT[dtype])
    torch.cuda.synchronize()
    assert np.array_equal(bits_of(S.reshape(-1), dtype), round_once(oracle.scale(s_store, dtype, scale), dtype))
    scaled = bits_of(S.reshape(-1), dtype)
    scaled = (scaled.view(np.float32) if dtype == "f32" else scaled).reshape(H * N, N)
    P = gu.run_softmax(S.view(H * N, N), H * N, N, dtype)
    gu.check_weights(gu.to_f64(P), oracle.softmax(scaled, dtype), dtype, f"three-kernel softmax {dtype}")
    # end to end against the weights of the exact scores: reported precision of the unfused path
    # (bf16 scores rounded twice on the way cannot meet the fused tolerance; fp32 does)
    if dtype == "f32":
        ref_p = oracle.attention_weights_bh(x.Q, x.K, dtype, scale)
        gu.check_weights(gu.to_f64(P).reshape(1, H, N, N), ref_p, dtype, "three-kernel end to end fp32",
                         abs_f32=2e-6)


def test_three_kernel_pipeline_in_a_captured_graph():
    """The entry points only launch kernels on the caller's stream (no allocation, no memset, no
    synchronisation), so a stream capture records them; every replay must give the eager bits, also
    with eager work and synchronisations between the replays."""
    N, d, H = 512, 64, 3
    scale = float(np.float32(1.0 / math.sqrt(d)))
    x = wl.fused_inputs("t", "bf16", 1, H, N, d, seed=2100, scale=1.0)
    Q, K = gu.to_dev(x.Q, "bf16"), gu.to_dev(x.K, "bf16")
    S = torch.empty((1, H, N, N), dtype=torch.bfloat16, device="cuda")
    P = torch.empty_like(S)

    def pipeline(stream):
        attnw.attnw_gemm_scores(Q, K, S, 1, H, N, d, 1.0, attnw.ATTNW_BF16, stream)
        attnw.attnw_scale(S, S, S.numel(), scale, attnw.ATTNW_BF16, stream)
        attnw.attnw_softmax(S.view(H * N, N), P.view(H * N, N), H * N, N, attnw.ATTNW_BF16, stream)

    pipeline(torch.cuda.current_stream())
    torch.cuda.synchronize()
    want = P.view(torch.int16).clone()

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        pipeline(side)                                    # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            pipeline(torch.cuda.current_stream())
    torch.cuda.synchronize()
    for rep in range(4):
        P.fill_(-3.0)                                     # eager work between the replays
        S.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(P.view(torch.int16), want), f"replay {rep}"


def test_two_launch_softmax_in_a_captured_graph():
    """Few very long rows: attnw_softmax is two launches (statistics of the pieces of a row through a table in
    P, then the weights).  Both are recorded by a stream capture and every replay gives the eager bits, whatever
    P held before."""
    rows, cols = 3, 300000
    s = wl.softmax_inputs("t", "bf16", rows, cols, seed=2200, sigma=2.0, peak_fraction=0.001)
    S = gu.to_dev(s.S, "bf16")
    P = torch.empty_like(S)
    attnw.attnw_softmax(S, P, rows, cols, attnw.ATTNW_BF16, torch.cuda.current_stream())
    torch.cuda.synchronize()
    want = P.view(torch.int16).clone()
    gu.check_weights(gu.to_f64(P), oracle.softmax(s.S, "bf16"), "bf16", "two-launch softmax, eager")

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        attnw.attnw_softmax(S, P, rows, cols, attnw.ATTNW_BF16, side)
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            attnw.attnw_softmax(S, P, rows, cols, attnw.ATTNW_BF16, torch.cuda.current_stream())
    torch.cuda.synchronize()
    for rep in range(3):
        P.fill_(float(rep) - 1.0)                         # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(P.view(torch.int16), want), f"replay {rep}"


def test_split_key_fused_in_a_captured_graph():
    """One head of a long sequence: attnw_fused is two launches (statistics of the key ranges through tables
    inside P, then the weights).  Recorded by a stream capture, every replay gives the eager bits whatever P held."""
    N, d = 2048, 128
    x = wl.fused_inputs("t", "bf16", 1, 1, N, d, seed=2300)
    Q, K = gu.to_dev(x.Q, "bf16"), gu.to_dev(x.K, "bf16")
    P = torch.empty((1, 1, N, N), dtype=torch.bfloat16, device="cuda")
    scale = float(x.scale)
    attnw.attnw_fused(Q, K, P, 1, 1, N, d, scale, attnw.ATTNW_BF16, torch.cuda.current_stream())
    torch.cuda.synchronize()
    want = P.view(torch.int16).clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        attnw.attnw_fused(Q, K, P, 1, 1, N, d, scale, attnw.ATTNW_BF16, side)
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            attnw.attnw_fused(Q, K, P, 1, 1, N, d, scale, attnw.ATTNW_BF16, torch.cuda.current_stream())
    torch.cuda.synchronize()
    for rep in range(3):
        P.fill_(float(rep) * 7.0 - 3.0)                   # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(P.view(torch.int16), want), f"replay {rep}"


def _captured_replays_match_eager(call, out, replays=3):
    """`call(stream)` enqueues the library call that writes `out`.  Eager once, then recorded by a stream capture;
    every replay must give the eager bits whatever `out` held before."""
    call(torch.cuda.current_stream())
    torch.cuda.synchronize()
    want = out.view(torch.int16).clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        call(side)
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            call(torch.cuda.current_stream())
    torch.cuda.synchronize()
    for rep in range(replays):
        out.fill_(float(rep) * 7.0 - 3.0)                 # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), want), f"replay {rep}"


def test_last_strip_launch_of_a_ragged_length_in_a_captured_graph():
    """32 heads of 2089 keys: the 41 queries past the last full 256-query strip are a second launch."""
    B, H, N, d = 1, 32, 2089, 128
    x = wl.fused_inputs("t", "bf16", B, H, N, d, seed=2400)
    Q, K = gu.to_dev(x.Q, "bf16"), gu.to_dev(x.K, "bf16")
    P = torch.empty((B, H, N, N), dtype=torch.bfloat16, device="cuda")
    _captured_replays_match_eager(lambda s: attnw.attnw_fused(Q, K, P, B, H, N, d, float(x.scale), attnw.ATTNW_BF16, s), P)


@pytest.mark.parametrize("what", ["fused", "scores", "attention"])
def test_many_short_sequences_in_a_captured_graph(what):
    """The kernels in which a wave works alone on a (head, 32 queries) pair (their grid comes from an occupancy query
    made once per process, at the first call)."""
    B, H, N, d = 300, 4, 49, 32
    x = wl.fused_inputs("t", "bf16", B, H, N, d, seed=2500)
    Q, K = gu.to_dev(x.Q, "bf16"), gu.to_dev(x.K, "bf16")
    sc = float(x.scale)
    if what == "attention":
        V = gu.to_dev(wl.value_inputs(x, seed=2501), "bf16")
        O = torch.empty((B, H, N, d), dtype=torch.bfloat16, device="cuda")
        _captured_replays_match_eager(lambda s: attnw.attnw_attention(Q, K, V, O, B, H, N, d, sc, attnw.ATTNW_BF16, s), O)
    else:
        fn = attnw.attnw_fused if what == "fused" else attnw.attnw_gemm_scores
        P = torch.empty((B, H, N, N), dtype=torch.bfloat16, device="cuda")
        _captured_replays_match_eager(lambda s: fn(Q, K, P, B, H, N, d, sc, attnw.ATTNW_BF16, s), P)


def test_attention_with_a_launch_for_the_last_strip_in_a_captured_graph():
    """Two launches per call (the full strips, then the last few queries with their keys spread over four waves)."""
    B, H, N, d = 1, 64, 1025, 64
    x = wl.fused_inputs("t", "bf16", B, H, N, d, seed=2600)
    Q, K = gu.to_dev(x.Q, "bf16"), gu.to_dev(x.K, "bf16")
    V = gu.to_dev(wl.value_inputs(x, seed=2601), "bf16")
    O = torch.empty((B, H, N, d), dtype=torch.bfloat16, device="cuda")
    _captured_replays_match_eager(lambda s: attnw.attnw_attention(Q, K, V, O, B, H, N, d, float(x.scale), attnw.ATTNW_BF16, s), O)
