"""GPU parity: the HIP path (through the C ABI) against the fp64 CPU oracle on
the same seeded inputs, element by element."""
import math

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


def _oracle_heads(x):
    return oracle.attention_weights_bh(x.Q, x.K, x.dtype, x.scale)


# ---- configuration 1: single head, fp32, N = 128, d = 64 ---------------------------------

def test_c1_fused_fp32():
    x = wl.c1()
    P = gu.run_fused(x, guard=4096)
    gu.check_weights(gu.to_f64(P), _oracle_heads(x), "f32", "c1 fused")


def test_c1_softmax_fp32_on_oracle_scores():
    """S = scale * Q K^T comes from the oracle, rounded once to fp32; the kernel's
    output is held against the oracle softmax of that same S and against the
    Q, K oracle itself."""
    x = wl.c1()
    s32 = oracle.scores(x.Q[0, 0], x.K[0, 0], "f32", x.scale).astype(np.float32)
    P = gu.run_softmax(gu.to_dev(s32, "f32"), 128, 128, "f32", guard=4096)
    got = gu.to_f64(P)
    gu.check_weights(got, oracle.softmax(s32, "f32"), "f32", "c1 softmax vs oracle softmax")
    gu.check_weights(got, _oracle_heads(x)[0, 0], "f32", "c1 softmax vs Q,K oracle")


# ---- configuration 2 recipe, reduced rows: several blocks and a ragged last block --------

def test_c2_recipe_small_bf16():
    s = wl.c2(rows=1027)
    P = gu.run_softmax(gu.to_dev(s.S, "bf16"), s.rows, s.cols, "bf16", guard=4096)
    gu.check_weights(gu.to_f64(P), oracle.softmax(s.S, "bf16"), "bf16", "c2 recipe, 1027 rows")


# ---- fused bf16, small shapes that span several tiles and ragged tails -------------------

@pytest.mark.parametrize("B,H,N,d", [(1, 1, 256, 64), (2, 3, 320, 128), (1, 2, 1024, 64), (1, 1, 520, 32),
                                     (1, 1, 200, 256), (1, 2, 136, 16), (1, 1, 72, 96)])
def test_fused_bf16_small(B, H, N, d):
    x = wl.fused_inputs("t", "bf16", B, H, N, d, seed=100 + N + d)
    P = gu.run_fused(x, guard=8192)
    gu.check_weights(gu.to_f64(P), _oracle_heads(x), "bf16", f"fused bf16 {B}x{H}x{N}x{d}")


# ---- ragged problems of several tiles on the general kernel: interior tiles take the unpredicated
# store path (past the caches when rows start on 64-byte boundaries: 992; through L2 otherwise: 1000, 500),
# the last key tile and the last strip the predicated one, odd lengths the element path; 300 heads put
# the problem on the wide-strip instantiation, d = 96 pads the rows of K in LDS.

@pytest.mark.parametrize("dtype,B,H,N,d", [("bf16", 1, 2, 1000, 128), ("bf16", 1, 2, 992, 64), ("bf16", 1, 1, 777, 64),
                                           ("bf16", 3, 100, 200, 64), ("bf16", 1, 2, 648, 96), ("bf16", 2, 150, 197, 64),
                                           ("f32", 1, 2, 500, 64), ("f32", 1, 1, 401, 32)])
def test_fused_ragged_multi_tile(dtype, B, H, N, d):
    x = wl.fused_inputs("t", dtype, B, H, N, d, seed=1500 + N + d, row_factor=(0.5, 2.0) if dtype == "bf16" else None)
    P = gu.run_fused(x, guard=8192)
    got = gu.to_f64(P)
    if B * H <= 4:
        gu.check_weights(got, _oracle_heads(x), dtype, f"ragged {dtype} {B}x{H}x{N}x{d}")
    else:   # many heads: the first, the last and two in the middle against the oracle, row sums everywhere
        flat = got.reshape(B * H, N, N)
        for bh in (0, 1, B * H // 2, B * H - 1):
            ref = oracle.attention_weights(x.Q.reshape(B * H, N, d)[bh], x.K.reshape(B * H, N, d)[bh], dtype, x.scale)
            gu.check_weights(flat[bh], ref, dtype, f"ragged {dtype} {B}x{H}x{N}x{d} head {bh}")
        assert np.abs(flat.sum(-1) - 1.0).max() <= (gu.ROWSUM_BF16 if dtype == "bf16" else gu.ROWSUM_F32)


# ---- ragged lengths (odd from 704, even from 1280) with enough 256-query strips for the chip: whole-line stores out of a ring of
# staged chunks laid out as the rows lie in memory.  The first tile of a row stores a window that begins before the
# row, interior tiles hold back up to four chunks for the next tile, the last tile of a row and the end of the rotated
# sweep flush what is left, chunks shared with the neighbouring rows go element by element; the last strip has waves
# without rows.  N a multiple of 8: rows on 16-byte boundaries (1376: on 64-byte boundaries, nothing is ever held
# back); 1284: rows at elements 0 or 4 of a chunk (8-byte staging writes), 1286: even elements (4-byte), odd N: any
# (2-byte).  d = 96 and 16 pad the rows of K on chip.

@pytest.mark.parametrize("B,H,N,d", [(1, 15, 1544, 64), (2, 17, 1288, 128), (1, 13, 2056, 128), (1, 17, 1416, 96),
                                     (1, 17, 1304, 16), (1, 12, 2200, 32), (1, 17, 1376, 64),
                                     (1, 20, 1025, 64), (1, 17, 1286, 128), (1, 17, 1284, 64), (2, 10, 1153, 128),
                                     (1, 13, 2049, 64), (1, 20, 1279, 32), (1, 17, 1281, 96), (1, 7, 4097, 128),
                                     (1, 25, 785, 64)])
@pytest.mark.parametrize("what", ["fused", "scores"])
def test_rows_on_16_byte_boundaries_take_whole_line_stores(B, H, N, d, what):
    assert N % 256 != 0 and N >= (704 if N % 2 else 1280) and B * H * ((N + 255) // 256) >= 100
    _ring_case(B, H, N, d, what)


def _ring_case(B, H, N, d, what, scale=None):
    x = wl.fused_inputs("t", "bf16", B, H, N, d, seed=1700 + N + d, scale=scale, row_factor=(0.5, 2.0))
    heads = sorted({0, 1, B * H // 2, B * H - 1})
    Qf, Kf = x.Q.reshape(B * H, N, d), x.K.reshape(B * H, N, d)
    if what == "fused":
        got = gu.to_f64(gu.run_fused(x, guard=8192)).reshape(B * H, N, N)
        for bh in heads:
            ref = oracle.attention_weights(Qf[bh], Kf[bh], "bf16", x.scale)
            gu.check_weights(got[bh], ref, "bf16", f"ring {B}x{H}x{N}x{d} head {bh}")
        assert np.abs(got.sum(-1) - 1.0).max() <= gu.ROWSUM_BF16
    else:
        got = gu.to_f64(gu.run_scores(x, guard=8192)).reshape(B * H, N, N)
        assert np.isfinite(got).all()
        for bh in heads:
            ref = oracle.scores(Qf[bh], Kf[bh], "bf16", x.scale)
            acc = d * 2.0 ** -24 * abs(float(x.scale)) * (np.abs(wl.widen(Qf[bh], "bf16")) @ np.abs(wl.widen(Kf[bh], "bf16")).T)
            assert (np.abs(got[bh] - ref) <= acc + 2.0 ** -8 * np.abs(ref) + 1e-30).all(), f"ring scores head {bh}"


# the last, partial strip as a launch of its own (32-query strips, keys over the 8 waves) where its workgroups would
# start another round on the chip's 256 compute units: 8, 1, 41 and 90 queries in it (1, 1, 2, 3 strips of the second
# launch), 128-query strips: 1 and 65
@pytest.mark.parametrize("B,H,N,d,scale", [(1, 16, 4104, 128, None), (1, 16, 4097, 64, -0.2), (1, 32, 2089, 128, None),
                                           (1, 51, 1370, 64, None), (1, 128, 513, 32, None), (1, 73, 961, 64, -0.1)])
@pytest.mark.parametrize("what", ["fused", "scores"])
def test_last_strip_of_a_ragged_length_as_a_launch_of_its_own(B, H, N, d, scale, what):
    BM = 256 if N >= (704 if N % 2 else 1280) and not (N % 2 and N < 1152 and d <= 64) else 128
    full, slots = B * H * (N // BM), 256 * (1 if BM == 256 else 2)
    assert 0 < N % BM <= 96 and -(-full // slots) < -(-(full + B * H) // slots)
    _ring_case(B, H, N, d, what, scale=scale)


@pytest.mark.parametrize("B,H,N,d", [(4, 50, 577, 64), (2, 60, 333, 32), (1, 100, 1001, 64), (3, 70, 321, 48), (1, 40, 1151, 16)])
@pytest.mark.parametrize("what", ["fused", "scores"])
def test_odd_lengths_of_a_few_hundred_take_the_ring_with_128_query_strips(B, H, N, d, what):
    assert N % 2 == 1 and 320 <= N < 1152 and d <= 64 and B * H * ((N + 127) // 128) >= 200
    _ring_case(B, H, N, d, what)


# ---- fused bf16, shapes served by the round-based kernel (N a multiple of 256, d = 64 or 128) ---
# 600 strips over 256 workgroups: strip lists that cross head boundaries; 20 strips: workgroups
# with one strip (a statistics round followed directly by a weights round) and idle ones;
# one head with many strips: long lists inside one head.

@pytest.mark.parametrize("B,H,N,d", [(3, 100, 256, 64), (1, 5, 512, 128), (1, 1, 2048, 128), (2, 2, 1536, 64),
                                     (1, 130, 256, 128)])
def test_fused_bf16_round_kernel_shapes(B, H, N, d):
    x = wl.fused_inputs("t", "bf16", B, H, N, d, seed=700 + H + N + d)
    P = gu.run_fused(x, guard=8192)
    gu.check_weights(gu.to_f64(P), _oracle_heads(x), "bf16", f"round kernel {B}x{H}x{N}x{d}")


# ---- fused bf16, d = 64, N = 512 or 1024: the kernel that keeps the scores of a strip in registers.
#      Many heads: strip lists that cross heads (K replaced in LDS); one head: short lists.  (d = 128, N = 512 would
#      fit as well but measured slower than the round-based kernel, 49.6 against 42.4 us for 192 heads: it is not
#      routed there; the shapes stay in the list as a test of that routing.)

@pytest.mark.parametrize("B,H,N,d", [(1, 1, 512, 64), (1, 3, 1024, 64), (2, 5, 512, 64), (1, 37, 1024, 64),
                                     (1, 2, 512, 128), (3, 90, 512, 128), (1, 300, 1024, 64)])
def test_fused_bf16_resident_kernel(B, H, N, d):
    x = wl.fused_inputs("t", "bf16", B, H, N, d, seed=900 + H + N + d, row_factor=(0.5, 2.5))
    P = gu.run_fused(x, guard=8192)
    if H <= 40:
        gu.check_weights(gu.to_f64(P), _oracle_heads(x), "bf16", f"resident kernel {B}x{H}x{N}x{d}")
    else:   # many heads: a spread of them against the oracle, every row sum
        got = gu.to_f64(P)
        for b, h in [(0, 0), (0, 1), (B - 1, H // 2), (B - 1, H - 2), (B - 1, H - 1)]:
            ref = oracle.attention_weights(x.Q[b, h], x.K[b, h], "bf16", x.scale)
            gu.check_weights(got[b, h], ref, "bf16", f"resident kernel {B}x{H}x{N}x{d} head ({b},{h})")
        assert np.abs(got.sum(-1) - 1.0).max() <= gu.ROWSUM_BF16


@pytest.mark.parametrize("N,d", [(512, 64), (1024, 64), (512, 128)])
def test_fused_bf16_resident_kernel_negative_scale_and_other_kernels(N, d, monkeypatch):
    x = wl.fused_inputs("t", "bf16", 1, 2, N, d, seed=17 + N + d, scale=-0.2, row_factor=(0.5, 3.0))
    ref = _oracle_heads(x)
    P = gu.run_fused(x, guard=4096)
    gu.check_weights(gu.to_f64(P), ref, "bf16", f"resident kernel, negative scale, N={N} d={d}")
    # the same problem through the round-based and the two-pass kernel
    for which in ("rounds", "twopass"):
        monkeypatch.setenv("ATTNW_FUSED_KERNEL", which)
        gu.check_weights(gu.to_f64(gu.run_fused(x, guard=4096)), ref, "bf16", f"{which} kernel, negative scale, N={N}")


@pytest.mark.parametrize("d", [64, 128])
def test_fused_bf16_round_kernel_negative_scale_and_sharp_rows(d):
    x = wl.fused_inputs("t", "bf16", 1, 3, 512, d, seed=31 + d, scale=-1.0 / math.sqrt(d), row_factor=(0.5, 3.0))
    P = gu.run_fused(x, guard=4096)
    gu.check_weights(gu.to_f64(P), _oracle_heads(x), "bf16", f"round kernel, negative scale, d={d}")


@pytest.mark.parametrize("N", [1, 2, 3, 4, 7, 17, 31, 33, 100, 129, 257])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_fused_ragged_n(N, dtype):
    x = wl.fused_inputs("t", dtype, 1, 2, N, 64, seed=200 + N)
    P = gu.run_fused(x, guard=4096)
    gu.check_weights(gu.to_f64(P), _oracle_heads(x), dtype, f"fused {dtype} N={N}")


@pytest.mark.parametrize("d", [4, 8, 12, 16, 20, 32, 36, 48, 64, 68, 80, 100, 128, 192, 252, 256])
def test_fused_fp32_all_d(d):
    x = wl.fused_inputs("t", "f32", 1, 1, 160, d, seed=300 + d)
    P = gu.run_fused(x, guard=4096)
    gu.check_weights(gu.to_f64(P), _oracle_heads(x), "f32", f"fused f32 d={d}")


def test_fused_sharp_and_flat_rows_bf16():
    """The long-row configuration's recipe (per-row factors in [0.5, 3]) at a size
    the oracle covers in full: mixes near-uniform and sharply peaked rows."""
    x = wl.fused_inputs("t", "bf16", 1, 2, 768, 64, seed=4, row_factor=(0.5, 3.0))
    P = gu.run_fused(x, guard=4096)
    gu.check_weights(gu.to_f64(P), _oracle_heads(x), "bf16", "sharp/flat rows")


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("scale", [0.0, -0.125, 0.5])
def test_fused_scale_values(dtype, scale):
    x = wl.fused_inputs("t", dtype, 1, 1, 192, 64, seed=17, scale=scale)
    P = gu.run_fused(x, guard=4096)
    ref = _oracle_heads(x)
    # The 1e-6 bound belongs to scores of unit spread (scale = 1/sqrt(d)).  An fp32
    # contraction of d terms leaves each scaled score with an error that grows like
    # |scale| * sqrt(d), and p inherits it relatively: widen the bound by that factor.
    abs_f32 = gu.ABS_F32 * max(1.0, abs(scale) * math.sqrt(64))
    gu.check_weights(gu.to_f64(P), ref, dtype, f"scale {scale}", abs_f32=abs_f32)
    if scale == 0.0:
        assert np.allclose(gu.to_f64(P), 1.0 / 192, rtol=4e-3)


def test_fused_zero_queries_uniform():
    x = wl.fused_inputs("t", "bf16", 1, 1, 256, 64, seed=5)
    x.Q[...] = 0
    P = gu.to_f64(gu.run_fused(x))
    assert np.array_equal(P, np.full_like(P, 1.0 / 256))      # 2^-8 is exact in bf16


def test_fused_is_deterministic_and_heads_independent():
    x = wl.fused_inputs("t", "bf16", 2, 2, 384, 64, seed=6)
    a = gu.run_fused(x)
    b = gu.run_fused(x)
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    y = wl.fused_inputs("t", "bf16", 2, 2, 384, 64, seed=6)
    y.K[1, 0] = wl.fused_inputs("t", "bf16", 1, 1, 384, 64, seed=7).K[0, 0]
    c = gu.run_fused(y)
    same = [[torch.equal(a[i, j].view(torch.int16), c[i, j].view(torch.int16)) for j in range(2)] for i in range(2)]
    assert same == [[True, True], [False, True]]


# ---- dedicated softmax: every dispatch path, ragged and in place ----------------------------

@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("cols", [1, 7, 8, 64, 520, 1000, 1024, 2049, 4096, 8192, 12288, 16384, 32768, 65536, 70000])
def test_softmax_cols(dtype, cols):
    rows = 9 if cols <= 16384 else 3
    s = wl.softmax_inputs("t", dtype, rows, cols, seed=400 + cols, sigma=2.0, peak_fraction=0.01)
    P = gu.run_softmax(gu.to_dev(s.S, dtype), rows, cols, dtype, guard=4096)
    gu.check_weights(gu.to_f64(P), oracle.softmax(s.S, dtype), dtype, f"softmax {dtype} cols={cols}")


# Short rows share a wave (4 to 32 lanes per row when rows start on 16-byte boundaries, 16 or 64 lanes
# with element accesses otherwise): many rows, a row count that leaves the last block partly empty.
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("cols", [3, 16, 24, 48, 100, 136, 197, 250, 256, 257, 1023])
def test_softmax_many_short_rows(dtype, cols):
    rows = 1003
    s = wl.softmax_inputs("t", dtype, rows, cols, seed=1600 + cols, sigma=2.0, peak_fraction=0.02)
    P = gu.run_softmax(gu.to_dev(s.S, dtype), rows, cols, dtype, guard=4096)
    gu.check_weights(gu.to_f64(P), oracle.softmax(s.S, dtype), dtype, f"softmax {dtype} {rows} x {cols}")


# Few very long rows: a row is cut into pieces, one workgroup each, every workgroup gathering the
# statistics of the whole row; odd lengths put the rows off the 16-byte boundaries (scalar head and tail).
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("rows,cols", [(3, 300000), (3, 300001), (2, 1048576 + 24), (5, 99999), (300, 20001)])
def test_softmax_long_rows(dtype, rows, cols):
    s = wl.softmax_inputs("t", dtype, rows, cols, seed=1700 + cols % 1000, sigma=2.0, peak_fraction=0.001)
    P = gu.run_softmax(gu.to_dev(s.S, dtype), rows, cols, dtype, guard=4096)
    gu.check_weights(gu.to_f64(P), oracle.softmax(s.S, dtype), dtype, f"softmax {dtype} {rows} x {cols}")


@pytest.mark.parametrize("src,dst", [("f32", "bf16"), ("bf16", "f32")])
@pytest.mark.parametrize("rows,cols", [(3, 300001), (1003, 100), (7, 70000)])
def test_softmax_cast_long_and_short_rows(src, dst, rows, cols):
    import paper_2407_13885_amd as attnw
    s = wl.softmax_inputs("t", src, rows, cols, seed=1800 + cols % 1000, sigma=2.0)
    S = gu.to_dev(s.S, src)
    P, canary = gu.empty_like_out((rows, cols), dst, guard=4096)
    attnw.attnw_softmax_cast(S, P, rows, cols, gu.DT[src], gu.DT[dst])
    torch.cuda.synchronize()
    assert gu.guards_intact(canary), "softmax wrote outside P"
    gu.check_weights(gu.to_f64(P), oracle.softmax(s.S, src), dst, f"softmax {src}->{dst} {rows} x {cols}")


# Many short rows off the 16-byte boundaries, or of one or two chunks (at least 1024 rows of fewer than 64 columns): whole chunks through LDS,
# 8, 4, 2 or 1 rows per chunk-aligned group.  Row counts that fill the last wave, leave it one row, end the matrix on
# a chunk boundary or inside a chunk (the last chunk then goes element by element); in place; rows of the lowest value.
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("cols", [1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 12, 16, 17, 20, 31, 33, 36, 49, 50, 52, 62, 63, 90, 100, 124,
                                  126, 196, 252])
def test_softmax_many_short_rows_off_the_chunk_boundaries(dtype, cols):
    for rows, inplace in ((1024, False), (1031, True), (4097, False)):
        s = wl.softmax_inputs("t", dtype, rows, cols, seed=2600 + cols + rows, sigma=2.0, peak_fraction=0.01)
        S = s.S.copy()
        low = np.float32(-3.3895314e38) if dtype == "f32" else np.uint16(0xff7f)
        S[5, :] = low                                # a fully masked row: uniform
        S[rows - 1, : cols // 2] = low
        P = gu.run_softmax(gu.to_dev(S, dtype), rows, cols, dtype, guard=0 if inplace else 4096, inplace=inplace)
        got = gu.to_f64(P)
        gu.check_weights(got, oracle.softmax(S, dtype), dtype, f"short rows {dtype} {rows} x {cols}")
        assert np.abs(got[5] - 1.0 / cols).max() <= (2.0 ** -8 if dtype == "bf16" else 1e-6) / cols


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("cols", [2048, 1001, 100, 2049, 70000, 300001])
def test_softmax_in_place(dtype, cols):
    s = wl.softmax_inputs("t", dtype, 21, cols, seed=500 + cols, sigma=2.0, peak_fraction=0.01)
    S = gu.to_dev(s.S, dtype)
    P = gu.run_softmax(S, 21, cols, dtype, inplace=True)
    assert P.data_ptr() == S.data_ptr()
    gu.check_weights(gu.to_f64(P), oracle.softmax(s.S, dtype), dtype, f"in-place {dtype} cols={cols}")


# Rows off the 16-byte boundaries that share a wave: the chunk two rows of a block share leaves as one store, put
# together in LDS behind a barrier that every load of the block precedes -- in place, a row count that leaves the last
# block partly empty, 16 and 32 lanes per row.
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("cols", [67, 197, 393, 251])
def test_softmax_in_place_rows_that_share_chunks_within_a_block(dtype, cols):
    rows = 1003
    s = wl.softmax_inputs("t", dtype, rows, cols, seed=520 + cols, sigma=2.0, peak_fraction=0.02)
    S = gu.to_dev(s.S, dtype)
    P = gu.run_softmax(S, rows, cols, dtype, inplace=True)
    assert P.data_ptr() == S.data_ptr()
    gu.check_weights(gu.to_f64(P), oracle.softmax(s.S, dtype), dtype, f"in-place {dtype} {rows} x {cols}")


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("cols", [7, 100, 1001, 2048, 2049, 70000, 300001])
def test_softmax_rows_of_the_lowest_finite_value(dtype, cols):
    """A fully masked row (every score the lowest finite value of the type) is finite input: Eq. 1 gives the
    uniform 1/cols, whichever kernel the row length selects.  Rows that hold one ordinary score among
    them put all the weight on it."""
    rows = 5
    s = wl.softmax_inputs("t", dtype, rows, cols, seed=2100 + cols, sigma=2.0)
    lowest = np.float32(-3.3895314e38)          # the lowest finite bf16 value, also an fp32 value
    S = s.S.copy()
    low = lowest if dtype == "f32" else np.uint16(0xff7f)
    S[0, :] = low
    S[2, :] = low
    S[3, :] = low
    S[3, cols // 2] = np.float32(1.5) if dtype == "f32" else np.uint16(0x3fc0)
    P = gu.run_softmax(gu.to_dev(S, dtype), rows, cols, dtype, guard=4096)
    got = gu.to_f64(P)
    gu.check_weights(got, oracle.softmax(S, dtype), dtype, f"masked rows {dtype} cols={cols}")
    assert np.allclose(got[0], 1.0 / cols, rtol=4e-3) and got[3, cols // 2] == 1.0


def test_softmax_large_offsets_fp32():
    """Eq. 1: a large common offset per row must cancel (fp32 keeps the 1e-6 bound)."""
    s = wl.softmax_inputs("t", "f32", 16, 512, seed=9, sigma=1.5)
    shifted = (s.S.astype(np.float64) + 1000.0 * (1 + np.arange(16)).reshape(16, 1)).astype(np.float32)
    P = gu.run_softmax(gu.to_dev(shifted, "f32"), 16, 512, "f32")
    gu.check_weights(gu.to_f64(P), oracle.softmax(shifted, "f32"), "f32", "shifted rows")


# ---- unfused pair: stage-wise parity --------------------------------------------------------

@pytest.mark.parametrize("dtype,N,d", [("bf16", 320, 64), ("bf16", 129, 128), ("f32", 200, 64), ("f32", 128, 256)])
def test_gemm_scores_and_unfused_pair(dtype, N, d):
    x = wl.fused_inputs("t", dtype, 1, 2, N, d, seed=600 + N)
    S = gu.run_scores(x, guard=4096)
    got = gu.to_f64(S)
    Qa, Ka = np.abs(wl.widen(x.Q, dtype)), np.abs(wl.widen(x.K, dtype))
    for h in range(2):
        ref = oracle.scores(x.Q[0, h], x.K[0, h], dtype, x.scale)
        # fp32 accumulation of d products: |err| <= d * 2^-24 * scale * sum|q||k| (first order),
        # then one rounding to the storage type
        acc_bound = d * 2.0 ** -24 * float(x.scale) * (Qa[0, h] @ Ka[0, h].T)
        store = (2.0 ** -8 if dtype == "bf16" else 2.0 ** -24) * np.abs(ref)
        assert (np.abs(got[0, h] - ref) <= acc_bound + store + 1e-30).all(), f"scores {dtype} head {h}"
    # second stage on the S actually produced
    P = gu.run_softmax(S.view(2 * N, N), 2 * N, N, dtype)
    s_host = S.view(2 * N, N).cpu()
    s_np = s_host.numpy() if dtype == "f32" else s_host.view(torch.int16).numpy().view(np.uint16)
    gu.check_weights(gu.to_f64(P), oracle.softmax(s_np, dtype), dtype, f"unfused softmax {dtype}")


# ---- score GEMM on the shapes the round-based kernel serves ------------------------------------

def _check_scores(x, S, what):
    got = gu.to_f64(S)
    d = x.Q.shape[-1]
    Qa, Ka = np.abs(wl.widen(x.Q, "bf16")), np.abs(wl.widen(x.K, "bf16"))
    B, H = x.Q.shape[:2]
    for b in range(B):
        for h in range(H):
            ref = oracle.scores(x.Q[b, h], x.K[b, h], "bf16", x.scale)
            acc_bound = d * 2.0 ** -24 * abs(float(x.scale)) * (Qa[b, h] @ Ka[b, h].T)
            assert (np.abs(got[b, h] - ref) <= acc_bound + 2.0 ** -8 * np.abs(ref) + 1e-30).all(), f"{what} head {b},{h}"


@pytest.mark.parametrize("B,H,N,d", [(3, 100, 256, 64), (1, 5, 512, 128), (2, 2, 1536, 64), (1, 1, 2048, 128)])
def test_gemm_scores_round_kernel_shapes(B, H, N, d):
    x = wl.fused_inputs("t", "bf16", B, H, N, d, seed=800 + H + N + d)
    _check_scores(x, gu.run_scores(x, guard=8192), f"round-kernel scores {B}x{H}x{N}x{d}")


def test_gemm_scores_round_kernel_negative_scale_matches_general_kernel(monkeypatch):
    x = wl.fused_inputs("t", "bf16", 1, 3, 512, 64, seed=77, scale=-0.37)
    S = gu.run_scores(x, guard=4096)
    _check_scores(x, S, "round-kernel scores, negative scale")
    # the general kernel accumulates in the same order: identical bits
    monkeypatch.setenv("ATTNW_FUSED_KERNEL", "twopass")
    S2 = gu.run_scores(x, guard=4096)
    assert torch.equal(S.view(torch.int16), S2.view(torch.int16))


# Rows that start on 16-byte boundaries are kept in registers as groups of 8 (a 16-bit type on either side) or 4
# elements, lanes per row and groups per lane chosen by the number of groups: the counts at which the choice
# changes, and one past each, for every pair of types.
@pytest.mark.parametrize("src,dst", [("bf16", "bf16"), ("f32", "f32"), ("f32", "bf16"), ("bf16", "f32")])
@pytest.mark.parametrize("groups", [64, 65, 128, 129, 192, 193, 256, 257, 320, 321, 512, 513, 1024, 1025, 1280, 1281,
                                    2048, 2049, 4096, 4097, 6144, 6145, 8192])
def test_softmax_groups_per_row_at_the_steps_of_the_launch_shapes(src, dst, groups):
    import paper_2407_13885_amd as attnw
    e = 4 if (src, dst) == ("f32", "f32") else 8
    cols = groups * e
    rows = 5 if groups <= 64 * 5 else 3
    s = wl.softmax_inputs("t", src, rows, cols, seed=2100 + groups, sigma=2.0, peak_fraction=0.005)
    S = gu.to_dev(s.S, src)
    P, canary = gu.empty_like_out((rows, cols), dst, guard=4096)
    attnw.attnw_softmax_cast(S, P, rows, cols, gu.DT[src], gu.DT[dst])
    torch.cuda.synchronize()
    assert gu.guards_intact(canary), "softmax wrote outside P"
    gu.check_weights(gu.to_f64(P), oracle.softmax(s.S, src), dst, f"softmax {src}->{dst} {rows} x {cols}")


@pytest.mark.parametrize("groups", [8193, 12288, 12289, 16384])
def test_softmax_fp32_rows_of_up_to_sixteen_groups_per_lane(groups):
    rows, cols = 3, groups * 4
    s = wl.softmax_inputs("t", "f32", rows, cols, seed=2200 + groups, sigma=2.0, peak_fraction=0.005)
    P = gu.run_softmax(gu.to_dev(s.S, "f32"), rows, cols, "f32", guard=4096)
    gu.check_weights(gu.to_f64(P), oracle.softmax(s.S, "f32"), "f32", f"softmax f32 {rows} x {cols}")


# ---- softmax with separate storage types for scores and weights ------------------------------------

@pytest.mark.parametrize("src,dst", [("f32", "bf16"), ("bf16", "f32")])
@pytest.mark.parametrize("cols", [8, 24, 1000, 2048, 2049, 16384, 40000])
def test_softmax_cast(src, dst, cols):
    import paper_2407_13885_amd as attnw
    rows = 37 if cols < 10000 else 5
    s = wl.softmax_inputs("t", src, rows, cols, seed=1300 + cols, sigma=2.0)
    S = gu.to_dev(s.S, src)
    P, canary = gu.empty_like_out((rows, cols), dst, guard=4096)
    attnw.attnw_softmax_cast(S, P, rows, cols, gu.DT[src], gu.DT[dst])
    torch.cuda.synchronize()
    assert gu.guards_intact(canary), "softmax wrote outside P"
    gu.check_weights(gu.to_f64(P), oracle.softmax(s.S, src), dst, f"softmax {src}->{dst} cols={cols}")


def test_softmax_cast_with_equal_types_is_attnw_softmax():
    import paper_2407_13885_amd as attnw
    s = wl.softmax_inputs("t", "bf16", 64, 2048, seed=7, sigma=2.0)
    S = gu.to_dev(s.S, "bf16")
    a = gu.run_softmax(S, 64, 2048, "bf16")
    b = torch.empty_like(a)
    attnw.attnw_softmax_cast(S, b, 64, 2048, attnw.ATTNW_BF16, attnw.ATTNW_BF16)
    torch.cuda.synchronize()
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))


# ---- concurrent callers ---------------------------------------------------------------------------

def test_calls_from_two_host_threads_on_two_streams():
    """The library keeps no mutable state between calls: two host threads, each on a stream of its own,
    get the bits a single caller gets."""
    import threading
    import paper_2407_13885_amd as attnw
    xs = [wl.fused_inputs("t", "bf16", 1, 4, 1024, 64, seed=50 + i) for i in range(2)]
    want = [gu.run_fused(x).view(torch.int16).clone() for x in xs]
    dev = [(gu.to_dev(x.Q, "bf16"), gu.to_dev(x.K, "bf16")) for x in xs]
    outs = [torch.empty((1, 4, 1024, 1024), dtype=torch.bfloat16, device="cuda") for _ in xs]
    streams = [torch.cuda.Stream() for _ in xs]
    torch.cuda.synchronize()
    errors = []

    def worker(i):
        try:
            x = xs[i]
            for _ in range(20):
                attnw.attnw_fused(dev[i][0], dev[i][1], outs[i], x.B, x.H, x.N, x.d, float(x.scale), attnw.ATTNW_BF16,
                                  streams[i])
                attnw.attnw_softmax(outs[i].view(-1, x.N), outs[i].view(-1, x.N), x.H * x.N, x.N, attnw.ATTNW_BF16,
                                    streams[i])
                attnw.attnw_fused(dev[i][0], dev[i][1], outs[i], x.B, x.H, x.N, x.d, float(x.scale), attnw.ATTNW_BF16,
                                  streams[i])
            streams[i].synchronize()
        except Exception as e:      # surfaced in the main thread
            errors.append(e)

    threads = [threading.Thread(target=worker, args=(i,)) for i in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    torch.cuda.synchronize()
    assert not errors, errors
    for i in range(2):
        assert torch.equal(outs[i].view(torch.int16), want[i]), f"thread {i}"


# ---- seeded random shapes: the boundaries between kernels and instantiations are crossed somewhere ---------

def _random_fused_shapes(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        dtype = "bf16" if rng.random() < 0.7 else "f32"
        d = int(rng.choice([16, 32, 48, 64, 80, 96, 128, 160, 256]))
        N = int(rng.choice([rng.integers(1, 40), rng.integers(40, 300), rng.integers(300, 900), 256, 512, 640, 768]))
        BH = int(rng.choice([1, 2, 3, 7, 40, 210])) if N <= 300 else int(rng.choice([1, 2, 5]))
        B = 1 if BH % 2 or rng.random() < 0.5 else 2
        scale = float(rng.choice([1.0 / math.sqrt(d), -1.0 / math.sqrt(d), 0.03]))
        out.append((dtype, B, BH // B, N, d, scale))
    return out


@pytest.mark.parametrize("dtype,B,H,N,d,scale", _random_fused_shapes(36, seed=20240713))
def test_fused_and_scores_random_shapes(dtype, B, H, N, d, scale):
    # (fp32: scores of unit spread, which is what the 1e-6 absolute bound belongs to; bf16: sharp and flat rows mixed)
    x = wl.fused_inputs("t", dtype, B, H, N, d, seed=7000 + 13 * N + d + H, scale=scale,
                        row_factor=(0.5, 2.0) if dtype == "bf16" else None)
    P = gu.run_fused(x, guard=4096)
    got = gu.to_f64(P).reshape(B * H, N, N)
    Qf, Kf = x.Q.reshape(B * H, N, d), x.K.reshape(B * H, N, d)
    heads = sorted({0, (B * H) // 2, B * H - 1})
    abs_f32 = gu.ABS_F32 * max(1.0, abs(scale) * math.sqrt(d))
    for bh in heads:
        ref = oracle.attention_weights(Qf[bh], Kf[bh], dtype, x.scale)
        gu.check_weights(got[bh], ref, dtype, f"random shape {dtype} {B}x{H}x{N}x{d} scale {scale:.3g} head {bh}", abs_f32=abs_f32)
    rs_tol = gu.ROWSUM_BF16 if dtype == "bf16" else gu.ROWSUM_F32
    assert np.abs(got.sum(-1) - 1.0).max() <= rs_tol
    # the score GEMM of the same problem: accumulation bound + one rounding, on the same heads
    S = gu.to_f64(gu.run_scores(x, guard=4096)).reshape(B * H, N, N)
    for bh in heads:
        ref = oracle.scores(Qf[bh], Kf[bh], dtype, x.scale)
        bound = d * 2.0 ** -24 * abs(scale) * (np.abs(wl.widen(Qf[bh], dtype)) @ np.abs(wl.widen(Kf[bh], dtype)).T)
        ulp = (2.0 ** -8 if dtype == "bf16" else 2.0 ** -24) * np.abs(ref)
        assert (np.abs(S[bh] - ref) <= bound + ulp + 1e-30).all(), f"scores {dtype} {B}x{H}x{N}x{d} head {bh}"


def _random_softmax_shapes(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        src = "bf16" if rng.random() < 0.6 else "f32"
        dst = src if rng.random() < 0.6 else ("f32" if src == "bf16" else "bf16")
        cols = int(rng.choice([rng.integers(1, 70), rng.integers(70, 1100), rng.integers(1100, 9000), rng.integers(9000, 80000),
                               8 * rng.integers(1, 1200), 1024, 2048, 4096]))
        rows = int(rng.integers(1, 600)) if cols < 9000 else int(rng.integers(1, 12))
        out.append((src, dst, rows, cols, bool(src == dst and rng.random() < 0.3)))
    return out


@pytest.mark.parametrize("src,dst,rows,cols,inplace", _random_softmax_shapes(40, seed=20240714))
def test_softmax_random_shapes(src, dst, rows, cols, inplace):
    import paper_2407_13885_amd as attnw
    s = wl.softmax_inputs("t", src, rows, cols, seed=9000 + rows + cols, sigma=2.5, peak_fraction=0.01)
    S = gu.to_dev(s.S, src)
    if inplace:
        P, canary = S, None
    else:
        P, canary = gu.empty_like_out((rows, cols), dst, guard=4096)
    attnw.attnw_softmax_cast(S, P, rows, cols, gu.DT[src], gu.DT[dst])
    torch.cuda.synchronize()
    if canary is not None:
        assert gu.guards_intact(canary), "softmax wrote outside P"
    gu.check_weights(gu.to_f64(P), oracle.softmax(s.S, src), dst, f"softmax {src}->{dst} {rows} x {cols} inplace={inplace}")


# ---- few strips: the keys of a strip are split over several workgroups, statistics through tables in P --------

# (d = 128 on one head: taken from the persistent kernel; the others: shapes of the general kernel)
@pytest.mark.parametrize("dtype,B,H,N,d,scale", [("bf16", 1, 1, 2048, 128, 0.0884), ("bf16", 1, 1, 4096, 128, -0.0884),
                                                 ("bf16", 1, 2, 3000, 64, 0.125), ("bf16", 1, 1, 1500, 96, 0.1),
                                                 ("bf16", 1, 2, 2176, 128, 0.0884), ("f32", 1, 1, 2048, 64, 0.125),
                                                 ("f32", 1, 2, 1026, 32, 0.17677669),
                                                 # rows of P off the 8-byte boundaries (tables of single floats) and, bf16
                                                 # with an odd length, off the 4-byte ones (a table then starts 2 bytes
                                                 # into its piece)
                                                 ("bf16", 1, 1, 2050, 128, 0.0884), ("f32", 1, 1, 1025, 64, 0.125),
                                                 ("bf16", 1, 1, 2051, 64, 0.125), ("bf16", 1, 2, 4097, 128, -0.0884),
                                                 ("bf16", 1, 3, 1283, 96, 0.1)])
def test_fused_and_scores_with_split_keys(dtype, B, H, N, d, scale):
    x = wl.fused_inputs("t", dtype, B, H, N, d, seed=8000 + N + d, scale=scale, row_factor=(0.5, 3.0) if dtype == "bf16" else None)
    P = gu.run_fused(x, guard=8192)
    got = gu.to_f64(P)
    rows = sorted({0, 1, 63, 64, 255, 256, N // 2, N - 257, N - 2, N - 1} | set(np.random.default_rng(N).integers(0, N, 24).tolist()))
    for h in range(H):
        ref = np.concatenate([oracle.attention_weights(x.Q[0, h], x.K[0, h], dtype, x.scale, rows=(r, r + 1)) for r in rows])
        gu.check_weights(got[0, h][rows], ref, dtype, f"split keys {dtype} {B}x{H}x{N}x{d} head {h}")
    rs_tol = gu.ROWSUM_BF16 if dtype == "bf16" else gu.ROWSUM_F32
    assert np.abs(got.sum(-1) - 1.0).max() <= rs_tol
    S = gu.to_f64(gu.run_scores(x, guard=8192))
    for h in range(H):
        ref = np.concatenate([oracle.scores(x.Q[0, h], x.K[0, h], dtype, x.scale, rows=(r, r + 1)) for r in rows])
        qa, ka = np.abs(wl.widen(x.Q[0, h], dtype))[rows], np.abs(wl.widen(x.K[0, h], dtype))
        bound = d * 2.0 ** -24 * abs(scale) * (qa @ ka.T) + (2.0 ** -8 if dtype == "bf16" else 2.0 ** -24) * np.abs(ref) + 1e-30
        assert (np.abs(S[0, h][rows] - ref) <= bound).all(), f"split-key scores {dtype} {N}x{d} head {h}"


def test_split_keys_match_the_unsplit_kernel_bit_for_bit_in_the_scores(monkeypatch):
    x = wl.fused_inputs("t", "bf16", 1, 1, 2048, 128, seed=8100)
    a = gu.run_scores(x, guard=4096)
    monkeypatch.setenv("ATTNW_FUSED_KERNEL", "twopass")     # the plain two-pass kernel: a workgroup per strip
    b = gu.run_scores(x, guard=4096)
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))
