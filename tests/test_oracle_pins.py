"""Pins for the fp64 CPU oracle: it is checked against what the paper's
definitions and the mathematics fix, never against itself.

Citations: Softmax section (unnumbered definition, Eq. 1), Multi-Head
Self-Attention section (Attention(Q,K,V) without the V product), fused-kernel
section (Q, K are n x d_k, P is n x n).
"""
import math
import os

import numpy as np
import pytest
import scipy.special

import oracle
from paper_2407_13885_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "softmax_closed_forms.txt")
TIGHT = 1e-12


def _rng(seed):
    return np.random.default_rng(seed)


def _closed_form_cases():
    cases = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            w, num, den = [p.split() for p in line.split("|")]
            cases.append(([float(x) for x in w], [float(x) for x in num], float(den[0])))
    return cases


# ---- closed forms (brute force, N <= 4) ---------------------------------------

@pytest.mark.parametrize("w,num,den", _closed_form_cases())
def test_softmax_closed_forms(w, num, den):
    z = np.log(np.array([w], dtype=np.float64))
    p = oracle.softmax(z, "f64")
    assert np.allclose(p[0], np.array(num) / den, rtol=1e-14, atol=0)


@pytest.mark.parametrize("w,num,den", _closed_form_cases())
def test_attention_closed_forms_via_d1(w, num, den):
    """d = 1, every query = 1, key_j = ln w_j, scale = 1  =>  every row is w / sum(w)."""
    n = len(w)
    Q = np.ones((n, 1))
    K = np.log(np.array(w, dtype=np.float64)).reshape(n, 1)
    p = oracle.attention_weights(Q, K, "f64", 1.0)
    for i in range(n):
        assert np.allclose(p[i], np.array(num) / den, rtol=1e-14, atol=0)


def test_n2_is_logistic():
    """N = 2: p = [sigma(s0 - s1), sigma(s1 - s0)] with sigma the logistic function."""
    for s0, s1 in [(0.3, -1.2), (5.0, 5.0), (-40.0, 3.0), (700.0, 690.0)]:
        p = oracle.softmax(np.array([[s0, s1]]), "f64")[0]
        assert math.isclose(p[0], 1.0 / (1.0 + math.exp(s1 - s0)), rel_tol=1e-14)
        assert math.isclose(p[1], 1.0 / (1.0 + math.exp(s0 - s1)), rel_tol=1e-14)


def test_hand_expanded_d2_pins_dot_product_and_scale():
    """Q = [[1, 2]], K = [[3, 4], [5, 6]] would need N == 2 rows of Q; use two
    different query rows so that a transposed operand or a dropped scale shows.

    scores (scale 1/2):  q0 = (1, 2):  [ (3+8)/2, (5+12)/2 ] = [5.5, 8.5]
                         q1 = (-1, 1): [ (-3+4)/2, (-5+6)/2 ] = [0.5, 0.5]
    """
    Q = np.array([[1.0, 2.0], [-1.0, 1.0]])
    K = np.array([[3.0, 4.0], [5.0, 6.0]])
    s = oracle.scores(Q, K, "f64", 0.5)
    assert np.array_equal(s, np.array([[5.5, 8.5], [0.5, 0.5]]))
    p = oracle.attention_weights(Q, K, "f64", 0.5)
    e3 = math.exp(3.0)
    assert np.allclose(p, [[1 / (1 + e3), e3 / (1 + e3)], [0.5, 0.5]], rtol=1e-14)


def test_scores_are_q_k_transposed_not_q_k():
    """With Q = I the scores are K^T: S_ij = k_j[i]."""
    K = np.array([[1.0, 2.0], [3.0, 4.0]])
    s = oracle.scores(np.eye(2), K, "f64", 1.0)
    assert np.array_equal(s, K.T)


# ---- invariants ---------------------------------------------------------------

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_rows_sum_to_one(dtype):
    x = wl.fused_inputs("t", dtype, 1, 2, 96, 32, seed=11)
    p = oracle.attention_weights_bh(x.Q, x.K, dtype, x.scale)
    assert np.abs(p.sum(-1) - 1.0).max() < TIGHT
    assert (p > 0).all()
    s = wl.softmax_inputs("t", dtype, 37, 301, seed=12, sigma=2.0, peak_fraction=0.01)
    ps = oracle.softmax(s.S, dtype)
    assert np.abs(ps.sum(-1) - 1.0).max() < TIGHT


@pytest.mark.parametrize("n", [1, 2, 3, 4, 17, 128])
def test_zero_queries_give_uniform(n):
    K = _rng(1).standard_normal((n, 8))
    p = oracle.attention_weights(np.zeros((n, 8)), K, "f64", 0.35)
    assert np.array_equal(p, np.full((n, n), 1.0 / n))


def test_equal_keys_give_uniform_and_n1_gives_one():
    Q = _rng(2).standard_normal((5, 4))
    K = np.tile(_rng(3).standard_normal((1, 4)), (5, 1))
    assert np.allclose(oracle.attention_weights(Q, K, "f64", 0.5), 0.2, rtol=1e-14)
    assert np.array_equal(oracle.attention_weights(Q[:1], K[:1], "f64", 0.5), [[1.0]])
    assert np.array_equal(oracle.softmax(np.array([[123.0]]), "f64"), [[1.0]])


@pytest.mark.parametrize("c", [1e3, -1e3, 0.5])
def test_shift_invariance_eq1(c):
    z = _rng(4).standard_normal((9, 33)) * 3.0
    shift = c * (1.0 + np.arange(9)).reshape(9, 1)   # a different constant per row
    assert np.abs(oracle.softmax(z + shift, "f64") - oracle.softmax(z, "f64")).max() < 1e-11


def test_plain_definition_equals_max_subtracted_form():
    """Eq. 1: both sides have the same value (small-magnitude inputs)."""
    z = _rng(5).standard_normal((7, 50)) * 2.0
    assert np.abs(oracle.softmax_plain(z, "f64") - oracle.softmax(z, "f64")).max() < 1e-15


def test_large_scores_do_not_overflow():
    z = np.array([[1000.0, 999.0, -1000.0]])
    p = oracle.softmax(z, "f64")[0]
    e = math.exp(-1.0)
    assert np.allclose(p, [1 / (1 + e), e / (1 + e), 0.0], rtol=1e-14, atol=1e-300)


def test_key_permutation_permutes_columns_and_query_permutation_rows():
    r = _rng(6)
    Q, K = r.standard_normal((12, 6)), r.standard_normal((12, 6))
    p = oracle.attention_weights(Q, K, "f64", 0.4)
    perm = r.permutation(12)
    pk = oracle.attention_weights(Q, K[perm], "f64", 0.4)
    assert np.abs(pk - p[:, perm]).max() < 1e-15
    pq = oracle.attention_weights(Q[perm], K, "f64", 0.4)
    assert np.abs(pq - p[perm, :]).max() < 1e-15


def test_rows_are_independent():
    r = _rng(7)
    Q, K = r.standard_normal((10, 4)), r.standard_normal((10, 4))
    p = oracle.attention_weights(Q, K, "f64", 0.5)
    Q2 = Q.copy()
    Q2[3] += 1.0
    p2 = oracle.attention_weights(Q2, K, "f64", 0.5)
    changed = np.abs(p2 - p).max(axis=1) > 0
    assert changed.tolist() == [i == 3 for i in range(10)]


def test_row_ranges_match_full_result():
    r = _rng(8)
    Q, K = r.standard_normal((20, 4)), r.standard_normal((20, 4))
    full = oracle.attention_weights(Q, K, "f64", 0.5)
    assert np.array_equal(oracle.attention_weights(Q, K, "f64", 0.5, rows=(7, 13)), full[7:13])
    z = r.standard_normal((20, 9))
    assert np.array_equal(oracle.softmax(z, "f64", rows=(19, 20)), oracle.softmax(z, "f64")[19:])
    assert np.array_equal(oracle.attention_weights(Q, K, "f64", 0.5, threads=1), full)


# ---- scale handling -------------------------------------------------------------

def test_scale_zero_is_uniform_and_doubling_scale_is_doubling_q():
    r = _rng(9)
    Q, K = r.standard_normal((6, 8)), r.standard_normal((6, 8))
    assert np.array_equal(oracle.attention_weights(Q, K, "f64", 0.0), np.full((6, 6), 1 / 6))
    a = oracle.attention_weights(Q, K, "f64", 0.5)
    b = oracle.attention_weights(2.0 * Q, K, "f64", 0.25)
    assert np.abs(a - b).max() < 1e-15


def test_scale_is_the_fp32_value_widened():
    """1/sqrt(128) is not exact in fp32: the oracle must use the fp32 number."""
    r = _rng(10)
    Q, K = r.standard_normal((8, 128)), r.standard_normal((8, 128))
    c32 = np.float32(1.0 / math.sqrt(128.0))
    got = oracle.scores(Q, K, "f64", c32)
    want = np.float64(c32) * (Q @ K.T)
    assert np.abs(got - want).max() < 1e-13
    off = (1.0 / math.sqrt(128.0)) * (Q @ K.T)
    assert np.abs(got - off).max() > 1e-10


# ---- storage formats --------------------------------------------------------------

def test_bf16_and_f32_inputs_are_widened_exactly():
    x = wl.fused_inputs("t", "bf16", 1, 1, 24, 16, seed=13)
    Qw, Kw = wl.widen(x.Q[0, 0], "bf16"), wl.widen(x.K[0, 0], "bf16")
    assert np.array_equal(oracle.attention_weights(x.Q[0, 0], x.K[0, 0], "bf16", x.scale),
                          oracle.attention_weights(Qw, Kw, "f64", x.scale))
    y = wl.fused_inputs("t", "f32", 1, 1, 24, 16, seed=14)
    assert np.array_equal(oracle.attention_weights(y.Q[0, 0], y.K[0, 0], "f32", y.scale),
                          oracle.attention_weights(y.Q[0, 0].astype(np.float64),
                                                   y.K[0, 0].astype(np.float64), "f64", y.scale))
    # bf16 1.0 = 0x3F80, -2.0 = 0xC000, 0.15625 = 0x3E20
    bits = np.array([[0x3F80, 0xC000, 0x3E20]], dtype=np.uint16)
    want = scipy.special.softmax(np.array([[1.0, -2.0, 0.15625]]), axis=-1)
    assert np.abs(oracle.softmax(bits, "bf16") - want).max() < 1e-15


# ---- library cross-checks (not the oracle) -------------------------------------------

@pytest.mark.parametrize("n,d", [(1, 4), (3, 1), (64, 32), (200, 64), (256, 128)])
def test_against_numpy_scipy(n, d):
    r = _rng(100 + n)
    Q, K = r.standard_normal((n, d)), r.standard_normal((n, d))
    c = np.float32(1.0 / math.sqrt(d))
    want = scipy.special.softmax(np.float64(c) * np.einsum("id,jd->ij", Q, K), axis=-1)
    assert np.abs(oracle.attention_weights(Q, K, "f64", c) - want).max() < TIGHT


def test_softmax_non_square_against_scipy():
    z = _rng(20).standard_normal((5, 77)) * 4.0
    assert np.abs(oracle.softmax(z, "f64") - scipy.special.softmax(z, axis=-1)).max() < TIGHT
    assert np.abs(oracle.softmax(z.T.copy(), "f64") - scipy.special.softmax(z.T, axis=-1)).max() < TIGHT


def test_bad_arguments_are_rejected():
    with pytest.raises(ValueError):
        oracle.softmax(np.zeros((2, 2)), "f64", rows=(1, 3))
    with pytest.raises(TypeError):
        oracle.softmax(np.zeros((2, 2), dtype=np.float32), "f64")


# ---- attention output  O = softmax(scale Q K^T) V  (Multi-Head Self-Attention section) -------------
# Pins chosen so that a transposed V, a contraction over the wrong axis, weights that are not
# normalised, or V rows matched to the wrong keys each fail at least one of them.

def test_output_with_one_hot_values_is_a_column_block_of_the_weights():
    r = _rng(30)
    N, d, dv = 12, 5, 7
    Q, K = r.standard_normal((N, d)), r.standard_normal((N, d))
    V = np.zeros((N, dv))
    V[np.arange(dv) + 2, np.arange(dv)] = 1.0          # V[j][t] = 1 iff j = t + 2
    O = oracle.attention_output(Q, K, V, "f64", 0.7)
    P = oracle.attention_weights(Q, K, "f64", 0.7)
    assert np.array_equal(O, P[:, 2:2 + dv])


def test_output_constant_values_and_zero_queries():
    r = _rng(31)
    N, d, dv = 9, 4, 6
    Q, K, V = r.standard_normal((N, d)), r.standard_normal((N, d)), r.standard_normal((N, dv))
    v = r.standard_normal(dv)
    O = oracle.attention_output(Q, K, np.tile(v, (N, 1)), "f64", 1.3)
    assert np.abs(O - v).max() < TIGHT                 # rows of the weights sum to 1
    O0 = oracle.attention_output(np.zeros((N, d)), K, V, "f64", 1.3)
    assert np.abs(O0 - V.mean(axis=0)).max() < TIGHT   # uniform weights: column means of V


def test_output_closed_form_two_keys():
    # d = 1, q_i = 1, k = (a, b): weights (s(a-b), s(b-a)), s the logistic function
    a, b = 0.25, -1.5
    Q = np.ones((2, 1)); K = np.array([[a], [b]]); V = np.array([[2.0, -1.0, 0.5], [10.0, 3.0, -4.0]])
    w0 = 1.0 / (1.0 + math.exp(b - a))
    want = w0 * V[0] + (1.0 - w0) * V[1]
    O = oracle.attention_output(Q, K, V, "f64", 1.0)
    assert np.abs(O - want).max() < TIGHT


def test_output_linear_in_values_and_invariant_under_joint_key_value_permutation():
    r = _rng(32)
    N, d, dv = 17, 8, 5
    Q, K = r.standard_normal((N, d)), r.standard_normal((N, d))
    V1, V2 = r.standard_normal((N, dv)), r.standard_normal((N, dv))
    O1, O2 = oracle.attention_output(Q, K, V1, "f64", 0.4), oracle.attention_output(Q, K, V2, "f64", 0.4)
    assert np.abs(oracle.attention_output(Q, K, 2.0 * V1 - 3.0 * V2, "f64", 0.4) - (2.0 * O1 - 3.0 * O2)).max() < 1e-13
    perm = r.permutation(N)
    assert np.abs(oracle.attention_output(Q, K[perm], V1[perm], "f64", 0.4) - O1).max() < 1e-13
    # permuting the values alone must change the result (V rows are tied to keys)
    assert np.abs(oracle.attention_output(Q, K, V1[perm], "f64", 0.4) - O1).max() > 1e-3


@pytest.mark.parametrize("n,d,dv", [(1, 4, 3), (50, 16, 16), (130, 64, 64)])
def test_output_against_numpy_scipy(n, d, dv):
    r = _rng(200 + n)
    Q, K, V = r.standard_normal((n, d)), r.standard_normal((n, d)), r.standard_normal((n, dv))
    c = np.float32(1.0 / math.sqrt(d))
    want = scipy.special.softmax(np.float64(c) * (Q @ K.T), axis=-1) @ V
    got, P = oracle.attention_output(Q, K, V, "f64", c, return_weights=True)
    assert np.abs(got - want).max() < 1e-13
    assert np.array_equal(P, oracle.attention_weights(Q, K, "f64", c))
    rows = oracle.attention_output(Q, K, V, "f64", c, rows=(n // 2, n))
    assert np.array_equal(rows, got[n // 2:])


# ---- the scaling step on its own (section "Fused Matrix Multiply + Scaling + Softmax") -------------

def test_scale_hand_values_and_powers_of_two():
    x = np.array([1.5, -2.25, 0.1, 0.0], dtype=np.float32)
    got = oracle.scale(x, "f32", 3.0)
    assert got.tolist() == [4.5, -6.75, 3.0 * float(np.float32(0.1)), 0.0]
    r = _rng(5)
    xb = wl.store(r.standard_normal(1000) * 4.0, "bf16")
    got = oracle.scale(xb, "bf16", 0.125)
    assert np.array_equal(got, np.ldexp(wl.widen(xb, "bf16"), -3))           # exponent shift only
    assert np.array_equal(oracle.scale(xb, "bf16", 1.0), wl.widen(xb, "bf16"))
    assert np.array_equal(oracle.scale(xb, "bf16", -1.0), -wl.widen(xb, "bf16"))


def test_scale_uses_the_fp32_scale_and_matches_numpy_and_the_score_oracle():
    r = _rng(6)
    x = wl.store(r.standard_normal((7, 33)), "f32")
    c = 1.0 / math.sqrt(128.0)
    got = oracle.scale(x, "f32", c)
    assert got.shape == x.shape
    assert np.array_equal(got, float(np.float32(c)) * x.astype(np.float64))
    assert not np.array_equal(got, c * x.astype(np.float64))                 # the double 1/sqrt(128) is another number
    # scores at scale c are c times the scores at scale 1
    Q, K = wl.store(r.standard_normal((9, 16)), "bf16"), wl.store(r.standard_normal((9, 16)), "bf16")
    s1 = oracle.scores(Q, K, "bf16", 1.0)
    np.testing.assert_allclose(oracle.scale(s1, "f64", c), oracle.scores(Q, K, "bf16", c), rtol=1e-15, atol=0)
