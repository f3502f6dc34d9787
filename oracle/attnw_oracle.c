/*
 * attnw_oracle.c -- TEST INFRASTRUCTURE, not part of the product.
 *
 * Plain, slow, fp64 CPU statement of what the attention-weight path computes,
 * written from the paper's definitions.  It shares no code, header, table or
 * helper with the HIP library and must never be called from the product path:
 * only the tests, the smoke check and the bench's cpu_baseline leg use it.
 *
 * What it follows:
 *   - attention weights  P = softmax(Q K^T / sqrt(d_k))   (Multi-Head
 *     Self-Attention section, definition of Attention(Q,K,V) without the V
 *     product, and the fused-kernel section: Q and K are n x d_k, P is n x n);
 *   - row softmax  sigma(Z)_ij = e^{Z_ij} / sum_k e^{Z_ik}   (Softmax section,
 *     unnumbered definition; m x n input, one distribution per row);
 *   - the max-subtracted form with m_i = max_j Z_ij   (Softmax section, Eq. 1),
 *     which has the same value and keeps exp() away from overflow;
 *   - the attention output  Attention(Q,K,V) = softmax(Q K^T / sqrt(d_k)) V
 *     (Multi-Head Self-Attention section; the section "Limitations and future
 *     Directions" names fusing this product into the kernel as the next step);
 *   - the scaling step on its own, scores divided by sqrt(d_k) as a separate
 *     pass over the matrix (section "Fused Matrix Multiply + Scaling +
 *     Softmax": the unfused pipeline runs multiply, scaling and softmax as
 *     three kernels).
 *
 * Readings taken where the paper is silent (all listed in the design notes):
 * the scale is the fp32 number the caller hands to the library, widened
 * exactly; inputs (fp32 or bf16) are widened exactly to fp64, so the oracle is
 * the true value of the function at the rounded inputs; dot products and row
 * sums are accumulated left to right in fp64; exp is libm's.
 *
 * Parity pins (tests/test_oracle_pins.py): closed forms for N <= 4, row sums,
 * uniform output for Q = 0, shift invariance (Eq. 1), key/query permutation,
 * agreement of the plain definition with the max-subtracted form, and a
 * cross-check against scipy/numpy on small cases; for the attention output:
 * one-hot V (output = columns of P), constant V, Q = 0 (column means of V),
 * linearity in V, joint permutation of keys and values, the N = 2 closed form;
 * for the scaling step: hand-computed products, powers of two (exponent shift
 * only), composition with the score oracle (scores at scale c = c * scores at
 * scale 1), numpy.  Nothing here is unpinned.
 *
 * No blocking, fusion or reordering: every function is the definition, row by
 * row.  OpenMP only splits independent rows across host threads.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1, ORACLE_F64 = 2 };

/* exact widening of one stored element to fp64 */
static double load_elem(const void *base, int dtype, int64_t idx)
{
    switch (dtype) {
    case ORACLE_F32:
        return (double)((const float *)base)[idx];
    case ORACLE_BF16: {
        /* bf16 is the upper half of an fp32 */
        uint32_t bits = (uint32_t)((const uint16_t *)base)[idx] << 16;
        float f;
        memcpy(&f, &bits, sizeof f);
        return (double)f;
    }
    default:
        return ((const double *)base)[idx];
    }
}

static int g_threads_used = 1;

/* number of host threads the last call actually ran on */
int oracle_threads_used(void) { return g_threads_used; }

static int pick_threads(int requested)
{
#ifdef _OPENMP
    int t = requested > 0 ? requested : omp_get_max_threads();
    return t < 1 ? 1 : t;
#else
    (void)requested;
    return 1;
#endif
}

/* Eq. 1 applied to one row of n scores, in place: z_j <- e^{z_j - m} / sum_k e^{z_k - m}. */
static void softmax_row_inplace(double *z, int64_t n)
{
    double m = z[0];
    for (int64_t j = 1; j < n; ++j)
        if (z[j] > m) m = z[j];
    double l = 0.0;
    for (int64_t j = 0; j < n; ++j) {
        z[j] = exp(z[j] - m);
        l += z[j];
    }
    for (int64_t j = 0; j < n; ++j)
        z[j] = z[j] / l;
}

/*
 * Scaled attention scores of one head, rows [row_begin, row_end):
 *   S_out[i - row_begin][j] = scale * sum_t Q[i][t] * K[j][t],  j = 0 .. N-1.
 * Q, K: [N][d] row-major in `dtype`.  S_out: [(row_end-row_begin)][N] fp64.
 */
int oracle_scores(const void *Q, const void *K, int dtype, int64_t N, int64_t d, float scale,
                  int64_t row_begin, int64_t row_end, double *S_out, int threads)
{
    if (!Q || !K || !S_out || N < 1 || d < 1 || row_begin < 0 || row_end > N || row_begin > row_end)
        return -1;
    const double c = (double)scale;
    const int nt = pick_threads(threads);
    g_threads_used = nt;
#pragma omp parallel for schedule(static) num_threads(nt)
    for (int64_t i = row_begin; i < row_end; ++i) {
        double *out = S_out + (i - row_begin) * N;
        for (int64_t j = 0; j < N; ++j) {
            double acc = 0.0;
            for (int64_t t = 0; t < d; ++t)
                acc += load_elem(Q, dtype, i * d + t) * load_elem(K, dtype, j * d + t);
            out[j] = c * acc;
        }
    }
    return 0;
}

/*
 * Attention weights of one head, rows [row_begin, row_end):
 *   P_out[i - row_begin][:] = softmax_j( scale * sum_t Q[i][t] K[j][t] ).
 */
int oracle_attention_weights(const void *Q, const void *K, int dtype, int64_t N, int64_t d, float scale,
                             int64_t row_begin, int64_t row_end, double *P_out, int threads)
{
    int rc = oracle_scores(Q, K, dtype, N, d, scale, row_begin, row_end, P_out, threads);
    if (rc) return rc;
    const int nt = pick_threads(threads);
#pragma omp parallel for schedule(static) num_threads(nt)
    for (int64_t r = 0; r < row_end - row_begin; ++r)
        softmax_row_inplace(P_out + r * N, N);
    return 0;
}

/*
 * Row softmax of rows [row_begin, row_end) of a [rows][cols] matrix in `dtype`
 * (Eq. 1).  P_out: [(row_end-row_begin)][cols] fp64.
 */
int oracle_softmax(const void *S, int dtype, int64_t rows, int64_t cols,
                   int64_t row_begin, int64_t row_end, double *P_out, int threads)
{
    if (!S || !P_out || rows < 1 || cols < 1 || row_begin < 0 || row_end > rows || row_begin > row_end)
        return -1;
    const int nt = pick_threads(threads);
    g_threads_used = nt;
#pragma omp parallel for schedule(static) num_threads(nt)
    for (int64_t i = row_begin; i < row_end; ++i) {
        double *out = P_out + (i - row_begin) * cols;
        for (int64_t j = 0; j < cols; ++j)
            out[j] = load_elem(S, dtype, i * cols + j);
        softmax_row_inplace(out, cols);
    }
    return 0;
}

/*
 * The Softmax section's definition taken literally, with no max subtraction:
 *   sigma(Z)_ij = e^{Z_ij} / sum_k e^{Z_ik}.
 * Only safe for small-magnitude inputs; exists so that a test can pin Eq. 1
 * (the two forms agree) against something other than the stable form itself.
 */
int oracle_softmax_plain(const void *S, int dtype, int64_t rows, int64_t cols, double *P_out)
{
    if (!S || !P_out || rows < 1 || cols < 1)
        return -1;
    for (int64_t i = 0; i < rows; ++i) {
        double *out = P_out + i * cols;
        double l = 0.0;
        for (int64_t j = 0; j < cols; ++j) {
            out[j] = exp(load_elem(S, dtype, i * cols + j));
            l += out[j];
        }
        for (int64_t j = 0; j < cols; ++j)
            out[j] = out[j] / l;
    }
    return 0;
}

/*
 * The scaling step alone:  Y_out[i] = scale * X[i]  in fp64 (exact: a 24-bit times an at most
 * 24-bit significand), X in `dtype`, scale the fp32 number widened exactly.
 */
int oracle_scale(const void *X, int dtype, int64_t count, float scale, double *Y_out)
{
    if (!X || !Y_out || count < 1)
        return -1;
    const double c = (double)scale;
    for (int64_t i = 0; i < count; ++i)
        Y_out[i] = c * load_elem(X, dtype, i);
    return 0;
}

/*
 * Attention output of one head, rows [row_begin, row_end):
 *   O_out[i - row_begin][t] = sum_j P[i][j] * V[j][t],  P = softmax_j(scale * Q K^T)  as above.
 * Q, K: [N][d], V: [N][dv] row-major in `dtype`.  O_out: [(row_end-row_begin)][dv] fp64.
 * scratch: [(row_end-row_begin)][N] fp64, receives P (the caller may want it for error bounds).
 */
int oracle_attention_output(const void *Q, const void *K, const void *V, int dtype, int64_t N, int64_t d, int64_t dv,
                            float scale, int64_t row_begin, int64_t row_end, double *O_out, double *scratch,
                            int threads)
{
    if (!V || !O_out || !scratch || dv < 1) return -1;
    int rc = oracle_attention_weights(Q, K, dtype, N, d, scale, row_begin, row_end, scratch, threads);
    if (rc) return rc;
    const int nt = pick_threads(threads);
#pragma omp parallel for schedule(static) num_threads(nt)
    for (int64_t r = 0; r < row_end - row_begin; ++r) {
        const double *p = scratch + r * N;
        for (int64_t t = 0; t < dv; ++t) {
            double acc = 0.0;
            for (int64_t j = 0; j < N; ++j)
                acc += p[j] * load_elem(V, dtype, j * dv + t);
            O_out[r * dv + t] = acc;
        }
    }
    return 0;
}
