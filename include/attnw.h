/*
 * attnw.h -- C ABI of libattnw: attention weights on AMD MI355X (gfx950).
 *
 *     P = softmax(scale * Q K^T)      row-wise over keys, for every (batch, head)
 *
 * The operation is the one the paper narrows its work to (Multi-Head
 * Self-Attention section: softmax(Q K^T / sqrt(d_k)) for one head; Softmax
 * section: the row softmax and its max-subtracted form, Eq. 1; fused-kernel
 * section: Q and K are n x d_k, the output is the n x n matrix of attention
 * weights).  Batch and head are independent repetitions of that problem.
 *
 * Conventions common to every entry point
 *   - All data pointers are DEVICE pointers owned by the caller; the library
 *     never allocates, frees, copies to the host or synchronises.
 *   - Arrays are dense row-major: Q, K are [B][H][N][d] (d fastest), P and S
 *     are [B][H][N][N] (key index fastest) or [rows][cols] (cols fastest).
 *   - `dtype` selects ONE element type for inputs and output: ATTNW_F32
 *     (IEEE binary32) or ATTNW_BF16 (upper 16 bits of a binary32).  All
 *     arithmetic between load and store is fp32 (bf16 inputs are multiplied on
 *     the matrix cores with fp32 accumulation); bf16 results are rounded once,
 *     to nearest even, at the store.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Work is enqueued on it and the call returns without waiting.  A call is
 *     one kernel launch (two for a softmax of few rows too long for the
 *     registers of a workgroup, and for attention weights of so few heads that
 *     the keys of a strip are split over workgroups -- the first launch then
 *     uses parts of P as scratch --, or whose last few queries of a ragged
 *     length get one or two launches of their own; two for an attention output
 *     whose last few queries of a ragged length get a launch of their own) and
 *     nothing else on the stream, so it can be
 *     recorded by stream capture and replayed as part of a graph.
 *   - Return value: ATTNW_OK (0) or a negative attnw_status.  Nothing throws or
 *     aborts.  Arguments are validated before any HIP call, in this order:
 *     dtype, negative dimensions, empty problem (a batch, head, row or column
 *     count of 0: returns ATTNW_OK, launches nothing, pointers not looked at),
 *     null pointers, size overflow, supported sizes, 16-byte alignment of each
 *     base pointer, overlap of output with inputs.
 *   - Inputs must be finite.  A NaN poisons its own row only.
 *   - The library keeps no mutable global state apart from a per-device cache
 *     of the compute-unit count and, per kernel for short sequences, of the
 *     number of its workgroups that a compute unit holds (queried once, at the
 *     first call that needs it); calls from several host threads on different
 *     streams are safe.
 *   - Environment: ATTNW_FUSED_KERNEL selects among the kernels behind
 *     attnw_fused / attnw_gemm_scores for bf16 shapes that several of them
 *     serve (read at every call; tests and measurements compare them):
 *       unset    N from 8 to 128 (d up to 128; not N above 96 with d above 96)
 *                or to 192 (d up to 64): a wave per head and 32 queries, scores
 *                in its registers;
 *                d = 64 and N = 512 or 1024, or d = 32 or 64 and N up to 608
 *                and not a multiple of 32: scores of a strip held in registers,
 *                one sweep; one
 *                to a few heads of 1024 to 8192 keys: scores held across a
 *                gang of workgroups; else N a multiple of 256 and d = 64 or
 *                128 (scores: d = 64): round-based kernel; else general kernel
 *       rounds   never the register-resident kernels
 *       twopass  always the general two-pass kernel
 *       gang     the gang kernel wherever it takes the shape
 *       tiny     the wave-per-head kernel wherever it takes the shape
 *     Weights of all of them agree to rounding of the row sum, scores bit for bit.
 *     The workgroups of the gang kernel wait for each other's row statistics
 *     inside one launch, so all of a gang must be running at once: the grid is
 *     what the chip holds and a gang is a run of consecutive workgroups, which a
 *     device that starts workgroups in order completes whatever runs beside the
 *     call.  Every wait is bounded all the same: should other work keep a member
 *     off the chip for some tenths of a second, the rows that wait for it come
 *     out as NaN instead of the device hanging.  ATTNW_FUSED_KERNEL=rounds keeps
 *     a process that shares the device with long-running kernels off it.
 */
#ifndef ATTNW_H
#define ATTNW_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ATTNW_F32 = 0,
    ATTNW_BF16 = 1
} attnw_dtype;

typedef enum {
    ATTNW_OK = 0,
    ATTNW_ERR_NULL = -1,        /* a required pointer is NULL */
    ATTNW_ERR_SHAPE = -2,       /* a negative dimension, or a product that overflows int64 */
    ATTNW_ERR_DTYPE = -3,       /* dtype is neither ATTNW_F32 nor ATTNW_BF16 */
    ATTNW_ERR_UNSUPPORTED = -4, /* d not a multiple of 16 (bf16) / 4 (fp32) or above 256; a dimension beyond the 32-bit grid limits */
    ATTNW_ERR_ALIGN = -5,       /* a base pointer is not 16-byte aligned */
    ATTNW_ERR_ALIAS = -6,       /* output overlaps an input */
    ATTNW_ERR_LAUNCH = -7       /* the HIP runtime refused the launch */
} attnw_status;

/*
 * Fused attention weights (matrix multiply + score scaling + row softmax in one
 * kernel; only P is written to device memory -- the paper's fused kernel).
 *
 *   P[b][h][i][j] = exp(s_ij - m_i) / sum_k exp(s_ik - m_i),
 *   s_ij = scale * sum_t Q[b][h][i][t] * K[b][h][j][t],   m_i = max_j s_ij.
 *
 * Q, K : [B][H][N][d], read only.         P : [B][H][N][N], written.
 * N >= 1 arbitrary; d <= 256 and a multiple of 16 (bf16) or of 4 (fp32): rows of
 * Q and K are whole 16-byte chunks; scale any finite float (0 gives the uniform
 * 1/N, negative values are honoured).  P must not overlap Q or K.
 * P is the only memory a call writes, and for some shapes it doubles as the
 * exchange area while the call runs: workgroups that share the keys of a row
 * park partial row statistics (maximum, sum) in parts of P that the same call
 * overwrites with weights before it completes, and read them back from there.
 * What P held before the call is never used; after the call every element of
 * P is a weight.
 */
int attnw_fused(const void *Q, const void *K, void *P,
                int64_t B, int64_t H, int64_t N, int64_t d,
                float scale, int dtype, void *stream);

/*
 * Dedicated row softmax over precomputed scores (the paper's Softmax kernel;
 * Softmax section, Eq. 1):  P[r][j] = exp(S[r][j] - m_r) / sum_k exp(S[r][k] - m_r).
 *
 * S : [rows][cols], read only.            P : [rows][cols], written.
 * rows, cols >= 1 arbitrary.  P == S exactly (in place) is allowed; any other
 * overlap is ATTNW_ERR_ALIAS.  (Fewer rows than compute units, each longer than
 * the registers of a workgroup hold, and not in place: two launches, the first
 * of which parks partial row statistics in P.)
 */
int attnw_softmax(const void *S, void *P, int64_t rows, int64_t cols,
                  int dtype, void *stream);

/*
 * The same row softmax with separate storage types for scores and weights
 * (e.g. fp32 scores in, bf16 weights out: 6 instead of 8 bytes of device
 * memory traffic per element, one rounding of the result).  The arithmetic in
 * between is fp32 whatever the types.
 *
 * S : [rows][cols] in `in_dtype`, read only.   P : [rows][cols] in `out_dtype`.
 * With in_dtype == out_dtype this is attnw_softmax (in place allowed); with
 * different types P must not overlap S at all.
 */
int attnw_softmax_cast(const void *S, void *P, int64_t rows, int64_t cols,
                       int in_dtype, int out_dtype, void *stream);

/*
 * First half of the unfused pair (matrix multiply + scaling as its own kernel,
 * scores round-trip through device memory -- the pipeline the paper's fused
 * kernel replaces):  S[b][h][i][j] = scale * sum_t Q[b][h][i][t] * K[b][h][j][t],
 * rounded once to `dtype`.  attnw_softmax(S, P, B*H*N, N, ...) completes the pair.
 * Same argument rules as attnw_fused.
 */
int attnw_gemm_scores(const void *Q, const void *K, void *S,
                      int64_t B, int64_t H, int64_t N, int64_t d,
                      float scale, int dtype, void *stream);

/*
 * Scaling as a kernel of its own:  Y[i] = scale * X[i],  i < count, the exact
 * product rounded once (to nearest even) to `dtype`.  With it the unfused
 * pipeline can be run as the three kernels the paper's section "Fused Matrix
 * Multiply + Scaling + Softmax" describes: attnw_gemm_scores with scale 1,
 * attnw_scale, attnw_softmax, each reading and writing device memory.
 *
 * X : count elements, read only.          Y : count elements, written.
 * count >= 1 arbitrary.  Y == X exactly (in place) is allowed; any other
 * overlap is ATTNW_ERR_ALIAS.  Finite inputs whose products stay in the normal
 * range of `dtype`.
 */
int attnw_scale(const void *X, void *Y, int64_t count, float scale,
                int dtype, void *stream);

/*
 * Attention output with the weights kept on chip (the product that the paper's
 * section "Limitations and future Directions" names as the next thing to fuse:
 * Attention(Q, K, V) = softmax(Q K^T / sqrt(d_k)) V, Multi-Head Self-Attention
 * section):
 *
 *   O[b][h][i][t] = sum_j P[b][h][i][j] * V[b][h][j][t],   P as in attnw_fused.
 *
 * Q, K, V : [B][H][N][d], read only.      O : [B][H][N][d], written, never read.
 * P is never written to device memory: one sweep over the keys with a running
 * row maximum and sum (Eq. 1 applied incrementally).
 * ATTNW_BF16: d a multiple of 16 up to 256, any N >= 1.  The weights are rounded
 * to bf16 before they multiply V on the matrix cores, the output once more at the
 * store.  (d up to 128 runs tiled through on-chip memory -- d = 32, 64, 128 with N
 * a multiple of 256 on the fast path, other head sizes padded on chip, other
 * lengths with the rows past the end clamped and masked; few heads are spread over
 * the chip by key ranges; sequences of up to 128 tokens with d = 64, or 160 with
 * d = 32, run a wave per head and 32 queries without on-chip tiles.  Larger d reads its
 * operands straight from device memory.  ATTNW_ATTENTION_KERNEL=tiny / =tiled in the
 * environment puts every shape that the wave-per-head kernel takes on it / none.)
 * ATTNW_F32: d a multiple of 4 up to 256, any N >= 1.  Both contractions on the
 * fp32 matrix instruction: fp32 products, sums and weights, no rounding but fp32's.
 * Anything else: ATTNW_ERR_UNSUPPORTED.  O must not overlap Q, K or V.
 * Validation order as for attnw_fused.
 */
int attnw_attention(const void *Q, const void *K, const void *V, void *O,
                    int64_t B, int64_t H, int64_t N, int64_t d,
                    float scale, int dtype, void *stream);

/* Human-readable name of a status code; never NULL. */
const char *attnw_status_string(int status);

/* Library version: major * 10000 + minor * 100 + patch. */
int attnw_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ATTNW_H */
