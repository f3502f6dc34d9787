// Internal interface between the C-ABI layer and the kernel translation units.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace attnw {

enum class DType : int { F32 = 0, BF16 = 1 };

// Row softmax, arguments already validated.  Returns the launch status.
hipError_t launch_softmax(DType in, DType out, const void* S, void* P, int64_t rows, int64_t cols, hipStream_t stream);

// Fused attention weights (scores_only = false) or scaled scores (scores_only = true).
hipError_t launch_qk(DType dt, bool scores_only, const void* Q, const void* K, void* out,
                     int64_t BH, int64_t N, int64_t d, float scale, hipStream_t stream);

// Compute units of the current device (256 if the query fails).
int compute_units();

// bf16, by the round-based kernel: fused attention weights (statistics of one strip gathered while the
// weights of the previous one are written) or, with scores_only, the scaled scores (one sweep per
// strip through the same staging and store path; d = 64 only).  Only for the shapes
// qk_rounds_supported() accepts.
bool qk_rounds_supported(int64_t BH, int64_t N, int64_t d);
hipError_t launch_qk_rounds(bool scores_only, const void* Q, const void* K, void* out, int64_t BH, int64_t N, int64_t d,
                            float scale, hipStream_t stream);

// Fused attention weights, bf16, d = 64, N = 512 or 1024: the scores of a 32-query strip stay in registers
// between the contraction and the normalisation (one sweep over the keys).
bool qk_resident_supported(int64_t BH, int64_t N, int64_t d);
hipError_t launch_qk_resident(const void* Q, const void* K, void* out, int64_t BH, int64_t N, float scale,
                              hipStream_t stream);

// Fused attention weights or scaled scores, bf16, d = 32 or 64, any N up to 608 (the odd lengths of a class token in
// front of a patch grid):
// scores of a 32-query strip resident in registers, the strip staged as the contiguous block of P that it is and
// written as aligned 16-byte chunks.
bool qk_flat_supported(int64_t BH, int64_t N, int64_t d);
hipError_t launch_qk_flat(bool scores_only, const void* Q, const void* K, void* out, int64_t BH, int64_t N, int64_t d,
                          float scale, hipStream_t stream);

// Fused attention weights or scaled scores, bf16, N <= 128, d a multiple of 16 up to 128, many heads: a wave per
// (head, 32 queries) with the K of the head as matrix operands in its registers, no LDS but the way out, no barriers.
bool qk_tiny_supported(int64_t BH, int64_t N, int64_t d);
hipError_t launch_qk_tiny(bool scores_only, const void* Q, const void* K, void* out, int64_t BH, int64_t N, int64_t d,
                          float scale, hipStream_t stream);

// Fused attention weights, bf16, d = 64 or 128, N a multiple of 512 from 1024 to 16384: the scores of a strip stay
// in the registers of the N / 512 workgroups that share its rows (one sweep over the keys; the workgroups exchange
// their row statistics through tables parked in P).  Two launches: table slots zeroed, then the kernel.
bool qk_gang_supported(int64_t BH, int64_t N, int64_t d);
hipError_t launch_qk_gang(const void* Q, const void* K, void* out, int64_t BH, int64_t N, int64_t d, float scale,
                          hipStream_t stream);

// Y = scale * X over count elements, rounded once to the storage type; X == Y allowed.
hipError_t launch_scale(DType dt, const void* X, void* Y, int64_t count, float scale, hipStream_t stream);

// Attention output O = softmax(scale Q K^T) V, bf16, d a multiple of 16 up to 128, any N >= 1 (tiled through LDS).
bool attention_supported(int64_t BH, int64_t N, int64_t d);
hipError_t launch_attention(const void* Q, const void* K, const void* V, void* O, int64_t BH, int64_t N, int64_t d,
                            float scale, hipStream_t stream);

// The same for fp32 (d a multiple of 4 up to 256, contractions on the fp32 matrix instruction) and for bf16 head sizes
// up to 256: one wave per 32 queries, operands straight from global memory.
bool attention_general_supported(DType dt, int64_t BH, int64_t N, int64_t d);
hipError_t launch_attention_general(DType dt, const void* Q, const void* K, const void* V, void* O, int64_t BH, int64_t N,
                                    int64_t d, float scale, hipStream_t stream);

// The same for many short sequences (bf16, d = 64 with N <= 128, d = 32 with N <= 224): a wave per (head, 32 queries), operands
// straight from global memory, the exponentials as they stand the operand of the second contraction.
bool attention_tiny_supported(int64_t BH, int64_t N, int64_t d);
bool prefers_attention_tiny(int64_t BH, int64_t N, int64_t d);
hipError_t launch_attention_tiny(const void* Q, const void* K, const void* V, void* O, int64_t BH, int64_t N, int64_t d,
                                 float scale, hipStream_t stream);

}  // namespace attnw
