// C ABI of libattnw (declared in include/attnw.h): argument validation on the
// host, then one kernel launch on the caller's stream.  No allocation, no
// synchronisation, no global mutable state.
#include "attnw.h"
#include "launchers.h"

#include <cstdlib>
#include <cstring>

#include <limits>

namespace {

constexpr int kVersion = 104;   // 0.1.4: major * 10000 + minor * 100 + patch; a patch step per entry point added since 0.1.0

bool mul_overflows(int64_t a, int64_t b, int64_t* out)
{
    return __builtin_mul_overflow(a, b, out);
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// half-open byte ranges [a, a+na) and [b, b+nb)
bool overlaps(const void* a, int64_t na, const void* b, int64_t nb)
{
    const uintptr_t a0 = reinterpret_cast<uintptr_t>(a), b0 = reinterpret_cast<uintptr_t>(b);
    return a0 < b0 + (uintptr_t)nb && b0 < a0 + (uintptr_t)na;
}

int elem_size(int dtype) { return dtype == ATTNW_F32 ? 4 : 2; }

// Shared by attnw_fused and attnw_gemm_scores: same arguments, same rules.
int run_qk(bool scores_only, const void* Q, const void* K, void* out, int64_t B, int64_t H, int64_t N, int64_t d,
           float scale, int dtype, void* stream)
{
    if (dtype != ATTNW_F32 && dtype != ATTNW_BF16) return ATTNW_ERR_DTYPE;
    if (B < 0 || H < 0 || N < 0 || d < 0) return ATTNW_ERR_SHAPE;
    if (B == 0 || H == 0 || N == 0) return ATTNW_OK;          // empty problem
    if (!Q || !K || !out) return ATTNW_ERR_NULL;
    int64_t BH, in_elems, out_elems, in_bytes, out_bytes;
    if (mul_overflows(B, H, &BH)) return ATTNW_ERR_SHAPE;
    if (mul_overflows(BH, N, &in_elems) || mul_overflows(in_elems, N, &out_elems) ||
        mul_overflows(in_elems, d, &in_elems))
        return ATTNW_ERR_SHAPE;
    const int es = elem_size(dtype);
    if (mul_overflows(in_elems, es, &in_bytes) || mul_overflows(out_elems, es, &out_bytes)) return ATTNW_ERR_SHAPE;
    // rows of Q and K are read as 16-byte chunks: 8 bf16 or 4 fp32 elements (bf16 additionally in whole
    // 32-byte contraction groups)
    const int64_t d_step = dtype == ATTNW_F32 ? 4 : 16;
    if (d < d_step || d > 256 || (d % d_step) != 0) return ATTNW_ERR_UNSUPPORTED;
    if (N > (int64_t)1 << 30) return ATTNW_ERR_UNSUPPORTED;
    // one workgroup per (head, strip of at least 64 queries), grid padded to a multiple of 8
    const int64_t strips = (N + 63) / 64;
    int64_t tiles;
    if (mul_overflows(BH, strips, &tiles) || tiles > (int64_t)std::numeric_limits<int32_t>::max() - 8)
        return ATTNW_ERR_UNSUPPORTED;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(out)) return ATTNW_ERR_ALIGN;
    if (overlaps(out, out_bytes, Q, in_bytes) || overlaps(out, out_bytes, K, in_bytes)) return ATTNW_ERR_ALIAS;

    const hipError_t e = attnw::launch_qk(static_cast<attnw::DType>(dtype), scores_only, Q, K, out, BH, N, d, scale,
                                          static_cast<hipStream_t>(stream));
    return e == hipSuccess ? ATTNW_OK : ATTNW_ERR_LAUNCH;
}

}  // namespace

extern "C" {

int attnw_fused(const void* Q, const void* K, void* P, int64_t B, int64_t H, int64_t N, int64_t d, float scale,
                int dtype, void* stream)
{
    return run_qk(false, Q, K, P, B, H, N, d, scale, dtype, stream);
}

int attnw_gemm_scores(const void* Q, const void* K, void* S, int64_t B, int64_t H, int64_t N, int64_t d, float scale,
                      int dtype, void* stream)
{
    return run_qk(true, Q, K, S, B, H, N, d, scale, dtype, stream);
}

int attnw_attention(const void* Q, const void* K, const void* V, void* O, int64_t B, int64_t H, int64_t N, int64_t d,
                    float scale, int dtype, void* stream)
{
    if (dtype != ATTNW_F32 && dtype != ATTNW_BF16) return ATTNW_ERR_DTYPE;
    if (B < 0 || H < 0 || N < 0 || d < 0) return ATTNW_ERR_SHAPE;
    if (B == 0 || H == 0 || N == 0) return ATTNW_OK;          // empty problem
    if (!Q || !K || !V || !O) return ATTNW_ERR_NULL;
    int64_t BH, elems, bytes;
    if (mul_overflows(B, H, &BH) || mul_overflows(BH, N, &elems) || mul_overflows(elems, d, &elems) ||
        mul_overflows(elems, elem_size(dtype), &bytes))
        return ATTNW_ERR_SHAPE;
    const attnw::DType dt = dtype == ATTNW_F32 ? attnw::DType::F32 : attnw::DType::BF16;
    const bool tiled = dtype == ATTNW_BF16 && attnw::attention_supported(BH, N, d);
    if (!tiled && !attnw::attention_general_supported(dt, BH, N, d)) return ATTNW_ERR_UNSUPPORTED;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O)) return ATTNW_ERR_ALIGN;
    if (overlaps(O, bytes, Q, bytes) || overlaps(O, bytes, K, bytes) || overlaps(O, bytes, V, bytes))
        return ATTNW_ERR_ALIAS;
    hipStream_t st = static_cast<hipStream_t>(stream);
    // many short sequences: the kernel in which a wave works alone on a (head, 32 queries) pair
    // (ATTNW_ATTENTION_KERNEL=tiny puts every shape it takes on it, =tiled none: tests and measurements compare them)
    if (dtype == ATTNW_BF16 && attnw::attention_tiny_supported(BH, N, d)) {
        const char* force = getenv("ATTNW_ATTENTION_KERNEL");
        const bool want = force ? strcmp(force, "tiny") == 0 : attnw::prefers_attention_tiny(BH, N, d);
        if (want) return attnw::launch_attention_tiny(Q, K, V, O, BH, N, d, scale, st) == hipSuccess ? ATTNW_OK : ATTNW_ERR_LAUNCH;
    }
    const hipError_t e = tiled ? attnw::launch_attention(Q, K, V, O, BH, N, d, scale, st)
                               : attnw::launch_attention_general(dt, Q, K, V, O, BH, N, d, scale, st);
    return e == hipSuccess ? ATTNW_OK : ATTNW_ERR_LAUNCH;
}

// Shared by attnw_softmax and attnw_softmax_cast.
static int run_softmax(const void* S, void* P, int64_t rows, int64_t cols, int in_dtype, int out_dtype, void* stream)
{
    if (in_dtype != ATTNW_F32 && in_dtype != ATTNW_BF16) return ATTNW_ERR_DTYPE;
    if (out_dtype != ATTNW_F32 && out_dtype != ATTNW_BF16) return ATTNW_ERR_DTYPE;
    if (rows < 0 || cols < 0) return ATTNW_ERR_SHAPE;
    if (rows == 0 || cols == 0) return ATTNW_OK;              // empty problem
    if (!S || !P) return ATTNW_ERR_NULL;
    int64_t elems, in_bytes, out_bytes;
    if (mul_overflows(rows, cols, &elems) || mul_overflows(elems, elem_size(in_dtype), &in_bytes) ||
        mul_overflows(elems, elem_size(out_dtype), &out_bytes))
        return ATTNW_ERR_SHAPE;
    // one workgroup per row (or per four rows): the grid's x extent is 32-bit
    if (rows > (int64_t)std::numeric_limits<int32_t>::max()) return ATTNW_ERR_UNSUPPORTED;
    if (!aligned16(S) || !aligned16(P)) return ATTNW_ERR_ALIGN;
    // in place only when every element is read and written at the same address
    if (!(S == P && in_dtype == out_dtype) && overlaps(P, out_bytes, S, in_bytes)) return ATTNW_ERR_ALIAS;

    const hipError_t e = attnw::launch_softmax(static_cast<attnw::DType>(in_dtype), static_cast<attnw::DType>(out_dtype),
                                               S, P, rows, cols, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? ATTNW_OK : ATTNW_ERR_LAUNCH;
}

int attnw_softmax(const void* S, void* P, int64_t rows, int64_t cols, int dtype, void* stream)
{
    return run_softmax(S, P, rows, cols, dtype, dtype, stream);
}

int attnw_softmax_cast(const void* S, void* P, int64_t rows, int64_t cols, int in_dtype, int out_dtype, void* stream)
{
    return run_softmax(S, P, rows, cols, in_dtype, out_dtype, stream);
}

int attnw_scale(const void* X, void* Y, int64_t count, float scale, int dtype, void* stream)
{
    if (dtype != ATTNW_F32 && dtype != ATTNW_BF16) return ATTNW_ERR_DTYPE;
    if (count < 0) return ATTNW_ERR_SHAPE;
    if (count == 0) return ATTNW_OK;                          // empty problem
    if (!X || !Y) return ATTNW_ERR_NULL;
    int64_t bytes;
    if (mul_overflows(count, elem_size(dtype), &bytes)) return ATTNW_ERR_SHAPE;
    if (!aligned16(X) || !aligned16(Y)) return ATTNW_ERR_ALIGN;
    if (X != Y && overlaps(Y, bytes, X, bytes)) return ATTNW_ERR_ALIAS;
    const hipError_t e = attnw::launch_scale(static_cast<attnw::DType>(dtype), X, Y, count, scale,
                                             static_cast<hipStream_t>(stream));
    return e == hipSuccess ? ATTNW_OK : ATTNW_ERR_LAUNCH;
}

const char* attnw_status_string(int status)
{
    switch (status) {
    case ATTNW_OK: return "ok";
    case ATTNW_ERR_NULL: return "null pointer";
    case ATTNW_ERR_SHAPE: return "bad shape (negative dimension or size overflow)";
    case ATTNW_ERR_DTYPE: return "unknown dtype";
    case ATTNW_ERR_UNSUPPORTED:
        return "unsupported dtype / head size / extent for this entry point (limits are listed per call in attnw.h)";
    case ATTNW_ERR_ALIGN: return "pointer not 16-byte aligned";
    case ATTNW_ERR_ALIAS: return "output overlaps an input";
    case ATTNW_ERR_LAUNCH: return "kernel launch failed";
    default: return "unknown status";
    }
}

int attnw_version(void) { return kVersion; }

}  // extern "C"
