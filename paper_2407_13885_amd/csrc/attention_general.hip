// Attention output  O = softmax(scale * Q K^T) V  for the element types and head sizes that the tiled
// bf16 kernel does not take: fp32 (d a multiple of 4 up to 256) and bf16 with 128 < d <= 256.
//
// (Paper: Multi-Head Self-Attention section, Attention(Q, K, V) = softmax(Q K^T / sqrt(d_k)) V; the product
// with V is what the section "Limitations and future Directions" names as the next thing to fuse.  The
// max-subtracted softmax of the Softmax section, Eq. 1, is applied incrementally as in the tiled kernel.)
//
// One wave per workgroup, 32 queries per wave, every wave walks all keys in sub-tiles of 32: no shared
// memory, no barriers, nothing crosses waves.  Operands come straight from global memory (K and V of a
// head are read by all the waves of the head: they live in the caches), which makes every row clamp and
// every padding a matter of the load's address or of a zero in its place.
//   S^T = K_sub * Q^T      on the matrix instruction of the element type (fp32: v_mfma_f32_32x32x2_f32, so
//                          the scores have fp32 products and sums; bf16: v_mfma_f32_32x32x16_bf16);
//                          lane (query l32, half h) holds keys 8i + 4h + j of its query.
//   p = 2^(c s - ref), running sum, reference exponent that follows the running maximum lazily.
//   O^T += V_sub^T * P^T   fp32: one v_mfma_f32_32x32x2_f32 per accumulator r -- it contracts the key pair
//                          (8(r/4) + r%4, 8(r/4) + 4 + r%4), whose weights ARE accumulator r of the two
//                          half-waves, against one float of V per lane (row = the key of the lane's half,
//                          column = 32b + l32): fp32 weights, fp32 products, no rounding before the store.
//                          bf16: as in the tiled kernel (weights rounded to bf16, 16 keys per instruction,
//                          the lane's 8 weights are its operand), the 8 values of V gathered by 2-byte loads.
#include "launchers.h"
#include "qk_common.h"

namespace attnw {
namespace {

__device__ __forceinline__ float half_max_g(float x)
{
#if defined(__HIP_DEVICE_COMPILE__)
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
#else
    return x;
#endif
}
__device__ __forceinline__ float half_sum_g(float x)
{
#if defined(__HIP_DEVICE_COMPILE__)
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
#else
    return x;
#endif
}

constexpr int largest_divisor_up_to_8(int n)
{
    int best = 1;
    for (int k = 2; k <= 8; ++k)
        if (n % k == 0) best = k;
    return best;
}

// DVB: 32-column blocks of an output row, ceil(d / 32); rows are handled as if they had 32 DVB elements (rb: bytes
// of a row in memory).  Every load is unconditional at a clamped address and replaced by zero afterwards where it
// lies past the end of the row -- loads under a branch would be waited for one by one -- and the loads of a batch
// (8 contraction groups of K, 4 keys of V) are issued together ahead of the matrix instructions that use them.
template <typename T, int DVB>
__global__ __launch_bounds__(64)
void attention_general_kernel(const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V, T* __restrict__ O,
                              int N, int rb, float c, uint32_t sign_flip, uint32_t strips, uint32_t total)
{
    constexpr int E = (int)sizeof(T);
    constexpr int G = DVB * E;                    // 32-byte contraction groups of a padded row (32 DVB elements)
    constexpr int GB = largest_divisor_up_to_8(G);   // groups per batch of loads
    constexpr bool QRES = G <= 8;                 // Q fragments stay in registers (else they are re-read per sub-tile)
    static_assert(DVB >= 1 && DVB <= 8 && G % GB == 0, "output accumulators: at most 128 registers");

    const uint32_t logical = xcd_contiguous_block_id(blockIdx.x, gridDim.x);
    if (logical >= total) return;
    const uint32_t bh = logical / strips;
    const uint32_t strip = logical - bh * strips;
    const int lane = threadIdx.x & 63;
    const int l32 = lane & 31;
    const int half = lane >> 5;
    const int d = rb / E;
    const int last_chunk = rb / 16 - 1;

    const char* Qh = reinterpret_cast<const char*>(Q) + (int64_t)bh * N * rb;
    const char* Kh = reinterpret_cast<const char*>(K) + (int64_t)bh * N * rb;
    const char* Vh = reinterpret_cast<const char*>(V) + (int64_t)bh * N * rb;
    char* Oh = reinterpret_cast<char*>(O) + (int64_t)bh * N * rb;
    const int q0 = strip * 32;
    auto row_in = [&](int r) __attribute__((always_inline)) { return min(r, N - 1); };   // every load stays inside the arrays

    // chunk 2g + half of a row (the k-range of the lane's half-wave in group g), zeros past the end of the row
    auto frag = [&](const char* row, int g) __attribute__((always_inline)) {
        const int ch = 2 * g + half;
        const u32x4 v = *reinterpret_cast<const u32x4*>(row + min(ch, last_chunk) * 16);
        return ch <= last_chunk ? v : u32x4{0u, 0u, 0u, 0u};
    };
    const char* qrow = Qh + (int64_t)row_in(q0 + l32) * rb;
    u32x4 qf[QRES ? G : 1];
    if constexpr (QRES) {
#pragma unroll
        for (int g = 0; g < G; ++g) qf[g] = frag(qrow, g) ^ sign_flip;
    }
    // the lane's column of every output block, clamped for the loads of V
    int vcol[DVB];
#pragma unroll
    for (int b = 0; b < DVB; ++b) vcol[b] = min(b * 32 + l32, d - 1) * E;

    f32x16 oacc[DVB];
#pragma unroll
    for (int b = 0; b < DVB; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[b][r] = 0.0f;
    float mb_run = kNegBig, l_run = 0.0f;
    constexpr float kLazy = 8.0f;                 // binades the maximum may run ahead of the reference exponent

    for (int key0 = 0; key0 < N; key0 += 32) {
        // ---- scores of 32 keys ---------------------------------------------------------------------------------
        f32x16 s;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = 0.0f;
        const char* krow = Kh + (int64_t)row_in(key0 + l32) * rb;
#pragma unroll
        for (int gb = 0; gb < G; gb += GB) {
            u32x4 kf[GB], qq[QRES ? 1 : GB];
#pragma unroll
            for (int g = 0; g < GB; ++g) {
                kf[g] = frag(krow, gb + g);
                if constexpr (!QRES) qq[g] = frag(qrow, gb + g) ^ sign_flip;
            }
#pragma unroll
            for (int g = 0; g < GB; ++g) {
                if constexpr (QRES) Mma<T>::run(s, kf[g], qf[gb + g]);
                else Mma<T>::run(s, kf[g], qq[g]);
            }
        }
        // ---- weights -------------------------------------------------------------------------------------------
        float tm = max3(s[0], s[1], s[2]);
#pragma unroll
        for (int r = 3; r < 15; r += 2) tm = max3(tm, s[r], s[r + 1]);
        const float mbn = half_max_g(fmaxf(tm, s[15])) * c;   // (keys past the end are copies of key N-1: no new maximum)
        if (__builtin_amdgcn_ballot_w64(mbn > mb_run + kLazy) != 0) {
            const float mb_new = fmaxf(mb_run, mbn);
            const float alpha = fast_exp2(mb_run - mb_new);   // exactly 1 for lanes whose exponent stands
            l_run *= alpha;
#pragma unroll
            for (int b = 0; b < DVB; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[b][r] *= alpha;
            mb_run = mb_new;
        }
        float p[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            p[r] = fast_exp2(__builtin_fmaf(s[r], c, -mb_run));
            // last sub-tile of a ragged length: keys past the end weigh nothing
            if (key0 + 4 * half + 8 * (r / 4) + (r % 4) >= N) p[r] = 0.0f;
        }
        float sum = p[0];
#pragma unroll
        for (int r = 1; r < 16; ++r) sum += p[r];
        l_run += sum;
        // ---- output accumulators -----------------------------------------------------------------------------------
        if constexpr (E == 4) {
            // accumulator r is the weight of key 8 (r / 4) + 4 half + r % 4: four keys (one r / 4) per batch
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                float vv[4][DVB];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const char* vrow = Vh + (int64_t)row_in(key0 + 8 * r4 + 4 * half + j) * rb;
#pragma unroll
                    for (int b = 0; b < DVB; ++b) {
                        const float v = *reinterpret_cast<const float*>(vrow + vcol[b]);
                        vv[j][b] = b * 32 + l32 < d ? v : 0.0f;
                    }
                }
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int b = 0; b < DVB; ++b)
                        oacc[b] = __builtin_amdgcn_mfma_f32_32x32x2f32(vv[j][b], p[4 * r4 + j], oacc[b], 0, 0, 0);
            }
        } else {
#pragma unroll
            for (int m = 0; m < 2; ++m) {
                u32x4 pw;
#pragma unroll
                for (int i = 0; i < 4; ++i) pw[i] = pack_bf16x2(p[8 * m + 2 * i], p[8 * m + 2 * i + 1]);
                // operand slot e of the lane <-> key 16m + 8 (e / 4) + 4 half + e % 4 (the key of accumulator 8m + e)
                u32x4 vf[DVB];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int e = 2 * i;
                    const char* vlo = Vh + (int64_t)row_in(key0 + 16 * m + 8 * (e / 4) + 4 * half + (e % 4)) * rb;
                    const char* vhi = Vh + (int64_t)row_in(key0 + 16 * m + 8 * (e / 4) + 4 * half + (e % 4) + 1) * rb;
#pragma unroll
                    for (int b = 0; b < DVB; ++b) {
                        const uint32_t lo = *reinterpret_cast<const uint16_t*>(vlo + vcol[b]);
                        const uint32_t hi = *reinterpret_cast<const uint16_t*>(vhi + vcol[b]);
                        vf[b][i] = b * 32 + l32 < d ? (lo | (hi << 16)) : 0u;
                    }
                }
#pragma unroll
                for (int b = 0; b < DVB; ++b) Mma<uint16_t>::run(oacc[b], vf[b], pw);
            }
        }
    }

    // ---- normalise, round once (bf16), store: a lane owns runs of 4 consecutive output columns of its query ----
    const float inv = 1.0f / half_sum_g(l_run);
    if (q0 + l32 >= N) return;
    char* orow = Oh + (int64_t)(q0 + l32) * rb;
#pragma unroll
    for (int b = 0; b < DVB; ++b)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int col = b * 32 + 8 * i + 4 * half;   // d is a multiple of 4: the run lies inside the row or past it
            if (col < d) {
                if constexpr (E == 4) {
                    f32x4 w = {oacc[b][4 * i] * inv, oacc[b][4 * i + 1] * inv, oacc[b][4 * i + 2] * inv, oacc[b][4 * i + 3] * inv};
                    *reinterpret_cast<f32x4*>(orow + col * 4) = w;
                } else {
                    u32x2 w = {pack_bf16x2(oacc[b][4 * i] * inv, oacc[b][4 * i + 1] * inv),
                               pack_bf16x2(oacc[b][4 * i + 2] * inv, oacc[b][4 * i + 3] * inv)};
                    *reinterpret_cast<u32x2*>(orow + col * 2) = w;
                }
            }
        }
}

template <typename T, int DVB>
hipError_t launch_general_t(const void* Q, const void* K, const void* V, void* O, int64_t BH, int N, int d, float scale,
                            hipStream_t stream)
{
    const uint32_t strips = (uint32_t)((N + 31) / 32);
    const uint64_t total = (uint64_t)BH * strips;
    const uint32_t grid = (uint32_t)((total + 7) / 8 * 8);
    const float c = fabsf(scale) * kLog2e;
    const uint32_t flip = scale < 0.0f ? Mma<T>::kSignMask : 0u;
    hipLaunchKernelGGL((attention_general_kernel<T, DVB>), dim3(grid), dim3(64), 0, stream, static_cast<const T*>(Q),
                       static_cast<const T*>(K), static_cast<const T*>(V), static_cast<T*>(O), N, d * (int)sizeof(T), c,
                       flip, strips, (uint32_t)total);
    return hipGetLastError();
}

template <typename T>
hipError_t launch_general_blocks(int blocks, const void* Q, const void* K, const void* V, void* O, int64_t BH, int N, int d,
                                 float scale, hipStream_t stream)
{
    switch (blocks) {
    case 1: return launch_general_t<T, 1>(Q, K, V, O, BH, N, d, scale, stream);
    case 2: return launch_general_t<T, 2>(Q, K, V, O, BH, N, d, scale, stream);
    case 3: return launch_general_t<T, 3>(Q, K, V, O, BH, N, d, scale, stream);
    case 4: return launch_general_t<T, 4>(Q, K, V, O, BH, N, d, scale, stream);
    case 5: return launch_general_t<T, 5>(Q, K, V, O, BH, N, d, scale, stream);
    case 6: return launch_general_t<T, 6>(Q, K, V, O, BH, N, d, scale, stream);
    case 7: return launch_general_t<T, 7>(Q, K, V, O, BH, N, d, scale, stream);
    case 8: return launch_general_t<T, 8>(Q, K, V, O, BH, N, d, scale, stream);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace

bool attention_general_supported(DType dt, int64_t BH, int64_t N, int64_t d)
{
    const int64_t step = dt == DType::F32 ? 4 : 16;
    if (d < step || d > 256 || (d % step) != 0) return false;
    if (N < 1 || N > ((int64_t)1 << 24)) return false;
    return BH * ((N + 31) / 32) <= (int64_t)0x7ffffff0;
}

hipError_t launch_attention_general(DType dt, const void* Q, const void* K, const void* V, void* O, int64_t BH, int64_t N,
                                    int64_t d, float scale, hipStream_t stream)
{
    const int blocks = (int)((d + 31) / 32);
    if (dt == DType::F32) return launch_general_blocks<float>(blocks, Q, K, V, O, BH, (int)N, (int)d, scale, stream);
    return launch_general_blocks<uint16_t>(blocks, Q, K, V, O, BH, (int)N, (int)d, scale, stream);
}

}  // namespace attnw
