// Fused attention weights  P = softmax(scale * Q K^T)  and, from the same tiling,
// the stand-alone scaled-score GEMM of the unfused pair.
//
// The paper's fused kernel (section "Fused Matrix Multiply + Scaling + Softmax")
// leaves a block of scores in each core's SRAM after the matrix multiply, scales
// it, reduces row maxima and row sums across the cores that share a row, and
// writes only the attention weights to DRAM.  On one MI355X compute unit a strip
// of BM query rows times all N keys does not fit on chip for the sizes of
// interest, so this kernel walks the keys twice instead: pass one multiplies a
// K tile (staged in LDS) with the strip's Q fragments (held in registers) on the
// matrix cores and folds the scores into a running row maximum and row sum
// (Softmax section, Eq. 1); pass two recomputes the same scores, turns them into
// weights with one fused multiply-add and one 2^x per element, rounds once and
// streams them to HBM.  Scores never leave the registers.
//
// Orientation: the MFMA computes the TRANSPOSED tile  (K tile) * (Q strip)^T, so
// that a lane's 16 accumulators are 16 keys of ONE query: row reductions stay
// inside the lane (plus one exchange between lanes l and l+32 at the end of pass
// one) and every lane owns runs of 4 consecutive keys for the store.
#include "device_utils.h"
#include "launchers.h"

namespace attnw {
namespace {

template <typename T> struct Mma;

// bf16: one 16-byte chunk holds 8 consecutive d-elements; lanes 0..31 carry chunk
// 2g, lanes 32..63 chunk 2g+1 of a 32-byte group = the k = 16 of one instruction.
template <> struct Mma<uint16_t> {
    static __device__ __forceinline__ void run(f32x16& acc, const u32x4& a, const u32x4& b)
    {
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b),
                                                      acc, 0, 0, 0);
    }
    static constexpr uint32_t kSignMask = 0x80008000u;
};

// fp32: a chunk holds 4 floats; the 32-byte group (8 floats) is contracted by four
// 32x32x2 instructions, instruction i taking floats i (lanes 0..31) and 4+i (lanes
// 32..63).  Any pairing is valid as long as both operands use the same one.
template <> struct Mma<float> {
    static __device__ __forceinline__ void run(f32x16& acc, const u32x4& a, const u32x4& b)
    {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a[i]), __uint_as_float(b[i]), acc, 0, 0, 0);
    }
    static constexpr uint32_t kSignMask = 0x80000000u;
};

// T      element type (uint16_t = bf16 bits, float)
// DB     padded bytes of one Q/K row held on chip (power of two, >= d * sizeof(T))
// BN     keys per LDS tile
// QB     32-query blocks per wave (a workgroup of 4 waves owns BM = 128 * QB queries)
// SCORES true: write scale * Q K^T (one pass); false: write the attention weights
template <typename T, int DB, int BN, int QB, bool SCORES>
__global__ __launch_bounds__(256, 2)
void qk_kernel(const T* __restrict__ Q, const T* __restrict__ K, T* __restrict__ out,
               int N, int d, float c, uint32_t sign_flip, uint32_t strips, uint32_t total_tiles)
{
    constexpr int ES = sizeof(T);
    constexpr int EPC = 16 / ES;              // elements per 16-byte chunk
    constexpr int QW = 32 * QB;               // queries per wave
    constexpr int BM = 4 * QW;                // queries per workgroup
    constexpr int G = DB / 32;                // 32-byte contraction groups per row
    constexpr int CPR = DB / 16;              // chunks per K row in LDS
    constexpr int KT = BN / 32;               // 32-key sub-tiles per K tile
    constexpr int K_TILE_BYTES = BN * DB;
    constexpr int LPT = BN * CPR / 256;       // K chunks each thread stages per tile
    constexpr int ST_PITCH = BN * ES + 16;    // staging row pitch (padded against bank conflicts)
    constexpr int ST_BYTES = QW * ST_PITCH;
    constexpr int CPS = BN * ES / 16;         // chunks per staging row
    constexpr int RPI = 64 / CPS;             // staging rows one store instruction covers
    constexpr int RPL = CPR >= 16 ? 1 : 16 / CPR;           // K rows per 256-byte LDS line
    constexpr int SWZ_MASK = (CPR >= 16 ? 16 : CPR) - 1;
    static_assert(BN % 32 == 0 && (BN * CPR) % 256 == 0 && CPS <= 64 && QW % RPI == 0, "tile shape");

    __shared__ __align__(16) char smem[2 * K_TILE_BYTES + 4 * ST_BYTES];

    const uint32_t logical = xcd_contiguous_block_id(blockIdx.x, gridDim.x);
    if (logical >= total_tiles) return;
    const uint32_t bh = logical / strips;
    const uint32_t strip = logical - bh * strips;

    const int tid = threadIdx.x;
    const int wave = tid >> 6;
    const int lane = tid & 63;
    const int l32 = lane & 31;
    const int half = lane >> 5;

    const int cpr_act = d * ES / 16;          // chunks of real data per row
    const int64_t row_bytes = (int64_t)d * ES;
    const char* Qh = reinterpret_cast<const char*>(Q) + (int64_t)bh * N * row_bytes;
    const char* Kh = reinterpret_cast<const char*>(K) + (int64_t)bh * N * row_bytes;
    T* out_h = out + (int64_t)bh * N * N;
    const int qw0 = strip * BM + wave * QW;   // first query of this wave

    char* const stage = smem + 2 * K_TILE_BYTES + wave * ST_BYTES;

    // ---- Q fragments: registers for the whole kernel --------------------------------
    u32x4 qf[QB][G];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const int q = qw0 + qb * 32 + l32;
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const int cq = 2 * g + half;
            u32x4 v = {0u, 0u, 0u, 0u};
            if (q < N && cq < cpr_act) v = *reinterpret_cast<const u32x4*>(Qh + (int64_t)q * row_bytes + cq * 16);
            qf[qb][g] = v ^ sign_flip;        // negative scale: softmax(-|c| s) = softmax(|c| (-Q) K^T)
        }
    }

    // ---- K tile staging ----------------------------------------------------------------
    const int n_tiles = (N + BN - 1) / BN;
    u32x4 kreg[LPT];
    auto k_fetch = [&](int tile) {
        const int k0 = tile * BN;
#pragma unroll
        for (int j = 0; j < LPT; ++j) {
            const int ci = tid + 256 * j;
            const int key = ci / CPR, ch = ci % CPR;
            u32x4 v = {0u, 0u, 0u, 0u};
            if (k0 + key < N && ch < cpr_act)
                v = *reinterpret_cast<const u32x4*>(Kh + (int64_t)(k0 + key) * row_bytes + ch * 16);
            kreg[j] = v;
        }
    };
    auto k_commit = [&](int buf) {
        char* base = smem + buf * K_TILE_BYTES;
#pragma unroll
        for (int j = 0; j < LPT; ++j) {
            const int ci = tid + 256 * j;
            const int key = ci / CPR, ch = ci % CPR;
            const int sw = ch ^ ((key / RPL) & SWZ_MASK);
            *reinterpret_cast<u32x4*>(base + key * DB + sw * 16) = kreg[j];
        }
    };

    // scores of sub-tile kt of the tile in `buf`: acc[qb][r] = q . k for key
    // kt*32 + 8*(r/4) + 4*half + r%4 and query qb*32 + l32
    auto mma_subtile = [&](int buf, int kt, f32x16 (&acc)[QB]) {
        const char* base = smem + buf * K_TILE_BYTES;
        const int key = kt * 32 + l32;
        const char* rowp = base + key * DB;
        const int swz = (key / RPL) & SWZ_MASK;
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[qb][r] = 0.0f;
#pragma unroll
        for (int g = 0; g < G; ++g) {
            if (2 * g < cpr_act) {            // wave-uniform: skip the zero padding of short rows
                const u32x4 a = *reinterpret_cast<const u32x4*>(rowp + (((2 * g + half) ^ swz) * 16));
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) Mma<T>::run(acc[qb], a, qf[qb][g]);
            }
        }
    };

    // move the wave's staged QW x BN block to global memory, 16 bytes per lane
    const bool vec_ok = (N % EPC) == 0;
    auto flush_stage = [&](int k0) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int it = 0; it < QW / RPI; ++it) {
            const int row = it * RPI + lane / CPS;
            const int ch = lane % CPS;
            const int q = qw0 + row;
            const int key0 = k0 + ch * EPC;
            const u32x4 v = *reinterpret_cast<const u32x4*>(stage + row * ST_PITCH + ch * 16);
            if (q < N && key0 < N) {
                T* dst = out_h + (int64_t)q * N + key0;
                if (vec_ok) {
                    __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(dst));
                } else {
                    const T* e = reinterpret_cast<const T*>(&v);
#pragma unroll
                    for (int i = 0; i < EPC; ++i)
                        if (key0 + i < N) dst[i] = e[i];
                }
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    };
    auto stage_put4 = [&](int qb, int kt, int r4, float v0, float v1, float v2, float v3) {
        char* p = stage + (qb * 32 + l32) * ST_PITCH + (kt * 32 + 8 * r4 + 4 * half) * ES;
        if constexpr (ES == 2) {
            u32x2 w = {pack_bf16x2(v0, v1), pack_bf16x2(v2, v3)};
            *reinterpret_cast<u32x2*>(p) = w;
        } else {
            u32x4 w = {__float_as_uint(v0), __float_as_uint(v1), __float_as_uint(v2), __float_as_uint(v3)};
            *reinterpret_cast<u32x4*>(p) = w;
        }
    };

    // ---- software pipeline over K tiles: fetch t+1 while computing t -------------------
    const int passes = SCORES ? 1 : 2;
    const int steps = passes * n_tiles;
    float m_run[QB], l_run[QB], bias[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) { m_run[qb] = kNegBig; l_run[qb] = 0.0f; bias[qb] = 0.0f; }

    k_fetch(0);
    k_commit(0);
    __syncthreads();

    for (int s = 0; s < steps; ++s) {
        const int tile = (s >= n_tiles) ? s - n_tiles : s;
        const bool second = s >= n_tiles;
        const int buf = s & 1;
        const int k0 = tile * BN;
        const bool tail = k0 + BN > N;
        if (s + 1 < steps) k_fetch((s + 1 >= n_tiles) ? s + 1 - n_tiles : s + 1);

#pragma unroll
        for (int kt = 0; kt < KT; ++kt) {
            if (k0 + kt * 32 >= N) break;     // uniform: nothing but padding left in this tile
            f32x16 acc[QB];
            mma_subtile(buf, kt, acc);
            const int kbase = k0 + kt * 32 + 4 * half;
            if constexpr (SCORES) {
#pragma unroll
                for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4)
                        stage_put4(qb, kt, r4, acc[qb][4 * r4] * c, acc[qb][4 * r4 + 1] * c,
                                   acc[qb][4 * r4 + 2] * c, acc[qb][4 * r4 + 3] * c);
            } else if (!second) {
                // pass one: running maximum and sum of exponentials (Eq. 1), per lane
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) {
                    if (tail) {
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            if (kbase + 8 * (r / 4) + (r % 4) >= N) acc[qb][r] = kNegBig;
                    }
                    float tm = max3(acc[qb][0], acc[qb][1], acc[qb][2]);
#pragma unroll
                    for (int r = 3; r < 15; r += 2) tm = max3(tm, acc[qb][r], acc[qb][r + 1]);
                    tm = fmaxf(tm, acc[qb][15]);
                    const float mn = fmaxf(m_run[qb], tm);
                    l_run[qb] *= fast_exp2((m_run[qb] - mn) * c);
                    m_run[qb] = mn;
                    const float mb = mn * c;
                    float sum = 0.0f;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        // fp32 results are held to an absolute bound: subtract first so
                        // that a large common offset cancels exactly
                        float e = (ES == 4) ? fast_exp2((acc[qb][r] - mn) * c)
                                            : fast_exp2(__builtin_fmaf(acc[qb][r], c, -mb));
                        if (tail && kbase + 8 * (r / 4) + (r % 4) >= N) e = 0.0f;
                        sum += e;
                    }
                    l_run[qb] += sum;
                }
            } else {
                // pass two: weights = 2^(c*s - bias), bias = c*m + log2(l)
#pragma unroll
                for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4) {
                        float p[4];
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            p[i] = (ES == 4) ? fast_exp2(__builtin_fmaf(acc[qb][4 * r4 + i] - m_run[qb], c, -bias[qb]))
                                             : fast_exp2(__builtin_fmaf(acc[qb][4 * r4 + i], c, -bias[qb]));
                        stage_put4(qb, kt, r4, p[0], p[1], p[2], p[3]);
                    }
            }
        }
        if (SCORES || second) flush_stage(k0);

        if (!SCORES && s == n_tiles - 1) {
            // lanes l and l+32 hold the two halves of each query's keys: merge them
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                const float mo = __shfl_xor(m_run[qb], 32, 64);
                const float lo = __shfl_xor(l_run[qb], 32, 64);
                const float mn = fmaxf(m_run[qb], mo);
                const float l = l_run[qb] * fast_exp2((m_run[qb] - mn) * c) + lo * fast_exp2((mo - mn) * c);
                m_run[qb] = mn;
                // bf16: bias = c*m + log2(l) folds max and normaliser into one constant;
                // fp32: the max is subtracted separately, bias = log2(l)
                bias[qb] = (ES == 4) ? fast_log2(l) : __builtin_fmaf(mn, c, fast_log2(l));
            }
        }

        if (s + 1 < steps) k_commit(buf ^ 1);
        __syncthreads();
    }
}

template <typename T, int DB, int BN, int QB>
hipError_t launch_shape(bool scores_only, const void* Q, const void* K, void* out, int64_t BH, int N, int d,
                        float scale, hipStream_t stream)
{
    constexpr int BM = 128 * QB;
    const uint32_t strips = (uint32_t)((N + BM - 1) / BM);
    const uint64_t total = (uint64_t)BH * strips;
    const uint32_t grid = (uint32_t)((total + 7) / 8 * 8);
    const T* q = static_cast<const T*>(Q);
    const T* k = static_cast<const T*>(K);
    T* o = static_cast<T*>(out);
    if (scores_only) {
        hipLaunchKernelGGL((qk_kernel<T, DB, BN, QB, true>), dim3(grid), dim3(256), 0, stream, q, k, o, N, d, scale, 0u,
                           strips, (uint32_t)total);
    } else {
        const float c = fabsf(scale) * kLog2e;
        const uint32_t flip = scale < 0.0f ? Mma<T>::kSignMask : 0u;
        hipLaunchKernelGGL((qk_kernel<T, DB, BN, QB, false>), dim3(grid), dim3(256), 0, stream, q, k, o, N, d, c, flip,
                           strips, (uint32_t)total);
    }
    return hipGetLastError();
}

template <typename T>
hipError_t launch_qk_t(bool scores_only, const void* Q, const void* K, void* out, int64_t BH, int N, int d,
                       float scale, hipStream_t stream)
{
    const int row_bytes = d * (int)sizeof(T);
    if (row_bytes <= 64) return launch_shape<T, 64, 64, 1>(scores_only, Q, K, out, BH, N, d, scale, stream);
    if (row_bytes <= 128) return launch_shape<T, 128, 64, 1>(scores_only, Q, K, out, BH, N, d, scale, stream);
    if (row_bytes <= 256) return launch_shape<T, 256, 64, 1>(scores_only, Q, K, out, BH, N, d, scale, stream);
    if (row_bytes <= 512) return launch_shape<T, 512, 32, 1>(scores_only, Q, K, out, BH, N, d, scale, stream);
    if constexpr (sizeof(T) == 4) return launch_shape<T, 1024, 32, 1>(scores_only, Q, K, out, BH, N, d, scale, stream);
    return hipErrorInvalidValue;   // unreachable: d <= 256 bounds row_bytes
}

}  // namespace

hipError_t launch_qk(DType dt, bool scores_only, const void* Q, const void* K, void* out,
                     int64_t BH, int64_t N, int64_t d, float scale, hipStream_t stream)
{
    if (dt == DType::F32) return launch_qk_t<float>(scores_only, Q, K, out, BH, (int)N, (int)d, scale, stream);
    return launch_qk_t<uint16_t>(scores_only, Q, K, out, BH, (int)N, (int)d, scale, stream);
}

}  // namespace attnw
