// Dedicated row softmax over precomputed scores (the paper's Softmax kernel:
// Softmax section, max-subtracted form of Eq. 1; its Grayskull version keeps one
// row of tiles resident in a core's SRAM and walks max -> subtract -> exp -> sum
// -> normalise).  Here a row lives in the registers of one wavefront (or of one
// workgroup for long rows): it is read from HBM once with 16-byte loads, reduced
// with cross-lane shuffles, and written once with 16-byte stores, so the kernel
// moves 2 * sizeof(T) bytes per element and nothing else.
#include "device_utils.h"
#include "launchers.h"

namespace attnw {
namespace {

template <typename T> struct Elem;

template <> struct Elem<float> {
    static constexpr int VEC = 4;   // elements per 16-byte chunk
    static __device__ __forceinline__ void unpack(const u32x4& v, float* x)
    {
#pragma unroll
        for (int i = 0; i < 4; ++i) x[i] = __uint_as_float(v[i]);
    }
    static __device__ __forceinline__ u32x4 pack(const float* x)
    {
        u32x4 v;
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = __float_as_uint(x[i]);
        return v;
    }
    static __device__ __forceinline__ float load1(const float* p) { return *p; }
    static __device__ __forceinline__ void store1(float* p, float v) { *p = v; }
};

template <> struct Elem<uint16_t> {   // bf16 bit patterns
    static constexpr int VEC = 8;
    static __device__ __forceinline__ void unpack(const u32x4& v, float* x)
    {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            x[2 * i] = bf16_lo_to_f32(v[i]);
            x[2 * i + 1] = bf16_hi_to_f32(v[i]);
        }
    }
    static __device__ __forceinline__ u32x4 pack(const float* x)
    {
        u32x4 v;
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = pack_bf16x2(x[2 * i], x[2 * i + 1]);
        return v;
    }
    static __device__ __forceinline__ float load1(const uint16_t* p) { return __uint_as_float((uint32_t)*p << 16); }
    static __device__ __forceinline__ void store1(uint16_t* p, float v) { *p = (uint16_t)(pack_bf16x2(v, 0.0f) & 0xffffu); }
};

// One row per TPR threads; every thread keeps R groups of E elements of the row in registers
// (E = the larger of the two types' elements per 16-byte chunk: a group is one chunk of the
// narrower type and one or two of the wider).  TPR == 64: four rows per 256-thread block,
// wave-local reductions only.  TPR > 64: one row per block, partial results meet in LDS.
// Requires cols to be a multiple of E (groups = cols / E <= R * TPR).
template <typename TI, typename TO, int R, int TPR>
__global__ __launch_bounds__(TPR == 64 ? 256 : TPR)
void softmax_rows_kernel(const TI* S, TO* P, int64_t rows, int groups)   // S == P (in place, TI == TO) is allowed
{
    constexpr int VI = Elem<TI>::VEC, VO = Elem<TO>::VEC;
    constexpr int E = VI > VO ? VI : VO;
    constexpr int CI = E / VI, CO = E / VO;     // 16-byte chunks per group on the way in / out
    constexpr int WAVES = (TPR == 64) ? 1 : TPR / 64;
    const int tid = (TPR == 64) ? (int)(threadIdx.x & 63) : (int)threadIdx.x;
    const int64_t row = (TPR == 64) ? (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6) : (int64_t)blockIdx.x;
    if (row >= rows) return;   // whole wave (TPR == 64) or whole block leaves together

    const u32x4* src = reinterpret_cast<const u32x4*>(S) + row * groups * CI;
    u32x4* dst = reinterpret_cast<u32x4*>(P) + row * groups * CO;

    u32x4 raw[R][CI];
#pragma unroll
    for (int k = 0; k < R; ++k) {
        const int c = tid + k * TPR;
        if (c < groups) {
#pragma unroll
            for (int j = 0; j < CI; ++j) raw[k][j] = __builtin_nontemporal_load(src + c * CI + j);
        }
    }

    float x[R][E];
    float m = -INFINITY;
#pragma unroll
    for (int k = 0; k < R; ++k) {
        const int c = tid + k * TPR;
        if (c < groups) {
#pragma unroll
            for (int j = 0; j < CI; ++j) Elem<TI>::unpack(raw[k][j], x[k] + j * VI);
        } else {
#pragma unroll
            for (int i = 0; i < E; ++i) x[k][i] = -INFINITY;
        }
#pragma unroll
        for (int i = 0; i < E; ++i) m = fmaxf(m, x[k][i]);
    }

    __shared__ float red[2][WAVES];
    m = wave_reduce_max(m);
    if constexpr (WAVES > 1) {
        if ((threadIdx.x & 63) == 0) red[0][threadIdx.x >> 6] = m;
        __syncthreads();
#pragma unroll
        for (int w = 0; w < WAVES; ++w) m = fmaxf(m, red[0][w]);
    }

    // e = exp(x - m) = 2^((x - m) * log2 e); the subtraction is done first so that
    // large common offsets cancel exactly.
    float l = 0.0f;
#pragma unroll
    for (int k = 0; k < R; ++k) {
#pragma unroll
        for (int i = 0; i < E; ++i) {
            x[k][i] = fast_exp2((x[k][i] - m) * kLog2e);
            l += x[k][i];
        }
    }
    l = wave_reduce_sum(l);
    if constexpr (WAVES > 1) {
        if ((threadIdx.x & 63) == 0) red[1][threadIdx.x >> 6] = l;
        __syncthreads();
        l = 0.0f;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) l += red[1][w];
    }
    const float inv = 1.0f / l;

#pragma unroll
    for (int k = 0; k < R; ++k) {
        const int c = tid + k * TPR;
        if (c < groups) {
#pragma unroll
            for (int i = 0; i < E; ++i) x[k][i] *= inv;
#pragma unroll
            for (int j = 0; j < CO; ++j) __builtin_nontemporal_store(Elem<TO>::pack(x[k] + j * VO), dst + c * CO + j);
        }
    }
}

// Any cols (ragged, unaligned rows, rows too long for registers): one row per
// 256-thread block, element-wise accesses, the row is read twice.
template <typename TI, typename TO>
__global__ __launch_bounds__(256)
void softmax_generic_kernel(const TI* S, TO* P, int64_t rows, int64_t cols)
{
    const int64_t row = blockIdx.x;
    if (row >= rows) return;
    const TI* src = S + row * cols;
    TO* dst = P + row * cols;

    // online (max, sum): after folding x, l = sum exp(x_k - m) over the k seen so far
    float m = kNegBig, l = 0.0f;
    for (int64_t j = threadIdx.x; j < cols; j += 256) {
        const float x = Elem<TI>::load1(src + j);
        const float mn = fmaxf(m, x);
        l = l * fast_exp2((m - mn) * kLog2e) + fast_exp2((x - mn) * kLog2e);
        m = mn;
    }
    // combine (m, l) pairs across the wave, then across the four waves
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const float mo = __shfl_xor(m, off, 64), lo = __shfl_xor(l, off, 64);
        const float mn = fmaxf(m, mo);
        l = l * fast_exp2((m - mn) * kLog2e) + lo * fast_exp2((mo - mn) * kLog2e);
        m = mn;
    }
    __shared__ float sm[4], sl[4];
    if ((threadIdx.x & 63) == 0) { sm[threadIdx.x >> 6] = m; sl[threadIdx.x >> 6] = l; }
    __syncthreads();   // also orders every read of pass one before any in-place write below
    m = fmaxf(fmaxf(sm[0], sm[1]), fmaxf(sm[2], sm[3]));
    l = 0.0f;
#pragma unroll
    for (int w = 0; w < 4; ++w) l += sl[w] * fast_exp2((sm[w] - m) * kLog2e);
    const float inv = 1.0f / l;
    for (int64_t j = threadIdx.x; j < cols; j += 256) {
        const float x = Elem<TI>::load1(src + j);
        Elem<TO>::store1(dst + j, fast_exp2((x - m) * kLog2e) * inv);
    }
}

template <typename TI, typename TO, int R, int TPR>
hipError_t launch_rows(const void* S, void* P, int64_t rows, int groups, hipStream_t stream)
{
    const int64_t blocks = (TPR == 64) ? (rows + 3) / 4 : rows;
    const int threads = (TPR == 64) ? 256 : TPR;
    hipLaunchKernelGGL((softmax_rows_kernel<TI, TO, R, TPR>), dim3((uint32_t)blocks), dim3(threads), 0, stream,
                       static_cast<const TI*>(S), static_cast<TO*>(P), rows, groups);
    return hipGetLastError();
}

template <typename TI, typename TO>
hipError_t launch_softmax_t(const void* S, void* P, int64_t rows, int64_t cols, hipStream_t stream)
{
    constexpr int E = Elem<TI>::VEC > Elem<TO>::VEC ? Elem<TI>::VEC : Elem<TO>::VEC;
    // Register-resident rows: up to 8 groups per thread when a group is 8 elements, 4 when both
    // types are fp32 (a thread's group is 8 resp. 4 fp32 values once unpacked).
    constexpr int MAXR = (E == 4) ? 4 : 8;
    if (cols % E == 0 && cols / E <= 1024 * MAXR) {
        const int groups = (int)(cols / E);
        if (groups <= 64) return launch_rows<TI, TO, 1, 64>(S, P, rows, groups, stream);
        if (groups <= 128) return launch_rows<TI, TO, 2, 64>(S, P, rows, groups, stream);
        if (groups <= 256) return launch_rows<TI, TO, 4, 64>(S, P, rows, groups, stream);
        if (groups <= 512) return launch_rows<TI, TO, 2, 256>(S, P, rows, groups, stream);
        if (groups <= 1024) return launch_rows<TI, TO, 4, 256>(S, P, rows, groups, stream);
        if (groups <= 2048) return launch_rows<TI, TO, 2, 1024>(S, P, rows, groups, stream);
        if (groups <= 4096) return launch_rows<TI, TO, 4, 1024>(S, P, rows, groups, stream);
        if constexpr (MAXR >= 8) return launch_rows<TI, TO, 8, 1024>(S, P, rows, groups, stream);
    }
    hipLaunchKernelGGL((softmax_generic_kernel<TI, TO>), dim3((uint32_t)rows), dim3(256), 0, stream,
                       static_cast<const TI*>(S), static_cast<TO*>(P), rows, cols);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_softmax(DType in, DType out, const void* S, void* P, int64_t rows, int64_t cols, hipStream_t stream)
{
    if (in == DType::F32)
        return out == DType::F32 ? launch_softmax_t<float, float>(S, P, rows, cols, stream)
                                 : launch_softmax_t<float, uint16_t>(S, P, rows, cols, stream);
    return out == DType::F32 ? launch_softmax_t<uint16_t, float>(S, P, rows, cols, stream)
                             : launch_softmax_t<uint16_t, uint16_t>(S, P, rows, cols, stream);
}

}  // namespace attnw
