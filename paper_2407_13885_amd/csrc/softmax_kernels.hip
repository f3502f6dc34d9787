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

// One row per TPR threads; every thread keeps R 16-byte chunks of the row in
// registers.  TPR == 64: four rows per 256-thread block, wave-local reductions
// only.  TPR > 64: one row per block, partial results meet in LDS.
// Requires cols to be a multiple of VEC (chunks = cols / VEC <= R * TPR).
template <typename T, int R, int TPR>
__global__ __launch_bounds__(TPR == 64 ? 256 : TPR)
void softmax_rows_kernel(const T* S, T* P, int64_t rows, int chunks)   // S == P (in place) is allowed
{
    constexpr int VEC = Elem<T>::VEC;
    constexpr int WAVES = (TPR == 64) ? 1 : TPR / 64;
    const int tid = (TPR == 64) ? (int)(threadIdx.x & 63) : (int)threadIdx.x;
    const int64_t row = (TPR == 64) ? (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6) : (int64_t)blockIdx.x;
    if (row >= rows) return;   // whole wave (TPR == 64) or whole block leaves together

    const u32x4* src = reinterpret_cast<const u32x4*>(S) + row * chunks;
    u32x4* dst = reinterpret_cast<u32x4*>(P) + row * chunks;

    u32x4 raw[R];
#pragma unroll
    for (int k = 0; k < R; ++k) {
        const int c = tid + k * TPR;
        if (c < chunks) raw[k] = __builtin_nontemporal_load(src + c);
    }

    float x[R][VEC];
    float m = -INFINITY;
#pragma unroll
    for (int k = 0; k < R; ++k) {
        const int c = tid + k * TPR;
        if (c < chunks) {
            Elem<T>::unpack(raw[k], x[k]);
        } else {
#pragma unroll
            for (int i = 0; i < VEC; ++i) x[k][i] = -INFINITY;
        }
#pragma unroll
        for (int i = 0; i < VEC; ++i) m = fmaxf(m, x[k][i]);
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
        for (int i = 0; i < VEC; ++i) {
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
        if (c < chunks) {
#pragma unroll
            for (int i = 0; i < VEC; ++i) x[k][i] *= inv;
            __builtin_nontemporal_store(Elem<T>::pack(x[k]), dst + c);
        }
    }
}

// Any cols (ragged, unaligned rows, rows too long for registers): one row per
// 256-thread block, element-wise accesses, the row is read twice.
template <typename T>
__global__ __launch_bounds__(256)
void softmax_generic_kernel(const T* S, T* P, int64_t rows, int64_t cols)
{
    const int64_t row = blockIdx.x;
    if (row >= rows) return;
    const T* src = S + row * cols;
    T* dst = P + row * cols;

    // online (max, sum): after folding x, l = sum exp(x_k - m) over the k seen so far
    float m = kNegBig, l = 0.0f;
    for (int64_t j = threadIdx.x; j < cols; j += 256) {
        const float x = Elem<T>::load1(src + j);
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
        const float x = Elem<T>::load1(src + j);
        Elem<T>::store1(dst + j, fast_exp2((x - m) * kLog2e) * inv);
    }
}

template <typename T, int R, int TPR>
hipError_t launch_rows(const void* S, void* P, int64_t rows, int chunks, hipStream_t stream)
{
    const int64_t blocks = (TPR == 64) ? (rows + 3) / 4 : rows;
    const int threads = (TPR == 64) ? 256 : TPR;
    hipLaunchKernelGGL((softmax_rows_kernel<T, R, TPR>), dim3((uint32_t)blocks), dim3(threads), 0, stream,
                       static_cast<const T*>(S), static_cast<T*>(P), rows, chunks);
    return hipGetLastError();
}

template <typename T>
hipError_t launch_softmax_t(const void* S, void* P, int64_t rows, int64_t cols, hipStream_t stream)
{
    constexpr int VEC = Elem<T>::VEC;
    // Register-resident rows: up to 8 chunks per thread for bf16, 4 for fp32 (a
    // thread's chunk is 8 resp. 4 fp32 values once unpacked).
    constexpr int MAXR = (sizeof(T) == 4) ? 4 : 8;
    if (cols % VEC == 0 && cols / VEC <= 1024 * MAXR) {
        const int chunks = (int)(cols / VEC);
        if (chunks <= 64) return launch_rows<T, 1, 64>(S, P, rows, chunks, stream);
        if (chunks <= 128) return launch_rows<T, 2, 64>(S, P, rows, chunks, stream);
        if (chunks <= 256) return launch_rows<T, 4, 64>(S, P, rows, chunks, stream);
        if (chunks <= 512) return launch_rows<T, 2, 256>(S, P, rows, chunks, stream);
        if (chunks <= 1024) return launch_rows<T, 4, 256>(S, P, rows, chunks, stream);
        if (chunks <= 2048) return launch_rows<T, 2, 1024>(S, P, rows, chunks, stream);
        if (chunks <= 4096) return launch_rows<T, 4, 1024>(S, P, rows, chunks, stream);
        if constexpr (MAXR >= 8) return launch_rows<T, 8, 1024>(S, P, rows, chunks, stream);
    }
    hipLaunchKernelGGL((softmax_generic_kernel<T>), dim3((uint32_t)rows), dim3(256), 0, stream,
                       static_cast<const T*>(S), static_cast<T*>(P), rows, cols);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_softmax(DType dt, const void* S, void* P, int64_t rows, int64_t cols, hipStream_t stream)
{
    if (dt == DType::F32) return launch_softmax_t<float>(S, P, rows, cols, stream);
    return launch_softmax_t<uint16_t>(S, P, rows, cols, stream);
}

}  // namespace attnw
