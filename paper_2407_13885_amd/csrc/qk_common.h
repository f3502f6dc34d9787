// Building blocks shared by the Q K^T kernels: MFMA wrappers per element type,
// direct global-to-LDS transfers, wait-count helpers and compile-time loop helpers.
#pragma once

#include "device_utils.h"

namespace attnw {

typedef const void __attribute__((address_space(1)))* global_cptr;
typedef void __attribute__((address_space(3)))* lds_ptr;

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

// vmcnt(0) with the other counters left alone (gfx9 encoding of s_waitcnt)
__device__ __forceinline__ void wait_vmem() { __builtin_amdgcn_s_waitcnt(0x0F70); }
// vmcnt(N): wait until at most the N youngest vector-memory operations are outstanding
template <int N> __device__ __forceinline__ void wait_vmem_le()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit field");
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// 16 bytes per lane from global memory straight into LDS (lane i lands at dst + 16*i;
// dst is wave-uniform).  The __restrict__ parameters give the transfer an alias scope of
// its own once inlined, which is what lets the compiler see that LDS reads from the
// OTHER tile buffer need not wait for it.
__device__ __forceinline__ void dma16(const char* __restrict__ src, char* __restrict__ dst)
{
    __builtin_amdgcn_global_load_lds((global_cptr)src, (lds_ptr)dst, 16, 0, 0);
}

// The same transfer issued from inline assembly, which the compiler's wait-count pass does not see: the
// only waits on it are the explicit vmcnt waits of the caller (vector-memory operations retire in order).
// lds_base = byte offset in LDS, wave-uniform, below 64 KiB (it travels in M0).
__device__ __forceinline__ void dma16_untracked(const char* src, uint32_t lds_base)
{
#if defined(__HIP_DEVICE_COMPILE__)
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_base), "v"(src) : "memory", "m0");
#endif
}

__device__ __forceinline__ uint32_t lds_offset_of(const void* p)
{
    return (uint32_t)(uintptr_t)(lds_ptr)(p);
}

template <int I> struct IC { static constexpr int value = I; };

// f(IC<0>{}), f(IC<1>{}), ... f(IC<N-1>{})
template <int N, typename F> __device__ __forceinline__ void static_for(F&& f)
{
    if constexpr (N > 0) {
        static_for<N - 1>(f);
        f(IC<N - 1>{});
    }
}

// Calls body(t, IC<buffer>) for t = first .. n-1 with the LDS buffer alternating from
// `buf_first`; the buffer is a compile-time constant inside body.
template <typename Body>
__device__ __forceinline__ void for_tiles(int first, int buf_first, int n, Body&& body)
{
    int t = first;
    if (buf_first == 1 && t < n) { body(t, IC<1>{}); ++t; }
    for (; t + 1 < n; t += 2) {
        body(t, IC<0>{});
        body(t + 1, IC<1>{});
    }
    if (t < n) body(t, IC<0>{});
}

}  // namespace attnw
