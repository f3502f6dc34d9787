// Attention output  O = softmax(scale * Q K^T) V  for MANY SHORT sequences (bf16, N <= 128, d = 32 or 64 -- windows
// of 49 or 64 tokens with a few heads each and thousands of windows per call): the product the paper's section
// "Limitations and future Directions" names as the next thing to fuse, on the shapes where a workgroup per
// (head, strip) spends its time in prologue and barriers.
//
// As in the kernel for the attention weights of such shapes, a WAVE works alone on a (head, block of 32 queries)
// pair: K and the block's Q rows come straight from global memory as matrix-instruction operands, S^T = K Q^T leaves
// the whole row of scores of a query in lanes l and l + 32, maximum and sum (Softmax section, Eq. 1) are register
// reductions and one lane exchange.  The exponentials, rounded to bf16, ARE the second operand of the next matrix
// instruction: a lane's 8 values of a 16-key step are keys 16 s + 8 (j / 4) + 4 half + j % 4, and the V operand is
// gathered with the same assignment -- the V of the head travels global memory -> the wave's private LDS area as it
// lies in memory (16 bytes per lane, no registers), and lane l of a half reads column l of its 8 rows, two bytes
// each --, so O^T = V^T P^T needs no exchange between lanes either.  The output is divided by the row sum at the
// end, staged row by row in LDS and stored as 16-byte chunks.  No barrier anywhere.
//
// Vector-memory operations retire in order, so operands are requested into the registers that the matrix
// instructions have just read -- K and Q of unit i + 1 after the score instructions of unit i, V of unit i + 1 (into
// the LDS area) after its output instructions -- and every unit issues the same number of loads, transfers and
// stores: the waits are then "all but the last n operations" and leave the stores of the previous unit in flight.
#include "launchers.h"
#include "qk_common.h"

namespace attnw {
namespace {

// waves per workgroup (independent of each other): four, or two where four waves' areas for V would take the LDS of a
// compute unit for one workgroup (d = 64 with more than 64 keys: 16 KiB of V per wave)
template <int NKB, int DB> constexpr int waves_of() { return NKB * DB > 4 ? 2 : 4; }

// NKB: 32-key blocks of a head (32 (NKB - 1) < N <= 32 NKB); DB: 32-column blocks of the head size (d = 32 DB)
template <int NKB, int DB>
__global__ __launch_bounds__((NKB * DB > 4 ? 128 : 256), 2)
void attention_tiny_kernel(const uint16_t* __restrict__ Q, const uint16_t* __restrict__ K, const uint16_t* __restrict__ V,
                           uint16_t* __restrict__ O, int N, float c, uint32_t sign_flip, uint32_t total_units)
{
    constexpr int kWaves = waves_of<NKB, DB>();
    constexpr int G = 2 * DB;                     // 16-element steps of the score contraction
    constexpr int D = 32 * DB;
    constexpr int ROW_B = 2 * D;                  // bytes of a row of Q, K, V, O
    constexpr int LAST = NKB - 1;                 // the block of keys that N may cut
    constexpr int PITCH = D + 8;                  // elements between staged rows of O (16 bytes x an odd number)
    constexpr int CPR = D / 8;                    // 16-byte chunks per row of O
    constexpr int NST = 32 * CPR / 64;            // store instructions per unit
    constexpr int NV = NKB * 32 * ROW_B / 1024;   // 1-KiB wave transfers that bring the V of a head
    constexpr int NQK = (NKB + 1) * G;            // 16-byte loads per lane that bring K and the Q rows of a unit
    __shared__ __align__(1024) char v_lds[kWaves][NV * 1024];   // (first in LDS: the transfers address the first 64 KiB)
    __shared__ __align__(16) uint16_t o_lds[kWaves][32 * PITCH];

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int l32 = lane & 31;
    const int half = lane >> 5;
    uint16_t* const blk = o_lds[wave];

    // this wave's units: a contiguous range of the global (head, query block) order
    const uint32_t nqb = (uint32_t)((N + 31) / 32);
    const uint32_t w = blockIdx.x * kWaves + wave, W = gridDim.x * kWaves;
    const uint32_t u_begin = (uint32_t)((uint64_t)w * total_units / W);
    const uint32_t u_end = (uint32_t)((uint64_t)(w + 1) * total_units / W);
    if (u_begin >= u_end) return;
    const bool cut = N != 32 * NKB;

    uint32_t h = u_begin / nqb;
    uint32_t qb = u_begin - h * nqb;

    u32x4 kf[NKB][G], qf[G];
    auto request_qk = [&](uint32_t hh, uint32_t qq) __attribute__((always_inline)) {
        const char* const Kh = reinterpret_cast<const char*>(K) + (int64_t)hh * N * ROW_B;
        const char* const Qh = reinterpret_cast<const char*>(Q) + (int64_t)hh * N * ROW_B;
        {
            const char* p = Qh + (int64_t)min((int)qq * 32 + l32, N - 1) * ROW_B + half * 16;
#pragma unroll
            for (int g = 0; g < G; ++g) qf[g] = *reinterpret_cast<const u32x4*>(p + g * 32);
        }
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb) {
            const char* p = Kh + (int64_t)min(kb * 32 + l32, N - 1) * ROW_B + half * 16;
#pragma unroll
            for (int g = 0; g < G; ++g) kf[kb][g] = *reinterpret_cast<const u32x4*>(p + g * 32);
        }
    };
    // V of head hh into the wave's LDS area as it lies in memory (lanes past the end repeat the last 16 bytes: rows past
    // N then hold finite values, and their weights are zero)
    // The transfers are issued from inline assembly: the compiler does not count them, so its own waits (for K and Q) are
    // computed as if they were not there -- they then wait for the transfers too, which is safe -- and the wait that
    // the V operands need is the explicit one in front of the second contraction.
    char* const v_area = v_lds[wave];
    const uint32_t v_base = lds_offset_of(v_area);
    const int v_chunks = N * (ROW_B / 16);
    auto request_v = [&](uint32_t hh) __attribute__((always_inline)) {
        const char* const Vh = reinterpret_cast<const char*>(V) + (int64_t)hh * N * ROW_B;
#pragma unroll
        for (int t = 0; t < NV; ++t) dma16_untracked(Vh + (int64_t)min(t * 64 + lane, v_chunks - 1) * 16, v_base + t * 1024);
    };
    // V operand of the 16-key step (kb, s) and column block db: element j = V[32 kb + 16 s + 8 (j / 4) + 4 half + j % 4][32 db + l32]
    const uint16_t* const v_lane = reinterpret_cast<const uint16_t*>(v_area) + 4 * half * D + l32;
    auto v_operand = [&](int kb, int s, int db) __attribute__((always_inline)) -> u32x4 {
        u32x4 f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int kc = kb * 32 + 16 * s + 8 * (i / 2) + 2 * (i % 2);
            const uint32_t lo = v_lane[kc * D + 32 * db], hi = v_lane[(kc + 1) * D + 32 * db];
            f[i] = lo | (hi << 16);
        }
        return f;
    };
    request_v(h);
    wait_vmem();                                  // (once per wave: the waits below assume a unit's worth of operations behind the transfers)
    request_qk(h, qb);

    // where in the staging area the chunks are that this lane stores (chunk lane + 64 it of a unit)
    int own_off[NST];
#pragma unroll
    for (int it = 0; it < NST; ++it) {
        const int ch = lane + 64 * it;
        own_off[it] = (ch / CPR) * PITCH + (ch % CPR) * 8;
    }

    auto unit = [&](uint32_t u) __attribute__((always_inline)) {
        const int q0 = (int)qb * 32;
        const int rows = min(32, N - q0);

        // ---- scores: X[kb][r] = q . k for key 32 kb + 8 (r / 4) + 4 half + r % 4 and query q0 + l32 ----------------
        f32x16 X[NKB];
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb) {
#pragma unroll
            for (int r = 0; r < 16; ++r) X[kb][r] = 0.0f;
#pragma unroll
            for (int g = 0; g < G; ++g) Mma<uint16_t>::run(X[kb], kf[kb][g], qf[g] ^ sign_flip);
        }
        // the operands of the next unit, into the registers the matrix instructions have just read (the last unit
        // requests itself again: every unit issues the same operations)
        uint32_t h1 = h, qb1 = qb;
        if (u + 1 < u_end && ++qb1 == nqb) {
            qb1 = 0;
            ++h1;
        }
        request_qk(h1, qb1);

        // ---- row statistics, exponentials in place (Eq. 1) ----------------------------------------------------------------
        // (keys past N carry the score of key N - 1, whose K row they loaded: the maximum is not theirs alone)
        float m = kNegBig;
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb) {
#pragma unroll
            for (int r = 0; r < 16; r += 2) m = max3(m, X[kb][r], X[kb][r + 1]);
        }
        m = fmaxf(m, __shfl_xor(m, 32, 64));      // lanes l and l + 32 hold the two halves of a query's keys
        const float mb = m * c;
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb) {
#pragma unroll
            for (int r = 0; r < 16; ++r) X[kb][r] = fast_exp2(__builtin_fmaf(X[kb][r], c, -mb));
        }
        if (cut) {                                // (wave-uniform) N cuts the last block: its keys past N do not count
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int key = LAST * 32 + 8 * (r / 4) + 4 * half + (r % 4);
                X[LAST][r] = key < N ? X[LAST][r] : 0.0f;
            }
        }
        float ls[4] = {0.0f, 0.0f, 0.0f, 0.0f};   // four chains of additions instead of one
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb) {
#pragma unroll
            for (int r = 0; r < 16; ++r) ls[r & 3] += X[kb][r];
        }
        float l = (ls[0] + ls[1]) + (ls[2] + ls[3]);
        l += __shfl_xor(l, 32, 64);
        const float inv = __builtin_amdgcn_rcpf(l);

        // ---- O^T = V^T P^T: the exponentials, rounded to bf16, are the second operand as they stand ------------------------
        // The V of this unit was requested after the output instructions of the unit before; younger than that are the
        // stores of that unit and the K / Q loads above.
        wait_vmem_le<NST + NQK>();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        f32x16 oacc[DB];
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[db][r] = 0.0f;
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                u32x4 pw;
#pragma unroll
                for (int i = 0; i < 4; ++i) pw[i] = pack_bf16x2(X[kb][8 * s + 2 * i], X[kb][8 * s + 2 * i + 1]);
#pragma unroll
                for (int db = 0; db < DB; ++db) Mma<uint16_t>::run(oacc[db], v_operand(kb, s, db), pw);
            }
        // (every lane is done reading V: what it read is in its registers before the transfers below can land)
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        request_v(h1);

        // ---- stage the block of O row by row: oacc[db][r] is column 32 db + 8 (r / 4) + 4 half + r % 4 of query l32 ---------
        if (l32 < rows) {
            uint16_t* const rowp = blk + l32 * PITCH;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const uint32_t w01 = pack_bf16x2(oacc[db][4 * r4] * inv, oacc[db][4 * r4 + 1] * inv);
                    const uint32_t w23 = pack_bf16x2(oacc[db][4 * r4 + 2] * inv, oacc[db][4 * r4 + 3] * inv);
                    *reinterpret_cast<u32x2*>(rowp + db * 32 + 8 * r4 + 4 * half) = u32x2{w01, w23};
                }
        }
        // (the lanes of a wave read what other lanes wrote: LDS serves a wave's operations in order)
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        // ---- the block leaves: NST store instructions whatever the number of rows (lanes without a chunk of their own
        // repeat the last one -- the same bytes to the same place)
        uint16_t* const gbase = O + ((int64_t)h * N + q0) * D;
        const int n_chunks = rows * CPR;
        const int last_off = (rows - 1) * PITCH + (CPR - 1) * 8;
        u32x4 v[NST];
        int ch[NST];
#pragma unroll
        for (int it = 0; it < NST; ++it) {
            const bool own = lane + 64 * it < n_chunks;
            ch[it] = own ? lane + 64 * it : n_chunks - 1;
            v[it] = *reinterpret_cast<const u32x4*>(blk + (own ? own_off[it] : last_off));
        }
#pragma unroll
        for (int it = 0; it < NST; ++it) __builtin_nontemporal_store(v[it], reinterpret_cast<u32x4*>(gbase + ch[it] * 8));
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();

        h = h1;
        qb = qb1;
    };
    // (the first unit stands in front of the loop so that every path into the loop's head has issued the same
    // operations -- the waits for the loads are computed from what all paths agree on)
    unit(u_begin);
    for (uint32_t u = u_begin + 1; u < u_end; ++u) unit(u);
}

template <int NKB, int DB>
hipError_t launch_t(const void* Q, const void* K, const void* V, void* O, int64_t BH, int N, float scale, hipStream_t stream)
{
    constexpr int kWaves = waves_of<NKB, DB>();
    const uint32_t total = (uint32_t)(BH * ((N + 31) / 32));
    static const int per_cu = [] {
        int n = 0;
        return hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, attention_tiny_kernel<NKB, DB>, 64 * kWaves, 0) == hipSuccess && n > 0 ? n : 2;
    }();
    const uint32_t resident = (uint32_t)compute_units() * (uint32_t)per_cu;
    const uint32_t want = (total + kWaves - 1) / kWaves;
    const uint32_t grid = want < resident ? want : resident;
    const float c = fabsf(scale) * kLog2e;
    const uint32_t flip = scale < 0.0f ? Mma<uint16_t>::kSignMask : 0u;
    hipLaunchKernelGGL((attention_tiny_kernel<NKB, DB>), dim3(grid), dim3(64 * kWaves), 0, stream,
                       static_cast<const uint16_t*>(Q), static_cast<const uint16_t*>(K), static_cast<const uint16_t*>(V),
                       static_cast<uint16_t*>(O), N, c, flip, total);
    return hipGetLastError();
}

}  // namespace

bool attention_tiny_supported(int64_t BH, int64_t N, int64_t d)
{
    if (N < 1 || N > (d == 32 ? 224 : 128) || (d != 32 && d != 64)) return false;   // (beyond: scores and operands exceed the registers)
    return BH * ((N + 31) / 32) <= (int64_t)0x7ffffff0;
}

// Measured against the tiled kernel, us (heads x N, d): 12288 x 49, 32 122 -> 30; 12288 x 64, 32 119 -> 38; 12288 x 100, 32
// 133 -> 81; 12288 x 128, 32 145 -> 137; 12288 x 49, 64 242 -> 57; 12288 x 64, 64 252 -> 90; 1024 x 32, 64 20 -> 4.3; 16 to 256
// heads: within 0.5 us of each other either way.  d = 64 beyond 64 keys (two waves per workgroup), 1024 heads: N = 65
// 22 -> 12, 96 26 -> 14, 100 26.5 -> 19, 128 29.5 -> 24.5; 12288 heads of N = 128: 307 -> 268.
// d = 32 beyond 128 keys (two waves per workgroup), 3072 heads: N = 129 52 -> 34, 144 60 -> 40, 160 55 -> 44; 197 57 -> 79 and
// 224 58 -> 91: not taken from 161 keys on.
bool prefers_attention_tiny(int64_t BH, int64_t N, int64_t d)
{
    (void)BH; (void)d;
    return N <= 160;
}

hipError_t launch_attention_tiny(const void* Q, const void* K, const void* V, void* O, int64_t BH, int64_t N, int64_t d,
                                 float scale, hipStream_t stream)
{
    const int n = (int)N;
    if (d == 32) {
        if (n <= 32) return launch_t<1, 1>(Q, K, V, O, BH, n, scale, stream);
        if (n <= 64) return launch_t<2, 1>(Q, K, V, O, BH, n, scale, stream);
        if (n <= 96) return launch_t<3, 1>(Q, K, V, O, BH, n, scale, stream);
        if (n <= 128) return launch_t<4, 1>(Q, K, V, O, BH, n, scale, stream);
        if (n <= 160) return launch_t<5, 1>(Q, K, V, O, BH, n, scale, stream);
        if (n <= 192) return launch_t<6, 1>(Q, K, V, O, BH, n, scale, stream);
        return launch_t<7, 1>(Q, K, V, O, BH, n, scale, stream);
    }
    if (n <= 32) return launch_t<1, 2>(Q, K, V, O, BH, n, scale, stream);
    if (n <= 64) return launch_t<2, 2>(Q, K, V, O, BH, n, scale, stream);
    if (n <= 96) return launch_t<3, 2>(Q, K, V, O, BH, n, scale, stream);
    return launch_t<4, 2>(Q, K, V, O, BH, n, scale, stream);
}

}  // namespace attnw
