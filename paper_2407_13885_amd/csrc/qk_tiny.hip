// Fused attention weights  P = softmax(scale * Q K^T)  and scaled scores for MANY SHORT sequences (bf16, N <= 128 with
// d a multiple of 16 up to 128, N <= 256 with d <= 64): windows of 49 or 64 tokens with three to thirty-two heads each and thousands of
// windows per call, sentences of up to 128 tokens.  One head is a few matrix instructions of work; a workgroup
// per (head, strip) spends its time in prologue and barriers, and of eight waves that split 256 keys only two
// have any.
//
// Here a WAVE works alone: a unit of work is a (head, block of 32 queries) pair, the wave holds the K of the head
// as matrix-instruction operands in registers (loaded straight from global memory, no LDS, nothing shared with
// other waves, hence no barrier anywhere), multiplies them with the block's Q fragments -- S^T = K Q^T, so that a
// lane's accumulators are keys of ONE query --, and the whole row of scores of a query sits in the two lanes l and
// l + 32: the row maximum and sum (Softmax section, Eq. 1) are register reductions and one lane exchange, the
// weights are formed where the contraction left the scores, as in the paper's fused kernel (section "Fused Matrix
// Multiply + Scaling + Softmax") with a core's SRAM replaced by a wave's registers.
//
// The way out is a private LDS area per wave.  The 32 rows of a block are one contiguous piece of P; the wave
// stages it there and stores it as 16-byte chunks, consecutive lanes consecutive chunks:
//   * N a multiple of 8 (rows of P start on 16-byte boundaries): staged row by row with a padded pitch (conflict-
//     free writes), every chunk lies inside one row;
//   * otherwise: staged exactly as the block lies in memory, element (row, key) at o + row N + key with o = the
//     block's first element index mod 8; chunks straddle rows, the first and last chunk of a block are shared
//     with the neighbouring blocks and only the block's own elements of them are stored, one by one.
// Staging writes are 8 bytes while N is a multiple of 4, 4 while it is even, else 2.
//
// Keys past N: K rows clamped to the last on the way in, scores replaced by a large negative number before the
// maximum, weights neither summed nor staged.  Queries past N: rows clamped on the way in, not staged.
#include "launchers.h"
#include "qk_common.h"

namespace attnw {
namespace {

constexpr int kTinyWaves = 4;                     // waves per workgroup (independent of each other)

// NKB: 32-key blocks of a head (N <= 32 NKB); G: 16-element steps of the contraction (d = 16 G)
//
// A wave's units follow each other in memory (blocks of a head, then the next head), so its output is ONE
// contiguous stream of P; a unit's whole 16-byte chunks leave at once and the elements behind the last chunk
// boundary are carried to the front of the staging area, where the next unit continues the chunk.  Only the first
// chunk of the stream (shared with the wave before) and what is left after the last unit are stored element by
// element, after the loop.
//
// Vector-memory operations retire in order: a wave that waits for a load also waits for every store it issued
// before that load.  The operands of unit i + 1 are therefore requested right after the matrix instructions of
// unit i have read theirs (into the same registers) -- behind the stores of unit i - 1, ahead of those of unit i --,
// and every unit issues the same number of store instructions (lanes without a chunk masked off), so that the wait
// for the operands at the top of unit i + 1 is "all but the last NST operations" and leaves the stores of unit i
// in flight.
template <int NKB, int G, bool SCORES>
__global__ __launch_bounds__(64 * kTinyWaves, 2)   // (two workgroups per compute unit at least: at most 256 registers,
                                                   // which also keeps the accumulators of the matrix instructions
                                                   // in ordinary vector registers)
void qk_tiny_kernel(const uint16_t* __restrict__ Q, const uint16_t* __restrict__ K, uint16_t* __restrict__ out, int N,
                    float c, uint32_t sign_flip, uint32_t total_units)
{
    constexpr int ROW_B = 32 * G;                 // bytes of a row of Q or K
    constexpr int BLK_ELEMS = 32 * 32 * NKB + 32 * 8;   // as in memory: 7 + 32 N; row by row: 32 (N + 8)
    constexpr int NST = 2 * NKB;                  // store instructions per unit: 64 chunks each, (7 + 32 * 32 NKB) / 8 at most
    constexpr int LAST = NKB - 1;                 // the block of keys that N may cut (32 LAST < N <= 32 NKB)
    constexpr bool LATE = NKB > 4;                // where in a unit the operands of the next one are requested
    // how an odd length is staged: 4-byte writes of pairs made up across the two half-waves, or element by element
    // (measured: 1024 heads of N = 197, d = 32 36 -> 28 us, of N = 129, d = 64 26 -> 24; 12288 heads of N = 49 26 -> 28)
    constexpr bool PAIRED = NKB > 4;
    __shared__ __align__(16) uint16_t blk_lds[kTinyWaves][BLK_ELEMS];
    __shared__ __align__(16) uint16_t lead_lds[kTinyWaves][8];
    __shared__ __align__(16) uint16_t dump_lds[kTinyWaves][40];   // where the keys past N of a block go (32 + a run of 4)

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int l32 = lane & 31;
    const int half = lane >> 5;
    uint16_t* const blk = blk_lds[wave];

    // this wave's units: a contiguous range of the global (head, query block) order
    const uint32_t nqb = (uint32_t)((N + 31) / 32);
    const uint32_t w = blockIdx.x * kTinyWaves + wave, W = gridDim.x * kTinyWaves;
    const uint32_t u_begin = (uint32_t)((uint64_t)w * total_units / W);
    const uint32_t u_end = (uint32_t)((uint64_t)(w + 1) * total_units / W);
    if (u_begin >= u_end) return;

    const bool cut = N != 32 * NKB;
    const bool rows16 = (N % 8) == 0;             // rows of P on 16-byte boundaries
    const int pitch = (N % 16) == 0 ? N + 8 : N;  // elements between staged rows (rows16: 16 bytes x an odd number)
    const int cpr = N / 8;                        // rows16: chunks per row
    const uint32_t cpr_inv = cpr > 0 ? (65536u + (uint32_t)cpr - 1u) / (uint32_t)cpr : 0u;   // ch / cpr = ch * cpr_inv >> 16 for ch < 4096

    // where in the staging area the chunks are that this lane stores (chunk lane + 64 it of a unit)
    int own_off[NST];
#pragma unroll
    for (int it = 0; it < NST; ++it) {
        const int ch = lane + 64 * it;
        const int row = (int)(((uint32_t)ch * cpr_inv) >> 16);
        own_off[it] = rows16 ? row * pitch + (ch - row * cpr) * 8 : ch * 8;
    }

    uint32_t h = u_begin / nqb;
    uint32_t qb = u_begin - h * nqb;

    u32x4 kf[NKB][G], qf[G];
    auto request = [&](uint32_t hh, uint32_t qq) __attribute__((always_inline)) {
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
    request(h, qb);

    // the stream: `lead` elements in front of it belong to the wave before (its first chunk is stored after the loop)
    const int lead = rows16 ? 0 : (int)((((int64_t)h * N + (int64_t)qb * 32) * N) & 7);
    bool lead_pending = lead != 0;
    bool lead_saved = false;
    int64_t lead_at = 0;                          // element index in P of the chunk with the foreign elements
    int o = lead;                                 // elements carried in front of the unit being staged
    int64_t e_next = 0;

    auto unit = [&](uint32_t u) __attribute__((always_inline)) {
        const int q0 = (int)qb * 32;
        const int rows = min(32, N - q0);
        const int64_t e0 = ((int64_t)h * N + q0) * N;   // first element of the block in P

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
        if constexpr (!LATE) request(h1, qb1);

        // ---- row statistics and weights in place (Eq. 1) ---------------------------------------------------------------
        float inv = c;                            // SCORES: the scale
        if constexpr (!SCORES) {
            // (keys past N carry the score of key N - 1, whose K row they loaded: the maximum is not theirs alone)
            float m = kNegBig;
#pragma unroll
            for (int kb = 0; kb < NKB; ++kb) {
#pragma unroll
                for (int r = 0; r < 16; r += 2) m = max3(m, X[kb][r], X[kb][r + 1]);
            }
            m = fmaxf(m, __shfl_xor(m, 32, 64));  // lanes l and l + 32 hold the two halves of a query's keys
            const float mb = m * c;
#pragma unroll
            for (int kb = 0; kb < NKB; ++kb) {
#pragma unroll
                for (int r = 0; r < 16; ++r) X[kb][r] = fast_exp2(__builtin_fmaf(X[kb][r], c, -mb));
            }
            if (cut) {                            // (wave-uniform) N cuts the last block: its keys past N do not count
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
            inv = __builtin_amdgcn_rcpf(l);
        }

        // ---- stage the block behind the `o` elements carried over ----------------------------------------------------
        uint32_t Wp[NKB][8];                      // the lane's 16 keys of a block as 8 pairs
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
            for (int i = 0; i < 8; ++i) Wp[kb][i] = pack_bf16x2(X[kb][2 * i] * inv, X[kb][2 * i + 1] * inv);
        if (l32 < rows) {
            uint16_t* const rowp = blk + o + l32 * pitch;
            // keys past N (last block only) go to a dump area instead: a select of the address, no branch
            uint16_t* const dumpp = dump_lds[wave] - LAST * 32;
            // GRAN bytes per staging write: 8 while N is a multiple of 4 (runs of 4 keys are whole or absent, and 8-byte
            // aligned), 4 while it is even, else 2
            const int par = (o + l32 * N) & 1;   // (odd N) the row starts on an odd element of the staging area
            auto stage = [&](auto granc) __attribute__((always_inline)) {
                constexpr int GRAN = decltype(granc)::value;
                uint32_t end_val = 0u;
                bool end_here = false;
#pragma unroll
                for (int kb = 0; kb < NKB; ++kb) {
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4) {
                        const int key = kb * 32 + 8 * r4 + 4 * half;
                        const uint32_t w01 = Wp[kb][2 * r4], w23 = Wp[kb][2 * r4 + 1];
                        auto at = [&](int k) __attribute__((always_inline)) -> uint16_t* {
                            if (kb < LAST) return rowp + k;
                            return (k < N ? rowp : dumpp) + k;
                        };
                        if constexpr (GRAN == 8) {
                            *reinterpret_cast<u32x2*>(at(key)) = u32x2{w01, w23};
                        } else if constexpr (GRAN == 4) {
                            *reinterpret_cast<uint32_t*>(at(key)) = w01;
                            *reinterpret_cast<uint32_t*>(at(key + 2)) = w23;
                        } else if constexpr (!PAIRED) {
                            *at(key) = (uint16_t)(w01 & 0xffffu);
                            *at(key + 1) = (uint16_t)(w01 >> 16);
                            *at(key + 2) = (uint16_t)(w23 & 0xffffu);
                            *at(key + 3) = (uint16_t)(w23 >> 16);
                        } else {
                            // Odd N: rows start on even and odd elements in turn (`par`), and 2-byte LDS writes are slow.
                            // A row that starts odd pairs its keys as (1, 2), (3, 4) ...: the second word of a run takes
                            // its upper half from the run that follows in memory, which the other half-wave's lane
                            // of the same row holds (half 0: same r4 of half 1; half 1: the next r4 of half 0) -- one lane
                            // exchange per run, two aligned 4-byte writes.  Words with a key past N go to the dump area;
                            // the one element per row without a partner in its own row follows below.
                            uint32_t nxt = 0u;    // this lane's first pair of the run after this one
                            if (r4 < 3) nxt = Wp[kb][2 * r4 + 2];
                            else if (kb + 1 < NKB) nxt = Wp[kb + 1][0];
                            uint32_t nw = w23;
#if defined(__HIP_DEVICE_COMPILE__)
                            const auto sw = __builtin_amdgcn_permlane32_swap(w01, nxt, false, false);
                            nw = half ? sw[0] : sw[1];
#endif
                            const uint32_t W1 = par ? __builtin_amdgcn_alignbit(w23, w01, 16) : w01;
                            const uint32_t W2 = par ? __builtin_amdgcn_alignbit(nw, w23, 16) : w23;
                            const int k1 = key + par, k2 = key + 2 + par;
                            uint16_t* const a1 = (kb < LAST || k1 + 1 < N) ? rowp + k1 : dumpp + key;
                            uint16_t* const a2 = (kb < LAST || k2 + 1 < N) ? rowp + k2 : dumpp + key + 2;
                            *reinterpret_cast<uint32_t*>(a1) = W1;
                            *reinterpret_cast<uint32_t*>(a2) = W2;
                            if (kb == LAST && !par) {     // the row's last element (N - 1 is even): the lower half of a word of its own
                                const bool c0 = key == N - 1, c2 = key + 2 == N - 1;
                                end_val = c0 ? w01 : (c2 ? w23 : end_val);
                                end_here = end_here || c0 || c2;
                            }
                        }
                    }
                }
                if constexpr (GRAN == 2 && PAIRED) {
                    // the element of a row whose partner in its word belongs to the neighbouring row: the first of a
                    // row that starts odd (key 0: half 0), the last of a row that starts even
                    uint16_t* ae = dump_lds[wave];
                    uint32_t ve = Wp[0][0];
                    if (par) ae = half == 0 ? rowp : ae;
                    else {
                        ae = end_here ? rowp + (N - 1) : ae;
                        ve = end_val;
                    }
                    *ae = (uint16_t)(ve & 0xffffu);
                }
            };
            if ((N & 3) == 0) stage(IC<8>{});
            else if ((N & 1) == 0) stage(IC<4>{});
            else stage(IC<2>{});
        }
        // (the lanes of a wave read what other lanes wrote: LDS serves a wave's operations in order)
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        // (more than four blocks of keys: the scores and the K operands together exceed the registers, so the request
        // waits until the scores have left them -- still ahead of this unit's stores)
        if constexpr (LATE) request(h1, qb1);

        // ---- whole chunks leave: NST store instructions whatever the length ----------------------------------------------
        const int staged = o + rows * N;          // elements in the area (rows16: o = 0, a multiple of 8)
        const int n_whole = staged / 8;
        uint16_t* const gbase = out + (e0 - o);   // 16-byte aligned
        const int skip = (lead_pending && n_whole > 0) ? 1 : 0;   // the chunk with the foreign elements is not stored whole
        if (skip) {
            if (lane == 0) *reinterpret_cast<u32x4*>(lead_lds[wave]) = *reinterpret_cast<const u32x4*>(blk);
            lead_at = e0 - o;
            lead_saved = true;
            lead_pending = false;
        }
        // (every lane stores: lanes without a chunk of their own repeat the last one, the lane of the skipped chunk its
        // neighbour -- the same bytes to the same place; N >= 8 leaves a unit at least four whole chunks)
        const int last_off = rows16 ? (rows - 1) * pitch + (cpr - 1) * 8 : (n_whole - 1) * 8;
        constexpr int BATCH = NST < 4 ? NST : 4;
#pragma unroll
        for (int it0 = 0; it0 < NST; it0 += BATCH) {
            u32x4 v[BATCH];
            int ch[BATCH];
#pragma unroll
            for (int i = 0; i < BATCH; ++i) {
                const int it = it0 + i;
                const bool own = lane + 64 * it < n_whole;
                ch[i] = own ? lane + 64 * it : n_whole - 1;
                int off = own ? own_off[it] : last_off;
                if (it == 0) {
                    const bool sk = skip != 0 && lane == 0;
                    ch[i] = sk ? 1 : ch[i];
                    off = sk ? 8 : off;
                }
                v[i] = *reinterpret_cast<const u32x4*>(blk + off);
            }
#pragma unroll
            for (int i = 0; i < BATCH; ++i) __builtin_nontemporal_store(v[i], reinterpret_cast<u32x4*>(gbase + ch[i] * 8));
        }
        // what is behind the last chunk boundary moves to the front of the area
        const int left = staged - n_whole * 8;
        if (lane == 0 && n_whole > 0 && !rows16)
            *reinterpret_cast<u32x4*>(blk) = *reinterpret_cast<const u32x4*>(blk + n_whole * 8);
        o = left;
        e_next = e0 + (int64_t)rows * N;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();

        h = h1;
        qb = qb1;
    };
    // (the first unit stands in front of the loop so that every path into the loop's head has issued the same
    // operations: loads, then NST stores -- the wait for the loads is computed from what all paths agree on)
    unit(u_begin);
    for (uint32_t u = u_begin + 1; u < u_end; ++u) unit(u);

    // ---- the two ends of the stream, element by element ------------------------------------------------------------------------
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    if (lane < 8) {
        if (lead_saved && lane >= lead) out[lead_at + lane] = lead_lds[wave][lane];
        // what the last unit left in front of the area: `o` elements that end at e_next (a stream that never reached a
        // chunk boundary still has the foreign elements in front)
        const int from = lead_pending ? lead : 0;
        if (lane >= from && lane < o) out[e_next - o + lane] = blk[lane];
    }
}

template <int NKB, int G>
hipError_t launch_tiny_t(bool scores_only, const void* Q, const void* K, void* out, int64_t BH, int N, float scale,
                         hipStream_t stream)
{
    const uint32_t total = (uint32_t)(BH * ((N + 31) / 32));
    // independent waves: as many as the chip holds at a time, each with a contiguous range of units
    static const int per_cu[2] = {
        [] { int n = 0; return hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, qk_tiny_kernel<NKB, G, false>, 64 * kTinyWaves, 0) == hipSuccess && n > 0 ? n : 2; }(),
        [] { int n = 0; return hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, qk_tiny_kernel<NKB, G, true>, 64 * kTinyWaves, 0) == hipSuccess && n > 0 ? n : 2; }()};
    const uint32_t resident = (uint32_t)compute_units() * (uint32_t)per_cu[scores_only ? 1 : 0];
    const uint32_t want = (total + kTinyWaves - 1) / kTinyWaves;
    const uint32_t grid = want < resident ? want : resident;
    const float c = scores_only ? scale : fabsf(scale) * kLog2e;
    const uint32_t flip = (!scores_only && scale < 0.0f) ? Mma<uint16_t>::kSignMask : 0u;
    if (scores_only)
        hipLaunchKernelGGL((qk_tiny_kernel<NKB, G, true>), dim3(grid), dim3(64 * kTinyWaves), 0, stream,
                           static_cast<const uint16_t*>(Q), static_cast<const uint16_t*>(K), static_cast<uint16_t*>(out), N, c,
                           flip, total);
    else
        hipLaunchKernelGGL((qk_tiny_kernel<NKB, G, false>), dim3(grid), dim3(64 * kTinyWaves), 0, stream,
                           static_cast<const uint16_t*>(Q), static_cast<const uint16_t*>(K), static_cast<uint16_t*>(out), N, c,
                           flip, total);
    return hipGetLastError();
}

template <int NKB>
hipError_t launch_tiny(bool scores_only, const void* Q, const void* K, void* out, int64_t BH, int N, int d, float scale,
                       hipStream_t stream)
{
    switch (d / 16) {
    case 1: return launch_tiny_t<NKB, 1>(scores_only, Q, K, out, BH, N, scale, stream);
    case 2: return launch_tiny_t<NKB, 2>(scores_only, Q, K, out, BH, N, scale, stream);
    case 3: return launch_tiny_t<NKB, 3>(scores_only, Q, K, out, BH, N, scale, stream);
    case 4: if constexpr (NKB <= 7) return launch_tiny_t<NKB, 4>(scores_only, Q, K, out, BH, N, scale, stream); else break;
    case 5: if constexpr (NKB <= 4) return launch_tiny_t<NKB, 5>(scores_only, Q, K, out, BH, N, scale, stream); else break;
    case 6: if constexpr (NKB <= 4) return launch_tiny_t<NKB, 6>(scores_only, Q, K, out, BH, N, scale, stream); else break;
    case 7: if constexpr (NKB < 4) return launch_tiny_t<NKB, 7>(scores_only, Q, K, out, BH, N, scale, stream); else break;
    case 8: if constexpr (NKB < 4) return launch_tiny_t<NKB, 8>(scores_only, Q, K, out, BH, N, scale, stream); else break;
    default: break;
    }
    return hipErrorInvalidValue;
}

}  // namespace

bool qk_tiny_supported(int64_t BH, int64_t N, int64_t d)
{
    if (N < 8 || N > 256 || d < 16 || d > 128 || (d % 16) != 0) return false;   // (N >= 8: see the stores of a unit)
    if (N > 96 && d > 96) return false;           // (operands and scores of a unit would not fit the registers)
    if (N > 128 && d > 64) return false;
    if (N > 224 && d > 48) return false;
    return BH * ((N + 31) / 32) <= (int64_t)0x7ffffff0;
}

hipError_t launch_qk_tiny(bool scores_only, const void* Q, const void* K, void* out, int64_t BH, int64_t N, int64_t d,
                          float scale, hipStream_t stream)
{
    if (N <= 32) return launch_tiny<1>(scores_only, Q, K, out, BH, (int)N, (int)d, scale, stream);
    if (N <= 64) return launch_tiny<2>(scores_only, Q, K, out, BH, (int)N, (int)d, scale, stream);
    if (N <= 96) return launch_tiny<3>(scores_only, Q, K, out, BH, (int)N, (int)d, scale, stream);
    if (N <= 128) return launch_tiny<4>(scores_only, Q, K, out, BH, (int)N, (int)d, scale, stream);
    if (N <= 160) return launch_tiny<5>(scores_only, Q, K, out, BH, (int)N, (int)d, scale, stream);
    if (N <= 192) return launch_tiny<6>(scores_only, Q, K, out, BH, (int)N, (int)d, scale, stream);
    if (N <= 224) return launch_tiny<7>(scores_only, Q, K, out, BH, (int)N, (int)d, scale, stream);
    return launch_tiny<8>(scores_only, Q, K, out, BH, (int)N, (int)d, scale, stream);
}

}  // namespace attnw
