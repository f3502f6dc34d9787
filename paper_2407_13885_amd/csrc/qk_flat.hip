// Fused attention weights  P = softmax(scale * Q K^T)  for SHORT sequences of ANY length (bf16, d = 32 or 64, N <= 608):
// the lengths of a class token in front of a patch grid -- 197, 257, 577 -- are odd, so no row of P but the
// first starts on a 16-byte boundary, and a kernel that stores pieces of rows is left with 2-byte stores.
//
// As in the kernel for N = 512 / 1024 (the shape of the paper's own fused kernel, section "Fused Matrix Multiply +
// Scaling + Softmax": the scores stay where the matrix multiply left them, the cores of a row exchange local maxima
// and sums, only then are the weights formed and written) a workgroup of eight waves keeps the K of a head in LDS
// and works on strips of 32 queries; wave w owns keys 32 NT w .. 32 NT (w + 1) of the row, its scores stay in
// registers from the contraction to the normalisation (Softmax section, Eq. 1, against the wave's own maximum; one
// exchange of (reference exponent, sum) pairs through LDS per strip).
//
// What is different is the way out.  The 32 rows of a strip are ONE contiguous block of 32 N elements of P (rows
// follow each other without padding), so the strip is staged in LDS exactly as it lies in memory -- element
// (row, key) at flat position o + row N + key, o = the block's first element index mod 8 -- and then leaves as the
// aligned 16-byte chunks that cover the block: consecutive lanes, consecutive chunks, whole lines whatever N is.
// Only the block's first and last chunk are shared with the neighbouring strips; of those the block's own elements
// are stored one by one.  Staging writes are 8 bytes while N is a multiple of 4 (positions stay on 8-byte
// boundaries), 4 bytes while it is even, else 2.
//
// Keys past N: their K rows are never copied (LDS holds whatever it held), their scores are replaced by a large
// negative number before the maximum and their weights never staged.  Queries past N (last strip): rows clamped on
// the way in, not staged.
#include "launchers.h"
#include "qk_common.h"

namespace attnw {
namespace {

constexpr int kFlatMaxN = 608;                    // 256 N bytes of LDS: K of a head and the blocks of two strips

// NT: 32-key pieces per wave (N <= 256 NT); GRAN: bytes of one staging write (8, 4 or 2)
//
// Strips are pipelined over one barrier each: iteration i computes the scores, exponentials and local statistics of
// strip i + 1 (published into the statistics buffer of its parity) and THEN turns the exponentials of strip i, whose
// statistics every wave published before the previous barrier, into weights in the block buffer of its parity; after
// the barrier the block leaves while the next iteration already computes.  Two register sets of exponentials, two
// statistics buffers, two block buffers.
// SCORES: write scale * Q K^T instead of the weights (the first stage of the unfused pipelines: no statistics, the same
//         way out); c is then the scale itself
// DB: bytes of a row of Q or K (64, 128: d = 32, 64)
template <int DB, int NT, int GRAN, bool SCORES>
__global__ __launch_bounds__(512)
void qk_flat_kernel(const uint16_t* __restrict__ Q, const uint16_t* __restrict__ K, uint16_t* __restrict__ out, int N,
                    float c, uint32_t sign_flip, uint32_t strips_per_head, uint32_t total_strips)
{
    constexpr int NW = 8, G = DB / 32, CPR = DB / 16, NTHREADS = 64 * NW;
    constexpr int KEYS = 32 * NT * NW;            // keys the waves cover
    constexpr int K_ROWS = KEYS < kFlatMaxN ? KEYS : kFlatMaxN;
    constexpr int K_BYTES = K_ROWS * DB;
    constexpr int BLOCK_BYTES = (32 * K_ROWS + 16) * 2;   // a strip's block as it lies in memory, its offset, the rest of its last chunk
    constexpr int STAT_FLOATS = 2 * NW * 32;
    constexpr int RPL = 16 / CPR, SWZ_MASK = CPR - 1;

    __shared__ __align__(1024) char lds[K_BYTES + 2 * BLOCK_BYTES + 2 * STAT_FLOATS * 4];
    char* const k_lds = lds;
    float* const stat = reinterpret_cast<float*>(lds + K_BYTES + 2 * BLOCK_BYTES);   // [parity][max, sum][wave][query]

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int l32 = lane & 31;
    const int half = lane >> 5;

    // this workgroup's strips: a contiguous range of the global (head, strip) order
    const uint32_t wg = xcd_contiguous_block_id(blockIdx.x, gridDim.x);
    const uint32_t s_begin = (uint32_t)((uint64_t)wg * total_strips / gridDim.x);
    const uint32_t s_end = (uint32_t)((uint64_t)(wg + 1) * total_strips / gridDim.x);
    if (s_begin >= s_end) return;

    // K in LDS: key * DB, the 16-byte chunk index XOR-swizzled by the key (conflict-free fragment reads)
    int frag_off[G];
    {
        const int swz = (l32 / RPL) & SWZ_MASK;
#pragma unroll
        for (int g = 0; g < G; ++g) frag_off[g] = l32 * DB + (((2 * g + half) ^ swz) * 16);
    }
    const int key_w0 = wave * NT * 32;            // first key of this wave
    const int k_chunks = N * CPR;                 // 16-byte chunks of a head's K

    // Q fragments of a strip (rows past the end read row N - 1; a negative scale negates Q)
    auto load_q = [&](u32x4 (&qf)[G], uint32_t strip_id) __attribute__((always_inline)) {
        const uint32_t bh = strip_id / strips_per_head;
        const int q0 = (int)(strip_id - bh * strips_per_head) * 32;
        const char* p = reinterpret_cast<const char*>(Q) + ((int64_t)bh * N + min(q0 + l32, N - 1)) * DB + half * 16;
#pragma unroll
        for (int g = 0; g < G; ++g) qf[g] = *reinterpret_cast<const u32x4*>(p + g * 32) ^ sign_flip;
    };
    uint32_t head_in_lds = 0xffffffffu;
    // the K of head bh replaces the one in LDS (every wave is past its last read of it: see the callers)
    auto k_switch = [&](uint32_t bh) __attribute__((always_inline)) {
        const char* Kh = reinterpret_cast<const char*>(K) + (int64_t)bh * N * DB;
        for (int s = tid; s < k_chunks; s += NTHREADS) {
            const int key = s / CPR;
            const int pos = (s % CPR) ^ ((key / RPL) & SWZ_MASK);
            *reinterpret_cast<u32x4*>(k_lds + key * DB + pos * 16) = *reinterpret_cast<const u32x4*>(Kh + (int64_t)s * 16);
        }
        __syncthreads();                          // K is in place
        head_in_lds = bh;
    };

    // scores of this wave's keys for the strip whose Q fragments are qf: S^T = K_piece * Q^T (a lane's 16 accumulators
    // are 16 keys of one query), exponentials against the wave's own maximum in their place, (reference exponent,
    // sum) published.  Returns the reference exponent.
    auto compute = [&](f32x16 (&X)[NT], const u32x4 (&qf)[G], uint32_t parity) __attribute__((always_inline)) -> float {
        float m = kNegBig;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
#pragma unroll
            for (int r = 0; r < 16; ++r) X[t][r] = 0.0f;
            const int kp = key_w0 + t * 32;       // first key of the piece
            if (kp < N) {                         // (wave-uniform) pieces past the end are not touched
                // (rows of K past N inside a piece hold stale data: finite or not, their scores are replaced below)
                const char* piece = k_lds + kp * DB;
#pragma unroll
                for (int g = 0; g < G; ++g)
                    Mma<uint16_t>::run(X[t], *reinterpret_cast<const u32x4*>(piece + frag_off[g]), qf[g]);
            }
            if constexpr (SCORES) continue;       // (keys past N are never staged)
            if (kp + 32 > N) {                    // (wave-uniform) the one piece that N cuts, and the pieces past it
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = kp + 8 * (r / 4) + 4 * half + (r % 4);
                    X[t][r] = key < N ? X[t][r] : kNegBig;
                }
            }
#pragma unroll
            for (int r = 0; r < 16; r += 2) m = max3(m, X[t][r], X[t][r + 1]);
        }
        if constexpr (SCORES) return c;           // the factor of every score
        m = fmaxf(m, __shfl_xor(m, 32, 64));      // lanes l and l + 32 hold the two halves of a query's keys
        const float mb = m * c;
        float l = 0.0f;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int kp = key_w0 + t * 32;
#pragma unroll
            for (int r = 0; r < 16; ++r) X[t][r] = fast_exp2(__builtin_fmaf(X[t][r], c, -mb));
            if (kp + 32 > N) {                    // (a wave without keys: mb = c * kNegBig, every exponential would be 1)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = kp + 8 * (r / 4) + 4 * half + (r % 4);
                    X[t][r] = key < N ? X[t][r] : 0.0f;
                }
            }
#pragma unroll
            for (int r = 0; r < 16; ++r) l += X[t][r];
        }
        l += __shfl_xor(l, 32, 64);
        if (half == 0) {
            float* const st = stat + parity * STAT_FLOATS;
            st[wave * 32 + l32] = mb;
            st[NW * 32 + wave * 32 + l32] = l;
        }
        return mb;
    };
    // exponentials of a strip -> weights, into the block buffer of its parity where they lie in memory
    auto finish = [&](const f32x16 (&X)[NT], float mb, uint32_t strip_id, uint32_t parity) __attribute__((always_inline)) {
        const uint32_t bh = strip_id / strips_per_head;
        const int q0 = (int)(strip_id - bh * strips_per_head) * 32;
        const int rows = min(32, N - q0);
        float inv = mb;                           // SCORES: the scale
        if constexpr (!SCORES) {
            const float* const st = stat + parity * STAT_FLOATS;
            float mbg = mb;
#pragma unroll
            for (int w = 0; w < NW; ++w) mbg = fmaxf(mbg, st[w * 32 + l32]);
            float lg = 0.0f;
#pragma unroll
            for (int w = 0; w < NW; ++w) lg += st[NW * 32 + w * 32 + l32] * fast_exp2(st[w * 32 + l32] - mbg);
            inv = fast_exp2(mb - mbg) * __builtin_amdgcn_rcpf(lg);
        }
        const int64_t e0 = ((int64_t)bh * N + q0) * N;                      // first element of the block in P
        const int o = (int)(e0 & 7);
        if (l32 < rows) {
            uint16_t* const rowp = reinterpret_cast<uint16_t*>(lds + K_BYTES + parity * BLOCK_BYTES) + o + l32 * N;
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const int kp = key_w0 + t * 32;
                if (kp >= N) break;               // (wave-uniform) pieces past the end
                const bool whole = kp + 32 <= N;  // (wave-uniform) every key of the piece exists
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const int key = kp + 8 * r4 + 4 * half;
                    const uint32_t w01 = pack_bf16x2(X[t][4 * r4] * inv, X[t][4 * r4 + 1] * inv);
                    const uint32_t w23 = pack_bf16x2(X[t][4 * r4 + 2] * inv, X[t][4 * r4 + 3] * inv);
                    if constexpr (GRAN == 8) {    // N a multiple of 4: runs of 4 keys are whole or absent, and 8-byte aligned
                        if (whole || key < N) *reinterpret_cast<u32x2*>(rowp + key) = u32x2{w01, w23};
                    } else if constexpr (GRAN == 4) {
                        if (whole || key < N) *reinterpret_cast<uint32_t*>(rowp + key) = w01;
                        if (whole || key + 2 < N) *reinterpret_cast<uint32_t*>(rowp + key + 2) = w23;
                    } else if (whole) {
                        // Odd N: rows start on even and odd elements in turn, and 2-byte LDS writes are slow.  A row that
                        // starts odd pairs its keys as (1, 2), (3, 4) ...: the second word of a run takes its upper half
                        // from the run that follows in memory, which the other half-wave's lane of the same row holds
                        // (half 0: same r4 of half 1; half 1: the next r4, or the next piece, of half 0) -- one lane
                        // exchange per run, two aligned 4-byte writes.  The wave's first key and, where its keys end
                        // (the next piece is another wave's, or past N), its last one have no partner here: 2 bytes each.
                        const int par = (o + l32 * N) & 1;
                        const bool more = r4 < 3 || (t + 1 < NT && kp + 32 < N);   // (wave-uniform) this wave holds the next run
                        uint32_t nxt = 0u;
                        if (r4 < 3) nxt = pack_bf16x2(X[t][4 * r4 + 4] * inv, X[t][4 * r4 + 5] * inv);
                        else if (t + 1 < NT) nxt = pack_bf16x2(X[t + 1 < NT ? t + 1 : t][0] * inv, X[t + 1 < NT ? t + 1 : t][1] * inv);
                        uint32_t nw = w23;
#if defined(__HIP_DEVICE_COMPILE__)
                        const auto sw = __builtin_amdgcn_permlane32_swap(w01, nxt, false, false);
                        nw = half ? sw[0] : sw[1];
#endif
                        const uint32_t W1 = par ? __builtin_amdgcn_alignbit(w23, w01, 16) : w01;
                        const uint32_t W2 = par ? __builtin_amdgcn_alignbit(nw, w23, 16) : w23;
                        *reinterpret_cast<uint32_t*>(rowp + key + par) = W1;
                        if (par && half && !more) rowp[key + 3] = (uint16_t)(w23 >> 16);
                        else *reinterpret_cast<uint32_t*>(rowp + key + 2 + par) = W2;
                        if (par && !half && t == 0 && r4 == 0) rowp[key] = (uint16_t)(w01 & 0xffffu);
                    } else {
                        if (key < N) rowp[key] = (uint16_t)(w01 & 0xffffu);
                        if (key + 1 < N) rowp[key + 1] = (uint16_t)(w01 >> 16);
                        if (key + 2 < N) rowp[key + 2] = (uint16_t)(w23 & 0xffffu);
                        if (key + 3 < N) rowp[key + 3] = (uint16_t)(w23 >> 16);
                    }
                }
            }
        }
    };
    // the block of a strip leaves as the aligned 16-byte chunks that cover it
    auto flush = [&](uint32_t strip_id, uint32_t parity) __attribute__((always_inline)) {
        const uint32_t bh = strip_id / strips_per_head;
        const int q0 = (int)(strip_id - bh * strips_per_head) * 32;
        const int rows = min(32, N - q0);
        const int64_t e0 = ((int64_t)bh * N + q0) * N;
        const int o = (int)(e0 & 7);
        const int first = o, last = o + rows * N;                          // its elements in the block buffer
        const int n_chunks = (last + 7) / 8;
        const uint16_t* const blk = reinterpret_cast<const uint16_t*>(lds + K_BYTES + parity * BLOCK_BYTES);
        uint16_t* const gbase = out + (e0 - o);                             // 16-byte aligned
        for (int ch = tid; ch < n_chunks; ch += NTHREADS) {
            const u32x4 v = *reinterpret_cast<const u32x4*>(blk + ch * 8);
            if (ch * 8 >= first && ch * 8 + 8 <= last) {
                __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(gbase + ch * 8));
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (ch * 8 + e >= first && ch * 8 + e < last)
                        gbase[ch * 8 + e] = (uint16_t)((e & 1) ? (v[e / 2] >> 16) : (v[e / 2] & 0xffffu));
            }
        }
    };

    f32x16 Xa[NT], Xb[NT];
    u32x4 qf[G];
    // ---- prologue: the first strip up to its statistics ----------------------------------------------------------
    load_q(qf, s_begin);
    k_switch(s_begin / strips_per_head);
    float mb_a = compute(Xa, qf, 0u), mb_b = 0.0f;
    if (s_begin + 1 < s_end) load_q(qf, s_begin + 1);
    __syncthreads();                              // its statistics are published

    // one iteration: strip `cur` (exponentials in X, reference exponent mb, parity p) is finished while strip cur + 1
    // is computed into Y; qf holds the fragments of cur + 1 on entry and of cur + 2 on exit
    auto iteration = [&](f32x16 (&X)[NT], float mb, f32x16 (&Y)[NT], float& mb_next, uint32_t cur, uint32_t p)
                         __attribute__((always_inline)) {
        const bool has_next = cur + 1 < s_end;
        if (has_next) {
            const uint32_t bh1 = (cur + 1) / strips_per_head;
            // (a new head: every wave is past its MFMAs of strip `cur` -- they precede the barrier before this iteration)
            if (bh1 != head_in_lds) k_switch(bh1);
            mb_next = compute(Y, qf, p ^ 1u);
            if (cur + 2 < s_end) load_q(qf, cur + 2);
        }
        finish(X, mb, cur, p);
        __syncthreads();                          // block `p` is complete, the statistics of cur + 1 are published
        // The Q fragments requested above are taken delivery of HERE, in front of the stores: vector-memory operations
        // retire in order and the number of stores below is not known to the compiler, so a wait for the fragments
        // placed after them would wait for every store to be acknowledged.
#pragma unroll
        for (int g = 0; g < G; ++g) asm volatile("" : "+v"(qf[g]));
        flush(cur, p);
    };
    for (uint32_t cur = s_begin; cur < s_end; cur += 2) {
        iteration(Xa, mb_a, Xb, mb_b, cur, 0u);
        if (cur + 1 < s_end) iteration(Xb, mb_b, Xa, mb_a, cur + 1, 1u);
    }
}

template <int DB, int NT, int GRAN>
hipError_t launch_flat_t(bool scores_only, const void* Q, const void* K, void* out, int64_t BH, int N, float scale, hipStream_t stream)
{
    const uint32_t strips_per_head = (uint32_t)((N + 31) / 32);
    const uint32_t total = (uint32_t)(BH * strips_per_head);
    // persistent workgroups, one per compute unit, each with a contiguous list of strips -- but not more workgroups
    // than give each at least four strips to spread the copy of K over
    // (N <= 256: two workgroups fit a compute unit's LDS, and one's waits are the other's work)
    uint32_t grid = (uint32_t)((compute_units() * (NT == 1 ? 2 : 1) + 7) / 8 * 8);
    const uint32_t want = (total + 3) / 4;
    if (grid > want) grid = (want + 7) / 8 * 8;
    const float c = scores_only ? scale : fabsf(scale) * kLog2e;
    const uint32_t flip = (!scores_only && scale < 0.0f) ? Mma<uint16_t>::kSignMask : 0u;
    if (scores_only)
        hipLaunchKernelGGL((qk_flat_kernel<DB, NT, GRAN, true>), dim3(grid), dim3(512), 0, stream, static_cast<const uint16_t*>(Q),
                           static_cast<const uint16_t*>(K), static_cast<uint16_t*>(out), N, c, flip, strips_per_head, total);
    else
        hipLaunchKernelGGL((qk_flat_kernel<DB, NT, GRAN, false>), dim3(grid), dim3(512), 0, stream, static_cast<const uint16_t*>(Q),
                           static_cast<const uint16_t*>(K), static_cast<uint16_t*>(out), N, c, flip, strips_per_head, total);
    return hipGetLastError();
}

template <int DB, int NT>
hipError_t launch_flat(bool scores_only, const void* Q, const void* K, void* out, int64_t BH, int N, float scale, hipStream_t stream)
{
    if (N % 4 == 0) return launch_flat_t<DB, NT, 8>(scores_only, Q, K, out, BH, N, scale, stream);
    if (N % 2 == 0) return launch_flat_t<DB, NT, 4>(scores_only, Q, K, out, BH, N, scale, stream);
    return launch_flat_t<DB, NT, 2>(scores_only, Q, K, out, BH, N, scale, stream);
}

template <int DB>
hipError_t launch_flat_d(bool scores_only, const void* Q, const void* K, void* out, int64_t BH, int N, float scale, hipStream_t stream)
{
    if (N <= 256) return launch_flat<DB, 1>(scores_only, Q, K, out, BH, N, scale, stream);
    if (N <= 512) return launch_flat<DB, 2>(scores_only, Q, K, out, BH, N, scale, stream);
    return launch_flat<DB, 3>(scores_only, Q, K, out, BH, N, scale, stream);
}

}  // namespace

bool qk_flat_supported(int64_t BH, int64_t N, int64_t d)
{
    // (d = 128 measured slower than the general kernel: K of a head and two blocks leave room for one workgroup per
    // compute unit -- 1024 heads of N = 197 91 -> 99 us, of N = 255 95 -> 125)
    if ((d != 32 && d != 64) || N < 1 || N > kFlatMaxN) return false;
    return BH * ((N + 31) / 32) <= (int64_t)0x7ffffff0;
}

hipError_t launch_qk_flat(bool scores_only, const void* Q, const void* K, void* out, int64_t BH, int64_t N, int64_t d,
                          float scale, hipStream_t stream)
{
    if (d == 32) return launch_flat_d<64>(scores_only, Q, K, out, BH, (int)N, scale, stream);
    return launch_flat_d<128>(scores_only, Q, K, out, BH, (int)N, scale, stream);
}

}  // namespace attnw
