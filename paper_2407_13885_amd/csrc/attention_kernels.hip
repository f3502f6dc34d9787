// Attention output  O = softmax(scale * Q K^T) V  with the attention weights kept on chip.
//
// The paper's section "Limitations and future Directions" names the product with V as the next thing
// to fuse into its kernel
// (Multi-Head Self-Attention section: Attention(Q, K, V) = softmax(Q K^T / sqrt(d_k)) V).  Once the
// weights are not written, nothing forces two sweeps over the keys: the max-subtracted softmax
// (Softmax section, Eq. 1) is applied incrementally -- a reference exponent that follows the running
// row maximum, a running sum l, and an output accumulator that is rescaled by 2^(old - new) whenever
// the reference moves -- and one sweep over the K and V tiles suffices.
//
// Work split: one workgroup of 8 waves per (head, strip of 8 * QW queries); every wave owns
// QW = 32 * QB queries and walks ALL keys, so no statistics cross waves.  (Problems of a few heads, the
// sizes the paper itself measures, have too few such strips for the chip: there the 8 waves are 2 query
// blocks x 4 key ranges -- a wave takes one 32-key sub-tile of every tile, and the four partial outputs
// of a query block, each with its own reference exponent and sum, are merged through LDS at the end.)
// Per 128-key tile:
//   K tile  [128 keys][d]      global -> LDS directly, chunk-swizzled as in the weight kernels;
//   V tile  transposed on the way into LDS as Vt[d][128 keys]: the second contraction runs over
//           keys, and a matrix-core operand wants its 8 contraction elements contiguous per lane.
// Per 32-key sub-tile and query block (all on v_mfma_f32_32x32x16_bf16, fp32 accumulate):
//   S^T = K_sub * Q^T          lane (query l32, half h) holds keys 8i + 4h + j of its query;
//   sub-tile max (shared by lanes l, l+32: both feed the same second contraction), p = 2^(c s - ref),
//   l += sum p (fp32), p rounded to bf16;
//   O^T += Vt_sub * P^T        lane (query l32, half h) holds O[query][8i + 4h + j] per 32-wide block.
// The k-index of the second contraction is a permutation of the keys chosen so that a lane's own
// 8 weights ARE its operand: slot 8h + e  <->  key 16m + 8 (e / 4) + 4h + e % 4.  Vt stores the keys
// of every 16-group in that order (bits 2 and 3 of the key index swapped).
#include "launchers.h"
#include "qk_common.h"

namespace attnw {
namespace {

// value of the other half-wave's lane (l ^ 32) combined with the own one
__device__ __forceinline__ float half_max(float x)
{
#if defined(__HIP_DEVICE_COMPILE__)
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
#else
    return x;
#endif
}
__device__ __forceinline__ float half_sum(float x)
{
#if defined(__HIP_DEVICE_COMPILE__)
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
#else
    return x;
#endif
}

template <int DB, int QB, int WK = 1>
struct AttnCfg {
    static constexpr int D = DB / 2;              // head dimension
    static constexpr int NW = 8;
    static constexpr int WQ = NW / WK;            // waves along the queries (WK: waves that share a query block)
    static constexpr int QW = 32 * QB;            // queries per wave
    static constexpr int BM = QW * WQ;            // queries per workgroup
    static constexpr int BN = 128;                // keys per tile
    static constexpr int G = DB / 32;             // 32-byte contraction groups per K row
    static constexpr int CPR = DB / 16;           // 16-byte chunks per K / V row
    static constexpr int DVB = D / 32;            // 32-wide blocks of the output row
    static constexpr int K_TILE_BYTES = BN * DB;
    static constexpr int K_LOADS = BN * CPR / 64 / NW;
    static constexpr int V_LOADS = 2 * CPR / NW;  // wave-wide loads of 64 keys x one chunk, per wave and tile
    static constexpr int VT_PITCH = BN * 2 + 16;  // bytes of one Vt row (one output column, 128 keys)
    static constexpr int VT_BYTES = D * VT_PITCH;
    static constexpr int RPL = CPR >= 16 ? 1 : 16 / CPR;
    static constexpr int SWZ_MASK = (CPR >= 16 ? 16 : CPR) - 1;
    // merging the WK partial results of a query block: per wave, reference exponent, sum and output accumulators
    static constexpr int MERGE_SLOTS = 2 + DVB * 16;
    static constexpr int MERGE_BYTES = WK > 1 ? NW * MERGE_SLOTS * 64 * 4 : 0;
    static constexpr int TILE_BYTES = 2 * K_TILE_BYTES + 2 * VT_BYTES;
    static constexpr int LDS_TOTAL = TILE_BYTES > MERGE_BYTES ? TILE_BYTES : MERGE_BYTES;
};

// TAIL: N is not a whole number of tiles / strips.  Rows past the end are read as row N-1 (every load
// stays inside the arrays), their weights are forced to 0 and their queries are not stored.
// PAD:  rows of Q, K, V and O are `rb` < DB bytes long (head sizes that are not 32, 64 or 128); on chip they are
// padded to DB: Q fragments and V columns past the end are zeros, K chunks past the end hold a copy of the row's
// first chunk (finite, and it meets the zero Q fragments), output columns past the end are not stored.
template <int DB, int QB, bool TAIL, bool PAD = false, int WK = 1>
__global__ __launch_bounds__(512)
void attention_kernel(const uint16_t* __restrict__ Q, const uint16_t* __restrict__ K, const uint16_t* __restrict__ V,
                      uint16_t* __restrict__ O, int N, int rb_arg, float c, uint32_t sign_flip, uint32_t strips, uint32_t total, int q_base)
{
    const int rb = PAD ? rb_arg : DB;             // bytes of a row in memory
    using C = AttnCfg<DB, QB, WK>;
    constexpr int NW = C::NW, QW = C::QW, BM = C::BM, BN = C::BN, G = C::G, CPR = C::CPR, DVB = C::DVB;
    constexpr int K_TILE_BYTES = C::K_TILE_BYTES, K_LOADS = C::K_LOADS, V_LOADS = C::V_LOADS;
    constexpr int VT_PITCH = C::VT_PITCH, VT_BYTES = C::VT_BYTES;
    static_assert(2 * K_TILE_BYTES <= 65536, "the K buffers sit in the first 64 KiB of LDS (transfer base register)");
    static_assert((2 * CPR) % NW == 0, "V tile load shape");
    static_assert(WK == 1 || (QB == 1 && 4 % WK == 0), "key ranges: whole sub-tiles of a tile, one query block per wave");

    __shared__ __align__(1024) char lds[C::LDS_TOTAL];
    char* const k_lds = lds;
    char* const vt_lds = lds + 2 * K_TILE_BYTES;

    const uint32_t logical = xcd_contiguous_block_id(blockIdx.x, gridDim.x);
    if (logical >= total) return;
    const uint32_t bh = logical / strips;
    const uint32_t strip = logical - bh * strips;

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int l32 = lane & 31;
    const int half = lane >> 5;

    const char* Qh = reinterpret_cast<const char*>(Q) + (int64_t)bh * N * rb;
    const char* Kh = reinterpret_cast<const char*>(K) + (int64_t)bh * N * rb;
    const char* Vh = reinterpret_cast<const char*>(V) + (int64_t)bh * N * rb;
    char* Oh = reinterpret_cast<char*>(O) + (int64_t)bh * N * rb;
    const int wq = wave / WK, wk = wave % WK;     // query block of the wave, its key range within every tile
    const int q0 = q_base + strip * BM + wq * QW;   // (q_base: the launch covers the strips from that query on)

    auto row_in = [&](int r) __attribute__((always_inline)) { return TAIL ? min(r, N - 1) : r; };

    // ---- Q fragments (a negative scale negates Q) ----------------------------------------------------
    u32x4 qf[QB][G];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
        for (int g = 0; g < G; ++g) {
            u32x4 v = {0u, 0u, 0u, 0u};
            if (!PAD || (2 * g + half) * 16 < rb)
                v = *reinterpret_cast<const u32x4*>(Qh + (int64_t)row_in(q0 + qb * 32 + l32) * rb + (2 * g + half) * 16) ^ sign_flip;
            qf[qb][g] = v;
        }

    // ---- per-lane constants ----------------------------------------------------------------------------
    // K tile transfer j of this lane: key within the tile (recomputed where a clamp needs it), byte offset in the tile
    // (s = (wave + NW j) 64 + lane is transfer j's chunk of the tile: its chunk within the row, and the bits of its key
    // that the swizzle takes, do not depend on j -- one offset per lane and a constant step per transfer, instead of
    // a 64-bit offset register pair per transfer)
    constexpr int KSTEP = NW * 64 / CPR;          // keys between transfers j and j + 1 of a lane
    static_assert((NW * 64) % CPR == 0 && KSTEP % C::RPL == 0 && (KSTEP / C::RPL) % (C::SWZ_MASK + 1) == 0, "K transfer shape");
    auto k_key = [&](int j) __attribute__((always_inline)) { return (wave * 64 + lane) / CPR + KSTEP * j; };
    int k_off0;
    {
        const int s = wave * 64 + lane;
        int ch = (s % CPR) ^ ((k_key(0) / C::RPL) & C::SWZ_MASK);
        if (PAD && ch * 16 >= rb) ch = 0;         // a padding chunk: any finite data of the row
        k_off0 = k_key(0) * rb + ch * 16;
    }
    auto k_off = [&](int j) __attribute__((always_inline)) { return k_off0 + j * KSTEP * rb; };
    const uint32_t k_lds_base = lds_offset_of(k_lds);
    int kfrag_off[G];
    {
        const int swz = (l32 / C::RPL) & C::SWZ_MASK;
#pragma unroll
        for (int g = 0; g < G; ++g) kfrag_off[g] = l32 * DB + (((2 * g + half) ^ swz) * 16);
    }
    // V tile: wave-wide load j covers 64 consecutive keys x one 16-byte chunk (8 output columns); the
    // 8 values go to 8 Vt rows at the key's permuted position (64 lanes -> 128 contiguous bytes per row)
    // (NW is even: the half of the tile is the same for every j, the chunk advances by NW / 2)
    static_assert(NW % 2 == 0, "V load shape");
    const int v_key0 = (wave & 1) * 64 + lane;
    auto v_key = [&](int) __attribute__((always_inline)) { return v_key0; };
    int v_off0, v_ldsoff0;
    {
        const int ch = wave >> 1;
        const int pos = (v_key0 & ~12) | ((v_key0 & 4) << 1) | ((v_key0 & 8) >> 1);   // bits 2 and 3 swapped
        v_off0 = v_key0 * rb + ch * 16;
        v_ldsoff0 = ch * 8 * VT_PITCH + pos * 2;
    }
    auto v_off = [&](int j) __attribute__((always_inline)) { return v_off0 + j * (NW / 2) * 16; };
    auto v_ldsoff = [&](int j) __attribute__((always_inline)) { return v_ldsoff0 + j * (NW / 2) * 8 * VT_PITCH; };
    // Vt fragment of (block dvb, sub-tile u, group m): row dvb*32 + l32, keys u*32 + 16m + 8*half ..
    const int vfrag_off = l32 * VT_PITCH + half * 16;

    const int n_tiles = (N + BN - 1) / BN;
    // rows past the end exist only in the last tile of a TAIL problem: there every row index is clamped
    // (the row a transfer reads moves, its place in LDS does not)
    auto k_issue = [&](int tile, int buf) __attribute__((always_inline)) {
        const char* tile_base = Kh + (int64_t)tile * BN * rb;
        const bool clamp = TAIL && tile == n_tiles - 1;
#pragma unroll
        for (int i = 0; i < K_LOADS; ++i) {
            const char* src = tile_base + k_off(i);
            if (clamp) src -= (int64_t)(tile * BN + k_key(i) - row_in(tile * BN + k_key(i))) * rb;
            dma16_untracked(src, k_lds_base + buf * K_TILE_BYTES + (wave + NW * i) * 1024);
        }
    };
    u32x4 vreg[V_LOADS];
    auto v_load = [&](int tile) __attribute__((always_inline)) {
        const char* tile_base = Vh + (int64_t)tile * BN * rb;
        const bool clamp = TAIL && tile == n_tiles - 1;
#pragma unroll
        for (int j = 0; j < V_LOADS; ++j) {
            const char* src = tile_base + v_off(j);
            if (clamp) src -= (int64_t)(tile * BN + v_key(j) - row_in(tile * BN + v_key(j))) * rb;
            if (PAD && (int)(((wave + NW * j) >> 1) * 16) >= rb) vreg[j] = u32x4{0u, 0u, 0u, 0u};   // columns past the end
            else vreg[j] = *reinterpret_cast<const u32x4*>(src);
        }
    };
    auto v_scatter = [&](int buf) __attribute__((always_inline)) {
        char* base = vt_lds + buf * VT_BYTES;
#pragma unroll
        for (int j = 0; j < V_LOADS; ++j)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint32_t w = vreg[j][e / 2];
                *reinterpret_cast<uint16_t*>(base + v_ldsoff(j) + e * VT_PITCH) = (uint16_t)((e & 1) ? (w >> 16) : (w & 0xffffu));
            }
    };

    f32x16 oacc[QB][DVB];
    float mb_run[QB], l_run[QB];
    constexpr float kLazy = 8.0f;    // binades the maximum may run ahead of the reference exponent
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        mb_run[qb] = kNegBig; l_run[qb] = 0.0f;
#pragma unroll
        for (int b = 0; b < DVB; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[qb][b][r] = 0.0f;
    }

    // one 128-key tile out of buffers `buf`
    // (maskc: the tile runs past N -- only the last tile of a TAIL problem is compiled with the masks)
    auto compute_tile = [&](auto bufc, int t, auto maskc) __attribute__((always_inline)) {
        constexpr int BUF = decltype(bufc)::value;
        constexpr bool MASK = decltype(maskc)::value != 0;
        const char* kb = k_lds + BUF * K_TILE_BYTES;
        const char* vb = vt_lds + BUF * VT_BYTES + vfrag_off;
#pragma unroll
        for (int uu = 0; uu < 4 / WK; ++uu) {
            const int u = wk + WK * uu;           // sub-tiles of this wave
            u32x4 kf[G];
#pragma unroll
            for (int g = 0; g < G; ++g) kf[g] = *reinterpret_cast<const u32x4*>(kb + u * 32 * DB + kfrag_off[g]);
            f32x16 s[QB];
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
#pragma unroll
                for (int r = 0; r < 16; ++r) s[qb][r] = 0.0f;
#pragma unroll
                for (int g = 0; g < G; ++g) Mma<uint16_t>::run(s[qb], kf[g], qf[qb][g]);
            }
            u32x4 vf[DVB][2];
#pragma unroll
            for (int b = 0; b < DVB; ++b)
#pragma unroll
                for (int m = 0; m < 2; ++m)
                    vf[b][m] = *reinterpret_cast<const u32x4*>(vb + b * 32 * VT_PITCH + (u * 32 + 16 * m) * 2);
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                // maximum of this sub-tile, shared by the two lanes of a query
                float tm = max3(s[qb][0], s[qb][1], s[qb][2]);
#pragma unroll
                for (int r = 3; r < 15; r += 2) tm = max3(tm, s[qb][r], s[qb][r + 1]);
                const float mbn = half_max(fmaxf(tm, s[qb][15])) * c;
                // The exponent the weights are taken against (mb_run) follows the running maximum lazily:
                // it moves only when some query of the wave exceeds it by more than kLazy binades.  Until
                // then weights up to 2^kLazy appear, which costs nothing (fp32 sums, and bf16 has the same
                // relative precision at every magnitude), and the 16 * DVB multiplies of the output
                // accumulator - needed at every new maximum otherwise, i.e. in most of the early sub-tiles
                // of a row - become rare.  Lanes whose exponent stands get the factor 2^0 = 1 exactly.
                if (__builtin_amdgcn_ballot_w64(mbn > mb_run[qb] + kLazy) != 0) {
                    const float mb_new = fmaxf(mb_run[qb], mbn);
                    const float alpha = fast_exp2(mb_run[qb] - mb_new);
                    l_run[qb] *= alpha;
#pragma unroll
                    for (int b = 0; b < DVB; ++b)
#pragma unroll
                        for (int r = 0; r < 16; ++r) oacc[qb][b][r] *= alpha;
                    mb_run[qb] = mb_new;
                }
                const float mb = mb_run[qb];
                float p[16];
#pragma unroll
                for (int r = 0; r < 16; ++r) p[r] = fast_exp2(__builtin_fmaf(s[qb][r], c, -mb));
                if constexpr (MASK) {
                    // keys past the end were read as key N-1 (their scores change no maximum): no weight
                    const int kbase = t * BN + u * 32 + 4 * half;
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (kbase + 8 * (r / 4) + (r % 4) >= N) p[r] = 0.0f;
                }
                float sum = p[0];
#pragma unroll
                for (int r = 1; r < 16; ++r) sum += p[r];
                l_run[qb] += sum;
                // a lane's weights of group m are accumulators 8m .. 8m+7: exactly its operand of the second contraction
#pragma unroll
                for (int m = 0; m < 2; ++m) {
                    u32x4 pw;
#pragma unroll
                    for (int i = 0; i < 4; ++i) pw[i] = pack_bf16x2(p[8 * m + 2 * i], p[8 * m + 2 * i + 1]);
#pragma unroll
                    for (int b = 0; b < DVB; ++b) Mma<uint16_t>::run(oacc[qb][b], vf[b][m], pw);
                }
            }
        }
    };

    // ---- prologue: tile 0 --------------------------------------------------------------------------------
    k_issue(0, 0);
    v_load(0);
    v_scatter(0);
    wait_vmem();
    __syncthreads();

    // ---- the sweep: while tile t is computed, K tile t+1 lands in the other buffer and V tile t+1 waits in registers
    auto iteration = [&](int t, auto bufc, auto maskc) __attribute__((always_inline)) {
        constexpr int BUF = decltype(bufc)::value;
        const int nxt = t + 1 < n_tiles ? t + 1 : 0;      // past the end: a valid tile, unused
        k_issue(nxt, BUF ^ 1);
        v_load(nxt);
        // (a wave whose queries all lie past the end -- the last strip of a ragged length -- only moves tiles and meets
        // the barriers: the waves that share its SIMD get the issue slots; measured on 192 heads of N = 577, d = 64:
        // 47.4 -> 43.0 us, 16 heads of N = 4097, d = 128: 249 -> 209 us.  The test stays outside compute_tile -- inside,
        // per query block, it cost the full strips 3-5 % -- and out of the key-range instantiations, which it slowed)
        if (!TAIL || WK > 1 || q0 < N) compute_tile(bufc, t, maskc);
        v_scatter(BUF ^ 1);
        wait_vmem();
        __syncthreads();
    };
    if constexpr (TAIL) {
        for_tiles(0, 0, n_tiles - 1, [&](int t, auto bufc) __attribute__((always_inline)) { iteration(t, bufc, IC<0>{}); });
        if (((n_tiles - 1) & 1) == 0) iteration(n_tiles - 1, IC<0>{}, IC<1>{});
        else iteration(n_tiles - 1, IC<1>{}, IC<1>{});
    } else {
        for (int t = 0; t < n_tiles; t += 2) {      // N is a multiple of two tiles
            iteration(t, IC<0>{}, IC<0>{});
            iteration(t + 1, IC<1>{}, IC<0>{});
        }
    }

    // ---- key ranges: merge the WK partial results of a query block ------------------------------------------------
    // Every wave parks its reference exponent, its sum and its accumulators in LDS (the tile buffers are free: the
    // sweep ended with a barrier); wave (wq, wk) then finishes output blocks wk, wk + WK, ..: with M the largest of
    // the WK exponents, partial j counts with the factor 2^(m_j - M) -- exactly 1 for the largest.
    if constexpr (WK > 1) {
        constexpr int SLOTS = C::MERGE_SLOTS;
        float* const part = reinterpret_cast<float*>(lds);
        float* const mine = part + wave * SLOTS * 64 + lane;
        mine[0] = mb_run[0];
        mine[64] = l_run[0];
#pragma unroll
        for (int b = 0; b < DVB; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) mine[(2 + b * 16 + r) * 64] = oacc[0][b][r];
        __syncthreads();
        const float* const grp = part + wq * WK * SLOTS * 64 + lane;
        float f[WK], M = grp[0];
#pragma unroll
        for (int j = 1; j < WK; ++j) M = fmaxf(M, grp[j * SLOTS * 64]);
        float L = 0.0f;
#pragma unroll
        for (int j = 0; j < WK; ++j) {
            f[j] = fast_exp2(grp[j * SLOTS * 64] - M);
            L = __builtin_fmaf(f[j], grp[j * SLOTS * 64 + 64], L);
        }
        const float inv = 1.0f / half_sum(L);
        if (TAIL && q0 + l32 >= N) return;        // (no barrier follows)
        char* orow = Oh + (int64_t)(q0 + l32) * rb + half * 8;
        for (int b = wk; b < DVB; b += WK)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float o[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    o[e] = 0.0f;
#pragma unroll
                    for (int j = 0; j < WK; ++j) o[e] = __builtin_fmaf(f[j], grp[(j * SLOTS + 2 + b * 16 + 4 * i + e) * 64], o[e]);
                }
                u32x2 w = {pack_bf16x2(o[0] * inv, o[1] * inv), pack_bf16x2(o[2] * inv, o[3] * inv)};
                if (!PAD || (b * 32 + 8 * i) * 2 + half * 8 < rb) *reinterpret_cast<u32x2*>(orow + (b * 32 + 8 * i) * 2) = w;
            }
        return;
    }

    // ---- normalise, round once, store: a lane owns runs of 4 consecutive output columns of its query -----------
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const float inv = 1.0f / half_sum(l_run[qb]);
        if (TAIL && q0 + qb * 32 + l32 >= N) continue;
        char* orow = Oh + (int64_t)(q0 + qb * 32 + l32) * rb + half * 8;
#pragma unroll
        for (int b = 0; b < DVB; ++b)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                u32x2 w = {pack_bf16x2(oacc[qb][b][4 * i] * inv, oacc[qb][b][4 * i + 1] * inv),
                           pack_bf16x2(oacc[qb][b][4 * i + 2] * inv, oacc[qb][b][4 * i + 3] * inv)};
                // (d is a multiple of 16: a run of four columns lies inside the row or past it)
                if (!PAD || (b * 32 + 8 * i) * 2 + half * 8 < rb) *reinterpret_cast<u32x2*>(orow + (b * 32 + 8 * i) * 2) = w;
            }
    }
}

// Queries [q_base, q_end) of every head (q_end < 0: up to N); q_base is a multiple of the strip height.
template <int DB, int QB, bool TAIL, bool PAD = false, int WK = 1>
hipError_t launch_attention_t(const void* Q, const void* K, const void* V, void* O, int64_t BH, int N, float scale,
                              hipStream_t stream, int d = DB / 2, int q_base = 0, int q_end = -1)
{
    using C = AttnCfg<DB, QB, WK>;
    const int rows = (q_end < 0 ? N : q_end) - q_base;
    const uint32_t strips = (uint32_t)((rows + C::BM - 1) / C::BM);
    const uint64_t total = (uint64_t)BH * strips;
    const uint32_t grid = (uint32_t)((total + 7) / 8 * 8);
    const float c = fabsf(scale) * kLog2e;
    const uint32_t flip = scale < 0.0f ? Mma<uint16_t>::kSignMask : 0u;
    hipLaunchKernelGGL((attention_kernel<DB, QB, TAIL, PAD, WK>), dim3(grid), dim3(512), 0, stream, static_cast<const uint16_t*>(Q),
                       static_cast<const uint16_t*>(K), static_cast<const uint16_t*>(V), static_cast<uint16_t*>(O), N, 2 * d,
                       c, flip, strips, (uint32_t)total, q_base);
    return hipGetLastError();
}

// A ragged length whose last strip (256 queries, 512 with two query blocks per wave) holds at most 64 queries, and whose partial strips start another round
// of workgroups on the chip: such a workgroup spends what ONE of its waves spends on a full strip -- the whole sweep
// over the keys -- on a few rows.  The partial strips are left out of the launch and follow as a second one with
// 64-query strips whose keys are spread over four waves (a quarter of the sweep per wave).  Measured: 64 heads of
// N = 2049, d = 64: 146 -> 103 us; 128 heads of N = 1025: 74 -> 66 us; 16 heads of N = 4097, d = 128: 209 -> 202 us
// (33 tiles at the load latency of a tile each: the second launch alone takes 60 us there).
template <int DB, int QB = 1>
hipError_t launch_attention_own_tail(const void* Q, const void* K, const void* V, void* O, int64_t BH, int N, float scale,
                                     hipStream_t stream, bool* taken)
{
    constexpr int BM = 256 * QB;
    const int64_t full = N / BM, tail_rows = N - full * BM;
    const int64_t slots = (int64_t)compute_units() * (DB == 64 && QB == 1 ? 2 : 1);   // (co-resident workgroups: registers)
    *taken = full >= 1 && tail_rows >= 1 && tail_rows <= 64 &&
             (BH * full + slots - 1) / slots < (BH * (full + 1) + slots - 1) / slots;
    if (!*taken) return hipSuccess;
    const hipError_t e = launch_attention_t<DB, QB, true>(Q, K, V, O, BH, N, scale, stream, DB / 2, 0, (int)(full * BM));
    if (e != hipSuccess) return e;
    return launch_attention_t<DB, 1, true, false, 4>(Q, K, V, O, BH, N, scale, stream, DB / 2, (int)(full * BM));
}

}  // namespace

// Problems with at most one 64-query strip per compute unit (twice that for d <= 64): the wide workgroups would leave
// most of the chip without work.  Measured, bf16, wide -> key ranges over waves: one head of d = 128, N = 1024
// 32 -> 19 us, 4096 104 -> 55, 16384 398 -> 227; four heads of N = 4096 106 -> 64 (eight: 111 -> 117, not taken);
// d = 64: one head of N = 4096 70 -> 29, eight heads 75 -> 62, sixteen 85 -> 121 (not taken).
static bool prefers_key_ranges(int64_t BH, int64_t N, int64_t d)
{
    return BH * ((N + 63) / 64) <= (int64_t)compute_units() * (d <= 64 ? 2 : 1);
}

bool attention_supported(int64_t BH, int64_t N, int64_t d)
{
    if (d < 16 || d > 128 || (d % 16) != 0) return false;
    if (N < 1 || N > ((int64_t)1 << 24)) return false;
    return BH * ((N + 255) / 256) <= (int64_t)0x7ffffff0;
}

hipError_t launch_attention(const void* Q, const void* K, const void* V, void* O, int64_t BH, int64_t N, int64_t d,
                            float scale, hipStream_t stream)
{
    // few heads: 64-query strips with the keys of a tile spread over four waves
    if (prefers_key_ranges(BH, N, d)) {
        if (d == 32) return launch_attention_t<64, 1, true, false, 4>(Q, K, V, O, BH, (int)N, scale, stream);
        if (d == 64) return launch_attention_t<128, 1, true, false, 4>(Q, K, V, O, BH, (int)N, scale, stream);
        if (d == 128) return launch_attention_t<256, 1, true, false, 4>(Q, K, V, O, BH, (int)N, scale, stream);
        if (d < 32) return launch_attention_t<64, 1, true, true, 4>(Q, K, V, O, BH, (int)N, scale, stream, (int)d);
        if (d < 64) return launch_attention_t<128, 1, true, true, 4>(Q, K, V, O, BH, (int)N, scale, stream, (int)d);
        return launch_attention_t<256, 1, true, true, 4>(Q, K, V, O, BH, (int)N, scale, stream, (int)d);
    }
    // head sizes between the powers of two: rows padded on chip, in the instantiation that also takes any length
    if (d != 32 && d != 64 && d != 128) {
        if (d <= 32) return launch_attention_t<64, 1, true, true>(Q, K, V, O, BH, (int)N, scale, stream, (int)d);
        if (d <= 64) return launch_attention_t<128, 1, true, true>(Q, K, V, O, BH, (int)N, scale, stream, (int)d);
        return launch_attention_t<256, 1, true, true>(Q, K, V, O, BH, (int)N, scale, stream, (int)d);
    }
    if (d == 32) {          // short rows: two query blocks per wave whenever that leaves enough workgroups
        const bool wide = N >= 2048 && BH * ((N + 511) / 512) >= 200;
        if ((N % 256) != 0) {
            bool taken;
            if (wide) {
                const hipError_t e = launch_attention_own_tail<64, 2>(Q, K, V, O, BH, (int)N, scale, stream, &taken);
                return taken ? e : launch_attention_t<64, 2, true>(Q, K, V, O, BH, (int)N, scale, stream);
            }
            const hipError_t e = launch_attention_own_tail<64>(Q, K, V, O, BH, (int)N, scale, stream, &taken);
            return taken ? e : launch_attention_t<64, 1, true>(Q, K, V, O, BH, (int)N, scale, stream);
        }
        return (wide && (N % 512) == 0) ? launch_attention_t<64, 2, false>(Q, K, V, O, BH, (int)N, scale, stream)
                                        : launch_attention_t<64, 1, false>(Q, K, V, O, BH, (int)N, scale, stream);
    }
    if ((N % 256) != 0) {   // any length: rows past the end are clamped and masked
        bool taken;
        if (d == 128) {
            const hipError_t e = launch_attention_own_tail<256>(Q, K, V, O, BH, (int)N, scale, stream, &taken);
            return taken ? e : launch_attention_t<256, 1, true>(Q, K, V, O, BH, (int)N, scale, stream);
        }
        // (512-query strips only where the rows a last strip leaves unused are a small share)
        if (N >= 2048 && BH * ((N + 511) / 512) >= 200) {
            const hipError_t e = launch_attention_own_tail<128, 2>(Q, K, V, O, BH, (int)N, scale, stream, &taken);
            return taken ? e : launch_attention_t<128, 2, true>(Q, K, V, O, BH, (int)N, scale, stream);
        }
        const hipError_t e = launch_attention_own_tail<128>(Q, K, V, O, BH, (int)N, scale, stream, &taken);
        return taken ? e : launch_attention_t<128, 1, true>(Q, K, V, O, BH, (int)N, scale, stream);
    }
    if (d == 128) return launch_attention_t<256, 1, false>(Q, K, V, O, BH, (int)N, scale, stream);
    // two query blocks per wave (512-query strips) when that still gives every compute unit a workgroup
    if ((N % 512) == 0 && BH * (N / 512) >= 200) return launch_attention_t<128, 2, false>(Q, K, V, O, BH, (int)N, scale, stream);
    return launch_attention_t<128, 1, false>(Q, K, V, O, BH, (int)N, scale, stream);
}

}  // namespace attnw
