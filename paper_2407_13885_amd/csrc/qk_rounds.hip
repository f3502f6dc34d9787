// Fused attention weights  P = softmax(scale * Q K^T)  for bf16 problems whose sizes are whole
// multiples of the tiling: the variant that keeps the HBM write stream busy all the time.
//
// The paper's fused kernel (section "Fused Matrix Multiply + Scaling + Softmax") holds a block of
// scores in each core's SRAM, reduces row maxima and sums across the cores of a row and writes only
// the attention weights.  A compute unit here cannot hold a strip of scores, so the scores of a
// strip are produced twice: once for the row statistics (running maximum and sum of exponentials,
// Softmax section, Eq. 1) and once for the weights.  Run one after the other, the two sweeps leave
// the memory system idle during the first and saturated during the second.  This kernel overlaps
// them across strips instead:
//
//   * a persistent workgroup owns a contiguous list of 32*WQ-query strips of one head after another;
//   * one sweep over the keys of the head (a "round") serves TWO strips: slot A = the strip whose
//     statistics are known (its weights are computed, rounded and written), slot B = the next
//     strip (its statistics are gathered).  The K tile staged in LDS and every K fragment read from
//     it feed both slots, so K is fetched once per round, not once per pass;
//   * at the end of a round the statistics of slot B are merged (lane halves, then the WK waves
//     that split the keys of a tile: the paper's local-then-global reduction across a row of
//     cores), slot B's strip moves to slot A and the next strip enters slot B.
// The first round of a list has no slot A and the last one no slot B.
//
// Inside a round, wave (wq, wk) owns queries wq*32 .. +32 of each slot and, of every K tile of
// BN = 64*WK keys, the two 32-key sub-tiles 2*wk, 2*wk+1.  One "step" = one sub-tile:
//   - VALU work on the scores of the current sub-tile (accumulator set `cur`),
//   - the MFMAs of the next sub-tile into the other accumulator set (`nxt`), one per chunk of VALU
//     work, so that the matrix pipe and the vector ALU are fed from the same instruction stream,
//   - the LDS reads of the K fragments of the sub-tile after next (a full step of latency slack).
// As in the two-pass kernel, the MFMA computes the transposed tile (K sub-tile) * (Q block)^T: a
// lane's 16 accumulators are 16 keys of one query.
//
// SCORES = true turns the same machinery into the score GEMM of the unfused pipelines: every round
// is a weights-only round of its own strip with p = scale * s in place of the exponential, no
// statistics and no handover (the staging and store path is what makes it worth sharing).
//
// Stores: slot A's rounded weights are staged in LDS as [query][key] rows and leave as 16 bytes per lane.  With
// rows of 128 bytes (d = 64, 128-query strips) two tiles are staged before they are stored, in an area that
// the two waves which split a tile's keys share: a store instruction then writes 512 contiguous bytes of two
// rows instead of 128 bytes of eight, which the memory system takes at a higher rate.
//
// K tiles travel global -> LDS directly (16 bytes per lane), double buffered.  The transfers are
// issued from inline assembly so that the only waits on them are the explicit vmcnt waits below:
// vector-memory operations retire in order, hence "at most n outstanding" with n = the number of
// younger stores leaves the stores in flight while the tile is known to have landed.
#include "launchers.h"
#include "qk_common.h"

namespace attnw {
namespace {

// PAIR: the weights of TWO consecutive tiles are staged before they are stored, in an area shared by the WK = 2
// waves that split the keys of a tile, so that a store instruction writes 512 contiguous bytes of each of two
// rows instead of 128 bytes of each of eight (measured store rate of that pattern at N = 16384: 6.3 against
// 5.5 TB/s).  Costs one more barrier per pair of tiles: the waves read each other's staged rows.
template <int DB, int WQ, int WK, bool PAIR = false>
struct RoundsCfg {
    static constexpr int SUBS = 2;                // 32-key sub-tiles per wave per K tile
    static constexpr int NBUF = 2;                // K tile buffers in LDS
    static constexpr int NW = WQ * WK;
    static constexpr int BS = 32 * WQ;            // queries per strip
    static constexpr int BN = 32 * SUBS * WK;     // keys per K tile
    static constexpr int G = DB / 32;             // 32-byte contraction groups per row
    static constexpr int CPR = DB / 16;           // 16-byte chunks per K row
    static constexpr int K_TILE_BYTES = BN * DB;
    static constexpr int LOADS = BN * CPR / 64 / NW;   // 1-KiB wave transfers per wave and tile
    static constexpr int SEG = PAIR ? 2 * BN * 2 : 32 * SUBS * 2;   // bytes of one staged row: the wave's keys of one tile, or all keys of two tiles
    static constexpr int ST_PITCH = SEG + 16;
    static constexpr int ST_BYTES = PAIR ? 32 * ST_PITCH / WK : 32 * ST_PITCH;   // per wave (PAIR: a share of the area of its WK waves)
    static constexpr int CPS = SEG / 16;          // chunks per staged row
    static constexpr int RPI = 64 / CPS;          // staged rows one store instruction covers
    static constexpr int NF = PAIR ? 32 / WK / RPI / 2 : 32 / RPI;   // store instructions per tile and wave (PAIR: 32 / WK rows every other tile, half per tile)
    static constexpr int NCH = 2 * G;             // chunks per step (one MFMA each when both slots are live)
    static constexpr int RPL = CPR >= 16 ? 1 : 16 / CPR;
    static constexpr int SWZ_MASK = (CPR >= 16 ? 16 : CPR) - 1;
    static constexpr int LDS_K = NBUF * K_TILE_BYTES;
    static constexpr int LDS_ST = NW * ST_BYTES;
    static constexpr int LDS_STAT = NW * 32 * 2 * 4;
    static constexpr int LDS_TOTAL = LDS_K + LDS_ST + LDS_STAT;
};

template <int DB, int WQ, int WK, bool SCORES, bool PAIR = false>
__global__ __launch_bounds__(64 * WQ * WK)
void qk_rounds_kernel(const uint16_t* __restrict__ Q, const uint16_t* __restrict__ K, uint16_t* __restrict__ out,
                      int N, float c, uint32_t sign_flip, uint32_t strips_per_head, uint32_t total_strips)
{
    using C = RoundsCfg<DB, WQ, WK, PAIR>;
    static_assert(!PAIR || WK == 2, "a pair of tiles is staged by the two waves that split a tile's keys");
    constexpr int SUBS = C::SUBS, NBUF = C::NBUF, NW = C::NW, BS = C::BS, BN = C::BN, G = C::G, CPR = C::CPR;
    constexpr int K_TILE_BYTES = C::K_TILE_BYTES, LOADS = C::LOADS, ST_PITCH = C::ST_PITCH;
    constexpr int ST_BYTES = C::ST_BYTES, CPS = C::CPS, RPI = C::RPI, NF = C::NF, NCH = C::NCH;
    static_assert(SUBS == 2 && NBUF == 2, "accumulator sets, fragment prefetch and buffers alternate per step / tile");
    static_assert(C::LDS_K <= 65536, "the K buffers sit in the first 64 KiB of LDS (transfer base register)");
    static_assert(NCH >= NF + 2 && 16 % NCH == 0, "chunk layout of a step");
    static_assert((BN * CPR) % (64 * NW) == 0, "tile transfer shape");

    __shared__ __align__(1024) char lds[C::LDS_TOTAL];
    char* const k_lds = lds;
    char* const st_lds = lds + C::LDS_K;
    float* const stat_lds = reinterpret_cast<float*>(lds + C::LDS_K + C::LDS_ST);

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wq = wave / WK, wk = wave % WK;
    const int lane = tid & 63;
    const int l32 = lane & 31;
    const int half = lane >> 5;

    // ---- this workgroup's strips: a contiguous range of the global (head, strip) order -------------
    const uint32_t wg = xcd_contiguous_block_id(blockIdx.x, gridDim.x);
    uint32_t s_cur = (uint32_t)((uint64_t)wg * total_strips / gridDim.x);
    const uint32_t s_end = (uint32_t)((uint64_t)(wg + 1) * total_strips / gridDim.x);

    // ---- per-lane constants -------------------------------------------------------------------------
    // K tile transfer: LDS slot s (16 bytes) holds chunk (key, ch) with s = key * CPR + (ch ^ swizzle(key));
    // the swizzle that keeps the fragment reads conflict-free is applied to the global address.
    int goff[LOADS];
#pragma unroll
    for (int j = 0; j < LOADS; ++j) {
        const int s = (wave + NW * j) * 64 + lane;
        const int key = s / CPR;
        const int ch = (s % CPR) ^ ((key / C::RPL) & C::SWZ_MASK);
        goff[j] = key * DB + ch * 16;
    }
    const uint32_t k_lds_base = lds_offset_of(k_lds);
    // fragment g of this wave's sub-tile u of a buffer: k_lds + buffer + u * 32 * DB + frag_off[g]
    int frag_off[G];
    {
        const int swz = (l32 / C::RPL) & C::SWZ_MASK;
#pragma unroll
        for (int g = 0; g < G; ++g) frag_off[g] = (wk * SUBS * 32 + l32) * DB + (((2 * g + half) ^ swz) * 16);
    }
    // staging rows of slot A: written as [query][key] runs of 4 keys, read back 16 bytes per lane
    // PAIR: one area of 32 rows per group of WK waves; a wave writes its keys of every row and reads whole rows
    // 32 / WK * wk .. of it.  Otherwise: a private area per wave.
    char* const stage = PAIR ? st_lds + wq * (32 * ST_PITCH) : st_lds + wave * ST_BYTES;
    const int rd_row0 = PAIR ? wk * (32 / WK) : 0;
    const char* const st_rd = stage + (rd_row0 + lane / CPS) * ST_PITCH + (lane % CPS) * 16;
    char* const st_wr = stage + l32 * ST_PITCH + (PAIR ? wk * (32 * C::SUBS * 2) : 0) + 8 * half;
    constexpr int NFL = PAIR ? 2 * NF : NF;       // staged rows a wave holds in registers between read-back and store
    uint32_t out_lane_off[NFL];
#pragma unroll
    for (int f = 0; f < NFL; ++f) out_lane_off[f] = (uint32_t)(((rd_row0 + f * RPI + lane / CPS) * N + (lane % CPS) * 8) * 2);

    const int n_tiles = N / BN;

    while (s_cur < s_end) {
        // ======== one segment: strips [s0, s1) of head bh ================================================
        const uint32_t bh = s_cur / strips_per_head;
        const uint32_t s0 = s_cur - bh * strips_per_head;
        const uint32_t seg_end = min(s_end, (bh + 1) * strips_per_head);
        const uint32_t s1 = seg_end - bh * strips_per_head;
        s_cur = seg_end;

        const char* Qh = reinterpret_cast<const char*>(Q) + (int64_t)bh * N * DB;
        const char* Kh = reinterpret_cast<const char*>(K) + (int64_t)bh * N * DB;
        char* const out_h = reinterpret_cast<char*>(out) + (int64_t)bh * N * (int64_t)N * 2;
        // Every workgroup starts its sweeps at a different tile and wraps around: with all workgroups
        // marching in step, the rows they write at one moment sit a whole row pitch apart and land on the
        // same few memory channels.
        // (PAIR: an even rotation keeps the two tiles of a staged pair adjacent and 512-byte aligned in the row)
        const int rot = (int)(((bh * strips_per_head + s0) * 7u) % (uint32_t)n_tiles) & (PAIR ? ~1 : ~0);
        // K tile of position t of a round's sweep (0 <= t < n_tiles + NBUF: the prefetch runs into the
        // next round, which walks the same rotated order)
        auto tile_at = [&](int t) __attribute__((always_inline)) {
            int x = t + rot;
            x = x >= n_tiles ? x - n_tiles : x;
            x = x >= n_tiles ? x - n_tiles : x;
            return x;
        };
        auto k_issue = [&](int t, int buf) __attribute__((always_inline)) {
            const char* tile_base = Kh + (int64_t)tile_at(t) * (BN * DB);
#pragma unroll
            for (int i = 0; i < LOADS; ++i)
                dma16_untracked(tile_base + goff[i], k_lds_base + buf * K_TILE_BYTES + (wave + NW * i) * 1024);
        };
        // Q fragments of one strip: lanes 0..31 carry the even 16-byte chunk of each 32-byte group,
        // lanes 32..63 the odd one.  A negative scale negates Q: softmax(-|c| s) = softmax(|c| (-Q) K^T).
        auto load_q = [&](u32x4 (&qf)[G], uint32_t strip) __attribute__((always_inline)) {
            const char* p = Qh + (int64_t)(strip * BS + wq * 32 + l32) * DB + half * 16;
#pragma unroll
            for (int g = 0; g < G; ++g) qf[g] = *reinterpret_cast<const u32x4*>(p + g * 32) ^ sign_flip;
        };

        u32x4 qf[2][G];        // [0] slot A (weights are written), [1] slot B (statistics)
        u32x4 kf[G];           // K fragments of the sub-tile whose MFMAs are issued next
        f32x16 accX[2], accY[2];
        float m_run = kNegBig, mb_run = kNegBig, l_run = 0.0f, bias = 0.0f;
        u32x4 fl[NFL];

        // ---- segment prologue: the transfers of the previous segment have drained, nobody reads LDS ----
        wait_vmem();
        __syncthreads();
#pragma unroll
        for (int b = 0; b < NBUF; ++b) k_issue(b, b);
        load_q(qf[SCORES ? 0 : 1], s0);
        wait_vmem_le<(NBUF - 1) * LOADS>();       // tile 0 (the younger Q loads only make this stricter)
        __syncthreads();

        // One step: see the head of the file.  t = position of the tile in the round's sweep.
        auto step = [&](auto bufc, auto uc, auto hasac, auto hasbc, auto flushc, f32x16 (&cur)[2], f32x16 (&nxt)[2],
                        int t, char* out_prev) __attribute__((always_inline)) {
            constexpr int BUF = decltype(bufc)::value;
            constexpr int U = decltype(uc)::value;
            constexpr bool HAS_A = decltype(hasac)::value != 0;
            constexpr bool HAS_B = decltype(hasbc)::value != 0;
            constexpr bool FLUSH_PREV = decltype(flushc)::value != 0;   // the previous tile's rows are still staged
            constexpr int BUF_NEXT_TILE = (BUF + 1) % NBUF;

            if constexpr (U == 0) {
                // Tile t+1 must have landed for every wave: its fragments are fetched during this tile.
                // Tile t's own buffer was read completely during tile t-1 and takes tile t+NBUF.
                // Younger than the transfer of tile t+1 are the NF stores of the previous tile's rows --
                // unless this round has not issued that many yet.
                // (PAIR: the first stores of a round are issued during its third tile)
                if (HAS_A && t >= NBUF + (PAIR ? 1 : 0)) wait_vmem_le<NF>();
                else wait_vmem();
                __syncthreads();
                k_issue(t + NBUF, BUF);
            }
            __builtin_amdgcn_sched_barrier(0);

            float pv[16];
            uint32_t pk[8];
            float mbl = 0.0f;
            static_for<NCH>([&](auto cic) __attribute__((always_inline)) {
                constexpr int ci = decltype(cic)::value;
                // ---- staged rows of the previous tile: read them all before this step's first staging write
                if constexpr (HAS_A && U == 0 && FLUSH_PREV && ci == 0 && (!PAIR || BUF == 0)) {
#pragma unroll
                    for (int f = 0; f < NFL; ++f) fl[f] = *reinterpret_cast<const u32x4*>(st_rd + f * RPI * ST_PITCH);
                    if constexpr (PAIR) {
                        // the rows were written by both waves of the group and the next pair's first write follows
                        // in this very step: every wave must have its rows in registers first
                        __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0)
                        __syncthreads();
                    }
                }
                // ---- slot A: p = 2^(c*s - (c*m + log2 l)), rounded once, 16 / NCH scores per chunk
                if constexpr (HAS_A) {
                    constexpr int EP = 16 / NCH;
#pragma unroll
                    for (int e = 0; e < EP; ++e) {
                        const int r = ci * EP + e;
                        if constexpr (SCORES) pv[r] = cur[0][r] * c;
                        else pv[r] = fast_exp2(__builtin_fmaf(cur[0][r], c, -bias));
                    }
                    constexpr int r_end = (ci + 1) * EP;
                    if constexpr (r_end % 2 == 0) {
#pragma unroll
                        for (int r = r_end - (EP >= 2 ? EP : 2); r < r_end; r += 2) pk[r / 2] = pack_bf16x2(pv[r], pv[r + 1]);
                    }
                    if constexpr (r_end % 4 == 0) {   // a run of 4 consecutive keys is complete
                        constexpr int r4 = r_end / 4 - 1;
                        u32x2 w = {pk[2 * r4], pk[2 * r4 + 1]};
                        *reinterpret_cast<u32x2*>(st_wr + (PAIR ? BUF * (BN * 2) : 0) + (U * 32 + 8 * r4) * 2) = w;
                    }
                }
                // ---- slot B: running maximum and sum of exponentials (Eq. 1); chunk 0 folds the maximum
                if constexpr (HAS_B) {
                    if constexpr (ci == 0) {
                        float tm = max3(cur[1][0], cur[1][1], cur[1][2]);
#pragma unroll
                        for (int r = 3; r < 15; r += 2) tm = max3(tm, cur[1][r], cur[1][r + 1]);
                        m_run = max3(tm, cur[1][15], m_run);
                        // the sum is kept relative to 2^mb with mb = fl(c * max): rescale by the difference of
                        // the ROUNDED exponents, which is exactly 0 while the maximum stands (a factor built
                        // from the unrounded product would drift the sum by an ulp per step, always the same way)
                        mbl = m_run * c;
                        l_run *= fast_exp2(mb_run - mbl);
                        mb_run = mbl;
                    } else {
                        constexpr int e0 = (ci - 1) * 16 / (NCH - 1), e1 = ci * 16 / (NCH - 1);
                        float ev[e1 - e0];
#pragma unroll
                        for (int r = e0; r < e1; ++r) ev[r - e0] = fast_exp2(__builtin_fmaf(cur[1][r], c, -mbl));
                        float sum = ev[0];
#pragma unroll
                        for (int r = 1; r < e1 - e0; ++r) sum += ev[r];
                        l_run += sum;
                    }
                }
                // ---- stores of the rows read in chunk 0 (past the caches: the weights are not read again)
                if constexpr (HAS_A && U == 0 && FLUSH_PREV && ci >= 2 && ci < 2 + NF) {
                    constexpr int f = (PAIR ? BUF * NF : 0) + ci - 2;   // PAIR: half of the rows per tile of the following pair
                    __builtin_nontemporal_store(fl[f], reinterpret_cast<u32x4*>(out_prev + out_lane_off[f]));
                }
                // ---- one MFMA of the next sub-tile; once both slots have used fragment g, fetch the same
                //      fragment of the sub-tile after next (tile t+1, same U)
                {
                    constexpr int g = ci / 2, slot = ci % 2;
                    if constexpr ((slot == 0 && HAS_A) || (slot == 1 && HAS_B)) {
                        if constexpr (g == 0) {
#pragma unroll
                            for (int r = 0; r < 16; ++r) nxt[slot][r] = 0.0f;
                        }
                        Mma<uint16_t>::run(nxt[slot], kf[g], qf[slot][g]);
                    }
                    if constexpr (slot == 1)
                        kf[g] = *reinterpret_cast<const u32x4*>(k_lds + BUF_NEXT_TILE * K_TILE_BYTES + U * 32 * DB + frag_off[g]);
                }
                // the chunk order is the schedule: keep the compiler from merging chunks
                __builtin_amdgcn_sched_barrier(0);
            });
        };

        auto tile_body = [&](int t, auto bufc, auto hasac, auto hasbc, auto flushc, char* out_rows) __attribute__((always_inline)) {
            char* out_prev = nullptr;
            if constexpr (decltype(hasac)::value != 0 && decltype(flushc)::value != 0) {
                if constexpr (PAIR) out_prev = out_rows + (int64_t)(tile_at(t - 2 - decltype(bufc)::value) * BN) * 2;   // first tile of the pair before
                else out_prev = out_rows + (int64_t)(tile_at(t - 1) * BN + wk * SUBS * 32) * 2;
            }
            step(bufc, IC<0>{}, hasac, hasbc, flushc, accX, accY, t, out_prev);
            step(bufc, IC<1>{}, hasac, hasbc, flushc, accY, accX, t, out_prev);
        };

        // One round: a full sweep over the keys; its first tile sits in buffer 0 (n_tiles is a multiple of NBUF).
        auto round = [&](auto hasac, auto hasbc, char* out_rows) __attribute__((always_inline)) {
            constexpr bool HAS_A = decltype(hasac)::value != 0;
            constexpr bool HAS_B = decltype(hasbc)::value != 0;
            // scores of the first sub-tile with this round's Q fragments, then the fragments of the second
#pragma unroll
            for (int g = 0; g < G; ++g) kf[g] = *reinterpret_cast<const u32x4*>(k_lds + frag_off[g]);
#pragma unroll
            for (int sl = 0; sl < 2; ++sl) {
                if ((sl == 0 && HAS_A) || (sl == 1 && HAS_B)) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) accX[sl][r] = 0.0f;
#pragma unroll
                    for (int g = 0; g < G; ++g) Mma<uint16_t>::run(accX[sl], kf[g], qf[sl][g]);
                }
            }
#pragma unroll
            for (int g = 0; g < G; ++g) kf[g] = *reinterpret_cast<const u32x4*>(k_lds + 32 * DB + frag_off[g]);
            // first group of NBUF tiles: nothing is staged before tile 0
            static_for<NBUF>([&](auto bc) __attribute__((always_inline)) {
                constexpr int b = decltype(bc)::value;
                if constexpr (b == 0 || PAIR) tile_body(b, bc, hasac, hasbc, IC<0>{}, out_rows);
                else tile_body(b, bc, hasac, hasbc, IC<1>{}, out_rows);
            });
            for (int t = NBUF; t < n_tiles; t += NBUF)
                static_for<NBUF>([&](auto bc) __attribute__((always_inline)) {
                    tile_body(t + decltype(bc)::value, bc, hasac, hasbc, IC<1>{}, out_rows);
                });
            // rows of the last tile
            if constexpr (HAS_A && PAIR) {
                // the last pair: every wave's rows of it are staged (barrier), then read by the group's other wave;
                // the second barrier keeps the next round's first staging write behind these reads
                char* out_prev = out_rows + (int64_t)(tile_at(n_tiles - 2) * BN) * 2;
                __syncthreads();
#pragma unroll
                for (int f = 0; f < NFL; ++f) fl[f] = *reinterpret_cast<const u32x4*>(st_rd + f * RPI * ST_PITCH);
                __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0)
                __syncthreads();
#pragma unroll
                for (int f = 0; f < NFL; ++f)
                    __builtin_nontemporal_store(fl[f], reinterpret_cast<u32x4*>(out_prev + out_lane_off[f]));
            } else if constexpr (HAS_A) {
                char* out_prev = out_rows + (int64_t)(tile_at(n_tiles - 1) * BN + wk * SUBS * 32) * 2;
#pragma unroll
                for (int f = 0; f < NF; ++f) {
                    const u32x4 v = *reinterpret_cast<const u32x4*>(st_rd + f * RPI * ST_PITCH);
                    __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(out_prev + out_lane_off[f]));
                }
            }
        };

        // After a round with slot B: merge its statistics (lanes l and l+32 hold the two halves of every
        // query's keys of this wave; the WK waves that share the queries each saw a slice of every
        // tile), fold maximum and normaliser into one constant and hand the strip over to slot A.
        // All exponents are the rounded mb = fl(c * max) the sums were built against.
        auto handover = [&]() __attribute__((always_inline)) {
            const float mo = __shfl_xor(mb_run, 32, 64);
            const float lo = __shfl_xor(l_run, 32, 64);
            float mb = fmaxf(mb_run, mo);
            float l = l_run * fast_exp2(mb_run - mb) + lo * fast_exp2(mo - mb);
            if constexpr (WK > 1) {
                if (half == 0) {
                    stat_lds[(wave * 32 + l32) * 2] = mb;
                    stat_lds[(wave * 32 + l32) * 2 + 1] = l;
                }
                __syncthreads();
#pragma unroll
                for (int o = 1; o < WK; ++o) {
                    const int other = wq * WK + (wk + o) % WK;
                    const float m2 = stat_lds[(other * 32 + l32) * 2];
                    const float l2 = stat_lds[(other * 32 + l32) * 2 + 1];
                    const float mx = fmaxf(mb, m2);
                    l = l * fast_exp2(mb - mx) + l2 * fast_exp2(m2 - mx);
                    mb = mx;
                }
                __syncthreads();      // the exchange buffer is written again after the next round
            }
            bias = mb + fast_log2(l);
#pragma unroll
            for (int g = 0; g < G; ++g) qf[0][g] = qf[1][g];
            m_run = kNegBig;
            mb_run = kNegBig;
            l_run = 0.0f;
        };
        auto rows_of = [&](uint32_t strip) __attribute__((always_inline)) {
            return out_h + (int64_t)(strip * BS + wq * 32) * (int64_t)N * 2;
        };

        if constexpr (SCORES) {
            // scaled scores: no statistics, every round writes its own strip
            for (uint32_t s = s0; s < s1; ++s) {
                if (s > s0) load_q(qf[0], s);
                round(IC<1>{}, IC<0>{}, rows_of(s));
            }
        } else {
            round(IC<0>{}, IC<1>{}, nullptr);                  // first strip: statistics only
            for (uint32_t s = s0 + 1; s < s1; ++s) {
                handover();
                load_q(qf[1], s);
                round(IC<1>{}, IC<1>{}, rows_of(s - 1));
            }
            handover();
            round(IC<1>{}, IC<0>{}, rows_of(s1 - 1));          // last strip: weights only
        }
    }
    wait_vmem();   // no K transfer may be in flight when the workgroup's LDS is released
}

template <int DB, int WQ, int WK, bool SCORES, bool PAIR = false>
hipError_t launch_rounds(const void* Q, const void* K, void* out, int64_t BH, int N, float scale, hipStream_t stream)
{
    using C = RoundsCfg<DB, WQ, WK, PAIR>;
    const uint32_t strips_per_head = (uint32_t)(N / C::BS);
    const uint32_t total = (uint32_t)(BH * strips_per_head);
    uint32_t grid = (uint32_t)((compute_units() + 7) / 8 * 8);
    if (grid > total) grid = (total + 7) / 8 * 8;
    // weights: exponent scale |scale| log2(e) with the sign folded into Q; scores: the scale itself
    const float c = SCORES ? scale : fabsf(scale) * kLog2e;
    const uint32_t flip = (!SCORES && scale < 0.0f) ? Mma<uint16_t>::kSignMask : 0u;
    hipLaunchKernelGGL((qk_rounds_kernel<DB, WQ, WK, SCORES, PAIR>), dim3(grid), dim3(64 * WQ * WK), 0, stream,
                       static_cast<const uint16_t*>(Q), static_cast<const uint16_t*>(K), static_cast<uint16_t*>(out), N, c,
                       flip, strips_per_head, total);
    return hipGetLastError();
}

}  // namespace

// compute units of the current device (persistent workgroups are sized by it); cached per device
int compute_units()
{
    static int cached[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    int n = __atomic_load_n(&cached[dev], __ATOMIC_RELAXED);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        __atomic_store_n(&cached[dev], n, __ATOMIC_RELAXED);
    }
    return n;
}

bool qk_rounds_supported(int64_t BH, int64_t N, int64_t d)
{
    // whole strips of 128 queries, an even number of 128-key tiles, rows of exactly 128 or 256 bytes,
    // strip count and per-head output within 32-bit offsets
    if (d != 64 && d != 128) return false;
    if (N < 256 || (N % 256) != 0 || N > 32768) return false;
    return BH * (N / 128) <= (int64_t)0x7fffffff;
}

hipError_t launch_qk_rounds(bool scores_only, const void* Q, const void* K, void* out, int64_t BH, int64_t N, int64_t d,
                            float scale, hipStream_t stream)
{
    auto go = [&](auto db, auto wq, auto wk) {
        constexpr int DB = decltype(db)::value, WQ = decltype(wq)::value, WK = decltype(wk)::value;
        return scores_only ? launch_rounds<DB, WQ, WK, true>(Q, K, out, BH, (int)N, scale, stream)
                           : launch_rounds<DB, WQ, WK, false>(Q, K, out, BH, (int)N, scale, stream);
    };
    if (d == 64) {
        // Few strips per workgroup: lists of 1 or 2 strips leave some workgroups with twice the work of
        // others and make the statistics-only and weights-only rounds a large share.  Strips of 64 queries
        // (2 x 4 waves, 256-key tiles) double the list lengths; K traffic per element doubles, which small
        // problems can afford.  (d = 128 has no LDS for 256-key tiles.)
        const int64_t strips128 = BH * (N / 128);
        if (strips128 < 4 * (int64_t)compute_units() && (N % 512) == 0) return go(IC<128>{}, IC<2>{}, IC<4>{});
        // 128-query strips: the weights of two tiles are staged before they are stored (512-byte runs per row)
        return scores_only ? launch_rounds<128, 4, 2, true, true>(Q, K, out, BH, (int)N, scale, stream)
                           : launch_rounds<128, 4, 2, false, true>(Q, K, out, BH, (int)N, scale, stream);
    }
    if (scores_only) return hipErrorInvalidValue;   // the caller keeps scores with 256-byte rows on the general kernel
    return launch_rounds<256, 4, 2, false>(Q, K, out, BH, (int)N, scale, stream);
}

}  // namespace attnw
