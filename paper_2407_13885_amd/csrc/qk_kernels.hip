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
// Work split inside a workgroup of WQ x WK waves: wave (wq, wk) owns QW = 32*QB
// queries (strip rows wq*QW ...) and, of every K tile of BN = 32*SUBS*WK keys,
// the SUBS 32-key sub-tiles wk*SUBS ...; partial row maxima / sums of the WK
// waves that share a query meet once, in LDS, between the passes -- the same
// local-then-global reduction the paper runs across a row of cores.
//
// Orientation: the MFMA computes the TRANSPOSED tile  (K tile) * (Q strip)^T, so
// that a lane's 16 accumulators are 16 keys of ONE query: row reductions stay
// inside the lane (plus one exchange between lanes l and l+32) and every lane
// owns runs of 4 consecutive keys for the store.
#include "launchers.h"
#include "qk_common.h"

#include <cstdlib>
#include <cstring>

namespace attnw {
namespace {

// T      element type (uint16_t = bf16 bits, float)
// DB     padded bytes of one Q/K row held on chip (power of two, >= d * sizeof(T))
// QB     32-query blocks per wave
// WQ,WK  waves along queries / along the keys of a tile
// SUBS   32-key sub-tiles per wave per K tile
// SCORES true: write scale * Q K^T (one pass); false: write the attention weights
// FAST   true: N is a multiple of the strip and of the K tile and rows are exactly
//        DB bytes, so no masking, clamping or store predicate is compiled in
// SPLIT  0: a workgroup sweeps all keys of its strip (both passes).
//        Problems with few strips (one head of a long sequence: the paper's own measurements are
//        on a single head) would leave most compute units idle that way; their keys are cut into
//        `kc_count` ranges of whole tiles, one workgroup per (strip, range), and the two passes
//        become two launches:
//        1: pass one over the workgroup's key range.  The ranges of a row must learn each other's
//           (maximum, sum) and the only memory a call may write is the output: the pair of range
//           k goes into slot k of a small table at the start of the row's piece of EVERY range
//           (kc_count * 8 bytes; a piece is at least two tiles long).
//        2: the workgroup reads, for each of its rows, the table at the start of the row's piece
//           of its OWN range -- nobody else touches that piece during this launch -- folds the
//           pairs into the row's maximum and sum and runs pass two over its range, overwriting
//           the tables with weights.  (The score GEMM needs no statistics: one launch of mode 2.)
// RING   (bf16, ragged lengths; 0 = off, else the bytes of one staging write: 8, 4 or 2.)  A piece of a row as a tile
//        leaves it starts and ends inside memory lines whenever the rows of the output do not start on 64-byte
//        boundaries, and lines written in parts cost a read-modify-write each; rows that do not even start on
//        16-byte boundaries (N not a multiple of 8: odd sequence lengths such as 197, 577, 1025) leave only
//        stores of 8, 4 or 2 bytes per lane.  With RING a wave walks whole tiles (WK = 1) and its staging row is a
//        ring of 16-byte chunks laid out as the row lies in MEMORY: an element goes to the chunk and the position
//        it has there (for rows off the 16-byte boundaries that shifts it by up to 7 elements against the tile,
//        hence the narrower staging writes -- 8 bytes while N is a multiple of 4, 4 while it is even, else 2).
//        After a tile the wave stores, of every row, the 16 chunks that END at the last 64-byte boundary inside
//        what it has computed -- the up to three chunks behind that boundary and the chunk that the next tile
//        completes stay in the ring and leave with the next tile.  Every such store is 16 bytes per lane and
//        covers whole lines.  Chunks that never become whole -- the two ends of a row, which share their chunk
//        with the neighbouring rows, and the place where the rotated sweep of the workgroup started -- are
//        written element by element.
template <typename T, int DB, int QB, int WQ, int WK, int SUBS, bool SCORES, bool FAST, int SPLIT = 0, int RING = 0>
__global__ __launch_bounds__(64 * WQ * WK)
void qk_kernel(const T* __restrict__ Q, const T* __restrict__ K, T* __restrict__ out,
               int N, int d, float c, uint32_t sign_flip, uint32_t strips, uint32_t total_tiles, int kc_count, int q_base)
{
    constexpr int ES = sizeof(T);
    constexpr int EPC = 16 / ES;              // elements per 16-byte chunk
    constexpr int NW = WQ * WK;               // waves per workgroup
    constexpr int QW = 32 * QB;               // queries per wave
    constexpr int BM = QW * WQ;               // queries per workgroup
    constexpr int BN = 32 * SUBS * WK;        // keys per LDS tile
    constexpr int G = DB / 32;                // 32-byte contraction groups per row
    constexpr int CPR = DB / 16;              // chunks per K row in LDS
    constexpr int K_TILE_BYTES = BN * DB;
    constexpr int LOADS = BN * CPR / 64 / NW; // 1-KiB wave loads each wave issues per tile
    constexpr int SEG = 32 * SUBS * ES;       // bytes of one staged row: the wave's keys of one tile
    constexpr int CPS = SEG / 16;             // chunks per staged row
    constexpr int RING_CH = CPS + 5;          // RING: chunks of the ring of a row (a tile, the chunks held back, the chunk it shares with the next)
    constexpr int ST_PITCH = (RING != 0 ? RING_CH * 16 : SEG) + 16;   // padded against bank conflicts
    constexpr int ST_BYTES = QW * ST_PITCH;
    constexpr int RPI = 64 / CPS;             // staged rows one store instruction covers
    constexpr int RPL = CPR >= 16 ? 1 : 16 / CPR;           // K rows per 256-byte LDS line
    constexpr int SWZ_MASK = (CPR >= 16 ? 16 : CPR) - 1;
    static_assert((BN * CPR) % (64 * NW) == 0 && CPS <= 64 && QW % RPI == 0, "tile shape");
    static_assert(RING == 0 || ((RING == 2 || RING == 4 || RING == 8) && !FAST && SPLIT == 0 && WK == 1 && QB == 1 && ES == 2 && CPS % 4 == 0),
                  "ring staging: a wave owns whole tiles of whole lines of 32 rows");

    __shared__ __align__(16) char k_lds0[K_TILE_BYTES];   // the two K tile buffers are separate
    __shared__ __align__(16) char k_lds1[K_TILE_BYTES];   // objects: see dma16
    __shared__ __align__(16) char st_lds[NW * ST_BYTES];
    __shared__ float stat_lds[SCORES ? 2 : NW * QW * 2];

    const uint32_t logical = xcd_contiguous_block_id(blockIdx.x, gridDim.x);
    if (logical >= total_tiles) return;
    uint32_t unit = logical;              // (head, strip) pair; with SPLIT the key range is the fastest index
    int kc = 0;
    if constexpr (SPLIT != 0) {
        kc = (int)(unit % (uint32_t)kc_count);
        unit /= (uint32_t)kc_count;
    }
    const uint32_t bh = unit / strips;
    const uint32_t strip = unit - bh * strips;

    const int tid = threadIdx.x;
    const int wave = tid >> 6;
    const int wq = wave / WK, wk = wave % WK;
    const int lane = tid & 63;
    const int l32 = lane & 31;
    const int half = lane >> 5;

    const int cpr_act = FAST ? CPR : d * ES / 16;   // chunks of real data per row
    const int row_bytes = FAST ? DB : d * ES;
    const char* Qh = reinterpret_cast<const char*>(Q) + (int64_t)bh * N * row_bytes;
    const char* Kh = reinterpret_cast<const char*>(K) + (int64_t)bh * N * row_bytes;
    T* out_h = out + (int64_t)bh * N * N;
    // (q_base: the launch covers the queries from there on -- the last, partial strip of a ragged length can be a
    // launch of its own with a workgroup shape that spreads its keys over the waves)
    const int qw0 = q_base + strip * BM + wq * QW;   // first query of this wave
    char* const stage = st_lds + wave * ST_BYTES;

    // ---- Q fragments: registers for the whole kernel --------------------------------
    u32x4 qf[QB][G];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const int q = qw0 + qb * 32 + l32;
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const int cq = 2 * g + half;
            u32x4 v = {0u, 0u, 0u, 0u};
            if (FAST || (q < N && cq < cpr_act))
                v = *reinterpret_cast<const u32x4*>(Qh + (int64_t)q * row_bytes + cq * 16);
            qf[qb][g] = v ^ sign_flip;        // negative scale: softmax(-|c| s) = softmax(|c| (-Q) K^T)
        }
    }

    // ---- K tiles: global memory -> LDS directly, 16 bytes per lane ------------------------
    // A wave-wide load fills 1 KiB of consecutive LDS; LDS slot s holds chunk
    // (key, ch) with s = key * CPR + (ch ^ swizzle(key)), so the swizzle that keeps
    // the MFMA operand reads conflict-free is applied to the global address.
    int key_of[LOADS], goff[LOADS];
#pragma unroll
    for (int j = 0; j < LOADS; ++j) {
        const int s = (wave + NW * j) * 64 + lane;
        const int key = s / CPR;
        int ch = (s % CPR) ^ ((key / RPL) & SWZ_MASK);
        ch = ch < cpr_act ? ch : 0;           // padding columns are never read: any valid address
        key_of[j] = key;
        goff[j] = key * row_bytes + ch * 16;
    }
    const int n_tiles_all = (N + BN - 1) / BN;
    // this workgroup's tiles: t0 .. t0 + n_tiles (all of them without SPLIT)
    auto range_begin = [&](int k) __attribute__((always_inline)) { return SPLIT != 0 ? n_tiles_all * k / kc_count : 0; };
    const int t0 = range_begin(kc);
    const int n_tiles = SPLIT != 0 ? range_begin(kc + 1) - t0 : n_tiles_all;
    // Every workgroup starts its sweep over the keys at a different tile and wraps
    // around.  With all workgroups marching in step, the rows they write at one moment
    // sit a whole row pitch apart and land on the same few memory channels; the
    // stagger spreads the store stream over all of them.
    const int rot = (int)((logical * 7u) % (uint32_t)n_tiles);
    auto tile_at = [&](int j) __attribute__((always_inline)) { const int t = j + rot; return t0 + (t >= n_tiles ? t - n_tiles : t); };
    auto k_issue = [&](int tile, auto bufc) __attribute__((always_inline)) {
        char* const k_buf = decltype(bufc)::value == 0 ? k_lds0 : k_lds1;
        const int k0 = tile * BN;
        const char* tile_base = Kh + (int64_t)k0 * row_bytes;
#pragma unroll
        for (int j = 0; j < LOADS; ++j) {
            const char* src = tile_base + goff[j];
            if (!FAST && k0 + BN > N) {       // last tile: keys past the end re-read key N-1 (masked later)
                const int kk = min(k0 + key_of[j], N - 1);
                src = Kh + (int64_t)kk * row_bytes + (goff[j] - key_of[j] * row_bytes);
            }
            dma16(src, k_buf + (wave + NW * j) * 1024);
        }
    };

    // scores of 32-key sub-tile `sub` of the tile in `buf`: acc[qb][r] = q . k for key
    // sub*32 + 8*(r/4) + 4*half + r%4 and query qb*32 + l32
    auto mma_subtile = [&](auto bufc, int sub, f32x16 (&acc)[QB]) {
        const int key = sub * 32 + l32;
        const char* rowp = (decltype(bufc)::value == 0 ? k_lds0 : k_lds1) + key * DB;
        const int swz = (key / RPL) & SWZ_MASK;
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[qb][r] = 0.0f;
#pragma unroll
        for (int g = 0; g < G; ++g) {
            // padding columns of short rows hold a copy of chunk 0 of the key (finite) and meet zero Q
            // fragments: no branch here, the loop stays one block the scheduler can interleave
            const u32x4 a = *reinterpret_cast<const u32x4*>(rowp + (((2 * g + half) ^ swz) * 16));
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) Mma<T>::run(acc[qb], a, qf[qb][g]);
        }
    };

    // move the wave's staged QW x (32*SUBS) block to global memory.  Three paths, chosen per wave and
    // tile (wave-uniform): every row and key of the block exists and rows are 16-byte aligned -> NST
    // unconditional 16-byte stores past the caches (the output is far larger than the K of a head, which
    // then stays in L2); aligned rows at an edge -> the same stores predicated; unaligned rows -> one
    // element per lane, a lane-contiguous run of every staged row.  Returns whether the first path ran:
    // only then is the number of store instructions issued known to the wait that follows.
    const bool wave_has_rows = FAST || qw0 < N;
    const bool vec_ok = FAST || (N % EPC) == 0;
    const bool rows_full = FAST || qw0 + QW <= N;
    // rows that do not start on a 64-byte boundary make every 128-byte piece of a store straddle memory
    // lines: such stores go through L2, which merges the pieces before they reach HBM
    const bool past_caches = FAST || (N * ES) % 64 == 0;
    T* const out_lane = out_h + (int64_t)(qw0 + lane / CPS) * N + (lane % CPS) * EPC;
    auto flush_stage = [&](int kseg0) __attribute__((always_inline)) -> bool {
      if constexpr (RING != 0) {
        return false;                         // (the ring has its own flush below)
      } else {
        const bool full = FAST || (rows_full && vec_ok && kseg0 + 32 * SUBS <= N);
        if (full && past_caches) {
#pragma unroll
            for (int it = 0; it < QW / RPI; ++it) {
                const int row = it * RPI + lane / CPS;
                const u32x4 v = *reinterpret_cast<const u32x4*>(stage + row * ST_PITCH + (lane % CPS) * 16);
                __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(out_lane + (int64_t)(it * RPI) * N + kseg0));
            }
        } else if (full) {
#pragma unroll
            for (int it = 0; it < QW / RPI; ++it) {
                const int row = it * RPI + lane / CPS;
                const u32x4 v = *reinterpret_cast<const u32x4*>(stage + row * ST_PITCH + (lane % CPS) * 16);
                *reinterpret_cast<u32x4*>(out_lane + (int64_t)(it * RPI) * N + kseg0) = v;
            }
        } else if (vec_ok) {
#pragma unroll
            for (int it = 0; it < QW / RPI; ++it) {
                const int row = it * RPI + lane / CPS;
                const u32x4 v = *reinterpret_cast<const u32x4*>(stage + row * ST_PITCH + (lane % CPS) * 16);
                if (qw0 + row < N && kseg0 + (lane % CPS) * EPC < N)
                    *reinterpret_cast<u32x4*>(out_lane + (int64_t)(it * RPI) * N + kseg0) = v;
            }
        } else {
            // rows off the 16-byte boundaries: groups of GB = 8, 4 or sizeof(T) bytes, the largest that the row
            // length is a multiple of (rows then start on multiples of it); a lane-contiguous run of every staged row
            auto store_groups = [&](auto gbc) __attribute__((always_inline)) {
                constexpr int GB = decltype(gbc)::value;          // bytes per lane
                constexpr int EG = GB / ES;                       // elements per lane
                constexpr int LPR = SEG / GB;                     // lanes per staged row
                constexpr int RPE = 64 / LPR;                     // staged rows one instruction covers
                static_assert(LPR <= 64 && QW % RPE == 0, "group store shape");
#pragma unroll 4
                for (int it = 0; it < QW / RPE; ++it) {
                    const int row = it * RPE + lane / LPR;
                    const int e = (lane % LPR) * EG;
                    const char* from = stage + row * ST_PITCH + e * ES;
                    T* to = out_h + (int64_t)(qw0 + row) * N + kseg0 + e;
                    if (qw0 + row < N && kseg0 + e < N) {         // (N is a multiple of EG: a group is inside or outside)
                        if constexpr (GB == 8) *reinterpret_cast<u32x2*>(to) = *reinterpret_cast<const u32x2*>(from);
                        else if constexpr (GB == 4) *reinterpret_cast<uint32_t*>(to) = *reinterpret_cast<const uint32_t*>(from);
                        else *to = *reinterpret_cast<const T*>(from);
                    }
                }
            };
            const int row_bytes_out = N * ES;
            if (row_bytes_out % 8 == 0) store_groups(IC<8>{});
            else if (ES == 2 && row_bytes_out % 4 == 0) store_groups(IC<4>{});
            else store_groups(IC<ES>{});
        }
        return full;
      }
    };
    // RING.  With o(r) = the element index of row r's first element in memory mod 8 and a(r) = its 16-byte chunk
    // index mod 4, element k of the j-th tile of the sweep (tile index t) lies in ring chunk
    // (CPS j + (k + o) / 8) mod RING_CH at position (k + o) % 8.  Window of row r after that tile: the CPS chunks
    // that start a(r) chunks before the chunk of the tile's first element, i.e. on a 64-byte boundary; `tail`: the
    // window after that one, what the tile has left behind -- after the last tile of a row (whose successor in the
    // rotated sweep is tile 0) and at the end of the sweep.  Chunk i of the window starts at row element
    // key0 = BN t + 8 (i - a) - o; available are the elements from BN t on (from the tile before on, if that was the
    // previous one of the sweep) up to the end of the tile or of the row.  A lane takes chunk i = lane % CPS of row
    // lane / CPS of every group of RPI rows.  Returns whether exactly NST unconditional stores were issued.
    int ring_p = 0;                           // ring chunk of the first element of the tile whose values are being staged
    auto ring_flush = [&](int j, bool tail) __attribute__((always_inline)) -> bool {
        const int pj = (CPS * j) % RING_CH;
        const int t = tile_at(j);
        const bool chained = j >= 1 && t >= 1;                 // the tile before in memory was the one before in the sweep
        const bool interior = !tail && chained && rows_full && (t + 1) * BN <= N;   // every chunk of every window is whole
        const int avail_lo = chained ? -(1 << 20) : t * BN;
        const int avail_hi = min(N, (t + 1) * BN);
#pragma unroll
        for (int it = 0; it < QW / RPI; ++it) {
            const int row = it * RPI + lane / CPS;
            const int i = lane % CPS + (tail ? CPS : 0);
            T* const row_ptr = out_h + (int64_t)(qw0 + row) * N;
            const int a = (int)((reinterpret_cast<uintptr_t>(row_ptr) >> 4) & 3);
            const int o = (int)((reinterpret_cast<uintptr_t>(row_ptr) >> 1) & 7);
            int x = pj - a + i;                // -3 .. 2 CPS + RING_CH
            x = x < 0 ? x + RING_CH : x;
            x = x >= RING_CH ? x - RING_CH : x;
            x = x >= RING_CH ? x - RING_CH : x;
            const int key0 = t * BN + (i - a) * EPC - o;
            const u32x4 v = *reinterpret_cast<const u32x4*>(stage + row * ST_PITCH + x * 16);
            if (interior) {
                __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(row_ptr + key0));
            } else if (qw0 + row < N) {
                const int lo = max(0, avail_lo - key0), hi = min(EPC, avail_hi - key0);
                if (lo == 0 && hi == EPC) {
                    *reinterpret_cast<u32x4*>(row_ptr + key0) = v;
                } else {
#pragma unroll
                    for (int e = 0; e < EPC; ++e)
                        if (e >= lo && e < hi) row_ptr[key0 + e] = (T)((e & 1) ? (v[e / 2] >> 16) : (v[e / 2] & 0xffffu));
                }
            }
        }
        return interior;
    };
    // the lane's row (QB = 1): where its 4 consecutive keys of a chunk pair land
    int ring_sel = 0, ring_off = 0;           // s = 4 half + o(r): element s + i of the pair of chunks (B, B + 1)
    if constexpr (RING != 0) {
        const int o = (int)((reinterpret_cast<uintptr_t>(out_h + (int64_t)(qw0 + l32) * N) >> 1) & 7);
        ring_sel = 4 * half + o;
        ring_off = l32 * ST_PITCH;
    }
    auto stage_put4 = [&](int qb, int u, int r4, float v0, float v1, float v2, float v3) __attribute__((always_inline)) {
        char* p = stage + (qb * 32 + l32) * ST_PITCH + (u * 32 + 8 * r4 + 4 * half) * ES;
        if constexpr (RING != 0) {
            int b0 = ring_p + (u * 32 + 8 * r4) * ES / 16;          // wave-uniform: chunk of the pair's first element for o = 0
            b0 = b0 >= RING_CH ? b0 - RING_CH : b0;
            const int b1 = b0 + 1 >= RING_CH ? 0 : b0 + 1;
            const uint32_t w01 = pack_bf16x2(v0, v1), w23 = pack_bf16x2(v2, v3);
            char* const rowp = stage + ring_off;
            auto at = [&](int i) __attribute__((always_inline)) {   // element ring_sel + i
                const int e = ring_sel + i;
                return rowp + (e >= 8 ? b1 : b0) * 16 + (e & 7) * 2;
            };
            if constexpr (RING == 8) {
                *reinterpret_cast<u32x2*>(at(0)) = u32x2{w01, w23};
            } else if constexpr (RING == 4) {
                *reinterpret_cast<uint32_t*>(at(0)) = w01;
                *reinterpret_cast<uint32_t*>(at(2)) = w23;
            } else {
                *reinterpret_cast<uint16_t*>(at(0)) = (uint16_t)(w01 & 0xffffu);
                *reinterpret_cast<uint16_t*>(at(1)) = (uint16_t)(w01 >> 16);
                *reinterpret_cast<uint16_t*>(at(2)) = (uint16_t)(w23 & 0xffffu);
                *reinterpret_cast<uint16_t*>(at(3)) = (uint16_t)(w23 >> 16);
            }
            return;
        }
        if constexpr (ES == 2) {
            u32x2 w = {pack_bf16x2(v0, v1), pack_bf16x2(v2, v3)};
            *reinterpret_cast<u32x2*>(p) = w;
        } else {
            u32x4 w = {__float_as_uint(v0), __float_as_uint(v1), __float_as_uint(v2), __float_as_uint(v3)};
            *reinterpret_cast<u32x4*>(p) = w;
        }
    };

    float m_run[QB], l_run[QB], bias[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) { m_run[qb] = kNegBig; l_run[qb] = 0.0f; bias[qb] = 0.0f; }

    // pass one on the scores of one 32-key sub-tile: running maximum and sum of
    // exponentials (Eq. 1), kept per lane; kbase = first key of this lane's first run
    auto fold_stats = [&](f32x16 (&acc)[QB], int kbase, auto tailc) {
        constexpr bool tail = decltype(tailc)::value != 0;   // this tile holds keys past N
        if constexpr (tail) {
            // (wave-uniform: lane 0's kbase is the sub-tile's first key) a sub-tile wholly past N adds nothing
            if (__builtin_amdgcn_readfirstlane(kbase) >= N) return;
        }
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            if constexpr (tail) {
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
                // fp32 results are held to an absolute bound: subtract first so that a
                // large common offset cancels exactly
                float e = (ES == 4) ? fast_exp2((acc[qb][r] - mn) * c) : fast_exp2(__builtin_fmaf(acc[qb][r], c, -mb));
                if constexpr (tail) {
                    if (kbase + 8 * (r / 4) + (r % 4) >= N) e = 0.0f;
                }
                sum += e;
            }
            l_run[qb] += sum;
        }
    };
    // pass two (or the score GEMM) on one sub-tile: final values, rounded, into the staging rows
    auto emit = [&](f32x16 (&acc)[QB], int u) {
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                float p[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float sc = acc[qb][4 * r4 + i];
                    if constexpr (SCORES) p[i] = sc * c;
                    else if constexpr (ES == 4) p[i] = fast_exp2(__builtin_fmaf(sc - m_run[qb], c, -bias[qb]));
                    else p[i] = fast_exp2(__builtin_fmaf(sc, c, -bias[qb]));   // 2^(c*s - c*m - log2 l)
                }
                stage_put4(qb, u, r4, p[0], p[1], p[2], p[3]);
            }
    };

    // ---- the sweep -------------------------------------------------------------------------
    // The K tiles of both passes form one sequence s = 0 .. S-1 (tile_at(s mod n_tiles),
    // LDS buffer s & 1).  A wave always has two things in flight: the MFMAs of its next
    // sub-tile and the VALU work on the scores of the previous one (two accumulator sets),
    // also across the workgroup barrier that ends a tile -- a wave that issued only
    // MFMAs, or only VALU work, between two barriers would leave the other unit idle.
    //   body(s):  [store the rows staged during s-1]
    //             for u < SUBS-1:  MFMA(s, u+1)  ||  VALU(s, u)
    //             wait for the DMA of tile s+1, barrier, start the DMA of tile s+2
    //             MFMA(s+1, 0)  ||  VALU(s, SUBS-1)
    constexpr int NST = QW / RPI;             // store instructions per flush
    f32x16 acc_a[QB], acc_b[QB];              // accumulator set of sub-tile u of buffer b: (b*SUBS + u) & 1
    auto acc_of = [&](auto slotc) __attribute__((always_inline)) -> f32x16 (&)[QB] {
        if constexpr ((decltype(slotc)::value & 1) == 0) return acc_a; else return acc_b;
    };

    // (maximum, sum) table of query q in the piece of key range k: pairs of floats at the first 4-byte boundary of the
    // piece (accessed as single floats; a piece of an odd-length bf16 row may start 2 bytes before it)
    auto table_of = [&](int q, int k) __attribute__((always_inline)) {
        char* const piece = reinterpret_cast<char*>(out_h) + ((int64_t)q * N + (int64_t)range_begin(k) * BN) * ES;
        return reinterpret_cast<float*>((reinterpret_cast<uintptr_t>(piece) + 3) & ~(uintptr_t)3);
    };
    if constexpr (SPLIT == 2 && !SCORES) {
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            const int q = qw0 + qb * 32 + l32;
            float mn = kNegBig, l = 0.0f;
            if (FAST || q < N) {
                const float* tab = table_of(q, kc);
                for (int k = 0; k < kc_count; ++k) {
                    const float pm = tab[2 * k], pl = tab[2 * k + 1];
                    const float mx = fmaxf(mn, pm);
                    l = l * fast_exp2((mn - mx) * c) + pl * fast_exp2((pm - mx) * c);
                    mn = mx;
                }
            } else {
                l = 1.0f;                     // a row past the end: nothing of it is stored
            }
            m_run[qb] = mn;
            bias[qb] = (ES == 4) ? fast_log2(l) : __builtin_fmaf(mn, c, fast_log2(l));
        }
    }

    k_issue(tile_at(0), IC<0>{});
    wait_vmem();       // (mode 2: also the table reads above -- they must be done before anyone stores)
    __syncthreads();
    k_issue(tile_at(1 % n_tiles), IC<1>{});
    mma_subtile(IC<0>{}, wk * SUBS, acc_of(IC<0>{}));

    // Nothing in a body depends on whether a next tile exists: past the end of the sequence
    // the extra DMA re-reads a valid tile and the extra MFMAs chew on stale LDS, both
    // unused -- a branch there would split the block the scheduler interleaves.
    auto body = [&](int j, auto bufc, auto writec, auto flushc, auto tailc) __attribute__((always_inline)) {
        constexpr int B = decltype(bufc)::value;
        constexpr bool WRITE = decltype(writec)::value != 0;   // this tile's results go to memory
        constexpr bool FLUSH = decltype(flushc)::value != 0;   // the previous tile's are still staged
        const int k0 = tile_at(j) * BN;
        bool counted = false;                                  // exactly NST stores were issued by this body
        if constexpr (FLUSH) {
            if constexpr (RING != 0) {
                counted = ring_flush(j - 1, false);
                if (tile_at(j - 1) == n_tiles - 1) {   // the sweep wraps to tile 0: nothing may stay behind
                    ring_flush(j - 1, true);
                    counted = false;
                }
            } else {
                counted = flush_stage(tile_at(j - 1) * BN + wk * SUBS * 32);
            }
        }
        if constexpr (RING != 0) ring_p = (CPS * j) % RING_CH;
        // (a wave whose queries all lie past the end -- the last strip of a ragged length -- only moves K tiles and
        //  meets the barriers: the strip then costs its workgroup a fraction of a full one)
        if (wave_has_rows) {
            static_for<SUBS - 1>([&](auto uc) __attribute__((always_inline)) {
                constexpr int u = decltype(uc)::value;
                mma_subtile(bufc, wk * SUBS + u + 1, acc_of(IC<B * SUBS + u + 1>{}));
                if constexpr (WRITE) emit(acc_of(IC<B * SUBS + u>{}), u);
                else fold_stats(acc_of(IC<B * SUBS + u>{}), k0 + (wk * SUBS + u) * 32 + 4 * half, tailc);
            });
        }
        // The DMA of tile s+1 is older than this body's stores and memory operations
        // retire in order, so the wait can leave the NST stores in flight.
        if constexpr (FAST && FLUSH) {
            wait_vmem_le<NST>();
        } else {
            if (!counted) wait_vmem();
            wait_vmem_le<NST>();
        }
        __syncthreads();
        k_issue(tile_at(j + 2 < n_tiles ? j + 2 : j + 2 - n_tiles), bufc);   // this tile's buffer is free now
        // Pin the transfer here: left alone, the scheduler sinks it to the end of the block,
        // right in front of the wait that needs it, and its whole latency is exposed.
        __builtin_amdgcn_sched_barrier(0);
        if (wave_has_rows) {
            mma_subtile(IC<1 - B>{}, wk * SUBS, acc_of(IC<(1 - B) * SUBS>{}));
            if constexpr (WRITE) emit(acc_of(IC<B * SUBS + SUBS - 1>{}), SUBS - 1);
            else fold_stats(acc_of(IC<B * SUBS + SUBS - 1>{}), k0 + (wk * SUBS + SUBS - 1) * 32 + 4 * half, tailc);
        }
    };
    // pass-one body of tile j: the instantiation with key masks only where the tile runs past N
    auto stats_body = [&](int j, auto bufc) __attribute__((always_inline)) {
        if constexpr (FAST) {
            body(j, bufc, IC<0>{}, IC<0>{}, IC<0>{});
        } else {
            if (tile_at(j) * BN + BN > N) body(j, bufc, IC<0>{}, IC<0>{}, IC<1>{});
            else body(j, bufc, IC<0>{}, IC<0>{}, IC<0>{});
        }
    };

    if constexpr (!SCORES && SPLIT != 2) {
        // ================= pass one =================================================================
        for_tiles(0, 0, n_tiles, stats_body);

        // lanes l and l+32 hold the two halves of each query's keys of this wave; the WK
        // waves that share these queries each saw a different slice of every tile
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            const float mo = __shfl_xor(m_run[qb], 32, 64);
            const float lo = __shfl_xor(l_run[qb], 32, 64);
            const float mn = fmaxf(m_run[qb], mo);
            l_run[qb] = l_run[qb] * fast_exp2((m_run[qb] - mn) * c) + lo * fast_exp2((mo - mn) * c);
            m_run[qb] = mn;
            if (WK > 1 && half == 0) {
                stat_lds[(wave * QW + qb * 32 + l32) * 2] = mn;
                stat_lds[(wave * QW + qb * 32 + l32) * 2 + 1] = l_run[qb];
            }
        }
        if constexpr (WK > 1) __syncthreads();
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            float mn = m_run[qb], l = l_run[qb];
            if constexpr (WK > 1) {
#pragma unroll
                for (int o = 1; o < WK; ++o) {
                    const int other = wq * WK + (wk + o) % WK;
                    const float mo = stat_lds[(other * QW + qb * 32 + l32) * 2];
                    const float lo = stat_lds[(other * QW + qb * 32 + l32) * 2 + 1];
                    const float mx = fmaxf(mn, mo);
                    l = l * fast_exp2((mn - mx) * c) + lo * fast_exp2((mo - mx) * c);
                    mn = mx;
                }
            }
            m_run[qb] = mn;
            // bf16: bias = c*m + log2(l) folds max and normaliser into one constant;
            // fp32: the max is subtracted separately, bias = log2(l)
            bias[qb] = (ES == 4) ? fast_log2(l) : __builtin_fmaf(mn, c, fast_log2(l));
            if constexpr (SPLIT == 1) {
                // this range's pair into slot kc of the row's table in every range (one lane per query)
                const int q = qw0 + qb * 32 + l32;
                if (wk == 0 && half == 0 && (FAST || q < N)) {
                    for (int k = 0; k < kc_count; ++k) {
                        float* tab = table_of(q, k);
                        tab[2 * kc] = mn;
                        tab[2 * kc + 1] = l;
                    }
                }
            }
        }
    }
    if constexpr (SPLIT == 1) {
        wait_vmem();       // no K transfer may be in flight when the workgroup's LDS is released
        return;
    }

    // ================= pass two (or the only pass of the score GEMM): compute, round, store ========
    // pass one consumed n_tiles buffers, so the first tile of this pass sits in buffer n_tiles & 1
    const int b0 = (SCORES || SPLIT == 2) ? 0 : (n_tiles & 1);
    if (b0 == 0) body(0, IC<0>{}, IC<1>{}, IC<0>{}, IC<0>{}); else body(0, IC<1>{}, IC<1>{}, IC<0>{}, IC<0>{});
    for_tiles(1, b0 ^ 1, n_tiles, [&](int j, auto bufc) __attribute__((always_inline)) { body(j, bufc, IC<1>{}, IC<1>{}, IC<0>{}); });
    wait_vmem();
    if constexpr (RING != 0) {
        ring_flush(n_tiles - 1, false);
        ring_flush(n_tiles - 1, true);        // the chunks held back behind the last 64-byte boundary
    } else {
        flush_stage(tile_at(n_tiles - 1) * BN + wk * SUBS * 32);
    }
}

// Key ranges per strip for a problem of `units` (head, strip) pairs whose rows have n_tiles K tiles: 1 (no
// split) when the strips alone give at least half of the compute units a workgroup; else enough ranges of
// at least two tiles for about two workgroups per compute unit, at most 16 (the table of a row is
// 8 bytes per range and sits inside the first tile of a piece).
int key_ranges(int64_t units, int n_tiles)
{
    const int64_t cus = compute_units();
    if (2 * units >= cus) return 1;
    int64_t k = (2 * cus + units - 1) / units;
    if (k > n_tiles / 2) k = n_tiles / 2;
    if (k > 16) k = 16;
    return k < 2 ? 1 : (int)k;
}

template <typename T, int DB, int QB, int WQ, int WK, int SUBS, bool FAST, bool SPLITTABLE>
hipError_t launch_variant(bool scores_only, const void* Q, const void* K, void* out, int64_t BH, int N, int d,
                          float scale, hipStream_t stream, bool allow_split)
{
    constexpr int BM = 32 * QB * WQ, BN = 32 * SUBS * WK;
    constexpr int threads = 64 * WQ * WK;
    const uint32_t strips = (uint32_t)((N + BM - 1) / BM);
    const T* q = static_cast<const T*>(Q);
    const T* k = static_cast<const T*>(K);
    T* o = static_cast<T*>(out);
    const float c = scores_only ? scale : fabsf(scale) * kLog2e;
    const uint32_t flip = (!scores_only && scale < 0.0f) ? Mma<T>::kSignMask : 0u;
    if constexpr (SPLITTABLE) {
        const int kc = allow_split ? key_ranges(BH * strips, (N + BN - 1) / BN) : 1;
        if (kc > 1) {
            const uint64_t total = (uint64_t)BH * strips * kc;
            if (total > 0x7ffffff0u) return hipErrorInvalidValue;
            const uint32_t grid = (uint32_t)((total + 7) / 8 * 8);
            if (scores_only) {
                hipLaunchKernelGGL((qk_kernel<T, DB, QB, WQ, WK, SUBS, true, FAST, 2>), dim3(grid), dim3(threads), 0,
                                   stream, q, k, o, N, d, c, flip, strips, (uint32_t)total, kc, 0);
            } else {
                hipLaunchKernelGGL((qk_kernel<T, DB, QB, WQ, WK, SUBS, false, FAST, 1>), dim3(grid), dim3(threads), 0,
                                   stream, q, k, o, N, d, c, flip, strips, (uint32_t)total, kc, 0);
                hipLaunchKernelGGL((qk_kernel<T, DB, QB, WQ, WK, SUBS, false, FAST, 2>), dim3(grid), dim3(threads), 0,
                                   stream, q, k, o, N, d, c, flip, strips, (uint32_t)total, kc, 0);
            }
            return hipGetLastError();
        }
    }
    const uint64_t total = (uint64_t)BH * strips;
    const uint32_t grid = (uint32_t)((total + 7) / 8 * 8);
    if (scores_only)
        hipLaunchKernelGGL((qk_kernel<T, DB, QB, WQ, WK, SUBS, true, FAST>), dim3(grid), dim3(threads), 0, stream, q, k,
                           o, N, d, c, flip, strips, (uint32_t)total, 1, 0);
    else
        hipLaunchKernelGGL((qk_kernel<T, DB, QB, WQ, WK, SUBS, false, FAST>), dim3(grid), dim3(threads), 0, stream, q,
                           k, o, N, d, c, flip, strips, (uint32_t)total, 1, 0);
    return hipGetLastError();
}

template <typename T, int DB, int QB, int WQ, int WK, int SUBS, bool SPLITTABLE = false>
hipError_t launch_shape(bool scores_only, const void* Q, const void* K, void* out, int64_t BH, int N, int d,
                        float scale, hipStream_t stream, bool allow_split = false)
{
    constexpr int BM = 32 * QB * WQ, BN = 32 * SUBS * WK;
    // whole strips, whole K tiles, unpadded rows: the variant without masks and predicates
    if (N % BM == 0 && N % BN == 0 && d * (int)sizeof(T) == DB)
        return launch_variant<T, DB, QB, WQ, WK, SUBS, true, SPLITTABLE>(scores_only, Q, K, out, BH, N, d, scale, stream, allow_split);
    return launch_variant<T, DB, QB, WQ, WK, SUBS, false, SPLITTABLE>(scores_only, Q, K, out, BH, N, d, scale, stream, allow_split);
}

// bf16, ragged lengths: 256-query strips, a wave per 32 queries that walks whole 128-key tiles and stores whole
// memory lines out of a ring laid out as the rows lie in memory (RING in qk_kernel).
template <int DB, int GRAN, int WQ>
hipError_t launch_ring_t(bool scores_only, const void* Q, const void* K, void* out, int64_t BH, int N, int d, float scale,
                         hipStream_t stream)
{
    constexpr int BM = 32 * WQ;
    uint32_t strips = (uint32_t)((N + BM - 1) / BM);
    const uint16_t* q = static_cast<const uint16_t*>(Q);
    const uint16_t* k = static_cast<const uint16_t*>(K);
    uint16_t* o = static_cast<uint16_t*>(out);
    const float c = scores_only ? scale : fabsf(scale) * kLog2e;
    const uint32_t flip = (!scores_only && scale < 0.0f) ? Mma<uint16_t>::kSignMask : 0u;
    // The last strip of a ragged length holds N % BM queries, and a workgroup of this shape spends on it what one of
    // its waves spends on a full strip (the waves without queries only help with the K tiles): about half the
    // time of a full workgroup.  Where those workgroups make the difference between one more round of workgroups
    // on the chip and none (N = 4104, 16 heads: 272 workgroups of 256-query strips on 256 compute units), the last
    // strip becomes a launch of its own: 32-query strips whose keys are spread over the 8 waves of a workgroup.
    // Measured, fused / scores in us, B1 H16 d = 128: N = 4104 296 / 226 -> 251 / 141, 4097 322 / 201 -> 266 / 156, 4100
    // 294 / 175 -> 222 / 139, 8200 929 -> 830 (4072, 16 full strips and nothing else: 203 - 210 / 131); 128 heads of N = 513,
    // d = 32: 53 -> 39.
    const int tail_rows = N % BM;
    const int64_t slots = (int64_t)compute_units() * (WQ == 8 ? 1 : 2);
    const int64_t full = BH * (int64_t)(N / BM);
    const bool own_tail = tail_rows != 0 && tail_rows <= 96 && full > 0 &&
                          (full + slots - 1) / slots < (full + BH + slots - 1) / slots;
    if (own_tail) strips -= 1;
    const uint64_t total = (uint64_t)BH * strips;
    const uint32_t grid = (uint32_t)((total + 7) / 8 * 8);
    if (scores_only)
        hipLaunchKernelGGL((qk_kernel<uint16_t, DB, 1, WQ, 1, 4, true, false, 0, GRAN>), dim3(grid), dim3(64 * WQ), 0, stream,
                           q, k, o, N, d, c, flip, strips, (uint32_t)total, 1, 0);
    else
        hipLaunchKernelGGL((qk_kernel<uint16_t, DB, 1, WQ, 1, 4, false, false, 0, GRAN>), dim3(grid), dim3(64 * WQ), 0, stream,
                           q, k, o, N, d, c, flip, strips, (uint32_t)total, 1, 0);
    if (own_tail) {
        // 32-query strips, the 128 keys of a tile over 4 waves; with so few strips their keys are split over workgroups as
        // for problems of a few heads (SPLIT in qk_kernel: statistics through tables in P, then the weights)
        const uint32_t tail_strips = (uint32_t)((tail_rows + 31) / 32);
        const int q_base = (int)strips * BM;
        const int kc = key_ranges((int64_t)BH * tail_strips, (N + 127) / 128);
        const uint64_t tail_total = (uint64_t)BH * tail_strips * kc;
        const uint32_t tail_grid = (uint32_t)((tail_total + 7) / 8 * 8);
        if (kc > 1) {
            if (scores_only) {
                hipLaunchKernelGGL((qk_kernel<uint16_t, DB, 1, 1, 4, 1, true, false, 2>), dim3(tail_grid), dim3(256), 0, stream,
                                   q, k, o, N, d, c, flip, tail_strips, (uint32_t)tail_total, kc, q_base);
            } else {
                hipLaunchKernelGGL((qk_kernel<uint16_t, DB, 1, 1, 4, 1, false, false, 1>), dim3(tail_grid), dim3(256), 0, stream,
                                   q, k, o, N, d, c, flip, tail_strips, (uint32_t)tail_total, kc, q_base);
                hipLaunchKernelGGL((qk_kernel<uint16_t, DB, 1, 1, 4, 1, false, false, 2>), dim3(tail_grid), dim3(256), 0, stream,
                                   q, k, o, N, d, c, flip, tail_strips, (uint32_t)tail_total, kc, q_base);
            }
        } else if (scores_only) {   // (unsplit: the 256 keys of a tile over 8 waves)
            hipLaunchKernelGGL((qk_kernel<uint16_t, DB, 1, 1, 8, 1, true, false>), dim3(tail_grid), dim3(512), 0, stream,
                               q, k, o, N, d, c, flip, tail_strips, (uint32_t)tail_total, 1, q_base);
        } else {
            hipLaunchKernelGGL((qk_kernel<uint16_t, DB, 1, 1, 8, 1, false, false>), dim3(tail_grid), dim3(512), 0, stream,
                               q, k, o, N, d, c, flip, tail_strips, (uint32_t)tail_total, 1, q_base);
        }
    }
    return hipGetLastError();
}
template <int DB, int WQ = 8>
hipError_t launch_ring(bool scores_only, const void* Q, const void* K, void* out, int64_t BH, int N, int d, float scale,
                       hipStream_t stream)
{
    // staging writes as wide as the rows' positions in memory allow (rows start on multiples of 2 N bytes)
    if (N % 4 == 0) return launch_ring_t<DB, 8, WQ>(scores_only, Q, K, out, BH, N, d, scale, stream);
    if (N % 2 == 0) return launch_ring_t<DB, 4, WQ>(scores_only, Q, K, out, BH, N, d, scale, stream);
    return launch_ring_t<DB, 2, WQ>(scores_only, Q, K, out, BH, N, d, scale, stream);
}

template <typename T>
hipError_t launch_qk_t(bool scores_only, const void* Q, const void* K, void* out, int64_t BH, int N, int d,
                       float scale, hipStream_t stream, bool allow_split)
{
    const int row_bytes = d * (int)sizeof(T);
    constexpr int QB = sizeof(T) == 2 ? 2 : 1;   // fp32 stages twice the bytes per key: half the queries per wave
    // wide strips (4 waves along the queries) when that still gives every compute unit work, also when it
    // does so only with the keys of a strip split over several workgroups (rows of 128 and 256 bytes)
    const int64_t wide_units = BH * ((N + 128 * QB - 1) / (128 * QB));
    const bool big = wide_units >= 200;
    // (not below 1024 keys: two launches of a few microseconds each cost more than the idle compute units)
    const bool split = allow_split && !big && N >= 1024 && row_bytes > 64 && row_bytes <= 256 &&
                       key_ranges(wide_units, (N + 127) / 128) > 1;
    if constexpr (sizeof(T) == 2) {
        // Ragged lengths with enough 256-query strips for the chip: 8 waves of 32 queries that each walk whole tiles
        // and store whole memory lines out of a ring (RING in qk_kernel).  Measured, general kernel -> this one,
        // fused / scores in us.  B1 H16 d128: N = 2056 223 / 110 -> 88 / 52, 4072 286 / 215 -> 240 / 168, 4097 462 / 322 ->
        // 325 / 201, 4100 398 / 265 -> 294 / 175, 4104 (a 17th strip of 8 rows) 369 / 242 -> 340 / 226, 8168 1069 / 828 ->
        // 929 / 711; 4000 (rows on 64-byte boundaries) 225 / 151 both.  B8 H16 d64: N = 1543 368 / 283 -> 300 / 213,
        // 1544 283 / 230 -> 259 / 169, 1284 209 / 157 -> 181 / 119; 1025 193 / 139 -> 182 / 126, B16 H16 N = 785 208 / 152 ->
        // 179 / 126; not taken: 1032 121 / 78 -> 163 / 104, 1030 144 / 93 -> 164 / 120, B16 H12 N = 577 105 / 77 -> 111 / 84,
        // B64 H16 N = 197 74 / 53 -> 95 / 77.  Odd lengths gain earlier: their alternative is 2-byte stores.
        // Odd lengths of a few hundred to a thousand (a class token in front of 24 x 24 or 32 x 32 patches) with d <= 64:
        // the same with 128-query strips (4 waves, two workgroups per compute unit).  B16 H12 N = 577: d = 64 107 / 77 ->
        // 98 / 66, d = 32 99 / 72 -> 78 / 58; B8 H16 N = 1025 193 / 139 -> 156 / 110 (182 / 126 with 256-query strips);
        // B32 H12 N = 257 75 / 53 both; B64 H16 N = 197 74 / 53 -> 91 / 72 (not taken); even lengths lose (578: 79 / 51 -> 84 / 59).
        if ((N & 1) && N >= 320 && N < 1152 && row_bytes <= 128 && BH * ((N + 127) / 128) >= 200) {
            if (row_bytes <= 64) return launch_ring<64, 4>(scores_only, Q, K, out, BH, N, d, scale, stream);
            return launch_ring<128, 4>(scores_only, Q, K, out, BH, N, d, scale, stream);
        }
        if (N >= ((N & 1) ? 704 : 1280) && (N % 256) != 0 && row_bytes <= 256 && BH * ((N + 255) / 256) >= 100) {
            if (row_bytes <= 64) return launch_ring<64>(scores_only, Q, K, out, BH, N, d, scale, stream);
            if (row_bytes <= 128) return launch_ring<128>(scores_only, Q, K, out, BH, N, d, scale, stream);
            return launch_ring<256>(scores_only, Q, K, out, BH, N, d, scale, stream);
        }
    }
    if (row_bytes <= 64)
        return big ? launch_shape<T, 64, QB, 4, 2, 2>(scores_only, Q, K, out, BH, N, d, scale, stream)
                   : launch_shape<T, 64, QB, 1, 2, 2>(scores_only, Q, K, out, BH, N, d, scale, stream);
    if (row_bytes <= 128)
        return (big || split) ? launch_shape<T, 128, QB, 4, 2, 2, true>(scores_only, Q, K, out, BH, N, d, scale, stream, split)
                              : launch_shape<T, 128, QB, 1, 2, 2>(scores_only, Q, K, out, BH, N, d, scale, stream);
    if (row_bytes <= 256)
        return (big || split) ? launch_shape<T, 256, QB, 4, 2, 2, true>(scores_only, Q, K, out, BH, N, d, scale, stream, split)
                              : launch_shape<T, 256, QB, 1, 2, 2>(scores_only, Q, K, out, BH, N, d, scale, stream);
    if (row_bytes <= 512) return launch_shape<T, 512, 1, 4, 2, 1>(scores_only, Q, K, out, BH, N, d, scale, stream);
    if constexpr (sizeof(T) == 4)
        return launch_shape<T, 1024, 1, 4, 1, 1>(scores_only, Q, K, out, BH, N, d, scale, stream);
    return hipErrorInvalidValue;   // unreachable: d <= 256 bounds row_bytes
}

// bf16 shapes the persistent kernels take: those the two-pass kernel with split keys serves better.  Measured
// on one head of d = 128 (persistent kernel -> split): N = 2048 37 -> 25 us, 4096 68 -> 37, 8192 130 -> 89,
// 16384 269 -> 223; with 128 strips of 2048 or 4096 keys, and at d = 64 (64-query strips: twice the strips),
// the persistent kernel is as fast or faster.
bool prefers_key_split(int64_t BH, int64_t N, int64_t d)
{
    if (d != 128 || N < 2048 || (N % 2) != 0) return false;
    const int64_t strips = BH * ((N + 127) / 128), cus = compute_units();
    return 4 * strips <= cus || (2 * strips <= cus && N >= 8192);
}

// Problems with less than one 128-query strip per compute unit (one to a few heads: the sizes the paper itself
// measures are single heads) leave the persistent two-sweep kernels without work for most of the chip, and the
// key split above pays for it with two launches.  The kernel that spreads the keys of a strip over a gang of
// workgroups keeps every compute unit busy on them.  Measured, one head, default -> gang: d = 128, N = 1024
// 20.8 -> 14.9 us, 2048 25.4 -> 17.1, 4096 36.5 -> 26.1 (two heads 70 -> 37.5, four 75 -> 58); d = 64, N = 2048
// 18.3 -> 11.2, 4096 32.5 -> 19.0, 8192 60 -> 44; from one strip per compute unit on, and at N = 16384, the
// two-sweep kernels are as fast or faster.
bool prefers_gang(int64_t BH, int64_t N, int64_t d)
{
    if (N < 1024 || N > 8192) return false;
    return BH * (N / 128) < (int64_t)compute_units();
}

}  // namespace

hipError_t launch_qk(DType dt, bool scores_only, const void* Q, const void* K, void* out,
                     int64_t BH, int64_t N, int64_t d, float scale, hipStream_t stream)
{
    if (dt == DType::F32) return launch_qk_t<float>(scores_only, Q, K, out, BH, (int)N, (int)d, scale, stream, true);
    // ATTNW_FUSED_KERNEL=twopass keeps bf16 problems on the two-pass kernel above, =rounds keeps short sequences
    // off the resident kernel (tests and measurements compare the three)
    // (read at every call: the parity tests switch it between calls; one getenv against a launch of microseconds)
    const char* force = getenv("ATTNW_FUSED_KERNEL");
    const bool twopass = force && strcmp(force, "twopass") == 0;
    const bool rounds = force && strcmp(force, "rounds") == 0;
    const bool gang = force && strcmp(force, "gang") == 0;
    const bool tiny = force && strcmp(force, "tiny") == 0;
    // Sequences of up to 128 tokens: the kernel in which a wave works alone on a (head, 32 queries) pair.  Measured
    // against the kernels below, fused / scores in us: 12288 heads of N = 49, d = 32 320 / 219 -> 27 / 26; 4096 heads of
    // N = 64, d = 32 69 / 35 -> 10 / 10; 1024 heads of d = 64: N = 33 14 / 11 -> 6 / 5.5, 64 20 / 12 -> 6 / 6, 100 22 / 17 -> 16 / 15,
    // 128 25 / 17 -> 18 / 17; 16 heads: N = 49, d = 32 8.9 / 6.3 -> 4.3 / 4.2, N = 127, d = 96 12.6 / 9.3 -> 6.8 / 6.1.  Not taken:
    // N = 128 with fewer than 512 (head, 32 queries) pairs (64 heads of d = 64: 5.4 / 3.8 against 5.7 / 5.1), scores of
    // lengths that are multiples of 32 with few pairs (256 heads of N = 128: 5.4 against 6.0; 192 heads of N = 128, d = 64:
    // 5.2 against 5.6; N = 64, d = 32, 384 pairs: 4.6 against 4.8 -- taken from 1024 pairs on, from 384 up to 96 tokens, and
    // for every head size above 64, whose rows the kernels below pad: 1536 heads of N = 32, d = 64 16.3 -> 4.7 us, 768
    // heads of N = 64, d = 64 9.2 -> 5.6, 384 heads of N = 128, d = 64 8.7 -> 7.8, 192 heads of N = 96, d = 128 12.5 -> 6.6).
    if (qk_tiny_supported(BH, N, d)) {
        const int64_t units = BH * ((N + 31) / 32);
        // 128 < N <= 256 (d <= 64; the operands of the next unit are requested later in a unit, two waves per SIMD), 1024 heads,
        // fused / scores against the kernels below: N = 129, d = 64 27 / 23 against 35 / 29; 160 30 / 25 against 45 / 25; 192
        // 38 / 33 against 49 / 27; 197 48 / 43 against 52 / 41; 223 50 / 47 against 51 / 43; 224 51 / 44 against 55 / 32; d = 32:
        // N = 144 12 / 12 against 22 / 19, 197 28 / 27 against 42 / 30, 256 31 / 28 against 42 / 27 (4096 heads: 159 / 157 against 141 / 96)
        const bool take = N <= 128 ? (scores_only ? ((N % 32) != 0 || units >= 1024 || (N <= 96 && units >= 384) || d > 64) : !(N == 128 && units < 512))
                                   : (scores_only ? ((N % 32) != 0 && (N <= 160 || (d <= 32 && (N & 1) && N <= 224)))
                                                  : (N <= 192 || ((d <= 32 || (N & 1)) && N <= 224)));
        if (tiny || (!force && take)) return launch_qk_tiny(scores_only, Q, K, out, BH, N, d, scale, stream);
    }
    // Short sequences whose length is not a multiple of 32 (d = 64; 197, 257, 577 ...): the kernel that stages a strip
    // as the contiguous block of P that it is.  Measured against the general kernel, us: B64 H16 N = 33 31 -> 14,
    // 65 34 -> 20, 100 26 -> 21, 161 66 -> 40, 197 74 -> 50, 200 50 -> 41; B32 H12 N = 257 75 -> 46, 300 52 -> 43; B16 H12
    // N = 400 40 -> 29, 520 58 -> 44, 577 84 -> 70, 578 78 -> 56, 600 60 -> 52, 607 84 -> 71; one head of N = 197 16 -> 5.5, 577
    // 34 -> 18.  Multiples of 32 stay where they were (128: 25 against 27, 256: 20 against 25, 320: 47 against 50, 576: 58
    // against 64).
    // (scores of even lengths leave the general kernel as fast: its 4-byte stores pair up; measured 100 <= N <= 584)
    if (!force && (N % 32) != 0 && (!scores_only || (N & 1)) && qk_flat_supported(BH, N, d))
        return launch_qk_flat(scores_only, Q, K, out, BH, N, d, scale, stream);
    if (!scores_only && qk_gang_supported(BH, N, d) && (gang || (!force && prefers_gang(BH, N, d))))
        return launch_qk_gang(Q, K, out, BH, N, d, scale, stream);
    if (!twopass && !(!rounds && prefers_key_split(BH, N, d))) {
        if (!scores_only && !rounds && qk_resident_supported(BH, N, d))
            return launch_qk_resident(Q, K, out, BH, N, scale, stream);
        // (scores with 256-byte rows stay on the general kernel: two co-resident workgroups of it stream them faster)
        if (qk_rounds_supported(BH, N, d) && (!scores_only || d == 64))
            return launch_qk_rounds(scores_only, Q, K, out, BH, N, d, scale, stream);
    }
    // (forced onto the two-pass kernel: the plain one, a workgroup per strip)
    return launch_qk_t<uint16_t>(scores_only, Q, K, out, BH, (int)N, (int)d, scale, stream, !twopass);
}

}  // namespace attnw
