// Fused attention weights  P = softmax(scale * Q K^T)  with the scores of a strip resident on chip
// ACROSS compute units: Q K^T and the exponentials are computed once, for rows far longer than one
// compute unit can hold.
//
// This is the paper's fused kernel as it stands (section "Fused Matrix Multiply + Scaling + Softmax"):
// the score matrix is spread over a grid of cores, every core keeps its block in SRAM, reduces it to
// local row maxima and sums, the cores of a ROW exchange them for the global ones, and only then are
// the weights formed and written.  Here a "core" is a workgroup: its block is 32 queries x KR keys of
// fp32 scores in registers (KR = 512 with eight waves, one workgroup per compute unit; KR = 256 with
// four waves, two workgroups per compute unit), the KR K rows it needs stay in LDS for all the strips
// of a head, and the G = N / KR workgroups that share the rows of a strip -- a "gang" -- exchange
// their (maximum, sum) pairs through device memory.
//
// Where it is used: problems of one to a few heads, with less than one 128-query strip per compute
// unit -- the sizes the paper itself measures are single heads.  The kernels that sweep the keys twice
// have a workgroup per strip and leave most of the chip idle there; this one puts every compute unit
// on the keys of the few strips (one head, d = 128: N = 1024 20.8 -> 14.9 us, 4096 36.5 -> 26.1 us).
// On large problems it is NOT faster than the two-sweep kernels, measured on one MI355X: B1 H16 N4096
// d128 177-196 us against 177-188 us; B1 H8 N16384 d64 1250-1420 us against 990 us.  The second sweep
// it saves is matrix-core work, which already hides behind the vector ALU, and the vector ALU gains
// nothing: the exponential that is saved comes back as the multiplication by the normaliser, and the
// exchange costs instructions of its own.  ATTNW_FUSED_KERNEL=gang forces it wherever it applies.
//
// The only memory a call may write is P, so the exchange tables live in P itself: the pair table of
// strip s of a workgroup is parked in the part of P that the SAME workgroup fills with the weights
// of the strip after its next one, s + 2.  Nobody else ever writes there, and the workgroup writes
// those weights, two iterations after it took their exponentials, only after it has folded every
// peer's table of strip s + 2 -- which a peer publishes only after it has folded the tables of strip
// s (fold, barrier, publish, in this order within an iteration).  One strip less of distance is not
// enough: a peer starts READING the tables of strip s only after it has published its table of strip
// s + 1, so a workgroup that had waited for that table could overwrite what the peer was about to
// read (seen as whole strips with wrong sums in a gang whose members ran at different speeds).  The
// tables of the last two strips of a list have no such strip: they are parked in the last strip's
// own block (rows 1 and 3) and the peers acknowledge having read them before the block is written.
// A small kernel launched in front zeroes the table slots (a slot is valid once its sum is non-zero:
// a sum of exponentials against the own maximum is at least 1).
//
// All workgroups of a gang must be running at the same time: the grid is exactly as many workgroups
// as the compute units hold at once (LDS and registers leave room for no more) and gangs are
// consecutive blocks of one XCD, so that on a device that hands out workgroups in block order a gang
// is complete as soon as its last member has a place, whatever else runs beside the kernel (complete
// gangs finish on their own and make room).  Every wait is bounded all the same: a gang member that
// does not show up within some tenths of a second turns the rows that wait for it into NaN instead
// of hanging the device.
//
// Per workgroup (wave w owns keys 64 w .. 64 w + 63 of the workgroup's KR, as two 32-key pieces; all
// waves work on the same 32 queries), iteration i of its strip list:
//   exps      strip i: local maximum m_w of the wave's 64 scores per query, e = 2^(c s - c m_w) in place
//             of the scores, local sum l_w (Softmax section, Eq. 1, against the wave's own maximum) --
//             with the MFMAs of strip i + 1 riding along, one per chunk of exponentials;
//   peers     strip i - 2: the peers' pair tables, fetched into LDS during the previous iteration (a
//             hop through device memory takes about half a microsecond, and a read issued behind
//             this wave's own stores would wait for them), are folded: wave w folds peers 4 w .. 4 w + 3;
//   exchange  one barrier: the waves' local pairs of strip i and their peer partials of strip i - 2
//             meet in LDS; the workgroup's pair of strip i is published, the fetch of the peers'
//             tables of strip i - 1 is started;
//   weights   strip i - 2:  p = e 2^(c m_w - c m) / l with the global m and l, rounded once, staged
//             per wave as [16 queries][64 keys] (or [8][64]: what the LDS has room for), stored past
//             the caches.
// Four accumulator sets rotate: scores being accumulated, exponentials being taken, and two strips of
// exponentials waiting for their peers.
#include "launchers.h"
#include "qk_common.h"

namespace attnw {
namespace {

template <int DB_, int NW_>
struct GangCfg {
    static constexpr int DB = DB_;                // bytes of a Q / K row: d = 64 or 128
    static constexpr int NW = NW_, NT = 2;        // waves per workgroup (8: one workgroup per compute unit, 4: two)
    static constexpr int G = DB / 32;             // 32-byte contraction groups per row
    static constexpr int CPR = DB / 16;           // 16-byte chunks per K row
    static constexpr int KR = 32 * NW * NT;       // keys per workgroup: 512 or 256
    static constexpr int PIECE_BYTES = 32 * DB;
    static constexpr int K_BYTES = KR * DB;
    static constexpr int K_CHUNKS_PER_LANE = K_BYTES / 16 / (64 * NW);
    static constexpr int K_BATCH = 4;             // chunks per lane in flight while K is copied
    static constexpr int SEG = 128;               // bytes of one staged row: the wave's 64 keys
    static constexpr int ST_ROWS = DB == 256 ? 8 : 16;   // queries staged at a time (what the LDS has room for)
    static constexpr int ST_PITCH = SEG + 16;
    static constexpr int ST_BYTES = ST_ROWS * ST_PITCH;
    static constexpr int CPS = SEG / 16;          // chunks per staged row
    static constexpr int RPI = 64 / CPS;          // staged rows one store instruction covers
    static constexpr int NF = ST_ROWS / RPI;      // store instructions per staged block
    static constexpr int NS = (32 / ST_ROWS) * NF;   // store instructions per wave and strip
    static constexpr int RPL = CPR >= 16 ? 1 : 16 / CPR;
    static constexpr int SWZ_MASK = (CPR >= 16 ? 16 : CPR) - 1;
    // workgroups per gang at most: a wave fetches the tables of four peers, 1 KiB, with one transfer
    static constexpr int MAXG = 4 * NW;
    static constexpr int LDS_TAB = MAXG / 4 * 1024 + 256;   // + the landing area of the warming reads (never looked at)
    static constexpr int LDS_STAT = 2 * 4 * NW * 32 * 4;   // strip parity x (local max, local sum, peer max, peer sum)
    static constexpr int LDS_ST = NW * ST_BYTES;
    static constexpr int LDS_TOTAL = LDS_TAB + LDS_STAT + LDS_ST + K_BYTES;
    static_assert(K_CHUNKS_PER_LANE % K_BATCH == 0, "K copy shape");
    static_assert(LDS_TOTAL <= (NW == 4 ? 80 : 160) * 1024, "tables, exchange buffers, staging rows and the K of the key range share the LDS");
};

constexpr int kSpinLimit = 1 << 18;               // fetches of a table before a peer is given up

__device__ __forceinline__ uint64_t load_slot(const uint64_t* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void store_slot(uint64_t* p, uint64_t v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint64_t pack_pair(float m, float l)
{
    return (uint64_t)__float_as_uint(m) | ((uint64_t)__float_as_uint(l) << 32);
}
// 16 bytes per lane from device memory (device scope: the data was written by another compute unit during this
// kernel) straight into LDS at lds_base + 16 * lane; not seen by the compiler's wait-count pass (see qk_common.h)
__device__ __forceinline__ void dma16_untracked_device_scope(const char* src, uint32_t lds_base)
{
#if defined(__HIP_DEVICE_COMPILE__)
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off sc1" ::"s"(lds_base), "v"(src) : "memory", "m0");
#endif
}
// The same through this XCD's L2 as it stands.  What it returns may be out of date (a slot that another XCD has
// filled meanwhile can still read as empty): good for a first look, never for the look that gives up waiting.
__device__ __forceinline__ void dma16_untracked_l2(const char* src, uint32_t lds_base)
{
#if defined(__HIP_DEVICE_COMPILE__)
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_base), "v"(src) : "memory", "m0");
#endif
}
// 4 bytes per lane into LDS at lds_base + 4 * lane: a read whose only purpose is to bring memory lines into L2
__device__ __forceinline__ void dma4_untracked_l2(const char* src, uint32_t lds_base)
{
#if defined(__HIP_DEVICE_COMPILE__)
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, off" ::"s"(lds_base), "v"(src) : "memory", "m0");
#endif
}

// Lanes of one wave hand data to each other through LDS inside divergent code (see the resident kernel).
__device__ __forceinline__ void wave_sync_lds_gang()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Where things are, shared by the two kernels.  A list = the strips [s_a, s_b) of the global (head, strip)
// order that one gang works through; it is cut into segments at head boundaries (K changes there).
struct GangWork {
    uint32_t gang, r, n_gangs, gsize;             // gang id, this workgroup's key range, gangs, workgroups per gang
    uint32_t s_a, s_b;
};
__device__ __forceinline__ GangWork gang_work(uint32_t gsize, uint32_t total_strips)
{
    GangWork w;
    const uint32_t per_xcd = gridDim.x >> 3;
    const uint32_t xcd = blockIdx.x & 7u, idx = blockIdx.x >> 3;
    const uint32_t gangs_per_xcd = per_xcd / gsize;
    w.gsize = gsize;
    w.n_gangs = 8u * gangs_per_xcd;
    w.gang = xcd * gangs_per_xcd + idx / gsize;
    w.r = idx % gsize;
    w.s_a = (uint32_t)((uint64_t)w.gang * total_strips / w.n_gangs);
    w.s_b = (uint32_t)((uint64_t)(w.gang + 1) * total_strips / w.n_gangs);
    return w;
}
// byte offset in P of key range j of row `row` of strip `strip` of head `bh`
__device__ __forceinline__ int64_t slot_offset(uint32_t bh, uint32_t strip, int row, uint32_t j, int N, int kr)
{
    return (((int64_t)bh * N + (int64_t)strip * 32 + row) * (int64_t)N + (int64_t)j * kr) * 2;
}

// Zeroes the table slots the main kernel waits on: row 0 of every block but the first two of a segment (the
// pairs of the strip two before), rows 1, 2 and 3 of the last block of a segment (its own pairs, the
// acknowledgements, the pairs of the strip before).
template <int KR>
__global__ __launch_bounds__(256)
void qk_gang_init_kernel(uint16_t* __restrict__ out, int N, uint32_t gsize, uint32_t strips_per_head, uint32_t total_strips)
{
    const GangWork w = gang_work(gsize, total_strips);
    char* const base = reinterpret_cast<char*>(out);
    const int tid = threadIdx.x;
    const int q = tid & 31;
    // one 32-lane group per strip, 8 strips per trip
    for (uint32_t s = w.s_a + (tid >> 5); s < w.s_b; s += 8) {
        const uint32_t bh = s / strips_per_head, strip = s - bh * strips_per_head;
        const uint32_t seg_first = max(w.s_a, bh * strips_per_head);   // first strip of the segment, global index
        const bool last = s + 1 == w.s_b || strip + 1 == strips_per_head;
        if (s - seg_first >= 2) *reinterpret_cast<uint64_t*>(base + slot_offset(bh, strip, 0, w.r, N, KR) + q * 8) = 0ull;
        if (last) {
#pragma unroll
            for (int row = 1; row <= 3; ++row)
                *reinterpret_cast<uint64_t*>(base + slot_offset(bh, strip, row, w.r, N, KR) + q * 8) = 0ull;
        }
    }
}

template <int DB, int NW_>
__global__ __launch_bounds__(64 * NW_, 2)
void qk_gang_kernel(const uint16_t* __restrict__ Q, const uint16_t* __restrict__ K, uint16_t* __restrict__ out,
                    int N, float c, uint32_t sign_flip, uint32_t gsize, uint32_t strips_per_head, uint32_t total_strips)
{
    using C = GangCfg<DB, NW_>;
    constexpr int G = C::G, CPR = C::CPR, NW = C::NW, NT = C::NT, KR = C::KR, PIECE_BYTES = C::PIECE_BYTES, NTHREADS = 64 * NW;
    constexpr int ST_PITCH = C::ST_PITCH, ST_BYTES = C::ST_BYTES, CPS = C::CPS, RPI = C::RPI, NF = C::NF, ST_ROWS = C::ST_ROWS;

    // the table landing area first: transfers into LDS address it through a 16-bit base
    __shared__ __align__(1024) char lds[C::LDS_TOTAL];
    char* const tab_lds = lds;
    float* const stat = reinterpret_cast<float*>(lds + C::LDS_TAB);   // [parity][kind][wave][query]
    char* const st_lds = lds + C::LDS_TAB + C::LDS_STAT;
    char* const k_lds = lds + C::LDS_TAB + C::LDS_STAT + C::LDS_ST;

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int l32 = lane & 31;
    const int half = lane >> 5;

    const GangWork w = gang_work(gsize, total_strips);
    if (w.s_a >= w.s_b) return;
    const uint32_t r = w.r;

    // K fragment (piece t, group g) of this wave: k_lds + t * PIECE_BYTES + (frag0 ^ 32 g): the chunk index 2 g + half
    // is XOR-swizzled by the key, and 2 g only touches bits that the rest of the offset leaves alone
    const int frag0 = (wave * NT * 32 + l32) * DB + ((half ^ ((l32 / C::RPL) & C::SWZ_MASK)) * 16);
    char* const stage = st_lds + wave * ST_BYTES;
    char* const st_wr = stage + (l32 % ST_ROWS) * ST_PITCH + 8 * half;
    const char* const st_rd = stage + (lane / CPS) * ST_PITCH + (lane % CPS) * 16;
    char* const out_base = reinterpret_cast<char*>(out);
    // tables of the four peers 4 wave .. 4 wave + 3 land at tab_wave as [peer][query] pairs
    char* const tab_wave = tab_lds + wave * 1024;
    const uint32_t tab_wave_base = lds_offset_of(tab_wave);
    const bool fetches = (uint32_t)(4 * wave) < w.gsize;   // this wave has peers to fetch (wave-uniform)
    const int n_fetch_waves = (int)(w.gsize + 3) / 4;
    const int own_wave = (int)(r / 4);            // the wave whose four "peers" include this workgroup itself
    const uint32_t warm_base = lds_offset_of(tab_lds + C::LDS_TAB - 256);
    constexpr int WARM_WAVE = NW - 1, WARM_AHEAD = 4;

    uint32_t parity = 0;
    bool dead = false;                            // a peer did not show up: stop waiting, poison the rows

    // MFMA a of a sweep: contraction group a / NT, key piece a % NT -- group-major, so that consecutive MFMAs go to
    // different accumulators and a Q fragment is free for the next strip's rows after NT MFMAs
    constexpr int NMMA = NT * G;
    auto k_frag = [&](auto ic) __attribute__((always_inline)) -> u32x4 {
        constexpr int a = decltype(ic)::value;
        return *reinterpret_cast<const u32x4*>(k_lds + (a % NT) * PIECE_BYTES + (frag0 ^ (32 * (a / NT))));
    };
    auto mma_step = [&](f32x16 (&A)[NT], const u32x4 (&q)[G], const u32x4& kf, auto ic) __attribute__((always_inline)) {
        constexpr int a = decltype(ic)::value;
        if constexpr (a / NT == 0) {
#pragma unroll
            for (int x = 0; x < 16; ++x) A[a % NT][x] = 0.0f;
        }
        Mma<uint16_t>::run(A[a % NT], kf, q[a / NT]);
    };

    // byte offset, inside the head's part of P, of key range j of row `row` of strip `strip` (N <= 16384: 32 bits)
    auto blk_off = [&](uint32_t strip, uint32_t row, uint32_t j) __attribute__((always_inline)) -> uint32_t {
        return ((strip * 32u + row) * (uint32_t)N + j * (uint32_t)KR) * 2u;
    };
    const uint32_t lane_out_off = (uint32_t)(((lane / CPS) * N + wave * 32 * NT + (lane % CPS) * 8) * 2);

    uint32_t s_cur = w.s_a;
    while (s_cur < w.s_b) {
        // ======== one segment: strips [s0, s0 + n) of head bh ===========================================
        const uint32_t bh = s_cur / strips_per_head;
        const uint32_t s0 = s_cur - bh * strips_per_head;
        const uint32_t seg_end = min(w.s_b, (bh + 1) * strips_per_head);
        const uint32_t n = seg_end - s_cur;
        s_cur = seg_end;
        char* const out_h = out_base + (int64_t)bh * N * (int64_t)N * 2;
        const char* const Qh = reinterpret_cast<const char*>(Q) + (int64_t)bh * N * DB;

        // ---- this workgroup's 512 K rows of the head into LDS, chunk-swizzled for the fragment reads ----------
        {
            const char* Kr = reinterpret_cast<const char*>(K) + ((int64_t)bh * N + (int64_t)r * KR) * DB;
            __syncthreads();                      // nobody reads the previous segment's K (or exchange buffers) any more
#pragma unroll
            for (int b = 0; b < C::K_CHUNKS_PER_LANE / C::K_BATCH; ++b) {
                u32x4 kv[C::K_BATCH];
#pragma unroll
                for (int j = 0; j < C::K_BATCH; ++j)
                    kv[j] = *reinterpret_cast<const u32x4*>(Kr + (uint32_t)(((b * C::K_BATCH + j) * NTHREADS + tid) * 16));
#pragma unroll
                for (int j = 0; j < C::K_BATCH; ++j) {
                    const int sl = (b * C::K_BATCH + j) * NTHREADS + tid;
                    const int key = sl / CPR;
                    const int pos = (sl % CPR) ^ ((key / C::RPL) & C::SWZ_MASK);
                    // a negative scale negates K: softmax(-|c| s) = softmax(|c| Q (-K)^T)
                    *reinterpret_cast<u32x4*>(k_lds + key * DB + pos * 16) = kv[j] ^ sign_flip;
                }
            }
            __syncthreads();
        }

        u32x4 qf[G];
        auto q_ptr = [&](uint32_t strip) __attribute__((always_inline)) -> const char* {
            return Qh + (uint32_t)((strip * 32 + l32) * DB + half * 16);
        };
        // byte offset in the head's part of P of the table of segment-relative strip i as published by key range j:
        // row 0 of the block of strip i + 2, or, for the last two strips of the segment, rows 3 and 1 of the last block
        auto table_off = [&](uint32_t i, uint32_t j) __attribute__((always_inline)) -> uint32_t {
            return i + 2 < n ? blk_off(s0 + i + 2, 0, j) : blk_off(s0 + n - 1, i + 1 == n ? 1 : 3, j);
        };
        // start the transfer of the tables of strip i of this wave's four peers into LDS (lane: peer lane / 16,
        // 16 bytes lane % 16 of its 256-byte table; a peer that does not exist, or this workgroup itself: the own table)
        auto tables_fetch = [&](uint32_t i, bool first_look) __attribute__((always_inline)) {
            uint32_t j = 4 * wave + lane / 16;
            j = j < w.gsize ? j : r;
            const char* src = out_h + table_off(i, j) + (lane % 16) * 16;
            if (first_look) dma16_untracked_l2(src, tab_wave_base);
            else dma16_untracked_device_scope(src, tab_wave_base);
        };
        // fold the pairs of strip i of this wave's peers (own workgroup: mw, lw) into (pm, pl).  The transfer was
        // started an iteration ago; `exact`: between it and now this wave issued exactly NS stores and G loads
        auto tables_fold = [&](uint32_t i, bool exact, float mw, float lw, float& pm, float& pl) __attribute__((always_inline)) {
            pm = kNegBig;
            pl = 0.0f;
            if (fetches) {
                if (!exact) wait_vmem();
                else if (wave == WARM_WAVE) wait_vmem_le<C::NS + G + 1>();   // (its warming read follows the transfer)
                else wait_vmem_le<C::NS + G>();
                asm volatile("" ::: "memory");
                const uint32_t j0 = 4 * wave + 2 * half;   // this lane's peers: j0, j0 + 1
                f32x2 pr[2];
                bool need[2];
#pragma unroll
                for (int k = 0; k < 2; ++k) {
                    need[k] = j0 + k < w.gsize && j0 + k != r;
                    pr[k] = *reinterpret_cast<const f32x2*>(tab_wave + (2 * half + k) * 256 + l32 * 8);
                }
                // stragglers: fetch again until every pair is there (a sum is never 0), a bounded number of times
                int tries = 0;
                while (__any((need[0] && pr[0][1] == 0.0f) || (need[1] && pr[1][1] == 0.0f)) && !dead) {
                    __builtin_amdgcn_s_sleep(4);
                    tables_fetch(i, false);
                    wait_vmem();
                    asm volatile("" ::: "memory");
#pragma unroll
                    for (int k = 0; k < 2; ++k)
                        pr[k] = *reinterpret_cast<const f32x2*>(tab_wave + (2 * half + k) * 256 + l32 * 8);
                    if (++tries > kSpinLimit) dead = true;
                }
#pragma unroll
                for (int k = 0; k < 2; ++k) {
                    float m2 = kNegBig, l2 = 0.0f;
                    if (need[k]) { m2 = pr[k][0]; l2 = pr[k][1]; }
                    else if (j0 + k == r) { m2 = mw; l2 = lw; }
                    const float mx = fmaxf(pm, m2);
                    pl = pl * fast_exp2(pm - mx) + l2 * fast_exp2(m2 - mx);
                    pm = mx;
                }
                const float mo = __shfl_xor(pm, 32, 64), lo = __shfl_xor(pl, 32, 64);
                const float mx = fmaxf(pm, mo);
                pl = pl * fast_exp2(pm - mx) + lo * fast_exp2(mo - mx);
                pm = mx;
            }
        };

        // ---- weights of a strip whose exponentials are in X: scale, round once, stage, store ----------------
        auto finalize = [&](f32x16 (&X)[NT], float inv, uint32_t strip) __attribute__((always_inline)) {
            char* const out_rows = out_h + blk_off(strip, 0, r);      // wave-uniform
            // every lane's 32 weights, rounded (once, outside the per-block predicate below: inside it the work
            // would be issued once per block)
            u32x2 wv[2][4];
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const f32x16& a = X[u];
                    wv[u][r4] = u32x2{pack_bf16x2(a[4 * r4] * inv, a[4 * r4 + 1] * inv),
                                      pack_bf16x2(a[4 * r4 + 2] * inv, a[4 * r4 + 3] * inv)};
                }
#pragma unroll
            for (int hb = 0; hb < 32 / ST_ROWS; ++hb) {   // queries ST_ROWS hb .. + ST_ROWS of the strip
                if (l32 / ST_ROWS == hb) {
#pragma unroll
                    for (int u = 0; u < 2; ++u)
#pragma unroll
                        for (int r4 = 0; r4 < 4; ++r4)
                            *reinterpret_cast<u32x2*>(st_wr + (u * 32 + 8 * r4) * 2) = wv[u][r4];
                }
                wave_sync_lds_gang();             // some of the lanes wrote, all of them read
                u32x4 v[NF];
#pragma unroll
                for (int f = 0; f < NF; ++f) v[f] = *reinterpret_cast<const u32x4*>(st_rd + f * RPI * ST_PITCH);
                wave_sync_lds_gang();             // the rows are in registers before the next block overwrites them
#pragma unroll
                for (int f = 0; f < NF; ++f)
                    __builtin_nontemporal_store(
                        v[f], reinterpret_cast<u32x4*>(out_rows + (uint32_t)((hb * ST_ROWS + f * RPI) * N * 2) + lane_out_off));
                __builtin_amdgcn_sched_barrier(0);
            }
        };

        // per strip state carried from the iteration that takes the exponentials to the one that writes, two
        // iterations later: the wave's exponent, the workgroup's pair
        float mb_1 = 0.0f, mw_1 = 0.0f, lw_1 = 0.0f, mb_2 = 0.0f, mw_2 = 0.0f, lw_2 = 0.0f;
        // ---- iteration i = 0 .. n + 1.  X: scores of strip i (none from i = n on); Y: receives the scores of strip
        //      i + 1; Z: exponentials of strip i - 2, written now (the set of strip i - 1 waits untouched)
        auto iteration = [&](f32x16 (&X)[NT], f32x16 (&Y)[NT], f32x16 (&Z)[NT], uint32_t i) __attribute__((always_inline)) {
            const bool live = i < n, fin = i >= 2, req = i >= 1 && i <= n;
            float* const st = stat + parity * (4 * NW * 32);
            float mb = 0.0f, l = 0.0f;
            if (live) {
                // ---- local maximum of this wave's 64 keys
                float m = kNegBig;
#pragma unroll
                for (int t = 0; t < NT; ++t) {
#pragma unroll
                    for (int x = 0; x < 16; x += 2) m = max3(m, X[t][x], X[t][x + 1]);
                }
                m = fmaxf(m, __shfl_xor(m, 32, 64));
                mb = m * c;
                // ---- exponentials in place of the scores, local sum; the next strip's sweep rides along
                constexpr int EPC = 16 * NT / NMMA;
                constexpr int LEAD = 2;
                u32x4 ring[LEAD];
                static_for<LEAD>([&](auto ic) __attribute__((always_inline)) { ring[decltype(ic)::value] = k_frag(ic); });
                // the Q rows of the strip after next replace each fragment as soon as its MFMAs are issued: nearly a
                // whole iteration passes before they are used
                const char* const qn = q_ptr(s0 + min(i + 2, n - 1));
                static_for<NMMA>([&](auto ic) __attribute__((always_inline)) {
                    constexpr int a = decltype(ic)::value;
#pragma unroll
                    for (int e = 0; e < EPC; ++e) {
                        const int idx = a * EPC + e;
                        const float x = fast_exp2(__builtin_fmaf(X[idx / 16][idx % 16], c, -mb));
                        X[idx / 16][idx % 16] = x;
                        l += x;
                    }
                    mma_step(Y, qf, ring[a % LEAD], ic);
                    if constexpr (a + LEAD < NMMA) ring[a % LEAD] = k_frag(IC<a + LEAD>{});
                    if constexpr (a % NT == NT - 1) qf[a / NT] = *reinterpret_cast<const u32x4*>(qn + (a / NT) * 32);
                    __builtin_amdgcn_sched_barrier(0);
                });
                l += __shfl_xor(l, 32, 64);
            }
            __builtin_amdgcn_sched_barrier(0);    // (the steps of an iteration stay in their order: registers)
            // ---- peers' pairs of strip i - 2 (fetched during the previous iteration)
            float pm = kNegBig, pl = 0.0f;
            if (fin) tables_fold(i - 2, i >= 3 && live, mw_2, lw_2, pm, pl);
            if (half == 0) {
                st[(0 * NW + wave) * 32 + l32] = mb;
                st[(1 * NW + wave) * 32 + l32] = l;
                st[(2 * NW + wave) * 32 + l32] = pm;
                st[(3 * NW + wave) * 32 + l32] = pl;
            }
            __syncthreads();
            // ---- this workgroup's pair of strip i: published for the peers
            // (wanted by the wave that publishes it and by the wave that folds it in with its peers' pairs)
            float mw = mb, lw = 0.0f;
            if (live && (wave == 0 || wave == own_wave)) {
#pragma unroll
                for (int v = 0; v < NW; ++v) mw = fmaxf(mw, st[(0 * NW + v) * 32 + l32]);
#pragma unroll
                for (int v = 0; v < NW; ++v) lw += st[(1 * NW + v) * 32 + l32] * fast_exp2(st[(0 * NW + v) * 32 + l32] - mw);
                if (wave == 0 && half == 0)
                    store_slot(reinterpret_cast<uint64_t*>(out_h + table_off(i, r)) + l32, pack_pair(mw, lw));
            }
            float inv = 0.0f;
            if (fin) {
                // (only the waves that have peers to fetch hold a partial)
                float mg = kNegBig;
#pragma unroll
                for (int v = 0; v < NW; ++v)
                    if (v < n_fetch_waves) mg = fmaxf(mg, st[(2 * NW + v) * 32 + l32]);
                float lg = 0.0f;
#pragma unroll
                for (int v = 0; v < NW; ++v)
                    if (v < n_fetch_waves) lg += st[(3 * NW + v) * 32 + l32] * fast_exp2(st[(2 * NW + v) * 32 + l32] - mg);
                inv = fast_exp2(mb_2 - mg) * __builtin_amdgcn_rcpf(lg);
            }
            __builtin_amdgcn_sched_barrier(0);
            // ---- the peers published their tables of strip i - 1 an iteration ago: start fetching them
            if (req && fetches) tables_fetch(i - 1, true);
            // one 4-byte read per memory line of the Q rows of a strip a few iterations ahead: the workgroups of the
            // gang all ask for them at the same moment later, and the rows would come from device memory then
            if (wave == WARM_WAVE && i >= 2 && live)
                dma4_untracked_l2(Qh + (uint32_t)(min(s0 + i + WARM_AHEAD, s0 + n - 1) * 32 * DB + (lane * 128) % (32 * DB)), warm_base);
            // ---- weights of strip i - 2
            if (fin) {
                if (i == n + 1) {
                    // The last strip's table sits in its own block (row 1): tell every peer that it has been read
                    // (slot r of row 2 of the peer's block) and wait for the same from them before writing.
                    // (the barrier above: every wave of this workgroup has read its peers' tables)
                    if (wave == 0) {
                        const uint32_t j = lane;
                        const bool peer = j < w.gsize && j != r;
                        if (peer) store_slot(reinterpret_cast<uint64_t*>(out_h + blk_off(s0 + n - 1, 2, j)) + r, 1ull);
                        if (peer) {
                            const uint64_t* mine = reinterpret_cast<const uint64_t*>(out_h + blk_off(s0 + n - 1, 2, r)) + j;
                            int tries = 0;
                            while (load_slot(mine) == 0ull && !dead) {
                                __builtin_amdgcn_s_sleep(4);
                                if (++tries > kSpinLimit) dead = true;
                            }
                        }
                        if (__any(dead) && lane == 0) st[0] = -1.0f;   // (a local exponent slot: not in use in this iteration)
                    }
                    __syncthreads();
                    dead = dead || st[0] == -1.0f;
                }
                dead = __any(dead);
                if (dead) inv = __builtin_nanf("");
                finalize(Z, inv, s0 + i - 2);
            }
            __builtin_amdgcn_sched_barrier(0);
            parity ^= 1u;
            mb_2 = mb_1; mw_2 = mw_1; lw_2 = lw_1;
            mb_1 = mb; mw_1 = mw; lw_1 = lw;
        };

        // ---- the pipeline over the segment's strips; the four sets rotate roles -----------------------------
        f32x16 acc_a[NT], acc_b[NT], acc_c[NT], acc_d[NT];
        {
            const char* const q0 = q_ptr(s0);
#pragma unroll
            for (int g = 0; g < G; ++g) qf[g] = *reinterpret_cast<const u32x4*>(q0 + g * 32);
            static_for<NMMA>([&](auto ic) __attribute__((always_inline)) {
                mma_step(acc_a, qf, k_frag(ic), ic);
                __builtin_amdgcn_sched_barrier(0);
            });
            const char* const q1 = q_ptr(s0 + min(1u, n - 1));
#pragma unroll
            for (int g = 0; g < G; ++g) qf[g] = *reinterpret_cast<const u32x4*>(q1 + g * 32);
        }
        for (uint32_t i = 0; i <= n + 1; i += 4) {
            iteration(acc_a, acc_b, acc_c, i);
            if (i + 1 <= n + 1) iteration(acc_b, acc_c, acc_d, i + 1);
            if (i + 2 <= n + 1) iteration(acc_c, acc_d, acc_a, i + 2);
            if (i + 3 <= n + 1) iteration(acc_d, acc_a, acc_b, i + 3);
        }
        wait_vmem();                              // no transfer into LDS is in flight when the segment ends
    }
}

template <int DB, int NW>
hipError_t launch_gang(const void* Q, const void* K, void* out, int64_t BH, int N, float scale, hipStream_t stream)
{
    using C = GangCfg<DB, NW>;
    const uint32_t gsize = (uint32_t)(N / C::KR);
    const uint32_t strips_per_head = (uint32_t)(N / 32);
    const uint32_t total = (uint32_t)(BH * strips_per_head);
    // 8 waves: a workgroup per compute unit; 4 waves: two (both kernels are built for exactly that many)
    const uint32_t per_xcd = (uint32_t)(compute_units() / 8) * (8 / NW);
    const uint32_t gangs_per_xcd = per_xcd / gsize;
    const uint32_t grid = 8u * gangs_per_xcd * gsize;
    const float c = fabsf(scale) * kLog2e;
    const uint32_t flip = scale < 0.0f ? Mma<uint16_t>::kSignMask : 0u;
    hipLaunchKernelGGL((qk_gang_init_kernel<C::KR>), dim3(grid), dim3(256), 0, stream, static_cast<uint16_t*>(out), N, gsize,
                       strips_per_head, total);
    hipLaunchKernelGGL((qk_gang_kernel<DB, NW>), dim3(grid), dim3(64 * NW), 0, stream, static_cast<const uint16_t*>(Q),
                       static_cast<const uint16_t*>(K), static_cast<uint16_t*>(out), N, c, flip, gsize, strips_per_head, total);
    return hipGetLastError();
}

}  // namespace

bool qk_gang_supported(int64_t BH, int64_t N, int64_t d)
{
    // rows of 128 or 256 bytes; whole key ranges of 256 keys (up to 4096 keys: 16 workgroups of four waves, two per
    // compute unit) or of 512 (up to 16384 keys: 32 workgroups of eight waves); at least two ranges
    if (d != 64 && d != 128) return false;
    if (compute_units() % 8 != 0 || compute_units() < 128) return false;
    const bool small = N % 256 == 0 && N >= 512 && N <= 4096;
    const bool large = N % 512 == 0 && N > 4096 && N <= 16384;
    if (!small && !large) return false;
    return BH * (N / 32) <= (int64_t)0x7ffffff0;
}

hipError_t launch_qk_gang(const void* Q, const void* K, void* out, int64_t BH, int64_t N, int64_t d, float scale,
                          hipStream_t stream)
{
    if (N <= 4096)
        return d == 64 ? launch_gang<128, 4>(Q, K, out, BH, (int)N, scale, stream)
                       : launch_gang<256, 4>(Q, K, out, BH, (int)N, scale, stream);
    return d == 64 ? launch_gang<128, 8>(Q, K, out, BH, (int)N, scale, stream)
                   : launch_gang<256, 8>(Q, K, out, BH, (int)N, scale, stream);
}

}  // namespace attnw

