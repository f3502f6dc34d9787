// Fused attention weights  P = softmax(scale * Q K^T)  for short sequences: the scores of a strip
// stay on chip between the contraction and the normalisation, so Q K^T is computed once.
//
// This is the shape of the paper's own fused kernel (section "Fused Matrix Multiply + Scaling +
// Softmax"): a block of scores is left in each core's SRAM by the matrix multiply, every core
// reduces its block to local row maxima and sums, the cores of a row exchange them for the global
// ones, and only then are the weights formed and written.  Here the "row of cores" is the eight
// waves of a workgroup and the "SRAM" their registers: a strip of 32 queries against N <= 1024
// keys is 32 x N fp32 scores = at most 64 registers per lane when each wave owns N/8 of the keys.
// Longer rows do not fit (the round-based and the two-pass kernels recompute the scores instead).
//
// A persistent workgroup per compute unit takes a contiguous list of (head, strip) pairs.  Per head
// it copies the whole K (N x 128 bytes <= 128 KiB) into LDS once, in matrix-core operand order
// after that a strip costs no K traffic and no waiting on memory:
//   sweep     wave w owns keys [w N/8, (w+1) N/8) of the row; piece t of them is multiplied with the
//             strip's 32 queries: S^T = K_piece * Q^T, a lane's 16 accumulators are 16 keys of one query;
//   local     per lane and wave: maximum m_w of its N/8 scores of a query, e = 2^(c s - c m_w) in place of
//             the scores and their sum l_w (Softmax section, Eq. 1, against the wave's own maximum);
//   global    the eight waves exchange (c m_w, l_w) through LDS (one barrier per strip):
//             m = max m_w, l = sum l_w 2^(c m_w - c m);
//   weights   p = e 2^(c m_w - c m) / l, rounded once to bf16, staged per wave as [16 queries][64 keys], re-read
//             16 bytes per lane and stored past the caches (8 rows x 128 bytes per instruction).
// The Q rows of the next strip are requested before the stores of the current one are issued:
// vector-memory operations retire in order, and a load behind a burst of stores would wait for it.
// While the exponentials of a strip are taken, the scores of the next strip of the same head are
// accumulated into a second register set, one MFMA per chunk of vector work.
#include "launchers.h"
#include "qk_common.h"

namespace attnw {
namespace {

// NW waves, all on the same 32 queries; wave w owns NT pieces of 32 keys: keys 32 NT w + 32 t + i.
template <int NW, int NT>
struct ResidentCfg {
    static constexpr int DB = 128;                // bytes of a Q / K row: d = 64
    static constexpr int G = DB / 32;             // 32-byte contraction groups per row
    static constexpr int CPR = DB / 16;           // 16-byte chunks per K row
    static constexpr int N = 32 * NW * NT;        // keys
    static constexpr int PIECE_BYTES = 32 * DB;
    static constexpr int K_BYTES = N * DB;
    static constexpr int K_CHUNKS_PER_LANE = K_BYTES / 16 / (64 * NW);
    static constexpr int SEG = 128;               // bytes of one staged row: two 32-key pieces
    static constexpr int ST_ROWS = 128 / NW;      // queries staged at a time (the staging area is 18 KiB in all)
    static constexpr int ST_PITCH = SEG + 16;
    static constexpr int ST_BYTES = ST_ROWS * ST_PITCH;
    static constexpr int CPS = SEG / 16;          // chunks per staged row
    static constexpr int RPI = 64 / CPS;          // staged rows one store instruction covers
    static constexpr int NF = ST_ROWS / RPI;      // store instructions per staged block
    static constexpr int RPL = 16 / CPR;
    static constexpr int SWZ_MASK = CPR - 1;
    static constexpr int LDS_ST = NW * ST_BYTES;
    static constexpr int LDS_STAT = 2 * 2 * NW * 32 * 4;   // (max, sum) x strip parity
    static constexpr int LDS_TOTAL = K_BYTES + LDS_ST + LDS_STAT;
    static constexpr int ST_BLOCKS = 32 / ST_ROWS;
    static_assert(NT % 2 == 0 && NT >= 2 && NT <= 4, "pieces are staged in pairs; 16 NT accumulators per lane");
    static_assert(NW == 8 || NW == 16, "workgroups of 512 or 1024 lanes");
    static_assert(ST_ROWS % RPI == 0 && K_BYTES % (16 * 64 * NW) == 0, "staging block and K copy shapes");
    static_assert(LDS_TOTAL <= 160 * 1024, "K of a head, the staging rows and the exchange buffers share the LDS");
};

// Lanes of one wave hand data to each other through LDS inside divergent code: without this the compiler
// is free to run the readers' side of a branch before the writers' side (LDS itself serves a wave in order).
__device__ __forceinline__ void wave_sync_lds()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int NW, int NT>
__global__ __launch_bounds__(64 * NW)
void qk_resident_kernel(const uint16_t* __restrict__ Q, const uint16_t* __restrict__ K, uint16_t* __restrict__ out,
                        float c, uint32_t sign_flip, uint32_t strips_per_head, uint32_t total_strips)
{
    using C = ResidentCfg<NW, NT>;
    constexpr int DB = C::DB, G = C::G, CPR = C::CPR, N = C::N, PIECE_BYTES = C::PIECE_BYTES, NTHREADS = 64 * NW;
    constexpr int ST_PITCH = C::ST_PITCH, ST_BYTES = C::ST_BYTES, CPS = C::CPS, RPI = C::RPI, NF = C::NF;
    constexpr int ST_ROWS = C::ST_ROWS, ST_BLOCKS = C::ST_BLOCKS;

    __shared__ __align__(1024) char lds[C::LDS_TOTAL];
    char* const k_lds = lds;
    char* const st_lds = lds + C::K_BYTES;
    float* const stat = reinterpret_cast<float*>(lds + C::K_BYTES + C::LDS_ST);   // [parity][max, sum][wave][query]

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int l32 = lane & 31;
    const int half = lane >> 5;

    // this workgroup's strips: a contiguous range of the global (head, strip) order
    const uint32_t wg = xcd_contiguous_block_id(blockIdx.x, gridDim.x);
    uint32_t s_cur = (uint32_t)((uint64_t)wg * total_strips / gridDim.x);
    const uint32_t s_end = (uint32_t)((uint64_t)(wg + 1) * total_strips / gridDim.x);

    // K in LDS: piece (w, t) = keys 32 NT w + 32 t .. + 32 at byte (w NT + t) PIECE_BYTES, i.e. simply key * DB;
    // within a row the 16-byte chunk index is XOR-swizzled by the key so that the fragment reads of 16
    // consecutive lanes cover all banks.  Fragment g of piece t of this wave:
    int frag_off[G];
    {
        const int swz = (l32 / C::RPL) & C::SWZ_MASK;
#pragma unroll
        for (int g = 0; g < G; ++g) frag_off[g] = (wave * NT * 32 + l32) * DB + (((2 * g + half) ^ swz) * 16);
    }
    char* const stage = st_lds + wave * ST_BYTES;
    char* const st_wr = stage + (l32 % ST_ROWS) * ST_PITCH + 8 * half;
    const char* const st_rd = stage + (lane / CPS) * ST_PITCH + (lane % CPS) * 16;

    // Q fragments of a strip (global strip index: Q is one dense array of rows): lanes 0..31 carry the even
    // 16-byte chunk of each 32-byte group, lanes 32..63 the odd one.  A negative scale negates Q:
    // softmax(-|c| s) = softmax(|c| (-Q) K^T).
    auto load_q = [&](u32x4 (&qf)[G], uint32_t strip_id) __attribute__((always_inline)) {
        const char* p = reinterpret_cast<const char*>(Q) + ((int64_t)strip_id * 32 + l32) * DB + half * 16;
#pragma unroll
        for (int g = 0; g < G; ++g) qf[g] = *reinterpret_cast<const u32x4*>(p + g * 32) ^ sign_flip;
    };
    // the K of one head, 16 bytes per lane and trip, on its way from memory to LDS
    u32x4 kv[C::K_CHUNKS_PER_LANE];
    auto k_request = [&](uint32_t head) __attribute__((always_inline)) {
        const char* Kh = reinterpret_cast<const char*>(K) + (int64_t)head * N * DB;
#pragma unroll
        for (int j = 0; j < C::K_CHUNKS_PER_LANE; ++j)
            kv[j] = *reinterpret_cast<const u32x4*>(Kh + (int64_t)(j * NTHREADS + tid) * 16);
    };
    auto k_place = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < C::K_CHUNKS_PER_LANE; ++j) {
            const int s = j * NTHREADS + tid;     // chunk index in the head's K: key = s / CPR, chunk = s % CPR
            const int key = s / CPR;
            const int pos = (s % CPR) ^ ((key / C::RPL) & C::SWZ_MASK);
            *reinterpret_cast<u32x4*>(k_lds + key * DB + pos * 16) = kv[j];
        }
    };

    uint32_t parity = 0;
    uint32_t head_in_lds = 0xffffffffu;
    // Q fragments of this strip and of the next one (requested before this strip's stores are issued:
    // vector-memory operations retire in order, and a load behind a burst of stores would wait for it)
    u32x4 qf[G], qf1[G];
    if (s_cur < s_end) load_q(qf, s_cur);
    // Two accumulator sets: while the exponentials of one strip are taken (vector ALU), the scores of the
    // next strip of the same head are accumulated into the other set (matrix cores), one MFMA per chunk of
    // vector work from the same instruction stream.
    f32x16 acc_a[NT], acc_b[NT];
    constexpr int NMMA = NT * G;                  // MFMAs of one sweep
    // fragment of MFMA i of a sweep: piece i / G, group i % G
    auto k_frag = [&](auto ic) __attribute__((always_inline)) -> u32x4 {
        constexpr int i = decltype(ic)::value;
        return *reinterpret_cast<const u32x4*>(k_lds + (i / G) * PIECE_BYTES + frag_off[i % G]);
    };
    auto mma_step = [&](f32x16 (&A)[NT], const u32x4 (&q)[G], const u32x4& kf, auto ic) __attribute__((always_inline)) {
        constexpr int i = decltype(ic)::value;
        if constexpr (i % G == 0) {
#pragma unroll
            for (int r = 0; r < 16; ++r) A[i / G][r] = 0.0f;
        }
        Mma<uint16_t>::run(A[i / G], kf, q[i % G]);
    };
    // a sweep on its own (first strip of a list or of a head)
    auto sweep = [&](f32x16 (&A)[NT], const u32x4 (&q)[G]) __attribute__((always_inline)) {
        static_for<NMMA>([&](auto ic) __attribute__((always_inline)) { mma_step(A, q, k_frag(ic), ic); });
    };

    // one strip whose scores are in X; if `ahead`, the scores of the next strip (Q fragments qn) go to Y
    auto strip_body = [&](f32x16 (&X)[NT], f32x16 (&Y)[NT], const u32x4 (&qn)[G], bool ahead, char* out_rows)
                          __attribute__((always_inline)) {
        // ---- local maximum: of this wave's N / NW keys only.  The exponentials are taken against it; the waves
        //      exchange (reference exponent, local sum) pairs once, after the exponentials, and every wave folds
        //      the difference to the global maximum into its normalising factor -- one barrier per strip, and
        //      the exponentials do not wait for the other waves.
        float* const stat_m = stat + parity * (2 * NW * 32);
        float* const stat_l = stat_m + NW * 32;
        float m = kNegBig;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
#pragma unroll
            for (int r = 0; r < 16; r += 2) m = max3(m, X[t][r], X[t][r + 1]);
        }
        m = fmaxf(m, __shfl_xor(m, 32, 64));      // lanes l and l + 32 hold the two halves of a query's keys

        // ---- exponentials in place of the scores and their local sum; the next strip's sweep rides along ----
        const float mb = m * c;
        float l = 0.0f;
        constexpr int EPC = 16 * NT / NMMA;       // scores per chunk: one MFMA each
        if (ahead) {
            constexpr int LEAD = 3;               // fragments are fetched this many chunks ahead
            u32x4 ring[LEAD];
            static_for<LEAD>([&](auto ic) __attribute__((always_inline)) { ring[decltype(ic)::value] = k_frag(ic); });
            static_for<NMMA>([&](auto ic) __attribute__((always_inline)) {
                constexpr int i = decltype(ic)::value;
#pragma unroll
                for (int e = 0; e < EPC; ++e) {
                    const int idx = i * EPC + e;
                    const float x = fast_exp2(__builtin_fmaf(X[idx / 16][idx % 16], c, -mb));
                    X[idx / 16][idx % 16] = x;
                    l += x;
                }
                mma_step(Y, qn, ring[i % LEAD], ic);
                if constexpr (i + LEAD < NMMA) ring[i % LEAD] = k_frag(IC<i + LEAD>{});
                __builtin_amdgcn_sched_barrier(0);   // the chunk order is the schedule
            });
        } else {
#pragma unroll
            for (int t = 0; t < NT; ++t) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    X[t][r] = fast_exp2(__builtin_fmaf(X[t][r], c, -mb));
                    l += X[t][r];
                }
            }
        }
        l += __shfl_xor(l, 32, 64);
        if (half == 0) {
            stat_m[wave * 32 + l32] = mb;
            stat_l[wave * 32 + l32] = l;
        }
        __syncthreads();
        // global reference exponent and sum (Eq. 1 with the maximum taken over all waves); all exponents are
        // the rounded mb = fl(c * max) the sums were built against, summed in the same order in every wave
        float mbg = mb;
#pragma unroll
        for (int w = 0; w < NW; ++w) mbg = fmaxf(mbg, stat_m[w * 32 + l32]);
        float lg = 0.0f;
#pragma unroll
        for (int w = 0; w < NW; ++w) lg += stat_l[w * 32 + l32] * fast_exp2(stat_m[w * 32 + l32] - mbg);
        const float inv = fast_exp2(mb - mbg) * __builtin_amdgcn_rcpf(lg);
        // The exchange buffers alternate between strips: a wave that has passed this barrier writes the other
        // pair next, and cannot pass the next barrier before every wave has read this one.
        parity ^= 1u;

        // ---- weights: scale, round once, stage [ST_ROWS queries][64 keys], store -----------------------
        char* const out_lane = out_rows + ((int64_t)(lane / CPS) * N + wave * 32 * NT + (lane % CPS) * 8) * 2;
        static_for<NT / 2>([&](auto pc) __attribute__((always_inline)) {
            constexpr int tp = decltype(pc)::value;
            // the lane's 32 weights of this pair of pieces, rounded once -- outside the per-block predicate below
            // (inside it the arithmetic would be issued once per block)
            u32x2 wv[2][4];
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const f32x16& a = X[2 * tp + u];
                    wv[u][r4] = u32x2{pack_bf16x2(a[4 * r4] * inv, a[4 * r4 + 1] * inv),
                                      pack_bf16x2(a[4 * r4 + 2] * inv, a[4 * r4 + 3] * inv)};
                }
#pragma unroll
            for (int hb = 0; hb < ST_BLOCKS; ++hb) {   // queries ST_ROWS hb .. + ST_ROWS of the strip
                if (l32 / ST_ROWS == hb) {
#pragma unroll
                    for (int u = 0; u < 2; ++u)
#pragma unroll
                        for (int r4 = 0; r4 < 4; ++r4)
                            *reinterpret_cast<u32x2*>(st_wr + (u * 32 + 8 * r4) * 2) = wv[u][r4];
                }
                wave_sync_lds();                  // some of the lanes wrote, all of them read
                u32x4 v[NF];
#pragma unroll
                for (int f = 0; f < NF; ++f) v[f] = *reinterpret_cast<const u32x4*>(st_rd + f * RPI * ST_PITCH);
                wave_sync_lds();                  // the rows are in registers before the next block overwrites them
#pragma unroll
                for (int f = 0; f < NF; ++f)
                    __builtin_nontemporal_store(
                        v[f], reinterpret_cast<u32x4*>(out_lane + ((int64_t)(hb * ST_ROWS + f * RPI) * N + 64 * tp) * 2));
            }
        });
    };

    bool swept = false;                           // the current strip's scores are already in its accumulator set
    auto one_strip = [&](f32x16 (&X)[NT], f32x16 (&Y)[NT], uint32_t strip_id) __attribute__((always_inline)) {
        const uint32_t bh = strip_id / strips_per_head;
        const uint32_t strip = strip_id - bh * strips_per_head;
        char* const out_rows = reinterpret_cast<char*>(out) + ((int64_t)bh * N + strip * 32) * (int64_t)N * 2;
        if (bh != head_in_lds) {
            // ======== a new head: its K replaces the previous one ========================================
            k_request(bh);
            __syncthreads();                      // nobody reads the previous head's K any more
            k_place();
            __syncthreads();                      // K is in place
            head_in_lds = bh;
        }
        load_q(qf1, strip_id + 1 < s_end ? strip_id + 1 : strip_id);
        const bool ahead = strip_id + 1 < s_end && (strip_id + 1) / strips_per_head == bh;
        if (!swept) sweep(X, qf);
        strip_body(X, Y, qf1, ahead, out_rows);
        swept = ahead;
#pragma unroll
        for (int g = 0; g < G; ++g) qf[g] = qf1[g];
    };
    // the two accumulator sets swap roles from strip to strip: the loop is unrolled by two so that each role
    // is a fixed set of registers
    for (uint32_t strip_id = s_cur; strip_id < s_end; strip_id += 2) {
        one_strip(acc_a, acc_b, strip_id);
        if (strip_id + 1 < s_end) one_strip(acc_b, acc_a, strip_id + 1);
    }
}

template <int NW, int NT>
hipError_t launch_resident(const void* Q, const void* K, void* out, int64_t BH, float scale, hipStream_t stream)
{
    const uint32_t strips_per_head = NW * NT;
    const uint32_t total = (uint32_t)(BH * strips_per_head);
    // persistent workgroups, one per compute unit, each with a contiguous list of strips
    uint32_t grid = (uint32_t)((compute_units() + 7) / 8 * 8);
    if (grid > total) grid = (total + 7) / 8 * 8;
    const float c = fabsf(scale) * kLog2e;
    const uint32_t flip = scale < 0.0f ? Mma<uint16_t>::kSignMask : 0u;
    hipLaunchKernelGGL((qk_resident_kernel<NW, NT>), dim3(grid), dim3(64 * NW), 0, stream, static_cast<const uint16_t*>(Q),
                       static_cast<const uint16_t*>(K), static_cast<uint16_t*>(out), c, flip, strips_per_head, total);
    return hipGetLastError();
}

}  // namespace

bool qk_resident_supported(int64_t BH, int64_t N, int64_t d)
{
    // rows of exactly 128 bytes; N / 8 keys per wave in whole pairs of 32-key pieces, at most 64 registers of scores
    if (d != 64 || (N != 512 && N != 1024)) return false;
    return BH * (N / 32) <= (int64_t)0x7ffffff0;
}

hipError_t launch_qk_resident(const void* Q, const void* K, void* out, int64_t BH, int64_t N, float scale, hipStream_t stream)
{
    if (N == 512) return launch_resident<8, 2>(Q, K, out, BH, scale, stream);
    return launch_resident<8, 4>(Q, K, out, BH, scale, stream);
}

}  // namespace attnw
