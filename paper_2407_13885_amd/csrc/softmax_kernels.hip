// Dedicated row softmax over precomputed scores (the paper's Softmax kernel:
// Softmax section, max-subtracted form of Eq. 1; its Grayskull version keeps one
// row of tiles resident in a core's SRAM and walks max -> subtract -> exp -> sum
// -> normalise).  Here a row lives in the registers of one wavefront (or of one
// workgroup for long rows): it is read from HBM once with 16-byte loads, reduced
// with cross-lane shuffles, and written once with 16-byte stores, so the kernel
// moves 2 * sizeof(T) bytes per element and nothing else.
#include "device_utils.h"
#include "launchers.h"

namespace attnw {
namespace {

template <typename T> struct Elem;

template <> struct Elem<float> {
    static constexpr int VEC = 4;   // elements per 16-byte chunk
    static __device__ __forceinline__ void unpack(const u32x4& v, float* x)
    {
#pragma unroll
        for (int i = 0; i < 4; ++i) x[i] = __uint_as_float(v[i]);
    }
    static __device__ __forceinline__ u32x4 pack(const float* x)
    {
        u32x4 v;
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = __float_as_uint(x[i]);
        return v;
    }
    static __device__ __forceinline__ float load1(const float* p) { return *p; }
    static __device__ __forceinline__ void store1(float* p, float v) { *p = v; }
};

template <> struct Elem<uint16_t> {   // bf16 bit patterns
    static constexpr int VEC = 8;
    static __device__ __forceinline__ void unpack(const u32x4& v, float* x)
    {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            x[2 * i] = bf16_lo_to_f32(v[i]);
            x[2 * i + 1] = bf16_hi_to_f32(v[i]);
        }
    }
    static __device__ __forceinline__ u32x4 pack(const float* x)
    {
        u32x4 v;
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = pack_bf16x2(x[2 * i], x[2 * i + 1]);
        return v;
    }
    static __device__ __forceinline__ float load1(const uint16_t* p) { return __uint_as_float((uint32_t)*p << 16); }
    static __device__ __forceinline__ void store1(uint16_t* p, float v) { *p = (uint16_t)(pack_bf16x2(v, 0.0f) & 0xffffu); }
};

// Maximum / sum over the TPR consecutive lanes (a power of two, at most 64) that share a row.
template <int TPR> __device__ __forceinline__ float lanes_reduce_max(float v)
{
#pragma unroll
    for (int off = (TPR < 64 ? TPR : 64) / 2; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}
template <int TPR> __device__ __forceinline__ float lanes_reduce_sum(float v)
{
#pragma unroll
    for (int off = (TPR < 64 ? TPR : 64) / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// One row per TPR threads; every thread keeps R groups of E elements of the row in registers
// (E = the larger of the two types' elements per 16-byte chunk: a group is one chunk of the
// narrower type and one or two of the wider).  TPR <= 64: 256 / TPR rows per 256-thread block,
// reductions among the lanes of a row only (short rows share a wave: with one wave per row a
// 96-byte row would keep 6 of 64 lanes busy).  TPR > 64: one row per block, partial results meet
// in LDS.  Requires cols to be a multiple of E (groups = cols / E <= R * TPR).
template <typename TI, typename TO, int R, int TPR>
__global__ __launch_bounds__(TPR <= 64 ? 256 : TPR)
void softmax_rows_kernel(const TI* S, TO* P, int64_t rows, int groups)   // S == P (in place, TI == TO) is allowed
{
    constexpr int VI = Elem<TI>::VEC, VO = Elem<TO>::VEC;
    constexpr int E = VI > VO ? VI : VO;
    constexpr int CI = E / VI, CO = E / VO;     // 16-byte chunks per group on the way in / out
    constexpr int WAVES = (TPR <= 64) ? 1 : TPR / 64;
    constexpr int RPB = (TPR <= 64) ? 256 / TPR : 1;   // rows per block
    const int tid = (TPR <= 64) ? (int)(threadIdx.x % TPR) : (int)threadIdx.x;
    const int64_t row = (TPR <= 64) ? (int64_t)blockIdx.x * RPB + (threadIdx.x / TPR) : (int64_t)blockIdx.x;
    if (row >= rows) return;   // all lanes of a row (TPR <= 64) or the whole block leave together

    const u32x4* src = reinterpret_cast<const u32x4*>(S) + row * groups * CI;
    u32x4* dst = reinterpret_cast<u32x4*>(P) + row * groups * CO;

    u32x4 raw[R][CI];
#pragma unroll
    for (int k = 0; k < R; ++k) {
        const int c = tid + k * TPR;
        if (c < groups) {
#pragma unroll
            for (int j = 0; j < CI; ++j) raw[k][j] = __builtin_nontemporal_load(src + c * CI + j);
        }
    }

    float x[R][E];
    float m = -INFINITY;
#pragma unroll
    for (int k = 0; k < R; ++k) {
        const int c = tid + k * TPR;
        if (c < groups) {
#pragma unroll
            for (int j = 0; j < CI; ++j) Elem<TI>::unpack(raw[k][j], x[k] + j * VI);
        } else {
#pragma unroll
            for (int i = 0; i < E; ++i) x[k][i] = -INFINITY;
        }
#pragma unroll
        for (int i = 0; i < E; ++i) m = fmaxf(m, x[k][i]);
    }

    __shared__ float red[2][WAVES];
    m = lanes_reduce_max<TPR>(m);
    if constexpr (WAVES > 1) {
        if ((threadIdx.x & 63) == 0) red[0][threadIdx.x >> 6] = m;
        __syncthreads();
#pragma unroll
        for (int w = 0; w < WAVES; ++w) m = fmaxf(m, red[0][w]);
    }

    // e = exp(x - m) = 2^((x - m) * log2 e); the subtraction is done first so that
    // large common offsets cancel exactly.
    float l = 0.0f;
#pragma unroll
    for (int k = 0; k < R; ++k) {
#pragma unroll
        for (int i = 0; i < E; ++i) {
            x[k][i] = fast_exp2((x[k][i] - m) * kLog2e);
            l += x[k][i];
        }
    }
    l = lanes_reduce_sum<TPR>(l);
    if constexpr (WAVES > 1) {
        if ((threadIdx.x & 63) == 0) red[1][threadIdx.x >> 6] = l;
        __syncthreads();
        l = 0.0f;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) l += red[1][w];
    }
    const float inv = 1.0f / l;

#pragma unroll
    for (int k = 0; k < R; ++k) {
        const int c = tid + k * TPR;
        if (c < groups) {
#pragma unroll
            for (int i = 0; i < E; ++i) x[k][i] *= inv;
#pragma unroll
            for (int j = 0; j < CO; ++j) __builtin_nontemporal_store(Elem<TO>::pack(x[k] + j * VO), dst + c * CO + j);
        }
    }
}

// Rows that do not start on 16-byte boundaries (cols not a multiple of the elements per chunk), same type in and
// out: the matrix is one contiguous array, so a row is still covered by ALIGNED 16-byte chunks -- the first and the
// last of them shared with the neighbouring rows.  A row is read as those chunks (elements of the neighbours masked
// out: the softmax does not care where in a chunk an element sits), kept in registers as in softmax_rows_kernel,
// and written back as whole chunks except the two shared ones, of which only the row's own elements are stored, one
// by one.  The chunk that would reach past the end of the matrix (last row) is read element by element.
// chunks of a row <= cols / V + 2 <= R * TPR.
template <typename T, int R, int TPR>
__global__ __launch_bounds__(TPR <= 64 ? 256 : TPR)
void softmax_rows_shifted_kernel(const T* S, T* P, int64_t rows, int cols)   // S == P (in place) is allowed
{
    constexpr int V = Elem<T>::VEC;
    constexpr int WAVES = (TPR <= 64) ? 1 : TPR / 64;
    constexpr int RPB = (TPR <= 64) ? 256 / TPR : 1;
    const int tid = (TPR <= 64) ? (int)(threadIdx.x % TPR) : (int)threadIdx.x;
    const int slot = (TPR <= 64) ? (int)(threadIdx.x / TPR) : 0;      // the row's place in the block
    const int64_t row = (TPR <= 64) ? (int64_t)blockIdx.x * RPB + slot : (int64_t)blockIdx.x;
    // (rows past the end -- the last block of several rows per block -- stay to the end: the block meets at a barrier)
    const bool active = row < rows;

    // (S and P are 16-byte aligned: chunk c of the arrays holds elements V c .. V c + V - 1)
    const int64_t e0 = row * cols;
    const int64_t c0 = e0 / V;
    const int rel0 = (int)(c0 * V - e0);                              // -V < rel0 <= 0: the first chunk's first element, relative to the row
    const int n_chunks = (cols - rel0 + V - 1) / V;
    const bool last_row = row == rows - 1;                            // its last chunk may reach past the end of the arrays
    const u32x4* const src = reinterpret_cast<const u32x4*>(S) + c0;
    u32x4* const dst = reinterpret_cast<u32x4*>(P) + c0;

    float x[R][V];
    float m = -INFINITY;
#pragma unroll
    for (int k = 0; k < R; ++k) {
        const int c = tid + k * TPR;
        const int rel = rel0 + c * V;                                 // row index of the chunk's first element
        const bool mine = active && c < n_chunks;
        const bool whole = mine && rel >= 0 && rel + V <= cols;
        if (__builtin_amdgcn_ballot_w64(mine && !whole) == 0) {       // (wave-uniform) no lane of the wave holds a shared chunk
            if (mine) Elem<T>::unpack(__builtin_nontemporal_load(src + c), x[k]);
            else {
#pragma unroll
                for (int i = 0; i < V; ++i) x[k][i] = -INFINITY;
            }
        } else {
            float y[V];
#pragma unroll
            for (int i = 0; i < V; ++i) y[i] = -INFINITY;
            if (mine && !(last_row && rel + V > cols)) Elem<T>::unpack(__builtin_nontemporal_load(src + c), y);
            else if (mine) {
#pragma unroll
                for (int i = 0; i < V; ++i)
                    if ((unsigned)(rel + i) < (unsigned)cols) y[i] = Elem<T>::load1(S + e0 + rel + i);
            }
#pragma unroll
            for (int i = 0; i < V; ++i) x[k][i] = (mine && (unsigned)(rel + i) < (unsigned)cols) ? y[i] : -INFINITY;
        }
#pragma unroll
        for (int i = 0; i < V; ++i) m = fmaxf(m, x[k][i]);
    }

    __shared__ float red[2][WAVES];
    m = lanes_reduce_max<TPR>(m);
    if constexpr (WAVES > 1) {
        if ((threadIdx.x & 63) == 0) red[0][threadIdx.x >> 6] = m;
        __syncthreads();
#pragma unroll
        for (int w = 0; w < WAVES; ++w) m = fmaxf(m, red[0][w]);
    }
    float l = 0.0f;
#pragma unroll
    for (int k = 0; k < R; ++k) {
#pragma unroll
        for (int i = 0; i < V; ++i) {
            x[k][i] = fast_exp2((x[k][i] - m) * kLog2e);   // masked elements: 2^-inf = 0
            l += x[k][i];
        }
    }
    l = lanes_reduce_sum<TPR>(l);
    if constexpr (WAVES > 1) {
        if ((threadIdx.x & 63) == 0) red[1][threadIdx.x >> 6] = l;
        __syncthreads();
        l = 0.0f;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) l += red[1][w];
    }
    const float inv = 1.0f / l;

    // The chunk that two rows of this block share leaves as ONE 16-byte store: the upper row parks its elements of it
    // (the weights of masked elements are zeros, so are their bits) and the lower row, whose first chunk it is, ORs its
    // own in.  Only the chunks shared with the rows of other blocks are still written element by element.
    // (in place: every load of the block precedes the barrier, the merged store follows it)
    // Where two or more rows share a wave (bf16: 200000 x 197 40.5 -> 34.5 us, 300000 x 131 48 -> 40, 100000 x 394
    // 34 -> 31.5); with a wave per row the barrier costs more than the element stores (24576 x 2047 43.5 -> 48).
    constexpr bool MERGE = TPR <= 32;
    __shared__ u32x4 edge[RPB];
    bool parked = false;                                   // this lane's last chunk left through `edge`
    if constexpr (MERGE) {
        const int c_last = n_chunks - 1;
#pragma unroll
        for (int k = 0; k < R; ++k) {
            const int c = tid + k * TPR;
            if (active && c == c_last && rel0 + c * V + V > cols && slot + 1 < RPB && row + 1 < rows) {
                float y[V];
#pragma unroll
                for (int i = 0; i < V; ++i) y[i] = x[k][i] * inv;   // (elements past the row: 0 * inv = 0)
                edge[slot] = Elem<T>::pack(y);
                parked = true;
            }
        }
        __syncthreads();
    }

#pragma unroll
    for (int k = 0; k < R; ++k) {
        const int c = tid + k * TPR;
        const int rel = rel0 + c * V;
        const bool mine = active && c < n_chunks;
        const bool whole = mine && rel >= 0 && rel + V <= cols;
#pragma unroll
        for (int i = 0; i < V; ++i) x[k][i] *= inv;
        if (whole) {
            __builtin_nontemporal_store(Elem<T>::pack(x[k]), dst + c);
        } else if (mine) {
            if (MERGE && c == 0 && rel < 0 && slot > 0) {            // shared with the row above, which is in this block
                const u32x4 a = edge[slot - 1], b = Elem<T>::pack(x[k]);
                __builtin_nontemporal_store(u32x4{a[0] | b[0], a[1] | b[1], a[2] | b[2], a[3] | b[3]}, dst + c);
            } else if (!(parked && c == n_chunks - 1)) {
#pragma unroll
                for (int i = 0; i < V; ++i)
                    if ((unsigned)(rel + i) < (unsigned)cols) Elem<T>::store1(P + e0 + rel + i, x[k][i]);
            }
        }
    }
}

// EG consecutive elements of type T (EG * sizeof(T) bytes, naturally aligned) <-> floats
template <typename T, int EG> __device__ __forceinline__ void load_group(const T* p, float* x)
{
    if constexpr (EG == 1) {
        x[0] = Elem<T>::load1(p);
    } else if constexpr (sizeof(T) == 2) {            // bf16: 2 or 4 elements = 4 or 8 bytes
        uint32_t w[EG / 2];
        if constexpr (EG == 2) w[0] = *reinterpret_cast<const uint32_t*>(p);
        else { const u32x2 v = *reinterpret_cast<const u32x2*>(p); w[0] = v[0]; w[1] = v[1]; }
#pragma unroll
        for (int i = 0; i < EG / 2; ++i) { x[2 * i] = bf16_lo_to_f32(w[i]); x[2 * i + 1] = bf16_hi_to_f32(w[i]); }
    } else {                                          // fp32: 2 or 4 elements = 8 or 16 bytes
        if constexpr (EG == 2) { const f32x2 v = *reinterpret_cast<const f32x2*>(p); x[0] = v[0]; x[1] = v[1]; }
        else { const f32x4 v = *reinterpret_cast<const f32x4*>(p); x[0] = v[0]; x[1] = v[1]; x[2] = v[2]; x[3] = v[3]; }
    }
}
template <typename T, int EG> __device__ __forceinline__ void store_group(T* p, const float* x)
{
    if constexpr (EG == 1) {
        Elem<T>::store1(p, x[0]);
    } else if constexpr (sizeof(T) == 2) {
        if constexpr (EG == 2) *reinterpret_cast<uint32_t*>(p) = pack_bf16x2(x[0], x[1]);
        else { u32x2 v = {pack_bf16x2(x[0], x[1]), pack_bf16x2(x[2], x[3])}; *reinterpret_cast<u32x2*>(p) = v; }
    } else {
        if constexpr (EG == 2) { f32x2 v = {x[0], x[1]}; *reinterpret_cast<f32x2*>(p) = v; }
        else { f32x4 v = {x[0], x[1], x[2], x[3]}; *reinterpret_cast<f32x4*>(p) = v; }
    }
}

// Short rows whose length is not a whole number of 16-byte chunks of both types (groups = cols / EG <= R * TPR):
// one row per TPR lanes, lane j holds groups j, j + TPR, ... of EG consecutive elements in registers, EG = the
// largest of 4, 2, 1 that divides cols (a row then starts on a multiple of EG elements: accesses of EG elements
// are naturally aligned).  The row is read once.
template <typename TI, typename TO, int R, int TPR, int EG>
__global__ __launch_bounds__(256)
void softmax_elem_kernel(const TI* S, TO* P, int64_t rows, int cols)
{
    constexpr int RPB = 256 / TPR;
    const int tid = (int)(threadIdx.x % TPR);
    const int64_t row = (int64_t)blockIdx.x * RPB + (threadIdx.x / TPR);
    if (row >= rows) return;
    const TI* src = S + row * cols;
    TO* dst = P + row * cols;
    const int groups = cols / EG;
    float x[R][EG];
    // absent elements are -inf: below every finite score, however low (a fully masked row of the lowest
    // finite value is uniform, Eq. 1), and 2^(-inf - m) = 0
    float m = -INFINITY;
#pragma unroll
    for (int k = 0; k < R; ++k) {
        const int g = tid + k * TPR;
        if (g < groups) {
            load_group<TI, EG>(src + g * EG, x[k]);
        } else {
#pragma unroll
            for (int i = 0; i < EG; ++i) x[k][i] = -INFINITY;
        }
#pragma unroll
        for (int i = 0; i < EG; ++i) m = fmaxf(m, x[k][i]);
    }
    m = lanes_reduce_max<TPR>(m);
    float l = 0.0f;
#pragma unroll
    for (int k = 0; k < R; ++k) {
#pragma unroll
        for (int i = 0; i < EG; ++i) {
            x[k][i] = fast_exp2((x[k][i] - m) * kLog2e);     // absent elements: 2^(-inf) = 0
            l += x[k][i];
        }
    }
    l = lanes_reduce_sum<TPR>(l);
    const float inv = 1.0f / l;
#pragma unroll
    for (int k = 0; k < R; ++k) {
        const int g = tid + k * TPR;
        if (g < groups) {
#pragma unroll
            for (int i = 0; i < EG; ++i) x[k][i] *= inv;
            store_group<TO, EG>(dst + g * EG, x[k]);
        }
    }
}

// Many short rows off the 16-byte boundaries (cols = 49, 33, 17 ...: a row per window of tokens) or of one or two chunks,
// scores and weights of one type.  G consecutive rows -- G = 8, 4, 2 or 1 (fp32: 4, 2, 1), the fewest whose G * cols elements are whole 16-byte chunks
// -- start on a chunk boundary again, so a WAVE takes RW rows (a multiple of G, at most 64) that are CW <= 64 whole chunks
// of memory: lane c < CW loads chunk c (16 bytes, consecutive lanes consecutive chunks) and parks it in the wave's LDS
// area as it lies in memory; then LPR lanes (a power of two, RW * LPR <= 64) share a row, each reads up to EPL of its
// elements from there (Eq. 1: maximum and sum over the lanes of the row by shuffles), writes the weights back in
// place, and lane c stores chunk c.  The rows are read and written once, 16 bytes per lane; no barrier (a wave's LDS
// operations are served in order).  The last chunk of the matrix, if the matrix does not end on a chunk boundary,
// is loaded and stored element by element.
template <typename T, int EPL>
__global__ __launch_bounds__(256)
void softmax_packed_kernel(const T* S, T* P, int64_t rows, int cols, int RW, int CW, int LPR)
{
    constexpr int V = Elem<T>::VEC;
    __shared__ __align__(16) T area_lds[4][64 * V];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    T* const area = area_lds[wave];
    const int64_t it = (int64_t)blockIdx.x * 4 + wave;        // this wave's rows: it * RW ... (the same for its chunks)
    const int64_t row0 = it * RW;
    if (row0 >= rows) return;
    const int n_rows = (int)(rows - row0 < RW ? rows - row0 : RW);
    const int n_elems = n_rows * cols;
    const int n_chunks = (n_elems + V - 1) / V;                // (the last one partial only at the end of the matrix)
    const int64_t e_base = row0 * cols;                        // a multiple of V
    const bool mine = lane < n_chunks;
    const bool partial = mine && (lane + 1) * V > n_elems;

    // ---- the chunks into LDS as they lie in memory ---------------------------------------------------------------------
    if (mine) {
        u32x4 v = {0u, 0u, 0u, 0u};
        if (!partial) {
            v = *reinterpret_cast<const u32x4*>(S + e_base + (int64_t)lane * V);
            *reinterpret_cast<u32x4*>(area + lane * V) = v;
        } else {
            for (int i = 0; lane * V + i < n_elems; ++i) area[lane * V + i] = S[e_base + lane * V + i];
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    // ---- LPR lanes per row --------------------------------------------------------------------------------------------------
    const int r = lane / LPR, part = lane - r * LPR;
    const int epl = (cols + LPR - 1) / LPR;                     // elements per lane (<= EPL)
    const int c0 = part * epl;
    const bool row_here = r < n_rows;
    T* const rowp = area + (row_here ? r : 0) * cols;
    float x[EPL];
    float m = -INFINITY;                                        // absent elements: below every finite score, 2^(-inf - m) = 0
#pragma unroll
    for (int i = 0; i < EPL; ++i) {
        const bool have = row_here && i < epl && c0 + i < cols;
        x[i] = have ? Elem<T>::load1(rowp + (have ? c0 + i : 0)) : -INFINITY;
        m = fmaxf(m, x[i]);
    }
    for (int off = LPR >> 1; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
    m = row_here ? m : 0.0f;                                    // (lanes without a row: keep the arithmetic finite)
    float l = 0.0f;
#pragma unroll
    for (int i = 0; i < EPL; ++i) {
        x[i] = fast_exp2((x[i] - m) * kLog2e);
        l += x[i];
    }
    for (int off = LPR >> 1; off > 0; off >>= 1) l += __shfl_xor(l, off, 64);
    const float inv = 1.0f / l;
#pragma unroll
    for (int i = 0; i < EPL; ++i)
        if (row_here && i < epl && c0 + i < cols) Elem<T>::store1(rowp + c0 + i, x[i] * inv);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    // ---- the chunks leave ----------------------------------------------------------------------------------------------------
    if (mine) {
        if (!partial) {
            const u32x4 v = *reinterpret_cast<const u32x4*>(area + lane * V);
            __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(P + e_base + (int64_t)lane * V));
        } else {
            for (int i = 0; lane * V + i < n_elems; ++i) P[e_base + lane * V + i] = area[lane * V + i];
        }
    }
}

// Rows that do not fit the registers of a workgroup, and long rows that do not start on 16-byte
// boundaries.  The row is read twice (statistics, then weights) with 16-byte accesses: the elements of
// a row in front of its first 16-byte boundary (of both the scores and the weights: they have the same
// element index) and behind its last whole group are handled one by one.
//
// MODE 0: one workgroup per row does both passes (the only mode that works in place, S == P).
// Few long rows would leave most of the chip idle that way: the row is then cut into `chunks` pieces, one
// workgroup each, and the call becomes two launches on the stream.
// MODE 1: the statistics (maximum, sum) of each piece.  The pieces of a row have to learn each other's
//         statistics, and the only memory the call may write is P: the workgroup of piece c stores its
//         pair into slot c of a small table at the start of EVERY piece's part of P (chunks * 8 bytes,
//         a piece is at least 16 KiB).
// MODE 2: the workgroup of a piece reads the table at the start of its OWN part of P -- nobody else reads
//         or writes that part during this launch -- folds the pairs into the row's maximum and sum, and
//         overwrites the part, table included, with the weights.
template <typename TI, typename TO, int T, int MODE>      // T threads per workgroup
__global__ __launch_bounds__(T)
void softmax_long_kernel(const TI* S, TO* P, int64_t rows, int64_t cols, int chunks)
{
    constexpr int VI = Elem<TI>::VEC, VO = Elem<TO>::VEC;
    constexpr int E = VI > VO ? VI : VO;
    constexpr int CI = E / VI, CO = E / VO;
    constexpr int WAVES = T / 64;
    constexpr int U = 2;                                   // groups in flight per thread
    const int64_t row = blockIdx.x / (uint32_t)chunks;
    const int chunk = (int)(blockIdx.x % (uint32_t)chunks);
    const int tid = (int)threadIdx.x;
    const TI* src = S + row * cols;
    TO* dst = P + row * cols;
    // base pointers are 16-byte aligned: element index (row * cols + j) a multiple of E puts both the
    // score and the weight of element j on a 16-byte boundary
    const int64_t head = min(cols, (int64_t)((E - (row * cols) % E) % E));
    const int64_t ngroups = (cols - head) / E;
    const int64_t tail0 = head + ngroups * E;
    const u32x4* vsrc = reinterpret_cast<const u32x4*>(src + head);
    u32x4* vdst = reinterpret_cast<u32x4*>(dst + head);
    // groups of this workgroup's piece (MODE 0: chunks == 1, the whole row)
    auto piece_begin = [&](int c) __attribute__((always_inline)) { return ngroups * c / chunks; };
    const int64_t g0 = piece_begin(chunk), g1 = piece_begin(chunk + 1);

    // ---- statistics: per-thread running maximum m and l = sum 2^((x - m) log2 e) -------------------------
    // "nothing seen yet" is (-inf, 0): any finite score, however low, replaces it (2^(-inf) = 0 clears the
    // empty sum); two empty pairs are merged with factor 1, never through -inf - (-inf)
    float m = -INFINITY, l = 0.0f;
    auto fold = [&](const float* x, int n) __attribute__((always_inline)) {
        float gm = x[0];
#pragma unroll
        for (int i = 1; i < n; ++i) gm = fmaxf(gm, x[i]);
        const float mn = fmaxf(m, gm);
        float sum = 0.0f;
#pragma unroll
        for (int i = 0; i < n; ++i) sum += fast_exp2((x[i] - mn) * kLog2e);
        l = l * fast_exp2((m - mn) * kLog2e) + sum;       // exactly l + sum while the maximum stands
        m = mn;
    };
    if constexpr (MODE != 2) {
        for (int64_t g = g0 + tid; g < g1; g += (int64_t)T * U) {
            u32x4 raw[U][CI];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int64_t gg = g + (int64_t)u * T;
                if (gg < g1) {
#pragma unroll
                    for (int j = 0; j < CI; ++j) raw[u][j] = vsrc[gg * CI + j];
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (g + (int64_t)u * T < g1) {
                    float x[E];
#pragma unroll
                    for (int j = 0; j < CI; ++j) Elem<TI>::unpack(raw[u][j], x + j * VI);
                    fold(x, E);
                }
            }
        }
        if (chunk == 0 && tid < head) { const float x = Elem<TI>::load1(src + tid); fold(&x, 1); }
        if (chunk == chunks - 1 && tail0 + tid < cols) { const float x = Elem<TI>::load1(src + tail0 + tid); fold(&x, 1); }
    } else {
        // the pairs of all pieces of the row, from the table in this piece's own part of P
        if (tid < chunks) {
            const f32x2 pr = reinterpret_cast<const f32x2*>(vdst + g0 * CO)[tid];
            m = pr[0];
            l = pr[1];
        }
    }

    // ---- (m, l) pairs of all threads folded into one ------------------------------------------------------
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const float mo = __shfl_xor(m, off, 64), lo = __shfl_xor(l, off, 64);
        const float mn = fmaxf(m, mo);
        const float fa = m == mn ? 1.0f : fast_exp2((m - mn) * kLog2e);
        const float fb = mo == mn ? 1.0f : fast_exp2((mo - mn) * kLog2e);
        l = l * fa + lo * fb;
        m = mn;
    }
    __shared__ float sm[WAVES], sl[WAVES];
    if ((tid & 63) == 0) { sm[tid >> 6] = m; sl[tid >> 6] = l; }
    // also orders every read above (the scores in place, the table in MODE 2) before any write below
    __syncthreads();
    m = sm[0];
#pragma unroll
    for (int w = 1; w < WAVES; ++w) m = fmaxf(m, sm[w]);
    l = 0.0f;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) l += sl[w] * fast_exp2((sm[w] - m) * kLog2e);

    if constexpr (MODE == 1) {
        // slot `chunk` of the table of every piece of this row
        if (tid < chunks) {
            f32x2 pr = {m, l};
            reinterpret_cast<f32x2*>(vdst + piece_begin(tid) * CO)[chunk] = pr;
        }
        return;
    }
    const float inv = 1.0f / l;

    // ---- weights of this workgroup's piece of the row ----------------------------------------------------
    for (int64_t g = g0 + tid; g < g1; g += (int64_t)T * U) {
        u32x4 raw[U][CI];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t gg = g + (int64_t)u * T;
            if (gg < g1) {
#pragma unroll
                for (int j = 0; j < CI; ++j) raw[u][j] = vsrc[gg * CI + j];
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t gg = g + (int64_t)u * T;
            if (gg < g1) {
                float x[E];
#pragma unroll
                for (int j = 0; j < CI; ++j) Elem<TI>::unpack(raw[u][j], x + j * VI);
#pragma unroll
                for (int i = 0; i < E; ++i) x[i] = fast_exp2((x[i] - m) * kLog2e) * inv;
#pragma unroll
                for (int j = 0; j < CO; ++j) __builtin_nontemporal_store(Elem<TO>::pack(x + j * VO), vdst + gg * CO + j);
            }
        }
    }
    if (chunk == 0 && tid < head)
        Elem<TO>::store1(dst + tid, fast_exp2((Elem<TI>::load1(src + tid) - m) * kLog2e) * inv);
    if (chunk == chunks - 1 && tail0 + tid < cols)
        Elem<TO>::store1(dst + tail0 + tid, fast_exp2((Elem<TI>::load1(src + tail0 + tid) - m) * kLog2e) * inv);
}

template <typename TI, typename TO, int R, int TPR>
hipError_t launch_rows(const void* S, void* P, int64_t rows, int groups, hipStream_t stream)
{
    constexpr int RPB = (TPR <= 64) ? 256 / TPR : 1;
    const int64_t blocks = (rows + RPB - 1) / RPB;
    const int threads = (TPR <= 64) ? 256 : TPR;
    hipLaunchKernelGGL((softmax_rows_kernel<TI, TO, R, TPR>), dim3((uint32_t)blocks), dim3(threads), 0, stream,
                       static_cast<const TI*>(S), static_cast<TO*>(P), rows, groups);
    return hipGetLastError();
}

template <typename TI, typename TO, int R, int TPR, int EG>
hipError_t launch_elem(const void* S, void* P, int64_t rows, int cols, hipStream_t stream)
{
    constexpr int RPB = 256 / TPR;
    hipLaunchKernelGGL((softmax_elem_kernel<TI, TO, R, TPR, EG>), dim3((uint32_t)((rows + RPB - 1) / RPB)), dim3(256), 0,
                       stream, static_cast<const TI*>(S), static_cast<TO*>(P), rows, cols);
    return hipGetLastError();
}

// cols <= 1024 with cols % EG == 0: lanes per row and groups per lane by the number of groups
template <typename TI, typename TO, int EG>
hipError_t launch_elem_groups(const void* S, void* P, int64_t rows, int cols, hipStream_t stream)
{
    const int groups = cols / EG;
    if (groups <= 16) return launch_elem<TI, TO, 1, 16, EG>(S, P, rows, cols, stream);
    if (groups <= 32) return launch_elem<TI, TO, 1, 32, EG>(S, P, rows, cols, stream);
    if (groups <= 64) return launch_elem<TI, TO, 1, 64, EG>(S, P, rows, cols, stream);
    if (groups <= 256) return launch_elem<TI, TO, 4, 64, EG>(S, P, rows, cols, stream);
    return launch_elem<TI, TO, 16 / EG, 64, EG>(S, P, rows, cols, stream);
}

// Shape of the packed kernel for rows of `cols` elements, or false if it does not take them: G rows per chunk-aligned
// group, GW groups per wave while rows and chunks stay within 64 and a lane's share of a row within 8 elements.
template <typename T>
bool packed_shape(int64_t cols, int* RW, int* CW, int* LPR, int* EPL)
{
    constexpr int V = Elem<T>::VEC;
    if (cols < 1) return false;
    int G = V;
    while (G > 1 && (cols * (G / 2)) % V == 0) G /= 2;
    const int64_t CG = cols * G / V;
    if (CG > 64) return false;
    int best = 0;
    for (int gw = 1; gw * G <= 64 && gw * CG <= 64; ++gw) {
        int lpr = 1;
        while (lpr * 2 * gw * G <= 64) lpr *= 2;
        if ((cols + lpr - 1) / lpr <= 8) best = gw;
    }
    if (best == 0) return false;
    *RW = best * G;
    *CW = (int)(best * CG);
    int lpr = 1;
    while (lpr * 2 * *RW <= 64) lpr *= 2;
    *LPR = lpr;
    *EPL = (int)((cols + lpr - 1) / lpr);
    return true;
}

template <typename T>
hipError_t launch_packed(const void* S, void* P, int64_t rows, int cols, int RW, int CW, int LPR, int EPL, hipStream_t stream)
{
    const int64_t its = (rows + RW - 1) / RW;
    if ((its + 3) / 4 > (int64_t)0x7fffffff) return hipErrorInvalidValue;
    const dim3 grid((uint32_t)((its + 3) / 4));
    const T* s_ = static_cast<const T*>(S);
    T* p_ = static_cast<T*>(P);
    if (EPL <= 2) hipLaunchKernelGGL((softmax_packed_kernel<T, 2>), grid, dim3(256), 0, stream, s_, p_, rows, cols, RW, CW, LPR);
    else if (EPL <= 4) hipLaunchKernelGGL((softmax_packed_kernel<T, 4>), grid, dim3(256), 0, stream, s_, p_, rows, cols, RW, CW, LPR);
    else hipLaunchKernelGGL((softmax_packed_kernel<T, 8>), grid, dim3(256), 0, stream, s_, p_, rows, cols, RW, CW, LPR);
    return hipGetLastError();
}

template <typename T, int R, int TPR>
hipError_t launch_rows_shifted(const void* S, void* P, int64_t rows, int64_t cols, hipStream_t stream)
{
    constexpr int RPB = (TPR <= 64) ? 256 / TPR : 1;
    const int64_t blocks = (rows + RPB - 1) / RPB;
    const int threads = (TPR <= 64) ? 256 : TPR;
    hipLaunchKernelGGL((softmax_rows_shifted_kernel<T, R, TPR>), dim3((uint32_t)blocks), dim3(threads), 0, stream,
                       static_cast<const T*>(S), static_cast<T*>(P), rows, (int)cols);
    return hipGetLastError();
}

template <typename TI, typename TO>
hipError_t launch_softmax_t(const void* S, void* P, int64_t rows, int64_t cols, hipStream_t stream)
{
    constexpr int E = Elem<TI>::VEC > Elem<TO>::VEC ? Elem<TI>::VEC : Elem<TO>::VEC;
    // Register-resident rows: a thread keeps up to 64 fp32 values (8 groups of 8 elements, 16 of 4).
    constexpr int MAXR = 64 / E;
    // (many rows of one or two chunks: most lanes of the kernel below would idle -- 2 * 10^6 rows of 8 bf16 values
    // 26 -> 12 us, 10^6 of 16 16.5 -> 13.5; from three chunks on the kernel below is as fast or faster)
    if constexpr (sizeof(TI) == sizeof(TO)) {
        int RW, CW, LPR, EPL;
        if (cols % E == 0 && cols / E <= 2 && rows >= 1024 && packed_shape<TI>(cols, &RW, &CW, &LPR, &EPL))
            return launch_packed<TI>(S, P, rows, (int)cols, RW, CW, LPR, EPL, stream);
    }
    if (cols % E == 0 && cols / E <= 1024 * MAXR) {
        const int groups = (int)(cols / E);
        if (groups <= 4) return launch_rows<TI, TO, 1, 4>(S, P, rows, groups, stream);
        if (groups <= 8) return launch_rows<TI, TO, 1, 8>(S, P, rows, groups, stream);
        if (groups <= 16) return launch_rows<TI, TO, 1, 16>(S, P, rows, groups, stream);
        if (groups <= 32) return launch_rows<TI, TO, 1, 32>(S, P, rows, groups, stream);
        if (groups <= 64) return launch_rows<TI, TO, 1, 64>(S, P, rows, groups, stream);
        if (groups <= 128) return launch_rows<TI, TO, 2, 64>(S, P, rows, groups, stream);
        // (lanes times groups per lane just above the row where it was measured to pay -- a shape with half of its
        // slots empty has half of the bytes in flight per compute unit; bf16: 100000 x 1032 83 -> 69 us,
        // 24576 x 2056 39 -> 36.5, 6000 x 8200 41 -> 34, 6000 x 10240 44 -> 40; fp32: 50000 x 516 39 -> 37;
        // three groups on 128 or 256 lanes, six on 256 and five of 4 elements: no faster than the next shape up)
        if (groups <= 192) return launch_rows<TI, TO, 3, 64>(S, P, rows, groups, stream);
        // (two waves per row here: 2 % faster than one wave with four groups per lane on 24576 x 2048 bf16)
        if (groups <= 256) return launch_rows<TI, TO, 2, 128>(S, P, rows, groups, stream);
        if constexpr (E == 8) {
            if (groups <= 320) return launch_rows<TI, TO, 5, 64>(S, P, rows, groups, stream);
        }
        if (groups <= 512) return launch_rows<TI, TO, 2, 256>(S, P, rows, groups, stream);
        if (groups <= 1024) return launch_rows<TI, TO, 4, 256>(S, P, rows, groups, stream);
        if constexpr (E == 8) {
            if (groups <= 1280) return launch_rows<TI, TO, 5, 256>(S, P, rows, groups, stream);
        }
        if (groups <= 2048) return launch_rows<TI, TO, 2, 1024>(S, P, rows, groups, stream);
        if (groups <= 4096) return launch_rows<TI, TO, 4, 1024>(S, P, rows, groups, stream);
        if (groups <= 6144) return launch_rows<TI, TO, 6, 1024>(S, P, rows, groups, stream);
        if constexpr (MAXR >= 16) {
            // (eight groups of 4 elements on 1024 lanes: the compiler spills registers for that one shape)
            if (groups <= 12288) return launch_rows<TI, TO, 12, 1024>(S, P, rows, groups, stream);
            return launch_rows<TI, TO, 16, 1024>(S, P, rows, groups, stream);
        } else {
            return launch_rows<TI, TO, 8, 1024>(S, P, rows, groups, stream);
        }
    }
    // many short rows off the chunk boundaries, one type: whole chunks through LDS
    if constexpr (sizeof(TI) == sizeof(TO)) {
        int RW, CW, LPR, EPL;
        // (from 64 columns on only where the chunks of a wave's rows keep most of its lanes busy; measured against the
        // kernel below, bf16: 300000 x 124 37 -> 30 us, 100000 x 252 26.5 -> 21, 300000 x 90 33 -> 30; with half the
        // lanes loading it loses: 200000 x 132 31 -> 37)
        if (cols < 256 && rows >= 1024 && packed_shape<TI>(cols, &RW, &CW, &LPR, &EPL) && (cols < 64 || CW >= 45))
            return launch_packed<TI>(S, P, rows, (int)cols, RW, CW, LPR, EPL, stream);
    }
    // rows off the 16-byte boundaries, same type in and out: aligned chunks all the same, the two shared with the
    // neighbouring rows handled element by element (from 64 columns on: below, the two shared chunks are most of a row)
    if constexpr (sizeof(TI) == sizeof(TO)) {
        const int64_t chunks = cols / E + 2;
        if (cols >= 64 && chunks <= 8192 && (rows + 15) / 16 <= (int64_t)0x7fffffff) {
            // (a row of 2^k - 1 elements needs 2^k / V or one more chunk: intermediate shapes keep the lanes busy)
            if (chunks <= 16) return launch_rows_shifted<TI, 1, 16>(S, P, rows, cols, stream);
            if (chunks <= 32) return launch_rows_shifted<TI, 2, 16>(S, P, rows, cols, stream);
            if (chunks <= 48) return launch_rows_shifted<TI, 3, 16>(S, P, rows, cols, stream);
            if (chunks <= 64) return launch_rows_shifted<TI, 2, 32>(S, P, rows, cols, stream);
            if (chunks <= 96) return launch_rows_shifted<TI, 3, 32>(S, P, rows, cols, stream);
            if (chunks <= 128) return launch_rows_shifted<TI, 2, 64>(S, P, rows, cols, stream);
            if (chunks <= 192) return launch_rows_shifted<TI, 3, 64>(S, P, rows, cols, stream);
            if (chunks <= 256) return launch_rows_shifted<TI, 2, 128>(S, P, rows, cols, stream);
            if (chunks <= 320) return launch_rows_shifted<TI, 5, 64>(S, P, rows, cols, stream);
            if (chunks <= 384) return launch_rows_shifted<TI, 3, 128>(S, P, rows, cols, stream);
            if (chunks <= 512) return launch_rows_shifted<TI, 2, 256>(S, P, rows, cols, stream);
            if (chunks <= 768) return launch_rows_shifted<TI, 3, 256>(S, P, rows, cols, stream);
            if (chunks <= 1024) return launch_rows_shifted<TI, 4, 256>(S, P, rows, cols, stream);
            if (chunks <= 1536) return launch_rows_shifted<TI, 6, 256>(S, P, rows, cols, stream);
            if (chunks <= 2048) return launch_rows_shifted<TI, 2, 1024>(S, P, rows, cols, stream);
            if (chunks <= 3072) return launch_rows_shifted<TI, 3, 1024>(S, P, rows, cols, stream);
            if (chunks <= 4096) return launch_rows_shifted<TI, 4, 1024>(S, P, rows, cols, stream);
            if (chunks <= 6144) return launch_rows_shifted<TI, 6, 1024>(S, P, rows, cols, stream);
            return launch_rows_shifted<TI, 8, 1024>(S, P, rows, cols, stream);
        }
    }
    // short rows of any length and alignment: in registers, in groups of 4, 2 or 1 elements
    if (cols <= 1024) {
        if (cols % 4 == 0) return launch_elem_groups<TI, TO, 4>(S, P, rows, (int)cols, stream);
        if (cols % 2 == 0) return launch_elem_groups<TI, TO, 2>(S, P, rows, (int)cols, stream);
        return launch_elem_groups<TI, TO, 1>(S, P, rows, (int)cols, stream);
    }
    // everything else: two reads of the row.  Few rows are cut into pieces so that about two workgroups per
    // compute unit have work (never in place; a piece is at least 2048 groups long: two per thread, and room for
    // the table of the pieces' statistics at its start)
    int64_t chunks = 1;
    if (S != P && rows < compute_units()) {   // (with a row per compute unit the second launch costs more than it gains)
        const int64_t want = (2 * compute_units() + rows - 1) / rows;
        const int64_t fit = cols / ((int64_t)E * 2048);
        chunks = want < fit ? want : fit;
        if (chunks < 1) chunks = 1;
        if (chunks > 1024) chunks = 1024;
    }
    if (rows * chunks > (int64_t)0x7fffffff) return hipErrorInvalidValue;
    const TI* s_ = static_cast<const TI*>(S);
    TO* p_ = static_cast<TO*>(P);
    const dim3 grid((uint32_t)(rows * chunks));
    if (chunks > 1) {
        hipLaunchKernelGGL((softmax_long_kernel<TI, TO, 1024, 1>), grid, dim3(1024), 0, stream, s_, p_, rows, cols, (int)chunks);
        hipLaunchKernelGGL((softmax_long_kernel<TI, TO, 1024, 2>), grid, dim3(1024), 0, stream, s_, p_, rows, cols, (int)chunks);
    } else if (cols / E < 4096) {   // a few groups per thread at most: a small workgroup, more of them per compute unit
        hipLaunchKernelGGL((softmax_long_kernel<TI, TO, 256, 0>), grid, dim3(256), 0, stream, s_, p_, rows, cols, 1);
    } else {
        hipLaunchKernelGGL((softmax_long_kernel<TI, TO, 1024, 0>), grid, dim3(1024), 0, stream, s_, p_, rows, cols, 1);
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_softmax(DType in, DType out, const void* S, void* P, int64_t rows, int64_t cols, hipStream_t stream)
{
    if (in == DType::F32)
        return out == DType::F32 ? launch_softmax_t<float, float>(S, P, rows, cols, stream)
                                 : launch_softmax_t<float, uint16_t>(S, P, rows, cols, stream);
    return out == DType::F32 ? launch_softmax_t<uint16_t, float>(S, P, rows, cols, stream)
                             : launch_softmax_t<uint16_t, uint16_t>(S, P, rows, cols, stream);
}

}  // namespace attnw
