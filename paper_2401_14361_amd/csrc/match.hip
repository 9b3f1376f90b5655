// Step 3 of the layer step: the EAMC match (Sec. 4.5 of the paper).
//
// Every stored request-level EAM is compared with the current EAM by the cosine of
// the flattened matrices; the closest one wins.  On the device this is a streaming
// reduction over the whole collection: traces are stored layer-major
// [L][n_cap][E], a workgroup owns a tile of consecutive traces and walks the layers,
// so each step reads one contiguous run of cells with 16-byte loads.  The query's
// rows sit in LDS.  Dot products are exact 64-bit integers; the arg-max compares
// dot_a^2 * |T_b|^2 with dot_b^2 * |T_a|^2 in 192-bit integer arithmetic, so the
// winner does not depend on floating-point rounding.
#include <stdlib.h>
#include <string.h>

#include <new>
#include <type_traits>
#include <vector>

#include <stdio.h>

#include "kernels.hpp"
#include "score.hpp"
#include "wtypes.hpp"

namespace moei {

namespace {

constexpr int kDotThreads = 256;
constexpr int kMaxE = 2048;
typedef unsigned __int128 u128;

struct DotArgs {
    const void* traces;   // [L][n_cap][E]
    const int32_t* q;     // [B][L][E]
    u64* part;            // [B][n_lsplit][n_cap]
    int n_cap, N, L, E, B;
    int L_scan;           // layers 0..L_scan-1 are read
    int lper;             // layers per split
    int n_lsplit;
    int TN;               // traces per tile
    int rowV;             // vectors per trace row
    int once;             // the scan exceeds the last-level cache: load with the non-temporal hint
    int lane_rows;        // a trace row's vectors sit in rowV consecutive lanes (see the kernel)
};

template <typename CT, int VEC>
struct CellVec;

template <>
struct CellVec<int32_t, 4> {
    using raw = int4;
    static __device__ __forceinline__ raw load(const int32_t* p) { return *reinterpret_cast<const int4*>(p); }
    static __device__ __forceinline__ raw load_once(const int32_t* p) {
        const uint4 v = load_once_16(p);
        return make_int4((int)v.x, (int)v.y, (int)v.z, (int)v.w);
    }
    static __device__ __forceinline__ u64 dot(raw v, const int32_t* q, u64 acc) {
        int4 qq = *reinterpret_cast<const int4*>(q);
        acc += (u64)(uint32_t)v.x * (uint32_t)qq.x;
        acc += (u64)(uint32_t)v.y * (uint32_t)qq.y;
        acc += (u64)(uint32_t)v.z * (uint32_t)qq.z;
        acc += (u64)(uint32_t)v.w * (uint32_t)qq.w;
        return acc;
    }
};

template <>
struct CellVec<int32_t, 1> {
    using raw = int32_t;
    static __device__ __forceinline__ raw load(const int32_t* p) { return *p; }
    static __device__ __forceinline__ raw load_once(const int32_t* p) { return *p; }
    static __device__ __forceinline__ u64 dot(raw v, const int32_t* q, u64 acc) {
        return acc + (u64)(uint32_t)v * (uint32_t)q[0];
    }
};

template <>
struct CellVec<uint16_t, 8> {
    using raw = uint4;
    static __device__ __forceinline__ raw load(const uint16_t* p) { return *reinterpret_cast<const uint4*>(p); }
    static __device__ __forceinline__ raw load_once(const uint16_t* p) { return load_once_16(p); }
    static __device__ __forceinline__ u64 dot(raw v, const int32_t* q, u64 acc) {
        int4 q0 = *reinterpret_cast<const int4*>(q);
        int4 q1 = *reinterpret_cast<const int4*>(q + 4);
        acc += (u64)(v.x & 0xffffu) * (uint32_t)q0.x;
        acc += (u64)(v.x >> 16) * (uint32_t)q0.y;
        acc += (u64)(v.y & 0xffffu) * (uint32_t)q0.z;
        acc += (u64)(v.y >> 16) * (uint32_t)q0.w;
        acc += (u64)(v.z & 0xffffu) * (uint32_t)q1.x;
        acc += (u64)(v.z >> 16) * (uint32_t)q1.y;
        acc += (u64)(v.w & 0xffffu) * (uint32_t)q1.z;
        acc += (u64)(v.w >> 16) * (uint32_t)q1.w;
        return acc;
    }
};

template <>
struct CellVec<uint16_t, 1> {
    using raw = uint16_t;
    static __device__ __forceinline__ raw load(const uint16_t* p) { return *p; }
    static __device__ __forceinline__ raw load_once(const uint16_t* p) { return *p; }
    static __device__ __forceinline__ u64 dot(raw v, const int32_t* q, u64 acc) {
        return acc + (u64)v * (uint32_t)q[0];
    }
};

// The query rows of a workgroup's layers, for its NB queries, into LDS.  A query's cells of these
// layers are contiguous: each thread copies every 256th of them, query after query, with no index
// arithmetic beyond an addition (an index split by division costs more instructions here than the
// scan's own multiply-adds), the loads of all queries for several rounds in flight together.
template <int NB>
__device__ __forceinline__ void stage_queries(const int32_t* __restrict__ q, int B, int L, int E, int b0, int l0, int nl,
                                              int q_stride, int32_t* qs) {
    const int per = nl * E;  // cells per query
    constexpr int R = NB >= 16 ? 3 : (NB >= 8 ? 6 : (NB >= 4 ? 12 : 16));  // rounds whose loads go out together
    for (int c0 = (int)threadIdx.x; c0 < per; c0 += R * kDotThreads) {
        int32_t v[NB][R];
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const int32_t* src = q + ((size_t)min(b0 + b, B - 1) * L + l0) * E;  // past B: a copy, stored as zeros
#pragma unroll
            for (int r = 0; r < R; ++r) v[b][r] = c0 + r * kDotThreads < per ? src[c0 + r * kDotThreads] : 0;
        }
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int r = 0; r < R; ++r)
                if (c0 + r * kDotThreads < per) qs[b * q_stride + c0 + r * kDotThreads] = b0 + b < B ? v[b][r] : 0;
    }
}

// Sum of a 64-bit value over each group of `group` consecutive lanes (a power of two up to 64; all 64
// lanes take part; every lane of a group ends with the group's sum): two-word adds with carry over
// DPP exchanges inside a row of 16 lanes, shuffles beyond.
__device__ __forceinline__ u64 add_step_dpp(u64 v, unsigned lo_o, unsigned hi_o) {
    const unsigned lo = (unsigned)v + lo_o;
    const unsigned hi = (unsigned)(v >> 32) + hi_o + (lo < lo_o ? 1u : 0u);
    return ((u64)hi << 32) | lo;
}
#define MOEI_GROUP_STEP(v, ctrl) (v) = add_step_dpp((v), MOEI_DPP_U32((unsigned)(v), ctrl), MOEI_DPP_U32((unsigned)((v) >> 32), ctrl))
__device__ __forceinline__ u64 group_sum_u64(u64 v, int group) {
    if (group >= 2) MOEI_GROUP_STEP(v, 0xB1);    // quad_perm [1,0,3,2]
    if (group >= 4) MOEI_GROUP_STEP(v, 0x4E);    // quad_perm [2,3,0,1]
    if (group >= 8) MOEI_GROUP_STEP(v, 0x141);   // row_half_mirror
    if (group >= 16) MOEI_GROUP_STEP(v, 0x140);  // row_mirror
    if (group >= 32) v += ((u64)__shfl_xor((unsigned)(v >> 32), 16, 64) << 32 | __shfl_xor((unsigned)v, 16, 64));
    if (group >= 64) v += ((u64)__shfl_xor((unsigned)(v >> 32), 32, 64) << 32 | __shfl_xor((unsigned)v, 32, 64));
    return v;
}

// The same for NB = 8 or 16 values per lane and groups of 16 lanes, at a quarter of the additions: at
// each level of the exchange a lane keeps one half of its values and hands the other half to its
// partner, which keeps that half (the partner at a level differs in that level's bit of the lane
// number; the partners are those of the patterns above).  Lane i of a group ends with the group's sum
// of value number i % NB.
template <int NB>
__device__ __forceinline__ u64 row16_sum_scatter(u64 (&v)[NB], int lane) {
    static_assert(NB == 8 || NB == 16, "eight or sixteen values");
#define MOEI_DPP_U64(x, ctrl) (((u64)MOEI_DPP_U32((unsigned)((x) >> 32), ctrl) << 32) | MOEI_DPP_U32((unsigned)(x), ctrl))
#define MOEI_SCATTER_LEVEL(n, bit, ctrl)                              \
    {                                                                 \
        const bool up = (lane & (bit)) != 0;                          \
        _Pragma("unroll") for (int k = 0; k < (n); ++k) {             \
            const u64 keep = up ? v[k + (n)] : v[k];                  \
            const u64 send = up ? v[k] : v[k + (n)];                  \
            v[k] = keep + MOEI_DPP_U64(send, ctrl);                   \
        }                                                             \
    }
    if constexpr (NB == 16) {
        MOEI_SCATTER_LEVEL(8, 8, 0x140)  // row_mirror
    } else {
#pragma unroll
        for (int k = 0; k < 8; ++k) MOEI_GROUP_STEP(v[k], 0x140);
    }
    MOEI_SCATTER_LEVEL(4, 4, 0x141)  // row_half_mirror
    MOEI_SCATTER_LEVEL(2, 2, 0x4E)   // quad_perm [2,3,0,1]
    MOEI_SCATTER_LEVEL(1, 1, 0xB1)   // quad_perm [1,0,3,2]
#undef MOEI_SCATTER_LEVEL
#undef MOEI_DPP_U64
    return v[0];
}

// grid (tiles, layer splits, query groups).  Thread t owns vectors p = j*256 + t (j < J) of its
// tile; vector p belongs to trace p / rowV of the tile in EVERY layer, so the accumulators
// live in registers across the whole layer walk.  A workgroup serves NB queries at once:
// every loaded vector is multiplied with all of them, so a batch reads the traces once per
// group of NB queries.
template <typename CT, int VEC, int J, int NB>
__global__ void __launch_bounds__(kDotThreads) eamc_dot_kernel(DotArgs a) {
    using CV = CellVec<CT, VEC>;
    extern __shared__ __align__(16) unsigned char smem[];
    int32_t* qs = reinterpret_cast<int32_t*>(smem);  // [NB][lper*E]
    const int q_stride = a.lper * a.E;
    const int q_bytes = ((NB * q_stride * 4) + 15) & ~15;
    u64* rowsum = reinterpret_cast<u64*>(smem + q_bytes);  // [NB][TN]

    const int tid = threadIdx.x;
    const int split = blockIdx.y;
    const int b0 = blockIdx.z * NB;
    const int l0 = split * a.lper;
    int nl = min(l0 + a.lper, a.L_scan) - l0;
    if (nl < 0) nl = 0;
    const int n0 = blockIdx.x * a.TN;
    const int tn = min(a.TN, a.N - n0);

    stage_queries<NB>(a.q, a.B, a.L, a.E, b0, l0, nl, q_stride, qs);
    // a.lane_rows: the vectors of a trace row lie in a.rowV consecutive lanes (a power of two that divides
    // the wavefront): their sums are added across those lanes and stored by the first of them; otherwise
    // the row sums are gathered with LDS atomics, which many lanes on one address make slow
    if (!a.lane_rows)
        for (int i = tid; i < NB * a.TN; i += kDotThreads) rowsum[i] = 0;
    __syncthreads();

    bool valid[J];
    int row[J], col[J];
    u64 acc[J][NB];
    const int nvec = tn * a.rowV;
#pragma unroll
    for (int j = 0; j < J; ++j) {
        int p = j * kDotThreads + tid;
        valid[j] = p < nvec;
        row[j] = valid[j] ? p / a.rowV : 0;
        col[j] = valid[j] ? (p - row[j] * a.rowV) * VEC : 0;
#pragma unroll
        for (int b = 0; b < NB; ++b) acc[j][b] = 0;
    }
    const size_t lstride = (size_t)a.n_cap * a.E;
    const CT* base = reinterpret_cast<const CT*>(a.traces) + ((size_t)l0 * a.n_cap + n0) * a.E + (size_t)tid * VEC;
    // The loads of the next layers are kept in flight by hand: a ring of kAhead layers of this thread's
    // vectors, a slot refilled as soon as its layer has been taken out.  A vector past the tile's end
    // reads the thread's first vector instead (in bounds; its sums are dropped at the end), so the loop
    // has no divergent branch.
    constexpr int kAhead = J <= 2 ? 4 : 2;
    size_t voff[J];
#pragma unroll
    for (int j = 0; j < J; ++j) voff[j] = valid[j] ? (size_t)j * kDotThreads * VEC : 0;
    const bool any = valid[0];  // the thread has a vector in this tile at all
    typename CV::raw ring[kAhead][J];
    auto fetch = [&](typename CV::raw* dst, int l) {
        const CT* src = base + (size_t)l * lstride;
#pragma unroll
        for (int j = 0; j < J; ++j) dst[j] = a.once ? CV::load_once(src + voff[j]) : CV::load(src + voff[j]);
    };
    if (any) {
#pragma unroll
        for (int d = 0; d < kAhead; ++d)
            if (d < nl) fetch(ring[d], d);
        for (int l0r = 0; l0r < nl; l0r += kAhead) {
#pragma unroll
            for (int d = 0; d < kAhead; ++d) {
                const int l = l0r + d;
                if (l < nl) {  // uniform over the workgroup
                    typename CV::raw v[J];
#pragma unroll
                    for (int j = 0; j < J; ++j) v[j] = ring[d][j];
                    if (l + kAhead < nl) fetch(ring[d], l + kAhead);
                    const int32_t* ql = qs + (size_t)l * a.E;
#pragma unroll
                    for (int j = 0; j < J; ++j)
#pragma unroll
                        for (int b = 0; b < NB; ++b) acc[j][b] = CV::dot(v[j], ql + b * q_stride + col[j], acc[j][b]);
                }
            }
        }
    }
    if (a.lane_rows && a.rowV == 16 && NB >= 8) {
        // 16 lanes per trace row and 8 or 16 queries: every lane ends with one query's row sum and stores it
        constexpr int NBS = NB >= 8 ? NB : 8;
        const int lane = tid & (kWave - 1);
#pragma unroll
        for (int j = 0; j < J; ++j) {
            u64 v[NBS];
#pragma unroll
            for (int b = 0; b < NBS; ++b) v[b] = (b < NB && valid[j]) ? acc[j][b < NB ? b : 0] : 0;
            const u64 t = row16_sum_scatter<NBS>(v, lane);
            if (valid[j] && (NB == 16 || (lane & 8) == 0)) rowsum[(lane & (NB - 1)) * a.TN + row[j]] = t;
        }
    } else if (a.lane_rows) {
        const bool first = (tid & (a.rowV - 1)) == 0;
#pragma unroll
        for (int j = 0; j < J; ++j)
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const u64 t = group_sum_u64(valid[j] ? acc[j][b] : 0, a.rowV);  // rows are valid or not as a whole
                if (first && valid[j]) rowsum[b * a.TN + row[j]] = t;
            }
    } else {
#pragma unroll
        for (int j = 0; j < J; ++j)
#pragma unroll
            for (int b = 0; b < NB; ++b)
                if (valid[j] && acc[j][b] != 0) atomicAdd(&rowsum[b * a.TN + row[j]], acc[j][b]);
    }
    __syncthreads();
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        if (b0 + b >= a.B) break;
        u64* out = a.part + ((size_t)(b0 + b) * a.n_lsplit + split) * a.n_cap + n0;
        for (int i = tid; i < tn; i += kDotThreads) out[i] = rowsum[b * a.TN + i];
    }
}

// ---- the batched scan on the matrix cores.  For several queries the scan is a matrix product,
// [traces x cells] . [cells x queries], with integer entries and an exact integer result.  Cells
// are split into 7-bit digits (c = sum_i d_i 128^i, 0 <= d_i < 128) and the digit planes are
// multiplied pairwise by the 8-bit integer matrix instruction (16 traces x 64 cells times 64 cells
// x 16 queries, 32-bit sums): products of equal weight 128^(i + j) share an accumulator, and the
// accumulators are combined in 64-bit arithmetic at the end of a tile, long before any of them can
// overflow, so the dot products are the same integers the kernel above forms.  The instruction
// does the sum over the cells: no sums across lanes are left, and the vector ALUs only cut digits,
// so the kernel runs close to the speed of the scan itself.  How many digit planes are needed is
// known on the host for the traces (the largest cell ever stored: DA) and found while staging for
// the queries (DB, per workgroup).
//
// grid (tiles of 64 traces, layer splits, groups of 16 queries), 4 wavefronts of 16 traces each.  A
// unit is 64 cells of one layer of 16 traces (4 KiB, rows of 256 bytes; half that with 2-byte cells).  The matrix instruction
// wants lane (r = lane % 16, g = lane / 16) to hold 16 cells of trace r, so a load into registers
// would bring 64 bytes of each of 16 rows per instruction, and the compiler moves such loads down
// to their use (a wavefront then has one unit in flight whatever ring the source spells out).  So
// the units go from global memory straight into a ring in LDS, whole rows at a time, as
// instructions the compiler leaves where they are, with wait counts written by hand; lane (r, g)
// then reads piece p = cells 16 p + 4 g .. + 3 of row r from LDS, and byte j of digit word p is the
// digit of cell 16 p + 4 g + j.  The query planes lie in LDS in the same order,
// [digit][query][unit][g][p][j], a lane reads its 16 bytes at once; the stride between queries is
// an odd number of 16-byte steps, so the sixteen lanes that read one g together touch every bank
// once.  Cells past E in a row's last unit are zero in the query planes.
typedef int i32x4 __attribute__((ext_vector_type(4)));
constexpr int kMmQueries = 16;
constexpr int kDigitBits = 7;
constexpr int kMaxDigits = 4;  // 28 bits: cells up to MOEI_MAX_COUNT (24 bits)
static_assert(MOEI_MAX_COUNT < (1 << (kDigitBits * kMaxDigits)), "four digits hold every cell");
// Units (of 64 cells) per tile and layer split: what 30 KiB of LDS hold of query planes (two
// workgroups of 48 KiB of rings each then share a compute unit).  An
// accumulator takes at most kMaxDigits digit pairs of 127 x 127 per cell, so it cannot overflow.
constexpr int kMmMaxUnits = 7;
constexpr int kMmRing = 3;           // units of a wavefront's ring: two in flight while one is multiplied
// f(0), f(1), ... while the index is below n (and below MAX), each call nested in the check before it
template <int U, int MAX, typename F>
__device__ __forceinline__ void nest_up(int n, F&& f) {
    if constexpr (U < MAX) {
        if (U < n) {
            f(std::integral_constant<int, U>{});
            nest_up<U + 1, MAX>(n, f);
        }
    }
}
static_assert((long)kMmMaxUnits * 64 * kMaxDigits * 127 * 127 < 0x7fffffffL, "32-bit sums hold a tile");

struct DotMmArgs {
    const void* traces;  // [L][n_cap][E] cells of 4 or 2 bytes
    const int32_t* q;    // [B][L][E]
    u64* part;           // [B][n_lsplit][n_cap]
    int n_cap, N, L, E, B;
    int L_scan, lper, n_lsplit;
    int nblk;      // units per trace row: ceil(E / 64)
    int n_tiles;   // tiles of 64 J traces
    int q_stride;  // bytes per query in a digit plane: lper * nblk * 64, rounded up to an odd number of 16-byte steps
};

// The first ND 7-bit digits of four cells, digit i of the four cells in the four bytes of d[i].  Byte
// permutes first gather byte j of the four cells into one word (two words for the two low bytes of
// each pair, two more to interleave the pairs), then each digit is cut from at most two byte planes
// with masks that keep every byte to itself: about half the instructions of shifting and masking
// the cells one by one.
template <int ND>
__device__ __forceinline__ void cut_digits(int4 x, int (&d)[ND]);
template <int ND>
__device__ __forceinline__ void cut_digits(i32x4 v, int (&d)[ND]) {
    cut_digits<ND>(make_int4(v[0], v[1], v[2], v[3]), d);
}
template <int ND>
__device__ __forceinline__ void cut_digits(int4 x, int (&d)[ND]) {
    static_assert(ND >= 1 && ND <= kMaxDigits, "one to four digits");
    // v_perm_b32: selector bytes 0..3 take bytes of the second operand, 4..7 of the first
    const unsigned p01 = __builtin_amdgcn_perm((unsigned)x.y, (unsigned)x.x, 0x05010400u);  // x.b0 y.b0 x.b1 y.b1
    const unsigned p23 = __builtin_amdgcn_perm((unsigned)x.w, (unsigned)x.z, 0x05010400u);  // z.b0 w.b0 z.b1 w.b1
    const unsigned b0 = __builtin_amdgcn_perm(p23, p01, 0x05040100u);                        // byte 0 of x y z w
    d[0] = (int)(b0 & 0x7f7f7f7fu);
    if constexpr (ND >= 2) {
        const unsigned b1 = __builtin_amdgcn_perm(p23, p01, 0x07060302u);  // byte 1 of x y z w
        d[1] = (int)(((b1 & 0x3f3f3f3fu) << 1) | ((b0 >> 7) & 0x01010101u));
        if constexpr (ND >= 3) {
            const unsigned q01 = __builtin_amdgcn_perm((unsigned)x.y, (unsigned)x.x, 0x07030602u);  // x.b2 y.b2 x.b3 y.b3
            const unsigned q23 = __builtin_amdgcn_perm((unsigned)x.w, (unsigned)x.z, 0x07030602u);
            const unsigned b2 = __builtin_amdgcn_perm(q23, q01, 0x05040100u);                        // byte 2 of x y z w
            d[2] = (int)(((b2 & 0x1f1f1f1fu) << 2) | ((b1 >> 6) & 0x03030303u));
            if constexpr (ND >= 4) {
                const unsigned b3 = __builtin_amdgcn_perm(q23, q01, 0x07060302u);  // byte 3 of x y z w
                d[3] = (int)(((b3 & 0x0f0f0f0fu) << 3) | ((b2 >> 5) & 0x07070707u));
            }
        }
    }
}
// The same for four 2-byte cells in two words (cells 0, 1 in w0, cells 2, 3 in w1): up to three digits.
template <int ND>
__device__ __forceinline__ void cut_digits16(unsigned w0, unsigned w1, int (&d)[ND]) {
    static_assert(ND >= 1 && ND <= 3, "16 bits are three digits at most");
    const unsigned b0 = __builtin_amdgcn_perm(w1, w0, 0x06040200u);  // the low bytes of the four cells
    d[0] = (int)(b0 & 0x7f7f7f7fu);
    if constexpr (ND >= 2) {
        const unsigned b1 = __builtin_amdgcn_perm(w1, w0, 0x07050301u);  // their high bytes
        d[1] = (int)(((b1 & 0x3f3f3f3fu) << 1) | ((b0 >> 7) & 0x01010101u));
        if constexpr (ND >= 3) d[2] = (int)((b1 >> 6) & 0x03030303u);
    }
}
__device__ __forceinline__ int digits_of(unsigned v) { return v >> 21 ? 4 : (v >> 14 ? 3 : (v >> 7 ? 2 : 1)); }
inline int digits_of_host(unsigned v) { return v >> 21 ? 4 : (v >> 14 ? 3 : (v >> 7 ? 2 : 1)); }

template <int DA, int CB>  // digit planes of the traces; bytes per stored cell (4 or 2)
__global__ void __launch_bounds__(kDotThreads) eamc_dot_mm_kernel(DotMmArgs a) {
    constexpr int UB = 64 * 16 * CB;      // bytes of a unit: 16 rows of 64 cells
    constexpr int RB = 64 * CB;           // bytes of a unit's row in LDS
    constexpr int NLD = UB / 1024;        // load instructions per unit
    constexpr int CPC = 16 / CB;          // cells per 16-byte chunk
    extern __shared__ __align__(16) unsigned char smem[];  // the wavefronts' rings, then [kMaxDigits][16][q_stride] query planes
    __shared__ unsigned s_or[kDotThreads / kWave];
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wv = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int lrow = lane & 15, lgrp = lane >> 4;
    const int split = blockIdx.y, b0 = blockIdx.z * kMmQueries;
    const int l0 = split * a.lper;
    const int nl = max(0, min(l0 + a.lper, a.L_scan) - l0);
    const int E = a.E, nblk = a.nblk, S = a.q_stride;
    const size_t plane = (size_t)kMmQueries * S;
    const int n_units = nl * nblk;  // units of the tile: at most kMmMaxUnits
    const int tile = blockIdx.x;
    unsigned char* planes = smem + (size_t)(kDotThreads / kWave) * kMmRing * UB;

    // 1. the query rows become digit planes in LDS (sixteen threads per query; thread i of them takes
    // the 16-byte pieces i, i + 16, ... of every layer's row - piece c4 = cells 4 c4 .. + 3: unit
    // c4 / 16, g = c4 % 4, p = c4 % 16 / 4 - eight layers' loads in flight together; a query past B
    // repeats the last one: its column is never stored)
    {
        constexpr int R = 8;
        const int qb = tid >> 4, qi = tid & 15;
        const int32_t* qsrc = a.q + ((size_t)min(b0 + qb, a.B - 1) * a.L + l0) * E;
        unsigned char* dst = planes + (size_t)qb * S;
        unsigned seen = 0;
        for (int c4 = qi; c4 < nblk * 16; c4 += 16) {
            const int word = ((c4 >> 4) << 6) + ((((c4 & 3) << 2) + ((c4 & 15) >> 2)) << 2);  // byte offset in the row's units
            for (int lr = 0; lr < nl; lr += R) {
                int4 x[R];
#pragma unroll
                for (int r = 0; r < R; ++r)
                    x[r] = (4 * c4 < E && lr + r < nl) ? *reinterpret_cast<const int4*>(qsrc + (size_t)(lr + r) * E + 4 * c4)
                                                       : make_int4(0, 0, 0, 0);
#pragma unroll
                for (int r = 0; r < R; ++r)
                    if (lr + r < nl) {
                        seen |= (unsigned)(x[r].x | x[r].y | x[r].z | x[r].w);
                        int dg[kMaxDigits];
                        cut_digits<kMaxDigits>(x[r], dg);
#pragma unroll
                        for (int d = 0; d < kMaxDigits; ++d)
                            *reinterpret_cast<int*>(dst + d * plane + (size_t)(lr + r) * nblk * 64 + word) = dg[d];
                    }
            }
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) seen |= (unsigned)__shfl_xor((int)seen, off, 64);
        if (lane == 0) s_or[wv] = seen;
    }

    // 2. the trace stream of this wavefront: 16 traces, unit after unit, through a ring of kMmRing
    // units in its own part of LDS.  A load instruction fills 1 KiB: rows 4 p .. 4 p + 3 of the unit
    // (4-byte cells: rows of 256 bytes, 16 chunks of 16 bytes) or rows 8 p .. 8 p + 7 (2-byte cells:
    // rows of 128 bytes, 8 chunks); the lane that fills chunk position q of row r brings the row's
    // chunk q ^ (r % 16) resp. q ^ (r / 2 % 8), so that the reads below touch every bank once.  An
    // address is a uniform part (layer, tile, unit) plus this lane's row and chunk as a 32-bit byte
    // offset.  Rows past N repeat the last trace (never stored); in a row's ragged last unit a
    // chunk past the row's end is read from the row's last chunk instead (it multiplies zeros).
    const char* tbytes = reinterpret_cast<const char*>(a.traces);
    const bool ragged = (E & 63) != 0;
    unsigned piece_full[NLD], piece_last[NLD];
#pragma unroll
    for (int p = 0; p < NLD; ++p) {
        const int row = CB == 4 ? 4 * p + (lane >> 4) : 8 * p + (lane >> 3);
        const unsigned r = (unsigned)(min(64 * tile + 16 * wv + row, a.N - 1) - 64 * tile);
        const int c = CB == 4 ? (lane & 15) ^ row : (lane & 7) ^ ((row >> 1) & 7);  // the chunk: cells CPC c .. of the unit
        piece_full[p] = (r * (unsigned)E + (unsigned)(CPC * c)) * CB;
        piece_last[p] = (r * (unsigned)E + (unsigned)min(64 * (nblk - 1) + CPC * c, E - CPC)) * CB;
    }
    const uint32_t my_ring = lds_address(smem) + (uint32_t)wv * (kMmRing * UB);
    int f_l = 0, f_blk = 0;  // the next unit to request
    auto fetch = [&](int slot) {
        const bool last = ragged && f_blk == nblk - 1;  // uniform
        const char* ubase = tbytes + (((size_t)(l0 + f_l) * a.n_cap + (size_t)64 * tile) * E) * CB +
                            (last ? (size_t)0 : (size_t)f_blk * RB);
#pragma unroll
        for (int p = 0; p < NLD; ++p)
            load16_to_lds(ubase + (last ? piece_last[p] : piece_full[p]), my_ring + (uint32_t)slot * UB + 1024u * p);
        if (++f_blk == nblk) {
            f_blk = 0;
            ++f_l;
        }
    };
#pragma unroll
    for (int d = 0; d < kMmRing; ++d)
        if (d < n_units) fetch(d);
    __syncthreads();  // the query planes are whole
    static_assert(kDotThreads / kWave == 4, "four wavefronts");
    const int DB = digits_of(s_or[0] | s_or[1] | s_or[2] | s_or[3]);  // uniform over the workgroup

    // 3. the products.  The walk over the tile's units is written out unit by unit, each nested in
    // the check that it exists, so ring slots and wait counts are compile-time constants.  A unit's
    // loads have landed once at most those of the units requested after it are outstanding; its
    // slot is requested again once its pieces have been read out of LDS.  The accumulators cannot
    // overflow inside a tile and are touched by the matrix instructions alone until its end.
    auto run = [&](auto db_tag) {
        constexpr int DBC = decltype(db_tag)::value;
        constexpr int NW = DA + DBC - 1;  // weights 128^0 .. 128^(NW - 1)
        const unsigned char* qrow = planes + (size_t)lrow * S + lgrp * 16;
        const unsigned char* ring = smem + (size_t)wv * (kMmRing * UB);
        i32x4 acc[NW];
#pragma unroll
        for (int w = 0; w < NW; ++w) acc[w] = i32x4{0, 0, 0, 0};
        nest_up<0, kMmMaxUnits>(n_units, [&](auto u_tag) {
            constexpr int U = decltype(u_tag)::value;
            constexpr int D = U % kMmRing;
            // units requested after this one: min(kMmRing - 1, n_units - 1 - U)
            if (U + 2 < n_units)
                wait_vm_fence<2 * NLD>();
            else if (U + 1 < n_units)
                wait_vm_fence<NLD>();
            else
                wait_vm_fence<0>();
            static_assert(kMmRing == 3, "the wait counts above are those of a ring of three");
            // lane (lrow, lgrp) takes piece p = cells 16 p + 4 lgrp .. + 3 of row lrow
            int dg[4][DA];
            const unsigned char* urow = ring + D * UB + lrow * RB;
            if constexpr (CB == 4) {
                i32x4 x[4];
#pragma unroll
                for (int p = 0; p < 4; ++p) x[p] = *reinterpret_cast<const i32x4*>(urow + (((4 * p + lgrp) ^ lrow) << 4));
#pragma unroll
                for (int p = 0; p < 4; ++p) cut_digits<DA>(x[p], dg[p]);
            } else {
                uint2 x[4];  // chunk 2 p + lgrp / 2, its half lgrp % 2
#pragma unroll
                for (int p = 0; p < 4; ++p)
                    x[p] = *reinterpret_cast<const uint2*>(urow + (((2 * p + (lgrp >> 1)) ^ ((lrow >> 1) & 7)) << 4) + 8 * (lgrp & 1));
#pragma unroll
                for (int p = 0; p < 4; ++p) cut_digits16<DA>(x[p].x, x[p].y, dg[p]);
            }
            i32x4 bq[DBC];
#pragma unroll
            for (int db = 0; db < DBC; ++db) bq[db] = *reinterpret_cast<const i32x4*>(qrow + db * plane + (size_t)U * 64);
            if (U + kMmRing < n_units) {
                wait_lds_fence();  // the slot has been read
                fetch(D);
            }
#pragma unroll
            for (int da = 0; da < DA; ++da) {
                const i32x4 ad = {dg[0][da], dg[1][da], dg[2][da], dg[3][da]};
#pragma unroll
                for (int db = 0; db < DBC; ++db)
                    acc[da + db] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ad, bq[db], acc[da + db], 0, 0, 0);
            }
        });
        // D[trace 4 lgrp + v][query lrow]
        if (b0 + lrow < a.B) {
            u64* out = a.part + ((size_t)(b0 + lrow) * a.n_lsplit + split) * a.n_cap;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                u64 t = 0;
#pragma unroll
                for (int w = 0; w < NW; ++w) t += (u64)(unsigned)acc[w][v] << (kDigitBits * w);
                const int n = 64 * tile + 16 * wv + 4 * lgrp + v;
                if (n < a.N) out[n] = t;
            }
        }
    };
    switch (DB) {
        case 1: run(std::integral_constant<int, 1>{}); break;
        case 2: run(std::integral_constant<int, 2>{}); break;
        case 3: run(std::integral_constant<int, 3>{}); break;
        default: run(std::integral_constant<int, 4>{}); break;
    }
}

struct Best {
    u64 dot;     // <q, T>
    u64 nt;      // |T|^2, never 0 here (an all-zero trace enters as dot 0, nt 1)
    double key;  // dot^2 / nt in fp64: decides all but near ties
    int idx;     // -1: none
};

__device__ __forceinline__ Best make_best(u64 dot, u64 nt, int idx) {
    Best b;
    b.dot = nt ? dot : 0;
    b.nt = nt ? nt : 1;
    b.key = ((double)b.dot * (double)b.dot) / (double)b.nt;
    b.idx = idx;
    return b;
}

// a.dot^2 * b.nt  vs  b.dot^2 * a.nt, exactly, as 192-bit integers.
__device__ __noinline__ int cmp_sim_exact(u64 adot, u64 ant, u64 bdot, u64 bnt) {
    u128 a2 = (u128)adot * adot, b2 = (u128)bdot * bdot;
    u128 al = (u128)(u64)a2 * bnt, ah = (u128)(u64)(a2 >> 64) * bnt + (al >> 64);
    u128 bl = (u128)(u64)b2 * ant, bh = (u128)(u64)(b2 >> 64) * ant + (bl >> 64);
    if (ah != bh) return ah > bh ? 1 : -1;
    u64 all = (u64)al, bll = (u64)bl;
    if (all != bll) return all > bll ? 1 : -1;
    return 0;
}

// The fp64 keys carry a relative error below 2^-50; a gap wider than 2^-48 settles the
// order, anything closer is decided by the exact integer comparison.
__device__ __forceinline__ int cmp_sim(Best a, Best b) {
    const double d = a.key - b.key;
    const double tol = fmax(a.key, b.key) * 0x1p-48;
    if (d > tol) return 1;
    if (d < -tol) return -1;
    return cmp_sim_exact(a.dot, a.nt, b.dot, b.nt);
}

// The better of two candidates, field by field (the structs stay in registers).
__device__ __forceinline__ Best pick(Best a, Best b) {
    bool take_b;
    if (b.idx < 0) {
        take_b = false;
    } else if (a.idx < 0) {
        take_b = true;
    } else {
        const int c = cmp_sim(a, b);
        take_b = c < 0 || (c == 0 && b.idx < a.idx);  // equal similarity: lowest trace index
    }
    Best r;
    r.dot = take_b ? b.dot : a.dot;
    r.nt = take_b ? b.nt : a.nt;
    r.key = take_b ? b.key : a.key;
    r.idx = take_b ? b.idx : a.idx;
    return r;
}

// A candidate moved across lanes by a DPP pattern / read from one lane through scalar registers.
template <int CTRL>
__device__ __forceinline__ Best best_dpp(Best me) {
    auto mv = [](unsigned v) { return MOEI_DPP_U32(v, CTRL); };
    auto mv64 = [&](u64 v) { return ((u64)mv((unsigned)(v >> 32)) << 32) | mv((unsigned)v); };
    Best o;
    o.dot = mv64(me.dot);
    o.nt = mv64(me.nt);
    o.key = __longlong_as_double((long long)mv64((u64)__double_as_longlong(me.key)));
    o.idx = (int)mv((unsigned)me.idx);
    return o;
}
__device__ __forceinline__ Best best_lane(Best me, int lane) {
    auto rd = [&](unsigned v) { return (unsigned)__builtin_amdgcn_readlane((int)v, lane); };
    auto rd64 = [&](u64 v) { return ((u64)rd((unsigned)(v >> 32)) << 32) | rd((unsigned)v); };
    Best o;
    o.dot = rd64(me.dot);
    o.nt = rd64(me.nt);
    o.key = __longlong_as_double((long long)rd64((u64)__double_as_longlong(me.key)));
    o.idx = (int)rd((unsigned)me.idx);
    return o;
}

// The same search on (key, index) alone: three registers per exchange instead of seven.  It is
// final only if no comparison on the way was a near tie (keys within 2^-48 of each other and
// not both zero); `tie` reports that, and the caller then repeats the search with the exact
// comparison.  Two zero keys are two zero similarities: the lower index wins, exactly.
struct KeyIdx {
    double key;
    int idx;
};
__device__ __forceinline__ KeyIdx pick_key(KeyIdx a, KeyIdx b, bool& tie) {
    if (b.idx < 0) return a;
    if (a.idx < 0) return b;
    const double d = a.key - b.key;
    const double tol = fmax(a.key, b.key) * 0x1p-48;
    bool take_b;
    if (d > tol) {
        take_b = false;
    } else if (d < -tol) {
        take_b = true;
    } else if (a.key == 0.0 && b.key == 0.0) {
        take_b = b.idx < a.idx;
    } else {
        tie = true;
        take_b = false;
    }
    KeyIdx r;
    r.key = take_b ? b.key : a.key;
    r.idx = take_b ? b.idx : a.idx;
    return r;
}
template <int CTRL>
__device__ __forceinline__ KeyIdx keyidx_dpp(KeyIdx me) {
    const u64 k = (u64)__double_as_longlong(me.key);
    KeyIdx o;
    o.key = __longlong_as_double((long long)(((u64)MOEI_DPP_U32((unsigned)(k >> 32), CTRL) << 32) | MOEI_DPP_U32((unsigned)k, CTRL)));
    o.idx = (int)MOEI_DPP_U32((unsigned)me.idx, CTRL);
    return o;
}
__device__ __forceinline__ KeyIdx keyidx_lane(KeyIdx me, int lane) {
    const u64 k = (u64)__double_as_longlong(me.key);
    KeyIdx o;
    o.key = __longlong_as_double((long long)(((u64)(unsigned)__builtin_amdgcn_readlane((int)(k >> 32), lane) << 32) |
                                             (unsigned)__builtin_amdgcn_readlane((int)k, lane)));
    o.idx = __builtin_amdgcn_readlane(me.idx, lane);
    return o;
}

__device__ __forceinline__ Best wave_pick_exact(Best me) {
    me = pick(me, best_dpp<0xB1>(me));   // quad_perm [1,0,3,2]
    me = pick(me, best_dpp<0x4E>(me));   // quad_perm [2,3,0,1]
    me = pick(me, best_dpp<0x141>(me));  // row_half_mirror
    me = pick(me, best_dpp<0x140>(me));  // row_mirror
    const Best r0 = best_lane(me, 0), r1 = best_lane(me, 16), r2 = best_lane(me, 32), r3 = best_lane(me, 48);
    return pick(pick(r0, r1), pick(r2, r3));
}

// The wavefront's best candidate, in every lane: DPP inside each row of 16 lanes (the order is
// total, so both partners of an exchange keep the same winner), then the four row winners
// through scalar registers.  All 64 lanes must be active.
__device__ __forceinline__ Best wave_pick(Best me) {
    bool tie = false;
    KeyIdx k{me.key, me.idx};
    k = pick_key(k, keyidx_dpp<0xB1>(k), tie);
    k = pick_key(k, keyidx_dpp<0x4E>(k), tie);
    k = pick_key(k, keyidx_dpp<0x141>(k), tie);
    k = pick_key(k, keyidx_dpp<0x140>(k), tie);
    const KeyIdx r0 = keyidx_lane(k, 0), r1 = keyidx_lane(k, 16), r2 = keyidx_lane(k, 32), r3 = keyidx_lane(k, 48);
    const KeyIdx w = pick_key(pick_key(r0, r1, tie), pick_key(r2, r3, tie), tie);
    if (__ballot(tie) != 0ull) return wave_pick_exact(me);  // uniform
    if (w.idx < 0) return make_best(0, 1, -1);
    // the winner's dot product and norm come from the lane that holds it
    const int owner = __builtin_amdgcn_readfirstlane(__ffsll((long long)__ballot(me.idx == w.idx)) - 1);
    return best_lane(me, owner);
}

__device__ __forceinline__ double cosine(u64 dot, u64 nq, u64 nt) {
    if (nq == 0 || nt == 0) return 0.0;
    return (double)dot / (sqrt((double)nq) * sqrt((double)nt));
}

constexpr int kPickThreads = 1024;
static_assert(kPickThreads == kScoreThreads, "the finishing workgroup of the match also runs the scoring");
constexpr int kPickChunk = kPickThreads;  // traces per workgroup: one per thread
constexpr int kPickWaves = kPickThreads / kWave;

struct PickArgs {
    const u64* part;    // [B][n_lsplit][n_cap]
    const u64* norm2;   // [n_cap]
    const int32_t* q;   // [B][L*E]
    int n_lsplit, n_cap, N, LE;
    u64* cand;          // [B][gridDim.x][2] winners of the workgroups (dot, nt) ...
    int32_t* cand_idx;  // [B][gridDim.x] ... and their trace indices
    unsigned* ticket;   // [B] arrival counters, zero between launches
    int32_t* best;
    float* best_sim;
    float* sims;
    int do_score;   // the finishing workgroup also scores the matched trace (B = 1)
    ScoreArgs sc;
};

// Workgroup winner among its wavefronts' winners; valid in every thread of wavefront 0.
__device__ __forceinline__ Best block_pick(Best me, u64* s_dot, u64* s_nt, int* s_idx) {
    const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x / kWave;
    me = wave_pick(me);
    __syncthreads();
    if (lane == 0) {
        s_dot[wv] = me.dot;
        s_nt[wv] = me.nt;
        s_idx[wv] = me.idx;
    }
    __syncthreads();
    Best r = make_best(0, 1, -1);
    if (wv == 0) {
        if (lane < kPickWaves && s_idx[lane] >= 0) r = make_best(s_dot[lane], s_nt[lane], s_idx[lane]);
        r = wave_pick(r);
    }
    return r;
}

// grid (workgroups over traces, B): sums the layer-split partial dots, writes similarities,
// picks the workgroup's best trace; the last workgroup to arrive picks among the winners.
__global__ void __launch_bounds__(kPickThreads) eamc_pick_kernel(PickArgs a) {
    __shared__ u64 s_dot[kPickWaves];
    __shared__ u64 s_nt[kPickWaves];
    __shared__ int s_idx[kPickWaves];
    __shared__ u64 s_nq;
    __shared__ unsigned s_ticket;
    const int b = blockIdx.y;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wv = tid / kWave;

    // One trace per thread (kPickChunk == kPickThreads).  Its partial dot products and norm are
    // requested first, so that they travel together with the query cells of the norm below: one trip
    // to memory instead of two.
    const int n = blockIdx.x * kPickChunk + tid;
    const bool have = n < a.N;
    u64 dot = 0, nt = 1;
    if (have) {
        const u64* pp = a.part + (size_t)b * a.n_lsplit * a.n_cap + n;
        nt = a.norm2[n];
        int s = 0;
        for (; s + 4 <= a.n_lsplit; s += 4) {  // the split partials are independent loads: four at a time
            const u64 v0 = pp[(size_t)s * a.n_cap], v1 = pp[(size_t)(s + 1) * a.n_cap];
            const u64 v2 = pp[(size_t)(s + 2) * a.n_cap], v3 = pp[(size_t)(s + 3) * a.n_cap];
            dot += (v0 + v1) + (v2 + v3);
        }
        for (; s < a.n_lsplit; ++s) dot += pp[(size_t)s * a.n_cap];
    }
    u64 nq = 0;
    for (int i = tid; i < a.LE; i += kPickThreads) {
        u64 v = (uint32_t)a.q[(size_t)b * a.LE + i];
        nq += v * v;
    }
    nq = wave_sum_u64_dpp(nq);
    if (lane == 0) s_dot[wv] = nq;
    __syncthreads();
    if (tid == 0) {
        u64 t = 0;
        for (int i = 0; i < kPickWaves; ++i) t += s_dot[i];
        s_nq = t;
    }
    __syncthreads();
    nq = s_nq;

    Best me = make_best(0, 1, -1);
    if (have) {
        if (a.sims) a.sims[(size_t)b * a.N + n] = (float)cosine(dot, nq, nt);
        me = make_best(dot, nt, n);
    }
    Best r = block_pick(me, s_dot, s_nt, s_idx);
    __shared__ int s_sn[2];
    __shared__ int s_best[kMaxMatchBatch];
    __shared__ HeadLds s_heads;
    __shared__ KeyLds s_keys;
    if (gridDim.x == 1) {
        if (tid == 0) {
            a.best[b] = r.idx;
            // (the winner carries its norm: no second trip to memory for it; an all-zero trace has dot 0)
            if (a.best_sim) a.best_sim[b] = r.idx >= 0 ? (float)cosine(r.dot, nq, r.nt) : 0.f;
            s_best[0] = r.idx;
        }
        if (a.do_score) score_and_heads(a.sc, s_heads, s_keys, s_sn, s_best, true);
        return;
    }
    // several workgroups: publish this one's winner, the last to arrive finishes
    const size_t cbase = (size_t)b * gridDim.x;
    if (tid == 0) {
        a.cand[(cbase + blockIdx.x) * 2] = r.dot;
        a.cand[(cbase + blockIdx.x) * 2 + 1] = r.nt;
        a.cand_idx[cbase + blockIdx.x] = r.idx;
        __threadfence();
        s_ticket = __hip_atomic_fetch_add(&a.ticket[b], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    if (s_ticket != gridDim.x - 1) return;
    if (tid == 0) __threadfence();  // one acquire for the workgroup (the winners are read past the caches anyway)
    __syncthreads();
    Best fin = make_best(0, 1, -1);
    for (int i = tid; i < (int)gridDim.x; i += kPickThreads) {
        const int idx = __hip_atomic_load(&a.cand_idx[cbase + i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (idx >= 0) {
            const u64 d = __hip_atomic_load(&a.cand[(cbase + i) * 2], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const u64 t = __hip_atomic_load(&a.cand[(cbase + i) * 2 + 1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            fin = pick(fin, make_best(d, t, idx));
        }
    }
    fin = block_pick(fin, s_dot, s_nt, s_idx);
    if (tid == 0) {
        a.best[b] = fin.idx;
        if (a.best_sim) a.best_sim[b] = fin.idx >= 0 ? (float)cosine(fin.dot, nq, fin.nt) : 0.f;
        a.ticket[b] = 0;  // ready for the next launch on this stream
        s_best[0] = fin.idx;
    }
    if (a.do_score) score_and_heads(a.sc, s_heads, s_keys, s_sn, s_best, true);
}

// ---- the m most similar traces of ONE query, most similar first (ties: lowest index)
constexpr int kTopmPerThread = 4;  // candidates a thread of the finishing workgroup may hold

struct TopmArgs {
    const u64* part;   // [n_lsplit][n_cap]
    const u64* norm2;  // [n_cap]
    const int32_t* q;  // [L*E]
    int n_lsplit, n_cap, N, LE, m;
    u64* cand;          // [gridDim.x * m][2]
    int32_t* cand_idx;  // [gridDim.x * m]
    unsigned* ticket;   // one arrival counter, zero between launches
    int32_t* top;       // [m], -1 beyond the stored traces
    float* top_sim;     // [m] or null
    float* sims;        // [N] or null
    int do_score;       // the finishing workgroup also scores the aggregate of the m traces
    ScoreArgs sc;
};

// m rounds of "best of the workgroup, then retire it".  Every wavefront keeps its own winner in
// LDS; after a round only the wavefront that held the overall winner searches again, the others'
// winners stand.  `local_best()` is the calling thread's best remaining candidate, `retire(idx)`
// removes a candidate from the calling thread, `emit(r, w)` is called by thread 0 with winner r.
template <typename LocalBest, typename Retire, typename Emit>
__device__ __forceinline__ void extract_top(int m, u64* s_dot, u64* s_nt, int* s_idx, int* s_win, LocalBest local_best,
                                            Retire retire, Emit emit) {
    const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x / kWave;
    bool stale = true;  // uniform over the wavefront: its LDS entry must be recomputed
    for (int r = 0; r < m; ++r) {
        if (stale) {
            const Best wb = wave_pick(local_best());
            if (lane == 0) {
                s_dot[wv] = wb.dot;
                s_nt[wv] = wb.nt;
                s_idx[wv] = wb.idx;
            }
            stale = false;
        }
        __syncthreads();
        if (wv == 0) {
            Best w = make_best(0, 1, -1);
            if (lane < kPickWaves && s_idx[lane] >= 0) w = make_best(s_dot[lane], s_nt[lane], s_idx[lane]);
            w = wave_pick(w);
            if (lane == 0) {
                *s_win = w.idx;
                emit(r, w);
            }
        }
        __syncthreads();
        const int win = *s_win;
        if (win >= 0) {
            retire(win);
            stale = s_idx[wv] == win;  // LDS read, the same in every lane
        }
    }
}

// grid (workgroups over traces): each workgroup extracts the m best of its 1024 traces by m
// rounds of the exact pick; the last workgroup to arrive extracts the m best of all winners.
__global__ void __launch_bounds__(kPickThreads) eamc_topm_kernel(TopmArgs a) {
    __shared__ u64 s_dot[kPickWaves];
    __shared__ u64 s_nt[kPickWaves];
    __shared__ int s_idx[kPickWaves];
    __shared__ u64 s_nq;
    __shared__ unsigned s_ticket;
    __shared__ int s_win;
    __shared__ int s_sn[2];
    __shared__ int s_best[kMaxMatchBatch];
    __shared__ HeadLds s_heads;
    __shared__ KeyLds s_keys;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wv = tid / kWave;
    const bool single = gridDim.x == 1;

    u64 nq = 0;
    for (int i = tid; i < a.LE; i += kPickThreads) {
        u64 v = (uint32_t)a.q[i];
        nq += v * v;
    }
    nq = wave_sum_u64_dpp(nq);
    if (lane == 0) s_dot[wv] = nq;
    __syncthreads();
    if (tid == 0) {
        u64 t = 0;
        for (int i = 0; i < kPickWaves; ++i) t += s_dot[i];
        s_nq = t;
    }
    __syncthreads();
    nq = s_nq;

    Best me = make_best(0, 1, -1);
    const int n = blockIdx.x * kPickChunk + tid;  // one trace per thread
    if (n < a.N) {
        const u64* pp = a.part + n;
        u64 dot = 0;
        for (int s = 0; s < a.n_lsplit; ++s) dot += pp[(size_t)s * a.n_cap];
        const u64 nt = a.norm2[n];
        if (a.sims) a.sims[n] = (float)cosine(dot, nq, nt);
        me = make_best(dot, nt, n);
    }
    extract_top(
        a.m, s_dot, s_nt, s_idx, &s_win, [&]() { return me; },
        [&](int win) {
            if (me.idx == win) me = make_best(0, 1, -1);
        },
        [&](int r, const Best& w) {
            if (single) {
                a.top[r] = w.idx;
                if (a.top_sim) a.top_sim[r] = w.idx >= 0 ? (float)cosine(w.dot, nq, w.nt) : 0.f;
                s_best[r] = w.idx;
            } else {
                const size_t ci = (size_t)blockIdx.x * a.m + r;
                a.cand[ci * 2] = w.dot;
                a.cand[ci * 2 + 1] = w.nt;
                a.cand_idx[ci] = w.idx;
            }
        });
    if (!single) {
        if (tid == 0) {
            __threadfence();
            s_ticket = __hip_atomic_fetch_add(a.ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();
        if (s_ticket != gridDim.x - 1) return;
        if (tid == 0) __threadfence();
        __syncthreads();
        const int total = (int)gridDim.x * a.m;  // the host keeps this within kTopmPerThread per thread
        Best mine[kTopmPerThread];
#pragma unroll
        for (int u = 0; u < kTopmPerThread; ++u) {
            const int i = tid + u * kPickThreads;
            mine[u] = make_best(0, 1, -1);
            if (i < total) {
                const int idx = __hip_atomic_load(&a.cand_idx[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (idx >= 0) {
                    const u64 d = __hip_atomic_load(&a.cand[(size_t)i * 2], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    const u64 t = __hip_atomic_load(&a.cand[(size_t)i * 2 + 1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    mine[u] = make_best(d, t, idx);
                }
            }
        }
        __syncthreads();  // the first phase is done with the LDS winners
        extract_top(
            a.m, s_dot, s_nt, s_idx, &s_win,
            [&]() {
                Best loc = mine[0];
#pragma unroll
                for (int u = 1; u < kTopmPerThread; ++u) loc = pick(loc, mine[u]);
                return loc;
            },
            [&](int win) {
#pragma unroll
                for (int u = 0; u < kTopmPerThread; ++u)
                    if (mine[u].idx == win) mine[u] = make_best(0, 1, -1);
            },
            [&](int r, const Best& w) {
                a.top[r] = w.idx;
                if (a.top_sim) a.top_sim[r] = w.idx >= 0 ? (float)cosine(w.dot, nq, w.nt) : 0.f;
                s_best[r] = w.idx;
            });
        if (tid == 0) *a.ticket = 0;  // ready for the next launch on this stream
    }
    if (a.do_score) score_and_heads(a.sc, s_heads, s_keys, s_sn, s_best, true);
}

struct Plan {
    int VEC, J, TN, rowV, n_tiles, n_lsplit, lper, NB;
    size_t smem;
};

Plan make_plan(const moei_eamc* c, int L_scan, int B) {
    static const int kTargetBlocks = getenv("MOEI_MATCH_BLOCKS") ? atoi(getenv("MOEI_MATCH_BLOCKS")) : 0;
    Plan p{};
    p.NB = B > 8 ? 16 : (B > 4 ? 8 : (B >= 3 ? 4 : (B == 2 ? 2 : 1)));  // queries served by one pass over the traces
    const int E = c->d.E;
    const int full = 16 / c->cell_bytes;
    p.VEC = (E % full == 0) ? full : 1;
    p.rowV = E / p.VEC;
    const long total_vec = (long)c->N * L_scan * p.rowV;
    // vectors per thread: fewer when the whole scan is small, and when many queries' accumulators need the registers
    const int jt = total_vec >= (1L << 20) ? (p.NB >= 8 ? 2 : 4) : 1;
    p.TN = (kDotThreads * jt) / p.rowV;
    if (p.TN < 1) p.TN = 1;
    p.J = (p.TN * p.rowV + kDotThreads - 1) / kDotThreads;
    if (p.J > 2 && p.NB > 4) p.NB = 4;  // very wide rows: the accumulators of 8 or 16 queries would not fit the registers
    p.n_tiles = (c->N + p.TN - 1) / p.TN;
    // aim at two rounds of workgroups over the chip (short scans too: 4.2 instead of 4.5 us for
    // 1,000 traces beside the streaming FFN); the query groups multiply the grid as well
    const int target = kTargetBlocks > 0 ? kTargetBlocks : 512;
    const int per_split = p.n_tiles * ((B + p.NB - 1) / p.NB);
    int want = (target + per_split - 1) / per_split;
    int lmax = L_scan < c->lsplit_max ? L_scan : c->lsplit_max;
    p.n_lsplit = want < 1 ? 1 : (want > lmax ? lmax : want);
    // LDS: the query rows of one split (for all NB queries) must fit in 48 KiB
    int min_split = (int)(((size_t)p.NB * L_scan * E * 4 + 49151) / 49152);
    if (p.n_lsplit < min_split) p.n_lsplit = min_split;
    p.lper = (L_scan + p.n_lsplit - 1) / p.n_lsplit;
    p.n_lsplit = (L_scan + p.lper - 1) / p.lper;
    p.smem = (((size_t)p.NB * p.lper * E * 4 + 15) & ~(size_t)15) + (size_t)p.NB * p.TN * 8;
    return p;
}

template <typename CT, int VEC, int NB>
int launch_dot_nb(const Plan& p, const DotArgs& a, dim3 grid, hipStream_t s) {
#define MOEI_DOT_CASE(JJ)                                                                              \
    case JJ:                                                                                           \
        launch(K_MATCH_DOT, eamc_dot_kernel<CT, VEC, JJ, NB>, grid, dim3(kDotThreads), p.smem, s, a);  \
        break;
    if constexpr (NB >= 8) {  // the plan gives batches of 8 and 16 queries at most two vectors per thread
        switch (p.J) {
            MOEI_DOT_CASE(1)
            MOEI_DOT_CASE(2)
            default:
                MOEI_FAIL(MOEI_EINVAL, "eamc_match: no kernel for %d vectors per thread and %d queries per pass", p.J, NB);
        }
    } else {
        switch (p.J) {
            MOEI_DOT_CASE(1)
            MOEI_DOT_CASE(2)
            MOEI_DOT_CASE(3)
            MOEI_DOT_CASE(4)
            MOEI_DOT_CASE(5)
            MOEI_DOT_CASE(6)
            MOEI_DOT_CASE(7)
            MOEI_DOT_CASE(8)
            default:
                MOEI_FAIL(MOEI_EINVAL, "eamc_match: no kernel for %d vectors per thread", p.J);
        }
    }
#undef MOEI_DOT_CASE
    MOEI_LAUNCH_CHECK();
    return MOEI_OK;
}

template <typename CT, int VEC>
int launch_dot_j(const Plan& p, const DotArgs& a, dim3 grid, hipStream_t s) {
    if (p.NB == 16) return launch_dot_nb<CT, VEC, 16>(p, a, grid, s);
    if (p.NB == 8) return launch_dot_nb<CT, VEC, 8>(p, a, grid, s);
    if (p.NB == 4) return launch_dot_nb<CT, VEC, 4>(p, a, grid, s);
    if (p.NB == 2) return launch_dot_nb<CT, VEC, 2>(p, a, grid, s);
    return launch_dot_nb<CT, VEC, 1>(p, a, grid, s);
}

// The plan of the matrix-core scan: tiles of 64 J traces, layer splits that keep the query planes of
// a split within 64 KiB of LDS (more splits where the tiles alone do not fill the chip).
struct MmPlan {
    bool ok;
    int n_tiles, n_lsplit, lper, nblk, q_stride, DA;
    size_t smem;
};

// The plan of the matrix-core scan: tiles of 64 traces and the layer splits that keep a split's units
// within kMmMaxUnits (more splits where the tiles alone do not fill the chip).
MmPlan make_mm_plan(const moei_eamc* c, int L_scan, int B) {
    static const int kTarget = getenv("MOEI_MATCH_MM_BLOCKS") ? atoi(getenv("MOEI_MATCH_MM_BLOCKS")) : 0;
    static const int kSplits = getenv("MOEI_MATCH_MM_SPLITS") ? atoi(getenv("MOEI_MATCH_MM_SPLITS")) : 0;
    MmPlan p{};
    const int E = c->d.E;
    p.nblk = (E + 63) / 64;
    const int lper_max = kMmMaxUnits / p.nblk;
    if (lper_max < 1) return p;
    p.n_tiles = (c->N + 63) / 64;
    const int groups = (B + kMmQueries - 1) / kMmQueries;
    const int target = kTarget > 0 ? kTarget : 512;
    const int lmax = L_scan < c->lsplit_max ? L_scan : c->lsplit_max;
    const int min_split = (L_scan + lper_max - 1) / lper_max;
    int want = kSplits > 0 ? kSplits : (target + p.n_tiles * groups - 1) / (p.n_tiles * groups);
    if (want < min_split) want = min_split;
    p.n_lsplit = want > lmax ? lmax : want;
    if (p.n_lsplit < min_split) return p;
    p.lper = (L_scan + p.n_lsplit - 1) / p.n_lsplit;
    p.n_lsplit = (L_scan + p.lper - 1) / p.lper;
    p.q_stride = p.lper * p.nblk * 64;
    if ((p.q_stride / 16) % 2 == 0) p.q_stride += 16;
    p.smem = (size_t)(kDotThreads / kWave) * kMmRing * (64 * 16 * c->cell_bytes) + (size_t)kMaxDigits * kMmQueries * p.q_stride;
    p.DA = digits_of_host((unsigned)c->max_cell);
    p.ok = true;
    return p;
}

int launch_dot_mm(const MmPlan& p, const DotMmArgs& a, int cell_bytes, dim3 grid, hipStream_t s) {
#define MOEI_MM_CASE(DD, CB_)                                                                         \
    case (DD) * 8 + (CB_): {                                                                          \
        static bool allowed = false; /* more than 64 KiB of dynamic LDS must be asked for once */     \
        if (!allowed) {                                                                               \
            MOEI_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(eamc_dot_mm_kernel<DD, CB_>),  \
                                         hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024));     \
            allowed = true;                                                                           \
        }                                                                                             \
        launch(K_MATCH_DOT, eamc_dot_mm_kernel<DD, CB_>, grid, dim3(kDotThreads), p.smem, s, a);     \
        break;                                                                                        \
    }
    switch (p.DA * 8 + cell_bytes) {
        MOEI_MM_CASE(1, 4)
        MOEI_MM_CASE(2, 4)
        MOEI_MM_CASE(3, 4)
        MOEI_MM_CASE(4, 4)
        MOEI_MM_CASE(1, 2)
        MOEI_MM_CASE(2, 2)
        MOEI_MM_CASE(3, 2)
        default:
            MOEI_FAIL(MOEI_EINVAL, "eamc_match: no matrix-core scan for %d digits of %d-byte cells", p.DA, cell_bytes);
    }
#undef MOEI_MM_CASE
    MOEI_LAUNCH_CHECK();
    return MOEI_OK;
}

size_t cells(const moei_eamc* c) { return (size_t)c->d.L * c->n_cap * c->d.E; }

}  // namespace

}  // namespace moei

using namespace moei;

extern "C" int moei_eamc_create(const moei_model_desc* desc, int32_t n_cap, int32_t cell_bytes, moei_eamc** out) {
    MOEI_REQUIRE(desc && out, "moei_eamc_create: null pointer");
    *out = nullptr;
    int rc = check_desc(desc);
    if (rc) return rc;
    MOEI_REQUIRE(n_cap >= 1, "moei_eamc_create: n_cap = %d must be positive", n_cap);
    MOEI_REQUIRE(cell_bytes == 4 || cell_bytes == 2, "moei_eamc_create: cell_bytes must be 4 or 2");
    MOEI_REQUIRE(desc->E <= kMaxE, "moei_eamc_create: E = %d exceeds %d", desc->E, kMaxE);
    moei_eamc* c = new (std::nothrow) moei_eamc();
    if (!c) MOEI_FAIL(MOEI_ENOMEM, "moei_eamc_create: out of host memory");
    c->d = *desc;
    c->n_cap = n_cap;
    c->cell_bytes = cell_bytes;
    c->lsplit_max = desc->L < 32 ? desc->L : 32;
    const size_t LE = (size_t)desc->L * desc->E;
    hipError_t e = hipMalloc(&c->d_traces, cells(c) * cell_bytes);
    if (e == hipSuccess) e = hipMalloc((void**)&c->d_norm2, (size_t)n_cap * 8);
    if (e == hipSuccess) e = hipMalloc((void**)&c->d_part, (size_t)kMaxMatchBatch * c->lsplit_max * n_cap * 8);
    const size_t n_blk_max = ((size_t)n_cap + kPickChunk - 1) / kPickChunk;
    if (e == hipSuccess) e = hipMalloc((void**)&c->d_cand, (size_t)kMaxMatchBatch * n_blk_max * 2 * 8);
    if (e == hipSuccess) e = hipMalloc((void**)&c->d_cand_idx, (size_t)kMaxMatchBatch * n_blk_max * 4);
    if (e == hipSuccess) e = hipMalloc((void**)&c->d_ticket, (size_t)kMaxMatchBatch * 4);
    if (e == hipSuccess) e = hipMemset(c->d_ticket, 0, (size_t)kMaxMatchBatch * 4);
    if (e == hipSuccess) e = hipMalloc((void**)&c->d_keys, 2 * LE * 8);
    if (e != hipSuccess) {
        moei_eamc_destroy(c);
        MOEI_FAIL(MOEI_ENOMEM, "moei_eamc_create: device allocation failed: %s", hipGetErrorString(e));
    }
    *out = c;
    return MOEI_OK;
}

extern "C" int moei_eamc_destroy(moei_eamc* c) {
    if (!c) return MOEI_OK;
    (void)hipFree(c->d_traces);
    (void)hipFree(c->d_norm2);
    (void)hipFree(c->d_part);
    (void)hipFree(c->d_cand);
    (void)hipFree(c->d_cand_idx);
    (void)hipFree(c->d_ticket);
    (void)hipFree(c->d_keys);
    delete c;
    return MOEI_OK;
}

extern "C" int moei_eamc_size(const moei_eamc* c) {
    MOEI_REQUIRE(c, "moei_eamc_size: null pointer");
    return c->N;
}

namespace {

int check_cells(const int32_t* p, size_t n, int cell_bytes, int32_t* largest) {
    const int32_t hi = cell_bytes == 2 ? 65535 : MOEI_MAX_COUNT;
    int32_t m = 0;
    for (size_t i = 0; i < n; ++i) {
        if (p[i] < 0 || p[i] > hi)
            MOEI_FAIL(MOEI_EINVAL, "EAM cell %zu holds %d, outside [0, %d]", i, p[i], hi);
        m = p[i] > m ? p[i] : m;
    }
    *largest = m;
    return MOEI_OK;
}

unsigned long long norm2_of(const int32_t* p, size_t n) {
    unsigned long long s = 0;
    for (size_t i = 0; i < n; ++i) s += (unsigned long long)p[i] * (unsigned long long)p[i];
    return s;
}

}  // namespace

extern "C" int moei_eamc_load(moei_eamc* c, const int32_t* h_traces, int32_t N) {
    MOEI_REQUIRE(c, "moei_eamc_load: null pointer");
    MOEI_REQUIRE(N >= 0, "moei_eamc_load: N = %d is negative", N);
    if (N > c->n_cap) MOEI_FAIL(MOEI_ECAPACITY, "moei_eamc_load: N = %d exceeds the capacity %d", N, c->n_cap);
    MOEI_REQUIRE(N == 0 || h_traces, "moei_eamc_load: null traces");
    const int L = c->d.L, E = c->d.E;
    const size_t LE = (size_t)L * E;
    int32_t largest = 0;
    if (N > 0) {  // refused input leaves the collection as it was
        int rc = check_cells(h_traces, (size_t)N * LE, c->cell_bytes, &largest);
        if (rc) return rc;
    }
    c->N = 0;
    c->max_cell = largest;
    if (N == 0) return MOEI_OK;
    // trace-major -> layer-major staging, one layer at a time
    std::vector<unsigned long long> norm((size_t)N);
    for (int n = 0; n < N; ++n) norm[n] = norm2_of(h_traces + (size_t)n * LE, LE);
    std::vector<unsigned char> stage;
    try {
        stage.resize((size_t)N * E * c->cell_bytes);
    } catch (...) {
        MOEI_FAIL(MOEI_ENOMEM, "moei_eamc_load: out of host memory");
    }
    for (int l = 0; l < L; ++l) {
        if (c->cell_bytes == 4) {
            int32_t* dst = reinterpret_cast<int32_t*>(stage.data());
            for (int n = 0; n < N; ++n) memcpy(dst + (size_t)n * E, h_traces + (size_t)n * LE + (size_t)l * E, (size_t)E * 4);
        } else {
            uint16_t* dst = reinterpret_cast<uint16_t*>(stage.data());
            for (int n = 0; n < N; ++n) {
                const int32_t* src = h_traces + (size_t)n * LE + (size_t)l * E;
                for (int e = 0; e < E; ++e) dst[(size_t)n * E + e] = (uint16_t)src[e];
            }
        }
        unsigned char* d = reinterpret_cast<unsigned char*>(c->d_traces) + (size_t)l * c->n_cap * E * c->cell_bytes;
        MOEI_HIP(hipMemcpy(d, stage.data(), stage.size(), hipMemcpyHostToDevice));
    }
    MOEI_HIP(hipMemcpy(c->d_norm2, norm.data(), (size_t)N * 8, hipMemcpyHostToDevice));
    c->N = N;
    return MOEI_OK;
}

extern "C" int moei_eamc_insert(moei_eamc* c, const int32_t* h_eam, int32_t victim) {
    MOEI_REQUIRE(c && h_eam, "moei_eamc_insert: null pointer");
    const int L = c->d.L, E = c->d.E;
    const size_t LE = (size_t)L * E;
    int32_t largest = 0;
    int rc = check_cells(h_eam, LE, c->cell_bytes, &largest);
    if (rc) return rc;
    int pos;
    if (c->N < c->n_cap) {
        pos = c->N;
    } else {
        MOEI_REQUIRE(victim >= 0 && victim < c->N, "moei_eamc_insert: victim %d outside [0, %d)", victim, c->N);
        pos = victim;
    }
    const size_t cb = c->cell_bytes;
    std::vector<uint16_t> narrow;
    const void* src = h_eam;
    if (cb == 2) {
        narrow.resize(LE);
        for (size_t i = 0; i < LE; ++i) narrow[i] = (uint16_t)h_eam[i];
        src = narrow.data();
    }
    unsigned char* dst = reinterpret_cast<unsigned char*>(c->d_traces) + (size_t)pos * E * cb;
    MOEI_HIP(hipMemcpy2D(dst, (size_t)c->n_cap * E * cb, src, (size_t)E * cb, (size_t)E * cb, L, hipMemcpyHostToDevice));
    unsigned long long n2 = norm2_of(h_eam, LE);
    MOEI_HIP(hipMemcpy(c->d_norm2 + pos, &n2, 8, hipMemcpyHostToDevice));
    if (pos == c->N) c->N += 1;
    if (largest > c->max_cell) c->max_cell = largest;  // (a replaced trace may have held the old maximum: the bound stays)
    return MOEI_OK;
}

extern "C" int moei_eamc_export(const moei_eamc* c, int32_t* h_traces, int32_t max_traces) {
    MOEI_REQUIRE(c && (h_traces || c->N == 0), "moei_eamc_export: null pointer");
    if (max_traces < c->N) MOEI_FAIL(MOEI_ECAPACITY, "moei_eamc_export: room for %d traces, %d stored", max_traces, c->N);
    const int L = c->d.L, E = c->d.E, N = c->N;
    if (N == 0) return MOEI_OK;
    const size_t cb = c->cell_bytes;
    std::vector<unsigned char> stage((size_t)N * E * cb);
    for (int l = 0; l < L; ++l) {
        const unsigned char* d = reinterpret_cast<const unsigned char*>(c->d_traces) + (size_t)l * c->n_cap * E * cb;
        MOEI_HIP(hipMemcpy(stage.data(), d, stage.size(), hipMemcpyDeviceToHost));
        for (int n = 0; n < N; ++n) {
            int32_t* dst = h_traces + ((size_t)n * L + l) * E;
            if (cb == 4) {
                memcpy(dst, stage.data() + (size_t)n * E * 4, (size_t)E * 4);
            } else {
                const uint16_t* s16 = reinterpret_cast<const uint16_t*>(stage.data()) + (size_t)n * E;
                for (int e = 0; e < E; ++e) dst[e] = s16[e];
            }
        }
    }
    return MOEI_OK;
}

// Checkpoint file (failure recovery, App. B.2): a 32-byte header - magic "MOEIEAMC", version 1,
// L, E, N, 4 reserved bytes as zero - then the traces as int32 [N][L][E], little endian.
namespace {
struct EamcFileHeader {
    char magic[8];
    int32_t version, L, E, N;
    int32_t reserved[2];
};
static_assert(sizeof(EamcFileHeader) == 32, "header layout");
const char kEamcMagic[8] = {'M', 'O', 'E', 'I', 'E', 'A', 'M', 'C'};
}  // namespace

extern "C" int moei_eamc_save(const moei_eamc* c, const char* path) {
    MOEI_REQUIRE(c && path, "moei_eamc_save: null pointer");
    std::vector<int32_t> host;
    try {
        host.resize((size_t)c->N * c->d.L * c->d.E);
    } catch (...) {
        MOEI_FAIL(MOEI_ENOMEM, "moei_eamc_save: out of host memory");
    }
    int rc = moei_eamc_export(c, host.data(), c->N);
    if (rc) return rc;
    FILE* f = fopen(path, "wb");
    if (!f) MOEI_FAIL(MOEI_ESTATE, "moei_eamc_save: cannot open %s for writing", path);
    EamcFileHeader h{};
    memcpy(h.magic, kEamcMagic, 8);
    h.version = 1;
    h.L = c->d.L;
    h.E = c->d.E;
    h.N = c->N;
    bool ok = fwrite(&h, sizeof(h), 1, f) == 1;
    if (ok && !host.empty()) ok = fwrite(host.data(), sizeof(int32_t), host.size(), f) == host.size();
    ok = (fclose(f) == 0) && ok;
    if (!ok) MOEI_FAIL(MOEI_ESTATE, "moei_eamc_save: writing %s failed", path);
    return MOEI_OK;
}

extern "C" int moei_eamc_restore(moei_eamc* c, const char* path) {
    MOEI_REQUIRE(c && path, "moei_eamc_restore: null pointer");
    FILE* f = fopen(path, "rb");
    if (!f) MOEI_FAIL(MOEI_ESTATE, "moei_eamc_restore: cannot open %s", path);
    EamcFileHeader h{};
    if (fread(&h, sizeof(h), 1, f) != 1 || memcmp(h.magic, kEamcMagic, 8) != 0 || h.version != 1) {
        fclose(f);
        MOEI_FAIL(MOEI_EINVAL, "moei_eamc_restore: %s is not an EAMC checkpoint", path);
    }
    if (h.L != c->d.L || h.E != c->d.E || h.N < 0 || h.N > c->n_cap) {
        fclose(f);
        MOEI_FAIL(MOEI_EINVAL, "moei_eamc_restore: checkpoint holds %d traces of %dx%d, the collection takes %d of %dx%d",
                  h.N, h.L, h.E, c->n_cap, c->d.L, c->d.E);
    }
    std::vector<int32_t> host;
    try {
        host.resize((size_t)h.N * h.L * h.E);
    } catch (...) {
        fclose(f);
        MOEI_FAIL(MOEI_ENOMEM, "moei_eamc_restore: out of host memory");
    }
    const bool ok = host.empty() || fread(host.data(), sizeof(int32_t), host.size(), f) == host.size();
    fclose(f);
    if (!ok) MOEI_FAIL(MOEI_EINVAL, "moei_eamc_restore: %s is truncated", path);
    return moei_eamc_load(c, host.data(), h.N);
}

namespace moei {

namespace {
// The partial dot products of B queries against every stored trace (layers 0..layer_hi).
int launch_dots(const moei_eamc* c, const int32_t* d_eam, int B, int layer_hi, int* n_lsplit, hipStream_t s) {
    const int L = c->d.L, E = c->d.E;
    *n_lsplit = 0;
    if (c->N == 0) return MOEI_OK;
    // a.  Three queries and more (five and more for rows of several units, where a split holds few layers):
    // the scan as a matrix product (rows of whole 16-byte pieces); it takes the same time
    // for 3 as for 16 queries.  Measured at 10,000 traces: 26 x 64 cells, 4 queries 27.8 against 28.2 us
    // and 16 queries 29.3 against 44.7 us; 59 x 160 cells, 4 queries 100 against 84 us and 16 queries 111
    // against 207 us.
    static const bool kNoMm = getenv("MOEI_MATCH_NO_MM") && atoi(getenv("MOEI_MATCH_NO_MM")) != 0;
    if (B >= (E <= 64 ? 3 : 5) && !kNoMm && E % (16 / c->cell_bytes) == 0 && (uintptr_t)d_eam % 16 == 0) {
        const MmPlan mp = make_mm_plan(c, layer_hi + 1, B);
        if (mp.ok) {
            *n_lsplit = mp.n_lsplit;
            DotMmArgs ma{c->d_traces, d_eam, c->d_part, c->n_cap, c->N, L, E, B,
                         layer_hi + 1, mp.lper, mp.n_lsplit, mp.nblk, mp.n_tiles, mp.q_stride};
            return launch_dot_mm(mp, ma, c->cell_bytes, dim3(mp.n_tiles, mp.n_lsplit, (B + kMmQueries - 1) / kMmQueries), s);
        }
    }
    // b.  One or two queries, other shapes: the scan on the vector ALUs
    Plan p = make_plan(c, layer_hi + 1, B);
    *n_lsplit = p.n_lsplit;
    if (p.n_lsplit > c->lsplit_max || p.smem > 64 * 1024)
        MOEI_FAIL(MOEI_ECAPACITY, "eamc_match: L*E = %d is too large for the match kernel's LDS staging", L * E);
    // a collection that fits the 256 MB last-level cache stays there between layer steps; a longer
    // scan is read once per match and should not displace other data
    const size_t scan_bytes = (size_t)c->N * (layer_hi + 1) * E * c->cell_bytes;
    DotArgs a{c->d_traces, d_eam, c->d_part, c->n_cap, c->N, L, E, B, layer_hi + 1, p.lper, p.n_lsplit, p.TN, p.rowV,
              scan_bytes > ((size_t)192 << 20),
              p.rowV <= kWave && (p.rowV & (p.rowV - 1)) == 0 && kDotThreads % p.rowV == 0};
    dim3 grid(p.n_tiles, p.n_lsplit, (B + p.NB - 1) / p.NB);
    if (c->cell_bytes == 4)
        return p.VEC == 4 ? launch_dot_j<int32_t, 4>(p, a, grid, s) : launch_dot_j<int32_t, 1>(p, a, grid, s);
    return p.VEC == 8 ? launch_dot_j<uint16_t, 8>(p, a, grid, s) : launch_dot_j<uint16_t, 1>(p, a, grid, s);
}
}  // namespace

int launch_match(const moei_eamc* c, const int32_t* d_eam, int B, int layer_hi, int32_t* d_best, float* d_best_sim,
                 float* d_sims, const ScoreArgs* score, hipStream_t s) {
    const int L = c->d.L, E = c->d.E;
    if (score && B != 1) MOEI_FAIL(MOEI_EINVAL, "match with scoring needs B = 1");
    int n_lsplit = 0;
    int rc = launch_dots(c, d_eam, B, layer_hi, &n_lsplit, s);
    if (rc) return rc;
    const int n_blk = c->N > 0 ? (c->N + kPickChunk - 1) / kPickChunk : 1;
    PickArgs pa{c->d_part, c->d_norm2, d_eam, n_lsplit, c->n_cap, c->N, L * E, c->d_cand, c->d_cand_idx,
                c->d_ticket, d_best, d_best_sim, d_sims, score != nullptr, score ? *score : ScoreArgs{}};
    launch(K_MATCH_ARGMAX, eamc_pick_kernel, dim3(n_blk, B), dim3(kPickThreads), 0, s, pa);
    MOEI_LAUNCH_CHECK();
    return MOEI_OK;
}

int launch_match_topm(const moei_eamc* c, const int32_t* d_eam, int layer_hi, int m, int32_t* d_top, float* d_top_sim,
                      float* d_sims, const ScoreArgs* score, hipStream_t s) {
    const int L = c->d.L, E = c->d.E;
    if (m < 1 || m > kMaxMatchBatch) MOEI_FAIL(MOEI_EINVAL, "eamc_match_topm: m = %d outside [1, %d]", m, kMaxMatchBatch);
    const int n_blk = c->N > 0 ? (c->N + kPickChunk - 1) / kPickChunk : 1;
    if ((long)n_blk * m > (long)kTopmPerThread * kPickThreads)
        MOEI_FAIL(MOEI_ECAPACITY, "eamc_match_topm: %d traces x m = %d exceed the finishing workgroup's %d candidates",
                  c->N, m, kTopmPerThread * kPickThreads);
    int n_lsplit = 0;
    int rc = launch_dots(c, d_eam, 1, layer_hi, &n_lsplit, s);
    if (rc) return rc;
    TopmArgs ta{c->d_part, c->d_norm2, d_eam, n_lsplit, c->n_cap, c->N, L * E, m, c->d_cand, c->d_cand_idx,
                c->d_ticket, d_top, d_top_sim, d_sims, score != nullptr, score ? *score : ScoreArgs{}};
    launch(K_MATCH_ARGMAX, eamc_topm_kernel, dim3(n_blk), dim3(kPickThreads), 0, s, ta);
    MOEI_LAUNCH_CHECK();
    return MOEI_OK;
}

}  // namespace moei

extern "C" int eamc_match(const moei_eamc* c, const int32_t* d_eam, int32_t B, int32_t layer_hi, int32_t* d_best,
                          float* d_best_sim, float* d_sims, void* stream) {
    MOEI_REQUIRE(c && d_eam && d_best, "eamc_match: null pointer");
    MOEI_REQUIRE(B >= 0 && B <= kMaxMatchBatch, "eamc_match: B = %d outside [0, %d]", B, kMaxMatchBatch);
    MOEI_REQUIRE(layer_hi >= 0 && layer_hi < c->d.L, "eamc_match: layer_hi = %d outside [0, %d)", layer_hi, c->d.L);
    if (B == 0) return MOEI_OK;
    return launch_match(c, d_eam, B, layer_hi, d_best, d_best_sim, d_sims, nullptr, as_stream(stream));
}

extern "C" int eamc_match_topm(const moei_eamc* c, const int32_t* d_eam, int32_t layer_hi, int32_t m, int32_t* d_top,
                               float* d_top_sim, float* d_sims, void* stream) {
    MOEI_REQUIRE(c && d_eam && d_top, "eamc_match_topm: null pointer");
    MOEI_REQUIRE(layer_hi >= 0 && layer_hi < c->d.L, "eamc_match_topm: layer_hi = %d outside [0, %d)", layer_hi, c->d.L);
    return launch_match_topm(c, d_eam, layer_hi, m, d_top, d_top_sim, d_sims, nullptr, as_stream(stream));
}
