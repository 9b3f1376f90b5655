// The prefill iteration of one MoE layer: all n prompt tokens pass the layer together.
//
// Sec. 4.3 of the paper: an iteration routes n tokens and every token adds its k picks to
// row l of the request's EAM.  Five launches:
//   1. prefill_route_kernel   router logits + softmax/top-k, one wavefront per token (the
//                             same summation order as the decode routing, so the same bits)
//   2. prefill_group_kernel   histogram of the picks -> EAM row; tokens grouped per expert in
//                             ascending token order, cut into items of <= 64 (long prompts: 256) tokens
//   3. prefill_gateup_kernel, prefill_down_kernel
//                             grouped SwiGLU expert FFN on the matrix cores as two tiled products
//                             per item; an expert's weights pass once per item
//   4. prefill_reduce_kernel  y[t] = sum of the token's rows, in pick order
// With tens of tokens per expert the layer is still bound by streaming the weights (one weight
// byte meets about as many flops as the item has tokens); the matrix cores keep the arithmetic
// off the critical path.  v_mfma_f32_16x16x32_bf16: A is 16 x 32 (lane l holds row l%16,
// k = 8*(l/16)..+8), B is 32 x 16 (lane l holds column l%16, same k), D is 16 x 16 (lane l holds
// column l%16, rows 4*(l/16)..+4).
#include <stdlib.h>
#include <string.h>

#include <type_traits>

#include "kernels.hpp"
#include "topk.hpp"
#include "wtypes.hpp"

namespace moei {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ bf16x8 ld_bf16x8(const uint16_t* p) { return *reinterpret_cast<const bf16x8*>(p); }

// LDS tiles of the matrix kernels hold rows of 128 bf16 (sixteen 16-byte chunks) with no padding;
// chunk c of row r sits at chunk position c ^ (r % 16).  Staging writes (sixteen lanes along one
// row) still cover 256 contiguous bytes, and operand reads (sixteen lanes = sixteen consecutive
// rows, the same logical chunk) land on sixteen different chunk positions: both are free of bank
// conflicts.  (Measured with a read probe on one CU: 5.0 time units per wavefront access, as for
// contiguous data; rows padded by 8 elements take 8.3, by 16 elements 5.0 for operand reads but 8.3
// for the staging pattern, unpadded unswizzled rows 32.)
constexpr int kTileK = 128;
__device__ __forceinline__ int swz(int row, int chunk) { return row * kTileK + ((chunk ^ (row & 15)) << 3); }
constexpr int kPfMaxE = 2048;

struct PItem {
    int32_t slot;       // cache slot of the expert
    int32_t ntok;       // tokens of the item, <= TM
    int32_t list_off;   // routed: position of the item's first token in perm / pgate
    int32_t first_tok;  // shared expert: tokens first_tok .. first_tok + ntok - 1 with weight 1; else -1
    int32_t row0;       // the item's first row of the activation / contribution buffers
    int32_t once;       // the expert has no other item: its weights are read once (non-temporal loads)
};

// ------------------------------------------------------------------ 1. routing of n tokens
// grid n: one workgroup of four wavefronts per token.  The token sits in LDS as fp32; logit
// rows are dealt to the wavefronts, eight rows' loads in flight per round trip; every row's sum
// runs over the chunks in ascending order, as in the decode routing.  Wavefront 0 then takes
// the top-k.
template <typename WT>
__global__ void __launch_bounds__(4 * kWave) prefill_route_kernel(const void* __restrict__ Wv,
                                                                  const float* __restrict__ bias,
                                                                  const void* __restrict__ Xv, int n, int H, int E, int k,
                                                                  int renorm, int vec_ok, int32_t* __restrict__ idx,
                                                                  float* __restrict__ w, int32_t* __restrict__ where,
                                                                  int32_t* __restrict__ flags) {
    using V = WVec<WT>;
    extern __shared__ __align__(16) float smem[];
    __shared__ int s_idx[kWave];
    __shared__ float s_w[kWave];
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    float* xs = smem;      // [H] the token, fp32
    float* z = smem + H;   // [E] its logits
    const int t = blockIdx.x;
    const WT* W = reinterpret_cast<const WT*>(Wv);
    const WT* x = reinterpret_cast<const WT*>(Xv) + (size_t)t * H;
    for (int c = tid; c < H; c += 4 * kWave) xs[c] = V::one(x + c);
    __syncthreads();
    constexpr int RB = 8;
    for (int e0 = wv * RB; e0 < E; e0 += 4 * RB) {
        float acc[RB];
#pragma unroll
        for (int q = 0; q < RB; ++q) acc[q] = 0.f;
        if (vec_ok) {
            for (int c = lane * V::N; c < H; c += kWave * V::N) {
                typename V::raw wr[RB];
#pragma unroll
                for (int q = 0; q < RB; ++q) wr[q] = V::load(W + (size_t)min(e0 + q, E - 1) * H + c);
                float xf[V::N];
#pragma unroll
                for (int q = 0; q < V::N; ++q) xf[q] = xs[c + q];
#pragma unroll
                for (int q = 0; q < RB; ++q) acc[q] = V::dot(wr[q], xf, acc[q]);
            }
        } else {
            for (int c = lane; c < H; c += kWave)
#pragma unroll
                for (int q = 0; q < RB; ++q)
                    acc[q] = __builtin_fmaf(V::one(W + (size_t)min(e0 + q, E - 1) * H + c), xs[c], acc[q]);
        }
#pragma unroll
        for (int q = 0; q < RB; ++q) {
            const float zq = wave_sum_dpp(acc[q]);
            if (lane == 0 && e0 + q < E) z[e0 + q] = zq + (bias ? bias[e0 + q] : 0.f);
        }
    }
    __syncthreads();
    if (wv != 0) return;
    int my_idx;
    float my_w;
    if (wave_logits_bad(z, E, lane)) {  // uniform: the token gets no picks and only its shared experts' output
        my_idx = -1;
        my_w = 0.f;
        if (lane == 0) atomicOr(flags, 4);
    } else if (E <= kRankMaxE) {
        const float sel = wave_topk_rank(z, E, k, renorm, lane, s_idx, s_w, false);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        my_idx = lane < k ? s_idx[lane] : -1;
        my_w = lane < k ? (renorm ? s_w[lane] / sel : s_w[lane]) : 0.f;
    } else {
        wave_topk(z, E, k, renorm, lane, my_idx, my_w);
    }
    if (lane < k) {
        idx[(size_t)t * k + lane] = my_idx;
        w[(size_t)t * k + lane] = my_w;
        where[(size_t)t * k + lane] = -1;  // no contribution row yet: the grouping names one per placed pick
    }
}

// ------------------------------------------------------------------ 2. grouping
struct GroupArgsP {
    const int32_t* idx;  // [n][k]
    const float* w;      // [n][k]
    int n, k, E, n_shared, TM;
    const int32_t* slot_of_row;  // [E]
    int shared_base;
    int32_t* eam_row;  // [E] row `layer` of the EAM
    int32_t* perm;     // [n*k] tokens grouped per expert, ascending token order inside an expert
    float* pgate;      // [n*k] their gate weights
    int32_t* where;    // [n*k] row (= position in perm) of every routed (token, pick)
    PItem* items;
    int32_t* meta;  // [0] = items in all, [1] = routed items
    int32_t* flags;
    int spread_shared;  // list the items so that all items of a shared expert fall on one XCD of the wide kernels
};

constexpr int kXcds = 8;  // workgroups are handed to the chip's 8 XCDs in turn
constexpr int kGrpThreads = 256;
constexpr int kGrpWaves = kGrpThreads / kWave;

// does token t pick expert e, and as which pick?  (-1: no)
__device__ __forceinline__ int pick_of(const GroupArgsP& g, int t, int e) {
    int j_hit = -1;
    if (t < g.n)
        for (int j = 0; j < g.k; ++j)
            if (g.idx[(size_t)t * g.k + j] == e) j_hit = j;
    return j_hit;
}

// tokens [w*span, (w+1)*span) belong to wavefront w of an expert's workgroup
__device__ __forceinline__ int group_span(int n) { return ((n + kGrpWaves - 1) / kGrpWaves + kWave - 1) / kWave * kWave; }

// 2. grid E, dynamic LDS E ints.  Every workgroup first forms the histogram of all picks for itself (a
// few thousand LDS additions: less than the launch a kernel of its own for it would cost) and, in
// the same pass, the count of its own expert per wavefront range; then offsets by a prefix over the
// counts, EAM row update, placement in ascending token order, the expert's items; workgroup 0 also
// lists the shared experts' items.
__global__ void __launch_bounds__(kGrpThreads) prefill_group_kernel(GroupArgsP g) {
    extern __shared__ int s_hist[];  // [E] tokens that pick each expert
    __shared__ int s_red[3][kGrpWaves];
    __shared__ int s_cw[kGrpWaves];  // tokens that pick this expert, per wavefront range
    const int e = blockIdx.x, tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    for (int f = tid; f < g.E; f += kGrpThreads) s_hist[f] = 0;
    __syncthreads();
    const int span = group_span(g.n);
    {
        // the picks of this wavefront's token range are one run of integers: read flat (a token's picks are
        // distinct, so the picks equal to e count the tokens that pick it), eight loads in flight per lane
        const int p0 = wv * span * g.k, p1 = min(g.n, (wv + 1) * span) * g.k;
        int c = 0;
        for (int i0 = p0; i0 < p1; i0 += 8 * kWave) {
            int f[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int i = i0 + u * kWave + lane;
                f[u] = i < p1 ? g.idx[i] : -1;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                if ((unsigned)f[u] < (unsigned)g.E) atomicAdd(&s_hist[f[u]], 1);  // (a token without a softmax has picks -1)
                c += f[u] == e ? 1 : 0;
            }
        }
        c = (int)wave_sum_u32_dpp((unsigned)c);
        if (lane == 0) s_cw[wv] = c;
    }
    __syncthreads();
    // tokens of the experts before this one (the grouped rows stay in expert order); items of the
    // experts that come before it in the item list, which runs from the expert with the most tokens to the
    // one with the fewest (equal counts: by index), so that the matrix kernels' longest workgroups start
    // first; items of all experts
    const int my_c = s_hist[e];
    int toks = 0, its = 0, its_all = 0;
    for (int f = tid; f < g.E; f += kGrpThreads) {
        const int c = s_hist[f];
        const int ni = (c + g.TM - 1) / g.TM;
        if (f < e) toks += c;
        if (c > my_c || (c == my_c && f < e)) its += ni;
        its_all += ni;
    }
    toks = (int)wave_sum_u32_dpp((unsigned)toks);
    its = (int)wave_sum_u32_dpp((unsigned)its);
    its_all = (int)wave_sum_u32_dpp((unsigned)its_all);
    if (lane == 0) {
        s_red[0][wv] = toks;
        s_red[1][wv] = its;
        s_red[2][wv] = its_all;
    }
    __syncthreads();
    int off = 0, ioff = 0, n_routed = 0, cnt = 0, before = 0;
    for (int w = 0; w < kGrpWaves; ++w) {
        off += s_red[0][w];
        ioff += s_red[1][w];
        n_routed += s_red[2][w];
        const int cw = s_cw[w];
        if (w < wv) before += cw;
        cnt += cw;
    }
    if (tid == 0) g.eam_row[e] += cnt;  // Sec. 4.3: the n tokens add n*k to row l
    int pos = before;
    for (int t0 = wv * span; t0 < min(g.n, (wv + 1) * span); t0 += 4 * kWave) {
        int jj[4];  // four 64-token groups' lookups go out together
#pragma unroll
        for (int u = 0; u < 4; ++u) jj[u] = pick_of(g, t0 + u * kWave + lane < min(g.n, (wv + 1) * span) ? t0 + u * kWave + lane : g.n, e);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int t = t0 + u * kWave + lane, j = jj[u];
            const unsigned long long mask = __ballot(j >= 0);
            if (j >= 0) {
                const int r = pos + __popcll(mask & ((1ull << lane) - 1ull));
                g.perm[off + r] = t;
                g.pgate[off + r] = g.w[(size_t)t * g.k + j];
                g.where[(size_t)t * g.k + j] = off + r;
            }
            pos += __popcll(mask);
        }
    }
    const int slot = g.slot_of_row[e];
    if (cnt > 0 && slot < 0 && tid == 0) atomicOr(g.flags, 2);
    // the shared experts' items come first in the list: they are full, and the matrix kernels' grids
    // start with the list's head, so the longest workgroups are not the last to start.  For the wide
    // kernels, which run item p on XCD p % 8, item `tile` of shared expert s sits at position
    // s + 8 * tile instead (and the routed items fill the other positions in their order): all items of
    // a shared expert then run on one XCD, several of them at a time, and its weights pass through
    // that L2 once for them.  (Needs at most 8 shared experts and enough routed items to leave no gap.)
    const int tiles = (g.n + g.TM - 1) / g.TM;
    const int n_sh_items = g.n_shared * tiles;
    const int free8 = kXcds - g.n_shared;  // routed positions per block of 8 among the first 8 * tiles
    const bool spread = g.spread_shared && g.n_shared > 0 && g.n_shared <= kXcds && n_routed >= tiles * free8;
    for (int it = tid; it * g.TM < cnt; it += kGrpThreads) {
        const int r = ioff + it;  // number of this item among the routed ones
        int p = n_sh_items + r;
        if (spread && r < tiles * free8) p = kXcds * (r / free8) + g.n_shared + r % free8;
        g.items[p] = PItem{slot, min(g.TM, cnt - it * g.TM), off + it * g.TM, -1, off + it * g.TM, cnt <= g.TM};
    }
    if (e == 0) {
        for (int q = tid; q < n_sh_items; q += kGrpThreads) {
            const int s = q / tiles, tile = q - s * tiles;
            g.items[spread ? s + kXcds * tile : q] =
                PItem{g.shared_base + s, min(g.TM, g.n - tile * g.TM), 0, tile * g.TM, g.n * g.k + s * g.n + tile * g.TM,
                      tiles == 1};
        }
        if (tid == 0) {
            g.meta[0] = n_routed + g.n_shared * tiles;
            g.meta[1] = n_routed;
        }
    }
}

// ------------------------------------------------------------------ 3. grouped expert FFN on the matrix cores
// Two tiled matrix products per item (an expert and up to TM = 64 or 128 of its tokens):
//   3a. act[row][u] = silu(<W_gate[u], x_row>) * <W_up[u], x_row> * gate_row      (K = H)
//   3b. yc[row][h]  = sum_u act[row][u] * W_down[h][u]                             (K = I)
// `row` numbers the (token, pick) pairs in grouped order, then the (shared expert, token)
// pairs.  The weights of an expert pass once per item, so long prompts take the larger items;
// the small operand (inputs / activations) goes through LDS in k-slices, double-buffered.  A
// workgroup has four wavefronts per 64 tokens of the item: wavefront w serves output group
// w % 4 (16 units / 128 columns) for tokens 64 * (w / 4) .. + 64.
constexpr int kTileTok = 64;      // tokens per item for short prompts: four 16-token blocks
constexpr int kTileTokBig = 128;  // for long prompts
constexpr int kGuUnits = 64;   // 3a: intermediate units per workgroup, 16 per wavefront
constexpr int kGuKS = 128;     // 3a: k-slice of inputs and weight rows in LDS
constexpr int kDnCols = 512;   // 3b: output columns per workgroup, 128 per wavefront
constexpr int kDnKS = 128;     // 3b: k-slice of the activations in LDS

struct MmArgs {
    const uint16_t* pool;
    size_t slot_elems;
    int n_slots_total;
    const PItem* items;
    const int32_t* meta;
    const uint16_t* X;  // [n][H] bf16
    const int32_t* perm;
    const float* pgate;
    uint16_t* act;  // [rows][I] bf16
    float* yc;      // [rows][H]
    int H, I;
    int32_t* flags;
    int n_ub;  // gate/up: blocks of 64 (wide kernel: 128) units;  down: blocks of 512 columns
    int n_cb;
    int dn_split;  // the down kernel takes an item in this many parts of TM tokens (items of the wide tile: 2)
};

// Workgroups are handed to the chip's 8 XCDs in turn, and every XCD has an L2 of its own.  The
// grids are one-dimensional and numbered so that one XCD always serves the same output blocks
// (unit blocks / column blocks, i.e. the same weight rows) for item after item: the items of
// one expert follow each other in the list, so the second and later ones find the expert's
// weights in that XCD's L2 instead of fetching them again.
__device__ __forceinline__ bool xcd_work(int n_blocks, int* item, int* block) {
    const int per = (n_blocks + kXcds - 1) / kXcds;  // output blocks per XCD
    const int v = blockIdx.x, xcd = v % kXcds, w = v / kXcds;
    *item = w / per;
    *block = xcd + kXcds * (w % per);
    return *block < n_blocks;
}

// The other way round, for the kernel whose workgroups each stream weights of their own: all output
// blocks of an item on one XCD, so that the item's input rows come through that L2 once.
__device__ __forceinline__ bool xcd_item_work(int n_blocks, int* item, int* block) {
    const int v = blockIdx.x, xcd = v % kXcds, w = v / kXcds;
    *block = w % n_blocks;
    *item = xcd + kXcds * (w / n_blocks);
    return true;
}


__device__ __forceinline__ float silu_f(float g) { return g / (1.0f + expf(-g)); }

// round-to-nearest-even fp32 -> bf16 bits (finite inputs)
__device__ __forceinline__ uint32_t bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

// 3a.  grid (ceil(I / 64), items).  D = A B with A = 16 weight rows (units) x 32 k, B = 32 k x 16
// tokens, both from LDS; a wavefront owns 16 units x 64 tokens (gate and up).  The weight rows
// are fetched in 256-byte runs (a k-slice of a row), the next slice into registers while the
// current one is multiplied.
template <int TM>
__global__ void __launch_bounds__(TM * 4) prefill_gateup_kernel(MmArgs a) {
    constexpr int kMmThreads = TM * 4;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    static_assert(kGuKS == kTileK && kDnKS == kTileK, "the LDS tiles are 128 elements wide");
    uint16_t* Xs = reinterpret_cast<uint16_t*>(smem_raw);  // [TM][128] inputs, chunks swizzled
    uint16_t* Ws = Xs + (size_t)TM * kTileK;               // [2 * kGuUnits][128] gate rows, then up rows
    __shared__ float s_gate[TM];
    int item, ub;
    if (!xcd_work(a.n_ub, &item, &ub)) return;
    if (item >= a.meta[0]) return;
    const PItem it = a.items[item];
    if (it.slot < 0 || it.slot >= a.n_slots_total) return;  // the down kernel writes the zeros and raises the flag
    const int H = a.H, I = a.I;
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wv = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int lrow = lane & 15, lgrp = lane >> 4;
    const int ug = wv & 3, tq = wv >> 2;  // unit group, token quarter
    const bool live = tq * 64 < it.ntok;  // a quarter past the item's tokens only helps staging
    const uint16_t* wslot = a.pool + (size_t)it.slot * a.slot_elems;
    const int u_wg = ub * kGuUnits;

    if (tid < TM) s_gate[tid] = tid < it.ntok ? (it.first_tok >= 0 ? 1.0f : a.pgate[it.list_off + tid]) : 0.f;
    constexpr int VPR = kGuKS / 8;                                // 16-byte vectors per row and slice
    constexpr int NX = TM * VPR / kMmThreads;                     // input vectors per thread and slice
    constexpr int NW = 2 * kGuUnits * VPR / kMmThreads;           // weight vectors per thread and slice
    const uint16_t* xsrc[NX];
#pragma unroll
    for (int j = 0; j < NX; ++j) {
        const int v = tid + kMmThreads * j, r = v / VPR;
        int tok = -1;
        if (r < it.ntok) tok = it.first_tok >= 0 ? it.first_tok + r : a.perm[it.list_off + r];
        xsrc[j] = tok >= 0 ? a.X + (size_t)tok * H + (v % VPR) * 8 : nullptr;
    }
    const uint16_t* wsrc[NW];
#pragma unroll
    for (int j = 0; j < NW; ++j) {
        const int v = tid + kMmThreads * j, rho = v / VPR;  // rho: 0..63 gate rows, 64..127 up rows
        const int u = min(u_wg + (rho & (kGuUnits - 1)), I - 1);  // rows past I are masked at the end
        wsrc[j] = wslot + (size_t)u * 3 * H + (rho >= kGuUnits ? H : 0) + (v % VPR) * 8;
    }
    const int n_slices = (H + kGuKS - 1) / kGuKS;
    uint4 xst[NX], wst[NW];
    auto fetch = [&](int s) {
#pragma unroll
        for (int j = 0; j < NW; ++j) {
            const int kk = s * kGuKS + ((tid + kMmThreads * j) % VPR) * 8;
            wst[j] = kk < H ? (it.once ? load_once_16(wsrc[j] + s * kGuKS) : *reinterpret_cast<const uint4*>(wsrc[j] + s * kGuKS))
                            : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int j = 0; j < NX; ++j) {
            const int kk = s * kGuKS + ((tid + kMmThreads * j) % VPR) * 8;
            xst[j] = (xsrc[j] && kk < H) ? *reinterpret_cast<const uint4*>(xsrc[j] + s * kGuKS) : make_uint4(0, 0, 0, 0);
        }
    };
    auto put = [&]() {
#pragma unroll
        for (int j = 0; j < NW; ++j) {
            const int v = tid + kMmThreads * j;
            *reinterpret_cast<uint4*>(Ws + swz(v / VPR, v % VPR)) = wst[j];
        }
#pragma unroll
        for (int j = 0; j < NX; ++j) {
            const int v = tid + kMmThreads * j;
            *reinterpret_cast<uint4*>(Xs + swz(v / VPR, v % VPR)) = xst[j];
        }
    };

    f32x4 G[4], U[4];
#pragma unroll
    for (int tb = 0; tb < 4; ++tb) G[tb] = U[tb] = f32x4{0.f, 0.f, 0.f, 0.f};
    // operand rows of this lane: 16 * block + lrow, so the swizzle key is lrow for every block
    const uint16_t* ag = Ws + (size_t)(16 * ug + lrow) * kTileK;
    const uint16_t* au = ag + (size_t)kGuUnits * kTileK;
    const uint16_t* xb = Xs + (size_t)(64 * tq + lrow) * kTileK;

    fetch(0);
    for (int s = 0; s < n_slices; ++s) {
        __syncthreads();  // the previous slice has been multiplied
        put();
        __syncthreads();
        if (s + 1 < n_slices) fetch(s + 1);  // on its way while this slice is multiplied
        const int steps = live ? min(kGuKS, H - s * kGuKS) / 32 : 0;
        for (int ks = 0; ks < steps; ++ks) {
            const int ko = ((ks * 4 + lgrp) ^ lrow) << 3;  // where this lane's 8 k-values of step ks sit in a row
            const bf16x8 cg = ld_bf16x8(ag + ko), cu = ld_bf16x8(au + ko);
#pragma unroll
            for (int tb = 0; tb < 4; ++tb) {
                const bf16x8 b = ld_bf16x8(xb + (size_t)tb * 16 * kTileK + ko);
                G[tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(cg, b, G[tb], 0, 0, 0);
                U[tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(cu, b, U[tb], 0, 0, 0);
            }
        }
    }
    // D[unit 4*lgrp + v][token lrow] -> activation, bf16, act[row][unit]
    const bool packed = (I & 3) == 0;
    const int u0 = u_wg + 16 * ug + lgrp * 4;
#pragma unroll
    for (int tb = 0; tb < 4; ++tb) {
        const int tok = tq * 64 + tb * 16 + lrow;
        if (tok >= it.ntok) continue;
        const float gw = s_gate[tok];
        uint16_t* dst_row = a.act + (size_t)(it.row0 + tok) * I;
        uint32_t h[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) h[v] = bf16_bits(silu_f(G[tb][v]) * U[tb][v] * gw);
        if (packed && u0 + 3 < I) {
            *reinterpret_cast<uint2*>(dst_row + u0) = make_uint2(h[0] | (h[1] << 16), h[2] | (h[3] << 16));
        } else {
#pragma unroll
            for (int v = 0; v < 4; ++v)
                if (u0 + v < I) dst_row[u0 + v] = (uint16_t)h[v];
        }
    }
}

// 3a, long prompts.  Above ~128 tokens per expert the layer is bound by how fast a compute unit can
// pull its operands in.  Measured on this part: 16-byte loads into registers deliver ~16 bytes per
// clock and CU even from L2 (9.5 TB/s over the chip, whatever the depth); loads that go from global
// memory straight into LDS ~3.5 times that, but by the cache line - a 64-byte piece of a line costs
// as much as the whole 128 bytes; a stream that misses L2 ~20 GB/s per CU with 64 KiB in flight.
// So this kernel gives every workgroup a weight stream of its own - 128 units (gate and up: 256
// rows) of one expert - and as many of the expert's tokens as the accumulators hold (256), and
// brings both operands in with loads straight into LDS, one cache line (64 k-values) of every row
// per stage.  The weights come from HBM and the inputs mostly from L2, and a wavefront's loads
// complete in order, so the two are loaded by different wavefronts into rings of their own:
// wavefronts 0..3 keep two stages of weight rows in flight (a ring of three), wavefronts 4..7 one
// stage of input rows (a ring of two); all unit blocks of an item run on one XCD, so the item's
// input rows pass through that L2 once.  Chunk c of ring row r sits at chunk position
// c ^ ((r >> 1) % 8): the sixteen lanes that read one operand (sixteen consecutive rows, the same
// chunk) then touch all 64 banks once.  A wavefront owns 32 units (two 16-row blocks of gate, two of
// up) x 128 tokens (the even or the odd 16-token blocks of the item, so that a partly filled item
// leaves both halves of the workgroup the same work; blocks without tokens are neither read nor
// multiplied), 32 accumulator tiles, and multiplies a stage in two halves of 32 k-values.
constexpr int kTileTokWide = 256;
constexpr int kWdUnits = 128;   // intermediate units per workgroup
constexpr int kWdKS = 64;       // k-values per stage: 128 bytes of a row
constexpr int kWdStagesW = 3;   // ring of weight stages
constexpr int kWdStagesX = 2;   // ring of input stages
constexpr int kWdThreads = 512;
constexpr int kWdStageElems = 256 * kWdKS;  // a stage of either ring: 256 rows
__device__ __forceinline__ int wd_pos(int row, int chunk) { return row * kWdKS + ((chunk ^ ((row >> 1) & 7)) << 3); }

// waits until at most `stages` * 8 of this wavefront's vector memory operations are outstanding
__device__ __forceinline__ void wait_but_stages(int stages) {
    // s_waitcnt: vmcnt in bits 3:0 and 15:14, expcnt 6:4 and lgkmcnt 11:8 left at their maxima
    if (stages >= 2)
        __builtin_amdgcn_s_waitcnt(0x4f70);  // 16
    else if (stages == 1)
        __builtin_amdgcn_s_waitcnt(0x0f78);  // 8
    else
        __builtin_amdgcn_s_waitcnt(0x0f70);
}

__global__ void __launch_bounds__(kWdThreads, 2) prefill_gateup_wide_kernel(MmArgs a) {
    constexpr int TM = kTileTokWide;
    constexpr int NLD = 8;        // loads per wavefront and stage, 8 rows each: four wavefronts fill 256 rows
    constexpr int NTB = TM / 32;  // 16-token blocks per wavefront: 8
    static_assert(2 * kWdUnits == 256 && TM == 256 && kWdThreads == 8 * kWave && kWdKS == 64, "four wavefronts load 256 rows of 128 bytes");
    extern __shared__ __align__(16) unsigned char smem_raw[];
    uint16_t* ring_w = reinterpret_cast<uint16_t*>(smem_raw);        // [kWdStagesW][256][64]
    uint16_t* ring_x = ring_w + (size_t)kWdStagesW * kWdStageElems;  // [kWdStagesX][256][64]
    int item, ub;
    if (!xcd_item_work(a.n_ub, &item, &ub)) return;
    if (item >= a.meta[0]) return;
    const PItem it = a.items[item];
    if (it.slot < 0 || it.slot >= a.n_slots_total) return;  // the down kernel writes the zeros and raises the flag
    const int H = a.H, I = a.I;
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wv = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int lrow = lane & 15, lgrp = lane >> 4;
    const int rg = wv & 3, th = wv >> 2;  // unit group (32 units); the even or the odd 16-token blocks
    // 16-token blocks of this wavefront that hold tokens of the item (blocks th, th + 2, ...)
    const int n_live = max(0, ((it.ntok + 15) / 16 - th + 1) / 2);
    const bool loads_w = wv < 4;  // else the inputs
    const uint16_t* wslot = a.pool + (size_t)it.slot * a.slot_elems;
    const int u_wg = ub * kWdUnits;

    // load j of this wavefront fills rows 8 * (4 * j + wv % 4) .. + 8 of a stage of its ring; this
    // lane brings chunk position lane % 8 of row .. + lane / 8.  Weight rows 0..127 are gate rows,
    // 128..255 up rows.  Units past I repeat unit I - 1 and tokens past the item repeat its first
    // token: what they yield is never stored.
    const uint16_t* src[NLD];
#pragma unroll
    for (int j = 0; j < NLD; ++j) {
        const int r = 8 * (4 * j + (wv & 3)) + (lane >> 3);
        const int c = (lane & 7) ^ ((r >> 1) & 7);
        if (loads_w) {
            const int u = min(u_wg + (r & (kWdUnits - 1)), I - 1);
            src[j] = wslot + (size_t)u * 3 * H + (r >= kWdUnits ? H : 0) + c * 8;
        } else {
            const int t = r < it.ntok ? r : 0;
            const int tok = it.first_tok >= 0 ? it.first_tok + t : a.perm[it.list_off + t];
            src[j] = a.X + (size_t)tok * H + c * 8;
        }
    }
    const int depth = loads_w ? kWdStagesW : kWdStagesX;  // uniform over the wavefront
    const uint32_t my_ring = lds_address(loads_w ? ring_w : ring_x) + (uint32_t)(8 * (wv & 3)) * (kWdKS * 2);
    // input rows past the item's tokens are not loaded (what the ring holds there is multiplied at most
    // within a token block that also holds tokens, and never stored): this wavefront's loads j < n_ld
    const int n_ld = loads_w ? NLD : min(NLD, max(0, (it.ntok - 8 * (wv & 3) + 31) / 32));
    auto issue = [&](int s) {
        const uint32_t st = my_ring + (uint32_t)(s % depth) * (kWdStageElems * 2);
#pragma unroll
        for (int j = 0; j < NLD; ++j)
            if (j < n_ld) load16_to_lds(src[j] + (size_t)s * kWdKS, st + (uint32_t)(32 * j) * (kWdKS * 2));
    };

    f32x4 G[2][NTB], U[2][NTB];
#pragma unroll
    for (int bl = 0; bl < 2; ++bl)
#pragma unroll
        for (int tb = 0; tb < NTB; ++tb) G[bl][tb] = U[bl][tb] = f32x4{0.f, 0.f, 0.f, 0.f};

    // The operands of a half stage are read into registers one half step before they are multiplied,
    // so the LDS reads of half step t + 1 run beside the matrix instructions of half step t, and a
    // ring slot is free again as soon as every wavefront has read both its halves.
    struct Ops {
        bf16x8 ag[2], au[2], b[NTB];
    };
    // NT: token blocks of this wavefront that are read and multiplied (the live ones, rounded up to even)
    auto read_ops = [&](int t, Ops& o, auto nt_tag) {  // half step t: stage t / 2, chunks 4 * (t % 2) .. + 4
        constexpr int NT = decltype(nt_tag)::value;
        const int s = t >> 1, c = 4 * (t & 1) + lgrp;
        const uint16_t* sw = ring_w + (size_t)(s % kWdStagesW) * kWdStageElems;
        const uint16_t* sx = ring_x + (size_t)(s % kWdStagesX) * kWdStageElems;
#pragma unroll
        for (int bl = 0; bl < 2; ++bl) {
            const int r = 32 * rg + 16 * bl + lrow;
            o.ag[bl] = ld_bf16x8(sw + wd_pos(r, c));
            o.au[bl] = ld_bf16x8(sw + wd_pos(kWdUnits + r, c));
        }
#pragma unroll
        for (int tb = 0; tb < NT; ++tb) o.b[tb] = ld_bf16x8(sx + wd_pos((2 * tb + th) * 16 + lrow, c));
    };
    auto multiply = [&](const Ops& o, auto nt_tag) {
        constexpr int NT = decltype(nt_tag)::value;
#pragma unroll
        for (int tb = 0; tb < NT; ++tb)
#pragma unroll
            for (int bl = 0; bl < 2; ++bl) {
                G[bl][tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(o.ag[bl], o.b[tb], G[bl][tb], 0, 0, 0);
                U[bl][tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(o.au[bl], o.b[tb], U[bl][tb], 0, 0, 0);
            }
    };
    const int n_slices = H / kWdKS;   // H is a multiple of 128: at least two stages
    const int n_half = 2 * n_slices;  // at least four half steps, an even number
    for (int s = 0; s < depth; ++s)
        if (s < n_slices) issue(s);
    static_assert(kWdStagesX == 2, "the wavefronts that load inputs wait for all their loads: their count per stage varies");
    if (loads_w)
        wait_but_stages(min(n_slices, depth) - 1);  // stage 0 has landed
    else if (n_ld > 0)
        wait_but_stages(0);  // (stage 1's loads with it)
    __syncthreads();
    // Half step t multiplies half t and reads half t + 1.  When that is the first half of stage s + 1
    // (t odd), the stage has landed for all once the wavefronts that load have seen their loads of it
    // complete and the barrier is passed; by then every wavefront has read both halves of stage s,
    // whose ring slots take stages s + 3 (weights) and s + 2 (inputs).  The loop is written once for
    // each count of token blocks a wavefront may have, and its last half step is peeled, so that no
    // path through a half step skips its reads.
    auto run = [&](auto nt_tag) {
        constexpr int NT = decltype(nt_tag)::value;
        Ops opA, opB;
        if constexpr (NT > 0) read_ops(0, opA, nt_tag);
        auto half = [&](int t, const Ops& cur, Ops& nxt, bool enters_stage) {
            if (enters_stage) {
                const int s = t >> 1;
                wait_but_stages(loads_w ? min(n_slices - 2 - s, depth - 2) : 0);  // stages younger than s + 1 that have been issued
                __syncthreads();
                if (s + depth < n_slices) issue(s + depth);
            }
            if constexpr (NT > 0) {
                read_ops(t + 1, nxt, nt_tag);
                multiply(cur, nt_tag);
            }
        };
        for (int t = 0; t + 2 < n_half; t += 2) {
            half(t, opA, opB, false);
            half(t + 1, opB, opA, true);
        }
        half(n_half - 2, opA, opB, false);
        if constexpr (NT > 0) multiply(opB, nt_tag);
    };
    switch ((n_live + 1) / 2) {  // uniform over the wavefront
        case 0: run(std::integral_constant<int, 0>{}); break;
        case 1: run(std::integral_constant<int, 2>{}); break;
        case 2: run(std::integral_constant<int, 4>{}); break;
        case 3: run(std::integral_constant<int, 6>{}); break;
        default: run(std::integral_constant<int, 8>{}); break;
    }
    // D[unit 4*lgrp + v][token lrow] -> activation, bf16, act[row][unit]
    const bool packed = (I & 3) == 0;
#pragma unroll
    for (int tb = 0; tb < NTB; ++tb) {
        const int tok = (2 * tb + th) * 16 + lrow;
        if (tok >= it.ntok) continue;
        const float gw = it.first_tok >= 0 ? 1.0f : a.pgate[it.list_off + tok];
        uint16_t* dst_row = a.act + (size_t)(it.row0 + tok) * I;
#pragma unroll
        for (int bl = 0; bl < 2; ++bl) {
            const int u0 = u_wg + 32 * rg + 16 * bl + lgrp * 4;
            uint32_t h[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) h[v] = bf16_bits(silu_f(G[bl][tb][v]) * U[bl][tb][v] * gw);
            if (packed && u0 + 3 < I) {
                *reinterpret_cast<uint2*>(dst_row + u0) = make_uint2(h[0] | (h[1] << 16), h[2] | (h[3] << 16));
            } else {
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    if (u0 + v < I) dst_row[u0 + v] = (uint16_t)h[v];
            }
        }
    }
}

// 3b.  grid (ceil(H / 512), items).  D = A B with A = 16 tokens x 32 units from LDS, B = 32 units x
// 16 columns of W_down.  The slot stores W_down unit-major, so a lane loads eight units x eight
// columns and transposes them in registers into eight operands of eight units each; the column
// a lane serves in matrix i is then col0 + 8*lrow + i (which 16 columns a matrix covers is only
// a labelling).  A wavefront owns 64 tokens x 128 columns.
template <int TM>
__global__ void __launch_bounds__(TM * 4, 2) prefill_down_kernel(MmArgs a) {  // two wavefronts per SIMD: 256 registers
    constexpr int kMmThreads = TM * 4;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    uint16_t* As = reinterpret_cast<uint16_t*>(smem_raw);  // [2][TM][128], chunks swizzled
    const int item = blockIdx.y / a.dn_split, part = blockIdx.y % a.dn_split;
    if (item >= a.meta[0]) return;
    PItem it = a.items[item];
    it.row0 += part * TM;  // this workgroup's TM tokens of the item
    it.ntok = min(TM, it.ntok - part * TM);
    if (it.ntok <= 0) return;
    const int H = a.H, I = a.I;
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wv = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int lrow = lane & 15, lgrp = lane >> 4;
    const int cg = wv & 3, tq = wv >> 2;  // column group, token quarter
    const int col0 = blockIdx.x * kDnCols + 128 * cg;
    // uniform over the wavefront: its columns exist and its quarter holds tokens of the item
    const bool active = col0 < H && tq * 64 < it.ntok;
    if (it.slot < 0 || it.slot >= a.n_slots_total) {  // not resident: the rows are zero, the flag says so
        if (tid == 0) atomicOr(a.flags, 1);
        const int c_end = min(H, (int)(blockIdx.x + 1) * kDnCols);
        for (int r = 0; r < it.ntok; ++r)
            for (int c = blockIdx.x * kDnCols + tid; c < c_end; c += kMmThreads) a.yc[(size_t)(it.row0 + r) * H + c] = 0.f;
        return;
    }
    const uint16_t* wd = a.pool + (size_t)it.slot * a.slot_elems + 2 * H + (col0 < H ? col0 : 0) + lrow * 8;

    constexpr int VPR = kDnKS / 8;             // 16
    constexpr int NV = TM * VPR / kMmThreads;  // 4
    // staging vector j of this thread: activation row tid / 16 + RPJ * j, chunk tid % 16 of the slice
    constexpr int RPJ = kMmThreads / VPR;
    const int srow = tid / VPR, schunk = tid % VPR;
    const uint16_t* abase = a.act + (size_t)(it.row0 + srow) * I + schunk * 8;
    const int n_slices = (I + kDnKS - 1) / kDnKS;
    uint4 stage[NV];
    auto fetch = [&](int s) {
        const bool in_k = s * kDnKS + schunk * 8 < I;
#pragma unroll
        for (int j = 0; j < NV; ++j)
            stage[j] = (in_k && srow + RPJ * j < it.ntok)
                           ? *reinterpret_cast<const uint4*>(abase + (size_t)RPJ * j * I + s * kDnKS)
                           : make_uint4(0, 0, 0, 0);
    };
    // RPJ is a multiple of 16: every staging vector of the thread has the swizzle key srow % 16
    auto put = [&](int buf) {
        uint16_t* dst = As + (size_t)buf * TM * kTileK + swz(srow, schunk);
#pragma unroll
        for (int j = 0; j < NV; ++j) *reinterpret_cast<uint4*>(dst + (size_t)RPJ * j * kTileK) = stage[j];
    };
    auto load_w = [&](int k0, uint4* dst) {  // units k0 + 8*lgrp + j (clamped: their activations are zero)
#pragma unroll
        for (int j = 0; j < 8; ++j)
            dst[j] = it.once ? load_once_16(wd + (size_t)min(k0 + lgrp * 8 + j, I - 1) * 3 * H)
                            : *reinterpret_cast<const uint4*>(wd + (size_t)min(k0 + lgrp * 8 + j, I - 1) * 3 * H);
    };

    f32x4 Y[4][8];
#pragma unroll
    for (int tb = 0; tb < 4; ++tb)
#pragma unroll
        for (int i = 0; i < 8; ++i) Y[tb][i] = f32x4{0.f, 0.f, 0.f, 0.f};

    fetch(0);
    put(0);
    __syncthreads();
    uint4 cur[8], nxt[8];
    if (active) load_w(0, cur);
    for (int s = 0; s < n_slices; ++s) {
        if (s + 1 < n_slices) fetch(s + 1);
        const uint16_t* ab = As + ((size_t)(s & 1) * TM + 64 * tq + lrow) * kTileK;
        const int k0 = s * kDnKS;
        const int steps = active ? (min(kDnKS, I - k0) + 31) / 32 : 0;
#pragma unroll 1
        for (int ks = 0; ks < steps; ++ks) {
            // the next step's weights (the next slice's first step after the last one; past the
            // end an in-bounds dummy)
            int kn = k0 + (ks + 1) * 32;
            if (kn >= I) kn = 0;
            load_w(kn, nxt);
            bf16x8 av[4];
#pragma unroll
            for (int tb = 0; tb < 4; ++tb)
                av[tb] = ld_bf16x8(ab + (size_t)tb * 16 * kTileK + (((ks * 4 + lgrp) ^ lrow) << 3));
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                uint32_t dw[4];
#pragma unroll
                for (int p = 0; p < 4; ++p) {
                    const uint32_t lo = reinterpret_cast<const uint32_t*>(&cur[2 * p])[i >> 1];
                    const uint32_t hi = reinterpret_cast<const uint32_t*>(&cur[2 * p + 1])[i >> 1];
                    dw[p] = (i & 1) ? __builtin_amdgcn_perm(hi, lo, 0x07060302u) : __builtin_amdgcn_perm(hi, lo, 0x05040100u);
                }
                bf16x8 wt;
                memcpy(&wt, dw, 16);
#pragma unroll
                for (int tb = 0; tb < 4; ++tb)
                    Y[tb][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[tb], wt, Y[tb][i], 0, 0, 0);
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) cur[j] = nxt[j];
        }
        if (s + 1 < n_slices) put((s + 1) & 1);
        __syncthreads();
    }
    if (!active) return;
    // D[token 4*lgrp + v][column lrow] of matrix i is column col0 + 8*lrow + i
#pragma unroll
    for (int tb = 0; tb < 4; ++tb)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int tok = tq * 64 + tb * 16 + lgrp * 4 + v;
            if (tok < it.ntok) {
                float* dst = a.yc + (size_t)(it.row0 + tok) * H + col0 + lrow * 8;
                *reinterpret_cast<float4*>(dst) = make_float4(Y[tb][0][v], Y[tb][1][v], Y[tb][2][v], Y[tb][3][v]);
                *reinterpret_cast<float4*>(dst + 4) = make_float4(Y[tb][4][v], Y[tb][5][v], Y[tb][6][v], Y[tb][7][v]);
            }
        }
}

// 3b, long prompts: the down product for items of up to 256 tokens, built like the wide gate/up
// kernel.  A workgroup forms 256 tokens x 256 columns; its stream of W_down (64 units x 256 columns
// = 64 rows of 512 bytes per stage, ring of three) and the item's activations (256 rows of 128 bytes
// per stage, ring of two) go from global memory straight into LDS, loaded by wavefronts 0..3 and
// 4..7; all column blocks of an item run on one XCD.  (The kernel above loads W_down into registers,
// every token quarter again: at 256 tokens that path, ~16 bytes per clock and CU, is what bounds
// it.)  A wavefront owns four 16-token blocks (blocks q, q + 4, ... of the item for quarter q) x 128
// columns: 32 accumulator tiles, which leave registers for one set of W_down pieces (eight units x
// eight columns per lane, transposed in registers as above) and two of activations.  So the
// activations of a half stage are read one half step ahead and the W_down pieces at its start, and
// each ring has a barrier of its own: before the first half of a stage the wavefronts that load
// W_down have seen that stage land (after the barrier the stage before it has been read by all and
// its slot is loaded again), before the second half the same for the activations of the next stage.
// Needs I % 64 == 0 and H % 256 == 0; other shapes take the kernel above, an item in two parts.
constexpr int kDwCols = 256;
constexpr int kDwKS = 64;
constexpr int kDwStagesW = 3;
constexpr int kDwStagesA = 2;
constexpr int kDwStageElemsW = kDwKS * kDwCols;       // 64 rows of 256 columns: 32 KiB
constexpr int kDwStageElemsA = kTileTokWide * kDwKS;  // 256 rows of 64 units: 32 KiB
// waits until at most `n` of this wavefront's vector memory operations are outstanding (n <= 32)
__device__ __forceinline__ void wait_vm(int n) {
    // s_waitcnt: vmcnt in bits 3:0 and 15:14, expcnt 6:4 and lgkmcnt 11:8 left at their maxima
#define MOEI_WAIT_CASE(v) case v: __builtin_amdgcn_s_waitcnt(0x0f70 | ((v) & 15) | (((v) >> 4) << 14)); break;
    switch (n) {
        MOEI_WAIT_CASE(0) MOEI_WAIT_CASE(1) MOEI_WAIT_CASE(2) MOEI_WAIT_CASE(3) MOEI_WAIT_CASE(4) MOEI_WAIT_CASE(5)
        MOEI_WAIT_CASE(6) MOEI_WAIT_CASE(7) MOEI_WAIT_CASE(8) MOEI_WAIT_CASE(9) MOEI_WAIT_CASE(10) MOEI_WAIT_CASE(11)
        MOEI_WAIT_CASE(12) MOEI_WAIT_CASE(13) MOEI_WAIT_CASE(14) MOEI_WAIT_CASE(15) MOEI_WAIT_CASE(16) MOEI_WAIT_CASE(17)
        MOEI_WAIT_CASE(18) MOEI_WAIT_CASE(19) MOEI_WAIT_CASE(20) MOEI_WAIT_CASE(21) MOEI_WAIT_CASE(22) MOEI_WAIT_CASE(23)
        MOEI_WAIT_CASE(24) MOEI_WAIT_CASE(25) MOEI_WAIT_CASE(26) MOEI_WAIT_CASE(27) MOEI_WAIT_CASE(28) MOEI_WAIT_CASE(29)
        MOEI_WAIT_CASE(30) MOEI_WAIT_CASE(31)
        default: __builtin_amdgcn_s_waitcnt(0x8f70); break;  // 32
    }
#undef MOEI_WAIT_CASE
}

__global__ void __launch_bounds__(kWdThreads, 2) prefill_down_wide_kernel(MmArgs a) {
    extern __shared__ __align__(16) unsigned char smem_raw[];
    uint16_t* ring_w = reinterpret_cast<uint16_t*>(smem_raw);         // [kDwStagesW][64][256]
    uint16_t* ring_a = ring_w + (size_t)kDwStagesW * kDwStageElemsW;  // [kDwStagesA][256][64], chunks swizzled
    int item, cb;
    xcd_item_work(a.n_cb, &item, &cb);
    if (item >= a.meta[0]) return;
    const PItem it = a.items[item];
    const int H = a.H, I = a.I;
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wv = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int lrow = lane & 15, lgrp = lane >> 4;
    const int cg = wv & 1, tq = wv >> 1;  // column group (128 columns), token quarter
    const int col_wg = cb * kDwCols;
    if (it.slot < 0 || it.slot >= a.n_slots_total) {  // not resident: the rows are zero, the flag says so
        if (tid == 0) atomicOr(a.flags, 1);
        for (int r = 0; r < it.ntok; ++r)
            for (int c = tid; c < kDwCols; c += kWdThreads) a.yc[(size_t)(it.row0 + r) * H + col_wg + c] = 0.f;
        return;
    }
    // 16-token blocks of this wavefront that hold tokens of the item (blocks tq, tq + 4, ...)
    const int n_live = max(0, ((it.ntok + 15) / 16 - tq + 3) / 4);
    const bool loads_w = wv < 4;  // else the activations
    const uint16_t* wd = a.pool + (size_t)it.slot * a.slot_elems + 2 * H + col_wg;

    // Weights: load j (of 8) of wavefront w fills rows 2 * (4 * j + w) .. + 2 of a stage (a row = 256
    // columns = 32 pieces); this lane brings piece lane % 32 of row .. + lane / 32.  Activations: load
    // j (of at most 8) fills rows 8 * (4 * j + w) .. + 8 (a row = 64 units = 8 pieces), chunk position
    // lane % 8 of row .. + lane / 8; rows past the item's tokens are not loaded (what the ring holds
    // there is multiplied at most within a token block that also holds tokens, never stored).  One
    // source address per lane; the loads of a stage lie a fixed number of rows apart.
    const uint16_t* src0;
    const int arow = 8 * (wv & 3) + (lane >> 3);  // this lane's row of an activation load, before 32 * j
    if (loads_w) {
        const int r = 2 * (wv & 3) + (lane >> 5);
        src0 = wd + (size_t)r * 3 * H + (lane & 31) * 8;
    } else {
        const int c = (lane & 7) ^ ((arow >> 1) & 7);  // rows 32 apart share the swizzle key
        src0 = a.act + (size_t)it.row0 * I + c * 8;
    }
    const int nld = loads_w ? 8 : min(8, max(0, (it.ntok - 8 * (wv & 3) + 31) / 32));  // loads per stage of this wavefront
    const uint32_t my_ring = lds_address(loads_w ? ring_w : ring_a) + (uint32_t)(wv & 3) * 1024;
    auto issue = [&](int s) {  // the calling wavefront's share of stage s of its ring
        if (loads_w) {
            const uint32_t st = my_ring + (uint32_t)(s % kDwStagesW) * (kDwStageElemsW * 2);
            const uint16_t* p = src0 + (size_t)s * kDwKS * 3 * H;
#pragma unroll
            for (int j = 0; j < 8; ++j) load16_to_lds(p + (size_t)j * 8 * 3 * H, st + (uint32_t)j * 4096);
        } else {
            const uint32_t st = my_ring + (uint32_t)(s % kDwStagesA) * (kDwStageElemsA * 2);
            const uint16_t* p = src0 + s * kDwKS;
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (j < nld) load16_to_lds(p + (uint32_t)min(arow + 32 * j, it.ntok - 1) * (uint32_t)I, st + (uint32_t)j * 4096);
        }
    };

    f32x4 Y[4][8];
#pragma unroll
    for (int tb = 0; tb < 4; ++tb)
#pragma unroll
        for (int i = 0; i < 8; ++i) Y[tb][i] = f32x4{0.f, 0.f, 0.f, 0.f};

    struct Acts {
        bf16x8 av[4];  // the token blocks' activations of a half stage
    };
    auto read_acts = [&](int t, Acts& o, auto nt_tag) {  // half step t: stage t / 2, units 32 * (t % 2) .. + 32
        constexpr int NT = decltype(nt_tag)::value;
        const uint16_t* sa = ring_a + (size_t)((t >> 1) % kDwStagesA) * kDwStageElemsA;
#pragma unroll
        for (int tb = 0; tb < NT; ++tb) o.av[tb] = ld_bf16x8(sa + wd_pos((4 * tb + tq) * 16 + lrow, 4 * (t & 1) + lgrp));
    };
    auto multiply = [&](int t, const Acts& o, auto nt_tag) {
        constexpr int NT = decltype(nt_tag)::value;
        const uint16_t* sw = ring_w + (size_t)((t >> 1) % kDwStagesW) * kDwStageElemsW;
        uint4 w[8];  // units 8 * lgrp + j of the half stage, columns 8 * lrow .. + 8 of the wavefront's 128
#pragma unroll
        for (int j = 0; j < 8; ++j)
            w[j] = *reinterpret_cast<const uint4*>(sw + (size_t)(32 * (t & 1) + 8 * lgrp + j) * kDwCols + cg * 128 + lrow * 8);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            uint32_t dw[4];
#pragma unroll
            for (int p2 = 0; p2 < 4; ++p2) {
                const uint32_t lo = reinterpret_cast<const uint32_t*>(&w[2 * p2])[i >> 1];
                const uint32_t hi = reinterpret_cast<const uint32_t*>(&w[2 * p2 + 1])[i >> 1];
                dw[p2] = (i & 1) ? __builtin_amdgcn_perm(hi, lo, 0x07060302u) : __builtin_amdgcn_perm(hi, lo, 0x05040100u);
            }
            bf16x8 wt;
            memcpy(&wt, dw, 16);
#pragma unroll
            for (int tb = 0; tb < NT; ++tb) Y[tb][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(o.av[tb], wt, Y[tb][i], 0, 0, 0);
        }
    };
    const int n_slices = I / kDwKS;  // I is a multiple of 64 here
    // both rings start full; stage 0 of both has landed for all after the first barrier
    if (loads_w) {
        for (int s = 0; s < kDwStagesW; ++s)
            if (s < n_slices) issue(s);
        wait_vm((min(n_slices, kDwStagesW) - 1) * 8);
    } else {
        for (int s = 0; s < kDwStagesA; ++s)
            if (s < n_slices) issue(s);
        wait_vm((min(n_slices, kDwStagesA) - 1) * nld);
    }
    __syncthreads();
    auto run = [&](auto nt_tag) {
        constexpr int NT = decltype(nt_tag)::value;
        Acts actA, actB;
        if constexpr (NT > 0) read_acts(0, actA, nt_tag);
        for (int s = 0; s < n_slices; ++s) {
            // first half of stage s: its W_down rows have landed (stages 0 .. s + 1 have been issued);
            // stage s - 1 has been read by all, its slot takes stage s + 2
            if (s >= 1) {
                if (loads_w) wait_vm(min(n_slices - 1 - s, 1) * 8);
                __syncthreads();
                if (loads_w && s + 2 < n_slices) issue(s + 2);
            }
            if constexpr (NT > 0) {
                read_acts(2 * s + 1, actB, nt_tag);
                multiply(2 * s, actA, nt_tag);
            }
            // second half: the activations of stage s + 1 (read during this half step) have landed; those of
            // stage s have been read by all, their slot takes stage s + 2
            if (s + 1 < n_slices) {
                if (!loads_w) wait_vm(0);
                __syncthreads();
                if (!loads_w && s + 2 < n_slices) issue(s + 2);
                if constexpr (NT > 0) read_acts(2 * s + 2, actA, nt_tag);
            }
            if constexpr (NT > 0) multiply(2 * s + 1, actB, nt_tag);
        }
    };
    switch ((n_live + 1) / 2) {  // uniform over the wavefront
        case 0: run(std::integral_constant<int, 0>{}); break;
        case 1: run(std::integral_constant<int, 2>{}); break;
        default: run(std::integral_constant<int, 4>{}); break;
    }
    // D[token 4*lgrp + v][column lrow] of matrix i is column col0 + 8*lrow + i
    const int col0 = col_wg + cg * 128;
#pragma unroll
    for (int tb = 0; tb < 4; ++tb)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int tok = (4 * tb + tq) * 16 + lgrp * 4 + v;
            if (tok < it.ntok) {
                float* dst = a.yc + (size_t)(it.row0 + tok) * H + col0 + lrow * 8;
                *reinterpret_cast<float4*>(dst) = make_float4(Y[tb][0][v], Y[tb][1][v], Y[tb][2][v], Y[tb][3][v]);
                *reinterpret_cast<float4*>(dst + 4) = make_float4(Y[tb][4][v], Y[tb][5][v], Y[tb][6][v], Y[tb][7][v]);
            }
        }
}

// ------------------------------------------------------------------ 4. y[t] = sum of the token's rows, in pick order
// grid n, one workgroup per token: the k picks' rows, then the shared experts' rows.
__global__ void __launch_bounds__(256) prefill_reduce_kernel(const float* __restrict__ yc,
                                                             const int32_t* __restrict__ where, int n, int k,
                                                             int n_shared, int H, float* __restrict__ y) {
    __shared__ int s_rows[kWave + kWave];
    const int t = blockIdx.x;
    const int nc = k + n_shared;
    if ((int)threadIdx.x < nc)
        s_rows[threadIdx.x] = (int)threadIdx.x < k ? where[(size_t)t * k + threadIdx.x] : n * k + ((int)threadIdx.x - k) * n + t;
    __syncthreads();
    for (int c = threadIdx.x; c < H / 4; c += 256) {
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int j = 0; j < nc; ++j) {
            if (s_rows[j] < 0) continue;  // a pick that was never placed (token without picks)
            const float4 v = *reinterpret_cast<const float4*>(yc + (size_t)s_rows[j] * H + c * 4);
            acc.x += v.x;
            acc.y += v.y;
            acc.z += v.z;
            acc.w += v.w;
        }
        *reinterpret_cast<float4*>(y + (size_t)t * H + c * 4) = acc;
    }
}

// 1, long prompts.  The routing kernel of short prompts spends its time on the multiply-adds of the
// logits (n x E x H of them on the vector ALUs: 46 us at 2,048 tokens).  Here they run on the matrix
// cores.  grid ceil(n / 16), eight wavefronts: a workgroup forms the logits of 16 tokens,
// D = A B with A = 16 router rows x 32 k and B = 32 k x 16 tokens.  Both operands pass through LDS
// with loads that go straight there (a compute unit takes in 16-byte register loads at a quarter of
// that rate, and the workgroup reads the whole router matrix): a stage holds 64 k-values (one cache
// line) of the 16 token rows and of every router row, laid out like a stage of the wide matrix
// kernels above, in a ring as deep as LDS allows; every wavefront loads its share of a stage's rows.
// Wavefront w multiplies the k-values 32 * (w / 4) .. + 32 of each stage for the 16-expert blocks
// w % 4, w % 4 + 4, ... (E <= 256: at most four), so each logit is formed as two partial sums, which
// are added in a fixed order with the bias once the ring is done and its LDS is free.  Then
// wavefront w takes the top-k of tokens w and w + 8 with the code of the kernel for short prompts.
// A logit's sum runs over k in the matrix instruction's order, not the decode routing's: the two
// agree to rounding, not bit for bit.
// A step of the loop is two LDS reads and one matrix instruction per block, so what the loop costs
// is its control: the count a wavefront waits for is a compile-time constant (the loop is written
// once per number of loads a wavefront has per stage, its last steps unrolled), and ring slots are
// counted, not divided.
constexpr int kRtTok = 16;
constexpr int kRtMaxE = 256;
constexpr int kRtKS = 64;  // k-values per stage: 128 bytes of a row
constexpr int kRtThreads = 512;
constexpr int kRtWaves = kRtThreads / kWave;
// rows of a stage: the 16 tokens, then the experts, in groups of 8 rows (what one load instruction of a wavefront fills)
__host__ __device__ inline int rt_row_groups(int E) { return kRtTok / 8 + (E + 7) / 8; }
__host__ __device__ inline int rt_stage_elems(int E) { return rt_row_groups(E) * 8 * kRtKS; }
// Ring depth for NB blocks per wavefront (E <= 64 NB): what a workgroup has in flight bounds its
// rate, so the ring takes the LDS a workgroup may have (160 KiB less the 4 KiB of the picks).
__host__ __device__ constexpr int rt_depth(int nb) { return nb == 1 ? 15 : (nb == 2 ? 8 : (nb == 3 ? 6 : 4)); }
static_assert(rt_depth(1) * (2 + 8) * 8 * kRtKS * 2 <= 156 * 1024 && rt_depth(2) * (2 + 16) * 8 * kRtKS * 2 <= 156 * 1024 &&
                  rt_depth(3) * (2 + 24) * 8 * kRtKS * 2 <= 156 * 1024 && rt_depth(4) * (2 + 32) * 8 * kRtKS * 2 <= 156 * 1024,
              "the ring fits");
inline int rt_blocks_per_wave(int E) { return ((E + 15) / 16 + 3) / 4; }
inline size_t rt_lds_bytes(int E) { return (size_t)rt_depth(rt_blocks_per_wave(E)) * rt_stage_elems(E) * 2; }

// waits until at most N of this wavefront's vector memory operations are outstanding
template <int N>
__device__ __forceinline__ void wait_vm_c() {
    static_assert(N >= 0 && N < 64, "vmcnt has six bits");
    __builtin_amdgcn_s_waitcnt(0x0f70 | (N & 15) | ((N >> 4) << 14));
}
// f(R), f(R - 1), ..., f(0), each with its argument as a compile-time constant
template <int R, typename F>
__device__ __forceinline__ void count_down(F&& f) {
    if constexpr (R >= 0) {
        f(std::integral_constant<int, R>{});
        count_down<R - 1>(f);
    }
}

template <int NB>  // blocks of 16 experts per wavefront: ceil(ceil(E / 16) / 4)
__global__ void __launch_bounds__(kRtThreads) prefill_route_wide_kernel(const uint16_t* __restrict__ W,
                                                                        const float* __restrict__ bias,
                                                                        const uint16_t* __restrict__ X, int n, int H, int E,
                                                                        int k, int renorm, int32_t* __restrict__ idx,
                                                                        float* __restrict__ w, int32_t* __restrict__ where,
                                                                        int32_t* __restrict__ flags) {
    constexpr int NLD = NB + 1;  // loads per wavefront and stage: ceil((2 + 8 * NB) / 8) row groups at most
    constexpr int DEPTH = rt_depth(NB);
    extern __shared__ __align__(16) unsigned char smem_raw[];
    uint16_t* ring = reinterpret_cast<uint16_t*>(smem_raw);  // [DEPTH][8 * row groups][64], chunks swizzled
    float* zs = reinterpret_cast<float*>(smem_raw);          // afterwards: [2][16][E] partial logits
    __shared__ int s_idx[kRtWaves][kWave];
    __shared__ float s_w[kRtWaves][kWave];
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wv = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int lrow = lane & 15, lgrp = lane >> 4;
    const int eb = wv & 3, kh = wv >> 2;
    const int t0 = blockIdx.x * kRtTok;
    const int n_groups = rt_row_groups(E);
    const int stage_elems = rt_stage_elems(E);
    // load j of this wavefront fills row group wv + 8 * j of a stage; this lane brings chunk position
    // lane % 8 of the group's row lane / 8.  Tokens past n repeat the last token and experts past E
    // the last expert: what they yield is never stored.
    const uint16_t* src[NLD];
#pragma unroll
    for (int j = 0; j < NLD; ++j) {
        const int r = 8 * (wv + kRtWaves * j) + (lane >> 3);
        const int c = (lane & 7) ^ ((r >> 1) & 7);
        src[j] = (r < kRtTok ? X + (size_t)min(t0 + r, n - 1) * H : W + (size_t)min(r - kRtTok, E - 1) * H) + c * 8;
    }
    const int n_ld = max(0, (n_groups - wv + kRtWaves - 1) / kRtWaves);  // row groups of this wavefront: <= NLD
    const int n_slices = H / kRtKS;
    // Every workgroup reads the same router rows, and the pieces of one stage lie a whole row apart.
    // Workgroups that share an L2 (every eighth one) therefore start at different slices of k and
    // wrap around, so that at any moment they ask different parts of the cache for their lines.
    const int first_slice = (int)((blockIdx.x / kXcds) * 2u % (unsigned)n_slices);
    const uint32_t my_ring = lds_address(ring) + (uint32_t)(8 * wv) * (kRtKS * 2);
    // the operand rows this lane reads in every stage (a block past the router's last row group reads
    // the last group instead: never stored)
    const int c_op = 4 * kh + lgrp;
    const int x_pos = wd_pos(lrow, c_op);
    int w_pos[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j) w_pos[j] = wd_pos(min(kRtTok + 16 * (eb + 4 * j) + lrow, 8 * n_groups - 1), c_op);
    f32x4 acc[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};

    auto run = [&](auto nld_tag) {
        constexpr int N = decltype(nld_tag)::value;  // this wavefront's loads per stage
        // stage s holds slice (first_slice + s) % n_slices and sits in ring slot s % DEPTH
        int issue_slice = first_slice, issue_slot = 0;
        auto issue = [&]() {
            const uint32_t st = my_ring + (uint32_t)issue_slot * (uint32_t)(stage_elems * 2);
#pragma unroll
            for (int j = 0; j < N; ++j)
                load16_to_lds(src[j] + (size_t)issue_slice * kRtKS, st + (uint32_t)(8 * kRtWaves * j) * (kRtKS * 2));
            if (++issue_slice == n_slices) issue_slice = 0;
            if (++issue_slot == DEPTH) issue_slot = 0;
        };
        int slot = 0;
        auto multiply = [&]() {
            const uint16_t* st = ring + (size_t)slot * stage_elems;
            const bf16x8 xb = ld_bf16x8(st + x_pos);
            bf16x8 wb[NB];
#pragma unroll
            for (int j = 0; j < NB; ++j) wb[j] = ld_bf16x8(st + w_pos[j]);
#pragma unroll
            for (int j = 0; j < NB; ++j) acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wb[j], xb, acc[j], 0, 0, 0);
            if (++slot == DEPTH) slot = 0;
        };
        for (int s = 0; s < DEPTH - 1; ++s)
            if (s < n_slices) issue();
        // Stage s has landed for all once every wavefront has seen its own loads of it complete and
        // the barrier is passed; by then every wavefront has multiplied stage s - 1, whose slot takes
        // stage s + DEPTH - 1.  While DEPTH - 2 younger stages are in flight the count to wait for is
        // (DEPTH - 2) N; the last steps, with R = DEPTH - 3 .. 0 younger stages, are unrolled.
        int s = 0;
        for (; s + DEPTH - 2 < n_slices; ++s) {
            wait_vm_c<(DEPTH - 2) * N>();
            __syncthreads();
            if (s + DEPTH - 1 < n_slices) issue();
            multiply();
        }
        count_down<DEPTH - 3>([&](auto r_tag) {
            constexpr int R = decltype(r_tag)::value;
            if (R < n_slices) {  // stage n_slices - 1 - R
                wait_vm_c<R * N>();
                __syncthreads();
                multiply();
            }
        });
    };
    switch (n_ld) {  // uniform over the wavefront
        case 0: run(std::integral_constant<int, 0>{}); break;
        case 1: run(std::integral_constant<int, 1>{}); break;
        case 2: run(std::integral_constant<int, NLD < 2 ? NLD : 2>{}); break;
        case 3: run(std::integral_constant<int, NLD < 3 ? NLD : 3>{}); break;
        case 4: run(std::integral_constant<int, NLD < 4 ? NLD : 4>{}); break;
        default: run(std::integral_constant<int, NLD>{}); break;
    }
    __syncthreads();  // the ring has been read: its LDS takes the partial logits
    // D[expert 4 * lgrp + v][token lrow]
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int e = 16 * (eb + 4 * j) + 4 * lgrp + v;
            if (e < E) zs[((size_t)kh * kRtTok + lrow) * E + e] = acc[j][v];
        }
    __syncthreads();
    for (int tt = wv; tt < kRtTok && t0 + tt < n; tt += kRtWaves) {  // uniform over the wavefront
        const int t = t0 + tt;
        float* z = zs + (size_t)tt * E;
        for (int e = lane; e < E; e += kWave) z[e] = (z[e] + z[(size_t)kRtTok * E + e]) + (bias ? bias[e] : 0.f);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();  // the logits are whole; the previous token's picks have been read
        int my_idx;
        float my_w;
        if (wave_logits_bad(z, E, lane)) {  // the token gets no picks and only its shared experts' output
            my_idx = -1;
            my_w = 0.f;
            if (lane == 0) atomicOr(flags, 4);
        } else {
            const float sel = wave_topk_rank(z, E, k, renorm, lane, s_idx[wv], s_w[wv], false);
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
            my_idx = lane < k ? s_idx[wv][lane] : -1;
            my_w = lane < k ? (renorm ? s_w[wv][lane] / sel : s_w[wv][lane]) : 0.f;
        }
        if (lane < k) {
            idx[(size_t)t * k + lane] = my_idx;
            w[(size_t)t * k + lane] = my_w;
            where[(size_t)t * k + lane] = -1;  // no contribution row yet: the grouping names one per placed pick
        }
    }
}

template <typename K>
int pf_allow_lds(K kernel, size_t bytes) {
    static const void* seen_fn[8];
    static size_t seen_bytes[8];
    static int n_seen = 0;
    if (bytes <= 64 * 1024) return MOEI_OK;
    const void* fn = reinterpret_cast<const void*>(kernel);
    for (int i = 0; i < n_seen; ++i)
        if (seen_fn[i] == fn && seen_bytes[i] >= bytes) return MOEI_OK;
    MOEI_HIP(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
    if (n_seen < 8) {
        seen_fn[n_seen] = fn;
        seen_bytes[n_seen++] = bytes;
    }
    return MOEI_OK;
}

}  // namespace

int prefill_check(const moei_model_desc& d) {
    if (d.wdtype != MOEI_WDTYPE_BF16) MOEI_FAIL(MOEI_EINVAL, "moe_prefill_layer: bf16 weights only");
    if (d.H % 128 != 0 || d.H > 4096)
        MOEI_FAIL(MOEI_ECAPACITY, "moe_prefill_layer: H = %d must be a multiple of 128 and at most 4096", d.H);
    if (d.I % 8 != 0) MOEI_FAIL(MOEI_ECAPACITY, "moe_prefill_layer: I = %d must be a multiple of 8", d.I);
    if (d.E > kPfMaxE) MOEI_FAIL(MOEI_ECAPACITY, "moe_prefill_layer: E = %d exceeds %d", d.E, kPfMaxE);
    return MOEI_OK;
}

size_t prefill_item_bytes() { return sizeof(PItem); }
namespace {
int max_items_for(const moei_model_desc& d, int n, int tm) {
    return (n * d.k + tm - 1) / tm + d.E + d.n_shared * ((n + tm - 1) / tm);
}
// tokens per item: the wide kernels' 256 once the average expert holds 48 tokens (measured on the
// 64-expert top-6 shape: 256 tokens 279 us per layer with 64-token items against 288 us, 512 tokens
// 330 against 325, 1,024 tokens 488 against 405)
int tile_tokens(const moei_model_desc& d, int n) {
    const char* v = getenv("MOEI_PREFILL_TILE");
    if (v && atoi(v) == kTileTok) return kTileTok;
    if (v && atoi(v) == kTileTokBig) return kTileTokBig;
    if (v && atoi(v) == kTileTokWide) return kTileTokWide;
    return (long)n * d.k >= (long)48 * d.E ? kTileTokWide : kTileTok;
}

template <int TM>
int launch_mm(const moei_model_desc& d, MmArgs a, int max_items, hipStream_t s) {
    const size_t dn_smem = (size_t)2 * TM * kTileK * 2;
    int rc = pf_allow_lds(prefill_down_kernel<TM>, dn_smem);
    if (rc) return rc;
    if (a.dn_split == 1) {
        const size_t gu_smem = (size_t)(TM + 2 * kGuUnits) * kTileK * 2;
        rc = pf_allow_lds(prefill_gateup_kernel<TM>, gu_smem);
        if (rc) return rc;
        a.n_ub = (d.I + kGuUnits - 1) / kGuUnits;
        const int gu_per = (a.n_ub + kXcds - 1) / kXcds;
        launch(K_PF_GATEUP, prefill_gateup_kernel<TM>, dim3(kXcds * gu_per * max_items), dim3(TM * 4), gu_smem, s, a);
    } else {  // items of the wide tile: TM is the down kernel's share of one
        const size_t gu_smem = (size_t)(kWdStagesW + kWdStagesX) * kWdStageElems * 2;
        rc = pf_allow_lds(prefill_gateup_wide_kernel, gu_smem);
        if (rc) return rc;
        a.n_ub = (d.I + kWdUnits - 1) / kWdUnits;
        const int item_rounds = (max_items + kXcds - 1) / kXcds;
        launch(K_PF_GATEUP, prefill_gateup_wide_kernel, dim3(kXcds * a.n_ub * item_rounds), dim3(kWdThreads), gu_smem, s, a);
    }
    MOEI_LAUNCH_CHECK();
    if (a.dn_split == 2 && d.I % kDwKS == 0 && d.H % kDwCols == 0) {
        const size_t dw_smem = (size_t)(kDwStagesW * kDwStageElemsW + kDwStagesA * kDwStageElemsA) * 2;
        rc = pf_allow_lds(prefill_down_wide_kernel, dw_smem);
        if (rc) return rc;
        a.n_cb = d.H / kDwCols;
        const int item_rounds = (max_items + kXcds - 1) / kXcds;
        launch(K_PF_DOWN, prefill_down_wide_kernel, dim3(kXcds * a.n_cb * item_rounds), dim3(kWdThreads), dw_smem, s, a);
        MOEI_LAUNCH_CHECK();
        return MOEI_OK;
    }
    launch(K_PF_DOWN, prefill_down_kernel<TM>, dim3((d.H + kDnCols - 1) / kDnCols, max_items * a.dn_split), dim3(TM * 4), dn_smem, s, a);
    MOEI_LAUNCH_CHECK();
    return MOEI_OK;
}
}  // namespace

// the scratch is sized for the small tile, which yields the most items
int prefill_max_items(const moei_model_desc& d, int n_max) { return max_items_for(d, n_max, kTileTok); }
size_t prefill_rows(const moei_model_desc& d, int n_max) { return (size_t)n_max * (d.k + d.n_shared); }

int launch_prefill(const moei_model_desc& d, const PrefillScratch& ps, const void* d_pool, size_t slot_elems,
                   int n_slots_total, const int32_t* d_slot_of_row, int shared_base, int32_t* d_eam_row,
                   const void* d_router_w, const float* d_router_bias, const void* d_X, int n, float* d_Y,
                   int32_t* d_flags, hipStream_t s) {
    int rc = prefill_check(d);
    if (rc) return rc;
    if (n > ps.n_max) MOEI_FAIL(MOEI_ECAPACITY, "moe_prefill_layer: n = %d exceeds the scratch for %d tokens", n, ps.n_max);
    if ((uintptr_t)d_X % 16 != 0 || (uintptr_t)d_pool % 16 != 0 || (slot_elems * 2) % 16 != 0 || (uintptr_t)d_Y % 16 != 0)
        MOEI_FAIL(MOEI_EINVAL, "moe_prefill_layer: buffers must be 16-byte aligned");
    const int vec_ok = (d.H % 8 == 0) && ((uintptr_t)d_router_w % 16 == 0);
    // long prompts: the logits on the matrix cores (that kernel takes 15 - 18 us whatever n; the kernel
    // with a workgroup per token takes 11 us at 256 tokens, 19 us at 512, 22 us at 1,024 and 46 us at 2,048)
    if (n >= 512 && d.E <= kRtMaxE && d.H % 128 == 0 && (uintptr_t)d_router_w % 16 == 0) {
        const int nbw = rt_blocks_per_wave(d.E);
        const dim3 rgrid((n + kRtTok - 1) / kRtTok), rblock(kRtThreads);
        const size_t rsmem = rt_lds_bytes(d.E);
        const uint16_t* rw = reinterpret_cast<const uint16_t*>(d_router_w);
        const uint16_t* rx = reinterpret_cast<const uint16_t*>(d_X);
        const int rn = (int)(d.renorm_topk != 0);
#define MOEI_ROUTE_CASE(NB_)                                                                                       \
    case NB_:                                                                                                      \
        rc = pf_allow_lds(prefill_route_wide_kernel<NB_>, rsmem);                                                  \
        if (rc) return rc;                                                                                         \
        launch(K_PF_ROUTE, prefill_route_wide_kernel<NB_>, rgrid, rblock, rsmem, s, rw, d_router_bias, rx, n, d.H, d.E, \
               d.k, rn, ps.d_idx, ps.d_w, ps.d_where, d_flags);                                                    \
        break;
        switch (nbw) {
            MOEI_ROUTE_CASE(1)
            MOEI_ROUTE_CASE(2)
            MOEI_ROUTE_CASE(3)
            default:
                MOEI_ROUTE_CASE(4)
        }
#undef MOEI_ROUTE_CASE
    } else {
        const size_t route_smem = ((size_t)d.H + (size_t)d.E) * sizeof(float);
        rc = pf_allow_lds(prefill_route_kernel<uint16_t>, route_smem);
        if (rc) return rc;
        launch(K_PF_ROUTE, prefill_route_kernel<uint16_t>, dim3(n), dim3(4 * kWave), route_smem, s, d_router_w,
               d_router_bias, d_X, n, d.H, d.E, d.k, (int)(d.renorm_topk != 0), vec_ok, ps.d_idx, ps.d_w, ps.d_where, d_flags);
    }
    MOEI_LAUNCH_CHECK();
    const int tm = tile_tokens(d, n);
    GroupArgsP g{ps.d_idx, ps.d_w, n, d.k, d.E, d.n_shared, tm, d_slot_of_row, shared_base, d_eam_row, ps.d_perm,
                 ps.d_pgate, ps.d_where, reinterpret_cast<PItem*>(ps.d_items), ps.d_meta, d_flags,
                 tm == kTileTokWide};
    launch(K_FFN_GROUP, prefill_group_kernel, dim3(d.E), dim3(kGrpThreads), (size_t)d.E * sizeof(int), s, g);
    MOEI_LAUNCH_CHECK();
    // the number of items is known on the device only: the grids cover the largest possible count
    const int max_items = max_items_for(d, n, tm);
    MmArgs a{reinterpret_cast<const uint16_t*>(d_pool), slot_elems, n_slots_total,
             reinterpret_cast<const PItem*>(ps.d_items), ps.d_meta, reinterpret_cast<const uint16_t*>(d_X), ps.d_perm,
             ps.d_pgate, ps.d_act, ps.d_yc, d.H, d.I, d_flags, 0, (d.H + kDnCols - 1) / kDnCols,
             tm == kTileTokWide ? 2 : 1};
    rc = tm == kTileTok ? launch_mm<kTileTok>(d, a, max_items, s) : launch_mm<kTileTokBig>(d, a, max_items, s);
    if (rc) return rc;
    launch(K_PF_REDUCE, prefill_reduce_kernel, dim3(n), dim3(256), 0, s, (const float*)ps.d_yc,
           (const int32_t*)ps.d_where, n, d.k, d.n_shared, d.H, d_Y);
    MOEI_LAUNCH_CHECK();
    return MOEI_OK;
}

}  // namespace moei
