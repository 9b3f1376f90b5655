// The prefill iteration of one MoE layer: all n prompt tokens pass the layer together.
//
// Sec. 4.3 of the paper: an iteration routes n tokens and every token adds its k picks to
// row l of the request's EAM.  Four launches:
//   1. prefill_route_kernel   router logits + softmax/top-k, one wavefront per token (the
//                             same summation order as the decode routing, so the same bits)
//   2. prefill_count_kernel / prefill_place_kernel
//                             histogram of the picks -> EAM row; tokens grouped per expert in
//                             ascending token order, cut into items of <= TM tokens
//   3. prefill_ffn_kernel     grouped SwiGLU expert FFN on the matrix cores: an item's tokens
//                             sit in LDS, the expert's weights stream past once per item
//   4. prefill_reduce_kernel  y[t] = sum of the token's partial rows, in pick order
// With tens of tokens per expert the layer is still bound by streaming the weights (one
// weight byte meets ~TM flops); the matrix cores only keep the arithmetic off the critical
// path.  v_mfma_f32_16x16x32_bf16: A is 16 x 32 (lane l holds row l%16, k = 8*(l/16)..+8),
// B is 32 x 16 (lane l holds column l%16, same k), D is 16 x 16 (lane l holds column l%16,
// rows 4*(l/16)..+4).
#include <string.h>

#include "kernels.hpp"
#include "topk.hpp"
#include "wtypes.hpp"

namespace moei {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kPfWaves = 8;
constexpr int kPfThreads = kPfWaves * kWave;
constexpr int kPfChunk = 16 * kPfWaves;  // intermediate units per chunk: 16 per wavefront
constexpr int kPfPad = 8;                // bf16 elements of padding per LDS row (bank spread)
constexpr int kPfMaxE = 2048;

struct PItem {
    int32_t slot;       // cache slot of the expert
    int32_t ntok;       // tokens of the item, <= TM
    int32_t list_off;   // routed: position of the item's first token in perm / pgate
    int32_t first_tok;  // shared expert: tokens first_tok .. first_tok + ntok - 1 with weight 1; else -1
};

// ------------------------------------------------------------------ 1. routing of n tokens
template <typename WT>
__global__ void __launch_bounds__(4 * kWave) prefill_route_kernel(const void* __restrict__ Wv,
                                                                  const float* __restrict__ bias,
                                                                  const void* __restrict__ Xv, int n, int H, int E, int k,
                                                                  int renorm, int vec_ok, int32_t* __restrict__ idx,
                                                                  float* __restrict__ w) {
    using V = WVec<WT>;
    extern __shared__ __align__(16) float smem[];
    __shared__ int s_idx[4][kWave];
    __shared__ float s_w[4][kWave];
    const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x / kWave;
    float* xs = smem + (size_t)wv * H;           // this wavefront's token, fp32
    float* z = smem + (size_t)4 * H + (size_t)wv * E;  // its logits
    const int t = blockIdx.x * 4 + wv;
    if (t >= n) return;  // uniform over the wavefront; no workgroup barrier below
    const WT* W = reinterpret_cast<const WT*>(Wv);
    const WT* x = reinterpret_cast<const WT*>(Xv) + (size_t)t * H;
    for (int c = lane; c < H; c += kWave) xs[c] = V::one(x + c);
    s_idx[wv][lane] = 0;  // NaN logits leave ranks unassigned: such picks then name expert 0
    s_w[wv][lane] = 0.f;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    // eight rows at a time, so that eight loads are in flight per round trip; every row's sum
    // runs over the chunks in ascending order, as in the decode routing
    constexpr int RB = 8;
    for (int e0 = 0; e0 < E; e0 += RB) {
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
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    int my_idx;
    float my_w;
    if (E <= kRankMaxE) {
        const float sel = wave_topk_rank(z, E, k, renorm, lane, s_idx[wv], s_w[wv], false);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        my_idx = lane < k ? s_idx[wv][lane] : -1;
        my_w = lane < k ? (renorm ? s_w[wv][lane] / sel : s_w[wv][lane]) : 0.f;
    } else {
        wave_topk(z, E, k, renorm, lane, my_idx, my_w);
    }
    if (lane < k) {
        idx[(size_t)t * k + lane] = my_idx;
        w[(size_t)t * k + lane] = my_w;
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
    int32_t* where;    // [n*k][2] (item, row) of every routed (token, pick)
    PItem* items;
    int32_t* meta;  // [0] = items in all, [1] = routed items
    int32_t* cntw;  // [E][4] tokens that pick the expert, per wavefront range of the grouping kernels
    int32_t* flags;
};

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

// 2a. grid E: how many tokens pick expert e, per wavefront range -> cntw[e][kGrpWaves]
__global__ void __launch_bounds__(kGrpThreads) prefill_count_kernel(GroupArgsP g) {
    const int e = blockIdx.x, lane = threadIdx.x & (kWave - 1), wv = threadIdx.x / kWave;
    const int span = group_span(g.n);
    int c = 0;
    for (int t0 = wv * span; t0 < min(g.n, (wv + 1) * span); t0 += kWave)
        c += __popcll(__ballot(pick_of(g, t0 + lane, e) >= 0));
    if (lane == 0) g.cntw[e * kGrpWaves + wv] = c;
}

// 2b. grid E: offsets by a prefix over the counts, EAM row update, placement in ascending
// token order, the expert's items; workgroup 0 also lists the shared experts' items.
__global__ void __launch_bounds__(kGrpThreads) prefill_place_kernel(GroupArgsP g) {
    __shared__ int s_red[3][kGrpWaves];
    const int e = blockIdx.x, tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    // tokens and items of the experts before this one, items of all experts
    int toks = 0, its = 0, its_all = 0;
    for (int f = tid; f < g.E; f += kGrpThreads) {
        int c = 0;
        for (int w = 0; w < kGrpWaves; ++w) c += g.cntw[f * kGrpWaves + w];
        const int ni = (c + g.TM - 1) / g.TM;
        if (f < e) {
            toks += c;
            its += ni;
        }
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
        const int cw = g.cntw[e * kGrpWaves + w];
        if (w < wv) before += cw;
        cnt += cw;
    }
    if (tid == 0) g.eam_row[e] += cnt;  // Sec. 4.3: the n tokens add n*k to row l
    const int span = group_span(g.n);
    int pos = before;
    for (int t0 = wv * span; t0 < min(g.n, (wv + 1) * span); t0 += kWave) {
        const int t = t0 + lane;
        const int j = pick_of(g, t, e);
        const unsigned long long mask = __ballot(j >= 0);
        if (j >= 0) {
            const int r = pos + __popcll(mask & ((1ull << lane) - 1ull));
            g.perm[off + r] = t;
            g.pgate[off + r] = g.w[(size_t)t * g.k + j];
            g.where[((size_t)t * g.k + j) * 2] = ioff + r / g.TM;
            g.where[((size_t)t * g.k + j) * 2 + 1] = r % g.TM;
        }
        pos += __popcll(mask);
    }
    const int slot = g.slot_of_row[e];
    if (cnt > 0 && slot < 0 && tid == 0) atomicOr(g.flags, 2);
    for (int it = tid; it * g.TM < cnt; it += kGrpThreads)
        g.items[ioff + it] = PItem{slot, min(g.TM, cnt - it * g.TM), off + it * g.TM, -1};
    if (e == 0) {
        const int tiles = (g.n + g.TM - 1) / g.TM;
        for (int q = tid; q < g.n_shared * tiles; q += kGrpThreads) {
            const int s = q / tiles, tile = q - s * tiles;
            g.items[n_routed + q] = PItem{g.shared_base + s, min(g.TM, g.n - tile * g.TM), 0, tile * g.TM};
        }
        if (tid == 0) {
            g.meta[0] = n_routed + g.n_shared * tiles;
            g.meta[1] = n_routed;
        }
    }
}

// ------------------------------------------------------------------ 3. grouped expert FFN on the matrix cores
struct PfArgs {
    const uint16_t* pool;
    size_t slot_elems;
    int n_slots_total;
    const PItem* items;
    const int32_t* meta;
    const uint16_t* X;  // [n][H] bf16
    const int32_t* perm;
    const float* pgate;
    float* part;  // [workgroups][seg_max][TM][H]
    int H, I, seg_max;
    int32_t* flags;
};

__device__ __forceinline__ bf16x8 ld_bf16x8(const uint16_t* p) { return *reinterpret_cast<const bf16x8*>(p); }

__device__ __forceinline__ float silu_f(float g) { return g / (1.0f + expf(-g)); }

// round-to-nearest-even fp32 -> bf16 bits (finite inputs)
__device__ __forceinline__ uint32_t bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

// The intermediate units of all items form one row space of n_items * I rows, split evenly
// into contiguous ranges, one per workgroup; a range is cut at item boundaries into
// segments.  Per segment: the item's tokens go to LDS (bf16, TM x H); per chunk of 128
// units, phase 1 forms gate and up pre-activations for 16 units per wavefront (K = H),
// the activations go to LDS as bf16 (TM x 128), phase 2 adds them times the down columns
// into the wavefront's share of y (128-column groups), which stays in registers until the
// segment ends.  TB = token blocks of 16 (TM = 16 TB), CGW = column groups per wavefront.
template <int TB, int CGW>
__global__ void __launch_bounds__(kPfThreads) prefill_ffn_kernel(PfArgs a) {
    constexpr int TM = 16 * TB;
    constexpr int PW = 4;  // k-steps of phase 1 in flight (2 loads each)
    extern __shared__ __align__(16) unsigned char smem_raw[];
    const int H = a.H, I = a.I;
    const int xs_stride = H + kPfPad;
    constexpr int act_stride = kPfChunk + kPfPad;
    uint16_t* Xs = reinterpret_cast<uint16_t*>(smem_raw);  // [TM][H + pad]
    uint16_t* Act = Xs + (size_t)TM * xs_stride;           // [TM][128 + pad]
    float* s_gate = reinterpret_cast<float*>(Act + (size_t)TM * act_stride);  // [TM]
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wv = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int lrow = lane & 15, lgrp = lane >> 4;
    const int n_items = a.meta[0];
    const long total = (long)n_items * I;
    const long R0 = total * blockIdx.x / gridDim.x, R1 = total * (blockIdx.x + 1) / gridDim.x;
    const int n_cg = H / 128;

    int seg = 0;
    for (long row = R0; row < R1 && seg < a.seg_max; ++seg) {
        const int item = (int)(row / I);
        const int r0 = (int)(row - (long)item * I);
        const int r1 = (int)min((long)I, r0 + (R1 - row));
        row += r1 - r0;
        const PItem it = a.items[item];
        const bool slot_ok = it.slot >= 0 && it.slot < a.n_slots_total;
        if (!slot_ok && tid == 0) atomicOr(a.flags, 1);
        const uint16_t* wslot = a.pool + (size_t)(slot_ok ? it.slot : 0) * a.slot_elems;
        __syncthreads();  // the previous segment is done with the LDS
        // the item's tokens: gate weights and inputs (rows beyond ntok are zero)
        if (tid < TM) {
            float gw = 0.f;
            if (tid < it.ntok && slot_ok) gw = it.first_tok >= 0 ? 1.0f : a.pgate[it.list_off + tid];
            s_gate[tid] = gw;
        }
        for (int v = tid; v < TM * (H / 8); v += kPfThreads) {
            const int r = v / (H / 8), c = v - r * (H / 8);
            uint4 val = make_uint4(0, 0, 0, 0);
            if (r < it.ntok) {
                const int tok = it.first_tok >= 0 ? it.first_tok + r : a.perm[it.list_off + r];
                val = *reinterpret_cast<const uint4*>(a.X + (size_t)tok * H + c * 8);
            }
            *reinterpret_cast<uint4*>(Xs + (size_t)r * xs_stride + c * 8) = val;
        }
        f32x4 Y[CGW][TB][8];
#pragma unroll
        for (int q = 0; q < CGW; ++q)
#pragma unroll
            for (int tb = 0; tb < TB; ++tb)
#pragma unroll
                for (int i = 0; i < 8; ++i) Y[q][tb][i] = f32x4{0.f, 0.f, 0.f, 0.f};

        for (int c0 = r0; c0 < r1; c0 += kPfChunk) {
            __syncthreads();  // inputs staged / the previous chunk's activations consumed
            // ---- phase 1: units c0 + 16 wv + (0..15), K = H in steps of 32
            {
                const int u = min(c0 + 16 * wv + lrow, r1 - 1);  // rows past the segment are masked below
                const uint16_t* wg = wslot + (size_t)u * 3 * H + lgrp * 8;
                const uint16_t* wu = wg + H;
                const uint16_t* xb = Xs + (size_t)lrow * xs_stride + lgrp * 8;
                f32x4 G[TB], U[TB];
#pragma unroll
                for (int tb = 0; tb < TB; ++tb) G[tb] = U[tb] = f32x4{0.f, 0.f, 0.f, 0.f};
                const int steps = H / 32;
                bf16x8 ag[PW], au[PW];
#pragma unroll
                for (int q = 0; q < PW; ++q) {
                    const int s = q < steps ? q : 0;
                    ag[q] = ld_bf16x8(wg + s * 32);
                    au[q] = ld_bf16x8(wu + s * 32);
                }
                for (int s0 = 0; s0 < steps; s0 += PW) {
#pragma unroll
                    for (int q = 0; q < PW; ++q) {
                        const int s = s0 + q;
                        const bf16x8 cg_ = ag[q], cu_ = au[q];
                        const int sn = s + PW < steps ? s + PW : 0;  // past the end: an in-bounds dummy
                        ag[q] = ld_bf16x8(wg + sn * 32);
                        au[q] = ld_bf16x8(wu + sn * 32);
                        if (s < steps) {
#pragma unroll
                            for (int tb = 0; tb < TB; ++tb) {
                                const bf16x8 b = ld_bf16x8(xb + (size_t)tb * 16 * xs_stride + s * 32);
                                G[tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(cg_, b, G[tb], 0, 0, 0);
                                U[tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(cu_, b, U[tb], 0, 0, 0);
                            }
                        }
                    }
                }
                // D[unit 4*lgrp + v][token lrow] -> activation, bf16, to Act[token][unit]
#pragma unroll
                for (int tb = 0; tb < TB; ++tb) {
                    const float gw = s_gate[tb * 16 + lrow];
                    uint32_t h[4];
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int unit = c0 + 16 * wv + lgrp * 4 + v;
                        const float act = unit < r1 ? silu_f(G[tb][v]) * U[tb][v] * gw : 0.f;
                        h[v] = bf16_bits(act);
                    }
                    uint2 packed = make_uint2(h[0] | (h[1] << 16), h[2] | (h[3] << 16));
                    *reinterpret_cast<uint2*>(Act + (size_t)(tb * 16 + lrow) * act_stride + 16 * wv + lgrp * 4) = packed;
                }
            }
            __syncthreads();
            // ---- phase 2: y[token][column group] += Act[token][unit] * W_down[unit][column]
#pragma unroll
            for (int q = 0; q < CGW; ++q) {
                const int cg = wv + kPfWaves * q;
                if (cg < n_cg) {  // uniform over the wavefront
                    const uint16_t* wd = wslot + 2 * H + cg * 128 + lrow * 8;
#pragma unroll 1
                    for (int ks = 0; ks < kPfChunk / 32; ++ks) {
                        // eight units for eight columns per lane, transposed in registers to eight
                        // columns of eight units each (the column a lane serves in matrix i is
                        // cg*128 + 8*lrow + i)
                        uint4 ld[8];
#pragma unroll
                        for (int j = 0; j < 8; ++j) {
                            const int unit = min(c0 + ks * 32 + lgrp * 8 + j, r1 - 1);
                            ld[j] = *reinterpret_cast<const uint4*>(wd + (size_t)unit * 3 * H);
                        }
                        bf16x8 av[TB];
#pragma unroll
                        for (int tb = 0; tb < TB; ++tb)
                            av[tb] = ld_bf16x8(Act + (size_t)(tb * 16 + lrow) * act_stride + ks * 32 + lgrp * 8);
#pragma unroll
                        for (int i = 0; i < 8; ++i) {
                            uint32_t dw[4];
#pragma unroll
                            for (int p = 0; p < 4; ++p) {
                                const uint32_t lo = reinterpret_cast<const uint32_t*>(&ld[2 * p])[i >> 1];
                                const uint32_t hi = reinterpret_cast<const uint32_t*>(&ld[2 * p + 1])[i >> 1];
                                dw[p] = (i & 1) ? __builtin_amdgcn_perm(hi, lo, 0x07060302u)
                                                : __builtin_amdgcn_perm(hi, lo, 0x05040100u);
                            }
                            bf16x8 wt;
                            memcpy(&wt, dw, 16);
#pragma unroll
                            for (int tb = 0; tb < TB; ++tb)
                                Y[q][tb][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[tb], wt, Y[q][tb][i], 0, 0, 0);
                        }
                    }
                }
            }
        }
        // ---- the segment's partial rows: D[token 4*lgrp + v][column lrow] of matrix i is column cg*128 + 8*lrow + i
        float* out = a.part + ((size_t)blockIdx.x * a.seg_max + seg) * TM * H;
#pragma unroll
        for (int q = 0; q < CGW; ++q) {
            const int cg = wv + kPfWaves * q;
            if (cg < n_cg) {
#pragma unroll
                for (int tb = 0; tb < TB; ++tb)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        float* dst = out + (size_t)(tb * 16 + lgrp * 4 + v) * H + cg * 128 + lrow * 8;
                        *reinterpret_cast<float4*>(dst) =
                            make_float4(Y[q][tb][0][v], Y[q][tb][1][v], Y[q][tb][2][v], Y[q][tb][3][v]);
                        *reinterpret_cast<float4*>(dst + 4) =
                            make_float4(Y[q][tb][4][v], Y[q][tb][5][v], Y[q][tb][6][v], Y[q][tb][7][v]);
                    }
            }
        }
    }
}

// ------------------------------------------------------------------ 4. y[t] = sum of the token's partial rows
// One workgroup per token.  The partial rows of contribution j (the k picks in pick order, then
// the shared experts) are those of the segments that cover its item; they are listed in LDS
// first and then added in list order.
constexpr int kPfListMax = 1024;
__global__ void __launch_bounds__(256) prefill_reduce_kernel(const float* __restrict__ part,
                                                             const int32_t* __restrict__ where,
                                                             const int32_t* __restrict__ meta, int n, int k, int n_shared,
                                                             int TM, int I, int H, int n_blocks, int seg_max,
                                                             float* __restrict__ y, int32_t* __restrict__ flags) {
    __shared__ int s_list[kPfListMax];
    __shared__ int s_n;
    const int t = blockIdx.x;
    const int n_items = meta[0], n_routed = meta[1];
    const long total = (long)n_items * I;
    if (threadIdx.x == 0) {
        int cnt = 0;
        const int tiles = (n + TM - 1) / TM;
        for (int j = 0; j < k + n_shared; ++j) {
            int item, row;
            if (j < k) {
                item = where[((size_t)t * k + j) * 2];
                row = where[((size_t)t * k + j) * 2 + 1];
            } else {
                item = n_routed + (j - k) * tiles + t / TM;
                row = t % TM;
            }
            const long lo = (long)item * I, hi = lo + I;
            int g = (int)(lo * n_blocks / total);
            while (g + 1 < n_blocks && total * (g + 1) / n_blocks <= lo) ++g;
            while (g > 0 && total * g / n_blocks > lo) --g;
            for (; g < n_blocks && total * g / n_blocks < hi; ++g) {
                const long b0 = total * g / n_blocks, b1 = total * (g + 1) / n_blocks;
                if (b1 <= lo || b1 == b0) continue;  // ends before the item, or an empty range
                const int seg = item - (int)(b0 / I);
                if (seg >= seg_max || cnt >= kPfListMax) {
                    atomicOr(flags, 4);
                    continue;
                }
                s_list[cnt++] = ((g * seg_max + seg) * TM + row);
            }
        }
        s_n = cnt;
    }
    __syncthreads();
    const int cnt = s_n;
    for (int c = threadIdx.x; c < H / 4; c += 256) {
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int e = 0; e < cnt; ++e) {
            const float4 v = *reinterpret_cast<const float4*>(part + (size_t)s_list[e] * H + c * 4);
            acc.x += v.x;
            acc.y += v.y;
            acc.z += v.z;
            acc.w += v.w;
        }
        *reinterpret_cast<float4*>(y + (size_t)t * H + c * 4) = acc;
    }
}

int g_pf_cus = 0;
int pf_compute_units() {
    if (g_pf_cus == 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
            n = 256;
        g_pf_cus = n;
    }
    return g_pf_cus;
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

int prefill_token_tile(const moei_model_desc& d) { return d.H <= 2048 ? 32 : 16; }

int prefill_check(const moei_model_desc& d) {
    if (d.wdtype != MOEI_WDTYPE_BF16) MOEI_FAIL(MOEI_EINVAL, "moe_prefill_layer: bf16 weights only");
    if (d.H % 128 != 0 || d.H > 4096)
        MOEI_FAIL(MOEI_ECAPACITY, "moe_prefill_layer: H = %d must be a multiple of 128 and at most 4096", d.H);
    if (d.E > kPfMaxE) MOEI_FAIL(MOEI_ECAPACITY, "moe_prefill_layer: E = %d exceeds %d", d.E, kPfMaxE);
    return MOEI_OK;
}

size_t prefill_item_bytes() { return sizeof(PItem); }
int prefill_max_items(const moei_model_desc& d, int n_max) {
    const int TM = prefill_token_tile(d);
    return (n_max * d.k + TM - 1) / TM + d.E + d.n_shared * ((n_max + TM - 1) / TM);
}
int prefill_seg_max(const moei_model_desc& d, int n_max) {
    const int G = pf_compute_units();
    return (prefill_max_items(d, n_max) + G - 1) / G + 1;
}
size_t prefill_part_floats(const moei_model_desc& d, int n_max) {
    return (size_t)pf_compute_units() * prefill_seg_max(d, n_max) * prefill_token_tile(d) * d.H;
}

int launch_prefill(const moei_model_desc& d, const PrefillScratch& ps, const void* d_pool, size_t slot_elems,
                   int n_slots_total, const int32_t* d_slot_of_row, int shared_base, int32_t* d_eam_row,
                   const void* d_router_w, const float* d_router_bias, const void* d_X, int n, float* d_Y,
                   int32_t* d_flags, hipStream_t s) {
    int rc = prefill_check(d);
    if (rc) return rc;
    if (n > ps.n_max) MOEI_FAIL(MOEI_ECAPACITY, "moe_prefill_layer: n = %d exceeds the scratch for %d tokens", n, ps.n_max);
    if ((uintptr_t)d_X % 16 != 0 || (uintptr_t)d_pool % 16 != 0 || (slot_elems * 2) % 16 != 0 || (uintptr_t)d_Y % 16 != 0)
        MOEI_FAIL(MOEI_EINVAL, "moe_prefill_layer: buffers must be 16-byte aligned");
    const int TM = prefill_token_tile(d);
    const int vec_ok = (d.H % 8 == 0) && ((uintptr_t)d_router_w % 16 == 0);
    const size_t route_smem = ((size_t)4 * d.H + (size_t)4 * d.E) * sizeof(float);
    rc = pf_allow_lds(prefill_route_kernel<uint16_t>, route_smem);
    if (rc) return rc;
    launch(K_ROUTE_TOPK, prefill_route_kernel<uint16_t>, dim3((n + 3) / 4), dim3(4 * kWave), route_smem, s, d_router_w,
           d_router_bias, d_X, n, d.H, d.E, d.k, (int)(d.renorm_topk != 0), vec_ok, ps.d_idx, ps.d_w);
    MOEI_LAUNCH_CHECK();
    GroupArgsP g{ps.d_idx, ps.d_w, n, d.k, d.E, d.n_shared, TM, d_slot_of_row, shared_base, d_eam_row, ps.d_perm,
                 ps.d_pgate, ps.d_where, reinterpret_cast<PItem*>(ps.d_items), ps.d_meta, ps.d_cntw, d_flags};
    launch(K_FFN_GROUP, prefill_count_kernel, dim3(d.E), dim3(kGrpThreads), 0, s, g);
    MOEI_LAUNCH_CHECK();
    launch(K_FFN_GROUP, prefill_place_kernel, dim3(d.E), dim3(kGrpThreads), 0, s, g);
    MOEI_LAUNCH_CHECK();
    const int G = pf_compute_units();
    PfArgs a{reinterpret_cast<const uint16_t*>(d_pool), slot_elems, n_slots_total,
             reinterpret_cast<const PItem*>(ps.d_items), ps.d_meta, reinterpret_cast<const uint16_t*>(d_X), ps.d_perm,
             ps.d_pgate, ps.d_part, d.H, d.I, ps.seg_max, d_flags};
    const size_t smem = ((size_t)TM * (d.H + kPfPad) + (size_t)TM * (kPfChunk + kPfPad)) * 2 + (size_t)TM * 4;
    if (TM == 32) {
        rc = pf_allow_lds(prefill_ffn_kernel<2, 2>, smem);
        if (rc) return rc;
        launch(K_FFN_FUSED, prefill_ffn_kernel<2, 2>, dim3(G), dim3(kPfThreads), smem, s, a);
    } else {
        rc = pf_allow_lds(prefill_ffn_kernel<1, 4>, smem);
        if (rc) return rc;
        launch(K_FFN_FUSED, prefill_ffn_kernel<1, 4>, dim3(G), dim3(kPfThreads), smem, s, a);
    }
    MOEI_LAUNCH_CHECK();
    launch(K_FFN_REDUCE, prefill_reduce_kernel, dim3(n), dim3(256), 0, s, (const float*)ps.d_part,
           (const int32_t*)ps.d_where, (const int32_t*)ps.d_meta, n, d.k, d.n_shared, TM, d.I, d.H, G, ps.seg_max, d_Y,
           d_flags);
    MOEI_LAUNCH_CHECK();
    return MOEI_OK;
}

}  // namespace moei
