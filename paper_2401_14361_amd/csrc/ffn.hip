// Step 5 of the layer step: the activated experts' FFN as a GEMV over cache slots.
//
// An expert is a feed-forward network (Sec. 2 of the paper); here in SwiGLU form,
//   o = W_down ( silu(W_gate x) * (W_up x) ),  y = sum_e w_e o_e.
// At batch 1 this is one flop per weight byte, so the kernels are pure weight
// streams: a wavefront owns a few matrix rows, reads them with 16-byte loads
// (8 bf16 or 4 fp32 per lane), multiplies with the fp32 copy of the input vector held
// in LDS, and finishes with a 64-lane butterfly sum.  The down projection is split
// over (expert, row group, column range); its partial results are added up in a
// fixed order by a last small kernel, so the output is deterministic.
#include <stdlib.h>

#include "kernels.hpp"
#include "wtypes.hpp"

namespace moei {

namespace {

constexpr int kFfnThreads = 256;
constexpr int kWavesPerBlock = kFfnThreads / kWave;

struct FfnArgs {
    const void* pool;
    size_t slot_elems;
    int n_slots_total;
    const int32_t* slot_ids;
    const float* gate_w;
    const void* x;
    float* act;   // [n_act][I]
    float* part;  // [n_act * ksplit][H]
    int H, I, ksplit, iper;
    int32_t* flags;
};

// act[e][i] = silu(<W_gate[i], x>) * <W_up[i], x>;  grid (ceil(I / (4R)), n_act)
template <typename WT, int R, bool VEC>
__global__ void __launch_bounds__(kFfnThreads) ffn_gate_up_kernel(FfnArgs a) {
    using V = WVec<WT>;
    extern __shared__ __align__(16) float xs[];
    const int e = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    const int H = a.H, I = a.I;
    const int i0 = (blockIdx.x * kWavesPerBlock + wv) * R;
    const int slot = a.slot_ids[e];
    if (slot < 0 || slot >= a.n_slots_total) {  // uniform over the workgroup
        if (lane == 0)
            for (int r = 0; r < R; ++r)
                if (i0 + r < I) a.act[(size_t)e * I + i0 + r] = 0.f;
        if (tid == 0) atomicOr(a.flags, 1);
        return;
    }
    stage_as_f32(reinterpret_cast<const WT*>(a.x), xs, H);
    __syncthreads();
    if (i0 >= I) return;
    const WT* Wg = reinterpret_cast<const WT*>(a.pool) + (size_t)slot * a.slot_elems;
    const WT* Wu = Wg + (size_t)I * H;
    const WT* rg[R];
    const WT* ru[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        int row = min(i0 + r, I - 1);  // tail rows recompute the last row and are not written
        rg[r] = Wg + (size_t)row * H;
        ru[r] = Wu + (size_t)row * H;
    }
    float ag[R], au[R];
#pragma unroll
    for (int r = 0; r < R; ++r) ag[r] = au[r] = 0.f;
    if (VEC) {
#pragma unroll 2
        for (int c = lane * V::N; c < H; c += kWave * V::N) {
            typename V::raw wg[R], wu[R];
#pragma unroll
            for (int r = 0; r < R; ++r) {
                wg[r] = V::load(rg[r] + c);
                wu[r] = V::load(ru[r] + c);
            }
            float xf[V::N];
#pragma unroll
            for (int i = 0; i < V::N; i += 4) *reinterpret_cast<float4*>(xf + i) = *reinterpret_cast<const float4*>(xs + c + i);
#pragma unroll
            for (int r = 0; r < R; ++r) {
                ag[r] = V::dot(wg[r], xf, ag[r]);
                au[r] = V::dot(wu[r], xf, au[r]);
            }
        }
    } else {
        for (int c = lane; c < H; c += kWave) {
            float xv = xs[c];
#pragma unroll
            for (int r = 0; r < R; ++r) {
                ag[r] = __builtin_fmaf(V::one(rg[r] + c), xv, ag[r]);
                au[r] = __builtin_fmaf(V::one(ru[r] + c), xv, au[r]);
            }
        }
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
        float g = wave_sum(ag[r]);
        float u = wave_sum(au[r]);
        if (lane == 0 && i0 + r < I) a.act[(size_t)e * I + i0 + r] = g / (1.0f + expf(-g)) * u;
    }
}

// part[e*ksplit + ks][h] = w_e * <W_down[h][i_lo:i_hi], act[e][i_lo:i_hi]>;
// grid (ceil(H / (4R)), ksplit, n_act)
template <typename WT, int R, bool VEC>
__global__ void __launch_bounds__(kFfnThreads) ffn_down_kernel(FfnArgs a) {
    using V = WVec<WT>;
    extern __shared__ __align__(16) float as[];
    const int e = blockIdx.z, ks = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    const int H = a.H, I = a.I;
    const int h0 = (blockIdx.x * kWavesPerBlock + wv) * R;
    float* out = a.part + ((size_t)e * a.ksplit + ks) * H;
    const int slot = a.slot_ids[e];
    const int i_lo = ks * a.iper;
    const int i_hi = min(I, i_lo + a.iper);
    if (slot < 0 || slot >= a.n_slots_total || i_lo >= i_hi) {  // uniform over the workgroup
        if (lane == 0)
            for (int r = 0; r < R; ++r)
                if (h0 + r < H) out[h0 + r] = 0.f;
        return;
    }
    const float gw = a.gate_w[e];
    const int ni = i_hi - i_lo;
    for (int i = tid; i < ni; i += kFfnThreads) as[i] = a.act[(size_t)e * I + i_lo + i] * gw;
    __syncthreads();
    if (h0 >= H) return;
    const WT* Wd = reinterpret_cast<const WT*>(a.pool) + (size_t)slot * a.slot_elems + (size_t)2 * I * H;
    const WT* rd[R];
#pragma unroll
    for (int r = 0; r < R; ++r) rd[r] = Wd + (size_t)min(h0 + r, H - 1) * I + i_lo;
    float acc[R];
#pragma unroll
    for (int r = 0; r < R; ++r) acc[r] = 0.f;
    if (VEC) {
#pragma unroll 2
        for (int c = lane * V::N; c < ni; c += kWave * V::N) {
            typename V::raw w[R];
#pragma unroll
            for (int r = 0; r < R; ++r) w[r] = V::load(rd[r] + c);
            float xf[V::N];
#pragma unroll
            for (int i = 0; i < V::N; i += 4) *reinterpret_cast<float4*>(xf + i) = *reinterpret_cast<const float4*>(as + c + i);
#pragma unroll
            for (int r = 0; r < R; ++r) acc[r] = V::dot(w[r], xf, acc[r]);
        }
    } else {
        for (int c = lane; c < ni; c += kWave) {
            float xv = as[c];
#pragma unroll
            for (int r = 0; r < R; ++r) acc[r] = __builtin_fmaf(V::one(rd[r] + c), xv, acc[r]);
        }
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
        float s = wave_sum(acc[r]);
        if (lane == 0 && h0 + r < H) out[h0 + r] = s;
    }
}

// y[h] = sum of the n_part partial rows, in index order.
__global__ void ffn_reduce_kernel(const float* __restrict__ part, int n_part, int H, float* __restrict__ y) {
    int h = blockIdx.x * blockDim.x + threadIdx.x;
    if (h >= H) return;
    float s = 0.f;
    for (int p = 0; p < n_part; ++p) s += part[(size_t)p * H + h];
    y[h] = s;
}

int env_int(const char* name, int dflt) {
    const char* v = getenv(name);
    if (!v || !*v) return dflt;
    return atoi(v);
}

template <typename WT, bool VEC>
int launch_ffn_typed(const FfnArgs& a, int n_act, int r1, int r2, float* d_y, hipStream_t s) {
    const int H = a.H, I = a.I;
    dim3 g1((I + kWavesPerBlock * r1 - 1) / (kWavesPerBlock * r1), n_act);
    size_t sm1 = (size_t)H * sizeof(float);
    switch (r1) {
        case 1: ffn_gate_up_kernel<WT, 1, VEC><<<g1, kFfnThreads, sm1, s>>>(a); break;
        case 2: ffn_gate_up_kernel<WT, 2, VEC><<<g1, kFfnThreads, sm1, s>>>(a); break;
        default: ffn_gate_up_kernel<WT, 4, VEC><<<g1, kFfnThreads, sm1, s>>>(a); break;
    }
    MOEI_LAUNCH_CHECK();
    dim3 g2((H + kWavesPerBlock * r2 - 1) / (kWavesPerBlock * r2), a.ksplit, n_act);
    size_t sm2 = (size_t)a.iper * sizeof(float);
    switch (r2) {
        case 1: ffn_down_kernel<WT, 1, VEC><<<g2, kFfnThreads, sm2, s>>>(a); break;
        case 2: ffn_down_kernel<WT, 2, VEC><<<g2, kFfnThreads, sm2, s>>>(a); break;
        default: ffn_down_kernel<WT, 4, VEC><<<g2, kFfnThreads, sm2, s>>>(a); break;
    }
    MOEI_LAUNCH_CHECK();
    ffn_reduce_kernel<<<(H + 255) / 256, 256, 0, s>>>(a.part, n_act * a.ksplit, H, d_y);
    MOEI_LAUNCH_CHECK();
    return MOEI_OK;
}

// Column ranges of the down projection: at most 4096 intermediate values per range,
// a multiple of 512 (one 16-byte load per lane of a wavefront covers 512 bf16).
int plan_ksplit(int I, int ksplit_max, int* iper) {
    int ks = (I + 4095) / 4096;
    ks = env_int("MOEI_FFN_KSPLIT", ks);
    if (ks < 1) ks = 1;
    if (ks > ksplit_max) ks = ksplit_max;
    int per = (I + ks - 1) / ks;
    per = (per + 511) / 512 * 512;
    *iper = per;
    return (I + per - 1) / per;
}

}  // namespace

int ffn_scratch_alloc(const moei_model_desc& d, int n_act_max, FfnScratch* out) {
    out->n_act_max = n_act_max;
    out->ksplit_max = (d.I + 511) / 512;
    hipError_t e = hipMalloc((void**)&out->d_act, (size_t)n_act_max * d.I * sizeof(float));
    if (e == hipSuccess)
        e = hipMalloc((void**)&out->d_part, (size_t)n_act_max * out->ksplit_max * d.H * sizeof(float));
    if (e != hipSuccess) {
        ffn_scratch_free(out);
        MOEI_FAIL(MOEI_ENOMEM, "FFN scratch allocation failed: %s", hipGetErrorString(e));
    }
    return MOEI_OK;
}

void ffn_scratch_free(FfnScratch* s) {
    (void)hipFree(s->d_act);
    (void)hipFree(s->d_part);
    s->d_act = s->d_part = nullptr;
}

int launch_expert_ffn(const moei_model_desc& d, const void* d_pool, size_t slot_elems, int n_slots_total,
                      const FfnScratch& scr, const int32_t* d_slot_ids, const float* d_gate_w, int n_act,
                      const void* d_x, float* d_y, int32_t* d_flags, hipStream_t s) {
    if (n_act == 0) {  // an empty sum: the reduction over zero partial rows writes zeros
        ffn_reduce_kernel<<<(d.H + 255) / 256, 256, 0, s>>>(scr.d_part, 0, d.H, d_y);
        MOEI_LAUNCH_CHECK();
        return MOEI_OK;
    }
    FfnArgs a{};
    a.pool = d_pool;
    a.slot_elems = slot_elems;
    a.n_slots_total = n_slots_total;
    a.slot_ids = d_slot_ids;
    a.gate_w = d_gate_w;
    a.x = d_x;
    a.act = scr.d_act;
    a.part = scr.d_part;
    a.H = d.H;
    a.I = d.I;
    a.flags = d_flags;
    a.ksplit = plan_ksplit(d.I, scr.ksplit_max, &a.iper);
    const int wb = d.wdtype == MOEI_WDTYPE_BF16 ? 2 : 4;
    const int n = 16 / wb;
    const bool vec = (d.H % n == 0) && (d.I % n == 0) && ((uintptr_t)d_pool % 16 == 0) && ((slot_elems * wb) % 16 == 0);
    auto rows = [](int r) { return r >= 4 ? 4 : (r >= 2 ? 2 : 1); };
    static const int r1 = rows(env_int("MOEI_FFN_R1", 2));
    static const int r2 = rows(env_int("MOEI_FFN_R2", 4));
    if (d.wdtype == MOEI_WDTYPE_BF16)
        return vec ? launch_ffn_typed<uint16_t, true>(a, n_act, r1, r2, d_y, s)
                   : launch_ffn_typed<uint16_t, false>(a, n_act, r1, r2, d_y, s);
    return vec ? launch_ffn_typed<float, true>(a, n_act, r1, r2, d_y, s)
               : launch_ffn_typed<float, false>(a, n_act, r1, r2, d_y, s);
}

}  // namespace moei
