// Step 4 of the layer step: PredictEAM aggregation + prefetch / eviction priorities.
//
// Prefetch score (Sec. 4.5 of the paper): the matched EAM's cell, normalised over
// its row, times the layer-proximity factor (1 - (i - l)/L) for future layers i > l.
// Eviction score (Alg. 1): (cell + eps)(1 - i/L) / row sum, lowest score evicted
// first.  Both are evaluated as one fp64 division of exact products so that equal
// rationals give equal keys; the orders are then produced by rank counting (a
// candidate's rank is the number of candidates that sort before it; ties go to the
// lower flat id, so ranks are unique) with wavefront ballots.
#include "kernels.hpp"
#include "score.hpp"

namespace moei {

namespace {

constexpr int kRankThreads = 256;

// One workgroup; see score_cells.
__global__ void __launch_bounds__(kScoreThreads) priority_score_kernel(ScoreArgs a) {
    __shared__ int s_n[2];
    __shared__ int s_best[kMaxMatchBatch];
    __shared__ HeadLds s_heads;
    __shared__ KeyLds s_keys;
    score_and_heads(a, s_heads, s_keys, s_n, s_best, false);
}

// grid (workgroups, 2 lists).  The workgroup stages the list's L*E keys in LDS; a wavefront
// then takes one candidate cell at a time, its 64 lanes compare that key with 64 keys per
// step, and the ballot population counts add up to the candidate's rank: the number of
// candidates that sort before it (smaller key, or equal key and lower flat id).
__global__ void __launch_bounds__(kRankThreads)
    priority_rank_kernel(const u64* __restrict__ keys_all, int LE, const int32_t* __restrict__ n_pf,
                         const int32_t* __restrict__ n_ev, int32_t* __restrict__ pf_order,
                         int32_t* __restrict__ ev_order) {
    extern __shared__ __align__(16) unsigned char smem_raw[];
    u64* keys = reinterpret_cast<u64*>(smem_raw);
    const int which = blockIdx.y;
    if ((which == 0 ? *n_pf : *n_ev) == 0) return;  // an empty list: nothing to order (uniform)
    const u64* src = keys_all + (size_t)which * LE;
    int32_t* order = which == 0 ? pf_order : ev_order;
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wv = __builtin_amdgcn_readfirstlane(tid / kWave);
    // stage the keys: eight independent loads in flight per thread
    for (int i0 = 0; i0 < LE; i0 += 8 * kRankThreads) {
        u64 v[8];
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const int i = i0 + r * kRankThreads + tid;
            v[r] = i < LE ? src[i] : kNone;
        }
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const int i = i0 + r * kRankThreads + tid;
            if (i < LE) keys[i] = v[r];
        }
    }
    __syncthreads();
    const int W = gridDim.x * (kRankThreads / kWave);
    for (int f = blockIdx.x * (kRankThreads / kWave) + wv; f < LE; f += W) {
        const u64 mine = keys[f];
        if (mine == kNone) continue;  // uniform over the wavefront
        int rank = 0;
        for (int g0 = 0; g0 < LE; g0 += 4 * kWave) {  // four LDS reads in flight, then four ballots
            u64 kg[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int g = g0 + u * kWave + lane;
                kg[u] = g < LE ? keys[g] : kNone;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int g = g0 + u * kWave + lane;
                const bool before = kg[u] < mine || (kg[u] == mine && g < f);  // a padding key is never before
                rank += __popcll(__ballot(before));
            }
        }
        if (lane == 0) order[rank] = f;
    }
}

}  // namespace

}  // namespace moei

namespace moei {

ScoreArgs make_score_args(const moei_eamc* c, const int32_t* d_best, int B, int cur_layer, const int32_t* d_slot_of,
                          float eps, const int32_t* d_cur_idx, int n_cur, float* d_prefetch, float* d_evict,
                          int32_t* d_n_pf, int32_t* d_n_ev) {
    return ScoreArgs{c->d_traces, c->cell_bytes, c->n_cap, c->N, c->d.L, c->d.E, d_best, B, cur_layer, d_slot_of,
                     (double)eps, d_cur_idx, d_cur_idx ? n_cur : 0, d_prefetch, d_evict, c->d_keys, d_n_pf, d_n_ev,
                     nullptr, nullptr, 0, 0, nullptr, nullptr, nullptr, nullptr, nullptr};
}

// The two orders from the keys that score_cells left in c->d_keys.
int launch_priority_rank(const moei_model_desc& d, const unsigned long long* d_keys, const int32_t* d_n_pf,
                         const int32_t* d_n_ev, int32_t* d_pf_order, int32_t* d_ev_order, hipStream_t s) {
    const size_t LE = (size_t)d.L * d.E;
    const size_t smem = LE * 8;
    if (smem > 64 * 1024) {
        static size_t allowed = 0;
        if (smem > allowed) {
            MOEI_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(priority_rank_kernel),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
            allowed = smem;
        }
    }
    // enough wavefronts that each ranks only a few cells
    int blocks = (int)((LE + 4 * (kRankThreads / kWave) - 1) / (4 * (kRankThreads / kWave)));
    blocks = blocks < 1 ? 1 : (blocks > 256 ? 256 : blocks);
    launch(K_PRIO_RANK, priority_rank_kernel, dim3(blocks, 2), dim3(kRankThreads), smem, s, (const u64*)d_keys,
           (int)LE, d_n_pf, d_n_ev, d_pf_order, d_ev_order);
    MOEI_LAUNCH_CHECK();
    return MOEI_OK;
}

}  // namespace moei

using namespace moei;

extern "C" int expert_priority(const moei_eamc* c, const int32_t* d_best, int32_t B, int32_t cur_layer,
                               const int32_t* d_slot_of, float eps, const int32_t* d_cur_idx, int32_t n_cur,
                               float* d_prefetch, float* d_evict, int32_t* d_pf_order, int32_t* d_n_pf,
                               int32_t* d_ev_order, int32_t* d_n_ev, void* stream) {
    MOEI_REQUIRE(c && d_best && d_slot_of && d_prefetch && d_evict && d_pf_order && d_n_pf && d_ev_order && d_n_ev,
                 "expert_priority: null pointer");
    MOEI_REQUIRE(B >= 1 && B <= kMaxMatchBatch, "expert_priority: B = %d outside [1, %d]", B, kMaxMatchBatch);
    MOEI_REQUIRE(cur_layer >= -1 && cur_layer < c->d.L, "expert_priority: cur_layer = %d outside [-1, %d)", cur_layer,
                 c->d.L);
    MOEI_REQUIRE(eps >= 0.f, "expert_priority: eps must not be negative");
    MOEI_REQUIRE(!d_cur_idx || (n_cur >= 0 && n_cur <= kMaxMatchBatch * c->d.E),
                 "expert_priority: n_cur = %d outside [0, %d]", n_cur, kMaxMatchBatch * c->d.E);
    hipStream_t s = as_stream(stream);
    ScoreArgs a = make_score_args(c, d_best, B, cur_layer, d_slot_of, eps, d_cur_idx, n_cur, d_prefetch, d_evict, d_n_pf,
                                  d_n_ev);
    launch(K_PRIO_SCORE, priority_score_kernel, dim3(1), dim3(kScoreThreads), 0, s, a);
    MOEI_LAUNCH_CHECK();
    return launch_priority_rank(c->d, c->d_keys, d_n_pf, d_n_ev, d_pf_order, d_ev_order, s);
}
