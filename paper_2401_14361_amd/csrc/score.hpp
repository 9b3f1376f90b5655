// Scoring of every (layer, expert) cell from the matched traces: shared by the stand-alone
// priority kernel and by the match kernel's finishing workgroup (fused layer step).
#pragma once

#include "kernels.hpp"

namespace moei {

#if defined(__HIPCC__)

typedef unsigned long long u64;
constexpr int kScoreThreads = 1024;
constexpr u64 kNone = ~0ull;

struct ScoreArgs {
    const void* traces;  // [L][n_cap][E]
    int cell_bytes, n_cap, N, L, E;
    const int32_t* best;  // [B]
    int B, cur_layer;
    const int32_t* slot_of;  // [L*E]
    double eps;
    const int32_t* cur_idx;  // [n_cur] experts of the current layer that are about to run, or null
    int n_cur;
    float* P;  // [L*E]
    float* V;  // [L*E]
    u64* keys;     // [2][L*E]: prefetch keys, eviction keys; kNone = not a candidate
    int32_t* n_pf;
    int32_t* n_ev;
    // h_pf / h_ev > 0: the scoring workgroup also writes that many leading entries of each order
    // (select_heads); the complete orders come from priority_rank_kernel over `keys`
    int32_t* pf_order;
    int32_t* ev_order;
    int h_pf, h_ev;
    // pinned host memory that receives what the synchronous layer step reads on the host (or null):
    // matched trace, list lengths, the heads, and - for the prefetch admission - the eviction scores
    int32_t* host_best;
    int32_t* host_n;        // [2]: n_pf, n_ev
    int32_t* host_pf_head;
    int32_t* host_ev_head;
    float* host_V;          // [L*E] or null
    // a host that polls instead of waiting for an event: after host_best has been written (and made
    // visible to the host) the step's number goes to *host_seq (pinned, or null)
    int32_t* host_seq;
    int32_t seq;
};

__device__ __forceinline__ uint32_t cell_at(const void* traces, int cell_bytes, size_t i) {
    return cell_bytes == 4 ? (uint32_t) reinterpret_cast<const int32_t*>(traces)[i]
                           : (uint32_t) reinterpret_cast<const uint16_t*>(traces)[i];
}

// Called by all kScoreThreads threads of ONE workgroup: scores for every cell, a 64-bit sort
// key per cell and list (kNone where the cell is not a candidate) and the two candidate
// counts.  One wavefront per layer row.  s_n[2] and s_best[kMaxMatchBatch] are LDS; with
// best_in_lds the caller has already put the matched trace indices (-1 = none) there.
// A copy of the keys in LDS for the head selection (models of up to kKeyLdsCells cells): the
// selection then needs no second trip to memory.
constexpr int kKeyLdsCells = 2048;
struct KeyLds {
    u64 k[2][kKeyLdsCells];
};

__device__ __forceinline__ void score_cells(const ScoreArgs& a, int* s_n, int* s_best, bool best_in_lds, u64* kp,
                                            u64* kv, KeyLds* lds_keys) {
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wv = tid / kWave;
    const int L = a.L, E = a.E, l = a.cur_layer;
    if (tid < 2) s_n[tid] = 0;
    if (!best_in_lds && tid < a.B) {
        const int n = a.best[tid];
        s_best[tid] = (n >= 0 && n < a.N) ? n : -1;
    }
    __syncthreads();
    constexpr int kPerLane = 4;  // cells of a row held in registers (rows up to 256 wide)
    int my_ev = 0, my_pf = 0;
    for (int i = wv; i < L; i += kScoreThreads / kWave) {
        // all of the row's loads go out together: matched cells, residency, current picks
        u64 tv[kPerLane];
        int sv[kPerLane];
        u64 rsum = 0;
        for (int r = 0; r * kWave < E; ++r) {
            const int j = lane + r * kWave;
            u64 t = 0;
            int slot = -1;
            if (j < E) {
                for (int b = 0; b < a.B; ++b) {
                    const int n = s_best[b];
                    if (n >= 0) t += cell_at(a.traces, a.cell_bytes, ((size_t)i * a.n_cap + n) * E + j);
                }
                if (r < kPerLane) slot = a.slot_of[(size_t)i * E + j];
            }
            if (r < kPerLane) {
                tv[r] = t;
                sv[r] = slot;
            }
            rsum += t;
        }
        int cur = -1;  // lane m holds pick m of the current layer (used for row l only)
        if (i == l && lane < a.n_cur) cur = a.cur_idx[lane];
        const u64 R = wave_sum_u64_dpp(rsum);
        const double den = (double)(R ? R : 1ull) * (double)L;
        for (int r = 0; r * kWave < E; ++r) {
            const int j = lane + r * kWave;
            u64 t = 0;
            int slot = -1;
            if (r < kPerLane) {
                t = tv[r];
                slot = sv[r];
            } else if (j < E) {
                for (int b = 0; b < a.B; ++b) {
                    const int n = s_best[b];
                    if (n >= 0) t += cell_at(a.traces, a.cell_bytes, ((size_t)i * a.n_cap + n) * E + j);
                }
                slot = a.slot_of[(size_t)i * E + j];
            }
            // is expert j one of the current picks?  (all 64 lanes take part in the shuffles)
            bool excluded = false;
            if (i == l) {
                for (int m0 = 0; m0 < a.n_cur; m0 += kWave) {
                    int c = cur;
                    if (m0 > 0) c = (m0 + lane < a.n_cur) ? a.cur_idx[m0 + lane] : -1;
                    const int lim = min(kWave, a.n_cur - m0);
                    for (int m = 0; m < lim; ++m) excluded |= (__shfl(c, m, kWave) == j);
                }
            }
            if (j >= E) continue;
            const size_t f = (size_t)i * E + j;
            const double td = (double)t;
            const double v = ((td + a.eps) * (double)(L - i)) / den;
            double p = 0.0;
            if (i > l && R > 0) p = (td * (double)(L - i + l)) / den;
            a.P[f] = (float)p;
            a.V[f] = (float)v;
            if (a.host_V) a.host_V[f] = (float)v;
            // positive doubles order like their bit patterns; ~bits turns descending into ascending
            const bool is_pf = i > l && p > 0.0 && slot < 0;
            const bool is_ev = slot >= 0 && !excluded;
            const u64 key_p = is_pf ? ~(u64)__double_as_longlong(p) : kNone;
            const u64 key_v = is_ev ? (u64)__double_as_longlong(v) : kNone;
            kp[f] = key_p;
            kv[f] = key_v;
            if (lds_keys) {
                lds_keys->k[0][f] = key_p;
                lds_keys->k[1][f] = key_v;
            }
            my_pf += is_pf;
            my_ev += is_ev;
        }
    }
    if (my_pf) atomicAdd(&s_n[0], my_pf);
    if (my_ev) atomicAdd(&s_n[1], my_ev);
    __syncthreads();
    if (tid == 0) {
        *a.n_pf = s_n[0];
        *a.n_ev = s_n[1];
        if (a.host_n) {
            a.host_n[0] = s_n[0];
            a.host_n[1] = s_n[1];
        }
        if (a.host_best) *a.host_best = s_best[0];
        if (a.host_seq) {
            __threadfence_system();  // the matched trace is in host memory before the number that announces it
            __hip_atomic_store(a.host_seq, a.seq, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        }
    }
}

// ---- heads of the two orders
// Alg. 1 evicts the expert of lowest priority: serving one layer's k picks consumes at most k entries
// of the eviction order, and prefetching looks at `depth` entries of the prefetch order.  The layer
// step therefore selects only those heads (h rounds of a workgroup-wide arg-min over the keys that
// score_cells has left in global memory); the complete orders are ranked from the same keys by
// priority_rank_kernel when somebody asks for them.
struct KeyId {
    u64 k;
    int id;
};
__device__ __forceinline__ KeyId keyid_min(KeyId a, KeyId b) {
    const bool take_b = b.k < a.k || (b.k == a.k && b.id < a.id);
    KeyId r;
    r.k = take_b ? b.k : a.k;
    r.id = take_b ? b.id : a.id;
    return r;
}
__device__ __forceinline__ unsigned wave_min_u32_dpp(unsigned v) {
    v = min(v, MOEI_DPP_U32(v, 0xB1));   // quad_perm [1,0,3,2]
    v = min(v, MOEI_DPP_U32(v, 0x4E));   // quad_perm [2,3,0,1]
    v = min(v, MOEI_DPP_U32(v, 0x141));  // row_half_mirror
    v = min(v, MOEI_DPP_U32(v, 0x140));  // row_mirror
    const unsigned a = (unsigned)__builtin_amdgcn_readlane((int)v, 0), b = (unsigned)__builtin_amdgcn_readlane((int)v, 16);
    const unsigned c = (unsigned)__builtin_amdgcn_readlane((int)v, 32), d = (unsigned)__builtin_amdgcn_readlane((int)v, 48);
    return min(min(a, b), min(c, d));
}
// smallest (key, id) of the wavefront, in every lane (all 64 lanes active): three one-word minima -
// the key's high word, the low word among the lanes that hold that high word, the id among the
// lanes that hold that key
__device__ __forceinline__ KeyId wave_keyid_min(KeyId v) {
    const unsigned hi = (unsigned)(v.k >> 32), lo = (unsigned)v.k;
    const unsigned mh = wave_min_u32_dpp(hi);
    const unsigned ml = wave_min_u32_dpp(hi == mh ? lo : 0xffffffffu);
    const unsigned mi = wave_min_u32_dpp((hi == mh && lo == ml) ? (unsigned)v.id : 0x7fffffffu);
    return KeyId{((u64)mh << 32) | ml, (int)mi};
}

constexpr int kSelWaves = 4;                     // wavefronts that search one list (one per SIMD)
constexpr int kSelThreads = kSelWaves * kWave;
constexpr int kSelOwn = 8;                       // keys a lane keeps in registers (models of up to 2048 cells)
constexpr int kHeadMax = 96;                     // most entries of a head (picks + prefetch candidates)
struct HeadLds {
    u64 key[2][kSelWaves][kHeadMax];
    int id[2][kSelWaves][kHeadMax];
};

// All kScoreThreads threads of the scoring workgroup call, after score_cells (whose closing barrier
// has made the keys visible).  Wavefronts 0..3 search the prefetch list, 4..7 the eviction list, the
// others only meet the barrier.  Lane t of a list's 256 owns cells t, t + 256, ...  First every
// wavefront extracts the h smallest (key, flat id) pairs of its own cells - h rounds of a DPP arg-min,
// no barrier: what remains after a round is what lies after its winner - then the list's first
// wavefront extracts the h smallest of the 4 h candidates the same way.
// Writes pf_order[0 .. min(h_pf, n_pf)) and ev_order[0 .. min(h_ev, n_ev)).
__device__ __forceinline__ void select_heads(const ScoreArgs& a, const u64* kp, const u64* kv, const int* s_n, HeadLds& hl) {
    const int tid = threadIdx.x;
    const int LE = a.L * a.E;
    const int list = tid / kSelThreads;          // 0, 1: searching; >= 2: idle
    const int ltid = tid % kSelThreads;
    const int lane = tid & (kWave - 1), lwave = ltid / kWave;
    const bool active = list < 2;
    const u64* keys = list == 0 ? kp : kv;
    int32_t* out = list == 0 ? a.pf_order : a.ev_order;
    int32_t* host_out = list == 0 ? a.host_pf_head : a.host_ev_head;
    int want = 0;
    if (active) want = list == 0 ? min(a.h_pf, s_n[0]) : min(a.h_ev, s_n[1]);
    want = min(want, kHeadMax);
    if (want > 0) {  // uniform over the wavefront
        const bool in_regs = LE <= kSelOwn * kSelThreads;
        u64 mine[kSelOwn];
#pragma unroll
        for (int r = 0; r < kSelOwn; ++r) {
            const int f = ltid + r * kSelThreads;
            mine[r] = (in_regs && f < LE) ? keys[f] : kNone;
        }
        bool have_last = false;
        KeyId last{0, -1};
        KeyId cur{kNone, 0x7fffffff};
        bool cur_valid = false;  // this lane's best remaining cell is known
        for (int round = 0; round < want; ++round) {
            if (!cur_valid) {
                cur = KeyId{kNone, 0x7fffffff};
                auto consider = [&](u64 k, int f) {
                    if (k == kNone) return;
                    if (have_last && (k < last.k || (k == last.k && f <= last.id))) return;
                    cur = keyid_min(cur, KeyId{k, f});
                };
                if (in_regs) {
#pragma unroll
                    for (int r = 0; r < kSelOwn; ++r) consider(mine[r], ltid + r * kSelThreads);
                } else {
                    for (int f = ltid; f < LE; f += kSelThreads) consider(keys[f], f);
                }
                cur_valid = true;
            }
            const KeyId w = wave_keyid_min(cur);
            if (lane == 0) {
                hl.key[list][lwave][round] = w.k;
                hl.id[list][lwave][round] = w.id;
            }
            last = w;
            have_last = true;
            if (cur.id == w.id) cur_valid = false;  // this lane's best has been taken: look for its next one
        }
    }
    __syncthreads();
    if (want > 0 && lwave == 0) {
        // 4 * want candidates, lane-major: candidate c = wave * want + round sits in lane c % 64
        constexpr int kPer = (kSelWaves * kHeadMax + kWave - 1) / kWave;
        const int total = kSelWaves * want;
        KeyId cand[kPer];
#pragma unroll
        for (int r = 0; r < kPer; ++r) {
            const int c = lane + r * kWave;
            cand[r] = c < total ? KeyId{hl.key[list][c / want][c % want], hl.id[list][c / want][c % want]} : KeyId{kNone, 0x7fffffff};
        }
        bool have_last = false;
        KeyId last{0, -1};
        for (int round = 0; round < want; ++round) {
            KeyId cur{kNone, 0x7fffffff};
#pragma unroll
            for (int r = 0; r < kPer; ++r) {
                const KeyId c = cand[r];
                if (c.k == kNone) continue;
                if (have_last && (c.k < last.k || (c.k == last.k && c.id <= last.id))) continue;
                cur = keyid_min(cur, c);
            }
            const KeyId w = wave_keyid_min(cur);
            if (lane == 0 && w.k != kNone) {
                out[round] = w.id;
                if (host_out) host_out[round] = w.id;
            }
            last = w;
            have_last = true;
        }
    }
}

// Scoring, then the heads of the orders when the caller has asked for them.
__device__ __forceinline__ void score_and_heads(const ScoreArgs& a, HeadLds& hl, KeyLds& kl, int* s_n, int* s_best,
                                                bool best_in_lds) {
    const int LE = a.L * a.E;
    const bool heads = a.h_pf > 0 || a.h_ev > 0;
    const bool in_lds = heads && LE <= kKeyLdsCells;
    score_cells(a, s_n, s_best, best_in_lds, a.keys, a.keys + LE, in_lds ? &kl : nullptr);
    if (heads) select_heads(a, in_lds ? kl.k[0] : a.keys, in_lds ? kl.k[1] : a.keys + LE, s_n, hl);
}

#endif

// priority.hip
ScoreArgs make_score_args(const moei_eamc* c, const int32_t* d_best, int B, int cur_layer, const int32_t* d_slot_of,
                          float eps, const int32_t* d_cur_idx, int n_cur, float* d_prefetch, float* d_evict,
                          int32_t* d_n_pf, int32_t* d_n_ev);
// the complete orders from the keys score_cells has left in d_keys[2][L*E]
int launch_priority_rank(const moei_model_desc& d, const unsigned long long* d_keys, const int32_t* d_n_pf,
                         const int32_t* d_n_ev, int32_t* d_pf_order, int32_t* d_ev_order, hipStream_t s);
// match.hip: the match, and - if `score` is given (B must be 1) - the scoring of the matched
// trace by the workgroup that finishes the match, in the same launch
int launch_match(const moei_eamc* c, const int32_t* d_eam, int B, int layer_hi, int32_t* d_best, float* d_best_sim,
                 float* d_sims, const ScoreArgs* score, hipStream_t s);
// the m most similar traces of one query; `score` (with B = m) scores their aggregate
int launch_match_topm(const moei_eamc* c, const int32_t* d_eam, int layer_hi, int m, int32_t* d_top, float* d_top_sim,
                      float* d_sims, const ScoreArgs* score, hipStream_t s);

}  // namespace moei
