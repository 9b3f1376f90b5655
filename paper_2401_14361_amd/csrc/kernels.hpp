// Internal interfaces between the translation units of the moei library.
#pragma once

#include <vector>

#include "common.hpp"

namespace moei {

// ----------------------------------------------------------------- route.hip
struct RouteFusedArgs {
    const void* W;               // router matrix [E][H] in the weight dtype
    const float* bias;           // [E] or null
    const void* x;               // [H] in the weight dtype
    int H, vec_ok;
    float* logits;               // [E] scratch, written then read by the last wavefront
    unsigned* ticket;            // arrival counter, zero between launches
    int E, k, renorm;
    int32_t* idx;                // [k] out
    float* w;                    // [k] out
    int32_t* eam;                // the request's EAM [L*E]; row `layer` is updated in place
    int32_t* snap;               // [L*E] copy of the updated EAM for the match on the side stream
    int LE, layer;
    const int32_t* slot_of_row;  // slot_of + layer*E
    int n_shared, shared_base;   // shared slot ids: shared_base + s
    int32_t* slot_ids;           // [k + n_shared] out
    float* gate;                 // [k + n_shared] out
    int32_t* flags;              // error flags (bit 1: pick not resident)
    int32_t* host_idx;           // [k] pinned host memory that receives the picks too (synchronous step), or null
};
int launch_route_fused(RouteFusedArgs a, int wdtype, hipStream_t s);
int launch_gather_slots(const int32_t* d_idx, int k, const int32_t* d_slot_of_row, int32_t* d_slot_ids,
                        int32_t* d_flags, hipStream_t s);

// ------------------------------------------------------------------ ffn.hip
struct FfnScratch {
    float* d_part = nullptr;  // [n_part][H] workgroup partial sums of y
    int n_part = 0;           // = workgroups of the fused kernel (one per compute unit)
    int n_act_max = 0;
};
int ffn_scratch_alloc(const moei_model_desc& d, int n_act_max, FfnScratch* out);
void ffn_scratch_free(FfnScratch* s);
int launch_expert_ffn(const moei_model_desc& d, const void* d_pool, size_t slot_elems, int n_slots_total,
                      const FfnScratch& scr, const int32_t* d_slot_ids, const float* d_gate_w, int n_act,
                      const void* d_x, float* d_y, int32_t* d_flags, hipStream_t s);

// the same with the partial rows in a static device array (no allocation anywhere on the path)
constexpr size_t kStaticPartFloats = (size_t)256 * 5120;  // 5 MiB: 256 workgroups x H = 5120
int static_part_ptr(float** out);
int launch_expert_ffn_static(const moei_model_desc& d, const void* d_pool, size_t slot_elems, int n_slots_total,
                             int n_part, const int32_t* d_slot_ids, const float* d_gate_w, int n_act, const void* d_x,
                             float* d_y, int32_t* d_flags, hipStream_t s);

// decode batch B > 1: tokens grouped per activated expert
int grouped_max_items(const moei_model_desc& d);
size_t grouped_item_bytes();
size_t grouped_part_floats(const moei_model_desc& d);
int launch_expert_ffn_grouped(const moei_model_desc& d, const void* d_pool, size_t slot_elems, void* d_items,
                              int32_t* d_n_items, float* d_part, const int32_t* d_slot_of_row, int shared_base,
                              const int32_t* d_idx, const float* d_w, int B, const void* d_x, float* d_y,
                              int32_t* d_flags, hipStream_t s);

// ---------------------------------------------------------------- prefill.hip
struct PrefillScratch {
    int n_max = 0;              // tokens the buffers are sized for
    int32_t* d_idx = nullptr;   // [n_max][k] picks
    float* d_w = nullptr;       // [n_max][k] gate weights
    int32_t* d_perm = nullptr;  // [n_max*k] tokens grouped per expert
    float* d_pgate = nullptr;   // [n_max*k] their gate weights
    int32_t* d_where = nullptr;  // [n_max*k] row of every (token, pick)
    void* d_items = nullptr;
    int32_t* d_meta = nullptr;  // [2]
    uint16_t* d_act = nullptr;  // [n_max*(k+n_shared)][I] activations, bf16
    float* d_yc = nullptr;      // [n_max*(k+n_shared)][H] contributions
};
int prefill_check(const moei_model_desc& d);
size_t prefill_item_bytes();
int prefill_max_items(const moei_model_desc& d, int n_max);
size_t prefill_rows(const moei_model_desc& d, int n_max);
int launch_prefill(const moei_model_desc& d, const PrefillScratch& ps, const void* d_pool, size_t slot_elems,
                   int n_slots_total, const int32_t* d_slot_of_row, int shared_base, int32_t* d_eam_row,
                   const void* d_router_w, const float* d_router_bias, const void* d_X, int n, float* d_Y,
                   int32_t* d_flags, hipStream_t s);

}  // namespace moei

// The EAM collection (Sec. 4.5): traces layer-major on the device.
struct moei_eamc {
    moei_model_desc d{};
    int32_t n_cap = 0;
    int32_t N = 0;
    int32_t cell_bytes = 4;
    int32_t max_cell = 0;                // no stored cell has ever been larger (kept by load and insert)
    void* d_traces = nullptr;            // [L][n_cap][E] cells
    unsigned long long* d_norm2 = nullptr;  // [n_cap] squared norms of the flattened traces
    unsigned long long* d_part = nullptr;   // [B_max][lsplit_max][n_cap] partial dot products
    int32_t lsplit_max = 0;
    unsigned long long* d_cand = nullptr;   // [B_max][workgroups][2] per-workgroup winners (dot, norm)
    int32_t* d_cand_idx = nullptr;          // [B_max][workgroups] their trace indices
    unsigned* d_ticket = nullptr;           // [B_max] arrival counters of the final pick
    // priority scratch
    unsigned long long* d_keys = nullptr;  // [2][L*E] sort keys (prefetch, evict)
};

namespace moei {
constexpr int kMaxMatchBatch = 16;
}
