// Arguments of the sampling kernels and their host-side launchers.
#pragma once

#include "nd_common.h"

namespace nd {

enum : int { kDrawUniform = 0, kDrawWeighted = 1, kDrawNode2vec = 2 };

// Everything a lane needs to make the draws of one step; passed by value.
struct DrawArgs {
    uint64_t seed;
    uint64_t ppr_thr;             // walk ends when R3 < ppr_thr; 0 = never
    uint32_t sample_base;         // id of the call's first sample
    uint32_t step;
    uint32_t m;                   // draws per (transit, sample) pair
    FastDiv div_m;                // by m
    FastDiv div_wprev;            // by the number of transit slots per sample
    uint32_t b_ret, b_com, b_far, b_max;  // node2vec biases, Q16
    int32_t max_attempts;
    int32_t has_prev;             // node2vec: a previous transit exists (step > 0)
    int32_t use_weights;
    int32_t lds_policy;
    const int32_t* prev_transit;  // node2vec: previous transit of every sample
    int32_t* out;                 // this step's output array
};

int sample_step_tp(const Graph& gr, int draw, const DrawArgs& a, const SchedParams& sp, StepCtl* ctl,
                   const int32_t* g_key, const int32_t* g_start, const int32_t* vals,
                   const int32_t* list_wg, const int32_t* chunk_gid, const int32_t* chunk_idx,
                   int64_t max_groups, int64_t max_wg, int64_t max_chunks, int64_t cap_wg,
                   int64_t cap_chunks, int num_cus, hipStream_t stream);

int sample_step_sp(const Graph& gr, int draw, const DrawArgs& a, const int32_t* src, int64_t n_slots,
                   int check_roots, uint32_t* status, hipStream_t stream);

// Layer (collective) sampling: one step for all samples.
struct LayerArgs {
    uint64_t seed;
    uint32_t sample_base;
    uint32_t step;
    uint32_t n_prev;              // transit slots per sample at this step
    uint32_t m;                   // draws per sample
    const int32_t* transits;      // num_samples * n_prev (roots or the previous layer)
    int32_t* out;                 // num_samples * m
    int32_t check_roots;
    uint32_t* status;
};
int layer_step(const Graph& gr, const LayerArgs& a, int64_t num_samples, hipStream_t stream);

}  // namespace nd
