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

// Device arrays and launch bounds of one transit-parallel step.
struct TpStep {
    StepCtl* ctl;
    const int32_t* keys;       // pairs sorted by transit: transit ...
    const int32_t* vals;       // ... and slot in the previous step's array
    const int32_t* g_key;      // distinct transits
    const int32_t* g_start;    // first pair of each transit's group (+ sentinel)
    const int32_t* list_wg;    // workgroup-class transits
    const int32_t* chunk_gid;  // grid-class chunks: transit ...
    const int32_t* chunk_idx;  // ... and chunk number
    uint32_t* heavy_bits;      // one bit per vertex: set for workgroup / grid class transits
    int64_t max_draws;         // host-known upper bounds that size the launches
    int64_t max_wg, max_chunks;
    int64_t cap_wg, cap_chunks;
};

int sample_step_tp(const Graph& gr, int draw, const DrawArgs& a, const SchedParams& sp,
                   const TpStep& t, hipStream_t stream);

int sample_step_sp(const Graph& gr, int draw, const DrawArgs& a, const int32_t* src, int64_t n_slots,
                   int check_roots, uint32_t* status, hipStream_t stream);

// Multi-dimensional walk (Section 3): the sample's root set lives in `state` (S * R vertices).
// init copies the roots (out-of-range ones become NULL and are reported), select writes the
// step's transit of every sample (the root picked with R2 of the step's generator call) and
// update puts the vertex the step added in the picked root's place.
int multirw_init(const Graph& gr, const int32_t* roots, int64_t n, int32_t* state, uint32_t* status,
                 hipStream_t stream);
int multirw_select(const int32_t* state, int64_t S, uint32_t R, uint64_t seed, uint32_t sample_base,
                   uint32_t step, int32_t* transits, hipStream_t stream);
int multirw_update(int32_t* state, int64_t S, uint32_t R, uint64_t seed, uint32_t sample_base,
                   uint32_t step, const int32_t* added, hipStream_t stream);

// Random walks grouped per window of samples (nd_walk.hip): all num_steps steps of DeepWalk, PPR,
// node2vec or the multi-dimensional walk, one launch per 128 steps.  d carries the draw's
// constants (seed, sample_base, PPR threshold, node2vec biases, LDS policy); window is 256, 1024 or
// 2048; heavy_min the number of pairs of one transit inside a window from which the whole
// workgroup serves it; ctl (may be null) receives per-step counters.
int walk_window_auto(int64_t S);
int walk_windows(const Graph& gr, int draw, bool multirw, const DrawArgs& d, int64_t S, int32_t num_steps,
                 int window, uint32_t heavy_min, int force_class, const int32_t* roots, int check_roots,
                 int32_t* const* step_out, uint32_t* status, StepCtl* ctl, int32_t* mrw_state, uint32_t R,
                 hipStream_t stream);

// Unique neighbours (Section 6.3) for one k-hop step whose first draw round has already been
// written to `out`: per sample, duplicates are removed (the lowest slot keeps the vertex) and
// the slots that lost draw again, sample-parallel, for rounds - 1 further attempts.
struct UniqueArgs {
    uint64_t seed;
    uint32_t sample_base;
    uint32_t step;
    uint32_t W;               // slots per sample at this step (at most ND_MAX_UNIQUE_SLOTS)
    uint32_t W_prev;          // slots per sample of the previous step (1 at step 0)
    FastDiv div_m;            // slot j descends from slot j / m of the previous step
    int32_t rounds;
    const int32_t* parents;   // roots (step 0) or the previous step's output
    int32_t* out;
};
int unique_step(const Graph& gr, const UniqueArgs& a, int64_t num_samples, hipStream_t stream);

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
    int32_t use_weights;          // entries weigh w_q(v,u) instead of c(v)
    uint32_t* status;
};
int layer_step(const Graph& gr, const LayerArgs& a, int64_t num_samples, hipStream_t stream);
// Once per device before the first layer_step (nd_graph_create does it): lifts the kernels' LDS limit.
int layer_prepare();

}  // namespace nd
