// Host-side launcher that gathers the per-step arrays into one record per sample.
#pragma once

#include "nd_common.h"

namespace nd {

// step_out and step_len are host arrays with num_steps entries; every step_len[i] is a multiple
// of S and below 2^31; samples receives S records of sum(step_len) / S ints.
int pack_samples(const int32_t* const* step_out, int32_t num_steps, const int64_t* step_len, int64_t S,
                 int32_t* samples, hipStream_t stream);

// Measurement: n_runs (a power of two below 2^31) runs of run_len (1..32) ints, scattered or in order.
int probe_store_runs(int32_t* out, int64_t n_runs, int32_t run_len, int scattered, hipStream_t stream);

}  // namespace nd
