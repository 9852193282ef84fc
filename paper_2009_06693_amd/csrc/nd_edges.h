// Host-side launchers for the edges between consecutive layers.
#pragma once

#include "nd_common.h"

namespace nd {

// Once per process and device, before the first count or fill (allows the kernels' LDS size).
int edges_prepare();

size_t edges_workspace_bytes(int64_t num_samples, int32_t n_prev);

// Row sizes and their exclusive scan: row_ptr receives num_samples * n_prev + 1 entries.
// The first word of the workspace is set to 1 if a vertex outside [-1, V) was met.
int edges_count(const Graph& gr, const int32_t* transits, int32_t n_prev, const int32_t* sampled,
                int32_t m, int64_t num_samples, int64_t* row_ptr, void* workspace, hipStream_t stream);

// Writes the rows; entries at or beyond `capacity` are dropped.
int edges_fill(const Graph& gr, const int32_t* transits, int32_t n_prev, const int32_t* sampled,
               int32_t m, int64_t num_samples, const int64_t* row_ptr, int32_t* edge_slot,
               int64_t capacity, hipStream_t stream);

}  // namespace nd
