// Output format 1 of the paper (Section 4.1, "Output format"): one record per
// sample that holds everything the sample gained at all steps, which is what
// consumers of random walks and layer samples read.  The sampling steps write
// one array per step (format 2); this file gathers them into records:
//
//     samples[s][off_i + j] = step_out[i][s * w_i + j],  off_i = w_0 + ... + w_{i-1}
//
// A step with several slots per sample moves runs of w_i ints, which coalesce on
// both sides.  Walk steps (w_i = 1) are a transpose of [steps][samples]; they go
// through an LDS tile of 32 steps x 64 samples so that reads are 256-byte rows of
// a step array and writes are 128-byte pieces of a record.
#include "nd_common.h"
#include "nd_pack.h"
#include "nd_philox.h"

namespace nd {

namespace {

constexpr int kTileSteps = 32;
constexpr int kTileSamples = 64;

struct WalkChunk {
    const int32_t* step[kTileSteps];  // step arrays of this chunk (w = 1)
    int32_t n_steps;                  // used entries
    int32_t first_col;                // record position of the chunk's first step
};

__global__ __launch_bounds__(256) void pack_walk_kernel(WalkChunk c, int64_t S, int64_t rec_len,
                                                        int32_t* __restrict__ samples) {
    __shared__ int32_t tile[kTileSteps][kTileSamples + 1];
    const int64_t s0 = (int64_t)blockIdx.x * kTileSamples;
    const int lane = threadIdx.x & 63, row = threadIdx.x >> 6;  // 4 rows of 64 lanes
    for (int i = row; i < c.n_steps; i += 4) {
        const int64_t s = s0 + lane;
        if (s < S) tile[i][lane] = c.step[i][s];
    }
    __syncthreads();
    // 8 samples x 32 steps per pass: a sample's 32 entries are consecutive in its record
    const int col = threadIdx.x & 31, sub = threadIdx.x >> 5;
    for (int r = sub; r < kTileSamples; r += 8) {
        const int64_t s = s0 + r;
        if (s < S && col < c.n_steps) samples[s * rec_len + c.first_col + col] = tile[col][r];
    }
}

__global__ __launch_bounds__(256) void pack_wide_kernel(const int32_t* __restrict__ src, int64_t n,
                                                        FastDiv div_w, int64_t rec_len, int32_t first_col,
                                                        int32_t* __restrict__ samples) {
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= n) return;
    const uint32_t s = fastdiv((uint32_t)e, div_w);
    const uint32_t j = (uint32_t)e - s * div_w.d;
    samples[(int64_t)s * rec_len + first_col + j] = src[e];
}

}  // namespace

int pack_samples(const int32_t* const* step_out, int32_t num_steps, const int64_t* step_len, int64_t S,
                 int32_t* samples, hipStream_t stream) {
    if (S == 0) return ND_OK;
    int64_t rec_len = 0;
    for (int32_t i = 0; i < num_steps; ++i) rec_len += step_len[i] / S;
    int64_t col = 0;
    int32_t i = 0;
    while (i < num_steps) {
        const int64_t w = step_len[i] / S;
        if (w == 1) {
            WalkChunk c{};
            c.first_col = (int32_t)col;
            while (i < num_steps && step_len[i] / S == 1 && c.n_steps < kTileSteps) {
                c.step[c.n_steps++] = step_out[i];
                ++i;
            }
            col += c.n_steps;
            const int64_t blocks = (S + kTileSamples - 1) / kTileSamples;
            hipLaunchKernelGGL(pack_walk_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, c, S, rec_len,
                               samples);
        } else {
            const int64_t n = step_len[i];
            const int64_t blocks = (n + 255) / 256;
            hipLaunchKernelGGL(pack_wide_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, step_out[i], n,
                               make_fastdiv((uint32_t)w), rec_len, (int32_t)col, samples);
            col += w;
            ++i;
        }
    }
    ND_HIP_CHECK(hipGetLastError());
    return ND_OK;
}

}  // namespace nd
