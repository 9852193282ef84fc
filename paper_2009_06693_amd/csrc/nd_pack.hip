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

// Measurement only: n_runs runs of run_len ints, one lane per int, run r at run position
// mix(r) (a bijection of [0, n_runs) for a power of two: odd multiplications and xor-shifts) or at r.
__device__ __forceinline__ uint32_t probe_mix(uint32_t x, uint32_t mask, int half) {
    x = (x * 0x9E3779B1u) & mask;
    x ^= x >> half;
    x = (x * 0x85EBCA6Bu) & mask;
    x ^= x >> half;
    x = (x * 0xC2B2AE35u) & mask;
    x ^= x >> half;
    return x;
}

__global__ __launch_bounds__(256) void probe_store_runs_kernel(int32_t* __restrict__ out, uint32_t n_runs,
                                                               FastDiv div_len, int scattered, int half) {
    // a 256-lane round covers 256 / run_len whole runs; a lane keeps its place j inside the run
    const uint32_t len = div_len.d;
    const uint32_t r_local = fastdiv(threadIdx.x, div_len), j = threadIdx.x - r_local * len;
    const uint32_t per_round = 256u / len;
    if (r_local >= per_round) return;
    for (uint64_t r = (uint64_t)blockIdx.x * per_round + r_local; r < n_runs; r += (uint64_t)gridDim.x * per_round) {
        const uint32_t dst = scattered ? probe_mix((uint32_t)r, n_runs - 1u, half) : (uint32_t)r;
        out[(uint64_t)dst * len + j] = (int32_t)r;
    }
}

}  // namespace

int probe_store_runs(int32_t* out, int64_t n_runs, int32_t run_len, int scattered, hipStream_t stream) {
    if (n_runs == 0) return ND_OK;
    int bits = 0;
    while ((1ll << bits) < n_runs) ++bits;
    hipLaunchKernelGGL(probe_store_runs_kernel, dim3(2048), dim3(256), 0, stream, out, (uint32_t)n_runs,
                       make_fastdiv((uint32_t)run_len), scattered, bits / 2 + 1);
    ND_HIP_CHECK(hipGetLastError());
    return ND_OK;
}

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
