// Scheduling index (Section 6.1.2 of the paper, "Scheduling"): from the pairs
// sorted by transit, (1) a segmented scan finds the distinct transits with the
// position and size of each one's group of samples, and (2) every transit is
// assigned to one of three classes by the number of neighbours it must
// produce; the workgroup and grid classes get compacted work lists, and the
// position of a transit in its list is its scheduling index.  All counts stay
// in device memory (StepCtl): the host never waits for them.
#include "nd_common.h"
#include "nd_wave.h"

namespace nd {

size_t seg_scratch_bytes(int64_t n_slots) {
    const int64_t tiles = (n_slots + kSegTile - 1) / kSegTile + 1;
    return (size_t)tiles * (kSegThreads / 64) * sizeof(uint32_t);  // one head count per wavefront
}

namespace {

constexpr int kSegWaves = kSegThreads / 64;
constexpr int kSegPerWave = kSegTile / kSegWaves;

// A pair is the head of its group when its transit differs from the previous pair's.
__device__ __forceinline__ bool is_head(const int32_t* __restrict__ keys, int64_t idx, int64_t P,
                                        int lane, int32_t* key_out) {
    int32_t k = idx < P ? keys[idx] : -2;
    int32_t prev = __shfl_up(k, 1, 64);
    if (lane == 0) prev = (idx > 0 && idx < P) ? keys[idx - 1] : -3;
    *key_out = k;
    return idx < P && k != prev;
}

// Heads among the 1,024 consecutive pairs of every wavefront; a lane looks at four
// consecutive keys per round (one 16-byte load) and compares them with each other, the first
// with the last key of the lane before.
__global__ __launch_bounds__(kSegThreads) void seg_count_kernel(const int32_t* __restrict__ keys,
                                                                const StepCtl* __restrict__ ctl,
                                                                uint32_t* __restrict__ wave_counts,
                                                                uint32_t* __restrict__ heavy_bits,
                                                                int64_t bit_words) {
    const int lane = lane_id(), wave = wave_id();
    // the marks of the previous step's heavy transits go (this step's are set by classify_kernel)
    if (heavy_bits != nullptr)
        for (int64_t w = (int64_t)blockIdx.x * kSegThreads + threadIdx.x; w < bit_words;
             w += (int64_t)gridDim.x * kSegThreads)
            heavy_bits[w] = 0u;
    const int64_t P = ctl->P;
    const int64_t base = (int64_t)blockIdx.x * kSegTile + (int64_t)wave * kSegPerWave;
    uint32_t cnt = 0;
    if (base + kSegPerWave <= P) {
        // a whole chunk (all but the last): every load is issued before the first comparison, and
        // the key before a round's first is the last key of the round before, passed in a register
        constexpr int kRounds = kSegPerWave / 256;
        const int4* kp = reinterpret_cast<const int4*>(keys + base) + lane;  // base is a multiple of 4
        int4 v[kRounds];
#pragma unroll
        for (int r = 0; r < kRounds; ++r) v[r] = kp[r * 64];
        int32_t before = base > 0 ? keys[base - 1] : -3;  // the same in all lanes
#pragma unroll
        for (int r = 0; r < kRounds; ++r) {
            int32_t prev = __shfl_up(v[r].w, 1, 64);
            if (lane == 0) prev = before;
            cnt += (v[r].x != prev ? 1u : 0u) + (v[r].y != v[r].x ? 1u : 0u) + (v[r].z != v[r].y ? 1u : 0u) +
                   (v[r].w != v[r].z ? 1u : 0u);
            before = __builtin_amdgcn_readlane(v[r].w, 63);
        }
    } else if (base < P) {
#pragma unroll
        for (int r = 0; r < kSegPerWave / 256; ++r) {
            const int64_t idx = base + r * 256 + lane * 4;
            int32_t k[4] = {-2, -2, -2, -2};
            if (idx + 3 < P) {
                const int4 v = *reinterpret_cast<const int4*>(keys + idx);  // idx is a multiple of 4
                k[0] = v.x; k[1] = v.y; k[2] = v.z; k[3] = v.w;
            } else {
                for (int e = 0; e < 4; ++e)
                    if (idx + e < P) k[e] = keys[idx + e];
            }
            int32_t prev = __shfl_up(k[3], 1, 64);
            if (lane == 0) prev = (idx > 0 && idx < P) ? keys[idx - 1] : -3;
            cnt += (idx < P && k[0] != prev) ? 1u : 0u;
            cnt += (idx + 1 < P && k[1] != k[0]) ? 1u : 0u;
            cnt += (idx + 2 < P && k[2] != k[1]) ? 1u : 0u;
            cnt += (idx + 3 < P && k[3] != k[2]) ? 1u : 0u;
        }
    }
    const uint32_t incl = wave_inclusive_scan(cnt, lane);
    if (lane == 63) wave_counts[(int64_t)blockIdx.x * kSegWaves + wave] = incl;
}

// One workgroup: exclusive scan of the per-wavefront head counts in place (a thread takes the
// four counts of one tile), publishes the number of groups and resets the class counters of
// the step.
static_assert(kSegWaves == 4, "seg_scan_kernel reads one tile's counts as a uint4");
__global__ __launch_bounds__(1024) void seg_scan_kernel(uint32_t* __restrict__ wave_counts,
                                                        int64_t num_tiles, StepCtl* __restrict__ ctl,
                                                        int32_t* __restrict__ g_start) {
    __shared__ uint32_t tmp[18];
    uint32_t carry = 0;
    for (int64_t base = 0; base < num_tiles; base += 1024) {
        const int64_t i = base + threadIdx.x;
        uint4 c = make_uint4(0u, 0u, 0u, 0u);
        if (i < num_tiles) c = reinterpret_cast<const uint4*>(wave_counts)[i];
        uint32_t total;
        const uint32_t ex = carry + block_exclusive_scan<uint32_t, 1024>(c.x + c.y + c.z + c.w, tmp, &total);
        if (i < num_tiles)
            reinterpret_cast<uint4*>(wave_counts)[i] = make_uint4(ex, ex + c.x, ex + c.x + c.y, ex + c.x + c.y + c.z);
        carry += total;
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        ctl->U = carry;
        ctl->n_wg = 0;
        ctl->n_grid = 0;
        ctl->n_chunks = 0;
        ctl->heavy_draws = 0;
        ctl->n_staged = 0;
        ctl->wg_cursor = 0;
        g_start[carry] = (int32_t)ctl->P;  // sentinel: end of the last group
    }
}

__global__ __launch_bounds__(kSegThreads) void seg_write_kernel(const int32_t* __restrict__ keys,
                                                                const StepCtl* __restrict__ ctl,
                                                                const uint32_t* __restrict__ tile_offs,
                                                                int32_t* __restrict__ g_key,
                                                                int32_t* __restrict__ g_start) {
    const int lane = lane_id(), wave = wave_id();
    const int64_t P = ctl->P;
    const int64_t base = (int64_t)blockIdx.x * kSegTile + (int64_t)wave * kSegPerWave;
    if (base >= P) return;
    uint32_t gid = tile_offs[(int64_t)blockIdx.x * kSegWaves + wave];  // groups that start before this wave
    // group ids by ballot prefix
    if (base + kSegPerWave <= P) {
        // a whole chunk (all but the last): all keys are requested first; the key before a round's
        // first is the last key of the round before, passed in a register
        constexpr int kRounds = kSegPerWave / 64;
        const int32_t* kp = keys + base + lane;
        int32_t k[kRounds];
#pragma unroll
        for (int r = 0; r < kRounds; ++r) k[r] = kp[r * 64];
        int32_t before = base > 0 ? keys[base - 1] : -3;  // the same in all lanes
#pragma unroll
        for (int r = 0; r < kRounds; ++r) {
            int32_t prev = __shfl_up(k[r], 1, 64);
            if (lane == 0) prev = before;
            const bool h = k[r] != prev;
            const uint64_t bal = __ballot(h);
            if (h) {
                const uint32_t g = gid + __builtin_amdgcn_mbcnt_hi((uint32_t)(bal >> 32),
                                                                   __builtin_amdgcn_mbcnt_lo((uint32_t)bal, 0u));
                g_key[g] = k[r];
                g_start[g] = (int32_t)(base + r * 64 + lane);
            }
            gid += (uint32_t)__popcll(bal);
            before = __builtin_amdgcn_readlane(k[r], 63);
        }
        return;
    }
    for (int r = 0; r < kSegPerWave / 64; ++r) {
        int32_t k;
        const int64_t idx = base + r * 64 + lane;
        const bool h = is_head(keys, idx, P, lane, &k);
        const uint64_t bal = __ballot(h);
        if (h) {
            const uint32_t g = gid + (uint32_t)__popcll(bal & lanes_below(lane));
            g_key[g] = k;
            g_start[g] = (int32_t)idx;
        }
        gid += (uint32_t)__popcll(bal);
    }
}


// Few pairs (a walk on a small graph): the three kernels above in one workgroup of 16
// wavefronts, each taking a sixteenth of the pairs - heads per wavefront, their prefix over
// the wavefronts, then the group table.  Saves two launches per step where a launch costs
// more than the work.
constexpr int64_t kSegSmallLimit = 8192;
__global__ __launch_bounds__(1024) void seg_small_kernel(const int32_t* __restrict__ keys,
                                                         StepCtl* __restrict__ ctl,
                                                         int32_t* __restrict__ g_key,
                                                         int32_t* __restrict__ g_start,
                                                         uint32_t* __restrict__ heavy_bits,
                                                         int64_t bit_words) {
    __shared__ uint32_t wsum[16];
    const int lane = lane_id(), wave = wave_id();
    if (heavy_bits != nullptr)  // the marks of the previous step's heavy transits go
        for (int64_t w = threadIdx.x; w < bit_words; w += 1024) heavy_bits[w] = 0u;
    const int64_t P = ctl->P;
    const int64_t per_wave = ((P + 15) / 16 + 63) / 64 * 64;
    const int64_t wb = (int64_t)wave * per_wave;
    const int64_t we = wb + per_wave < P ? wb + per_wave : P;
    uint32_t cnt = 0;
    for (int64_t i = wb; i < we; i += 64) {
        int32_t k;
        cnt += (uint32_t)__popcll(__ballot(is_head(keys, i + lane, P, lane, &k)));
    }
    if (lane == 0) wsum[wave] = cnt;
    __syncthreads();
    uint32_t gid = 0, total = 0;
    for (int w = 0; w < 16; ++w) {
        gid += w < wave ? wsum[w] : 0u;
        total += wsum[w];
    }
    for (int64_t i = wb; i < we; i += 64) {
        int32_t k;
        const bool h = is_head(keys, i + lane, P, lane, &k);
        const uint64_t bal = __ballot(h);
        if (h) {
            const uint32_t g = gid + (uint32_t)__popcll(bal & lanes_below(lane));
            g_key[g] = k;
            g_start[g] = (int32_t)(i + lane);
        }
        gid += (uint32_t)__popcll(bal);
    }
    if (threadIdx.x == 0) {
        ctl->U = total;
        ctl->n_wg = 0;
        ctl->n_grid = 0;
        ctl->n_chunks = 0;
        ctl->heavy_draws = 0;
        ctl->n_staged = 0;
        ctl->wg_cursor = 0;
        g_start[total] = (int32_t)P;  // sentinel: end of the last group
    }
}

// One lane per transit, 1024 transits per workgroup round.  List space is
// reserved with one atomic per class per round (counts are combined with wave64
// ballots and a small LDS table first), so list order follows transit order
// inside a round.  Workgroup- and grid-class transits are marked in heavy_bits
// so that the sub-wavefront kernel leaves their pairs alone.
__global__ __launch_bounds__(256) void classify_kernel(const int32_t* __restrict__ g_key,
                                                       const int32_t* __restrict__ g_start,
                                                       StepCtl* __restrict__ ctl, SchedParams sp,
                                                       int32_t* __restrict__ list_wg,
                                                       int32_t* __restrict__ chunk_gid,
                                                       int32_t* __restrict__ chunk_idx,
                                                       int64_t max_chunks,
                                                       uint32_t* __restrict__ heavy_bits) {
    constexpr int R = 4;
    __shared__ uint32_t s_wg[R * 4 + 1], s_ch[R * 4 + 1], s_stat[2], s_grid[R * 4], s_heavy[R * 4];
    const int lane = lane_id(), wave = wave_id();
    const int64_t U = ctl->U;
    const int64_t stride = (int64_t)gridDim.x * 256 * R;
    for (int64_t base = (int64_t)blockIdx.x * 256 * R; base < U; base += stride) {
        int cls[R];
        uint32_t draws[R], wgrank[R], chexcl[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int64_t g = base + r * 256 + threadIdx.x;
            cls[r] = -1;
            draws[r] = 0;
            if (g < U) {
                draws[r] = (uint32_t)(g_start[g + 1] - g_start[g]) * (uint32_t)sp.m;
                cls[r] = class_of(draws[r], sp);
            }
            const uint64_t b_wg = __ballot(cls[r] == ND_CLASS_WORKGROUP);
            wgrank[r] = (uint32_t)__popcll(b_wg & lanes_below(lane));
            const uint32_t chunks = cls[r] == ND_CLASS_GRID
                                        ? (draws[r] + (uint32_t)sp.wg_max - 1u) / (uint32_t)sp.wg_max
                                        : 0u;
            const uint32_t incl = wave_inclusive_scan(chunks, lane);
            chexcl[r] = incl - chunks;
            const uint32_t heavy = wave_inclusive_scan(cls[r] == ND_CLASS_SUBWAVE ? 0u : draws[r], lane);
            const uint64_t b_grid = __ballot(cls[r] == ND_CLASS_GRID);
            if (lane == 63) {
                s_wg[r * 4 + wave] = (uint32_t)__popcll(b_wg);
                s_ch[r * 4 + wave] = incl;
                s_grid[r * 4 + wave] = (uint32_t)__popcll(b_grid);
                s_heavy[r * 4 + wave] = heavy;
            }
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            uint32_t run_wg = 0, run_ch = 0, n_grid = 0, heavy = 0;
            for (int i = 0; i < R * 4; ++i) {
                const uint32_t a = s_wg[i], b = s_ch[i];
                s_wg[i] = run_wg;
                s_ch[i] = run_ch;
                run_wg += a;
                run_ch += b;
                n_grid += s_grid[i];
                heavy += s_heavy[i];
            }
            // a round without workgroup- or grid-class transits touches no global counter
            s_stat[0] = run_wg ? atomicAdd(&ctl->n_wg, run_wg) : 0u;
            s_stat[1] = run_ch ? atomicAdd(&ctl->n_chunks, run_ch) : 0u;
            if (n_grid) atomicAdd(&ctl->n_grid, n_grid);
            if (heavy) atomicAdd(&ctl->heavy_draws, heavy);
        }
        __syncthreads();
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int64_t g = base + r * 256 + threadIdx.x;
            if (cls[r] == ND_CLASS_WORKGROUP) {
                list_wg[s_stat[0] + s_wg[r * 4 + wave] + wgrank[r]] = (int32_t)g;
            } else if (cls[r] == ND_CLASS_GRID) {
                const uint32_t cbase = s_stat[1] + s_ch[r * 4 + wave] + chexcl[r];
                const uint32_t chunks = (draws[r] + (uint32_t)sp.wg_max - 1u) / (uint32_t)sp.wg_max;
                for (uint32_t c = 0; c < chunks; ++c) {
                    if ((int64_t)(cbase + c) < max_chunks) {  // capacity is sized so this always holds
                        chunk_gid[cbase + c] = (int32_t)g;
                        chunk_idx[cbase + c] = (int32_t)c;
                    }
                }
            }
            if (heavy_bits != nullptr &&
                (cls[r] == ND_CLASS_WORKGROUP || cls[r] == ND_CLASS_GRID)) {
                const uint32_t v = (uint32_t)g_key[g];
                atomicOr(&heavy_bits[v >> 5], 1u << (v & 31u));
            }
        }
        __syncthreads();  // the LDS table is rewritten by the next round
    }
}

}  // namespace

int build_groups(const int32_t* sorted_keys, int64_t max_pairs, StepCtl* ctl, int32_t* g_key,
                 int32_t* g_start, uint32_t* tile_counts, uint32_t* heavy_bits, int64_t bit_words,
                 hipStream_t stream) {
    if (max_pairs <= kSegSmallLimit) {
        hipLaunchKernelGGL(seg_small_kernel, dim3(1), dim3(1024), 0, stream, sorted_keys, ctl, g_key, g_start,
                           heavy_bits, bit_words);
        ND_HIP_CHECK(hipGetLastError());
        return ND_OK;
    }
    int64_t tiles = (max_pairs + kSegTile - 1) / kSegTile;
    if (tiles < 1) tiles = 1;
    hipLaunchKernelGGL(seg_count_kernel, dim3((unsigned)tiles), dim3(kSegThreads), 0, stream,
                       sorted_keys, ctl, tile_counts, heavy_bits, bit_words);
    hipLaunchKernelGGL(seg_scan_kernel, dim3(1), dim3(1024), 0, stream, tile_counts, tiles, ctl, g_start);
    hipLaunchKernelGGL(seg_write_kernel, dim3((unsigned)tiles), dim3(kSegThreads), 0, stream,
                       sorted_keys, ctl, tile_counts, g_key, g_start);
    ND_HIP_CHECK(hipGetLastError());
    return ND_OK;
}

int classify_groups(const int32_t* g_key, const int32_t* g_start, int64_t max_groups, StepCtl* ctl,
                    const SchedParams& sp, int32_t* list_wg, int32_t* chunk_gid, int32_t* chunk_idx,
                    int64_t max_chunks, uint32_t* heavy_bits, hipStream_t stream) {
    int64_t blocks = (max_groups + 1023) / 1024;
    if (blocks < 1) blocks = 1;
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(classify_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, g_key, g_start,
                       ctl, sp, list_wg, chunk_gid, chunk_idx, max_chunks, heavy_bits);
    ND_HIP_CHECK(hipGetLastError());
    return ND_OK;
}

}  // namespace nd
