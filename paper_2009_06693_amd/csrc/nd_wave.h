// Wave64 and workgroup scan primitives (ballot / shuffle based).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace nd {

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & 63); }
__device__ __forceinline__ int wave_id() { return (int)(threadIdx.x >> 6); }

__device__ __forceinline__ uint64_t lanes_below(int lane) { return (1ull << lane) - 1ull; }

// A value that is the same in every lane of the wavefront, moved to scalar registers: the compiler
// cannot see that (threadIdx.x >> 6 and whatever is loaded through it look divergent), and loops
// and branches on such a value would otherwise run on execution masks instead of scalar branches.
__device__ __forceinline__ uint32_t wave_uniform(uint32_t x) {
    return (uint32_t)__builtin_amdgcn_readfirstlane((int)x);
}
__device__ __forceinline__ int32_t wave_uniform(int32_t x) { return __builtin_amdgcn_readfirstlane(x); }
__device__ __forceinline__ uint64_t wave_uniform(uint64_t x) {
    return ((uint64_t)wave_uniform((uint32_t)(x >> 32)) << 32) | wave_uniform((uint32_t)x);
}
__device__ __forceinline__ int64_t wave_uniform(int64_t x) { return (int64_t)wave_uniform((uint64_t)x); }

// Inclusive sum across the 64 lanes of a wavefront for 32-bit values, in six DPP additions: four
// shifts inside the rows of 16 lanes (a lane outside the row contributes 0), then lane 15 of rows
// 0 and 2 into rows 1 and 3, then lane 31 into rows 2 and 3.  Every lane must be active.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_moved(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROW_MASK, 0xf, true);
}
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v, int /*lane*/) {
    v += dpp_moved<0x111, 0xf>(v);  // row_shr:1
    v += dpp_moved<0x112, 0xf>(v);  // row_shr:2
    v += dpp_moved<0x114, 0xf>(v);  // row_shr:4
    v += dpp_moved<0x118, 0xf>(v);  // row_shr:8
    v += dpp_moved<0x142, 0xa>(v);  // row_bcast:15 into rows 1 and 3
    v += dpp_moved<0x143, 0xc>(v);  // row_bcast:31 into rows 2 and 3
    return v;
}

// The lanes of the wavefront that hold digit d (among the lanes of `candidates`): one ballot per
// digit bit, the bit spread over the lane's word so that "my bit equals theirs" is one XNOR per half.
template <int BITS>
__device__ __forceinline__ uint64_t digit_peers_fixed(uint32_t d, uint64_t candidates) {
    uint32_t lo = (uint32_t)candidates, hi = (uint32_t)(candidates >> 32);
#pragma unroll
    for (int b = 0; b < BITS; ++b) {
        const uint32_t mine = (uint32_t)__builtin_amdgcn_sbfe((int)d, (uint32_t)b, 1u);  // all ones or zero
        const uint64_t theirs = __ballot(mine != 0u);
        lo &= ~((uint32_t)theirs ^ mine);
        hi &= ~((uint32_t)(theirs >> 32) ^ mine);
    }
    return ((uint64_t)hi << 32) | lo;
}
__device__ __forceinline__ uint64_t digit_peers(uint32_t d, uint64_t candidates, int bits) {
    switch (bits) {  // the same for the whole launch
        case 8: return digit_peers_fixed<8>(d, candidates);
        case 7: return digit_peers_fixed<7>(d, candidates);
        case 6: return digit_peers_fixed<6>(d, candidates);
        case 5: return digit_peers_fixed<5>(d, candidates);
        case 4: return digit_peers_fixed<4>(d, candidates);
        case 3: return digit_peers_fixed<3>(d, candidates);
        case 2: return digit_peers_fixed<2>(d, candidates);
        default: return digit_peers_fixed<1>(d, candidates);
    }
}

// Inclusive scan across the 64 lanes of a wavefront (any type, through shuffles).
template <typename T>
__device__ __forceinline__ T wave_inclusive_scan(T x, int lane) {
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        T y = __shfl_up(x, d, 64);
        if (lane >= d) x += y;
    }
    return x;
}

// Exclusive scan over a workgroup of THREADS lanes (THREADS a multiple of 64, at
// most 1024).  `tmp` is shared memory with at least THREADS/64 + 1 entries.
// Returns the exclusive prefix of x; *total receives the workgroup's sum.
// Contains two barriers; every thread of the workgroup must call it.
template <typename T, int THREADS>
__device__ __forceinline__ T block_exclusive_scan(T x, T* tmp, T* total) {
    constexpr int W = THREADS / 64;
    const int lane = lane_id(), wave = wave_id();
    const T incl = wave_inclusive_scan(x, lane);
    if (lane == 63) tmp[wave] = incl;
    __syncthreads();
    if (wave == 0) {
        T w = lane < W ? tmp[lane] : (T)0;
        T wi = wave_inclusive_scan(w, lane);
        if (lane < W) tmp[lane] = wi - w;
        if (lane == W - 1) tmp[W] = wi;
    }
    __syncthreads();
    const T base = tmp[wave];
    *total = tmp[W];
    return base + incl - x;
}

}  // namespace nd
