// Device-side random numbers and integer helpers.
//
// Philox4x32-10 (Salmon, Moraes, Dror, Shaw, "Parallel random numbers: as easy
// as 1, 2, 3", SC'11): a counter-based generator, so a draw is a pure function
// of (seed, sample, slot, step, attempt) and the grouping of samples by transit
// (Section 5.2 of the NextDoor paper) cannot change what is drawn.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "nd_common.h"

namespace nd {

struct Rand4 {
    uint32_t r0, r1, r2, r3;
};

__device__ __forceinline__ Rand4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                               uint32_t k0, uint32_t k1) {
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return Rand4{c0, c1, c2, c3};
}

// Counter layout of every draw: (sample id, slot within the sample, step, attempt).
__device__ __forceinline__ Rand4 draw4(uint64_t seed, uint32_t sample_id, uint32_t slot,
                                       uint32_t step, uint32_t attempt) {
    return philox4x32_10(sample_id, slot, step, attempt, (uint32_t)seed, (uint32_t)(seed >> 32));
}

__device__ __forceinline__ uint32_t mulhi32(uint32_t a, uint32_t b) { return __umulhi(a, b); }
__device__ __forceinline__ uint64_t mulhi64(uint64_t a, uint64_t b) { return __umul64hi(a, b); }
__device__ __forceinline__ uint64_t cat64(uint32_t hi, uint32_t lo) { return ((uint64_t)hi << 32) | lo; }

__device__ __forceinline__ uint32_t fastdiv(uint32_t n, const FastDiv& f) {
    return f.d == 1 ? n : (__umulhi(n, f.magic) >> f.shift);
}

}  // namespace nd
