// Grouping (transit, slot) pairs by transit vertex: a stable least-significant-
// digit radix sort on the transit id, hand-written for gfx950.
//
// This is the first stage of the scheduling index of Section 6.1.2 of the
// paper (the map from every transit to the samples that hold it), which
// Section 8.1 reports as a radix sort of the samples keyed on the transit.
// The paper used a vendor sort; here each pass is three kernels:
//   upsweep    per-tile digit histogram in LDS              (reads 4 B / pair)
//   binscan    per-digit exclusive scan over the tiles
//   downsweep  stable in-tile ranking with wave64 ballots, tile-local reorder
//              in LDS, coalesced scatter                    (reads 8, writes 8 B / pair)
// The first pass is fused with transit enumeration and output compaction: it
// reads the previous step's output array directly (the slot index is the
// implicit value), drops slots without a transit and (in its upsweep) writes
// NULL into the children of those slots, so later passes and the sampling
// kernels only ever see live pairs.
#include "nd_common.h"
#include "nd_philox.h"
#include "nd_wave.h"

namespace nd {

SortPlan make_sort_plan(int64_t n_slots, int64_t V, int group_bits) {
    SortPlan p{};
    int nbits = 1;
    while ((1ll << nbits) < V) ++nbits;
    int shift = 0;
    if (group_bits > 0 && group_bits < nbits) {  // the low bits of the key are left unsorted
        shift = nbits - group_bits;
        nbits = group_bits;
    }
    p.passes = (nbits + kMaxRadixBits - 1) / kMaxRadixBits;
    for (int i = 0; i < p.passes; ++i) {
        // the wider digits go last: pass 0 also carries the slots without a transit, so its tiles
        // hold fewer live pairs and fewer bins keep its scattered runs longer
        p.bits[i] = nbits / p.passes + (i >= p.passes - nbits % p.passes ? 1 : 0);
        p.shift[i] = shift;
        shift += p.bits[i];
    }
    // Small inputs use small tiles: more workgroups in flight and a shorter dependent chain
    // per tile (the sort is latency-bound there); large inputs use large tiles, whose longer
    // per-digit runs make the scatter's stores contiguous.
    p.tile = n_slots <= kSmallSortLimit ? kSmallSortThreads * kSmallSortItems : kSortThreads * kSortItems;
    p.max_tiles = (n_slots + p.tile - 1) / p.tile;
    if (p.max_tiles < 1) p.max_tiles = 1;
    return p;
}

size_t sort_hist_bytes(const SortPlan& p) {
    int maxbits = 0;
    for (int i = 0; i < p.passes; ++i) maxbits = p.bits[i] > maxbits ? p.bits[i] : maxbits;
    // per-(digit, tile) counts followed by the per-digit totals
    return ((size_t)(1 << maxbits) * (size_t)p.max_tiles + 256) * sizeof(uint32_t);
}

namespace {


// FIRST: keys are the raw transit array (negative = no transit), n = n_slots;
// the pass also performs the output compaction's other half: the m children of
// every slot without a transit receive NULL.  A wavefront's 64 consecutive
// slots own 64*m consecutive output entries, which it fills with contiguous
// 16-byte stores; which parent is dead comes from a ballot, not from memory.
// otherwise: keys are live pairs, n = ctl->P.
template <bool FIRST, int THREADS, int ITEMS>
__global__ __launch_bounds__(THREADS) void upsweep_kernel(
    const int32_t* __restrict__ keys, int64_t n_slots, const StepCtl* __restrict__ ctl, int shift,
    int bits, uint32_t* __restrict__ hist, int64_t num_tiles, int32_t V, int check_range,
    uint32_t* __restrict__ status, int32_t* __restrict__ fill_out, FastDiv div_m, int aligned16) {
    __shared__ uint32_t h[1 << kMaxRadixBits];
    const int tid = threadIdx.x, lane = lane_id();
    const int nbins = 1 << bits;
    const uint32_t mask = (uint32_t)nbins - 1u;
    const int64_t n = FIRST ? n_slots : (int64_t)ctl->P;
    constexpr int kTile = THREADS * ITEMS;
    const int64_t base = (int64_t)blockIdx.x * kTile;
    if (tid < nbins) h[tid] = 0;
    __syncthreads();
    bool bad = false;
    if (!FIRST && base < n) {
        // live pairs only: four consecutive keys per lane and load (the tile base is a multiple of 4)
#pragma unroll 4
        for (int i = tid * 4; i < kTile; i += THREADS * 4) {
            const int64_t idx = base + i;
            if (idx + 3 < n) {
                const int4 v = *reinterpret_cast<const int4*>(keys + idx);
                atomicAdd(&h[((uint32_t)v.x >> shift) & mask], 1u);
                atomicAdd(&h[((uint32_t)v.y >> shift) & mask], 1u);
                atomicAdd(&h[((uint32_t)v.z >> shift) & mask], 1u);
                atomicAdd(&h[((uint32_t)v.w >> shift) & mask], 1u);
            } else {
                for (int e = 0; e < 4; ++e)
                    if (idx + e < n) atomicAdd(&h[((uint32_t)keys[idx + e] >> shift) & mask], 1u);
            }
        }
    }
    if (FIRST && base < n) {
        // all of the thread's keys are requested before the first is looked at
        int32_t mine[ITEMS];
        if (base + kTile <= n) {  // a whole tile (all but the last): nothing to test
            const int32_t* kp = keys + base + tid;
#pragma unroll
            for (int r = 0; r < ITEMS; ++r) mine[r] = kp[r * THREADS];
        } else {
#pragma unroll
            for (int r = 0; r < ITEMS; ++r) {
                const int64_t idx = base + r * THREADS + tid;
                mine[r] = idx < n ? keys[idx] : ND_NULL_VERTEX;
            }
        }
#pragma unroll
        for (int r = 0; r < ITEMS; ++r) {
            const int64_t idx = base + r * THREADS + tid;  // a wavefront covers 64 consecutive slots
            int32_t k = mine[r];
            if (idx < n) {
                if (FIRST && (k >= V || k < ND_NULL_VERTEX)) {
                    bad = true;
                    k = ND_NULL_VERTEX;
                }
                if (k >= 0) atomicAdd(&h[((uint32_t)k >> shift) & mask], 1u);
            }
            if (FIRST && fill_out != nullptr) {
                const uint64_t dead = __ballot(idx < n && k < 0);
                if (dead != 0) {  // uniform for the wavefront
                    const uint32_t m = div_m.d;
                    const int64_t slot0 = idx - lane;
                    const int64_t out0 = slot0 * (int64_t)m;
                    int64_t cnt = n - slot0;  // slots of this group of 64 that exist
                    cnt = cnt > 64 ? 64 : cnt;
                    const uint32_t n_out = (uint32_t)cnt * m;
                    int32_t* dst = fill_out + out0;
                    if (aligned16 && m >= 3u) {
                        // four entries per lane: with m >= 3 they have at most two parents
                        for (uint32_t o = (uint32_t)lane * 4u; o < n_out; o += 256u) {
                            const uint32_t p0 = fastdiv(o, div_m);
                            const uint32_t last = o + 3u < n_out ? o + 3u : n_out - 1u;
                            const uint32_t p3 = fastdiv(last, div_m);
                            const bool d0 = (dead >> p0) & 1ull, d3 = (dead >> p3) & 1ull;
                            if (d0 && d3 && o + 3u < n_out) {
                                *reinterpret_cast<int4*>(dst + o) = make_int4(-1, -1, -1, -1);
                            } else if (d0 || d3) {
                                for (uint32_t e = o; e <= last; ++e)
                                    if ((dead >> fastdiv(e, div_m)) & 1ull) dst[e] = ND_NULL_VERTEX;
                            }
                        }
                    } else {
                        for (uint32_t o = (uint32_t)lane; o < n_out; o += 64u)
                            if ((dead >> fastdiv(o, div_m)) & 1ull) dst[o] = ND_NULL_VERTEX;
                    }
                }
            }
        }
    }
    if (FIRST && check_range && bad) atomicOr(status, 1u);
    __syncthreads();
    if (tid < nbins) hist[(int64_t)tid * num_tiles + blockIdx.x] = h[tid];
}

// One workgroup per digit value: exclusive scan of that digit's per-tile counts,
// in place; the digit's total goes to bin_total[digit].
constexpr int kBinscanThreads = 1024;
constexpr int64_t kFusedScanTiles = 64;  // up to here the downsweep scans the tiles itself
__global__ __launch_bounds__(kBinscanThreads) void binscan_kernel(uint32_t* __restrict__ hist,
                                                                  uint32_t* __restrict__ bin_total,
                                                                  int64_t num_tiles) {
    __shared__ uint32_t tmp[kBinscanThreads / 64 + 1];
    uint32_t* row = hist + (int64_t)blockIdx.x * num_tiles;
    uint32_t carry = 0;
    for (int64_t base = 0; base < num_tiles; base += kBinscanThreads) {
        const int64_t i = base + threadIdx.x;
        const uint32_t x = i < num_tiles ? row[i] : 0u;
        uint32_t total;
        const uint32_t ex = block_exclusive_scan<uint32_t, kBinscanThreads>(x, tmp, &total);
        if (i < num_tiles) row[i] = carry + ex;
        carry += total;
        __syncthreads();
    }
    if (threadIdx.x == 0) bin_total[blockIdx.x] = carry;
}

template <bool FIRST, int THREADS, int ITEMS>
__global__ __launch_bounds__(THREADS) void downsweep_kernel(
    const int32_t* __restrict__ keys_in, const int32_t* __restrict__ vals_in, int64_t n_slots,
    StepCtl* __restrict__ ctl, int shift, int bits, const uint32_t* __restrict__ hist,
    const uint32_t* __restrict__ bin_total, int64_t num_tiles, int32_t* __restrict__ keys_out,
    int32_t* __restrict__ vals_out, int32_t V) {
    constexpr int kTile = THREADS * ITEMS;
    constexpr int kWaves = THREADS / 64;
    constexpr int kPerWave = kTile / kWaves;  // consecutive keys owned by one wave
    static_assert(THREADS >= (1 << kMaxRadixBits), "one thread per digit value");
    __shared__ uint32_t wave_hist[kWaves][1 << kMaxRadixBits];
    __shared__ uint32_t digit_start[1 << kMaxRadixBits];
    __shared__ uint32_t global_base[1 << kMaxRadixBits];
    __shared__ uint32_t scan_tmp[kWaves + 2];
    __shared__ int32_t skeys[kTile];
    __shared__ int32_t svals[kTile];

    const int tid = threadIdx.x, lane = lane_id(), wave = wave_id();
    const int nbins = 1 << bits;
    const uint32_t mask = (uint32_t)nbins - 1u;
    const int64_t n = FIRST ? n_slots : (int64_t)ctl->P;
    const int64_t base = (int64_t)blockIdx.x * kTile;

    // Global start of every digit = exclusive scan of the digit totals; the sum
    // of the totals is the number of live pairs, which pass 0 publishes.
    // With few tiles the scan over the tiles is not a kernel of its own (bin_total is null):
    // every workgroup adds up its digit's row of raw per-tile counts itself.
    {
        uint32_t t = 0, before = 0;
        if (tid < nbins) {
            const uint32_t* row = hist + (int64_t)tid * num_tiles;
            if (bin_total != nullptr) {
                t = bin_total[tid];
                before = row[blockIdx.x];
            } else {
#pragma unroll 8
                for (int tt = 0; tt < (int)num_tiles; ++tt) {  // independent loads, at most 64
                    const uint32_t c = row[tt];
                    t += c;
                    before += tt < (int)blockIdx.x ? c : 0u;
                }
            }
        }
        uint32_t total;
        const uint32_t ex = block_exclusive_scan<uint32_t, THREADS>(t, scan_tmp, &total);
        if (tid < nbins) global_base[tid] = ex + before;
        if (FIRST && blockIdx.x == 0 && tid == 0) ctl->P = total;
    }
    if (base >= n) return;  // uniform for the workgroup
    for (int i = tid; i < kWaves * (1 << kMaxRadixBits); i += THREADS)
        (&wave_hist[0][0])[i] = 0;

    int32_t key[ITEMS], val[ITEMS];
    uint32_t rank[ITEMS];
    if (base + kTile <= n) {  // a whole tile (all but the last): nothing to test, one base address
        const int64_t first = base + (int64_t)wave * kPerWave + lane;
        const int32_t* kp = keys_in + first;
        const int32_t* vp = FIRST ? nullptr : vals_in + first;
#pragma unroll
        for (int r = 0; r < ITEMS; ++r) {
            int32_t k = kp[r * 64];
            if (FIRST && (k >= V || k < 0)) k = ND_NULL_VERTEX;
            key[r] = k;
            val[r] = FIRST ? (int32_t)(first + r * 64) : vp[r * 64];
        }
    } else {
#pragma unroll
        for (int r = 0; r < ITEMS; ++r) {
            const int64_t idx = base + (int64_t)wave * kPerWave + r * 64 + lane;
            int32_t k = ND_NULL_VERTEX, v = 0;
            if (idx < n) {
                k = keys_in[idx];
                if (FIRST) {
                    if (k >= V || k < 0) k = ND_NULL_VERTEX;
                    v = (int32_t)idx;
                } else {
                    v = vals_in[idx];
                }
            }
            key[r] = k;
            val[r] = v;
        }
    }
    // Pass 0 sees the slots without a transit as well (nearly half of them in the k-hop
    // workload on a graph with many isolated vertices).  The wave squeezes them out of its
    // 1024 slots first, through its own part of the reorder buffer and keeping the order, so
    // that the ranking below spends its ballots on live pairs only.
    uint32_t wave_live = (uint32_t)kPerWave;
    int32_t* stage_k = skeys + wave * kPerWave;
    int32_t* stage_v = svals + wave * kPerWave;
    if (FIRST) {
        uint32_t cnt = 0;
#pragma unroll
        for (int r = 0; r < ITEMS; ++r) {
            const bool live = key[r] >= 0;
            const uint64_t bal = __ballot(live);
            if (live) {
                const uint32_t p = cnt + (uint32_t)__popcll(bal & lanes_below(lane));
                stage_k[p] = key[r];
                stage_v[p] = val[r];
            }
            cnt += (uint32_t)__popcll(bal);
        }
        wave_live = cnt;
    }
    __syncthreads();
    if (FIRST) {
#pragma unroll
        for (int r = 0; r < ITEMS; ++r) {
            const uint32_t i = (uint32_t)(r * 64 + lane);
            const bool live = i < wave_live;
            key[r] = live ? stage_k[live ? i : 0u] : ND_NULL_VERTEX;
            val[r] = live ? stage_v[live ? i : 0u] : 0;
        }
    }

    // Stable rank inside the wave's 1024 consecutive keys: for every group of 64
    // keys, the lanes holding the same digit are found with one ballot per digit
    // bit; the lowest such lane advances the wave's running count of the digit.
    // Every live lane reads the count before that lane writes it: the LDS executes
    // a wavefront's operations in order.
#pragma unroll
    for (int r = 0; r < ITEMS; ++r) {
        if ((uint32_t)(r * 64) >= wave_live) {  // the same for the whole wave: nothing left to rank
            rank[r] = 0;
            continue;
        }
        const bool live = key[r] >= 0;
        const uint32_t d = ((uint32_t)key[r] >> shift) & mask;
        const uint64_t peers = digit_peers(d, __ballot(live), bits);
        const uint32_t below = __builtin_amdgcn_mbcnt_hi((uint32_t)(peers >> 32),
                                                         __builtin_amdgcn_mbcnt_lo((uint32_t)peers, 0u));
        uint32_t old = 0;
        if (live) {
            old = wave_hist[wave][d];
            if (below == 0u) wave_hist[wave][d] = old + (uint32_t)__popcll(peers);
        }
        // the next group of 64 keys reads these counters
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        __builtin_amdgcn_wave_barrier();
        rank[r] = old + below;
    }
    __syncthreads();

    // Per digit: exclusive scan over the waves (in place) and over the digits.
    {
        uint32_t cnt = 0;
        if (tid < nbins) {
#pragma unroll
            for (int w = 0; w < kWaves; ++w) {
                const uint32_t t = wave_hist[w][tid];
                wave_hist[w][tid] = cnt;
                cnt += t;
            }
        }
        uint32_t total;
        const uint32_t ex = block_exclusive_scan<uint32_t, THREADS>(cnt, scan_tmp, &total);
        if (tid < nbins) digit_start[tid] = ex;
        if (tid == 0) scan_tmp[kWaves + 1] = total;  // live keys of the tile
    }
    __syncthreads();
    const uint32_t tile_live = wave_uniform(scan_tmp[kWaves + 1]);

#pragma unroll
    for (int r = 0; r < ITEMS; ++r) {
        if (key[r] >= 0) {
            const uint32_t d = ((uint32_t)key[r] >> shift) & mask;
            const uint32_t pos = digit_start[d] + wave_hist[wave][d] + rank[r];
            skeys[pos] = key[r];
            svals[pos] = val[r];
        }
    }
    __syncthreads();

    for (uint32_t i = tid; i < tile_live; i += THREADS) {
        const int32_t k = skeys[i];
        const uint32_t d = ((uint32_t)k >> shift) & mask;
        const uint32_t g = global_base[d] + (i - digit_start[d]);
        keys_out[g] = k;
        vals_out[g] = svals[i];
    }
}

template <int THREADS, int ITEMS>
int sort_pairs_impl(const int32_t* src, int64_t n_slots, int32_t V, const SortPlan& plan,
                    int32_t* keysA, int32_t* valsA, int32_t* keysB, int32_t* valsB, uint32_t* hist,
                    StepCtl* ctl, int32_t* fill_out, int32_t m, uint32_t* status_word,
                    int32_t** keys_out, int32_t** vals_out, hipStream_t stream) {
    const int64_t tiles = plan.max_tiles;
    int maxbits = 0;
    for (int i = 0; i < plan.passes; ++i) maxbits = plan.bits[i] > maxbits ? plan.bits[i] : maxbits;
    uint32_t* bin_total = hist + (size_t)(1 << maxbits) * (size_t)tiles;
    const int32_t* kin = src;
    const int32_t* vin = nullptr;
    int32_t* kout = keysA;
    int32_t* vout = valsA;
    for (int p = 0; p < plan.passes; ++p) {
        const int bits = plan.bits[p], shift = plan.shift[p];
        if (p == 0) {
            hipLaunchKernelGGL((upsweep_kernel<true, THREADS, ITEMS>), dim3((unsigned)tiles),
                               dim3(THREADS), 0, stream, kin, n_slots, ctl, shift, bits, hist, tiles, V,
                               status_word != nullptr ? 1 : 0, status_word, fill_out,
                               make_fastdiv((uint32_t)m), ((uintptr_t)fill_out & 15u) == 0 ? 1 : 0);
        } else {
            hipLaunchKernelGGL((upsweep_kernel<false, THREADS, ITEMS>), dim3((unsigned)tiles),
                               dim3(THREADS), 0, stream, kin, n_slots, ctl, shift, bits, hist, tiles, V,
                               0, (uint32_t*)nullptr, (int32_t*)nullptr, make_fastdiv(1u), 0);
        }
        // the launch of a scan kernel costs more than 64 loads per digit in every workgroup
        const bool own_scan = tiles > kFusedScanTiles;
        const uint32_t* totals = own_scan ? bin_total : nullptr;
        if (own_scan)
            hipLaunchKernelGGL(binscan_kernel, dim3(1u << bits), dim3(kBinscanThreads), 0, stream, hist,
                               bin_total, tiles);
        if (p == 0) {
            hipLaunchKernelGGL((downsweep_kernel<true, THREADS, ITEMS>), dim3((unsigned)tiles),
                               dim3(THREADS), 0, stream, kin, vin, n_slots, ctl, shift, bits, hist,
                               totals, tiles, kout, vout, V);
        } else {
            hipLaunchKernelGGL((downsweep_kernel<false, THREADS, ITEMS>), dim3((unsigned)tiles),
                               dim3(THREADS), 0, stream, kin, vin, n_slots, ctl, shift, bits, hist,
                               totals, tiles, kout, vout, V);
        }
        kin = kout;
        vin = vout;
        if (kout == keysA) {
            kout = keysB;
            vout = valsB;
        } else {
            kout = keysA;
            vout = valsA;
        }
    }
    ND_HIP_CHECK(hipGetLastError());
    *keys_out = const_cast<int32_t*>(kin);
    *vals_out = const_cast<int32_t*>(vin);
    return ND_OK;
}

}  // namespace

int sort_pairs(const int32_t* src, int64_t n_slots, int32_t V, const SortPlan& plan, int32_t* keysA,
               int32_t* valsA, int32_t* keysB, int32_t* valsB, uint32_t* hist, StepCtl* ctl,
               int32_t* fill_out, int32_t m, uint32_t* status_word, int32_t** keys_out,
               int32_t** vals_out, hipStream_t stream) {
    if (plan.tile == kSmallSortThreads * kSmallSortItems)
        return sort_pairs_impl<kSmallSortThreads, kSmallSortItems>(
            src, n_slots, V, plan, keysA, valsA, keysB, valsB, hist, ctl, fill_out, m, status_word,
            keys_out, vals_out, stream);
    return sort_pairs_impl<kSortThreads, kSortItems>(src, n_slots, V, plan, keysA, valsA, keysB, valsB,
                                                     hist, ctl, fill_out, m, status_word, keys_out,
                                                     vals_out, stream);
}

}  // namespace nd
