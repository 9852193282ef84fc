// Edges between consecutive layers (Section 4.2 of the paper, "Importance
// Sampling": in FastGCN / LADIES style sampling every sample carries the
// adjacency matrix between the transits of a step and the vertices the step
// added; the paper's `next` adds an edge between the new vertex and every
// transit that has it as a neighbour).
//
// The paper's kernel tests each new vertex against each transit.  Here one
// workgroup per sample puts the sample's new vertices into an LDS hash table
// once and then streams the adjacency lists of the sample's transits through
// it: a wavefront reads 64 consecutive adjacency entries per iteration
// (coalesced) and probes the table, so the cost is one LDS probe per adjacency
// entry instead of a binary search per (transit, new vertex) pair.
//
// Output is one CSR over the rows (sample, transit slot).  A row lists the new
// slots j whose vertex is a neighbour of the row's transit, ordered by (vertex
// id, j) - the order a walk down the ascending adjacency list meets them - so
// the result is unique.  To make that order cheap the sample's (vertex, slot)
// pairs are sorted once in LDS (bitonic network); the hash table maps a vertex
// to its run in the sorted list.  A table entry is one 32-bit word (fingerprint
// of the vertex, start and length of the run) in a table four times the number
// of slots, so that a miss - the common case - costs little more than one LDS
// read; a fingerprint match is confirmed against the sorted list.
//
// Two passes share the kernel: counting (row sizes, then a device-wide
// exclusive scan into 64-bit row pointers) and filling.
#include "nd_common.h"
#include "nd_edges.h"
#include "nd_wave.h"

namespace nd {

namespace {

constexpr int kEdgeThreads = 1024;  // two workgroups (48 KB of LDS each) fill a CU's 32 wave slots
constexpr int kEdgeUnroll = 4;      // adjacency loads in flight per lane
constexpr int kMaxSlots = 2048;  // new vertices per sample (ND_MAX_EDGE_SLOTS)
constexpr int kScanThreads = 256;
constexpr int kScanItems = 16;
constexpr int kScanTile = kScanThreads * kScanItems;

struct EdgeArgs {
    const int32_t* transits;  // [S][n_prev]
    const int32_t* sampled;   // [S][m]
    uint32_t n_prev, m;
    uint32_t m2;              // power of two >= m
    uint32_t hash_shift;      // 32 - log2(4 * m2)
    int32_t* counts;          // count pass: [S * n_prev]
    const int64_t* row_ptr;   // fill pass
    int32_t* edge_slot;
    int64_t capacity;
    uint32_t* status;
};

// Table entry: bits 0-10 first position of the vertex's run in the sorted list, bits 11-22 the
// run's length (1..2048), bits 23-31 a fingerprint of the vertex.  All ones = empty (no run is
// 4,095 long).
constexpr uint32_t kEmpty = 0xFFFFFFFFu;
__device__ __forceinline__ uint32_t hash_vertex(int32_t v) { return (uint32_t)v * 0x9E3779B1u; }
__device__ __forceinline__ uint32_t fingerprint(uint32_t h) { return (h >> 9) & 0x1FFu; }

template <typename OffT, bool FILL>
__global__ __launch_bounds__(kEdgeThreads) void edges_kernel(GraphView<OffT> g, EdgeArgs a) {
    __shared__ uint64_t s_sorted[kMaxSlots];   // (vertex << 32 | slot), ascending; ~0 = none
    __shared__ uint32_t table[4 * kMaxSlots];  // entries as described above
    const uint32_t b = blockIdx.x;
    const uint32_t tid = threadIdx.x;
    const uint32_t mask = 4u * a.m2 - 1u;
    const int32_t* sampled = a.sampled + (uint64_t)b * a.m;
    bool bad = false;

    for (uint32_t i = tid; i < a.m2; i += kEdgeThreads) {
        uint64_t key = ~0ull;
        if (i < a.m) {
            int32_t v = sampled[i];
            if (v >= g.V || v < ND_NULL_VERTEX) {
                bad = true;
                v = ND_NULL_VERTEX;
            }
            if (v >= 0) key = ((uint64_t)(uint32_t)v << 32) | i;
        }
        s_sorted[i] = key;
    }
    for (uint32_t i = tid; i < 4u * a.m2; i += kEdgeThreads) table[i] = kEmpty;
    __syncthreads();

    // bitonic sorting network over m2 keys
    for (uint32_t k = 2; k <= a.m2; k <<= 1) {
        for (uint32_t j = k >> 1; j > 0; j >>= 1) {
            for (uint32_t i = tid; i < a.m2; i += kEdgeThreads) {
                const uint32_t p = i ^ j;
                if (p > i) {
                    const uint64_t x = s_sorted[i], y = s_sorted[p];
                    const bool ascending = (i & k) == 0;
                    if ((x > y) == ascending) {
                        s_sorted[i] = y;
                        s_sorted[p] = x;
                    }
                }
            }
            __syncthreads();
        }
    }

    // the first entry of every run of equal vertices puts the run into the table (the table has
    // four times as many places as there can be runs, so the probe loops end)
    for (uint32_t k = tid; k < a.m2; k += kEdgeThreads) {
        const uint64_t key = s_sorted[k];
        if (key == ~0ull) continue;
        const int32_t v = (int32_t)(key >> 32);
        if (k > 0 && (int32_t)(s_sorted[k - 1] >> 32) == v) continue;
        uint32_t lo = k + 1, hi = a.m2;  // first position after k whose vertex differs
        while (lo < hi) {
            const uint32_t mid = (lo + hi) >> 1;
            if ((int32_t)(s_sorted[mid] >> 32) == v) lo = mid + 1;
            else hi = mid;
        }
        const uint32_t h = hash_vertex(v);
        const uint32_t entry = (fingerprint(h) << 23) | ((lo - k) << 11) | k;
        uint32_t pos = h >> a.hash_shift;
        while (atomicCAS(&table[pos], kEmpty, entry) != kEmpty) pos = (pos + 1u) & mask;
    }
    __syncthreads();

    const int lane = lane_id();
    for (uint32_t t = wave_id(); t < a.n_prev; t += kEdgeThreads / 64) {
        const uint64_t row = (uint64_t)b * a.n_prev + t;
        int32_t tv = a.transits[row];
        if (tv >= g.V || tv < ND_NULL_VERTEX) {
            bad = true;
            tv = ND_NULL_VERTEX;
        }
        uint32_t count = 0;
        int64_t wbase = 0;
        if constexpr (FILL) wbase = a.row_ptr[row];
        if (tv >= 0) {
            const uint64_t rs = (uint64_t)g.off[tv];
            const uint64_t deg = (uint64_t)g.off[tv + 1] - rs;
            for (uint64_t e0 = 0; e0 < deg; e0 += 64 * kEdgeUnroll) {
                int32_t u[kEdgeUnroll];
#pragma unroll
                for (int r = 0; r < kEdgeUnroll; ++r) {  // all loads first: the loop is latency bound
                    const uint64_t e = e0 + (uint64_t)r * 64 + lane;
                    u[r] = e < deg ? g.col[rs + e] : ND_NULL_VERTEX;
                }
#pragma unroll
                for (int r = 0; r < kEdgeUnroll; ++r) {
                    uint32_t c = 0, k = 0;
                    if (u[r] >= 0) {
                        const uint32_t h = hash_vertex(u[r]);
                        const uint32_t fp = fingerprint(h);
                        uint32_t pos = h >> a.hash_shift;
                        uint32_t en;
                        while ((en = table[pos]) != kEmpty) {  // ends: the table is never full
                            if ((en >> 23) == fp && (int32_t)(s_sorted[en & 0x7FFu] >> 32) == u[r]) {
                                k = en & 0x7FFu;
                                c = (en >> 11) & 0xFFFu;
                                break;
                            }
                            pos = (pos + 1u) & mask;
                        }
                    }
                    if constexpr (FILL) {
                        if (e0 + (uint64_t)r * 64 < deg) {  // same for the whole wavefront
                            // the 64 lanes hold runs (k, c); their entries are written in lane order,
                            // 64 at a time, each output position finding its lane by a search over
                            // the running sums
                            const uint32_t incl = wave_inclusive_scan(c, lane);
                            const uint32_t total = __shfl(incl, 63, 64);
                            const uint32_t ex = incl - c;
                            for (uint32_t base = 0; base < total; base += 64) {
                                const uint32_t p = base + lane;
                                uint32_t owner = 0;
#pragma unroll
                                for (uint32_t step = 32; step > 0; step >>= 1)
                                    if (__shfl(incl, (int)(owner + step - 1), 64) <= p) owner += step;
                                owner &= 63u;
                                const uint32_t ok = __shfl(k, (int)owner, 64);
                                const uint32_t oex = __shfl(ex, (int)owner, 64);
                                if (p < total && wbase + p < a.capacity)
                                    a.edge_slot[wbase + p] = (int32_t)(uint32_t)s_sorted[ok + (p - oex)];
                            }
                            wbase += total;
                        }
                    } else {
                        count += c;
                    }
                }
            }
        }
        if constexpr (!FILL) {
            const uint32_t incl = wave_inclusive_scan(count, lane);
            if (lane == 63) a.counts[row] = (int32_t)incl;
        }
    }
    if (bad && a.status) atomicOr(a.status, 1u);
}

__global__ void edges_clear_status_kernel(uint32_t* status) { *status = 0u; }

// ---- exclusive scan of n int32 counts into n + 1 int64 row pointers (reduce, scan the tile
// sums in one workgroup, scan again with the tile's base)
__global__ __launch_bounds__(kScanThreads) void scan_sums_kernel(const int32_t* counts, int64_t n,
                                                                 int64_t* sums) {
    __shared__ int64_t tmp[kScanThreads / 64 + 1];
    const int64_t base = (int64_t)blockIdx.x * kScanTile;
    int64_t s = 0;
    for (int i = 0; i < kScanItems; ++i) {
        const int64_t p = base + (int64_t)i * kScanThreads + threadIdx.x;
        if (p < n) s += counts[p];
    }
    int64_t total;
    block_exclusive_scan<int64_t, kScanThreads>(s, tmp, &total);
    if (threadIdx.x == 0) sums[blockIdx.x] = total;
}

__global__ __launch_bounds__(kScanThreads) void scan_top_kernel(int64_t* sums, int64_t tiles) {
    __shared__ int64_t tmp[kScanThreads / 64 + 1];
    int64_t carry = 0;
    for (int64_t base = 0; base < tiles; base += kScanThreads) {
        const int64_t p = base + threadIdx.x;
        const int64_t x = p < tiles ? sums[p] : 0;
        int64_t total;
        const int64_t ex = block_exclusive_scan<int64_t, kScanThreads>(x, tmp, &total);
        if (p < tiles) sums[p] = carry + ex;
        carry += total;
        __syncthreads();
    }
    if (threadIdx.x == 0) sums[tiles] = carry;
}

__global__ __launch_bounds__(kScanThreads) void scan_write_kernel(const int32_t* counts, int64_t n,
                                                                  const int64_t* sums, int64_t tiles,
                                                                  int64_t* row_ptr) {
    __shared__ int64_t tmp[kScanThreads / 64 + 1];
    // a thread owns kScanItems consecutive counts, so that one workgroup scan orders the tile
    const int64_t first = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanItems;
    int32_t c[kScanItems];
    int64_t s = 0;
    for (int i = 0; i < kScanItems; ++i) {
        c[i] = first + i < n ? counts[first + i] : 0;
        s += c[i];
    }
    int64_t total;
    int64_t run = sums[blockIdx.x] + block_exclusive_scan<int64_t, kScanThreads>(s, tmp, &total);
    for (int i = 0; i < kScanItems; ++i) {
        if (first + i < n) row_ptr[first + i] = run;
        run += c[i];
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) row_ptr[n] = sums[tiles];
}

inline int64_t scan_tiles(int64_t n) { return (n + kScanTile - 1) / kScanTile; }

inline uint32_t pow2_at_least(uint32_t x) {
    uint32_t p = 64;
    while (p < x) p <<= 1;
    return p;
}

inline EdgeArgs make_args(const int32_t* transits, int32_t n_prev, const int32_t* sampled, int32_t m) {
    EdgeArgs a{};
    a.transits = transits;
    a.sampled = sampled;
    a.n_prev = (uint32_t)n_prev;
    a.m = (uint32_t)m;
    a.m2 = pow2_at_least((uint32_t)m);
    uint32_t lg = 0;
    while ((1u << lg) < 4u * a.m2) ++lg;
    a.hash_shift = 32u - lg;
    return a;
}

}  // namespace

size_t edges_workspace_bytes(int64_t num_samples, int32_t n_prev) {
    const int64_t rows = num_samples * (int64_t)n_prev;
    const size_t counts = ((size_t)(rows > 0 ? rows : 1) * 4 + 255) / 256 * 256;
    return 256 + counts + (size_t)(scan_tiles(rows) + 1) * 8 + 256;
}

int edges_count(const Graph& gr, const int32_t* transits, int32_t n_prev, const int32_t* sampled,
                int32_t m, int64_t num_samples, int64_t* row_ptr, void* workspace, hipStream_t stream) {
    const int64_t rows = num_samples * (int64_t)n_prev;
    char* ws = (char*)workspace;
    uint32_t* status = (uint32_t*)ws;
    int32_t* counts = (int32_t*)(ws + 256);
    const size_t counts_bytes = ((size_t)(rows > 0 ? rows : 1) * 4 + 255) / 256 * 256;
    int64_t* sums = (int64_t*)(ws + 256 + counts_bytes);
    const int64_t tiles = scan_tiles(rows);
    hipLaunchKernelGGL(edges_clear_status_kernel, dim3(1), dim3(1), 0, stream, status);
    if (num_samples > 0) {
        EdgeArgs a = make_args(transits, n_prev, sampled, m);
        a.counts = counts;
        a.status = status;
        if (gr.off64)
            hipLaunchKernelGGL((edges_kernel<int64_t, false>), dim3((unsigned)num_samples),
                               dim3(kEdgeThreads), 0, stream, view_of<int64_t>(gr), a);
        else
            hipLaunchKernelGGL((edges_kernel<int32_t, false>), dim3((unsigned)num_samples),
                               dim3(kEdgeThreads), 0, stream, view_of<int32_t>(gr), a);
        hipLaunchKernelGGL(scan_sums_kernel, dim3((unsigned)tiles), dim3(kScanThreads), 0, stream, counts,
                           rows, sums);
    }
    hipLaunchKernelGGL(scan_top_kernel, dim3(1), dim3(kScanThreads), 0, stream, sums, tiles);
    hipLaunchKernelGGL(scan_write_kernel, dim3((unsigned)(tiles > 0 ? tiles : 1)), dim3(kScanThreads), 0,
                       stream, counts, rows, sums, tiles, row_ptr);
    ND_HIP_CHECK(hipGetLastError());
    return ND_OK;
}

int edges_fill(const Graph& gr, const int32_t* transits, int32_t n_prev, const int32_t* sampled,
               int32_t m, int64_t num_samples, const int64_t* row_ptr, int32_t* edge_slot,
               int64_t capacity, hipStream_t stream) {
    if (num_samples == 0) return ND_OK;
    EdgeArgs a = make_args(transits, n_prev, sampled, m);
    a.row_ptr = row_ptr;
    a.edge_slot = edge_slot;
    a.capacity = capacity;
    a.status = nullptr;
    if (gr.off64)
        hipLaunchKernelGGL((edges_kernel<int64_t, true>), dim3((unsigned)num_samples), dim3(kEdgeThreads),
                           0, stream, view_of<int64_t>(gr), a);
    else
        hipLaunchKernelGGL((edges_kernel<int32_t, true>), dim3((unsigned)num_samples), dim3(kEdgeThreads),
                           0, stream, view_of<int32_t>(gr), a);
    ND_HIP_CHECK(hipGetLastError());
    return ND_OK;
}

}  // namespace nd
