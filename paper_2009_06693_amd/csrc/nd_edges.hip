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
// of slots; a fingerprint match is confirmed against the sorted list.
//
// Nine adjacency entries in ten are of no sample vertex, and the kernel is bound by instruction
// issue, not by the 4 bytes per entry it streams.  So an entry first tests one bit of a 65,536-bit
// map of the sample's vertices (no loop, no divergence); the few that pass are packed, in order,
// into a queue of the wavefront in LDS, and the table is probed by a full wavefront of queued
// entries at a time.
//
// Two passes share the kernel: counting (row sizes, then a device-wide
// exclusive scan into 64-bit row pointers) and filling.
#include <type_traits>

#include "nd_common.h"
#include "nd_edges.h"
#include "nd_wave.h"

namespace nd {

namespace {

constexpr int kEdgeThreads = 1024;  // two workgroups (76 KB of LDS each) fill a CU's 32 wave slots
constexpr int kEdgeUnroll = 4;      // adjacency loads in flight per lane and step
constexpr uint32_t kBatch = 64 * kEdgeUnroll;  // adjacency entries a wavefront takes per step
constexpr int kBitWords = 2048;     // the vertex map: 65,536 bits, indexed by the vertex id folded to 16 bits
constexpr uint32_t kQueueCap = 64 + kBatch;    // fewer than 64 left over plus one step's entries
constexpr int kMaxSlots = 2048;  // new vertices per sample (ND_MAX_EDGE_SLOTS)
constexpr size_t kEdgeLdsBytes = (size_t)kMaxSlots * 8 + (size_t)4 * kMaxSlots * 4 + (size_t)kBitWords * 4 +
                                 (size_t)(kEdgeThreads / 64) * kQueueCap * 4;
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
// The vertex's bit in the 65,536-bit map: the id folded to 16 bits.  Two shifts and an exclusive or,
// where the multiplicative hash costs a quarter-rate multiply per adjacency entry, and neighbouring
// ids - an ascending adjacency list is full of them - read the same or neighbouring words of LDS.
__device__ __forceinline__ uint32_t map_bit(int32_t v) { return ((uint32_t)v ^ ((uint32_t)v >> 16)) & 0xFFFFu; }

// one wavefront: its LDS operations complete in order; keeps the compiler from moving them
__device__ __forceinline__ void wave_lds_order() {
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

template <typename OffT, bool FILL>
__global__ __launch_bounds__(kEdgeThreads) void edges_kernel(GraphView<OffT> g, EdgeArgs a) {
    extern __shared__ __align__(16) unsigned char s_dyn[];
    uint64_t* s_sorted = (uint64_t*)s_dyn;                // [kMaxSlots] (vertex << 32 | slot), ascending; ~0 = none
    uint32_t* table = (uint32_t*)(s_sorted + kMaxSlots);  // [4 * kMaxSlots] entries as described above
    uint32_t* s_bits = table + 4 * kMaxSlots;             // [kBitWords] bit set: some sample vertex hashes here
    int32_t* s_queue = (int32_t*)(s_bits + kBitWords);    // per wavefront: entries that passed the bit test
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
    for (uint32_t i = tid; i < (uint32_t)kBitWords; i += kEdgeThreads) s_bits[i] = 0u;
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
        const uint32_t bi = map_bit(v);
        atomicOr(&s_bits[bi >> 5], 1u << (bi & 31u));
    }
    __syncthreads();

    // ---- the wavefronts stream the adjacency lists of the sample's transits, a row at a time each.
    // Everything about a row is the same in all lanes of its wavefront and is kept in scalar
    // registers.  The loop runs over steps of up to kBatch entries of a row; the entries of the next
    // step (the same row's or the next row's) are requested before the current step is worked on,
    // and so are, one and two rows ahead, the offsets and the transit of the rows to come.
    constexpr uint32_t kStride = kEdgeThreads / 64;
    const int lane = lane_id();
    const uint32_t wave = wave_uniform((uint32_t)wave_id());
    int32_t* queue = s_queue + wave * kQueueCap;
    const uint64_t row0 = (uint64_t)b * a.n_prev;

    auto transit_of = [&](uint32_t row) -> int32_t {  // as stored; NULL beyond the last row
        return row < a.n_prev ? a.transits[row0 + row] : ND_NULL_VERTEX;
    };
    auto checked = [&](int32_t v) -> int32_t {
        v = wave_uniform(v);
        if (v >= g.V || v < ND_NULL_VERTEX) {
            bad = true;
            v = ND_NULL_VERTEX;
        }
        return v;
    };
    // the row whose entries are being requested
    uint32_t t = wave;
    uint64_t rs = 0, deg = 0;   // where its adjacency list starts and how long it is (0: nothing to stream)
    uint64_t e0 = 0;            // the next entry of it to request
    int64_t wb = 0;             // FILL: where its output starts
    // one row ahead: transit known, offsets (FILL: row pointers) requested; two ahead: transit requested
    int32_t tv_a = ND_NULL_VERTEX, tv_b = ND_NULL_VERTEX;
    OffT off_a0 = 0, off_a1 = 0;
    int64_t rp_a0 = 0, rp_a1 = 0;
    auto request_a = [&]() {
        off_a0 = off_a1 = 0;
        if (tv_a >= 0) {
            off_a0 = g.off[tv_a];
            off_a1 = g.off[tv_a + 1];
        }
        if constexpr (FILL) {
            rp_a0 = rp_a1 = 0;
            if (t + kStride < a.n_prev) {
                rp_a0 = a.row_ptr[row0 + t + kStride];
                rp_a1 = a.row_ptr[row0 + t + kStride + 1];
            }
        }
    };
    auto advance = [&]() {
        t += kStride;
        rs = wave_uniform((uint64_t)off_a0);
        deg = wave_uniform((uint64_t)off_a1) - rs;
        if constexpr (FILL) {
            wb = wave_uniform(rp_a0);
            if (wave_uniform(rp_a1) == wb) deg = 0;  // the counting pass found nothing in this row
        }
        e0 = 0;
        tv_a = checked(tv_b);
        request_a();
        tv_b = transit_of(t + 2 * kStride);
    };
    auto skip_empty_rows = [&]() {
        while (t < a.n_prev && deg == 0) {
            if constexpr (!FILL)
                if (lane == 0) a.counts[row0 + t] = 0;
            advance();
        }
    };
    auto request_entries = [&](int32_t (&u)[kEdgeUnroll]) {
        const int32_t* p = g.col + rs + e0;
        const uint64_t left = deg - e0;
        const uint32_t cnt = left < kBatch ? (uint32_t)left : kBatch;
        if (cnt == kBatch) {  // a full step, the common case: nothing to test
#pragma unroll
            for (int r = 0; r < kEdgeUnroll; ++r) u[r] = p[r * 64 + lane];
            return;
        }
#pragma unroll
        for (int r = 0; r < kEdgeUnroll; ++r) {
            u[r] = ND_NULL_VERTEX;
            // the test is the same in all lanes; inside the last 64 entries a lane past the end
            // reads the last entry again instead of branching (and drops it when it looks at it:
            // looking at it here would wait for each load in turn)
            if ((uint32_t)r * 64u < cnt) {
                const uint32_t e = (uint32_t)r * 64u + (uint32_t)lane;
                u[r] = p[e < cnt ? e : cnt - 1u];
            }
        }
    };

    {   // the pipeline's first row is loaded directly
        const int32_t tv = checked(transit_of(t));
        if (tv >= 0) {
            rs = wave_uniform((uint64_t)g.off[tv]);
            deg = wave_uniform((uint64_t)g.off[tv + 1]) - rs;
        }
        if constexpr (FILL) {
            if (t < a.n_prev) {
                wb = wave_uniform(a.row_ptr[row0 + t]);
                if (wave_uniform(a.row_ptr[row0 + t + 1]) == wb) deg = 0;
            }
        }
        tv_a = checked(transit_of(t + kStride));
        request_a();
        tv_b = transit_of(t + 2 * kStride);
    }
    skip_empty_rows();
    int32_t u_next[kEdgeUnroll];
#pragma unroll
    for (int r = 0; r < kEdgeUnroll; ++r) u_next[r] = 0;
    if (t < a.n_prev) request_entries(u_next);

    uint32_t queued = 0;  // entries in the queue (the same in all lanes)
    uint32_t count = 0;   // counting pass: my share of the row's edges
    int64_t wbase = wb;   // filling pass: where the row's next edge goes
    while (t < a.n_prev) {
        // ---- the step whose entries have been requested
        int32_t u[kEdgeUnroll];
#pragma unroll
        for (int r = 0; r < kEdgeUnroll; ++r) {
            u[r] = u_next[r];
            // taken here, before the requests below are issued: loads return in order, and a wait
            // for these entries placed after those requests would wait for them as well
            asm volatile("" : "+v"(u[r]));
        }
        const uint64_t left = deg - e0;
        const uint32_t cnt = left < kBatch ? (uint32_t)left : kBatch;
        const bool row_ends = left <= kBatch;
        const uint32_t t_now = t;
        // ---- request the next step's entries before working on this one
        if (row_ends) {
            advance();
            skip_empty_rows();
        } else {
            e0 += kBatch;
        }
        if (t < a.n_prev) request_entries(u_next);

        // ---- entries that pass the bit test join the queue, in order.  Two copies of the code: a
        // full step (the common case) tests nothing but the bit.
        auto enqueue = [&](auto full_step) {
            constexpr bool kFull = decltype(full_step)::value;
#pragma unroll
            for (int r = 0; r < kEdgeUnroll; ++r) {
                if (!kFull && (uint32_t)r * 64u >= cnt) break;  // the same for the whole wavefront
                const uint32_t bi = map_bit(u[r]);
                bool pass = ((s_bits[bi >> 5] >> (bi & 31u)) & 1u) != 0u;
                if (!kFull) pass = pass && (uint32_t)r * 64u + (uint32_t)lane < cnt;
                const uint64_t votes = __ballot(pass);
                const uint32_t ahead = __builtin_amdgcn_mbcnt_hi((uint32_t)(votes >> 32),
                                                                 __builtin_amdgcn_mbcnt_lo((uint32_t)votes, 0u));
                // no branch: a lane that does not pass writes to the queue's spare last place
                queue[pass ? queued + ahead : kQueueCap - 1u] = u[r];
                queued += (uint32_t)__popcll(votes);
            }
        };
        if (cnt == kBatch) enqueue(std::true_type{});
        else enqueue(std::false_type{});
        wave_lds_order();

        // ---- the table is probed by 64 queued entries at a time (by what is left when the row ends)
        uint32_t head = 0;
        while (queued - head >= 64u || (row_ends && head < queued)) {
            const uint32_t n = queued - head < 64u ? queued - head : 64u;
            const int32_t v = (uint32_t)lane < n ? queue[head + lane] : ND_NULL_VERTEX;
            uint32_t c = 0, k = 0;
            if (v >= 0) {
                const uint32_t h = hash_vertex(v);
                const uint32_t fp = fingerprint(h);
                uint32_t pos = h >> a.hash_shift;
                uint32_t en;
                while ((en = table[pos]) != kEmpty) {  // ends: the table is never full
                    if ((en >> 23) == fp && (int32_t)(s_sorted[en & 0x7FFu] >> 32) == v) {
                        k = en & 0x7FFu;
                        c = (en >> 11) & 0xFFFu;
                        break;
                    }
                    pos = (pos + 1u) & mask;
                }
            }
            if constexpr (FILL) {
                // the lanes hold runs (k, c), most of them empty or one entry long: a lane writes
                // its run entry by entry from the running sum of the lanes below it (the loop is
                // the same in all lanes and ends with the longest run)
                const uint32_t incl = wave_inclusive_scan(c, lane);
                const uint32_t total = (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
                const uint32_t ex = incl - c;
                if (__ballot(c > 8u) == 0ull) {
                    for (uint32_t i = 0; __ballot(i < c) != 0ull; ++i)
                        if (i < c && wbase + ex + i < a.capacity)
                            a.edge_slot[wbase + ex + i] = (int32_t)(uint32_t)s_sorted[k + i];
                    wbase += total;
                    head += n;
                    continue;
                }
                // a vertex held by many slots: the entries are written in lane order, 64 at a
                // time, each output position finding its lane by a search over the running sums
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
            } else {
                count += c;
            }
            head += n;
        }
        if (row_ends) {
            if constexpr (!FILL) {
                const uint32_t incl = wave_inclusive_scan(count, lane);
                if (lane == 63) a.counts[row0 + t_now] = (int32_t)incl;
                count = 0;
            }
            queued = 0;
            wbase = wb;  // of the row the next step belongs to
            wave_lds_order();
        } else if (head > 0u) {  // fewer than 64 are left: they move to the front
            const uint32_t rest = queued - head;
            const int32_t moved = (uint32_t)lane < rest ? queue[head + lane] : 0;
            wave_lds_order();
            if ((uint32_t)lane < rest) queue[lane] = moved;
            queued = rest;
            wave_lds_order();
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

// Dynamic LDS above the 64 KB default has to be allowed once per kernel; done when a graph is
// created so that the entry points themselves only launch.
int edges_prepare() {
#define ND_EDGES_ALLOW(OFFT, FILL)                                                              \
    ND_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(&edges_kernel<OFFT, FILL>),  \
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)kEdgeLdsBytes))
    ND_EDGES_ALLOW(int64_t, true);
    ND_EDGES_ALLOW(int64_t, false);
    ND_EDGES_ALLOW(int32_t, true);
    ND_EDGES_ALLOW(int32_t, false);
#undef ND_EDGES_ALLOW
    return ND_OK;
}

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
                               dim3(kEdgeThreads), kEdgeLdsBytes, stream, view_of<int64_t>(gr), a);
        else
            hipLaunchKernelGGL((edges_kernel<int32_t, false>), dim3((unsigned)num_samples),
                               dim3(kEdgeThreads), kEdgeLdsBytes, stream, view_of<int32_t>(gr), a);
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
                           kEdgeLdsBytes, stream, view_of<int64_t>(gr), a);
    else
        hipLaunchKernelGGL((edges_kernel<int32_t, true>), dim3((unsigned)num_samples), dim3(kEdgeThreads),
                           kEdgeLdsBytes, stream, view_of<int32_t>(gr), a);
    ND_HIP_CHECK(hipGetLastError());
    return ND_OK;
}

}  // namespace nd
