// Edges between consecutive layers (Section 4.2 of the paper, "Importance
// Sampling": in FastGCN / LADIES style sampling every sample carries the
// adjacency matrix between the transits of a step and the vertices the step
// added; the paper's `next` adds an edge between the new vertex and every
// transit that has it as a neighbour).
//
// The paper's kernel tests each new vertex against each transit.  Here one
// workgroup per sample puts the sample's new vertices into an LDS hash table
// once and then streams the adjacency lists of the sample's transits through
// it, 64 consecutive (coalesced) entries per wavefront load, so the cost is
// per adjacency entry instead of a binary search per (transit, new vertex) pair.
//
// Output is one CSR over the rows (sample, transit slot).  A row lists the new
// slots j whose vertex is a neighbour of the row's transit, ordered by (vertex
// id, j) - the order a walk down the ascending adjacency list meets them - so
// the result is unique.  To make that order cheap the sample's (vertex, slot)
// pairs are sorted once in LDS (a radix sort); the hash table maps a vertex to
// its run in the sorted list.  A table entry is one 32-bit word (fingerprint of
// the vertex, start and length of the run) in a table twice the number of
// slots; a fingerprint match is confirmed against the sorted list.
//
// Nine adjacency entries in ten are of no sample vertex, and the kernel is bound as much by
// instruction issue as by the 4 bytes per entry it streams.  So an entry first tests one bit of a 65,536-bit
// map of the sample's vertices (no loop, no divergence); the few that pass are packed, in order,
// into a queue of the wavefront in LDS, and the table is probed by a full wavefront of queued
// entries at a time.
//
// The sample's transit slots are sorted by vertex as well: a vertex that several slots hold (layer
// samples hold well-connected vertices many times over) is streamed once, and what is found goes to
// the row of each of those slots.  The wavefronts take the distinct transits from a counter.
//
// Two passes share the kernel: counting (row sizes, then a device-wide
// exclusive scan into 64-bit row pointers) and filling.
#include <type_traits>

#include "nd_common.h"
#include "nd_edges.h"
#include "nd_wave.h"

namespace nd {

namespace {

constexpr int kEdgeThreads = 1024;  // two workgroups (78 KB of LDS each) fill a CU's 32 wave slots
constexpr int kBitWords = 2048;     // the vertex map: 65,536 bits, indexed by the vertex id folded to 16 bits
constexpr uint32_t kQueueCap = 64 + 64;        // fewer than 64 left over plus a quarter step's entries
constexpr uint32_t kOutCap = 64 + 64;          // filling pass: edges of the current transit not yet written
constexpr int kMaxSlots = 2048;  // new vertices per sample (ND_MAX_EDGE_SLOTS)
constexpr int kChunk = 2048;     // transit slots of a sample that are sorted and de-duplicated together
constexpr size_t kEdgeLdsBytes = (size_t)kMaxSlots * 8 + (size_t)2 * kMaxSlots * 4 +
                                 (size_t)(kEdgeThreads / 64) * (kQueueCap + kOutCap) * 4 + (size_t)kChunk * 8 +
                                 (size_t)kChunk * 2;
constexpr int kScanThreads = 256;
constexpr int kScanItems = 16;
constexpr int kScanTile = kScanThreads * kScanItems;

struct EdgeArgs {
    const int32_t* transits;  // [S][n_prev]
    const int32_t* sampled;   // [S][m]
    uint32_t n_prev, m;
    uint32_t m2;              // power of two >= m
    uint32_t hash_shift;      // 32 - log2(2 * m2)
    int32_t* counts;          // count pass: [S * n_prev]
    const int64_t* row_ptr;   // fill pass
    int32_t* edge_slot;
    int64_t capacity;
    uint32_t* status;
    int vertex_bits;          // bits of the largest vertex id
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

// Sorts the n2 (a power of two, at most 2 * kEdgeThreads) keys (vertex << 32 | slot) of an LDS array
// by vertex; the slots arrive ascending and the sort is stable, so the keys end ascending.  Every
// thread of the workgroup calls it, after a barrier that made the keys visible, and it ends with
// one.  An LSD radix sort over the vertex's bits plus one (missing keys are all ones and must end
// behind the largest vertex), 8 bits per pass: a wavefront owns 128 consecutive keys, ranks them
// with one ballot per digit bit, the per-wavefront digit counts are scanned, and the keys, which
// sit in registers meanwhile, go back to their places.  Three passes for 4 M vertices where a
// bitonic network takes 66 compare-exchange steps (54 us per workgroup through LDS, 32 us in
// registers with lane exchanges: more than streaming the adjacency lists of 64 transits).
// hist: kEdgeThreads / 64 rows of 256 counters; digit_start: 256 entries; scan_tmp: for the scan.
__device__ __forceinline__ void sort_keys_lds(uint64_t* keys, uint32_t n2, uint32_t tid, int vertex_bits,
                                              uint32_t* hist, uint32_t* digit_start, uint32_t* scan_tmp) {
    constexpr uint32_t T = (uint32_t)kEdgeThreads;
    const bool two = n2 > T;  // the same for the whole workgroup
    const uint32_t wave = tid >> 6, lane = tid & 63u;
    const uint32_t per_wave = two ? 128u : 64u;
    const uint32_t at0 = wave * per_wave + lane, at1 = at0 + 64u;
    uint32_t* my_hist = hist + wave * 256u;
    const int total_bits = vertex_bits + 1;
    const int passes = (total_bits + 7) / 8;
    int shift = 0;
    for (int pass = 0; pass < passes; ++pass) {
        const int bits = total_bits / passes + (pass >= passes - total_bits % passes ? 1 : 0);
        const uint32_t dmask = (1u << bits) - 1u;
        const uint64_t k0 = at0 < n2 ? keys[at0] : ~0ull;
        const uint64_t k1 = (two && at1 < n2) ? keys[at1] : ~0ull;
        for (uint32_t i = lane; i < 256u; i += 64u) my_hist[i] = 0u;
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        __builtin_amdgcn_wave_barrier();
        const uint32_t d0 = ((uint32_t)(k0 >> 32) >> shift) & dmask;
        const uint32_t d1 = ((uint32_t)(k1 >> 32) >> shift) & dmask;
        uint32_t r0, r1 = 0;
        {
            const uint64_t peers = digit_peers(d0, ~0ull, bits);
            const uint32_t below = __builtin_amdgcn_mbcnt_hi((uint32_t)(peers >> 32),
                                                             __builtin_amdgcn_mbcnt_lo((uint32_t)peers, 0u));
            const uint32_t old = my_hist[d0];  // read by all lanes before the lowest peer writes it
            if (below == 0u) my_hist[d0] = old + (uint32_t)__popcll(peers);
            __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
            __builtin_amdgcn_wave_barrier();
            r0 = old + below;
        }
        if (two) {
            const uint64_t peers = digit_peers(d1, ~0ull, bits);
            const uint32_t below = __builtin_amdgcn_mbcnt_hi((uint32_t)(peers >> 32),
                                                             __builtin_amdgcn_mbcnt_lo((uint32_t)peers, 0u));
            const uint32_t old = my_hist[d1];
            if (below == 0u) my_hist[d1] = old + (uint32_t)__popcll(peers);
            __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
            __builtin_amdgcn_wave_barrier();
            r1 = old + below;
        }
        __syncthreads();
        uint32_t cnt = 0;
        if (tid < (1u << bits)) {  // per digit: exclusive scan over the wavefronts, in place
#pragma unroll
            for (uint32_t w = 0; w < T / 64u; ++w) {
                const uint32_t t = hist[w * 256u + tid];
                hist[w * 256u + tid] = cnt;
                cnt += t;
            }
        }
        uint32_t total;
        const uint32_t ex = block_exclusive_scan<uint32_t, kEdgeThreads>(cnt, scan_tmp, &total);
        if (tid < (1u << bits)) digit_start[tid] = ex;
        __syncthreads();
        // every key is in a register: the array can be overwritten
        if (at0 < n2) keys[digit_start[d0] + my_hist[d0] + r0] = k0;
        if (two && at1 < n2) keys[digit_start[d1] + my_hist[d1] + r1] = k1;
        __syncthreads();
        shift += bits;
    }
}

// Two workgroups of 1,024 threads per compute unit are eight wavefronts per SIMD.  That takes at most
// 64 vector registers and, on this register file (800 scalar registers per SIMD), at most 96 scalar
// registers per wavefront: left to itself the compiler uses more scalar registers than that, which
// silently halves the occupancy, so the bound is stated (the surplus goes to lanes of a vector register).
template <typename OffT, bool FILL>
__global__ __launch_bounds__(kEdgeThreads) __attribute__((amdgpu_waves_per_eu(8, 8)))
void edges_kernel(GraphView<OffT> g, EdgeArgs a) {
    extern __shared__ __align__(16) unsigned char s_dyn[];
    uint64_t* s_sorted = (uint64_t*)s_dyn;                // [kMaxSlots] (vertex << 32 | slot), ascending; ~0 = none
    uint32_t* table = (uint32_t*)(s_sorted + kMaxSlots);  // [2 * kMaxSlots] entries as described above
    int32_t* s_queue = (int32_t*)(table + 2 * kMaxSlots);  // per wavefront: entries that passed the bit test
    int32_t* s_out = s_queue + (kEdgeThreads / 64) * kQueueCap;  // per wavefront: edges waiting to be written
    uint64_t* s_trans = (uint64_t*)(s_out + (kEdgeThreads / 64) * kOutCap);  // [kChunk] (transit << 32 | slot), sorted
    uint16_t* s_heads = (uint16_t*)(s_trans + kChunk);    // [kChunk] where each distinct transit starts in s_trans
    // bit set: some sample vertex hashes here.  Declared statically so that its address is a constant
    // of the instruction that reads it (one read per adjacency entry).
    __shared__ uint32_t s_bits[kBitWords];
    __shared__ uint32_t s_scan[kEdgeThreads / 64 + 1];
    __shared__ uint32_t s_items[3];                       // distinct transits and live slots of the chunk; next item to hand out
    // Adjacency loads in flight per lane and step: eight where the kernel then still fits 64 vector
    // registers (two workgroups per compute unit), four in the filling pass over 64-bit offsets.
    constexpr int kEdgeUnroll = (FILL && sizeof(OffT) == 8) ? 4 : 8;
    constexpr uint32_t kBatch = 64 * kEdgeUnroll;  // adjacency entries a wavefront takes per step
    const uint32_t b = blockIdx.x;
    const uint32_t tid = threadIdx.x;
    const uint32_t mask = 2u * a.m2 - 1u;
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
    for (uint32_t i = tid; i < 2u * a.m2; i += kEdgeThreads) table[i] = kEmpty;
    for (uint32_t i = tid; i < (uint32_t)kBitWords; i += kEdgeThreads) s_bits[i] = 0u;
    __syncthreads();

    sort_keys_lds(s_sorted, a.m2, tid, a.vertex_bits, (uint32_t*)s_queue, (uint32_t*)s_heads, s_scan);

    // the first entry of every run of equal vertices puts the run into the table (the table has
    // twice as many places as there can be runs, so the probe loops end)
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
        atomicOr(&s_bits[bi >> 5], 0x80000000u >> (bi & 31u));  // counted from the top: the test is a shift and a sign
    }
    __syncthreads();

    // ---- The sample's transits, kChunk slots at a time, are sorted by vertex in LDS: layer samples
    // hold well-connected vertices many times over (569 distinct among the 2,048 transits of the
    // benchmark's second step), and a vertex's adjacency list is streamed once for all the slots
    // that hold it.  The wavefronts then take one distinct transit each at a time.
    // Everything about such an item is the same in all lanes of its wavefront and is kept in scalar
    // registers.  The loop runs over steps of up to kBatch entries of a list; the entries of the next
    // step (the same item's or the next item's) and the offsets of the item after are requested
    // before the current step is worked on.
    const int lane = lane_id();
    const uint32_t wave = wave_uniform((uint32_t)wave_id());
    int32_t* queue = s_queue + wave * kQueueCap;
    int32_t* obuf = s_out + wave * kOutCap;
    const uint64_t row0 = (uint64_t)b * a.n_prev;

    for (uint32_t chunk0 = 0; chunk0 < a.n_prev; chunk0 += (uint32_t)kChunk) {
        const uint32_t n_chunk = a.n_prev - chunk0 < (uint32_t)kChunk ? a.n_prev - chunk0 : (uint32_t)kChunk;
        uint32_t n2 = 64;
        while (n2 < n_chunk) n2 <<= 1;
        for (uint32_t i = tid; i < n2; i += kEdgeThreads) {
            uint64_t key = ~0ull;
            if (i < n_chunk) {
                int32_t v = a.transits[row0 + chunk0 + i];
                if (v >= g.V || v < ND_NULL_VERTEX) {
                    bad = true;
                    v = ND_NULL_VERTEX;
                }
                if (v >= 0) key = ((uint64_t)(uint32_t)v << 32) | (chunk0 + i);
                else if (!FILL) a.counts[row0 + chunk0 + i] = 0;  // a slot without a transit has no edges
            }
            s_trans[i] = key;
        }
        __syncthreads();
        sort_keys_lds(s_trans, n2, tid, a.vertex_bits, (uint32_t*)s_queue, (uint32_t*)s_heads, s_scan);
        {   // where the distinct transits start (two positions per thread: n2 <= 2 * kEdgeThreads)
            bool head[2];
            uint32_t mine = 0, live = 0;
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const uint32_t i = tid * 2u + (uint32_t)e;
                head[e] = false;
                if (i < n2 && s_trans[i] != ~0ull) {
                    ++live;
                    head[e] = i == 0 || (uint32_t)(s_trans[i - 1] >> 32) != (uint32_t)(s_trans[i] >> 32);
                }
                mine += head[e] ? 1u : 0u;
            }
            // one scan for both counts (each at most 2,048): heads in the low half, live slots in the high
            uint32_t total;
            uint32_t at = block_exclusive_scan<uint32_t, kEdgeThreads>(mine | (live << 16), s_scan, &total) & 0xFFFFu;
            if (tid == 0) {
                s_items[0] = total & 0xFFFFu;
                s_items[1] = total >> 16;
                s_items[2] = 0;
            }
#pragma unroll
            for (int e = 0; e < 2; ++e)
                if (head[e]) s_heads[at++] = (uint16_t)(tid * 2u + (uint32_t)e);
        }
        __syncthreads();
        const uint32_t n_items = wave_uniform(s_items[0]);
        const uint32_t n_live = wave_uniform(s_items[1]);  // the live slots are the first n_live of s_trans

        // the item whose entries are being requested: positions [p0, p1) of s_trans hold its slots
        // the wavefronts take the items in order from a counter: lists differ in length by orders of
        // magnitude, and a fixed share per wavefront leaves most of them waiting for the slowest
        auto claim = [&]() -> uint32_t {
            uint32_t i = 0;
            if (lane == 0) i = atomicAdd(&s_items[2], 1u);
            return wave_uniform(i);
        };
        uint32_t item = claim();
        uint32_t item_next = claim();  // its offsets are requested while `item` is worked on
        uint32_t p0 = 0, p1 = 0;
        uint64_t rs = 0;            // where its adjacency list starts
        uint32_t deg = 0;           // how long it is (0: nothing to stream); a list has fewer than 2^31 entries
        uint32_t e0 = 0;            // the next entry of it to request
        // one item ahead: offsets (FILL: row pointers of its first slot) requested
        OffT off_a0 = 0, off_a1 = 0;
        int64_t rp_a0 = 0, rp_a1 = 0;
        auto slots_of = [&](uint32_t it, uint32_t* first, uint32_t* last) {
            *first = s_heads[it];
            *last = it + 1u < n_items ? (uint32_t)s_heads[it + 1u] : n_live;
        };
        auto request_a = [&](uint32_t it) {  // offsets and row pointers of item `it`
            off_a0 = off_a1 = 0;
            rp_a0 = rp_a1 = 0;
            if (it < n_items) {
                const uint64_t key = s_trans[s_heads[it]];
                const int32_t v = wave_uniform((int32_t)(uint32_t)(key >> 32));
                off_a0 = g.off[v];
                off_a1 = g.off[v + 1];
                if constexpr (FILL) {
                    const uint32_t slot = wave_uniform((uint32_t)key);
                    rp_a0 = a.row_ptr[row0 + slot];
                    rp_a1 = a.row_ptr[row0 + slot + 1];
                }
            }
        };
        bool no_edges = false;  // FILL: the counting pass found nothing for this item
        auto adopt = [&]() {     // the item ahead becomes the item being requested
            rs = wave_uniform((uint64_t)off_a0);
            deg = (uint32_t)(wave_uniform((uint64_t)off_a1) - rs);
            if constexpr (FILL) {
                no_edges = wave_uniform(rp_a1) == wave_uniform(rp_a0);
                if (no_edges) deg = 0;
            }
            e0 = 0;
            if (item < n_items) slots_of(item, &p0, &p1);
            request_a(item_next);
        };
        // an item without entries to stream: its slots' counts are 0 (counting pass), nothing else
        auto skip_empty_items = [&]() {
            while (item < n_items && deg == 0) {
                if constexpr (!FILL)
                    for (uint32_t d = p0 + (uint32_t)lane; d < p1; d += 64u)
                        a.counts[row0 + (uint32_t)s_trans[d]] = 0;
                item = item_next;
                item_next = claim();
                adopt();
            }
        };
        auto request_entries = [&](int32_t (&u)[kEdgeUnroll]) {
            const int32_t* p = g.col + rs + e0;
            const uint32_t left = deg - e0;
            const uint32_t cnt = left < kBatch ? left : kBatch;
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

        request_a(item);
        adopt();
        skip_empty_items();
        int32_t u_next[kEdgeUnroll];
#pragma unroll
        for (int r = 0; r < kEdgeUnroll; ++r) u_next[r] = 0;
        if (item < n_items) request_entries(u_next);

        uint32_t queued = 0;  // entries in the queue (the same in all lanes)
        uint32_t count = 0;   // counting pass: my share of the item's edges
        uint32_t done = 0;    // filling pass: edges of the item written so far (to each of its slots' rows)
        uint32_t ofill = 0;   // filling pass: edges of the item waiting in obuf
        while (item < n_items) {
            // ---- the step whose entries have been requested
            int32_t u[kEdgeUnroll];
#pragma unroll
            for (int r = 0; r < kEdgeUnroll; ++r) {
                u[r] = u_next[r];
                // taken here, before the requests below are issued: loads return in order, and a wait
                // for these entries placed after those requests would wait for them as well
                asm volatile("" : "+v"(u[r]));
            }
            const uint32_t left = deg - e0;
            const uint32_t cnt = left < kBatch ? left : kBatch;
            const bool row_ends = left <= kBatch;
            const uint32_t q0 = p0, q1 = p1;  // the slots of the item being worked on
            // ---- request the next step's entries before working on this one
            if (row_ends) {
                item = item_next;
                item_next = claim();
                adopt();
                skip_empty_items();
            } else {
                e0 += kBatch;
            }
            if (item < n_items) request_entries(u_next);

            // ---- entries that pass the bit test join the queue, in order, 64 at a time; the table is
            // probed by 64 queued entries at a time (by what is left when the item ends).
            // Filling pass: the edges found are collected in obuf, in order, and leave 64 at a time, one
            // coalesced store per slot that holds the item's transit.
            auto write_out = [&](uint32_t nf) {  // the first nf (at most 64) entries of obuf, to every row of the item
                const int32_t val = (uint32_t)lane < nf ? obuf[lane] : 0;
                for (uint32_t d0 = q0; d0 < q1; d0 += 64u) {
                    // the rows of up to 64 slots at a time: their starts come by one load, a lane per slot
                    const uint32_t nd = q1 - d0 < 64u ? q1 - d0 : 64u;
                    int64_t my_row = 0;
                    if ((uint32_t)lane < nd) my_row = a.row_ptr[row0 + (uint32_t)s_trans[d0 + lane]];
                    for (uint32_t dd = 0; dd < nd; ++dd) {
                        const int64_t wbase =
                            (int64_t)(((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)(my_row >> 32), dd) << 32) |
                                      (uint32_t)__builtin_amdgcn_readlane((int)my_row, dd)) + done;
                        if ((uint32_t)lane < nf && wbase + lane < a.capacity) a.edge_slot[wbase + lane] = val;
                    }
                }
                done += nf;
            };
#pragma unroll
            for (int r = 0; r < kEdgeUnroll; ++r) {
                const bool in_step = cnt == kBatch || (uint32_t)r * 64u < cnt;  // the same for the whole wavefront
                if (in_step) {
                    const uint32_t bi = map_bit(u[r]);
                    const bool pass = (int32_t)(s_bits[bi >> 5] << (bi & 31u)) < 0;
                    // The lanes past the list's end (its last step only) are struck from the votes, a
                    // scalar operation, and not from `pass`: such a lane that passes writes to the place
                    // after the last live entry (at most the spare one), which nothing reads.
                    const uint32_t live = cnt - (uint32_t)r * 64u;
                    const uint64_t votes = __ballot(pass) & (live >= 64u ? ~0ull : (1ull << live) - 1ull);
                    const uint32_t at = __builtin_amdgcn_mbcnt_hi((uint32_t)(votes >> 32),
                                                                  __builtin_amdgcn_mbcnt_lo((uint32_t)votes, queued));
                    // no branch: a lane that does not pass writes to the queue's spare last place
                    queue[pass ? at : kQueueCap - 1u] = u[r];
                    queued += (uint32_t)__popcll(votes);
                    wave_lds_order();
                }
                const bool last = row_ends && r == kEdgeUnroll - 1;
                while (queued >= 64u || (last && queued > 0u)) {
                // 64 queued entries (or, at the item's end, what is left)
                const uint32_t n = queued < 64u ? queued : 64u;
                const int32_t v = (uint32_t)lane < n ? queue[lane] : ND_NULL_VERTEX;
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
                    // the lanes hold runs (k, c); their entries go to obuf in lane order, 64 positions
                    // at a time: a lane with a short run writes it itself, a long run (a vertex held by
                    // many slots) is spread by a search over the running sums
                    const uint32_t incl = wave_inclusive_scan(c, lane);
                    const uint32_t total = (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
                    const uint32_t ex = incl - c;
                    if (total <= 64u && __ballot(c > 8u) == 0ull) {
                        for (uint32_t i = 0; __ballot(i < c) != 0ull; ++i)
                            if (i < c) obuf[ofill + ex + i] = (int32_t)(uint32_t)s_sorted[k + i];
                        ofill += total;
                        wave_lds_order();
                        if (ofill >= 64u) {
                            write_out(64u);
                            const int32_t moved = (uint32_t)lane < ofill - 64u ? obuf[64 + lane] : 0;
                            wave_lds_order();
                            if ((uint32_t)lane < ofill - 64u) obuf[lane] = moved;
                            ofill -= 64u;
                            wave_lds_order();
                        }
                    } else {
                        for (uint32_t base = 0; base < total; base += 64u) {
                            const uint32_t p = base + lane;
                            uint32_t owner = 0;
#pragma unroll
                            for (uint32_t step = 32; step > 0; step >>= 1)
                                if (__shfl(incl, (int)(owner + step - 1), 64) <= p) owner += step;
                            owner &= 63u;
                            const uint32_t ok = __shfl(k, (int)owner, 64);
                            const uint32_t oex = __shfl(ex, (int)owner, 64);
                            const uint32_t nb = total - base < 64u ? total - base : 64u;
                            if (p < total) obuf[ofill + lane] = (int32_t)(uint32_t)s_sorted[ok + (p - oex)];
                            ofill += nb;
                            wave_lds_order();
                            if (ofill >= 64u) {
                                write_out(64u);
                                const int32_t moved = (uint32_t)lane < ofill - 64u ? obuf[64 + lane] : 0;
                                wave_lds_order();
                                if ((uint32_t)lane < ofill - 64u) obuf[lane] = moved;
                                ofill -= 64u;
                                wave_lds_order();
                            }
                        }
                    }
                } else {
                    count += c;
                }
                // what is left of the queue moves to the front
                const uint32_t rest = queued - n;
                const int32_t moved = (uint32_t)lane < rest ? queue[n + lane] : 0;
                wave_lds_order();
                if ((uint32_t)lane < rest) queue[lane] = moved;
                queued = rest;
                wave_lds_order();
                }
                if (last) {  // the item ends
                    if constexpr (!FILL) {
                        const uint32_t incl = wave_inclusive_scan(count, lane);
                        const uint32_t total = (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
                        for (uint32_t d = q0 + (uint32_t)lane; d < q1; d += 64u)
                            a.counts[row0 + (uint32_t)s_trans[d]] = (int32_t)total;
                        count = 0;
                    } else {
                        if (ofill > 0u) write_out(ofill);
                        ofill = 0;
                        done = 0;
                        wave_lds_order();
                    }
                }
            }
        }
        __syncthreads();  // the chunk's sorted transits are replaced by the next chunk's
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

inline EdgeArgs make_args(const Graph& gr, const int32_t* transits, int32_t n_prev, const int32_t* sampled,
                          int32_t m) {
    EdgeArgs a{};
    a.transits = transits;
    a.sampled = sampled;
    a.n_prev = (uint32_t)n_prev;
    a.m = (uint32_t)m;
    a.m2 = pow2_at_least((uint32_t)m);
    uint32_t lg = 0;
    while ((1u << lg) < 2u * a.m2) ++lg;
    a.hash_shift = 32u - lg;
    a.vertex_bits = 1;
    while (a.vertex_bits < 31 && (1ll << a.vertex_bits) < gr.V) ++a.vertex_bits;
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
        EdgeArgs a = make_args(gr, transits, n_prev, sampled, m);
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
    EdgeArgs a = make_args(gr, transits, n_prev, sampled, m);
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
