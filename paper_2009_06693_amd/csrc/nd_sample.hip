// Sampling kernels for individual transit sampling (random walks and k-hop;
// Section 6.1 of the paper).
//
// The three scheduling classes of Section 6.1.2 (Table "Types of kernels"),
// re-derived for 64-lane wavefronts and run as one launch per step:
//   sub-wavefront  one lane per draw over the pairs sorted by transit; the
//                  draws of one (transit, sample) pair sit on consecutive lanes,
//                  so the sample's new vertices leave in one contiguous store
//                  (the paper's sub-warps, Section 6.1.1), and neighbouring
//                  lanes read the same or neighbouring adjacency lists, which
//                  the caches serve once.  No LDS; three-round software pipeline.
//   workgroup      one 1,024-lane workgroup at a time per transit, handed out
//                  by a device-side cursor; the adjacency list (and the weight
//                  running sums) are staged in LDS when they fit and the reuse
//                  pays for the copy, otherwise read from global memory
//                  ("Caching", Section 6.1.2).
//   grid           a transit with more draws than one workgroup handles is cut
//                  into chunks that go through the same kernel and cursor as the
//                  workgroup class, every chunk staging the list.
// plus the sample-parallel kernel of Section 5.1 (one lane per output slot, no
// grouping), kept as the ablation baseline, the per-sample kernel that removes
// repeated neighbours (Section 6.3) and the small kernels of the
// multi-dimensional walk.
//
// What a lane draws is the same in all of them: one Philox call per
// (sample, slot, step, attempt), so they produce identical outputs.
#include "nd_common.h"
#include "nd_philox.h"
#include "nd_wave.h"
#include "nd_sample.h"
#include "nd_draw.h"

namespace nd {

namespace {

// q: slot of the transit in the previous step's array; jj: which of its m draws.
template <int DRAW, typename OffT>
__device__ __forceinline__ int32_t draw_for_slot(const GraphView<OffT>& g, const DrawArgs& a,
                                                 int32_t v, uint32_t deg, uint32_t q, uint32_t jj,
                                                 const int32_t* adj, const uint64_t* cum,
                                                 const uint32_t* wq) {
    const uint32_t s = fastdiv(q, a.div_wprev);
    const uint32_t slot = (q - s * a.div_wprev.d) * a.m + jj;
    const uint32_t sid = a.sample_base + s;
    if (DRAW == kDrawUniform) return draw_uniform(a, deg, sid, slot, adj);
    if (DRAW == kDrawWeighted) return draw_weighted(a, deg, sid, slot, adj, cum);
    return draw_node2vec(g, a, v, deg, sid, a.has_prev ? a.prev_transit[s] : ND_NULL_VERTEX, adj, wq);
}

// ---------------------------------------------------------------- sample-parallel (Section 5.1)
template <int DRAW, typename OffT>
__global__ __launch_bounds__(256) void sample_sp_kernel(GraphView<OffT> g, DrawArgs a,
                                                        const int32_t* __restrict__ src,
                                                        int64_t n_slots, int check_roots,
                                                        uint32_t* __restrict__ status) {
    const int64_t o = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (o >= n_slots * (int64_t)a.m) return;
    const uint32_t q = fastdiv((uint32_t)o, a.div_m);
    const uint32_t jj = (uint32_t)o - q * a.m;
    int32_t v = src[q];
    if (v >= g.V || v < ND_NULL_VERTEX) {
        if (check_roots) atomicOr(status, 1u);
        v = ND_NULL_VERTEX;
    }
    int32_t res = ND_NULL_VERTEX;
    if (v >= 0) {
        const uint64_t rs = (uint64_t)g.off[v];
        const uint32_t deg = row_length(g, v, rs);
        if (deg > 0)
            res = draw_for_slot<DRAW>(g, a, v, deg, q, jj, g.col + rs,
                                      DRAW == kDrawWeighted ? g.cumq + rs : nullptr,
                                      (DRAW == kDrawNode2vec && a.use_weights) ? g.wq + rs : nullptr);
    }
    a.out[o] = res;
}

// ---------------------------------------------------------------- sub-wavefront class
// One lane per draw over the pairs sorted by transit: draw d belongs to pair
// d / m, so the m draws of a (transit, sample) pair sit on m consecutive lanes
// (one contiguous store per sample) and consecutive pairs share or neighbour
// each other's transit (row offsets and adjacency lines are fetched once per
// wavefront instruction and reused from cache).  Transits that classify_groups
// handed to the workgroup or grid class are marked in a bitmap and skipped.
// What a lane needs to know about its pair before it can draw.
struct PairCtx {
    uint64_t rs;    // first adjacency entry of the transit
    uint32_t deg;   // 0: nothing to draw (dead end)
    uint32_t q;     // slot of the pair in the previous step's array
    int32_t v;      // transit
    bool mine;      // the pair exists and its transit is not left to another class
};

// Branch-free on purpose: every load is issued unconditionally (from a clamped, always valid
// index), so the loads of the U pairs a lane handles per round are in flight together.
// Loading a pair is two dependent steps - the sorted pair itself, then the row offsets of its
// transit - which the pipelined loop issues in different rounds.
struct PairKey {
    int32_t v;      // transit
    uint32_t q;     // slot of the pair in the previous step's array
    bool in_range;  // the pair exists
};

__device__ __forceinline__ PairKey load_pair_key(const int32_t* __restrict__ keys,
                                                 const int32_t* __restrict__ vals, uint32_t pi,
                                                 uint32_t P) {
    PairKey k;
    const uint32_t pc = pi < P ? pi : P - 1u;  // P >= 1 whenever a lane gets here
    k.v = keys[pc];
    k.q = (uint32_t)vals[pc];
    k.in_range = pi < P;
    return k;
}

template <bool HEAVY, typename OffT>
__device__ __forceinline__ PairCtx load_pair_row(const GraphView<OffT>& g, const uint32_t* heavy_bits,
                                                 const PairKey& k) {
    PairCtx c;
    c.v = k.v;
    c.q = k.q;
    uint32_t heavy = 0;
    if (HEAVY) heavy = (heavy_bits[(uint32_t)c.v >> 5] >> ((uint32_t)c.v & 31u)) & 1u;
    c.rs = (uint64_t)g.off[c.v];
    c.deg = row_length(g, c.v, c.rs);
    c.mine = k.in_range && heavy == 0u;
    return c;
}

template <bool HEAVY, typename OffT>
__device__ __forceinline__ PairCtx load_pair(const GraphView<OffT>& g,
                                             const int32_t* __restrict__ keys,
                                             const int32_t* __restrict__ vals,
                                             const uint32_t* heavy_bits, uint32_t pi, uint32_t P) {
    return load_pair_row<HEAVY>(g, heavy_bits, load_pair_key(keys, vals, pi, P));
}

template <int DRAW, typename OffT>
__device__ __forceinline__ int32_t draw_pair(const GraphView<OffT>& g, const DrawArgs& a,
                                             const PairCtx& c, uint32_t jj) {
    if (DRAW == kDrawUniform) {
        // straight-line: the generator runs on every lane, the gather reads entry 0 of the
        // adjacency array for lanes that have nothing to draw
        const uint32_t s = fastdiv(c.q, a.div_wprev);
        const uint32_t slot = (c.q - s * a.div_wprev.d) * a.m + jj;
        const Rand4 r = draw4(a.seed, a.sample_base + s, slot, a.step, 0u);
        const bool live = c.mine && c.deg > 0u && !(a.ppr_thr != 0 && (uint64_t)r.r3 < a.ppr_thr);
        const uint64_t e = live ? c.rs + mulhi32(r.r0, c.deg) : 0ull;
        const int32_t u = g.col[e];
        return live ? u : ND_NULL_VERTEX;
    }
    if (!c.mine || c.deg == 0) return ND_NULL_VERTEX;
    return draw_for_slot<DRAW>(g, a, c.v, c.deg, c.q, jj, g.col + c.rs,
                               DRAW == kDrawWeighted ? g.cumq + c.rs : nullptr,
                               (DRAW == kDrawNode2vec && a.use_weights) ? g.wq + c.rs : nullptr);
}

// The loop of the sub-wavefront kernel.  HEAVY: some transits of this step belong to the
// workgroup / grid class and must be skipped (looked up in the bitmap).
template <int DRAW, bool HEAVY, typename OffT>
__device__ __forceinline__ void sub_loop(const GraphView<OffT>& g, const DrawArgs& a, uint32_t P,
                                         const int32_t* __restrict__ keys,
                                         const int32_t* __restrict__ vals,
                                         const uint32_t* heavy_bits, uint32_t pairs_per_block,
                                         uint32_t tid, uint32_t block, uint32_t blocks) {
    // tid, block, blocks: position of this lane in a grid of 256-lane groups (four of them share
    // one workgroup of the launch)
    // independent pairs in flight per lane (the looping draws gain nothing from a second one)
    constexpr int U = DRAW == kDrawUniform ? 2 : 1;
    if (pairs_per_block != 0u) {
        // A workgroup round covers pairs_per_block whole pairs: a lane keeps its draw index jj
        // and walks over pairs, so no division sits in the loop.  U pairs are fetched before the
        // first draw so that their memory latencies overlap; they are adjacent blocks of the
        // sorted array, so the whole grid works on one contiguous window of transits at a time
        // (that window is what L2 keeps hot).
        const uint32_t pl = fastdiv(tid, a.div_m);
        const uint32_t jj = tid - pl * a.m;
        if (pl >= pairs_per_block) return;
        const uint32_t stride = blocks * pairs_per_block * U;
        uint32_t pi = block * pairs_per_block * U + pl;
        if (pi >= P) return;
        // Software pipeline, three rounds deep: the sorted pairs of round i + 2 and the row offsets
        // of round i + 1 are requested before round i draws, and round i's stores are issued last,
        // so a lane never waits for two dependent loads in one round and neither the stores'
        // acknowledgements nor the next loads are waited for while the generator runs.
        PairCtx cur[U];
        PairKey key1[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            cur[u] = load_pair<HEAVY>(g, keys, vals, heavy_bits, pi + u * pairs_per_block, P);
            key1[u] = load_pair_key(keys, vals, pi + stride + u * pairs_per_block, P);
        }
        for (; pi < P; pi += stride) {
            PairKey key2[U];
            PairCtx nxt[U];
            int32_t res[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                // pi + 2 * stride stays below 2^32: P < 2^31 and a stride is at most a few million
                key2[u] = load_pair_key(keys, vals, pi + 2u * stride + u * pairs_per_block, P);
                nxt[u] = load_pair_row<HEAVY>(g, heavy_bits, key1[u]);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) res[u] = draw_pair<DRAW>(g, a, cur[u], jj);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (cur[u].mine) a.out[cur[u].q * a.m + jj] = res[u];  // below 2^31 by the call's plan
                cur[u] = nxt[u];
                key1[u] = key2[u];
            }
        }
    } else {
        const uint32_t total = P * a.m;
        const uint32_t stride = blocks * 256u;
        for (uint32_t d = block * 256u + tid; d < total; d += stride) {
            const uint32_t pi = fastdiv(d, a.div_m);
            const uint32_t jj = d - pi * a.m;
            const PairCtx c = load_pair<HEAVY>(g, keys, vals, heavy_bits, pi, P);
            const int32_t res = draw_pair<DRAW>(g, a, c, jj);
            if (c.mine) a.out[c.q * a.m + jj] = res;
        }
    }
}

// ---------------------------------------------------------------- workgroup and grid classes
constexpr int kWgThreads = 1024;

template <int DRAW>
struct StageCap {  // adjacency entries that fit the 64 KB of LDS a workgroup stages into
    static constexpr uint32_t value =
        DRAW == kDrawUniform ? 16384u : (DRAW == kDrawWeighted ? 5120u : 8192u);
};

// Draws d in [d0, d1) of group gid, by one workgroup.
template <int DRAW, typename OffT>
__device__ __forceinline__ void workgroup_draws(const GraphView<OffT>& g, const DrawArgs& a,
                                                StepCtl* ctl, const int32_t* __restrict__ g_key,
                                                const int32_t* __restrict__ g_start,
                                                const int32_t* __restrict__ vals, uint32_t gid,
                                                uint32_t d0, uint32_t d1, int32_t* lds_col,
                                                uint64_t* lds_cum, uint32_t* lds_wq) {
    constexpr uint32_t cap = StageCap<DRAW>::value;
    const int32_t v = g_key[gid];
    const uint32_t start = (uint32_t)g_start[gid];
    const uint64_t rs = (uint64_t)g.off[v];
    const uint32_t deg = row_length(g, v, rs);
    const uint32_t ndraws = d1 - d0;
    bool stage = deg > 0 && deg <= cap;
    if (a.lds_policy == 1) stage = false;
    else if (a.lds_policy == 0) stage = stage && deg >= 1024u && deg / 4u <= ndraws;
    const int32_t* adj = g.col + rs;
    const uint64_t* cum = DRAW == kDrawWeighted ? g.cumq + rs : nullptr;
    const uint32_t* wq = (DRAW == kDrawNode2vec && a.use_weights) ? g.wq + rs : nullptr;
    if (stage) {
        for (uint32_t i = threadIdx.x; i < deg; i += kWgThreads) {
            lds_col[i] = adj[i];
            if (DRAW == kDrawWeighted) lds_cum[i] = cum[i];
            if (DRAW == kDrawNode2vec && a.use_weights) lds_wq[i] = wq[i];
        }
        if (threadIdx.x == 0) atomicAdd(&ctl->n_staged, 1u);
        __syncthreads();
        adj = lds_col;
        if (DRAW == kDrawWeighted) cum = lds_cum;
        if (DRAW == kDrawNode2vec && a.use_weights) wq = lds_wq;
    }
    for (uint32_t d = d0 + threadIdx.x; d < d1; d += kWgThreads) {
        const uint32_t pi = fastdiv(d, a.div_m);
        const uint32_t jj = d - pi * a.m;
        const uint32_t q = (uint32_t)vals[start + pi];
        int32_t res = ND_NULL_VERTEX;
        if (deg > 0) res = draw_for_slot<DRAW>(g, a, v, deg, q, jj, adj, cum, wq);
        a.out[(uint64_t)q * a.m + jj] = res;
    }
}

// One launch per step for all three classes.  Every workgroup first serves the workgroup and
// grid classes: it takes work items from a device-side cursor - items [0, n_wg) are the
// workgroup-class transits (one workgroup does the whole transit), items [n_wg, n_wg + n_chunks)
// are the chunks of the grid-class transits (many workgroups share one transit) - until the
// cursor runs out.  Then it turns into four independent 256-lane groups of the lane-per-draw
// loop over all pairs (sub-wavefront class), which skips the pairs of transits marked in
// heavy_bits.  A forced class runs only its half.
template <int DRAW, typename OffT>
__global__ __launch_bounds__(kWgThreads) void sample_tp_kernel(
    GraphView<OffT> g, DrawArgs a, SchedParams sp, StepCtl* __restrict__ ctl,
    const int32_t* __restrict__ keys, const int32_t* __restrict__ vals,
    const int32_t* __restrict__ g_key, const int32_t* __restrict__ g_start,
    const int32_t* __restrict__ list_wg, const int32_t* __restrict__ chunk_gid,
    const int32_t* __restrict__ chunk_idx, uint32_t cap_wg, uint32_t cap_chunks,
    const uint32_t* __restrict__ heavy_bits, uint32_t pairs_per_block, int do_heavy, int do_lanes) {
    constexpr uint32_t cap = StageCap<DRAW>::value;
    __shared__ int32_t lds_col[cap];
    __shared__ uint64_t lds_cum[DRAW == kDrawWeighted ? cap : 1];
    __shared__ uint32_t lds_wq[DRAW == kDrawNode2vec ? cap : 1];
    __shared__ uint32_t s_item;
    if (do_heavy) {
        uint32_t n_wg = ctl->n_wg, n_chunks = ctl->n_chunks;
        if (n_wg > cap_wg) n_wg = cap_wg;              // the lists are sized so this never bites
        if (n_chunks > cap_chunks) n_chunks = cap_chunks;
        const uint32_t n_items = n_wg + n_chunks;
        for (;;) {
            if (threadIdx.x == 0) s_item = atomicAdd(&ctl->wg_cursor, 1u);
            __syncthreads();
            const uint32_t i = wave_uniform(s_item);  // the item's description stays in scalar registers
            if (i >= n_items) break;  // uniform: every wave of the workgroup leaves here
            const bool grid = i >= n_wg;
            const uint32_t gid = (uint32_t)(grid ? chunk_gid[i - n_wg] : list_wg[i]);
            const uint32_t size = (uint32_t)(g_start[gid + 1] - g_start[gid]);
            const uint32_t draws = size * a.m;
            uint32_t d0 = 0, d1 = draws;
            if (grid) {
                d0 = (uint32_t)chunk_idx[i - n_wg] * (uint32_t)sp.wg_max;
                d1 = d0 + (uint32_t)sp.wg_max < draws ? d0 + (uint32_t)sp.wg_max : draws;
            }
            workgroup_draws<DRAW, OffT>(g, a, ctl, g_key, g_start, vals, gid, d0, d1, lds_col, lds_cum,
                                        lds_wq);
            __syncthreads();  // s_item and the LDS copy are rewritten by the next item
        }
    }
    if (do_lanes) {  // no barrier from here on
        const uint32_t P = ctl->P;
        const uint32_t tid = threadIdx.x & 255u;
        // Four 256-lane groups per workgroup; group i of workgroup b is number i * gridDim.x + b,
        // so that neighbouring rounds go to different workgroups (CUs) and a small step still
        // uses every CU.
        const uint32_t blocks = gridDim.x * (kWgThreads / 256);
        const uint32_t block = (threadIdx.x >> 8) * gridDim.x + blockIdx.x;
        // no transit went to the other classes this step: nothing to look up in the bitmap
        if (heavy_bits != nullptr && (ctl->n_wg | ctl->n_chunks) != 0u)
            sub_loop<DRAW, true>(g, a, P, keys, vals, heavy_bits, pairs_per_block, tid, block, blocks);
        else
            sub_loop<DRAW, false>(g, a, P, keys, vals, heavy_bits, pairs_per_block, tid, block, blocks);
    }
}

template <int DRAW, typename OffT>
int launch_tp(const Graph& gr, const DrawArgs& a, const SchedParams& sp, const TpStep& t,
              hipStream_t stream) {
    const GraphView<OffT> g = view_of<OffT>(gr);
    const bool lanes = sp.force_class == ND_CLASS_AUTO || sp.force_class == ND_CLASS_SUBWAVE;
    const bool heavy = sp.force_class != ND_CLASS_SUBWAVE;
    // Workgroups that are all resident at once (two per CU: 8 waves per SIMD), fewer when the
    // step is small: one per 1,024 draws for the lane-per-draw part, one per heavy item.
    const int64_t places = (int64_t)gr.num_cus * 2;
    int64_t blocks = 1;
    const int64_t rounds = (t.max_draws + 255) / 256;   // upper bound
    if (lanes) blocks = rounds < places ? rounds : places;
    if (heavy && t.max_wg + t.max_chunks > blocks) blocks = t.max_wg + t.max_chunks;
    blocks = blocks < 1 ? 1 : (blocks > places ? places : blocks);
    // whole pairs per 256-lane round when that idles under a tenth of the lanes
    uint32_t ppb = a.m <= 256u ? 256u / a.m : 0u;
    if (ppb * a.m < 231u) ppb = 0u;
    mark_phase(lanes ? ND_PHASE_SAMPLE_SUB : ND_PHASE_SAMPLE_WG, stream);
    hipLaunchKernelGGL((sample_tp_kernel<DRAW, OffT>), dim3((unsigned)blocks), dim3(kWgThreads), 0,
                       stream, g, a, sp, t.ctl, t.keys, t.vals, t.g_key, t.g_start, t.list_wg,
                       t.chunk_gid, t.chunk_idx, (uint32_t)t.cap_wg, (uint32_t)t.cap_chunks,
                       sp.force_class == ND_CLASS_AUTO ? (const uint32_t*)t.heavy_bits : nullptr, ppb,
                       heavy ? 1 : 0, lanes ? 1 : 0);
    ND_HIP_CHECK(hipGetLastError());
    return ND_OK;
}

template <int DRAW, typename OffT>
int launch_sp(const Graph& gr, const DrawArgs& a, const int32_t* src, int64_t n_slots,
              int check_roots, uint32_t* status, hipStream_t stream) {
    const GraphView<OffT> g = view_of<OffT>(gr);
    const int64_t total = n_slots * (int64_t)a.m;
    if (total == 0) return ND_OK;
    const int64_t blocks = (total + 255) / 256;
    hipLaunchKernelGGL((sample_sp_kernel<DRAW, OffT>), dim3((unsigned)blocks), dim3(256), 0, stream, g,
                       a, src, n_slots, check_roots, status);
    ND_HIP_CHECK(hipGetLastError());
    return ND_OK;
}

// ---------------------------------------------------------------- unique neighbours (Section 6.3)
// One group of lanes per sample.  The paper removes duplicates with a per-sample sort and scan;
// here the vertices a sample holds live in an LDS hash table (open addressing, at least twice
// as many buckets as slots).  Every bucket remembers the best claim on its vertex: 0 once a
// slot holds it, otherwise the lowest slot index (+1) proposing it this round - an atomicMin,
// so the outcome does not depend on the order in which lanes arrive.  Slots that lose draw
// again straight from the graph (the paper's sample-parallel refill).  A slot whose parent's
// slots already hold as many distinct vertices as the parent's row has entries can only draw a
// held vertex; it ends empty at once instead of drawing in vain for the rounds that are left.
// The kernel is bound by instruction issue, so idle lanes are what it pays for:
//  * the group is sized to the sample, THREADS * kPerThread >= W slots: half a wavefront for the
//    25-slot first hop of GraphSAGE, a whole one, four slots per lane, for its 250-slot second hop;
//  * after the first round the slots still open are few and scattered, so they are packed into a
//    queue in LDS and the later rounds run lane-per-queue-entry, with the counter-based generator
//    keyed by the slot the entry names;
//  * groups of a wavefront or less share a 256-lane workgroup, each with its own table and queues,
//    and every group walks over samples with a stride.
template <int THREADS>
__device__ __forceinline__ void group_sync() {
    if (THREADS > 64) {
        __syncthreads();
    } else {  // part of one wavefront: its LDS operations complete in order; keep the compiler from moving them
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
}
// true when x is non-zero in any lane of the group; group_lanes: the group's lanes within its wavefront
template <int THREADS>
__device__ __forceinline__ int group_or(int x, uint64_t group_lanes) {
    if (THREADS > 64) return __syncthreads_or(x);
    group_sync<THREADS>();
    const int r = (__ballot(x != 0) & group_lanes) != 0ull;
    group_sync<THREADS>();
    return r;
}
// A queue place for every lane with flag set (any order).  A group inside one wavefront counts in a
// register (*fill, the same in all its lanes); a four-wavefront group counts in LDS (*fill_lds).
// Every lane of the group calls it, in converged code.
template <int THREADS>
__device__ __forceinline__ uint32_t group_reserve(bool flag, uint64_t group_lanes, uint32_t* fill, uint32_t* fill_lds) {
    const uint64_t votes = __ballot(flag) & group_lanes;
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t before = (uint32_t)__popcll(votes & ((1ull << lane) - 1ull));
    const uint32_t n = (uint32_t)__popcll(votes);
    if (THREADS > 64) {
        uint32_t base = 0;
        if (lane == 0 && n > 0) base = atomicAdd(fill_lds, n);
        base = (uint32_t)__shfl((int)base, 0, 64);
        return base + before;
    }
    const uint32_t base = *fill;
    *fill = base + n;
    return base + before;
}

template <typename OffT, int THREADS, int kPerThread>
__global__ __launch_bounds__(256) void unique_kernel(GraphView<OffT> g, UniqueArgs a, uint32_t num_samples) {
    static_assert(THREADS == 32 || THREADS == 64 || THREADS == 256, "a group is half a wavefront, one, or four");
    constexpr int SUBS = 256 / THREADS;  // groups (samples in flight) per workgroup
    constexpr uint32_t kSlots = THREADS * kPerThread;
    constexpr uint32_t kBuckets = 2 * kSlots;
    static_assert(kSlots <= 65536, "queue entries are 16-bit slot numbers");
    __shared__ int32_t h_key_all[SUBS][kBuckets];     // vertex of the bucket, NULL = empty
    __shared__ uint32_t h_claim_all[SUBS][kBuckets];  // 0 = held by a slot, else lowest proposing slot + 1
    __shared__ uint16_t q_all[SUBS][2][kSlots];       // slots still open: this round's queue and the next's
    __shared__ uint32_t q_fill[2];                    // queue lengths of a four-wavefront group
    __shared__ uint32_t p_held_all[SUBS][kSlots];     // per parent: distinct vertices its slots hold
    const uint32_t sub = threadIdx.x / (uint32_t)THREADS;
    const uint32_t tix = threadIdx.x % (uint32_t)THREADS;  // my place in the group
    // two half-wavefront groups share a wavefront and diverge where their samples differ
    const uint64_t group_lanes = THREADS == 32 ? 0xFFFFFFFFull << (threadIdx.x & 32u) : ~0ull;
    int32_t* h_key = h_key_all[sub];
    uint32_t* h_claim = h_claim_all[sub];
    uint32_t* p_held = p_held_all[sub];
    const uint32_t W = a.W;
    uint32_t buckets = 64;                  // power of two, at least 2 W
    while (buckets < 2u * W) buckets <<= 1;
    const uint32_t mask = buckets - 1u;

    // proposes vertex c for slot j; returns the bucket of c.  The table never holds more than W
    // distinct vertices (every proposed vertex is held by the end of its round) in at least 2 W
    // buckets, so a free or matching bucket is found long before the probe bound.
    auto propose = [&](int32_t c, uint32_t j) -> uint32_t {
        uint32_t b = ((uint32_t)c * 2654435761u) & mask;
        for (uint32_t probe = 0; probe < buckets; ++probe) {
            const int32_t old = atomicCAS(&h_key[b], ND_NULL_VERTEX, c);
            if (old == ND_NULL_VERTEX || old == c) break;
            b = (b + 1u) & mask;
        }
        atomicMin(&h_claim[b], j + 1u);
        return b;
    };

    for (uint32_t s = blockIdx.x * SUBS + sub; s < num_samples; s += gridDim.x * SUBS) {  // the same s in the whole group
        int32_t* out_row = a.out + (uint64_t)s * W;
        // ---- round 0 was drawn by the step's ordinary kernels: every vertex in the row is a candidate
        int32_t cand[kPerThread];               // candidate of my slot t (NULL: nothing to place)
        int any_candidate = 0;
#pragma unroll
        for (int t = 0; t < kPerThread; ++t) {
            const uint32_t j = tix + (uint32_t)t * (uint32_t)THREADS;
            cand[t] = j < W ? out_row[j] : ND_NULL_VERTEX;
            any_candidate |= cand[t] >= 0 ? 1 : 0;
        }
        if (!group_or<THREADS>(any_candidate, group_lanes)) continue;  // uniform: a sample without live parents is done
        for (uint32_t b = tix; b < buckets; b += (uint32_t)THREADS) {
            h_key[b] = ND_NULL_VERTEX;
            h_claim[b] = 0xFFFFFFFFu;
        }
        for (uint32_t pj = tix; pj < a.W_prev; pj += (uint32_t)THREADS) p_held[pj] = 0;
        if (THREADS > 64 && tix == 0) q_fill[0] = 0;
        group_sync<THREADS>();
        uint32_t where[kPerThread];
#pragma unroll
        for (int t = 0; t < kPerThread; ++t) {
            where[t] = 0;
            if (cand[t] >= 0) where[t] = propose(cand[t], tix + (uint32_t)t * (uint32_t)THREADS);
        }
        group_sync<THREADS>();
        bool won[kPerThread];
#pragma unroll
        for (int t = 0; t < kPerThread; ++t)
            won[t] = cand[t] >= 0 && h_claim[where[t]] == tix + (uint32_t)t * (uint32_t)THREADS + 1u;
        group_sync<THREADS>();                  // every claim has been read
        // a winner keeps what the step's kernels wrote and marks its bucket as held: whoever proposes
        // that vertex later loses; a loser queues for the next round
        uint32_t cur = 0;                       // the queue being read
        uint32_t fill = 0;                      // entries in the queue being written (group inside one wavefront)
#pragma unroll
        for (int t = 0; t < kPerThread; ++t) {
            if (won[t]) {
                h_claim[where[t]] = 0u;
                atomicAdd(&p_held[fastdiv(tix + (uint32_t)t * (uint32_t)THREADS, a.div_m)], 1u);
            }
            const bool open = cand[t] >= 0 && !won[t];
            const uint32_t at = group_reserve<THREADS>(open, group_lanes, &fill, &q_fill[0]);
            if (open) q_all[sub][0][at] = (uint16_t)(tix + (uint32_t)t * (uint32_t)THREADS);
        }
        if (THREADS > 64 && tix == 0) q_fill[1] = 0;
        group_sync<THREADS>();
        uint32_t L = THREADS > 64 ? q_fill[0] : fill;  // slots still open (uniform in the group)

        // ---- later rounds: one lane per queue entry
        for (int32_t r = 1; r < a.rounds && L > 0; ++r) {
            uint32_t jq[kPerThread];
#pragma unroll
            for (int p = 0; p < kPerThread; ++p) {
                const uint32_t e = tix + (uint32_t)p * (uint32_t)THREADS;
                cand[p] = ND_NULL_VERTEX;
                where[p] = 0;
                jq[p] = 0;
                if (e >= L) continue;
                const uint32_t j = q_all[sub][cur][e];
                const uint32_t pj = fastdiv(j, a.div_m);
                const int32_t v = a.parents[(uint64_t)s * a.W_prev + pj];  // live: it drew in round 0
                const uint64_t rs = (uint64_t)g.off[v];
                const uint32_t deg = row_length(g, v, rs);
                if (p_held[pj] >= deg) {
                    // the parent's slots already hold as many distinct vertices as its row has entries:
                    // whatever this slot draws is held, now and in every later round
                    out_row[j] = ND_NULL_VERTEX;
                    continue;
                }
                const Rand4 rn = draw4(a.seed, a.sample_base + s, j, a.step, (uint32_t)r);
                cand[p] = g.col[rs + mulhi32(rn.r0, deg)];
                jq[p] = j;
                where[p] = propose(cand[p], j);
            }
            group_sync<THREADS>();
#pragma unroll
            for (int p = 0; p < kPerThread; ++p) won[p] = cand[p] >= 0 && h_claim[where[p]] == jq[p] + 1u;
            group_sync<THREADS>();              // every claim has been read
            fill = 0;
#pragma unroll
            for (int p = 0; p < kPerThread; ++p) {
                if (won[p]) {
                    h_claim[where[p]] = 0u;
                    out_row[jq[p]] = cand[p];
                    atomicAdd(&p_held[fastdiv(jq[p], a.div_m)], 1u);
                }
                const bool open = cand[p] >= 0 && !won[p];
                const uint32_t at = group_reserve<THREADS>(open, group_lanes, &fill, &q_fill[cur ^ 1u]);
                if (open) q_all[sub][cur ^ 1u][at] = (uint16_t)jq[p];
            }
            if (THREADS > 64 && tix == 0) q_fill[cur] = 0;  // everybody read it two barriers ago
            group_sync<THREADS>();
            cur ^= 1u;
            L = THREADS > 64 ? q_fill[cur] : fill;
        }
        // ---- a slot that never won a vertex of its own ends empty
#pragma unroll
        for (int p = 0; p < kPerThread; ++p) {
            const uint32_t e = tix + (uint32_t)p * (uint32_t)THREADS;
            if (e < L) out_row[q_all[sub][cur][e]] = ND_NULL_VERTEX;
        }
        group_sync<THREADS>();  // table and queues are rebuilt for the group's next sample
    }
}

// ---------------------------------------------------------------- multi-dimensional walk
__global__ __launch_bounds__(256) void mrw_init_kernel(const int32_t* __restrict__ roots, int64_t n,
                                                       int32_t V, int32_t* __restrict__ state,
                                                       uint32_t* __restrict__ status) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    int32_t v = roots[i];
    if (v >= V || v < ND_NULL_VERTEX) {
        atomicOr(status, 1u);
        v = ND_NULL_VERTEX;
    }
    state[i] = v;
}

// UPDATE = false: transits[s] = the picked root.  UPDATE = true: the picked root becomes added[s].
template <bool UPDATE>
__global__ __launch_bounds__(256) void mrw_pick_kernel(int32_t* __restrict__ state, int64_t S,
                                                       uint32_t R, uint64_t seed, uint32_t sample_base,
                                                       uint32_t step, int32_t* __restrict__ transits,
                                                       const int32_t* __restrict__ added) {
    const int64_t s = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (s >= S) return;
    const Rand4 r = draw4(seed, sample_base + (uint32_t)s, 0u, step, 0u);
    const uint32_t pick = mulhi32(r.r2, R);
    if (UPDATE) {
        const int32_t v = added[s];
        if (v >= 0) state[s * (int64_t)R + pick] = v;
    } else {
        transits[s] = state[s * (int64_t)R + pick];
    }
}

}  // namespace

int unique_step(const Graph& gr, const UniqueArgs& a, int64_t num_samples, hipStream_t stream) {
    if (num_samples == 0) return ND_OK;
#define ND_UNIQUE_LAUNCH(THREADS, PER)                                                              \
    do {                                                                                            \
        const int subs = 256 / (THREADS);                                                           \
        int64_t blocks = (num_samples + subs - 1) / subs;                                           \
        const int64_t cap = (int64_t)gr.num_cus * 48; /* measured: 16 to 128 per unit within 4 % */ \
        if (blocks > cap) blocks = cap; /* every group walks over samples with a stride */          \
        if (gr.off64)                                                                               \
            hipLaunchKernelGGL((unique_kernel<int64_t, THREADS, PER>), dim3((unsigned)blocks),      \
                               dim3(256), 0, stream, view_of<int64_t>(gr), a, (uint32_t)num_samples); \
        else                                                                                        \
            hipLaunchKernelGGL((unique_kernel<int32_t, THREADS, PER>), dim3((unsigned)blocks),      \
                               dim3(256), 0, stream, view_of<int32_t>(gr), a, (uint32_t)num_samples); \
    } while (0)
    // up to 256 slots at most one wavefront per sample (its barriers cost nothing), more lanes above
    if (a.W <= 32) ND_UNIQUE_LAUNCH(32, 1);
    else if (a.W <= 64) ND_UNIQUE_LAUNCH(64, 1);
    else if (a.W <= 128) ND_UNIQUE_LAUNCH(64, 2);
    else if (a.W <= 256) ND_UNIQUE_LAUNCH(64, 4);
    else if (a.W <= 512) ND_UNIQUE_LAUNCH(256, 2);
    else if (a.W <= 1024) ND_UNIQUE_LAUNCH(256, 4);
    else ND_UNIQUE_LAUNCH(256, 8);
#undef ND_UNIQUE_LAUNCH
    ND_HIP_CHECK(hipGetLastError());
    return ND_OK;
}

int multirw_init(const Graph& gr, const int32_t* roots, int64_t n, int32_t* state, uint32_t* status,
                 hipStream_t stream) {
    if (n == 0) return ND_OK;
    hipLaunchKernelGGL(mrw_init_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, roots,
                       n, (int32_t)gr.V, state, status);
    ND_HIP_CHECK(hipGetLastError());
    return ND_OK;
}

int multirw_select(const int32_t* state, int64_t S, uint32_t R, uint64_t seed, uint32_t sample_base,
                   uint32_t step, int32_t* transits, hipStream_t stream) {
    if (S == 0) return ND_OK;
    hipLaunchKernelGGL(mrw_pick_kernel<false>, dim3((unsigned)((S + 255) / 256)), dim3(256), 0, stream,
                       const_cast<int32_t*>(state), S, R, seed, sample_base, step, transits,
                       (const int32_t*)nullptr);
    ND_HIP_CHECK(hipGetLastError());
    return ND_OK;
}

int multirw_update(int32_t* state, int64_t S, uint32_t R, uint64_t seed, uint32_t sample_base,
                   uint32_t step, const int32_t* added, hipStream_t stream) {
    if (S == 0) return ND_OK;
    hipLaunchKernelGGL(mrw_pick_kernel<true>, dim3((unsigned)((S + 255) / 256)), dim3(256), 0, stream,
                       state, S, R, seed, sample_base, step, (int32_t*)nullptr, added);
    ND_HIP_CHECK(hipGetLastError());
    return ND_OK;
}

#define ND_DISPATCH(DRAWV, CALL)                                                         \
    do {                                                                                 \
        if (gr.off64) {                                                                  \
            using OffT = int64_t;                                                        \
            if ((DRAWV) == kDrawUniform) { constexpr int D = kDrawUniform; return CALL; } \
            if ((DRAWV) == kDrawWeighted) { constexpr int D = kDrawWeighted; return CALL; } \
            { constexpr int D = kDrawNode2vec; return CALL; }                            \
        } else {                                                                         \
            using OffT = int32_t;                                                        \
            if ((DRAWV) == kDrawUniform) { constexpr int D = kDrawUniform; return CALL; } \
            if ((DRAWV) == kDrawWeighted) { constexpr int D = kDrawWeighted; return CALL; } \
            { constexpr int D = kDrawNode2vec; return CALL; }                            \
        }                                                                                \
    } while (0)

int sample_step_tp(const Graph& gr, int draw, const DrawArgs& a, const SchedParams& sp,
                   const TpStep& t, hipStream_t stream) {
    ND_DISPATCH(draw, (launch_tp<D, OffT>(gr, a, sp, t, stream)));
}

int sample_step_sp(const Graph& gr, int draw, const DrawArgs& a, const int32_t* src, int64_t n_slots,
                   int check_roots, uint32_t* status, hipStream_t stream) {
    ND_DISPATCH(draw, (launch_sp<D, OffT>(gr, a, src, n_slots, check_roots, status, stream)));
}

}  // namespace nd
