// Random walks with the scheduling index built per window of samples, in LDS.
//
// Section 6.1.2 of the paper builds the transit-to-sample map of a step with a
// GPU-wide radix sort and scan, which Section 8.1 measures at up to 40 % of a
// walk's time: a walk step draws one neighbour per sample, so grouping moves
// more bytes than sampling does.  Here a workgroup owns a window of consecutive
// samples for the whole walk and keeps their (transit, sample) pairs in its
// LDS: at every step it
//   1. enters the transit of every live slot in a table in LDS that counts the
//      window's pairs per transit (transit enumeration),
//   2. lets the slots of a transit with few pairs in the window draw at once, one
//      lane per pair in slot order (sub-wavefront class: what such a small group
//      could share, the caches share for it),
//   3. sorts the pairs of the transits with many pairs by transit with a stable
//      least-significant-digit radix sort, ranking with wave64 ballots (the
//      scheme of the GPU-wide sort), and finds the group heads where the transit
//      changes,
//   4. serves those groups workgroup-wide, the adjacency list staged in LDS when
//      it fits (workgroup class); when the sub-wavefront class is forced, all
//      pairs are sorted and drawn one lane per pair in transit order,
//   5. hands every grouped sample its new vertex through LDS, so the step's
//      output leaves in slot order as whole cache lines.
// One launch covers up to 128 steps; nothing is exchanged between workgroups,
// so there is no GPU-wide sort, scan or barrier.  What is drawn is the same
// Philox call per (sample, step, attempt) as everywhere else: outputs are
// identical to those of the GPU-wide grouping and of the sample-parallel kernel.
#include "nd_common.h"
#include "nd_philox.h"
#include "nd_wave.h"
#include "nd_sample.h"
#include "nd_draw.h"

namespace nd {

namespace {

constexpr int kWalkChunk = 128;        // steps per launch: their output pointers are kernel arguments
constexpr uint32_t kDoneMark = 0x8000u;  // set in a pair's slot entry once a heavy group has served it

struct WalkArgs {
    DrawArgs d;                // step, has_prev, out and prev_transit are set per step by the kernel
    uint32_t S;                // samples of the call
    uint32_t first_step, n_steps;
    int32_t key_bits;          // bits of a vertex id
    uint32_t heavy_min;        // pairs of one transit inside a window from which the workgroup class takes over
    int32_t force_class;       // nd_sched_class
    int32_t V;
    int32_t check_roots;
    const int32_t* roots;      // the call's roots (samples, or samples * R for the multi-dimensional walk)
    const int32_t* cur_src;    // first_step > 0: output of step first_step - 1
    const int32_t* prev_src;   // node2vec, first_step > 0: roots (first_step == 1) or output of step first_step - 2
    uint32_t* status;
    StepCtl* ctl;              // ctl[step]: counters of the call, added to by every window
    int32_t* state;            // multi-dimensional walk: the samples' root sets (S * R)
    uint32_t R;
    int32_t* out[kWalkChunk];
};

// One draw, out of line where the inlined code is long (the rejection loop of node2vec), so that
// the unrolled per-slot loops below stay small.  What it needs travels by value, in registers: a
// structure handed over by reference has to live in scratch memory, and then for the whole kernel,
// so that every other use of the graph's pointers would go through scratch as well.
template <typename OffT>
__device__ __noinline__ int32_t draw_n2v_call(const OffT* off, const int32_t* col, const uint32_t* wq_row,
                                              const uint32_t* maxwq, uint64_t seed, uint32_t step,
                                              uint32_t b_ret, uint32_t b_com, uint32_t b_far, uint32_t b_max,
                                              int32_t max_attempts, int32_t has_prev, int32_t v, uint32_t deg,
                                              uint32_t sid, int32_t t_prev, const int32_t* adj) {
    const GraphView<OffT> g{off, col, nullptr, nullptr, maxwq, 0};
    DrawArgs d;  // only the fields the draw reads are set
    d.seed = seed;
    d.step = step;
    d.b_ret = b_ret;
    d.b_com = b_com;
    d.b_far = b_far;
    d.b_max = b_max;
    d.max_attempts = max_attempts;
    d.has_prev = has_prev;
    d.use_weights = wq_row != nullptr;
    return draw_node2vec(g, d, v, deg, sid, t_prev, adj, wq_row);
}

template <int DRAW, typename OffT>
__device__ __forceinline__ int32_t draw_one(const GraphView<OffT>& g, const DrawArgs& d, int32_t v,
                                            uint64_t rs, uint32_t deg, uint32_t sid, int32_t t_prev,
                                            const int32_t* adj) {
    if (deg == 0) return ND_NULL_VERTEX;
    if (DRAW == kDrawUniform) return draw_uniform(d, deg, sid, 0u, adj);
    if (DRAW == kDrawWeighted) return draw_weighted(d, deg, sid, 0u, adj, g.cumq + rs);
    return draw_n2v_call<OffT>(g.off, g.col, d.use_weights ? g.wq + rs : nullptr, g.maxwq, d.seed, d.step, d.b_ret,
                               d.b_com, d.b_far, d.b_max, d.max_attempts, d.has_prev, v, deg, sid, t_prev, adj);
}

// Bucket of the per-window transit table: [63:48] tag of the step that wrote it, [47:32] number
// of the window's pairs on this transit, [31:0] the transit.  A bucket whose tag is not the
// current step's is free, so the table is never cleared.
__device__ __forceinline__ uint32_t tab_tag(unsigned long long w) { return (uint32_t)(w >> 48); }
__device__ __forceinline__ uint32_t tab_count(unsigned long long w) { return (uint32_t)(w >> 32) & 0xFFFFu; }

template <int DRAW, bool MRW, typename OffT, int THREADS, int ITEMS>
__global__ __launch_bounds__(THREADS) void walk_window_kernel(GraphView<OffT> g, WalkArgs a) {
    constexpr int N = THREADS * ITEMS;
    constexpr int WAVES = THREADS / 64;
    constexpr uint32_t NB = 2u * N;          // buckets: at most N distinct transits, so at most half full
    static_assert(THREADS >= 256 && N < (int)kDoneMark, "one thread per digit value; slot index below the mark bit");
    __shared__ unsigned long long s_tab[NB]; // transit -> number of pairs in the window, this step
    __shared__ int32_t s_key[2][N];          // transits of the pairs to be grouped (ping-pong of the sort)
    __shared__ uint16_t s_val[2][N];         // their slot inside the window
    __shared__ int32_t s_res[N];             // new vertex of every grouped slot
    __shared__ int32_t s_prev[DRAW == kDrawNode2vec ? N : 1];  // node2vec: previous transit of grouped slots
    __shared__ uint32_t s_hist[WAVES][256];
    __shared__ uint32_t s_digit_start[256];
    __shared__ uint32_t s_tmp[WAVES + 2];
    __shared__ uint32_t s_cnt[3][4];         // per step (three sets used in turn): grouped pairs, live pairs,
                                             // distinct transits, heavy transits

    const int tid = threadIdx.x, lane = lane_id(), wv = wave_id();
    const uint32_t base_slot = blockIdx.x * (uint32_t)N;
    const uint32_t n_here = a.S - base_slot < (uint32_t)N ? a.S - base_slot : (uint32_t)N;
    const bool all_grouped = a.force_class != ND_CLASS_AUTO;  // a forced class sees every pair

    int passes = (a.key_bits + 7) / 8;
    if (passes < 1) passes = 1;

    for (uint32_t i = tid; i < NB; i += THREADS) s_tab[i] = 0ull;  // tag 0: no step
    if (tid < 12) (&s_cnt[0][0])[tid] = 0;

    // ---- state of my slots: slot l = it * THREADS + tid of the window
    int32_t cur[ITEMS], prev[ITEMS];
    uint32_t pick[ITEMS];
    if (MRW && a.first_step == 0) {  // the window's root sets, checked once
        const uint64_t rb = (uint64_t)base_slot * a.R;
        const uint32_t cnt = n_here * a.R;  // below 2^31 by the call's plan
        bool bad = false;
        for (uint32_t i = tid; i < cnt; i += THREADS) {
            int32_t v = a.roots[rb + i];
            if (v >= a.V || v < ND_NULL_VERTEX) {
                bad = true;
                v = ND_NULL_VERTEX;
            }
            a.state[rb + i] = v;
        }
        if (bad) atomicOr(a.status, 1u);
    }
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
        const uint32_t l = (uint32_t)(it * THREADS + tid);
        cur[it] = ND_NULL_VERTEX;
        prev[it] = ND_NULL_VERTEX;
        pick[it] = 0;
        if (!MRW && l < n_here) {
            if (a.first_step == 0) {
                int32_t v = a.roots[base_slot + l];
                if (v >= a.V || v < ND_NULL_VERTEX) {
                    if (a.check_roots) atomicOr(a.status, 1u);
                    v = ND_NULL_VERTEX;
                }
                cur[it] = v;
            } else {
                cur[it] = a.cur_src[base_slot + l];
                if (DRAW == kDrawNode2vec && a.prev_src != nullptr) prev[it] = a.prev_src[base_slot + l];
            }
        }
    }
    __syncthreads();  // table and counters cleared; the root sets written above are visible

    for (uint32_t si = 0; si < a.n_steps; ++si) {
        const uint32_t step = a.first_step + si;
        DrawArgs d = a.d;
        d.step = step;
        d.has_prev = step > 0;
        uint32_t* cnt_now = s_cnt[si % 3u];
        const unsigned long long tag = (unsigned long long)(si + 1u) << 48;

        // ---- 1. transit enumeration: every live slot enters its transit in the window's table
        uint32_t bucket[ITEMS];
        uint32_t first_w = 0, live_w = 0;  // of my wavefront: transits entered first, live slots
#pragma unroll
        for (int it = 0; it < ITEMS; ++it) {
            const uint32_t l = (uint32_t)(it * THREADS + tid);
            if (MRW) {
                cur[it] = ND_NULL_VERTEX;
                if (l < n_here) {
                    const Rand4 r = draw4(d.seed, d.sample_base + base_slot + l, 0u, step, 0u);
                    pick[it] = mulhi32(r.r2, a.R);
                    cur[it] = a.state[(uint64_t)(base_slot + l) * a.R + pick[it]];
                }
            }
            bucket[it] = 0;
            bool entered = false;
            if (cur[it] >= 0) {
                const uint32_t key = (uint32_t)cur[it];
                uint32_t b = (key * 2654435761u) >> 7 & (NB - 1u);
                for (uint32_t probe = 0; probe < NB; ++probe) {  // the table is at most half full
                    const unsigned long long old = s_tab[b];
                    if (tab_tag(old) != si + 1u) {                // free: claim it with count 1
                        if (atomicCAS(&s_tab[b], old, tag | (1ull << 32) | key) == old) {
                            entered = true;
                            break;
                        }
                        continue;                                 // somebody else took it: look again
                    }
                    if ((uint32_t)old == key) {
                        atomicAdd(&s_tab[b], 1ull << 32);
                        break;
                    }
                    b = (b + 1u) & (NB - 1u);
                }
                bucket[it] = b;
            }
            first_w += (uint32_t)__popcll(__ballot(entered));
            live_w += (uint32_t)__popcll(__ballot(cur[it] >= 0));
        }
        {   // counters of the step (one LDS atomic per wave)
            if (lane == 63) {
                if (first_w) atomicAdd(&cnt_now[2], first_w);
                if (live_w) atomicAdd(&cnt_now[1], live_w);
            }
            // The next step's set was last used two steps ago.  A thread can lag behind thread 0 by
            // less than one step (two barriers per step), so nobody can still be reading it; with
            // two sets a thread that has not yet read this step's pair count could see it cleared.
            if (tid == 0)
                for (int c = 0; c < 4; ++c) s_cnt[(si + 1u) % 3u][c] = 0;
        }
        __syncthreads();

        // ---- 2. a transit with few pairs in the window has little to share that the caches do not give
        //         anyway: its slots draw at once, in slot order.  Slots of the transits with many pairs
        //         (heavy_min or more) go on to be grouped.
        int32_t next[ITEMS];
        bool grouped[ITEMS];
        uint64_t rs[ITEMS];
        uint32_t deg[ITEMS];
#pragma unroll
        for (int it = 0; it < ITEMS; ++it) {
            const bool alive = cur[it] >= 0;
            grouped[it] = alive && (all_grouped || tab_count(s_tab[bucket[it]]) >= a.heavy_min);
            next[it] = ND_NULL_VERTEX;
            const int32_t v = alive && !grouped[it] ? cur[it] : 0;  // all row offsets first: independent loads
            rs[it] = (uint64_t)g.off[v];
            deg[it] = row_length(g, v, rs[it]);
        }
#pragma unroll
        for (int it = 0; it < ITEMS; ++it) {
            const uint32_t l = (uint32_t)(it * THREADS + tid);
            const uint64_t bal = __ballot(grouped[it]);
            uint32_t at = 0;
            if (lane == 0 && bal != 0) at = atomicAdd(&cnt_now[0], (uint32_t)__popcll(bal));
            at = __shfl(at, 0, 64);
            if (grouped[it]) {
                const uint32_t pos = at + (uint32_t)__popcll(bal & lanes_below(lane));
                s_key[0][pos] = cur[it];
                s_val[0][pos] = (uint16_t)l;
                if (DRAW == kDrawNode2vec) s_prev[l] = prev[it];
            } else if (cur[it] >= 0) {
                next[it] = draw_one<DRAW, OffT>(g, d, cur[it], rs[it], deg[it], d.sample_base + base_slot + l,
                                                prev[it], g.col + rs[it]);
            }
        }
        __syncthreads();
        const uint32_t P = wave_uniform(cnt_now[0]);  // pairs to group

        if (P > 0) {  // uniform for the workgroup
            // ---- 3. stable LSD radix sort of the P pairs by transit
            uint32_t chunk = ((P + WAVES - 1) / WAVES + 63u) & ~63u;  // consecutive pairs per wave
            const uint32_t w_begin = (uint32_t)wv * chunk;
            int shift = 0;
            for (int pass = 0; pass < passes; ++pass) {
                const int bits = a.key_bits / passes + (pass >= passes - a.key_bits % passes ? 1 : 0);
                const uint32_t mask = (1u << bits) - 1u;
                const int in = pass & 1, ob = in ^ 1;
                for (int i = tid; i < WAVES * 256; i += THREADS) (&s_hist[0][0])[i] = 0;
                __syncthreads();
                int32_t key[ITEMS];
                uint16_t val[ITEMS];
                uint32_t rank[ITEMS];
#pragma unroll
                for (int r = 0; r < ITEMS; ++r) {
                    key[r] = ND_NULL_VERTEX;
                    val[r] = 0;
                    rank[r] = 0;
                    if ((uint32_t)(r * 64) >= chunk) continue;  // the same for the whole wave
                    const uint32_t idx = w_begin + (uint32_t)(r * 64 + lane);
                    const bool live = idx < P;
                    if (live) {
                        key[r] = s_key[in][idx];
                        val[r] = s_val[in][idx];
                    }
                    const uint32_t dg = ((uint32_t)key[r] >> shift) & mask;
                    const uint64_t peers = digit_peers(dg, __ballot(live), bits);
                    const uint32_t below = __builtin_amdgcn_mbcnt_hi((uint32_t)(peers >> 32),
                                                                     __builtin_amdgcn_mbcnt_lo((uint32_t)peers, 0u));
                    uint32_t old = 0;
                    if (live) {  // every live lane reads the count before the lowest of its peers writes it
                        old = s_hist[wv][dg];
                        if (below == 0u) s_hist[wv][dg] = old + (uint32_t)__popcll(peers);
                    }
                    // the next 64 pairs read these counters
                    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
                    __builtin_amdgcn_wave_barrier();
                    rank[r] = old + below;
                }
                __syncthreads();
                {
                    uint32_t cnt = 0;
                    if (tid < (1 << bits)) {
#pragma unroll
                        for (int w = 0; w < WAVES; ++w) {
                            const uint32_t t = s_hist[w][tid];
                            s_hist[w][tid] = cnt;
                            cnt += t;
                        }
                    }
                    uint32_t total;
                    const uint32_t ex = block_exclusive_scan<uint32_t, THREADS>(cnt, s_tmp, &total);
                    if (tid < (1 << bits)) s_digit_start[tid] = ex;
                }
                __syncthreads();
#pragma unroll
                for (int r = 0; r < ITEMS; ++r) {
                    if (key[r] >= 0) {
                        const uint32_t dg = ((uint32_t)key[r] >> shift) & mask;
                        const uint32_t pos = s_digit_start[dg] + s_hist[wv][dg] + rank[r];
                        s_key[ob][pos] = key[r];
                        s_val[ob][pos] = val[r];
                    }
                }
                __syncthreads();
                shift += bits;
            }
            const int fb = passes & 1;             // buffer that holds the sorted pairs
            int32_t* skey = s_key[fb];
            uint16_t* sval = s_val[fb];
            int32_t* stage = s_key[fb ^ 1];        // free now: LDS copy of a heavy transit's list
            uint16_t* heavy_list = s_val[fb ^ 1];  // free now: first pair of the groups the whole workgroup serves

            // ---- 4a. segments and classes: a pair is the head of its group when the transit changes; a
            //          group with at least heavy_min pairs goes to the workgroup class
            if (a.force_class != ND_CLASS_SUBWAVE) {
#pragma unroll
                for (int i = 0; i < ITEMS; ++i) {
                    const uint32_t p = (uint32_t)(i * THREADS + tid);
                    if ((uint32_t)(i * THREADS) >= P) break;  // uniform
                    const int32_t k = p < P ? skey[p] : -2;
                    int32_t before = __shfl_up(k, 1, 64);
                    if (lane == 0) before = (p > 0 && p < P) ? skey[p - 1] : -3;
                    if (p < P && k != before) {
                        const uint32_t last = p + a.heavy_min - 1u;
                        if (a.force_class == ND_CLASS_WORKGROUP || (last < P && skey[last] == k))
                            heavy_list[atomicAdd(&cnt_now[3], 1u)] = (uint16_t)p;
                    }
                }
                __syncthreads();
            }
            const uint32_t n_heavy = wave_uniform(cnt_now[3]);
            uint32_t n_staged = 0, heavy_draws = 0;
            for (uint32_t hi = 0; hi < n_heavy; ++hi) {  // uniform trip count
                const uint32_t p0 = heavy_list[hi];
                const int32_t v = skey[p0];
                uint32_t lo = p0 + 1u, hi_p = P;          // end of the group: first pair with another transit
                while (lo < hi_p) {
                    const uint32_t mid = (lo + hi_p) >> 1;
                    if (skey[mid] == v) lo = mid + 1u;
                    else hi_p = mid;
                }
                const uint32_t p1 = lo;
                const uint64_t hrs = (uint64_t)g.off[v];
                const uint32_t hdeg = row_length(g, v, hrs);
                bool do_stage = hdeg > 0 && hdeg <= (uint32_t)N && d.lds_policy != 1;
                if (d.lds_policy == 0) do_stage = do_stage && hdeg >= 128u && hdeg / 4u <= p1 - p0;
                const int32_t* adj = g.col + hrs;
                if (do_stage) {
                    for (uint32_t i = tid; i < hdeg; i += THREADS) stage[i] = adj[i];
                    __syncthreads();
                    adj = stage;
                    ++n_staged;
                }
                heavy_draws += p1 - p0;
                for (uint32_t p = p0 + tid; p < p1; p += THREADS) {
                    const uint32_t l = sval[p];
                    s_res[l] = draw_one<DRAW, OffT>(g, d, v, hrs, hdeg, d.sample_base + base_slot + l,
                                                    s_prev[DRAW == kDrawNode2vec ? l : 0], adj);
                    sval[p] = (uint16_t)(l | kDoneMark);
                }
                __syncthreads();  // the staged list is replaced by the next group's
            }

            // ---- 4b. the other groups, one lane per pair in transit order
            if (a.force_class != ND_CLASS_WORKGROUP) {
#pragma unroll
                for (int i = 0; i < ITEMS; ++i) {
                    if ((uint32_t)(i * THREADS) >= P) break;  // uniform
                    const uint32_t p = (uint32_t)(i * THREADS + tid);
                    if (p >= P) continue;
                    const uint32_t l = sval[p];
                    if (l & kDoneMark) continue;
                    const int32_t v = skey[p];
                    const uint64_t prs = (uint64_t)g.off[v];
                    const uint32_t pdeg = row_length(g, v, prs);
                    s_res[l] = draw_one<DRAW, OffT>(g, d, v, prs, pdeg, d.sample_base + base_slot + l,
                                                    s_prev[DRAW == kDrawNode2vec ? l : 0], g.col + prs);
                }
            }
            if (tid == 0 && a.ctl != nullptr) {
                StepCtl* c = a.ctl + step;
                if (n_heavy) atomicAdd(&c->n_wg, n_heavy);
                if (n_staged) atomicAdd(&c->n_staged, n_staged);
                if (heavy_draws) atomicAdd(&c->heavy_draws, heavy_draws);
            }
            __syncthreads();
        }
        if (tid == 0 && a.ctl != nullptr && cnt_now[1] != 0) {
            atomicAdd(&a.ctl[step].P, cnt_now[1]);
            atomicAdd(&a.ctl[step].U, cnt_now[2]);
        }

        // ---- 5. every slot takes its new vertex; the step's output leaves in slot order
        int32_t* out = a.out[si];
#pragma unroll
        for (int it = 0; it < ITEMS; ++it) {
            const uint32_t l = (uint32_t)(it * THREADS + tid);
            if (l >= n_here) continue;
            const int32_t nv = grouped[it] ? s_res[l] : next[it];
            out[base_slot + l] = nv;
            if (MRW) {
                if (nv >= 0) a.state[(uint64_t)(base_slot + l) * a.R + pick[it]] = nv;
            } else {
                prev[it] = cur[it];
                cur[it] = nv;
            }
        }
    }
}

template <int DRAW, bool MRW, typename OffT>
int launch_windows(const Graph& gr, const WalkArgs& a, int window, hipStream_t stream) {
    const GraphView<OffT> g = view_of<OffT>(gr);
    if (window == 256) {
        const unsigned blocks = (unsigned)((a.S + 255u) / 256u);
        hipLaunchKernelGGL((walk_window_kernel<DRAW, MRW, OffT, 256, 1>), dim3(blocks), dim3(256), 0, stream, g, a);
    } else if (window == 1024) {
        const unsigned blocks = (unsigned)((a.S + 1023u) / 1024u);
        hipLaunchKernelGGL((walk_window_kernel<DRAW, MRW, OffT, 256, 4>), dim3(blocks), dim3(256), 0, stream, g, a);
    } else {
        const unsigned blocks = (unsigned)((a.S + 2047u) / 2048u);
        hipLaunchKernelGGL((walk_window_kernel<DRAW, MRW, OffT, 256, 8>), dim3(blocks), dim3(256), 0, stream, g, a);
    }
    ND_HIP_CHECK(hipGetLastError());
    return ND_OK;
}

template <typename OffT>
int dispatch_windows(const Graph& gr, int draw, bool multirw, const WalkArgs& a, int window,
                     hipStream_t stream) {
    if (multirw) return launch_windows<kDrawUniform, true, OffT>(gr, a, window, stream);
    if (draw == kDrawUniform) return launch_windows<kDrawUniform, false, OffT>(gr, a, window, stream);
    if (draw == kDrawWeighted) return launch_windows<kDrawWeighted, false, OffT>(gr, a, window, stream);
    return launch_windows<kDrawNode2vec, false, OffT>(gr, a, window, stream);
}

}  // namespace

int walk_window_auto(int64_t S) {
    // Windows of 256 samples (one per lane) give the most workgroups to overlap, which is what a
    // latency-bound walk step needs; measured on 4 K to 57 K walks they are 2x to 3.4x faster than
    // 1,024-sample windows.  Once the call saturates the memory system (millions of walks) the
    // window size no longer matters (7.56 / 7.36 / 7.27 ms for 256 / 1,024 / 2,048 on 4.19 M walks).
    return S >= (1 << 21) ? 1024 : 256;
}

int walk_windows(const Graph& gr, int draw, bool multirw, const DrawArgs& d, int64_t S, int32_t num_steps,
                 int window, uint32_t heavy_min, int force_class, const int32_t* roots, int check_roots,
                 int32_t* const* step_out, uint32_t* status, StepCtl* ctl, int32_t* mrw_state, uint32_t R,
                 hipStream_t stream) {
    if (S == 0) return ND_OK;
    WalkArgs a{};
    a.d = d;
    a.S = (uint32_t)S;
    a.key_bits = 1;
    while ((1ll << a.key_bits) < gr.V) ++a.key_bits;
    a.heavy_min = heavy_min;
    a.force_class = force_class;
    a.V = (int32_t)gr.V;
    a.check_roots = check_roots;
    a.roots = roots;
    a.status = status;
    a.ctl = ctl;
    a.state = mrw_state;
    a.R = R;
    for (int32_t first = 0; first < num_steps; first += kWalkChunk) {
        const int32_t n = num_steps - first < kWalkChunk ? num_steps - first : kWalkChunk;
        a.first_step = (uint32_t)first;
        a.n_steps = (uint32_t)n;
        a.cur_src = first > 0 ? step_out[first - 1] : nullptr;
        a.prev_src = first == 0 ? nullptr : (first == 1 ? roots : step_out[first - 2]);
        for (int32_t i = 0; i < kWalkChunk; ++i) a.out[i] = i < n ? step_out[first + i] : nullptr;
        mark_phase(ND_PHASE_WALK_WINDOW, stream);
        const int rc = gr.off64 ? dispatch_windows<int64_t>(gr, draw, multirw, a, window, stream)
                                : dispatch_windows<int32_t>(gr, draw, multirw, a, window, stream);
        if (rc != ND_OK) return rc;
    }
    return ND_OK;
}

}  // namespace nd
