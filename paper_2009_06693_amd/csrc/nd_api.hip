// C ABI: argument checking, workspace layout and the per-step loop that the
// host drives (Section 6 of the paper: the host coordinates the steps, the GPU
// executes them).  The host only enqueues kernels: every count a later kernel
// needs (live pairs, distinct transits, class sizes) stays in device memory,
// so nd_sample never waits for the GPU.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <vector>

#include "nd_common.h"
#include "nd_edges.h"
#include "nd_pack.h"
#include "nd_sample.h"

struct nd_graph {
    nd::Graph* g;
};

namespace nd {

namespace {

thread_local char g_error[512] = "";

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct Plan {
    int app = 0, mode = 0, k = 0;
    int collective = 0;
    int64_t S = 0;             // samples
    int64_t max_slots = 0;     // longest transit array over the steps (pair capacity)
    int64_t max_out = 0;       // longest output array
    int32_t sub_max = 16384, wg_max = 65536;
    int64_t cap_wg = 0, cap_chunks = 0;
    // workspace offsets
    size_t o_ctl = 0, o_keysA = 0, o_valsA = 0, o_keysB = 0, o_valsB = 0, o_hist = 0, o_tiles = 0,
           o_gkey = 0, o_gstart = 0, o_list_wg = 0, o_chunk_gid = 0, o_chunk_idx = 0, o_bits = 0,
           total = 0;
    int64_t bit_words = 0;
    size_t hist_bytes = 0;     // largest histogram over the steps' sort plans
    int64_t state_len = 0;     // multi-dimensional walk: vertices in the samples' root sets
    size_t o_state = 0, o_transits = 0;
    int window = 0;            // walks grouped per window of this many samples (0: GPU-wide grouping)
    uint32_t heavy_min = 64;   // pairs of one transit in a window from which the workgroup class serves it
};

int64_t step_fanout(int app, const nd_params* p, int i) {
    return (app == ND_KHOP || app == ND_LAYER) ? (int64_t)p->fanout[i] : 1;
}

// Length of step i's transit array and output array.
void step_shape(const Plan& pl, const nd_params* p, int i, int64_t* n_slots, int64_t* n_out) {
    if (pl.app == ND_LAYER) {
        *n_slots = pl.S * (i == 0 ? (int64_t)p->roots_per_sample : (int64_t)p->fanout[i - 1]);
        *n_out = pl.S * (int64_t)p->fanout[i];
        return;
    }
    int64_t w = 1;
    for (int l = 0; l < i; ++l) w *= step_fanout(pl.app, p, l);
    *n_slots = pl.S * w;
    *n_out = pl.S * w * step_fanout(pl.app, p, i);
}

int check_params(const Graph& g, int app, const nd_params* p, int64_t num_roots, Plan* pl) {
    if (p->struct_size != sizeof(nd_params)) {
        set_error("nd_params.struct_size is %u, expected %zu (call nd_params_init)", p->struct_size,
                  sizeof(nd_params));
        return ND_ERR_BAD_ARGUMENT;
    }
    if (app < ND_DEEPWALK || app > ND_MULTIRW) {
        set_error("unknown app %d", app);
        return ND_ERR_BAD_ARGUMENT;
    }
    if (p->mode != ND_MODE_TRANSIT_PARALLEL && p->mode != ND_MODE_SAMPLE_PARALLEL) {
        set_error("unknown mode %d", p->mode);
        return ND_ERR_BAD_ARGUMENT;
    }
    if (num_roots < 0) {
        set_error("num_roots is negative");
        return ND_ERR_BAD_ARGUMENT;
    }
    const bool walk = app == ND_DEEPWALK || app == ND_PPR || app == ND_NODE2VEC || app == ND_MULTIRW;
    if (p->num_steps < 1 || p->num_steps > (walk ? ND_MAX_WALK_STEPS : ND_MAX_FANOUT_STEPS)) {
        set_error("num_steps %d outside [1, %d]", p->num_steps,
                  walk ? ND_MAX_WALK_STEPS : ND_MAX_FANOUT_STEPS);
        return ND_ERR_BAD_ARGUMENT;
    }
    if (p->use_weights && !g.wq) {
        set_error("use_weights set but the graph was created without weights");
        return ND_ERR_NO_WEIGHTS;
    }
    if (p->use_weights && app != ND_LAYER && (!walk || app == ND_MULTIRW)) {
        set_error("use_weights applies to DeepWalk, PPR, node2vec and layer sampling only");
        return ND_ERR_BAD_ARGUMENT;
    }
    if (p->sched_force_class < ND_CLASS_AUTO || p->sched_force_class > ND_CLASS_GRID ||
        p->sched_sub_max < 0 || p->sched_wg_max < 0 || p->lds_stage_policy < 0 ||
        p->lds_stage_policy > 2 || p->sched_group_bits < 0 || p->sched_group_bits > 31 ||
        (p->sched_group_bits > 0 && p->sched_force_class != ND_CLASS_AUTO &&
         p->sched_force_class != ND_CLASS_SUBWAVE)) {
        set_error("bad scheduling override");
        return ND_ERR_BAD_ARGUMENT;
    }
    if (p->sched_window != 0 && p->sched_window != -1 && p->sched_window != 256 && p->sched_window != 1024 &&
        p->sched_window != 2048) {
        set_error("sched_window must be 0, -1, 256, 1024 or 2048");
        return ND_ERR_BAD_ARGUMENT;
    }
    if (p->sched_window > 0 && (!walk || p->sched_group_bits > 0 || p->sched_force_class == ND_CLASS_GRID)) {
        set_error("sched_window applies to random walks, without sched_group_bits and without the grid class");
        return ND_ERR_BAD_ARGUMENT;
    }
    pl->app = app;
    pl->mode = p->mode;
    pl->k = p->num_steps;
    pl->collective = app == ND_LAYER;
    pl->sub_max = p->sched_sub_max ? p->sched_sub_max : 16384;
    pl->wg_max = p->sched_wg_max ? p->sched_wg_max : 65536;
    if (pl->wg_max < pl->sub_max) {
        set_error("sched_wg_max below sched_sub_max");
        return ND_ERR_BAD_ARGUMENT;
    }
    if (p->unique_rounds < 0 || p->unique_rounds > 64 || (p->unique_rounds > 0 && app != ND_KHOP)) {
        set_error("unique_rounds must be in [0, 64] and applies to k-hop only");
        return ND_ERR_BAD_ARGUMENT;
    }
    if (app == ND_PPR && !(p->term_prob >= 0.0 && p->term_prob <= 1.0)) {
        set_error("term_prob outside [0, 1]");
        return ND_ERR_BAD_ARGUMENT;
    }
    if (app == ND_NODE2VEC) {
        if (p->bias_convention != 0 && p->bias_convention != 1) {
            set_error("bias_convention must be 0 or 1");
            return ND_ERR_BAD_ARGUMENT;
        }
        if (p->n2v_max_attempts < 0 || p->n2v_max_attempts > 4096) {
            set_error("n2v_max_attempts outside [0, 4096]");
            return ND_ERR_BAD_ARGUMENT;
        }
        if (!(p->p > 0.0) || !(p->q > 0.0)) {
            set_error("node2vec p and q must be positive");
            return ND_ERR_BAD_ARGUMENT;
        }
    }
    if (app == ND_LAYER) {
        if (p->roots_per_sample < 1 || p->roots_per_sample > ND_MAX_LAYER_TRANSITS) {
            set_error("roots_per_sample outside [1, %d]", ND_MAX_LAYER_TRANSITS);
            return ND_ERR_BAD_ARGUMENT;
        }
        if (num_roots % p->roots_per_sample) {
            set_error("num_roots is not a multiple of roots_per_sample");
            return ND_ERR_BAD_ARGUMENT;
        }
        if (g.max_degree >= (1ll << 24)) {
            set_error("layer sampling needs every degree below 2^24");
            return ND_ERR_TOO_LARGE;
        }
        pl->S = num_roots / p->roots_per_sample;
    } else if (app == ND_MULTIRW) {
        if (p->roots_per_sample < 1 || p->roots_per_sample > ND_MAX_LAYER_TRANSITS) {
            set_error("roots_per_sample outside [1, %d]", ND_MAX_LAYER_TRANSITS);
            return ND_ERR_BAD_ARGUMENT;
        }
        if (num_roots % p->roots_per_sample) {
            set_error("num_roots is not a multiple of roots_per_sample");
            return ND_ERR_BAD_ARGUMENT;
        }
        pl->S = num_roots / p->roots_per_sample;
        pl->state_len = num_roots;
    } else {
        pl->S = num_roots;
    }
    if ((uint64_t)pl->S + p->sample_id_base >= (1ull << 32) || p->sample_id_base >= (1ull << 32)) {
        set_error("sample ids (sample_id_base + samples) must stay below 2^32");
        return ND_ERR_TOO_LARGE;
    }
    if (app == ND_KHOP || app == ND_LAYER) {
        for (int i = 0; i < p->num_steps; ++i) {
            const int lim = app == ND_LAYER ? ND_MAX_LAYER_TRANSITS : (1 << 20);
            if (p->fanout[i] < 1 || p->fanout[i] > lim) {
                set_error("fanout[%d] = %d outside [1, %d]", i, p->fanout[i], lim);
                return ND_ERR_BAD_ARGUMENT;
            }
        }
    }
    pl->window = 0;
    if (walk && p->mode == ND_MODE_TRANSIT_PARALLEL) {
        const bool overridden = p->sched_force_class != ND_CLASS_AUTO || p->sched_sub_max != 0 ||
                                p->sched_wg_max != 0 || p->sched_group_bits != 0;
        if (p->sched_window > 0) pl->window = p->sched_window;
        else if (p->sched_window == 0 && !overridden) pl->window = walk_window_auto(pl->S);
        if (pl->window > 0 && p->sched_window > 0 && p->sched_sub_max > 0)
            pl->heavy_min = (uint32_t)p->sched_sub_max + 1u;
    }
    pl->max_slots = 0;
    pl->max_out = 0;
    double guard = 1.0;
    for (int i = 0; i < pl->k; ++i) {
        guard = (app == ND_KHOP) ? guard * p->fanout[i] : 1.0;
        if ((double)pl->S * guard >= 2147483648.0) {
            set_error("a step would have 2^31 or more slots");
            return ND_ERR_TOO_LARGE;
        }
        int64_t ns, no;
        step_shape(*pl, p, i, &ns, &no);
        if (ns >= (1ll << 31) || no >= (1ll << 31)) {
            set_error("a step would have 2^31 or more slots");
            return ND_ERR_TOO_LARGE;
        }
        if (ns > pl->max_slots) pl->max_slots = ns;
        if (no > pl->max_out) pl->max_out = no;
        if (p->unique_rounds > 0 && pl->S > 0 && no / pl->S > ND_MAX_UNIQUE_SLOTS) {
            set_error("unique neighbours need at most %d slots per sample and step (step %d has %lld)",
                      ND_MAX_UNIQUE_SLOTS, i, (long long)(no / pl->S));
            return ND_ERR_BAD_ARGUMENT;
        }
        const size_t hb = sort_hist_bytes(make_sort_plan(ns, g.V, p->sched_group_bits));
        if (hb > pl->hist_bytes) pl->hist_bytes = hb;
    }
    return ND_OK;
}

void layout(Plan* pl, int64_t V) {
    size_t o = sizeof(WsHeader);
    pl->o_ctl = o;
    o = align_up(o + sizeof(StepCtl) * (size_t)pl->k);
    if (pl->app == ND_MULTIRW) {
        pl->o_state = o; o = align_up(o + (size_t)(pl->state_len > 0 ? pl->state_len : 1) * 4);
        pl->o_transits = o; o = align_up(o + (size_t)(pl->S > 0 ? pl->S : 1) * 4);
    }
    if (pl->mode == ND_MODE_TRANSIT_PARALLEL && !pl->collective && pl->window == 0) {
        const size_t n = (size_t)(pl->max_slots > 0 ? pl->max_slots : 1);
        pl->o_keysA = o; o = align_up(o + n * 4);
        pl->o_valsA = o; o = align_up(o + n * 4);
        pl->o_keysB = o; o = align_up(o + n * 4);
        pl->o_valsB = o; o = align_up(o + n * 4);
        pl->o_hist = o; o = align_up(o + pl->hist_bytes);
        pl->o_tiles = o; o = align_up(o + seg_scratch_bytes(pl->max_slots));
        pl->o_gkey = o; o = align_up(o + n * 4);
        pl->o_gstart = o; o = align_up(o + (n + 1) * 4);
        // Capacities.  Without a forced class a workgroup-class transit has more than
        // sub_max draws and a grid-class transit more than wg_max, which bounds their number.
        const int64_t by_draws_wg = pl->max_out / pl->sub_max + 64;
        pl->cap_wg = by_draws_wg < pl->max_slots ? by_draws_wg : pl->max_slots;
        pl->cap_chunks = 2 * (pl->max_out / pl->wg_max) + 64;
        // a forced class can put every transit in one list
        pl->cap_wg = pl->max_slots > pl->cap_wg ? pl->max_slots : pl->cap_wg;
        pl->cap_chunks += pl->max_slots;
        pl->o_list_wg = o; o = align_up(o + (size_t)pl->cap_wg * 4);
        pl->o_chunk_gid = o; o = align_up(o + (size_t)pl->cap_chunks * 4);
        pl->o_chunk_idx = o; o = align_up(o + (size_t)pl->cap_chunks * 4);
        pl->bit_words = (V + 31) / 32;
        pl->o_bits = o; o = align_up(o + (size_t)pl->bit_words * 4);
    }
    pl->total = o;
}

__global__ void init_header_kernel(WsHeader* h, uint32_t num_steps, StepCtl* ctl, uint32_t* bits,
                                   int64_t bit_words) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i == 0) {
        h->status = 0;
        h->num_steps = num_steps;
    }
    if (i < num_steps) ctl[i] = StepCtl{};
    if (i < bit_words) bits[i] = 0;
}

__global__ void publish_counts_kernel(const StepCtl* ctl, int64_t* counts) {
    counts[0] = ctl->P;
    counts[1] = ctl->U;
}

int run_unique(const Graph& g, const nd_params* params, uint64_t seed, int step, int64_t S,
               int64_t n_slots, int64_t n_out, int32_t m, const int32_t* parents, int32_t* out,
               hipStream_t stream) {
    UniqueArgs u{};
    u.seed = seed;
    u.sample_base = (uint32_t)params->sample_id_base;
    u.step = (uint32_t)step;
    u.W = (uint32_t)(n_out / S);
    u.W_prev = (uint32_t)(n_slots / S);
    u.div_m = make_fastdiv((uint32_t)m);
    u.rounds = params->unique_rounds;
    u.parents = parents;
    u.out = out;
    mark_phase(ND_PHASE_UNIQUE, stream);
    return unique_step(g, u, S, stream);
}

uint32_t q16(double x) {
    const double q = std::floor(x * 65536.0 + 0.5);
    if (!(q >= 1.0) || q > 16777216.0) return 0;
    return (uint32_t)q;
}

}  // namespace

namespace {
struct Profiler {
    bool on = false;
    bool overflow = false;
    std::vector<hipEvent_t> events;   // pool, created on enable
    std::vector<int> phase;           // phase that starts at event i
    size_t used = 0;
};
thread_local Profiler g_prof;
constexpr size_t kMaxEvents = 16384;
}  // namespace

void mark_phase(int phase, hipStream_t stream) {
    Profiler& p = g_prof;
    if (!p.on) return;
    if (p.used >= p.events.size()) {
        p.overflow = true;
        return;
    }
    if (hipEventRecord(p.events[p.used], stream) != hipSuccess) return;
    p.phase[p.used] = phase;
    ++p.used;
}

void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof(g_error), fmt, ap);
    va_end(ap);
}

}  // namespace nd

using namespace nd;

extern "C" {

const char* nd_last_error(void) { return g_error; }

int nd_profile_enable(int on) {
    Profiler& p = g_prof;
    if (on && p.events.empty()) {
        p.events.resize(kMaxEvents);
        p.phase.assign(kMaxEvents, ND_PHASE_NONE);
        for (size_t i = 0; i < kMaxEvents; ++i) ND_HIP_CHECK(hipEventCreate(&p.events[i]));
    }
    if (!on && !p.events.empty()) {
        for (hipEvent_t e : p.events) (void)hipEventDestroy(e);
        p.events.clear();
        p.phase.clear();
    }
    p.on = on != 0;
    p.used = 0;
    p.overflow = false;
    return ND_OK;
}

int nd_profile_read(double* ms, int64_t* intervals) {
    Profiler& p = g_prof;
    if (!ms || !intervals) {
        set_error("ms or intervals is NULL");
        return ND_ERR_NULL_POINTER;
    }
    if (!p.on) {
        set_error("profiling is not enabled on this thread");
        return ND_ERR_BAD_ARGUMENT;
    }
    if (p.used > 0) ND_HIP_CHECK(hipEventSynchronize(p.events[p.used - 1]));
    for (size_t i = 0; i + 1 < p.used; ++i) {
        const int ph = p.phase[i];
        if (ph < 0 || ph >= ND_PHASE_COUNT) continue;
        float t = 0.f;
        ND_HIP_CHECK(hipEventElapsedTime(&t, p.events[i], p.events[i + 1]));
        ms[ph] += (double)t;
        intervals[ph] += 1;
    }
    const bool overflow = p.overflow;
    p.used = 0;
    p.overflow = false;
    if (overflow) {
        set_error("more than %zu phase marks between two reads; the rest were dropped", kMaxEvents);
        return ND_ERR_BAD_ARGUMENT;
    }
    return ND_OK;
}
int nd_version(void) { return ND_VERSION; }

void nd_params_init(nd_params* p) {
    if (!p) return;
    memset(p, 0, sizeof(*p));
    p->struct_size = (uint32_t)sizeof(nd_params);
    p->num_steps = 1;
    p->p = 1.0;
    p->q = 1.0;
    p->n2v_max_attempts = 64;
    p->roots_per_sample = 1;
    p->mode = ND_MODE_TRANSIT_PARALLEL;
    p->sched_force_class = ND_CLASS_AUTO;
}

int nd_graph_create(nd_graph** out, int64_t V, int64_t E, const void* row_offsets,
                    int offsets_are_int64, const int32_t* col_indices, const float* weights_or_null,
                    int src_is_device, void* hip_stream) {
    if (!out) {
        set_error("out is NULL");
        return ND_ERR_NULL_POINTER;
    }
    *out = nullptr;
    if (!row_offsets || (!col_indices && E > 0)) {
        set_error("row_offsets or col_indices is NULL");
        return ND_ERR_NULL_POINTER;
    }
    if (V < 1 || V >= (1ll << 31) || E < 0) {
        set_error("V must be in [1, 2^31) and E >= 0 (V=%lld, E=%lld)", (long long)V, (long long)E);
        return ND_ERR_TOO_LARGE;
    }
    if (!offsets_are_int64 && E >= (1ll << 31)) {
        set_error("E >= 2^31 needs int64 offsets");
        return ND_ERR_TOO_LARGE;
    }
    Graph* g = nullptr;
    const int rc = graph_create(&g, V, E, row_offsets, offsets_are_int64 ? 1 : 0, col_indices,
                                weights_or_null, src_is_device, (hipStream_t)hip_stream);
    if (rc != ND_OK) return rc;
    if (layer_prepare() != ND_OK || edges_prepare() != ND_OK) {
        graph_destroy(g);
        return ND_ERR_HIP;
    }
    nd_graph* h = new nd_graph{g};
    *out = h;
    return ND_OK;
}

int nd_graph_destroy(nd_graph* h) {
    if (!h) return ND_OK;
    graph_destroy(h->g);
    delete h;
    return ND_OK;
}

int nd_graph_info(const nd_graph* h, int64_t* V, int64_t* E, int* has_weights, int* offsets_are_int64) {
    if (!h) {
        set_error("graph is NULL");
        return ND_ERR_NULL_POINTER;
    }
    if (V) *V = h->g->V;
    if (E) *E = h->g->E;
    if (has_weights) *has_weights = h->g->wq != nullptr;
    if (offsets_are_int64) *offsets_are_int64 = h->g->off64;
    return ND_OK;
}

int nd_sample_query(const nd_graph* h, int app, const nd_params* params, int64_t num_roots,
                    int32_t* num_steps, int64_t* step_len, size_t* workspace_bytes) {
    if (!h || !params) {
        set_error("graph or params is NULL");
        return ND_ERR_NULL_POINTER;
    }
    Plan pl;
    const int rc = check_params(*h->g, app, params, num_roots, &pl);
    if (rc != ND_OK) return rc;
    layout(&pl, h->g->V);
    if (num_steps) *num_steps = pl.k;
    if (step_len) {
        for (int i = 0; i < pl.k; ++i) {
            int64_t ns, no;
            step_shape(pl, params, i, &ns, &no);
            step_len[i] = no;
        }
    }
    if (workspace_bytes) *workspace_bytes = pl.total;
    return ND_OK;
}

// The body of nd_sample and nd_sample_static.  fixed_scratch: the workspace is the library's
// own array of a fixed size, so a call that needs more is told the limit, not a size to bring.
static int sample_impl(const nd_graph* h, int app, const nd_params* params, const int32_t* roots_dev,
                       int64_t num_roots, uint64_t seed, int32_t* const* step_out_dev,
                       void* workspace_dev, size_t workspace_bytes, bool fixed_scratch,
                       hipStream_t stream) {
    const Graph& g = *h->g;
    Plan pl;
    int rc = check_params(g, app, params, num_roots, &pl);
    if (rc != ND_OK) return rc;
    layout(&pl, g.V);
    if (fixed_scratch && workspace_bytes < pl.total) {
        set_error("this call needs %zu bytes of scratch; nd_sample_static has %zu (ND_STATIC_SCRATCH_BYTES): "
                  "use fewer roots per call or nd_sample with a workspace", pl.total, workspace_bytes);
        return ND_ERR_TOO_LARGE;
    }
    if (workspace_bytes < pl.total || ((uintptr_t)workspace_dev % kAlign) != 0) {
        set_error("workspace needs %zu bytes aligned to %zu (got %zu)", pl.total, kAlign,
                  workspace_bytes);
        return ND_ERR_WORKSPACE;
    }
    for (int i = 0; i < pl.k; ++i) {
        int64_t ns, no;
        step_shape(pl, params, i, &ns, &no);
        if (!step_out_dev[i] && no > 0) {
            set_error("step_out_dev[%d] is NULL", i);
            return ND_ERR_NULL_POINTER;
        }
    }
    char* ws = (char*)workspace_dev;
    WsHeader* hdr = (WsHeader*)ws;
    StepCtl* ctl = (StepCtl*)(ws + pl.o_ctl);
    mark_phase(ND_PHASE_INIT, stream);
    {
        const int64_t n_init = pl.bit_words > pl.k ? pl.bit_words : pl.k;
        hipLaunchKernelGGL(init_header_kernel, dim3((unsigned)((n_init + 255) / 256)), dim3(256), 0,
                           stream, hdr, (uint32_t)pl.k, ctl, (uint32_t*)(ws + pl.o_bits), pl.bit_words);
    }
    ND_HIP_CHECK(hipGetLastError());
    if (pl.S == 0) {
        mark_phase(ND_PHASE_NONE, stream);
        return ND_OK;
    }

    if (app == ND_LAYER) {
        for (int i = 0; i < pl.k; ++i) {
            LayerArgs a{};
            a.seed = seed;
            a.sample_base = (uint32_t)params->sample_id_base;
            a.step = (uint32_t)i;
            a.n_prev = (uint32_t)(i == 0 ? params->roots_per_sample : params->fanout[i - 1]);
            a.m = (uint32_t)params->fanout[i];
            a.transits = i == 0 ? roots_dev : step_out_dev[i - 1];
            a.out = step_out_dev[i];
            a.check_roots = i == 0;
            a.use_weights = params->use_weights;
            a.status = &hdr->status;
            mark_phase(ND_PHASE_LAYER, stream);
            rc = layer_step(g, a, pl.S, stream);
            if (rc != ND_OK) return rc;
        }
        mark_phase(ND_PHASE_NONE, stream);
        return ND_OK;
    }

    // individual transit sampling: walks and k-hop
    int draw = kDrawUniform;
    if (app == ND_NODE2VEC) draw = kDrawNode2vec;
    else if (params->use_weights) draw = kDrawWeighted;
    DrawArgs a{};
    a.seed = seed;
    a.sample_base = (uint32_t)params->sample_id_base;
    a.ppr_thr = app == ND_PPR ? (uint64_t)std::floor(params->term_prob * 4294967296.0) : 0;
    a.use_weights = params->use_weights ? 1 : 0;
    a.lds_policy = params->lds_stage_policy;
    a.max_attempts = params->n2v_max_attempts;
    if (app == ND_NODE2VEC) {
        if (params->bias_convention == 0) {
            a.b_ret = q16(1.0 / params->p);
            a.b_com = q16(1.0);
            a.b_far = q16(1.0 / params->q);
        } else {
            a.b_ret = q16(params->p);
            a.b_com = q16(1.0 / params->q);
            a.b_far = q16(1.0);
        }
        if (!a.b_ret || !a.b_com || !a.b_far) {
            set_error("node2vec biases must lie in [2^-16, 2^8] after rounding to Q16");
            return ND_ERR_BAD_ARGUMENT;
        }
        a.b_max = a.b_ret > a.b_com ? a.b_ret : a.b_com;
        a.b_max = a.b_far > a.b_max ? a.b_far : a.b_max;
    }

    const bool multirw = app == ND_MULTIRW;
    int32_t* mrw_state = (int32_t*)(ws + pl.o_state);
    int32_t* mrw_transits = (int32_t*)(ws + pl.o_transits);
    const uint32_t mrw_R = (uint32_t)params->roots_per_sample;
    if (pl.window > 0) {  // walks grouped per window of samples, inside LDS
        rc = walk_windows(g, draw, multirw, a, pl.S, pl.k, pl.window, pl.heavy_min, params->sched_force_class,
                          roots_dev, 1, step_out_dev, &hdr->status, ctl, multirw ? mrw_state : nullptr,
                          multirw ? mrw_R : 1u, stream);
        if (rc != ND_OK) return rc;
        mark_phase(ND_PHASE_NONE, stream);
        return ND_OK;
    }
    if (multirw) {
        rc = multirw_init(g, roots_dev, pl.state_len, mrw_state, &hdr->status, stream);
        if (rc != ND_OK) return rc;
    }

    for (int i = 0; i < pl.k; ++i) {
        int64_t n_slots, n_out;
        step_shape(pl, params, i, &n_slots, &n_out);
        const int32_t m = (int32_t)step_fanout(app, params, i);
        const int32_t* src = i == 0 ? roots_dev : step_out_dev[i - 1];
        if (multirw) {  // the step's transits are the picked roots, not the previous output
            n_slots = pl.S;
            rc = multirw_select(mrw_state, pl.S, mrw_R, seed, a.sample_base, (uint32_t)i, mrw_transits,
                                stream);
            if (rc != ND_OK) return rc;
            src = mrw_transits;
        }
        a.step = (uint32_t)i;
        a.m = (uint32_t)m;
        a.div_m = make_fastdiv((uint32_t)m);
        a.div_wprev = make_fastdiv((uint32_t)(n_slots / pl.S));
        a.has_prev = i > 0;
        a.prev_transit = i == 0 ? nullptr : (i == 1 ? roots_dev : step_out_dev[i - 2]);
        a.out = step_out_dev[i];
        if (pl.mode == ND_MODE_SAMPLE_PARALLEL) {
            mark_phase(ND_PHASE_SAMPLE_SP, stream);
            rc = sample_step_sp(g, draw, a, src, n_slots, i == 0 && !multirw, &hdr->status, stream);
            if (rc != ND_OK) return rc;
            if (params->unique_rounds > 0) {
                rc = run_unique(g, params, seed, i, pl.S, n_slots, n_out, m, src, step_out_dev[i], stream);
                if (rc != ND_OK) return rc;
            }
            if (multirw) {
                rc = multirw_update(mrw_state, pl.S, mrw_R, seed, a.sample_base, (uint32_t)i,
                                    step_out_dev[i], stream);
                if (rc != ND_OK) return rc;
            }
            continue;
        }
        SchedParams sp{m, pl.sub_max, pl.wg_max, params->sched_force_class};
        const bool coarse = params->sched_group_bits > 0;  // grouped by id prefix: no groups, one class
        if (coarse) sp.force_class = ND_CLASS_SUBWAVE;
        const SortPlan plan = make_sort_plan(n_slots, g.V, params->sched_group_bits);
        int32_t *keys = nullptr, *vals = nullptr;
        mark_phase(ND_PHASE_SORT, stream);
        rc = sort_pairs(src, n_slots, (int32_t)g.V, plan, (int32_t*)(ws + pl.o_keysA),
                        (int32_t*)(ws + pl.o_valsA), (int32_t*)(ws + pl.o_keysB),
                        (int32_t*)(ws + pl.o_valsB), (uint32_t*)(ws + pl.o_hist), ctl + i,
                        step_out_dev[i], m, (i == 0 && !multirw) ? &hdr->status : nullptr, &keys, &vals,
                        stream);
        if (rc != ND_OK) return rc;
        int32_t* g_key = (int32_t*)(ws + pl.o_gkey);
        int32_t* g_start = (int32_t*)(ws + pl.o_gstart);
        int32_t* list_wg = (int32_t*)(ws + pl.o_list_wg);
        int32_t* chunk_gid = (int32_t*)(ws + pl.o_chunk_gid);
        int32_t* chunk_idx = (int32_t*)(ws + pl.o_chunk_idx);
        uint32_t* heavy_bits = sp.force_class == ND_CLASS_AUTO ? (uint32_t*)(ws + pl.o_bits) : nullptr;
        if (!coarse) {
            mark_phase(ND_PHASE_GROUP, stream);
            rc = build_groups(keys, n_slots, ctl + i, g_key, g_start, (uint32_t*)(ws + pl.o_tiles), heavy_bits,
                              pl.bit_words, stream);
            if (rc != ND_OK) return rc;
            rc = classify_groups(g_key, g_start, n_slots, ctl + i, sp, list_wg, chunk_gid, chunk_idx,
                                 pl.cap_chunks, heavy_bits, stream);
            if (rc != ND_OK) return rc;
        }
        // work-list bounds for this step's launch shapes
        int64_t max_wg = n_out / pl.sub_max + 1;
        int64_t max_chunks = 2 * (n_out / pl.wg_max) + 1;
        if (sp.force_class != ND_CLASS_AUTO) {
            max_wg = n_slots;
            max_chunks += n_slots;
        }
        if (max_wg > n_slots) max_wg = n_slots;
        TpStep t{};
        t.ctl = ctl + i;
        t.keys = keys;
        t.vals = vals;
        t.g_key = g_key;
        t.g_start = g_start;
        t.list_wg = list_wg;
        t.chunk_gid = chunk_gid;
        t.chunk_idx = chunk_idx;
        t.heavy_bits = heavy_bits;
        t.max_draws = n_out;
        t.max_wg = max_wg;
        t.max_chunks = max_chunks;
        t.cap_wg = pl.cap_wg;
        t.cap_chunks = pl.cap_chunks;
        rc = sample_step_tp(g, draw, a, sp, t, stream);
        if (rc != ND_OK) return rc;
        if (params->unique_rounds > 0) {
            rc = run_unique(g, params, seed, i, pl.S, n_slots, n_out, m, src, step_out_dev[i], stream);
            if (rc != ND_OK) return rc;
        }
        if (multirw) {
            rc = multirw_update(mrw_state, pl.S, mrw_R, seed, a.sample_base, (uint32_t)i,
                                step_out_dev[i], stream);
            if (rc != ND_OK) return rc;
        }
    }
    mark_phase(ND_PHASE_NONE, stream);
    return ND_OK;
}

int nd_sample(const nd_graph* h, int app, const nd_params* params, const int32_t* roots_dev,
              int64_t num_roots, uint64_t seed, int32_t* const* step_out_dev, void* workspace_dev,
              size_t workspace_bytes, void* hip_stream) {
    if (!h || !params || !step_out_dev || !workspace_dev || (!roots_dev && num_roots > 0)) {
        set_error("a required pointer is NULL");
        return ND_ERR_NULL_POINTER;
    }
    return sample_impl(h, app, params, roots_dev, num_roots, seed, step_out_dev, workspace_dev,
                       workspace_bytes, false, (hipStream_t)hip_stream);
}

// ---------------------------------------------------------------- scratch owned by the library
// nd_sample_static's workspace: one array per GPU, part of the loaded code object.  In host
// code the array's name is only a handle for hipGetSymbolAddress; its device address is looked
// up once per device and that pointer is what kernels receive.
static __device__ __align__(256) unsigned char nd_static_scratch[ND_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

__global__ void publish_status_kernel(const WsHeader* hdr, uint32_t* status_out) {
    *status_out = hdr->status;
}

// Device address of the current device's copy of the array (looked up on first use).
int static_scratch(void** out) {
    int dev = -1;
    ND_HIP_CHECK(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) {
        set_error("device %d is outside the %d devices nd_sample_static keeps scratch for", dev,
                  kMaxDevices);
        return ND_ERR_BAD_ARGUMENT;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        ND_HIP_CHECK(hipGetSymbolAddress(&p, HIP_SYMBOL(nd_static_scratch)));
        if (!p || ((uintptr_t)p % kAlign) != 0) {
            set_error("the library's scratch array has no usable device address");
            return ND_ERR_HIP;
        }
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return ND_OK;
}
}  // namespace

int nd_sample_static(const nd_graph* h, int app, const nd_params* params, const int32_t* roots_dev,
                     int64_t num_roots, uint64_t seed, int32_t* const* step_out_dev,
                     uint32_t* status_dev, void* hip_stream) {
    if (!h || !params || !step_out_dev || (!roots_dev && num_roots > 0)) {
        set_error("a required pointer is NULL");
        return ND_ERR_NULL_POINTER;
    }
    int dev = -1;
    ND_HIP_CHECK(hipGetDevice(&dev));
    if (dev != h->g->device) {
        set_error("the graph lives on device %d but device %d is current", h->g->device, dev);
        return ND_ERR_BAD_ARGUMENT;
    }
    void* scratch = nullptr;
    int rc = static_scratch(&scratch);
    if (rc != ND_OK) return rc;
    hipStream_t stream = (hipStream_t)hip_stream;
    rc = sample_impl(h, app, params, roots_dev, num_roots, seed, step_out_dev, scratch,
                     (size_t)ND_STATIC_SCRATCH_BYTES, true, stream);
    if (rc != ND_OK) return rc;
    if (status_dev) {
        hipLaunchKernelGGL(publish_status_kernel, dim3(1), dim3(1), 0, stream, (const WsHeader*)scratch,
                           status_dev);
        ND_HIP_CHECK(hipGetLastError());
    }
    return ND_OK;
}

int nd_sample_status(const void* workspace_dev, void* hip_stream) {
    if (!workspace_dev) {
        set_error("workspace is NULL");
        return ND_ERR_NULL_POINTER;
    }
    uint32_t status = 0;
    ND_HIP_CHECK(hipMemcpyAsync(&status, workspace_dev, sizeof(status), hipMemcpyDeviceToHost,
                                (hipStream_t)hip_stream));
    ND_HIP_CHECK(hipStreamSynchronize((hipStream_t)hip_stream));
    if (status & 1u) {
        set_error("a root was outside [0, V); it was treated as NULL");
        return ND_ERR_BAD_ROOT;
    }
    return ND_OK;
}

int nd_sample_stats(const void* workspace_dev, void* hip_stream, int32_t max_steps, int64_t* stats) {
    if (!workspace_dev || !stats) {
        set_error("workspace or stats is NULL");
        return ND_ERR_NULL_POINTER;
    }
    if (max_steps < 0) {
        set_error("max_steps is negative");
        return ND_ERR_BAD_ARGUMENT;
    }
    hipStream_t stream = (hipStream_t)hip_stream;
    WsHeader hdr;
    ND_HIP_CHECK(hipMemcpyAsync(&hdr, workspace_dev, sizeof(hdr), hipMemcpyDeviceToHost, stream));
    ND_HIP_CHECK(hipStreamSynchronize(stream));
    int n = (int)hdr.num_steps < max_steps ? (int)hdr.num_steps : max_steps;
    if (n > ND_MAX_WALK_STEPS) n = ND_MAX_WALK_STEPS;
    static thread_local StepCtl host_ctl[ND_MAX_WALK_STEPS];
    if (n > 0) {
        ND_HIP_CHECK(hipMemcpyAsync(host_ctl, (const char*)workspace_dev + sizeof(WsHeader),
                                    sizeof(StepCtl) * (size_t)n, hipMemcpyDeviceToHost, stream));
        ND_HIP_CHECK(hipStreamSynchronize(stream));
    }
    for (int i = 0; i < max_steps; ++i) {
        int64_t* s = stats + (size_t)i * 8;
        for (int j = 0; j < 8; ++j) s[j] = 0;
        if (i < n) {
            s[0] = host_ctl[i].P;
            s[1] = host_ctl[i].U;
            s[2] = (int64_t)host_ctl[i].U - host_ctl[i].n_wg - host_ctl[i].n_grid;
            s[3] = host_ctl[i].n_wg;
            s[4] = host_ctl[i].n_grid;
            s[5] = host_ctl[i].n_chunks;
            s[6] = host_ctl[i].n_staged;
            s[7] = host_ctl[i].heavy_draws;
        }
    }
    return ND_OK;
}

size_t nd_group_workspace_bytes(int64_t n, int64_t V) {
    if (n < 0 || V < 1) return 0;
    const size_t cnt = (size_t)(n > 0 ? n : 1);
    const SortPlan sp = make_sort_plan(n, V);
    return align_up(sizeof(StepCtl)) + 4 * align_up(cnt * 4) + align_up(sort_hist_bytes(sp)) +
           align_up(seg_scratch_bytes(n));
}

int nd_group_by_transit(const int32_t* transits_dev, int64_t n, int64_t V,
                        int32_t* sorted_transits_dev, int32_t* sorted_slots_dev,
                        int32_t* group_transit_dev, int32_t* group_start_dev, int64_t* counts_dev,
                        void* workspace_dev, size_t workspace_bytes, void* hip_stream) {
    if ((n > 0 && (!transits_dev || !sorted_transits_dev || !sorted_slots_dev || !group_transit_dev)) ||
        !group_start_dev || !counts_dev || !workspace_dev) {
        set_error("a required pointer is NULL");
        return ND_ERR_NULL_POINTER;
    }
    if (n < 0 || n >= (1ll << 31) || V < 1 || V >= (1ll << 31)) {
        set_error("n and V must be below 2^31");
        return ND_ERR_TOO_LARGE;
    }
    if (workspace_bytes < nd_group_workspace_bytes(n, V) || ((uintptr_t)workspace_dev % kAlign) != 0) {
        set_error("workspace needs %zu bytes aligned to %zu", nd_group_workspace_bytes(n, V), kAlign);
        return ND_ERR_WORKSPACE;
    }
    hipStream_t stream = (hipStream_t)hip_stream;
    const size_t cnt = (size_t)(n > 0 ? n : 1);
    const SortPlan sp = make_sort_plan(n, V);
    char* ws = (char*)workspace_dev;
    StepCtl* ctl = (StepCtl*)ws;
    size_t o = align_up(sizeof(StepCtl));
    int32_t* keysA = (int32_t*)(ws + o); o += align_up(cnt * 4);
    int32_t* valsA = (int32_t*)(ws + o); o += align_up(cnt * 4);
    int32_t* keysB = (int32_t*)(ws + o); o += align_up(cnt * 4);
    int32_t* valsB = (int32_t*)(ws + o); o += align_up(cnt * 4);
    uint32_t* hist = (uint32_t*)(ws + o); o += align_up(sort_hist_bytes(sp));
    uint32_t* tiles = (uint32_t*)(ws + o);
    int32_t *keys = nullptr, *vals = nullptr;
    int rc = sort_pairs(transits_dev, n, (int32_t)V, sp, keysA, valsA, keysB, valsB, hist, ctl, nullptr,
                        1, nullptr, &keys, &vals, stream);
    if (rc != ND_OK) return rc;
    rc = build_groups(keys, n, ctl, group_transit_dev, group_start_dev, tiles, nullptr, 0, stream);
    if (rc != ND_OK) return rc;
    if (n > 0) {
        ND_HIP_CHECK(hipMemcpyAsync(sorted_transits_dev, keys, (size_t)n * 4, hipMemcpyDeviceToDevice, stream));
        ND_HIP_CHECK(hipMemcpyAsync(sorted_slots_dev, vals, (size_t)n * 4, hipMemcpyDeviceToDevice, stream));
    }
    hipLaunchKernelGGL(publish_counts_kernel, dim3(1), dim3(1), 0, stream, ctl, counts_dev);
    ND_HIP_CHECK(hipGetLastError());
    return ND_OK;
}

static int check_edge_args(const nd_graph* g, const int32_t* transits_dev, int32_t n_prev,
                           const int32_t* sampled_dev, int32_t m, int64_t num_samples) {
    if (!g || !g->g || (num_samples > 0 && (!transits_dev || !sampled_dev))) {
        set_error("a required pointer is NULL");
        return ND_ERR_NULL_POINTER;
    }
    if (n_prev < 1 || m < 1 || num_samples < 0) {
        set_error("n_prev and m must be at least 1 and num_samples not negative");
        return ND_ERR_BAD_ARGUMENT;
    }
    if (m > ND_MAX_EDGE_SLOTS || num_samples * (int64_t)n_prev >= (1ll << 31) ||
        num_samples * (int64_t)m >= (1ll << 31)) {
        set_error("at most %d new vertices per sample, and fewer than 2^31 transit slots and new slots per call",
                  ND_MAX_EDGE_SLOTS);
        return ND_ERR_TOO_LARGE;
    }
    return ND_OK;
}

size_t nd_layer_edges_workspace_bytes(int64_t num_samples, int32_t n_prev) {
    if (num_samples < 0 || n_prev < 1) return 0;
    return edges_workspace_bytes(num_samples, n_prev);
}

int nd_layer_edges_count(const nd_graph* g, const int32_t* transits_dev, int32_t n_prev,
                         const int32_t* sampled_dev, int32_t m, int64_t num_samples,
                         int64_t* row_ptr_dev, void* workspace_dev, size_t workspace_bytes,
                         void* hip_stream) {
    int rc = check_edge_args(g, transits_dev, n_prev, sampled_dev, m, num_samples);
    if (rc != ND_OK) return rc;
    if (!row_ptr_dev || !workspace_dev) {
        set_error("a required pointer is NULL");
        return ND_ERR_NULL_POINTER;
    }
    if (workspace_bytes < edges_workspace_bytes(num_samples, n_prev) ||
        ((uintptr_t)workspace_dev % kAlign) != 0) {
        set_error("workspace needs %zu bytes aligned to %zu", edges_workspace_bytes(num_samples, n_prev), kAlign);
        return ND_ERR_WORKSPACE;
    }
    return edges_count(*g->g, transits_dev, n_prev, sampled_dev, m, num_samples, row_ptr_dev,
                       workspace_dev, (hipStream_t)hip_stream);
}

int nd_layer_edges_fill(const nd_graph* g, const int32_t* transits_dev, int32_t n_prev,
                        const int32_t* sampled_dev, int32_t m, int64_t num_samples,
                        const int64_t* row_ptr_dev, int32_t* edge_slot_dev, int64_t capacity,
                        void* hip_stream) {
    int rc = check_edge_args(g, transits_dev, n_prev, sampled_dev, m, num_samples);
    if (rc != ND_OK) return rc;
    if (!row_ptr_dev || (capacity > 0 && !edge_slot_dev)) {
        set_error("a required pointer is NULL");
        return ND_ERR_NULL_POINTER;
    }
    if (capacity < 0) {
        set_error("capacity is negative");
        return ND_ERR_BAD_ARGUMENT;
    }
    return edges_fill(*g->g, transits_dev, n_prev, sampled_dev, m, num_samples, row_ptr_dev,
                      edge_slot_dev, capacity, (hipStream_t)hip_stream);
}

int nd_layer_edges_status(const void* workspace_dev, void* hip_stream) {
    if (!workspace_dev) {
        set_error("a required pointer is NULL");
        return ND_ERR_NULL_POINTER;
    }
    uint32_t word = 0;
    ND_HIP_CHECK(hipMemcpyAsync(&word, workspace_dev, 4, hipMemcpyDeviceToHost, (hipStream_t)hip_stream));
    ND_HIP_CHECK(hipStreamSynchronize((hipStream_t)hip_stream));
    if (word) {
        set_error("a transit or a new vertex was outside [-1, V)");
        return ND_ERR_BAD_ROOT;
    }
    return ND_OK;
}

int nd_probe_store_runs(int32_t* out_dev, int64_t n_runs, int32_t run_len, int scattered, void* hip_stream) {
    if (!out_dev) {
        set_error("out_dev is NULL");
        return ND_ERR_NULL_POINTER;
    }
    if (n_runs < 1 || n_runs >= (1ll << 31) || (n_runs & (n_runs - 1)) != 0 || run_len < 1 || run_len > 32) {
        set_error("n_runs must be a power of two below 2^31 and run_len in [1, 32]");
        return ND_ERR_BAD_ARGUMENT;
    }
    return probe_store_runs(out_dev, n_runs, run_len, scattered, (hipStream_t)hip_stream);
}

int nd_samples_pack(const int32_t* const* step_out_dev, int32_t num_steps, const int64_t* step_len,
                    int64_t num_samples, int32_t* samples_dev, void* hip_stream) {
    if (num_steps < 1 || num_steps > ND_MAX_WALK_STEPS || num_samples < 0) {
        set_error("num_steps must be in [1, %d] and num_samples not negative", ND_MAX_WALK_STEPS);
        return ND_ERR_BAD_ARGUMENT;
    }
    if (!step_out_dev || !step_len || (num_samples > 0 && !samples_dev)) {
        set_error("a required pointer is NULL");
        return ND_ERR_NULL_POINTER;
    }
    int64_t record = 0;
    for (int32_t i = 0; i < num_steps; ++i) {
        if (step_len[i] < 0 || step_len[i] >= (1ll << 31)) {
            set_error("step %d has %lld entries; at most 2^31 - 1", i, (long long)step_len[i]);
            return ND_ERR_TOO_LARGE;
        }
        if (num_samples > 0) {
            if (step_len[i] == 0 || step_len[i] % num_samples != 0) {
                set_error("step %d: %lld entries is not a positive multiple of the %lld samples", i,
                          (long long)step_len[i], (long long)num_samples);
                return ND_ERR_BAD_ARGUMENT;
            }
            if (!step_out_dev[i]) {
                set_error("a required pointer is NULL");
                return ND_ERR_NULL_POINTER;
            }
            record += step_len[i] / num_samples;
        }
    }
    if (record >= (1ll << 31)) {
        set_error("a record of %lld entries is too long", (long long)record);
        return ND_ERR_TOO_LARGE;
    }
    return pack_samples(step_out_dev, num_steps, step_len, num_samples, samples_dev, (hipStream_t)hip_stream);
}

}  // extern "C"
