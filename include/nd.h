/*
 * nd.h - C ABI of the transit-parallel graph sampling library for one AMD
 * MI355X (gfx950).
 *
 * The calls follow the problem statement of the NextDoor paper (Section 3 and
 * Section 4.1): the inputs are a graph, an initial set of samples (roots), and
 * a sampling application with its parameters; the output is the expanded
 * samples, one int32 array per step, resident in device memory (Section 4.1,
 * "Output format", the per-step form).  Every step is executed transit-
 * parallel (Section 5.2 and Section 6): the (transit, sample-slot) pairs of the
 * step are grouped by transit vertex with a radix sort and a segmented scan,
 * the transits are split into three scheduling classes by the number of
 * neighbours they must produce (Section 6.1.2, Table "Types of kernels"), and
 * one launch per step draws the neighbours of all three classes.  Random walks
 * by default group per window of samples inside a workgroup's LDS instead
 * (nd_params.sched_window).
 *
 * Conventions
 *   - All functions return 0 on success or a negative nd_status code; the
 *     message of the last failure on the calling thread is nd_last_error().
 *     No exception crosses this boundary and no argument is a C++ or torch
 *     type.
 *   - "host" / "device" after a pointer says where the memory must live.
 *   - The NULL vertex is -1 (ND_NULL_VERTEX).  A sample slot whose transit is
 *     NULL, or has no out-edges, receives NULL at this and all later steps
 *     (Section 4.1: `next` may return NULL; a walk without transits has ended).
 *   - Random numbers: Philox4x32-10 with key = (seed low word, seed high word)
 *     and counter = (sample_id_base + sample index, slot within the sample,
 *     step, attempt).  The output therefore depends only on (graph, app,
 *     params, roots, seed) and never on how samples are grouped, scheduled or
 *     split over calls.
 */
#ifndef ND_H_
#define ND_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ND_VERSION 100
#define ND_NULL_VERTEX (-1)
#define ND_MAX_FANOUT_STEPS 8 /* k-hop / layer steps */
#define ND_MAX_WALK_STEPS 4096
#define ND_MAX_LAYER_TRANSITS 4096 /* roots_per_sample and layer fanouts */
#define ND_MAX_UNIQUE_SLOTS 2048    /* slots per sample and step with unique_rounds > 0 */

typedef enum nd_status {
    ND_OK = 0,
    ND_ERR_NULL_POINTER = -1,
    ND_ERR_BAD_ARGUMENT = -2,  /* sizes, enum values, parameter ranges */
    ND_ERR_BAD_GRAPH = -3,     /* CSR fails validation (see nd_graph_create) */
    ND_ERR_BAD_WEIGHT = -4,    /* weight not finite, <= 0 or >= 2^15, or a row total >= 2^39 */
    ND_ERR_NO_WEIGHTS = -5,    /* use_weights on a graph created without weights */
    ND_ERR_WORKSPACE = -6,     /* workspace too small or misaligned */
    ND_ERR_HIP = -7,           /* a HIP runtime call failed */
    ND_ERR_BAD_ROOT = -8,      /* reported by nd_sample_status: a root outside [0, V) */
    ND_ERR_TOO_LARGE = -9      /* V >= 2^31, too many samples or slots for 32-bit ids */
} nd_status;

/* Sampling applications (Section 3 and Section 4.2 of the paper). */
typedef enum nd_app {
    ND_DEEPWALK = 0, /* fixed-length static walk, uniform or weight-proportional      */
    ND_PPR = 1,      /* static walk that ends with probability term_prob per step     */
    ND_NODE2VEC = 2, /* second-order walk, rejection sampling with bias p, q          */
    ND_KHOP = 3,     /* GraphSAGE k-hop: fanout[i] uniform neighbours per transit     */
    ND_LAYER = 4,    /* collective: fanout[i] draws from the transits' combined       */
                     /* neighbourhood, LADIES-style weights                           */
    ND_MULTIRW = 5   /* multi-dimensional walk: a sample owns roots_per_sample roots;  */
                     /* each step picks one uniformly, adds a uniform neighbour of it  */
                     /* and puts that neighbour in the picked root's place             */
} nd_app;

/* Execution strategy.  Both give identical outputs. */
typedef enum nd_mode {
    ND_MODE_TRANSIT_PARALLEL = 0, /* the paper's method (Section 5.2, Section 6)     */
    ND_MODE_SAMPLE_PARALLEL = 1   /* one lane per (sample, slot), no grouping          */
                                  /* (Section 5.1), kept as the ablation baseline     */
} nd_mode;

/* Scheduling classes (Section 6.1.2), re-derived for 64-lane wavefronts. */
typedef enum nd_sched_class {
    ND_CLASS_AUTO = -1,
    ND_CLASS_SUBWAVE = 0,   /* several transits share one wavefront                   */
    ND_CLASS_WORKGROUP = 1, /* one workgroup per transit, adjacency list in LDS       */
    ND_CLASS_GRID = 2       /* one transit spread over many workgroups                */
} nd_sched_class;

typedef struct nd_params {
    uint32_t struct_size;      /* sizeof(nd_params), set by nd_params_init             */
    int32_t num_steps;         /* walks: walk length (PPR: the cap that replaces the   */
                               /* paper's unbounded step count); k-hop, layer: number  */
                               /* of entries used in fanout[]                          */
    int32_t fanout[ND_MAX_FANOUT_STEPS]; /* k-hop: neighbours per transit; layer:     */
                               /* vertices per sample, at each step                    */
    int32_t use_weights;       /* walks: draw proportionally to the edge weight; layer: */
                               /* an entry of the combined neighbourhood weighs its edge */
                               /* weight instead of 1 / deg(transit)^2 (with weights     */
                               /* 1 / (deg(v) deg(u)): symmetric normalisation)          */
    int32_t bias_convention;   /* node2vec: 0 = return 1/p, common neighbour 1,        */
                               /* farther 1/q (the node2vec definition); 1 = p, 1/q, 1 */
                               /* (the wording of Section 4.2)                         */
    double p, q;               /* node2vec hyper-parameters                            */
    double term_prob;          /* PPR: probability of ending the walk at each step     */
    int32_t roots_per_sample;  /* layer: roots that form one sample (batch); multi-    */
                               /* dimensional walk: roots a sample owns (at most 4,096) */
    int32_t n2v_max_attempts;  /* node2vec: rejection attempts before the exact        */
                               /* fallback draw; part of the output's definition       */
    uint64_t sample_id_base;   /* id of this call's first sample in the random-number  */
                               /* counter: a call on roots[a:b] with base a reproduces */
                               /* that slice of the call on all roots                  */
    int32_t mode;              /* nd_mode                                              */
    int32_t sched_force_class; /* nd_sched_class; anything but AUTO is for tests       */
    int32_t sched_sub_max;     /* largest draw count (pairs x fanout) of a transit     */
                               /* handled lane-per-draw (0: the default, 16,384)       */
    int32_t sched_wg_max;      /* largest draw count handled by one workgroup; also    */
                               /* the chunk a grid-class transit is cut into           */
                               /* (0: the default, 65,536); not below sched_sub_max    */
    int32_t lds_stage_policy;  /* 0: stage the adjacency list in LDS when it fits and  */
                               /* pays; 1: never stage; 2: stage whenever it fits      */
    int32_t unique_rounds;     /* k-hop: 0 = neighbours are drawn with replacement; r > 0 = */
                               /* unique neighbours (Section 6.3): within a sample and step */
                               /* no vertex appears twice; a slot that drew a vertex already */
                               /* held by a lower slot draws again (attempt 1 .. r-1) and is */
                               /* NULL if it never finds a free one.  Needs at most 2,048    */
                               /* slots per sample and step.                                 */
    int32_t sched_group_bits;  /* 0: group by the exact transit (the paper's scheduling   */
                               /* index, three classes).  b > 0: group only by the top b  */
                               /* bits of the transit's id - fewer radix passes, no       */
                               /* segment scan or classification; every draw then goes    */
                               /* through the lane-per-draw kernel, which needs transits  */
                               /* to be near each other, not equal.  Same output.         */
    int32_t sched_window;      /* random walks: scope of the grouping by transit.              */
                               /* -1: all samples of the call (GPU-wide sort and scan, three   */
                               /* classes); 256, 1024 or 2048: windows of that many            */
                               /* consecutive samples, each kept by one workgroup for the      */
                               /* whole walk (pairs per transit counted in LDS; a transit with */
                               /* many pairs in its window is sorted out, grouped and served   */
                               /* workgroup-wide from LDS, the others lane-per-pair;           */
                               /* sched_sub_max then is the largest number of pairs of one     */
                               /* transit in a window served lane-per-pair, default 63; no     */
                               /* grid class); 0: windows for walks unless sched_force_class,  */
                               /* sched_sub_max, sched_wg_max or sched_group_bits is set.      */
                               /* Same output.                                                 */
    int32_t reserved[2];
} nd_params;

typedef struct nd_graph nd_graph; /* opaque; owned by the library */

/* Fills *p with the defaults (n2v_max_attempts = 64, p = q = 1, mode =
 * transit-parallel, class AUTO, everything else 0). */
void nd_params_init(nd_params* p);

/*
 * Copies a CSR graph into device memory owned by the library (Section 5.1:
 * the graph lives in GPU global memory) and, when weights are given, builds
 * what the paper's Vertex class offers (Section 4.1): per vertex the largest
 * edge weight and the running sums of its edge weights.  Weights are
 * quantised once to integers, w_q = floor(w * 2^16 + 0.5), and all later
 * arithmetic on them is integer.
 *
 *   row_offsets      V+1 entries, int32 (offsets_are_int64 = 0) or int64; host or device
 *   col_indices      E entries, int32; every row strictly ascending (no duplicates)
 *   weights_or_null  E float32 entries or NULL
 *   src_is_device    0: the three arrays are host memory; 1: device memory
 *   hip_stream       hipStream_t to work on (NULL = the default stream); the call
 *                    returns after the work on it has completed
 *
 * Errors: ND_ERR_NULL_POINTER; ND_ERR_TOO_LARGE (V >= 2^31 or V < 1 ...);
 * ND_ERR_BAD_GRAPH (offsets[0] != 0, offsets not monotone, offsets[V] != E, a
 * column outside [0, V), a row not strictly ascending); ND_ERR_BAD_WEIGHT;
 * ND_ERR_HIP.  On error *out is NULL and nothing stays allocated.
 */
int nd_graph_create(nd_graph** out, int64_t V, int64_t E, const void* row_offsets,
                    int offsets_are_int64, const int32_t* col_indices,
                    const float* weights_or_null, int src_is_device, void* hip_stream);

/*
 * Ends the life of the graph's device copy (Section 5.1: the graph stays in GPU
 * global memory for as long as samples are drawn from it; Section 6.4: one copy
 * per GPU).  Frees everything nd_graph_create allocated.  Accepts NULL.  No
 * nd_sample call on this graph may still be running.
 */
int nd_graph_destroy(nd_graph* g);

/* V, E, whether weights are present, and the width of the stored offsets. */
int nd_graph_info(const nd_graph* g, int64_t* V, int64_t* E, int* has_weights,
                  int* offsets_are_int64);

/*
 * Sizes of one nd_sample call (Section 4.1, "Output format": the second form,
 * one array per step whose length follows from the number of samples and the
 * application's steps(), stepSize(i) and sampleSize(i); Section 4.1's
 * stepTransits fixes how many transits, hence slots, step i has).
 *   num_roots        walks and k-hop: one sample per root; layer and multi-
 *                    dimensional walk: a multiple of roots_per_sample (one sample
 *                    per group of consecutive roots)
 *   num_steps        out: number of per-step output arrays
 *   step_len         out, host, at least num_steps entries (ND_MAX_WALK_STEPS is
 *                    always enough): int32 elements of each step's array.
 *                    Walks: S.  k-hop: S * fanout[0] * ... * fanout[i].
 *                    Layer: num_samples * fanout[i].
 *   workspace_bytes  out: device scratch nd_sample needs for these arguments
 */
int nd_sample_query(const nd_graph* g, int app, const nd_params* params, int64_t num_roots,
                    int32_t* num_steps, int64_t* step_len, size_t* workspace_bytes);

/*
 * Runs every step of the application for all roots (Section 3: starting from
 * the initial samples, each step takes the step's transit vertices of every
 * sample and adds vertices drawn from their neighbourhoods, individually per
 * transit or collectively per sample; Section 4.1: the run ends after steps()
 * steps; Section 5.2 and Section 6: every step is executed transit-parallel),
 * asynchronously on hip_stream, allocating nothing.
 *
 *   roots_dev        device, num_roots int32 vertices.  A root outside [0, V) is
 *                    treated as NULL and recorded (see nd_sample_status).
 *   seed             Philox key
 *   step_out_dev     host array of num_steps device pointers, caller-allocated,
 *                    step i holding step_len[i] int32.  Layouts:
 *                      walks   out[i][s]             vertex walk s adds at step i
 *                      k-hop   out[i][s*W_i + j]     slot j of sample s; its parent
 *                                                    is slot j / fanout[i] of step i-1
 *                      layer   out[i][b*fanout[i]+j] j-th vertex of sample b's layer i
 *                    Roots are not repeated in the output.
 *   workspace_dev    device scratch of at least workspace_bytes, 256-byte aligned;
 *                    owned by the caller, reusable by the next call on the same
 *                    stream
 *
 * The call only launches kernels (no allocation, no memset or copy, no wait
 * for the device, no read-back), so it can be recorded into a HIP graph with
 * stream capture and replayed; calls that use different workspaces and output
 * arrays may run at the same time on different streams.
 *
 * Errors (checked before anything is launched): ND_ERR_NULL_POINTER,
 * ND_ERR_BAD_ARGUMENT, ND_ERR_NO_WEIGHTS, ND_ERR_WORKSPACE, ND_ERR_TOO_LARGE,
 * ND_ERR_HIP.
 */
int nd_sample(const nd_graph* g, int app, const nd_params* params, const int32_t* roots_dev,
              int64_t num_roots, uint64_t seed, int32_t* const* step_out_dev, void* workspace_dev,
              size_t workspace_bytes, void* hip_stream);

/*
 * nd_sample for callers that cannot allocate device memory and have no
 * workspace to bring: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, same kernels and the same
 * outputs as nd_sample, but the scratch is an array of
 * ND_STATIC_SCRATCH_BYTES that is part of the library's code object (every GPU
 * the library runs on holds its own copy until the process ends).  The call
 * allocates and frees nothing, on the host side of HIP or in the library.
 *
 *   status_dev       device, one uint32, or NULL: receives what nd_sample_status
 *                    would report (bit 0 set: a root was outside [0, V)), written
 *                    by the last kernel of the call on hip_stream
 *
 * The graph's device must be current.  A call whose nd_sample_query
 * workspace_bytes exceeds ND_STATIC_SCRATCH_BYTES fails with ND_ERR_TOO_LARGE
 * before anything is launched (split the roots over several calls with
 * sample_id_base, or use nd_sample).  All calls on one GPU share that GPU's
 * array, which keeps the previous call's contents (the call clears what must
 * start at zero): calls that overlap in time on one GPU, on whatever streams,
 * race and give undefined outputs.  Other errors as nd_sample.
 */
#define ND_STATIC_SCRATCH_BYTES (32u << 20)
int nd_sample_static(const nd_graph* g, int app, const nd_params* params, const int32_t* roots_dev,
                     int64_t num_roots, uint64_t seed, int32_t* const* step_out_dev,
                     uint32_t* status_dev, void* hip_stream);

/*
 * Waits for hip_stream and reports what the last nd_sample that used this
 * workspace recorded on the device: ND_OK, or ND_ERR_BAD_ROOT.
 */
int nd_sample_status(const void* workspace_dev, void* hip_stream);

/*
 * Per-step scheduling statistics of the last transit-parallel nd_sample on
 * this workspace (waits for hip_stream).  stats receives, for each of the
 * first max_steps steps, 8 int64 values: live pairs, distinct transits,
 * transits in the sub-wavefront / workgroup / grid class, grid chunks,
 * work items staged in LDS, draws made by the workgroup and grid classes.  Evidence
 * for Section 6.1.2's partition.
 */
int nd_sample_stats(const void* workspace_dev, void* hip_stream, int32_t max_steps,
                    int64_t* stats);

/*
 * The scheduling-index build on its own (Section 6.1.2, "Scheduling"; Section
 * 8.1): groups the live entries of a transit array by transit vertex.
 *
 *   transits_dev     device, n int32: transit of every slot (negative = no transit)
 *   V                transits are < V
 *   sorted_transits_dev, sorted_slots_dev   device, n int32 each: the live pairs
 *                    ordered by transit, slots of equal transits ascending
 *   group_transit_dev, group_start_dev      device, n and n+1 int32: distinct
 *                    transits ascending and the position of each one's first pair;
 *                    group_start[num_groups] = number of live pairs
 *   counts_dev       device, 2 int64: number of live pairs, number of groups
 *   workspace_dev    device scratch, nd_group_workspace_bytes(n, V) bytes
 */
size_t nd_group_workspace_bytes(int64_t n, int64_t V);
int nd_group_by_transit(const int32_t* transits_dev, int64_t n, int64_t V,
                        int32_t* sorted_transits_dev, int32_t* sorted_slots_dev,
                        int32_t* group_transit_dev, int32_t* group_start_dev, int64_t* counts_dev,
                        void* workspace_dev, size_t workspace_bytes, void* hip_stream);

/*
 * Edges between consecutive layers (Section 4.2, "Importance Sampling": every
 * sample carries the adjacency matrix between the transits of a step and the
 * vertices the step added; an edge is recorded between a new vertex and every
 * transit that has it as a neighbour).  Works on any pair of per-sample vertex
 * arrays, e.g. the roots and step 0, or steps i-1 and i, of a layer call.
 *
 *   transits_dev     device, num_samples * n_prev int32 (negative = empty slot)
 *   sampled_dev      device, num_samples * m int32 (negative = empty slot),
 *                    m <= ND_MAX_EDGE_SLOTS
 *   row_ptr_dev      device, num_samples * n_prev + 1 int64: one CSR over the
 *                    rows (sample b, transit slot t), row b * n_prev + t
 *   edge_slot_dev    device, capacity int32: a row lists every new slot j of the
 *                    same sample with sampled[b][j] in adj(transits[b][t]), ordered
 *                    by (vertex id, j); a vertex held by several slots gives one
 *                    entry per slot
 *   workspace_dev    device scratch of nd_layer_edges_workspace_bytes bytes,
 *                    256-byte aligned, owned by the caller
 *
 * nd_layer_edges_count writes row_ptr (asynchronously on hip_stream); the caller
 * reads row_ptr[num_samples * n_prev], allocates that many entries and calls
 * nd_layer_edges_fill with the same arguments.  Entries at or beyond capacity are
 * not written.  A vertex outside [-1, V) counts as an empty slot and is recorded:
 * nd_layer_edges_status waits for the stream and returns ND_ERR_BAD_ROOT then.
 * Neither call allocates.  Errors: ND_ERR_NULL_POINTER, ND_ERR_BAD_ARGUMENT,
 * ND_ERR_TOO_LARGE, ND_ERR_WORKSPACE, ND_ERR_HIP.
 */
#define ND_MAX_EDGE_SLOTS 2048
size_t nd_layer_edges_workspace_bytes(int64_t num_samples, int32_t n_prev);
int nd_layer_edges_count(const nd_graph* g, const int32_t* transits_dev, int32_t n_prev,
                         const int32_t* sampled_dev, int32_t m, int64_t num_samples,
                         int64_t* row_ptr_dev, void* workspace_dev, size_t workspace_bytes,
                         void* hip_stream);
int nd_layer_edges_fill(const nd_graph* g, const int32_t* transits_dev, int32_t n_prev,
                        const int32_t* sampled_dev, int32_t m, int64_t num_samples,
                        const int64_t* row_ptr_dev, int32_t* edge_slot_dev, int64_t capacity,
                        void* hip_stream);
int nd_layer_edges_status(const void* workspace_dev, void* hip_stream);

/*
 * Output format 1 of Section 4.1 ("Output format": an array of samples, each
 * holding all vertices sampled at all steps, as consumers of random walks and
 * layer samples read them).  nd_sample writes format 2 (one array per step);
 * this call gathers those arrays into one record per sample:
 *
 *   samples[s * record + off_i + j] = step_out[i][s * w_i + j]
 *   w_i = step_len[i] / num_samples,  off_i = w_0 + ... + w_{i-1},  record = sum of w_i
 *
 *   step_out_dev   host array of num_steps device pointers (as given to nd_sample)
 *   step_len       host array of num_steps lengths (as returned by nd_sample_query),
 *                  each a positive multiple of num_samples
 *   num_samples    walks and k-hop: the number of roots; layer and multi-
 *                  dimensional walk: num_roots / roots_per_sample
 *   samples_dev    device, num_samples * record int32
 *
 * A walk's record is its path without the root; a k-hop record lists hop 1,
 * then hop 2, ...  Asynchronous on hip_stream; allocates nothing.  Errors:
 * ND_ERR_NULL_POINTER, ND_ERR_BAD_ARGUMENT, ND_ERR_TOO_LARGE, ND_ERR_HIP.
 */
int nd_samples_pack(const int32_t* const* step_out_dev, int32_t num_steps, const int64_t* step_len,
                    int64_t num_samples, int32_t* samples_dev, void* hip_stream);

/*
 * Phase timing, for measurement.  After nd_profile_enable(1) on a thread, the
 * nd_sample calls of that thread bracket every phase of every step with HIP
 * events on their stream (a few microseconds per step; no synchronisation).
 * nd_profile_read waits for the recorded events, adds the elapsed milliseconds
 * and the number of intervals of every phase since the previous read to
 * ms[ND_PHASE_COUNT] and intervals[ND_PHASE_COUNT] (the caller zeroes them),
 * and resets the recording.  At most 16384 events are kept between reads;
 * later marks are dropped and nd_profile_read then returns ND_ERR_BAD_ARGUMENT.
 * The sampling phases contain exactly one kernel launch per interval.
 */
typedef enum nd_phase {
    ND_PHASE_NONE = -1,
    ND_PHASE_INIT = 0,        /* workspace header / bitmap reset                    */
    ND_PHASE_SORT = 1,        /* transit enumeration, NULL fill + radix sort        */
    ND_PHASE_GROUP = 2,       /* segmented scan + classification                    */
    ND_PHASE_SAMPLE_SUB = 3,  /* the step's sampling kernel (all three classes)     */
    ND_PHASE_SAMPLE_WG = 4,   /* the same kernel when a heavy class is forced       */
    ND_PHASE_SAMPLE_SP = 5,   /* sample-parallel kernel (ablation mode)             */
    ND_PHASE_LAYER = 6,       /* collective (layer) kernel                          */
    ND_PHASE_UNIQUE = 7,      /* duplicate removal and refill (unique neighbours)   */
    ND_PHASE_WALK_WINDOW = 8, /* walk kernel with per-window grouping in LDS (one   */
                              /* launch per 128 steps)                              */
    ND_PHASE_COUNT = 9
} nd_phase;
int nd_profile_enable(int on);
int nd_profile_read(double* ms, int64_t* intervals);

/*
 * Store-pattern probe, for measurement (Section 6.1.1: the point of sub-warp
 * execution is that a sample's new vertices leave in one coalesced write; this
 * call measures what such writes cost on this GPU when the runs land at
 * scattered places, as they do after grouping by transit).  Writes n_runs runs of
 * run_len int32 each into out_dev (n_runs * run_len entries; n_runs a power of
 * two, run_len in [1, 32]): run r goes to run position mix(r), a fixed pseudo-random
 * bijection of [0, n_runs), when scattered != 0, to position r otherwise; every entry of out_dev is
 * written exactly once.  Asynchronous on hip_stream; allocates nothing.
 * Errors: ND_ERR_NULL_POINTER, ND_ERR_BAD_ARGUMENT, ND_ERR_HIP.
 */
int nd_probe_store_runs(int32_t* out_dev, int64_t n_runs, int32_t run_len, int scattered, void* hip_stream);

/* Message of the last failure of a call of this library on the calling thread (the paper's system
 * reports errors through its host program; this ABI returns a status code and keeps the text here).
 * The pointer stays valid until the thread's next failing call. */
const char* nd_last_error(void);
/* ND_VERSION of the loaded library. */
int nd_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ND_H_ */
