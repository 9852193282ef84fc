// Internal declarations shared by the library's translation units.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "../../include/nd.h"

namespace nd {

constexpr int kWave = 64;

// ---------------------------------------------------------------- errors
void set_error(const char* fmt, ...);
#define ND_HIP_CHECK(expr)                                                              \
    do {                                                                                \
        hipError_t e_ = (expr);                                                         \
        if (e_ != hipSuccess) {                                                         \
            nd::set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, __LINE__); \
            return ND_ERR_HIP;                                                          \
        }                                                                               \
    } while (0)

// ---------------------------------------------------------------- phase timing (measurement only)
// When enabled on the calling thread, every call of mark_phase records a HIP
// event on the stream; the time between two marks is charged to the phase of
// the first.  ND_PHASE_NONE closes the current interval.
void mark_phase(int phase, hipStream_t stream);

// ---------------------------------------------------------------- graph
struct Graph {
    int64_t V = 0, E = 0;
    int off64 = 0;              // width of row offsets as stored
    void* off = nullptr;        // V+1 int32 or int64 (device)
    int32_t* col = nullptr;     // E (device)
    uint32_t* wq = nullptr;     // E quantised weights (device) or null
    uint64_t* cumq = nullptr;   // E inclusive running sums of wq per row (device) or null
    uint32_t* maxwq = nullptr;  // V largest wq per row (device) or null
    int device = 0;
    int num_cus = 256;
    int64_t max_degree = 0;
};

// Device-side view passed to kernels by value.
template <typename OffT>
struct GraphView {
    const OffT* off;
    const int32_t* col;
    const uint32_t* wq;
    const uint64_t* cumq;
    const uint32_t* maxwq;
    int32_t V;
};

template <typename OffT>
inline GraphView<OffT> view_of(const Graph& g) {
    return GraphView<OffT>{(const OffT*)g.off, g.col, g.wq, g.cumq, g.maxwq, (int32_t)g.V};
}

// Length of row v, given where it starts.  A row is shorter than 2^32, so the low words of the two
// offsets suffice, and with 64-bit offsets the high word of the second one is not fetched: a
// register that a load in flight is about to fill and nobody reads is reused at once, and that use
// waits for the load (in the k-hop loop this cost a tenth of the kernel's time).
template <typename OffT>
__device__ __forceinline__ uint32_t row_length(const GraphView<OffT>& g, int32_t v, uint64_t row_start) {
    return reinterpret_cast<const uint32_t*>(g.off + v + 1)[0] - (uint32_t)row_start;
}

int graph_create(Graph** out, int64_t V, int64_t E, const void* off, int off64, const int32_t* col,
                 const float* w, int src_is_device, hipStream_t stream);
void graph_destroy(Graph* g);

// ---------------------------------------------------------------- division by a runtime constant
// Exact floor(n / d) for 0 <= n < 2^31 and 1 <= d < 2^31:
// q = mulhi32(n, magic) >> shift with magic = ceil(2^(32+shift) / d) (Granlund-Montgomery,
// valid because n < 2^31 leaves one bit of headroom).
struct FastDiv {
    uint32_t d, magic, shift;
};
inline FastDiv make_fastdiv(uint32_t d) {
    FastDiv f;
    f.d = d;
    if (d == 1) {
        f.magic = 0;
        f.shift = 0;
        return f;
    }
    uint32_t s = 0;
    while ((1ull << s) < d) ++s;  // s = ceil(log2 d)
    f.shift = s - 1;
    f.magic = (uint32_t)(((1ull << (32 + s - 1)) + d - 1) / d);
    return f;
}

// ---------------------------------------------------------------- per-step control block (device)
// Written by the grouping kernels, read by the kernels that follow on the same
// stream; the host never reads it inside nd_sample.
struct StepCtl {
    uint32_t P;             // live pairs of the step
    uint32_t U;             // distinct transits
    uint32_t n_wg;          // transits in the workgroup class
    uint32_t n_grid;        // transits in the grid class
    uint32_t n_chunks;      // grid chunks
    uint32_t reserved0;
    uint32_t n_staged;      // workgroup/grid work items that staged their list in LDS
    uint32_t wg_cursor;     // next workgroup-class item to hand out
    uint32_t reserved1;
    uint32_t heavy_draws;   // draws of the workgroup- and grid-class transits
    uint32_t pad[6];
};
static_assert(sizeof(StepCtl) == 64, "one control block per 64 bytes");

struct WsHeader {
    uint32_t status;        // bit 0: a root was out of range
    uint32_t num_steps;
    uint32_t pad[62];
};
static_assert(sizeof(WsHeader) == 256, "header is one 256-byte block");

// ---------------------------------------------------------------- radix sort plan
constexpr int kSortThreads = 512;       // large inputs: 8,192 keys per tile
constexpr int kSortItems = 16;
constexpr int kSmallSortThreads = 256;  // small inputs: 2,048 keys per tile
constexpr int kSmallSortItems = 8;
constexpr int64_t kSmallSortLimit = 1 << 23;
constexpr int kMaxRadixBits = 8;

struct SortPlan {
    int passes;
    int bits[4];
    int shift[4];
    int tile;               // keys per tile
    int64_t max_tiles;      // tiles of the slot array (pass 0); later passes never need more
};
// group_bits > 0: sort on the top group_bits bits of the key only.
SortPlan make_sort_plan(int64_t n_slots, int64_t V, int group_bits = 0);
size_t sort_hist_bytes(const SortPlan& p);

// Pass 0 reads `src` (n_slots transits, negative = no transit, implicit value = index)
// and, if fill_out is given, writes ND_NULL_VERTEX into the m children of every dead slot.
// The sorted pairs end in (keys_out, vals_out) which is one of the two buffer pairs.
int sort_pairs(const int32_t* src, int64_t n_slots, int32_t V, const SortPlan& plan,
               int32_t* keysA, int32_t* valsA, int32_t* keysB, int32_t* valsB, uint32_t* hist,
               StepCtl* ctl, int32_t* fill_out, int32_t m, uint32_t* status_word,
               int32_t** keys_out, int32_t** vals_out, hipStream_t stream);

// ---------------------------------------------------------------- scheduling index
constexpr int kSegThreads = 256;
constexpr int kSegItems = 16;
constexpr int kSegTile = kSegThreads * kSegItems;
size_t seg_scratch_bytes(int64_t n_slots);
// heavy_bits (may be null): the per-vertex marks of the previous step are cleared on the way.
int build_groups(const int32_t* sorted_keys, int64_t max_pairs, StepCtl* ctl, int32_t* g_key,
                 int32_t* g_start, uint32_t* tile_counts, uint32_t* heavy_bits, int64_t bit_words,
                 hipStream_t stream);

struct SchedParams {
    int32_t m;              // draws per pair
    int32_t sub_max;        // draws <= sub_max: sub-wavefront class
    int32_t wg_max;         // draws <= wg_max: workgroup class; chunk size of the grid class
    int32_t force_class;    // nd_sched_class
};
// Scheduling class of a transit that must produce `draws` neighbours
// (Section 6.1.2, Table "Types of kernels", with wave64 thresholds).
__host__ __device__ inline int class_of(uint32_t draws, const SchedParams& sp) {
    if (sp.force_class != ND_CLASS_AUTO) return sp.force_class;
    if (draws <= (uint32_t)sp.sub_max) return ND_CLASS_SUBWAVE;
    if (draws <= (uint32_t)sp.wg_max) return ND_CLASS_WORKGROUP;
    return ND_CLASS_GRID;
}
// Fills the workgroup list and the grid chunk list and marks their transits in heavy_bits
// (one bit per vertex; may be null when a class is forced).
int classify_groups(const int32_t* g_key, const int32_t* g_start, int64_t max_groups, StepCtl* ctl,
                    const SchedParams& sp, int32_t* list_wg, int32_t* chunk_gid, int32_t* chunk_idx,
                    int64_t max_chunks, uint32_t* heavy_bits, hipStream_t stream);

}  // namespace nd
