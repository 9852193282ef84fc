// CSR loader: copies the graph to device memory, validates it there and builds
// the per-vertex weight data the paper's Vertex class offers (Section 4.1:
// degree, largest edge weight, running sums of the edge weights).
#include <cmath>
#include <cstdio>
#include <new>

#include "nd_common.h"
#include "nd_wave.h"

namespace nd {

namespace {

enum : uint32_t {
    kBadFirst = 1u,      // offsets[0] != 0
    kBadMonotone = 2u,   // offsets decrease somewhere or leave [0, E]
    kBadLast = 4u,       // offsets[V] != E
    kBadColumn = 8u,     // a column outside [0, V)
    kBadOrder = 16u,     // a row not strictly ascending
    kBadWeight = 32u,    // weight not finite, <= 0 or >= 2^15
    kBadRowTotal = 64u   // a row's quantised weights sum to 2^39 or more
};

template <typename OffT>
__global__ void check_offsets_kernel(const OffT* __restrict__ off, int64_t V, int64_t E,
                                     uint32_t* __restrict__ flags,
                                     unsigned long long* __restrict__ max_degree) {
    const int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    uint32_t bad = 0;
    if (v == 0 && off[0] != 0) bad |= kBadFirst;
    if (v == 0 && (int64_t)off[V] != E) bad |= kBadLast;
    if (v < V) {
        const int64_t a = (int64_t)off[v], b = (int64_t)off[v + 1];
        if (a > b || a < 0 || b > E) bad |= kBadMonotone;
        else atomicMax(max_degree, (unsigned long long)(b - a));
    }
    if (bad) atomicOr(flags, bad);
}

// One wavefront per row, 64 entries at a time: columns in range and strictly
// ascending; with weights, quantise (w_q = floor(w * 2^16 + 0.5), evaluated in
// double), accumulate the running sums (a wave scan per 64 entries plus the sum
// carried from the entries before) and the row maximum.  Rows are dealt to the
// wavefronts round robin, so a row of any length costs its wavefront
// ceil(deg / 64) rounds and the long rows of a skewed graph do not serialise.
template <typename OffT>
__global__ __launch_bounds__(256) void check_rows_kernel(const OffT* __restrict__ off, const int32_t* __restrict__ col,
                                                         const float* __restrict__ w, int64_t V,
                                                         uint32_t* __restrict__ wq, uint64_t* __restrict__ cumq,
                                                         uint32_t* __restrict__ maxwq, uint32_t* __restrict__ flags) {
    const int lane = lane_id();
    const int64_t wave0 = ((int64_t)blockIdx.x * 256 + threadIdx.x) >> 6;
    const int64_t n_waves = ((int64_t)gridDim.x * 256) >> 6;
    uint32_t bad = 0;
    for (int64_t v = wave0; v < V; v += n_waves) {  // the same v on every lane of the wave
        const int64_t lo = (int64_t)off[v], hi = (int64_t)off[v + 1];
        unsigned long long run = 0;
        uint32_t mx = 0;
        for (int64_t base = lo; base < hi; base += 64) {
            const int64_t e = base + lane;
            const bool in = e < hi;
            const int32_t c = in ? col[e] : 0;
            int32_t before = __shfl_up(c, 1, 64);
            if (lane == 0) before = e > lo ? col[e - 1] : -1;
            if (in && (c < 0 || (int64_t)c >= V)) bad |= kBadColumn;
            if (in && c <= before) bad |= kBadOrder;
            if (w) {
                uint32_t q = 0;
                if (in) {
                    const float x = w[e];
                    q = 1;
                    if (!(x > 0.0f) || !(x < 32768.0f)) bad |= kBadWeight;
                    else q = (uint32_t)floor((double)x * 65536.0 + 0.5);
                    wq[e] = q;
                    if (q > mx) mx = q;
                }
                const unsigned long long incl = wave_inclusive_scan((unsigned long long)q, lane);
                if (in) cumq[e] = run + incl;
                run += __shfl(incl, 63, 64);
            }
        }
        if (w) {
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) {
                const uint32_t o = __shfl_xor(mx, d, 64);
                mx = o > mx ? o : mx;
            }
            if (lane == 0) maxwq[v] = mx;
            if (run >= (1ull << 39)) bad |= kBadRowTotal;
        }
    }
    if (bad) atomicOr(flags, bad);
}

void free_graph(Graph* g) {
    if (!g) return;
    (void)hipFree(g->off);
    (void)hipFree(g->col);
    (void)hipFree(g->wq);
    (void)hipFree(g->cumq);
    (void)hipFree(g->maxwq);
    delete g;
}

template <typename OffT>
int validate_and_build(Graph* g, const float* w_dev, uint32_t* flags_dev, hipStream_t stream) {
    const int threads = 256;
    const int64_t blocks = (g->V + threads) / threads;  // covers v == V-1 and the v == 0 checks
    hipLaunchKernelGGL(check_offsets_kernel<OffT>, dim3((unsigned)blocks), dim3(threads), 0, stream,
                       (const OffT*)g->off, g->V, g->E, flags_dev,
                       (unsigned long long*)(flags_dev + 2));
    ND_HIP_CHECK(hipGetLastError());
    uint32_t flags = 0;
    unsigned long long max_degree = 0;
    ND_HIP_CHECK(hipMemcpyAsync(&flags, flags_dev, sizeof(flags), hipMemcpyDeviceToHost, stream));
    ND_HIP_CHECK(hipMemcpyAsync(&max_degree, flags_dev + 2, sizeof(max_degree), hipMemcpyDeviceToHost,
                                stream));
    ND_HIP_CHECK(hipStreamSynchronize(stream));
    g->max_degree = (int64_t)max_degree;
    if (flags) {
        set_error("bad CSR offsets:%s%s%s", (flags & kBadFirst) ? " offsets[0] != 0;" : "",
                  (flags & kBadMonotone) ? " offsets not monotone within [0, E];" : "",
                  (flags & kBadLast) ? " offsets[V] != E;" : "");
        return ND_ERR_BAD_GRAPH;
    }
    // rows may only be walked once the offsets are known to be sane
    {   // one wavefront per row; enough workgroups to fill the chip several times, never more than rows / 4
        int64_t row_blocks = (g->V + 3) / 4;
        const int64_t cap = (int64_t)g->num_cus * 16;
        if (row_blocks > cap) row_blocks = cap;
        hipLaunchKernelGGL(check_rows_kernel<OffT>, dim3((unsigned)row_blocks), dim3(256), 0, stream,
                           (const OffT*)g->off, g->col, w_dev, g->V, g->wq, g->cumq, g->maxwq, flags_dev);
    }
    ND_HIP_CHECK(hipGetLastError());
    ND_HIP_CHECK(hipMemcpyAsync(&flags, flags_dev, sizeof(flags), hipMemcpyDeviceToHost, stream));
    ND_HIP_CHECK(hipStreamSynchronize(stream));
    if (flags & (kBadColumn | kBadOrder)) {
        set_error("bad CSR rows:%s%s", (flags & kBadColumn) ? " a column is outside [0, V);" : "",
                  (flags & kBadOrder) ? " a row is not strictly ascending (unsorted or duplicate);" : "");
        return ND_ERR_BAD_GRAPH;
    }
    if (flags & (kBadWeight | kBadRowTotal)) {
        set_error("bad weights:%s%s",
                  (flags & kBadWeight) ? " a weight is not finite, <= 0 or >= 2^15;" : "",
                  (flags & kBadRowTotal) ? " a row's quantised weights sum to 2^39 or more;" : "");
        return ND_ERR_BAD_WEIGHT;
    }
    return ND_OK;
}

}  // namespace

int graph_create(Graph** out, int64_t V, int64_t E, const void* off, int off64, const int32_t* col,
                 const float* w, int src_is_device, hipStream_t stream) {
    Graph* g = new (std::nothrow) Graph;
    if (!g) {
        set_error("out of host memory");
        return ND_ERR_HIP;
    }
    g->V = V;
    g->E = E;
    g->off64 = off64;
    float* w_dev = nullptr;
    uint32_t* flags_dev = nullptr;
    int rc = ND_OK;
    auto body = [&]() -> int {
        ND_HIP_CHECK(hipGetDevice(&g->device));
        ND_HIP_CHECK(hipDeviceGetAttribute(&g->num_cus, hipDeviceAttributeMultiprocessorCount, g->device));
        if (g->num_cus < 1) g->num_cus = 1;
        const size_t off_bytes = (size_t)(V + 1) * (off64 ? 8 : 4);
        const size_t e_alloc = (size_t)(E > 0 ? E : 1);
        const hipMemcpyKind kind = src_is_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice;
        ND_HIP_CHECK(hipMalloc(&g->off, off_bytes));
        ND_HIP_CHECK(hipMalloc((void**)&g->col, e_alloc * 4));
        ND_HIP_CHECK(hipMalloc((void**)&flags_dev, 256));
        ND_HIP_CHECK(hipMemsetAsync(flags_dev, 0, 256, stream));
        ND_HIP_CHECK(hipMemcpyAsync(g->off, off, off_bytes, kind, stream));
        if (E > 0) ND_HIP_CHECK(hipMemcpyAsync(g->col, col, (size_t)E * 4, kind, stream));
        if (w) {
            ND_HIP_CHECK(hipMalloc((void**)&w_dev, e_alloc * 4));
            ND_HIP_CHECK(hipMalloc((void**)&g->wq, e_alloc * 4));
            ND_HIP_CHECK(hipMalloc((void**)&g->cumq, e_alloc * 8));
            ND_HIP_CHECK(hipMalloc((void**)&g->maxwq, (size_t)V * 4));
            if (E > 0) ND_HIP_CHECK(hipMemcpyAsync(w_dev, w, (size_t)E * 4, kind, stream));
        }
        return off64 ? validate_and_build<int64_t>(g, w_dev, flags_dev, stream)
                     : validate_and_build<int32_t>(g, w_dev, flags_dev, stream);
    };
    rc = body();
    (void)hipStreamSynchronize(stream);
    (void)hipFree(w_dev);
    (void)hipFree(flags_dev);
    if (rc != ND_OK) {
        free_graph(g);
        *out = nullptr;
        return rc;
    }
    *out = g;
    return ND_OK;
}

void graph_destroy(Graph* g) { free_graph(g); }

}  // namespace nd
