// Collective transit sampling (Section 6.2 of the paper; layer sampling with
// LADIES-style importance weights, Section 4.2 "Importance Sampling").
//
// The paper materialises every sample's combined neighbourhood in global
// memory (transit-parallel copy of whole adjacency lists) and then draws from
// it sample-parallel.  On this GPU the copy is the dominant traffic, so the
// combined neighbourhood stays implicit: it is the concatenation, in slot
// order, of the transits' adjacency lists, described by a running sum of
// per-transit masses deg(v) * c(v) kept in LDS; a draw picks a position in the
// concatenation by inverse transform (binary search over the running sums,
// then an integer division by c(v) inside the chosen list) and reads that one
// neighbour.  One workgroup per sample, as in the paper's sample-parallel draw.
// A transit's degree and row start are fetched once per (sample, transit slot).
//
// c(v) = floor(2^48 / deg(v)^2) is the fixed-point squared entry of the
// row-normalised adjacency matrix, so a vertex is drawn with probability
// proportional to its squared column norm restricted to the transit rows.
#include "nd_common.h"
#include "nd_philox.h"
#include "nd_sample.h"
#include "nd_wave.h"

namespace nd {

namespace {

// 512 lanes per sample: the transits' 24 bytes each of LDS allow three workgroups per CU, and the
// draws are chains of dependent reads, so the wider workgroup (24 waves per CU) hides more latency
constexpr int kLayerThreads = 512;

// Exact floor(num / c) for num < 2^24 * c: the quotient is estimated in double precision
// (relative error 2^-52, so off by at most one for a quotient below 2^24) and corrected with
// integer arithmetic.
__device__ __forceinline__ uint64_t div_small_quotient(uint64_t num, uint64_t c) {
    uint64_t q = (uint64_t)((double)num / (double)c);
    int64_t r = (int64_t)(num - q * c);
    if (r < 0) {
        --q;
        r += (int64_t)c;
    }
    if (r >= (int64_t)c) ++q;
    return q;
}

// Dynamic LDS: per transit slot the running sum of masses, the weight c(v) and the first
// adjacency entry of the transit (24 bytes), so a draw touches global memory once.
// WEIGHTED: an entry from transit v to u weighs the graph's quantised edge weight w_q(v,u); the
// mass of a transit is its row's weight sum and the place inside the row is found by a search
// over the row's running sums (global memory).
template <typename OffT, bool WEIGHTED>
__global__ __launch_bounds__(kLayerThreads) void layer_kernel(GraphView<OffT> g, LayerArgs a) {
    extern __shared__ uint64_t lds[];
    uint64_t* s_incl = lds;
    uint64_t* s_c = lds + a.n_prev;
    uint64_t* s_rs = lds + 2 * (size_t)a.n_prev;
    __shared__ uint64_t scan_tmp[kLayerThreads / 64 + 1];
    const uint32_t b = blockIdx.x;
    const int32_t* transits = a.transits + (uint64_t)b * a.n_prev;

    uint64_t carry = 0;
    bool bad = false;
    for (uint32_t base = 0; base < a.n_prev; base += kLayerThreads) {
        const uint32_t t = base + threadIdx.x;
        uint64_t mass = 0, c = 0, rs = 0;
        if (t < a.n_prev) {
            int32_t v = transits[t];
            if (v >= g.V || v < ND_NULL_VERTEX) {
                bad = true;
                v = ND_NULL_VERTEX;
            }
            if (v >= 0) {
                rs = (uint64_t)g.off[v];
                const uint64_t deg = (uint64_t)g.off[v + 1] - rs;
                if (deg > 0) {
                    if (WEIGHTED) {
                        c = deg;  // the row length takes the weight's place
                        mass = g.cumq[rs + deg - 1];
                    } else {
                        c = (1ull << 48) / (deg * deg);
                        mass = deg * c;
                    }
                }
            }
        }
        uint64_t total;
        const uint64_t ex = block_exclusive_scan<uint64_t, kLayerThreads>(mass, scan_tmp, &total);
        if (t < a.n_prev) {
            s_incl[t] = carry + ex + mass;
            s_c[t] = c;
            s_rs[t] = rs;
        }
        carry += total;
        __syncthreads();
    }
    if (a.check_roots && bad) atomicOr(a.status, 1u);
    const uint64_t total = carry;

    for (uint32_t j = threadIdx.x; j < a.m; j += kLayerThreads) {
        int32_t res = ND_NULL_VERTEX;
        if (total > 0) {
            const Rand4 r = draw4(a.seed, a.sample_base + b, j, a.step, 0u);
            const uint64_t x = mulhi64(cat64(r.r0, r.r1), total);
            uint32_t lo = 0, hi = a.n_prev - 1;
            while (lo < hi) {  // first transit whose running sum exceeds x
                const uint32_t mid = (lo + hi) >> 1;
                if (s_incl[mid] > x) hi = mid;
                else lo = mid + 1;
            }
            const uint64_t before = lo ? s_incl[lo - 1] : 0ull;
            uint64_t idx;
            if (WEIGHTED) {  // first entry of the row whose running sum exceeds what is left of x
                const uint64_t* cum = g.cumq + s_rs[lo];
                const uint64_t rest = x - before;
                uint64_t l = 0, h = s_c[lo] - 1;
                while (l < h) {
                    const uint64_t mid = (l + h) >> 1;
                    if (cum[mid] > rest) h = mid;
                    else l = mid + 1;
                }
                idx = l;
            } else {
                idx = div_small_quotient(x - before, s_c[lo]);
            }
            res = g.col[s_rs[lo] + idx];
        }
        a.out[(uint64_t)b * a.m + j] = res;
    }
}

}  // namespace

// Dynamic LDS above the 64 KB default has to be allowed once per kernel; done when a graph is
// created so that layer_step itself only launches.
int layer_prepare() {
#define ND_LAYER_ALLOW(OFFT, W)                                                                 \
    ND_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(&layer_kernel<OFFT, W>),     \
                                     hipFuncAttributeMaxDynamicSharedMemorySize,                \
                                     ND_MAX_LAYER_TRANSITS * 24))
    ND_LAYER_ALLOW(int64_t, true);
    ND_LAYER_ALLOW(int64_t, false);
    ND_LAYER_ALLOW(int32_t, true);
    ND_LAYER_ALLOW(int32_t, false);
#undef ND_LAYER_ALLOW
    return ND_OK;
}

int layer_step(const Graph& gr, const LayerArgs& a, int64_t num_samples, hipStream_t stream) {
    if (num_samples == 0) return ND_OK;
    const size_t lds_bytes = (size_t)a.n_prev * 24;  // at most 96 KB of the 160 KB per CU
#define ND_LAYER_LAUNCH(OFFT, W)                                                                    \
    hipLaunchKernelGGL((layer_kernel<OFFT, W>), dim3((unsigned)num_samples), dim3(kLayerThreads),  \
                       lds_bytes, stream, view_of<OFFT>(gr), a)
    if (gr.off64) {
        if (a.use_weights) ND_LAYER_LAUNCH(int64_t, true);
        else ND_LAYER_LAUNCH(int64_t, false);
    } else {
        if (a.use_weights) ND_LAYER_LAUNCH(int32_t, true);
        else ND_LAYER_LAUNCH(int32_t, false);
    }
#undef ND_LAYER_LAUNCH
    ND_HIP_CHECK(hipGetLastError());
    return ND_OK;
}

}  // namespace nd
