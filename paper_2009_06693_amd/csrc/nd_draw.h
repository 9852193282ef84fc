// What one lane draws (Section 4.2 of the paper: the `next` functions of the
// applications), shared by every sampling kernel: uniform neighbour (DeepWalk,
// PPR, k-hop), weight-proportional neighbour by inverse transform, node2vec by
// rejection sampling.  One Philox call per (sample, slot, step, attempt).
#pragma once

#include "nd_common.h"
#include "nd_philox.h"
#include "nd_sample.h"

namespace nd {

constexpr uint32_t kOneQ16 = 65536u;

// ---------------------------------------------------------------- one draw
// adj / cum / wq point at the transit's row (global memory or its LDS copy).

template <typename OffT>
__device__ __forceinline__ bool row_contains(const GraphView<OffT>& g, uint64_t rs, uint32_t deg,
                                             int32_t u) {
    uint32_t lo = 0, hi = deg;
    while (lo < hi) {
        const uint32_t mid = (lo + hi) >> 1;
        const int32_t c = g.col[rs + mid];
        if (c < u) lo = mid + 1;
        else hi = mid;
    }
    return lo < deg && g.col[rs + lo] == u;
}

// Uniform neighbour (DeepWalk, PPR, k-hop): index = high word of R0 * degree.
__device__ __forceinline__ int32_t draw_uniform(const DrawArgs& a, uint32_t deg, uint32_t sid,
                                                uint32_t slot, const int32_t* adj) {
    const Rand4 r = draw4(a.seed, sid, slot, a.step, 0u);
    if (a.ppr_thr != 0 && (uint64_t)r.r3 < a.ppr_thr) return ND_NULL_VERTEX;
    return adj[mulhi32(r.r0, deg)];
}

// Weight-proportional neighbour: inverse transform on the row's running sums.
__device__ __forceinline__ int32_t draw_weighted(const DrawArgs& a, uint32_t deg, uint32_t sid,
                                                 uint32_t slot, const int32_t* adj,
                                                 const uint64_t* cum) {
    const Rand4 r = draw4(a.seed, sid, slot, a.step, 0u);
    if (a.ppr_thr != 0 && (uint64_t)r.r3 < a.ppr_thr) return ND_NULL_VERTEX;
    const uint64_t x = mulhi64(cat64(r.r0, r.r1), cum[deg - 1]);
    uint32_t lo = 0, hi = deg - 1;
    while (lo < hi) {
        const uint32_t mid = (lo + hi) >> 1;
        if (cum[mid] > x) hi = mid;
        else lo = mid + 1;
    }
    return adj[lo];
}

// node2vec (Section 4.2): rejection sampling under the envelope
// maxEdgeWeight(v) * largest bias; the bias of candidate u depends on its
// relation to t, the transit of the previous step.  The membership search in
// t's row is skipped when both possible biases give the same verdict.
template <typename OffT>
__device__ __forceinline__ uint32_t n2v_bias(const GraphView<OffT>& g, const DrawArgs& a, int32_t t,
                                             uint64_t rs_t, uint32_t deg_t, int32_t u) {
    if (!a.has_prev) return kOneQ16;
    if (u == t) return a.b_ret;
    // values, not a choice between two members: the latter is a choice between two addresses and
    // keeps the whole structure in memory
    const uint32_t b_com = a.b_com, b_far = a.b_far;
    return row_contains(g, rs_t, deg_t, u) ? b_com : b_far;
}

// t: the transit of the previous step (read only when a.has_prev).
template <typename OffT>
__device__ __forceinline__ int32_t draw_node2vec(const GraphView<OffT>& g, const DrawArgs& a,
                                                 int32_t v, uint32_t deg, uint32_t sid,
                                                 int32_t t_prev, const int32_t* adj,
                                                 const uint32_t* wq) {
    const uint32_t maxw = a.use_weights ? g.maxwq[v] : kOneQ16;
    const uint64_t envelope = (uint64_t)maxw * (a.has_prev ? a.b_max : kOneQ16);
    int32_t t = ND_NULL_VERTEX;
    uint64_t rs_t = 0;
    uint32_t deg_t = 0;
    if (a.has_prev) {
        t = t_prev;
        rs_t = (uint64_t)g.off[t];
        deg_t = row_length(g, t, rs_t);
    }
    const uint32_t b_com = a.b_com, b_far = a.b_far;  // values: see n2v_bias
    const uint32_t b_lo = b_com < b_far ? b_com : b_far;
    const uint32_t b_hi = b_com < b_far ? b_far : b_com;
    for (int32_t att = 0; att < a.max_attempts; ++att) {
        const Rand4 r = draw4(a.seed, sid, 0u, a.step, (uint32_t)att);
        const uint32_t e = mulhi32(r.r0, deg);
        const int32_t u = adj[e];
        const uint64_t y = mulhi64(cat64(r.r1, r.r2), envelope);
        const uint64_t w = a.use_weights ? wq[e] : kOneQ16;
        if (!a.has_prev) {
            if (y < w * kOneQ16) return u;
        } else if (u == t) {
            if (y < w * a.b_ret) return u;
        } else if (y < w * b_lo) {
            return u;
        } else if (y < w * b_hi) {
            const uint32_t bias = row_contains(g, rs_t, deg_t, u) ? b_com : b_far;
            if (y < w * bias) return u;
        }
    }
    // exact fallback: inverse transform over all biased weights of the row
    const Rand4 r = draw4(a.seed, sid, 0u, a.step, (uint32_t)a.max_attempts);
    uint64_t Z = 0;
    for (uint32_t e = 0; e < deg; ++e) {
        const uint64_t w = a.use_weights ? wq[e] : kOneQ16;
        Z += w * n2v_bias(g, a, t, rs_t, deg_t, adj[e]);
    }
    const uint64_t x = mulhi64(cat64(r.r0, r.r1), Z);
    uint64_t run = 0;
    for (uint32_t e = 0; e < deg; ++e) {
        const uint64_t w = a.use_weights ? wq[e] : kOneQ16;
        run += w * n2v_bias(g, a, t, rs_t, deg_t, adj[e]);
        if (run > x) return adj[e];
    }
    return adj[deg - 1];  // not reached: x < Z
}

}  // namespace nd
