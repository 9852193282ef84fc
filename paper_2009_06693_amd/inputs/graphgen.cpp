// Seeded synthetic graph generators (R-MAT, Chung-Lu) producing a symmetrised,
// self-loop-free, duplicate-free CSR with ascending rows, plus symmetric
// float32 edge weights.
//
// This file is input plumbing shared by the tests, the benchmark, the CPU
// oracle and the GPU library: it holds none of the sampling method's
// arithmetic.  Its random numbers come from a counter-based 64-bit mixer
// (SplitMix64 finaliser) keyed on (seed, stream, index), so the output is a
// pure function of the arguments and does not depend on the thread count.
//
// The graphs stand in for the SNAP graphs of the paper's evaluation
// (Section 8, Table "Graph used in our evaluation"), which are not available
// offline; the weights follow the paper's recipe of drawing each edge weight
// uniformly from [1, 5).

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <vector>
#include <omp.h>

namespace {

inline uint64_t mix64(uint64_t z) {
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

inline uint64_t rnd(uint64_t seed, uint64_t stream, uint64_t index) {
    return mix64(mix64(mix64(seed) ^ (stream * 0xD6E8FEB86659FD93ull)) + index);
}

inline double u01(uint64_t r) { return (double)(r >> 11) * (1.0 / 9007199254740992.0); }

struct Csr {
    int64_t V = 0, E = 0;
    std::vector<int64_t> off;
    std::vector<int32_t> col;
};

// keys: (u << 32) | v for each directed entry.  Sorts, removes duplicates,
// builds CSR.  Parallel bucket sort on the source vertex.
void build_csr(std::vector<uint64_t>& keys, int64_t V, Csr& g) {
    const int64_t n = (int64_t)keys.size();
    int shift = 0;
    while ((V >> shift) > 4096) ++shift;
    const int64_t nb = (V >> shift) + 1;
    std::vector<int64_t> cnt(nb + 1, 0);
    for (int64_t i = 0; i < n; ++i) cnt[(keys[i] >> 32 >> shift) + 1]++;
    for (int64_t b = 0; b < nb; ++b) cnt[b + 1] += cnt[b];
    std::vector<uint64_t> tmp(n);
    {
        std::vector<int64_t> pos(cnt.begin(), cnt.end() - 1);
        for (int64_t i = 0; i < n; ++i) tmp[pos[keys[i] >> 32 >> shift]++] = keys[i];
    }
    std::vector<int64_t> uniq(nb, 0);
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t b = 0; b < nb; ++b) {
        uint64_t* lo = tmp.data() + cnt[b];
        uint64_t* hi = tmp.data() + cnt[b + 1];
        std::sort(lo, hi);
        uniq[b] = std::unique(lo, hi) - lo;
    }
    int64_t E = 0;
    for (int64_t b = 0; b < nb; ++b) E += uniq[b];
    g.V = V;
    g.E = E;
    g.off.assign(V + 1, 0);
    g.col.resize(E);
    int64_t w = 0;
    for (int64_t b = 0; b < nb; ++b) {
        const uint64_t* p = tmp.data() + cnt[b];
        for (int64_t i = 0; i < uniq[b]; ++i) {
            g.off[(p[i] >> 32) + 1]++;
            g.col[w++] = (int32_t)(p[i] & 0xFFFFFFFFull);
        }
    }
    for (int64_t v = 0; v < V; ++v) g.off[v + 1] += g.off[v];
    keys.clear();
    keys.shrink_to_fit();
}

// Sum of (i + i0)^(-alpha) over i in [0, V), accumulated in fixed blocks so the
// result does not depend on the thread count.  If cum is given it receives the
// inclusive running sums.
double powsum(int64_t V, double i0, double alpha, double* cum) {
    const int64_t B = 65536, nb = (V + B - 1) / B;
    std::vector<double> part(nb);
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < nb; ++b) {
        double s = 0.0;
        const int64_t hi = std::min(V, (b + 1) * B);
        for (int64_t i = b * B; i < hi; ++i) {
            s += std::pow((double)i + i0, -alpha);
            if (cum) cum[i] = s;
        }
        part[b] = s;
    }
    double s = 0.0;
    std::vector<double> base(nb);
    for (int64_t b = 0; b < nb; ++b) {
        base[b] = s;
        s += part[b];
    }
    if (cum) {
#pragma omp parallel for schedule(static)
        for (int64_t b = 0; b < nb; ++b) {
            const int64_t hi = std::min(V, (b + 1) * B);
            for (int64_t i = b * B; i < hi; ++i) cum[i] += base[b];
        }
    }
    return s;
}

// Relabels vertices by a seeded random permutation (rank of a per-vertex hash),
// so that vertex ids carry no degree order, as in real edge lists.
void relabel(std::vector<uint64_t>& keys, int64_t V, uint64_t seed) {
    std::vector<int64_t> perm(V);
    std::vector<uint64_t> h(V);
    for (int64_t i = 0; i < V; ++i) {
        perm[i] = i;
        h[i] = rnd(seed, 7, (uint64_t)i);
    }
    std::sort(perm.begin(), perm.end(), [&](int64_t x, int64_t y) {
        return h[x] < h[y] || (h[x] == h[y] && x < y);
    });
    std::vector<int32_t> newid(V);
    for (int64_t r = 0; r < V; ++r) newid[perm[r]] = (int32_t)r;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < (int64_t)keys.size(); ++i) {
        uint64_t u = (uint64_t)newid[keys[i] >> 32], v = (uint64_t)newid[keys[i] & 0xFFFFFFFFull];
        keys[i] = (u << 32) | v;
    }
}

Csr* make_rmat(int scale, int64_t num_edges, double a, double b, double c, uint64_t seed) {
    const int64_t V = (int64_t)1 << scale;
    std::vector<uint64_t> keys((size_t)num_edges * 2);
    const double ab = a + b, abc = a + b + c;
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < num_edges; ++e) {
        uint64_t u = 0, v = 0;
        for (int l = 0; l < scale; ++l) {
            double r = u01(rnd(seed, 1 + l, (uint64_t)e));
            uint64_t bu = 0, bv = 0;
            if (r < a) {
            } else if (r < ab) {
                bv = 1;
            } else if (r < abc) {
                bu = 1;
            } else {
                bu = 1;
                bv = 1;
            }
            u = (u << 1) | bu;
            v = (v << 1) | bv;
        }
        keys[2 * e] = (u << 32) | v;
        keys[2 * e + 1] = (v << 32) | u;
    }
    // drop self loops
    keys.erase(std::remove_if(keys.begin(), keys.end(),
                              [](uint64_t k) { return (k >> 32) == (k & 0xFFFFFFFFull); }),
               keys.end());
    relabel(keys, V, seed);
    Csr* g = new Csr;
    build_csr(keys, V, *g);
    return g;
}

// Chung-Lu multigraph model: both endpoints of every undirected edge are drawn
// independently with probability proportional to an expected-degree sequence
// w_i = (i + i0)^(-1/(gamma-1)), with i0 chosen so that the largest expected
// degree is max_expected_degree; then self loops and duplicates are removed and
// the vertices are relabelled at random.
Csr* make_chung_lu(int64_t V, int64_t num_undirected, double gamma, double max_expected_degree,
                   uint64_t seed) {
    const double alpha = 1.0 / (gamma - 1.0);
    // Bisection on log(i0): the largest expected degree 2*M*w_0/sum(w) falls as i0 grows.
    auto dmax_of = [&](double i0) {
        return 2.0 * (double)num_undirected * std::pow(i0, -alpha) / powsum(V, i0, alpha, nullptr);
    };
    double lo = 0.0, hi = std::log((double)V * 64.0);  // i0 in [1, 64 V]
    double i0 = 1.0;
    if (dmax_of(1.0) > max_expected_degree) {
        for (int iter = 0; iter < 48; ++iter) {
            double mid = 0.5 * (lo + hi);
            if (dmax_of(std::exp(mid)) > max_expected_degree) lo = mid; else hi = mid;
        }
        i0 = std::exp(hi);
    }
    std::vector<double> cum(V);
    const double s = powsum(V, i0, alpha, cum.data());
    std::vector<uint64_t> keys((size_t)num_undirected * 2);
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < num_undirected; ++e) {
        uint64_t ends[2];
        for (int k = 0; k < 2; ++k) {
            double x = u01(rnd(seed, 101 + k, (uint64_t)e)) * s;
            int64_t idx = std::upper_bound(cum.begin(), cum.end(), x) - cum.begin();
            if (idx >= V) idx = V - 1;
            ends[k] = (uint64_t)idx;
        }
        keys[2 * e] = (ends[0] << 32) | ends[1];
        keys[2 * e + 1] = (ends[1] << 32) | ends[0];
    }
    keys.erase(std::remove_if(keys.begin(), keys.end(),
                              [](uint64_t k) { return (k >> 32) == (k & 0xFFFFFFFFull); }),
               keys.end());
    relabel(keys, V, seed);
    Csr* g = new Csr;
    build_csr(keys, V, *g);
    return g;
}

}  // namespace

extern "C" {

void* gg_rmat(int scale, int64_t num_edges, double a, double b, double c, uint64_t seed) {
    if (scale < 1 || scale > 30 || num_edges < 0) return nullptr;
    return make_rmat(scale, num_edges, a, b, c, seed);
}

void* gg_chung_lu(int64_t V, int64_t num_undirected, double gamma, double max_expected_degree,
                  uint64_t seed) {
    if (V < 2 || V >= ((int64_t)1 << 31) || num_undirected < 0 || gamma <= 1.0) return nullptr;
    return make_chung_lu(V, num_undirected, gamma, max_expected_degree, seed);
}

int64_t gg_num_vertices(void* h) { return ((Csr*)h)->V; }
int64_t gg_num_entries(void* h) { return ((Csr*)h)->E; }

// Copies the CSR out.  off_is_int64 selects the width of `off` (V+1 entries).
void gg_copy(void* h, void* off, int off_is_int64, int32_t* col) {
    Csr* g = (Csr*)h;
    if (off_is_int64) {
        std::memcpy(off, g->off.data(), sizeof(int64_t) * (g->V + 1));
    } else {
        int32_t* o = (int32_t*)off;
        for (int64_t i = 0; i <= g->V; ++i) o[i] = (int32_t)g->off[i];
    }
    std::memcpy(col, g->col.data(), sizeof(int32_t) * g->E);
}

void gg_free(void* h) { delete (Csr*)h; }

// Symmetric weights in [lo, hi): the weight of entry (u, v) is a function of
// the unordered pair {u, v} and the seed, so both directions agree.
void gg_weights(int64_t V, const int64_t* off, const int32_t* col, double lo, double hi,
                uint64_t seed, float* w) {
#pragma omp parallel for schedule(dynamic, 4096)
    for (int64_t u = 0; u < V; ++u) {
        for (int64_t e = off[u]; e < off[u + 1]; ++e) {
            uint64_t v = (uint64_t)col[e];
            uint64_t a = (uint64_t)u < v ? (uint64_t)u : v, b = (uint64_t)u < v ? v : (uint64_t)u;
            double x = lo + (hi - lo) * u01(rnd(seed, 55, (a << 32) | b));
            float f = (float)x;
            if (f >= (float)hi) f = std::nextafterf((float)hi, (float)lo);
            w[e] = f;
        }
    }
}

// Seeded permutation of [0, n) (Fisher-Yates driven by the counter mixer).
void gg_permutation(int64_t n, uint64_t seed, int32_t* out) {
    for (int64_t i = 0; i < n; ++i) out[i] = (int32_t)i;
    for (int64_t i = n - 1; i > 0; --i) {
        uint64_t r = rnd(seed, 77, (uint64_t)i);
        int64_t j = (int64_t)(((unsigned __int128)r * (uint64_t)(i + 1)) >> 64);
        int32_t t = out[i];
        out[i] = out[j];
        out[j] = t;
    }
}

}  // extern "C"
