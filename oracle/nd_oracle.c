/*
 * CPU oracle for graph sampling in the "sample by sample" form.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow,
 * single-threaded statement of what the sampling applications of the paper
 * (Section 3, "An Abstraction for Graph Sampling", and Section 4.2, "Use
 * Cases") compute, written as the definition:
 *
 *     for every sample s:  for every step i:  for every slot j:  draw
 *
 * Grouping samples by transit vertex (Section 5.2) changes which thread makes
 * a draw and when, not what is drawn, so when every random number is a pure
 * function of (seed, sample, step, slot, attempt) the transit-parallel result
 * equals this loop nest exactly.  The GPU library shares no code with this
 * file; only tests, the smoke check and the benchmark's CPU-baseline leg may
 * call it.
 *
 * Conventions fixed here because the paper leaves them open (each is listed
 * with its reason in the design notes):
 *   - random numbers: Philox4x32-10 (Salmon et al., SC'11), key = the two
 *     halves of the 64-bit seed, counter = (sample id, slot, step, attempt);
 *   - uniform index in [0, d): high 32 bits of R0 * d;
 *   - float edge weights are quantised once to Q16 integers, and every later
 *     comparison is integer;
 *   - NULL vertex = -1; a NULL or dead-end transit yields NULL from then on.
 *
 * Parity pins: every function below is pinned by tests/test_oracle_*.py
 * (known-answer vectors, closed-form probabilities, brute-force enumeration,
 * hand-worked walks, reductions between applications).  The paper prints no
 * sampled outputs, so agreement with the authors' own implementation is
 * "parity unpinned".
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>

#define NDO_NULL (-1)
#define NDO_ONE_Q16 65536u

typedef struct ndo_graph {
    int64_t V, E;
    int64_t* off;    /* V+1 row offsets */
    int32_t* col;    /* E neighbours, each row ascending */
    uint32_t* wq;    /* E quantised weights, or NULL when the graph has none */
    uint64_t* cumq;  /* E inclusive running sums of wq inside each row, or NULL */
    uint32_t* maxwq; /* V largest wq of each row (0 for empty rows), or NULL */
} ndo_graph;

/* ------------------------------------------------------------------------ */
/* Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as   */
/* easy as 1, 2, 3", SC'11): ten rounds of two 32x32->64 multiplications     */
/* with a Weyl key schedule.                                                 */
/* ------------------------------------------------------------------------ */
void ndo_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* One generator call for (sample id, slot, step, attempt) under a 64-bit seed. */
static void draw4(uint64_t seed, uint32_t sample_id, uint32_t slot, uint32_t step,
                  uint32_t attempt, uint32_t r[4]) {
    uint32_t ctr[4] = {sample_id, slot, step, attempt};
    uint32_t key[2] = {(uint32_t)(seed & 0xFFFFFFFFu), (uint32_t)(seed >> 32)};
    ndo_philox4x32_10(ctr, key, r);
}

uint64_t ndo_mulhi64(uint64_t a, uint64_t b) {
    return (uint64_t)(((unsigned __int128)a * b) >> 64);
}

/* Uniform index in [0, d), d >= 1: floor(r * d / 2^32). */
uint32_t ndo_uniform_index(uint32_t r, uint32_t d) {
    return (uint32_t)(((uint64_t)r * d) >> 32);
}

/* ------------------------------------------------------------------------ */
/* Graph: CSR plus, for weighted graphs, what the paper's Vertex class       */
/* offers (Section 4.1): the largest edge weight and the running sum of the  */
/* edge weights of every vertex, here on Q16 integers.                       */
/* ------------------------------------------------------------------------ */
void ndo_graph_destroy(ndo_graph* g) {
    if (!g) return;
    free(g->off); free(g->col); free(g->wq); free(g->cumq); free(g->maxwq);
    free(g);
}

ndo_graph* ndo_graph_create(int64_t V, int64_t E, const int64_t* off, const int32_t* col,
                            const float* w) {
    ndo_graph* g = (ndo_graph*)calloc(1, sizeof(ndo_graph));
    if (!g) return NULL;
    g->V = V; g->E = E;
    g->off = (int64_t*)malloc(sizeof(int64_t) * (size_t)(V + 1));
    g->col = (int32_t*)malloc(sizeof(int32_t) * (size_t)(E > 0 ? E : 1));
    if (!g->off || !g->col) { ndo_graph_destroy(g); return NULL; }
    memcpy(g->off, off, sizeof(int64_t) * (size_t)(V + 1));
    if (E > 0) memcpy(g->col, col, sizeof(int32_t) * (size_t)E);
    if (w) {
        g->wq = (uint32_t*)malloc(sizeof(uint32_t) * (size_t)(E > 0 ? E : 1));
        g->cumq = (uint64_t*)malloc(sizeof(uint64_t) * (size_t)(E > 0 ? E : 1));
        g->maxwq = (uint32_t*)calloc((size_t)(V > 0 ? V : 1), sizeof(uint32_t));
        if (!g->wq || !g->cumq || !g->maxwq) { ndo_graph_destroy(g); return NULL; }
        for (int64_t v = 0; v < V; ++v) {
            uint64_t run = 0;
            uint32_t mx = 0;
            for (int64_t e = off[v]; e < off[v + 1]; ++e) {
                uint32_t q = (uint32_t)floor((double)w[e] * 65536.0 + 0.5);
                g->wq[e] = q;
                run += q;
                g->cumq[e] = run;
                if (q > mx) mx = q;
            }
            g->maxwq[v] = mx;
        }
    }
    return g;
}

static int64_t degree(const ndo_graph* g, int32_t v) { return g->off[v + 1] - g->off[v]; }

static int valid_vertex(const ndo_graph* g, int32_t v) { return v >= 0 && (int64_t)v < g->V; }

/* Weighted index by inverse transform on the row's integer running sums:
 * x = floor(r64 * total / 2^64), result = first j whose running sum exceeds x. */
int64_t ndo_weighted_index(const ndo_graph* g, int32_t v, uint32_t r0, uint32_t r1) {
    const int64_t lo = g->off[v], d = degree(g, v);
    const uint64_t total = g->cumq[lo + d - 1];
    const uint64_t x = ndo_mulhi64(((uint64_t)r0 << 32) | r1, total);
    for (int64_t j = 0; j < d; ++j)
        if (g->cumq[lo + j] > x) return j;
    return d - 1; /* not reached: x < total */
}

/* 1 if u is in the (ascending) row of t. */
static int has_edge(const ndo_graph* g, int32_t t, int32_t u) {
    for (int64_t e = g->off[t]; e < g->off[t + 1]; ++e)
        if (g->col[e] == u) return 1;
    return 0;
}

/* ------------------------------------------------------------------------ */
/* DeepWalk (Section 3, "Random walks"): a fixed-length static walk; one new */
/* vertex per step, a neighbour of the previous vertex chosen uniformly or   */
/* in proportion to the edge weight.  out[i*S + s] is the vertex walk s adds */
/* at step i.                                                                */
/* ------------------------------------------------------------------------ */
int ndo_deepwalk(const ndo_graph* g, int use_weights, const int32_t* roots, int64_t S,
                 uint64_t sample_id_base, uint64_t seed, int32_t L, int32_t* out) {
    if (use_weights && !g->wq) return -1;
    for (int64_t s = 0; s < S; ++s) {
        int32_t v = valid_vertex(g, roots[s]) ? roots[s] : NDO_NULL;
        for (int32_t i = 0; i < L; ++i) {
            int32_t next = NDO_NULL;
            if (v != NDO_NULL && degree(g, v) > 0) {
                uint32_t r[4];
                draw4(seed, (uint32_t)(sample_id_base + (uint64_t)s), 0u, (uint32_t)i, 0u, r);
                int64_t j = use_weights ? ndo_weighted_index(g, v, r[0], r[1])
                                        : (int64_t)ndo_uniform_index(r[0], (uint32_t)degree(g, v));
                next = g->col[g->off[v] + j];
            }
            out[(int64_t)i * S + s] = next;
            v = next;
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Personalised PageRank walk (Section 3): a variable-length static walk     */
/* that ends with a user-given probability at every step; the paper's        */
/* unbounded step count is replaced by the cap L.  The coin (R3 of the same  */
/* generator call as the draw) is tossed before the draw; a walk that ended  */
/* adds NULL at this and every later step.                                   */
/* ------------------------------------------------------------------------ */
int ndo_ppr(const ndo_graph* g, int use_weights, double term_prob, const int32_t* roots, int64_t S,
            uint64_t sample_id_base, uint64_t seed, int32_t L, int32_t* out) {
    if (use_weights && !g->wq) return -1;
    if (!(term_prob >= 0.0) || term_prob > 1.0) return -2;
    const uint64_t thr = (uint64_t)floor(term_prob * 4294967296.0);
    for (int64_t s = 0; s < S; ++s) {
        int32_t v = valid_vertex(g, roots[s]) ? roots[s] : NDO_NULL;
        for (int32_t i = 0; i < L; ++i) {
            int32_t next = NDO_NULL;
            if (v != NDO_NULL && degree(g, v) > 0) {
                uint32_t r[4];
                draw4(seed, (uint32_t)(sample_id_base + (uint64_t)s), 0u, (uint32_t)i, 0u, r);
                if ((uint64_t)r[3] >= thr) { /* walk goes on */
                    int64_t j = use_weights ? ndo_weighted_index(g, v, r[0], r[1])
                                            : (int64_t)ndo_uniform_index(r[0], (uint32_t)degree(g, v));
                    next = g->col[g->off[v] + j];
                }
            }
            out[(int64_t)i * S + s] = next;
            v = next;
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------ */
/* node2vec (Section 4.2): a second-order walk.  With t the transit of the   */
/* previous step and v the current one, edge (v,u) has weight                */
/* w(v,u) * bias, bias = b_ret if u == t, b_com if u is a neighbour of t,    */
/* b_far otherwise; the next vertex is found by rejection sampling under the */
/* envelope maxEdgeWeight(v) * max bias: propose an edge uniformly, accept   */
/* with probability (its weight) / envelope.  After max_attempts rejections  */
/* an exact inverse-transform draw over all biased weights is made instead.  */
/* The first step has no t and uses bias 1 for every edge.                   */
/* b_ret, b_com, b_far are Q16 integers.                                     */
/* ------------------------------------------------------------------------ */
static uint32_t n2v_edge_weight(const ndo_graph* g, int use_weights, int64_t e) {
    return use_weights ? g->wq[e] : NDO_ONE_Q16;
}

static uint64_t n2v_biased_weight(const ndo_graph* g, int use_weights, int has_t, int32_t t,
                                  int64_t e, uint32_t b_ret, uint32_t b_com, uint32_t b_far) {
    const int32_t u = g->col[e];
    uint32_t bias;
    if (!has_t) bias = NDO_ONE_Q16;
    else if (u == t) bias = b_ret;
    else if (has_edge(g, t, u)) bias = b_com;
    else bias = b_far;
    return (uint64_t)n2v_edge_weight(g, use_weights, e) * bias;
}

int ndo_node2vec_q16(const ndo_graph* g, int use_weights, uint32_t b_ret, uint32_t b_com,
                     uint32_t b_far, int32_t max_attempts, const int32_t* roots, int64_t S,
                     uint64_t sample_id_base, uint64_t seed, int32_t L, int32_t* out) {
    if (use_weights && !g->wq) return -1;
    uint32_t b_max = b_ret;
    if (b_com > b_max) b_max = b_com;
    if (b_far > b_max) b_max = b_far;
    for (int64_t s = 0; s < S; ++s) {
        const uint32_t sid = (uint32_t)(sample_id_base + (uint64_t)s);
        int32_t t = NDO_NULL; /* transit of the previous step */
        int32_t v = valid_vertex(g, roots[s]) ? roots[s] : NDO_NULL;
        for (int32_t i = 0; i < L; ++i) {
            int32_t next = NDO_NULL;
            if (v != NDO_NULL && degree(g, v) > 0) {
                const int has_t = (i > 0);
                const int64_t lo = g->off[v], d = degree(g, v);
                const uint32_t maxw = use_weights ? g->maxwq[v] : NDO_ONE_Q16;
                const uint64_t envelope = (uint64_t)maxw * (has_t ? b_max : NDO_ONE_Q16);
                int accepted = 0;
                for (int32_t a = 0; a < max_attempts && !accepted; ++a) {
                    uint32_t r[4];
                    draw4(seed, sid, 0u, (uint32_t)i, (uint32_t)a, r);
                    const int64_t e = lo + ndo_uniform_index(r[0], (uint32_t)d);
                    const uint64_t y = ndo_mulhi64(((uint64_t)r[1] << 32) | r[2], envelope);
                    const uint64_t T = n2v_biased_weight(g, use_weights, has_t, t, e, b_ret, b_com, b_far);
                    if (y < T) { next = g->col[e]; accepted = 1; }
                }
                if (!accepted) {
                    uint32_t r[4];
                    draw4(seed, sid, 0u, (uint32_t)i, (uint32_t)max_attempts, r);
                    uint64_t Z = 0;
                    for (int64_t e = lo; e < lo + d; ++e)
                        Z += n2v_biased_weight(g, use_weights, has_t, t, e, b_ret, b_com, b_far);
                    const uint64_t x = ndo_mulhi64(((uint64_t)r[0] << 32) | r[1], Z);
                    uint64_t run = 0;
                    for (int64_t e = lo; e < lo + d; ++e) {
                        run += n2v_biased_weight(g, use_weights, has_t, t, e, b_ret, b_com, b_far);
                        if (run > x) { next = g->col[e]; break; }
                    }
                }
            }
            out[(int64_t)i * S + s] = next;
            t = v;
            v = next;
        }
    }
    return 0;
}

/* Q16 bias: floor(x * 2^16 + 0.5); 0 when outside [1, 2^24] (caller rejects). */
uint32_t ndo_q16(double x) {
    double q = floor(x * 65536.0 + 0.5);
    if (!(q >= 1.0) || q > 16777216.0) return 0;
    return (uint32_t)q;
}

/* convention 0: node2vec as defined by its authors (return 1/p, common
 * neighbour 1, farther 1/q).  convention 1: the three cases as Section 4.2 of
 * the paper words them (u == t: p; neighbour of t: 1/q; otherwise 1). */
int ndo_node2vec(const ndo_graph* g, int use_weights, double p, double q, int convention,
                 int32_t max_attempts, const int32_t* roots, int64_t S, uint64_t sample_id_base,
                 uint64_t seed, int32_t L, int32_t* out) {
    uint32_t b_ret, b_com, b_far;
    if (convention == 0) { b_ret = ndo_q16(1.0 / p); b_com = ndo_q16(1.0); b_far = ndo_q16(1.0 / q); }
    else if (convention == 1) { b_ret = ndo_q16(p); b_com = ndo_q16(1.0 / q); b_far = ndo_q16(1.0); }
    else return -3;
    if (!b_ret || !b_com || !b_far || max_attempts < 0) return -2;
    return ndo_node2vec_q16(g, use_weights, b_ret, b_com, b_far, max_attempts, roots, S,
                            sample_id_base, seed, L, out);
}

/* ------------------------------------------------------------------------ */
/* MultiDimensional random walk (Section 3; Section 4.2, figure "Multi       */
/* Dimensional Random Walk"): a sample owns R root vertices.  At every step  */
/* stepTransits picks one of them uniformly, next adds a uniform neighbour   */
/* of the picked root to the sample, and that neighbour takes the picked     */
/* root's place.  Both choices come from the step's single generator call:   */
/* the root index from R2, the neighbour index from R0.  A picked root that  */
/* is NULL or has no out-edge adds NULL and leaves the roots as they are.    */
/* roots: S*R vertices (sample-major); out[i*S + s] as for the other walks.  */
/* ------------------------------------------------------------------------ */
int ndo_multirw(const ndo_graph* g, int32_t R, const int32_t* roots, int64_t S,
                uint64_t sample_id_base, uint64_t seed, int32_t L, int32_t* out) {
    if (R < 1) return -2;
    int32_t* cur = (int32_t*)malloc(sizeof(int32_t) * (size_t)R);
    if (!cur) return -5;
    for (int64_t s = 0; s < S; ++s) {
        for (int32_t k = 0; k < R; ++k) {
            const int32_t v = roots[s * R + k];
            cur[k] = valid_vertex(g, v) ? v : NDO_NULL;
        }
        for (int32_t i = 0; i < L; ++i) {
            uint32_t r[4];
            draw4(seed, (uint32_t)(sample_id_base + (uint64_t)s), 0u, (uint32_t)i, 0u, r);
            const uint32_t pick = ndo_uniform_index(r[2], (uint32_t)R);
            const int32_t t = cur[pick];
            int32_t next = NDO_NULL;
            if (t != NDO_NULL && degree(g, t) > 0) {
                next = g->col[g->off[t] + ndo_uniform_index(r[0], (uint32_t)degree(g, t))];
                cur[pick] = next;
            }
            out[(int64_t)i * S + s] = next;
        }
    }
    free(cur);
    return 0;
}

/* ------------------------------------------------------------------------ */
/* k-hop neighbourhood sampling (Section 3; GraphSAGE's 2-hop sampler in     */
/* Section 4.2): at step i every vertex added at step i-1 (the root at step  */
/* 0) is a transit and contributes fanout[i] neighbours drawn uniformly and  */
/* independently (with replacement).  Step i of sample s fills slots         */
/* j in [0, W_i), W_i = fanout[0]*...*fanout[i]; slot j descends from slot   */
/* j / fanout[i] of step i-1.  The steps are laid end to end in `out`:       */
/* step i starts at S * (W_0 + ... + W_{i-1}) and holds out_i[s*W_i + j].    */
/* ------------------------------------------------------------------------ */
int ndo_khop(const ndo_graph* g, const int32_t* fanout, int32_t k, const int32_t* roots, int64_t S,
             uint64_t sample_id_base, uint64_t seed, int32_t* out) {
    int64_t step_base = 0, W_prev = 1;
    const int32_t* prev = NULL;
    for (int32_t i = 0; i < k; ++i) {
        const int64_t m = fanout[i];
        if (m < 1) return -2;
        const int64_t W = W_prev * m;
        int32_t* cur = out + step_base;
        for (int64_t s = 0; s < S; ++s) {
            for (int64_t j = 0; j < W; ++j) {
                int32_t parent;
                if (i == 0) parent = valid_vertex(g, roots[s]) ? roots[s] : NDO_NULL;
                else parent = prev[s * W_prev + j / m];
                int32_t next = NDO_NULL;
                if (parent != NDO_NULL && degree(g, parent) > 0) {
                    uint32_t r[4];
                    draw4(seed, (uint32_t)(sample_id_base + (uint64_t)s), (uint32_t)j, (uint32_t)i, 0u, r);
                    next = g->col[g->off[parent] + ndo_uniform_index(r[0], (uint32_t)degree(g, parent))];
                }
                cur[s * W + j] = next;
            }
        }
        prev = cur;
        step_base += S * W;
        W_prev = W;
    }
    return 0;
}

/* ------------------------------------------------------------------------ */
/* k-hop sampling with unique neighbours (Section 6.3): within one sample and */
/* one step no vertex may appear twice.  Round 0 is the ordinary step (every  */
/* slot with a live parent draws, attempt 0).  Duplicates are then removed:   */
/* among slots holding the same vertex the lowest slot keeps it.  The slots   */
/* that lost draw again from their own parent (attempt 1, 2, ... - the        */
/* paper's sample-parallel refill), and a new candidate is accepted only if   */
/* no slot already holds its vertex, lower slots first.  After `rounds`       */
/* rounds a slot that is still open gets NULL.  Layout as ndo_khop.           */
/* ------------------------------------------------------------------------ */
int ndo_khop_unique(const ndo_graph* g, const int32_t* fanout, int32_t k, int32_t rounds,
                    const int32_t* roots, int64_t S, uint64_t sample_id_base, uint64_t seed,
                    int32_t* out) {
    if (rounds < 1) return -2;
    int64_t step_base = 0, W_prev = 1;
    const int32_t* prev = NULL;
    for (int32_t i = 0; i < k; ++i) {
        const int64_t m = fanout[i];
        if (m < 1) return -2;
        const int64_t W = W_prev * m;
        int32_t* cur = out + step_base;
        char* open = (char*)malloc((size_t)W);
        if (!open) return -5;
        for (int64_t s = 0; s < S; ++s) {
            int32_t* row = cur + s * W;
            for (int64_t j = 0; j < W; ++j) {
                const int32_t parent = i == 0 ? (valid_vertex(g, roots[s]) ? roots[s] : NDO_NULL)
                                              : prev[s * W_prev + j / m];
                row[j] = NDO_NULL;
                open[j] = parent != NDO_NULL && degree(g, parent) > 0;
            }
            for (int32_t r = 0; r < rounds; ++r) {
                for (int64_t j = 0; j < W; ++j) {  /* lower slots first */
                    if (!open[j]) continue;
                    const int32_t parent = i == 0 ? roots[s] : prev[s * W_prev + j / m];
                    uint32_t rn[4];
                    draw4(seed, (uint32_t)(sample_id_base + (uint64_t)s), (uint32_t)j, (uint32_t)i,
                          (uint32_t)r, rn);
                    const int32_t cand =
                        g->col[g->off[parent] + ndo_uniform_index(rn[0], (uint32_t)degree(g, parent))];
                    int taken = 0;
                    for (int64_t q = 0; q < W && !taken; ++q)
                        if (row[q] == cand) taken = 1;
                    if (!taken) {
                        row[j] = cand;
                        open[j] = 0;
                    }
                }
            }
        }
        free(open);
        prev = cur;
        step_base += S * W;
        W_prev = W;
    }
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Layer sampling with LADIES-style importance weights (Section 3, "Layer    */
/* Sampling"; Section 4.2, "Importance Sampling"): collective transit        */
/* sampling.  At step i a sample draws fanout[i] vertices from the combined  */
/* neighbourhood of all its transits, i.e. the concatenation, in slot order, */
/* of the adjacency lists of the vertices it added at step i-1 (its roots at */
/* step 0; NULL entries contribute nothing; repeated transits repeat their   */
/* lists).  An entry that comes from transit v carries weight                */
/* c(v) = floor(2^48 / deg(v)^2), the fixed-point form of the squared entry  */
/* 1/deg(v)^2 of the row-normalised adjacency matrix, so a vertex u is drawn */
/* with probability proportional to the sum of c(v) over the transit rows    */
/* that contain u: the squared norm of u's column restricted to those rows.  */
/* The draw is an inverse transform over the concatenation:                  */
/* x = floor(r64 * total / 2^64), total = sum over transits of deg*c.        */
/* Samples are batches of roots_per_sample roots; step i writes              */
/* out_i[b*fanout[i] + j], steps laid end to end.                            */
/* ------------------------------------------------------------------------ */
int ndo_layer(const ndo_graph* g, int32_t roots_per_sample, const int32_t* fanout, int32_t k,
              const int32_t* roots, int64_t num_samples, uint64_t sample_id_base, uint64_t seed,
              int32_t* out) {
    int64_t step_base = 0;
    const int32_t* prev = roots;
    int64_t n_prev = roots_per_sample;
    for (int32_t i = 0; i < k; ++i) {
        const int64_t m = fanout[i];
        if (m < 1) return -2;
        int32_t* cur = out + step_base;
        for (int64_t b = 0; b < num_samples; ++b) {
            const int32_t* transits = prev + b * n_prev;
            uint64_t total = 0;
            for (int64_t t = 0; t < n_prev; ++t) {
                const int32_t v = transits[t];
                if (!valid_vertex(g, v)) continue;
                const uint64_t d = (uint64_t)degree(g, v);
                if (d == 0) continue;
                if (d >= (1u << 24)) return -4;
                total += d * ((((uint64_t)1) << 48) / (d * d));
            }
            for (int64_t j = 0; j < m; ++j) {
                int32_t next = NDO_NULL;
                if (total > 0) {
                    uint32_t r[4];
                    draw4(seed, (uint32_t)(sample_id_base + (uint64_t)b), (uint32_t)j, (uint32_t)i, 0u, r);
                    const uint64_t x = ndo_mulhi64(((uint64_t)r[0] << 32) | r[1], total);
                    uint64_t before = 0; /* mass of the lists in front of the current one */
                    for (int64_t t = 0; t < n_prev; ++t) {
                        const int32_t v = transits[t];
                        if (!valid_vertex(g, v)) continue;
                        const uint64_t d = (uint64_t)degree(g, v);
                        if (d == 0) continue;
                        const uint64_t c = (((uint64_t)1) << 48) / (d * d);
                        if (before + d * c > x) {
                            next = g->col[g->off[v] + (int64_t)((x - before) / c)];
                            break;
                        }
                        before += d * c;
                    }
                }
                cur[b * m + j] = next;
            }
        }
        prev = cur;
        n_prev = m;
        step_base += num_samples * m;
    }
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Layer sampling with the graph's own edge weights: an entry of the         */
/* combined neighbourhood that comes from transit v and points to u carries  */
/* the quantised weight w_q(v,u), so u is drawn with probability             */
/* proportional to the sum of w(v,u) over the transit rows that contain u.   */
/* With w(v,u) = 1 / (deg(v) deg(u)) this is the squared column norm of the  */
/* symmetrically normalised adjacency matrix restricted to the transit rows  */
/* (the LADIES criterion; Section 4.2 leaves the criterion to `next`).       */
/* Same inverse transform as above: x = floor(r64 * total / 2^64), total =   */
/* sum over transits of the row's weight sum; inside the chosen row the      */
/* first entry whose running sum exceeds what is left of x.                  */
/* ------------------------------------------------------------------------ */
int ndo_layer_weighted(const ndo_graph* g, int32_t roots_per_sample, const int32_t* fanout, int32_t k,
                       const int32_t* roots, int64_t num_samples, uint64_t sample_id_base,
                       uint64_t seed, int32_t* out) {
    if (!g->cumq) return -5;
    int64_t step_base = 0;
    const int32_t* prev = roots;
    int64_t n_prev = roots_per_sample;
    for (int32_t i = 0; i < k; ++i) {
        const int64_t m = fanout[i];
        if (m < 1) return -2;
        int32_t* cur = out + step_base;
        for (int64_t b = 0; b < num_samples; ++b) {
            const int32_t* transits = prev + b * n_prev;
            uint64_t total = 0;
            for (int64_t t = 0; t < n_prev; ++t) {
                const int32_t v = transits[t];
                if (!valid_vertex(g, v) || degree(g, v) == 0) continue;
                total += g->cumq[g->off[v + 1] - 1];
            }
            for (int64_t j = 0; j < m; ++j) {
                int32_t next = NDO_NULL;
                if (total > 0) {
                    uint32_t r[4];
                    draw4(seed, (uint32_t)(sample_id_base + (uint64_t)b), (uint32_t)j, (uint32_t)i, 0u, r);
                    const uint64_t x = ndo_mulhi64(((uint64_t)r[0] << 32) | r[1], total);
                    uint64_t before = 0; /* weight of the lists in front of the current one */
                    for (int64_t t = 0; t < n_prev && next == NDO_NULL; ++t) {
                        const int32_t v = transits[t];
                        if (!valid_vertex(g, v) || degree(g, v) == 0) continue;
                        const uint64_t row = g->cumq[g->off[v + 1] - 1];
                        if (before + row > x) {
                            for (int64_t e = g->off[v]; e < g->off[v + 1]; ++e)
                                if (g->cumq[e] > x - before) { next = g->col[e]; break; }
                        }
                        before += row;
                    }
                }
                cur[b * m + j] = next;
            }
        }
        prev = cur;
        n_prev = m;
        step_base += num_samples * m;
    }
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Edges between consecutive layers (Section 4.2, "Importance Sampling": a   */
/* sample records the edges between the transit vertices of a step and the   */
/* vertices the step adds).  For sample b, transit slot t and new slot j the */
/* edge (t, j) exists when both slots hold a vertex and sampled[b][j] is in  */
/* the adjacency list of transits[b][t].  The result is one CSR over the     */
/* rows (b, t): row_ptr has S*n_prev + 1 entries, edge_slot lists a row's j  */
/* in the order of (vertex id, j), which is the order in which a walk down   */
/* the (ascending) adjacency list meets them.  A vertex drawn into several   */
/* slots contributes each of them.  edge_slot may be NULL to count only.     */
/* ------------------------------------------------------------------------ */
typedef struct { int32_t v, j; } slot_of_vertex;

static int by_vertex_then_slot(const void* a, const void* b) {
    const slot_of_vertex *x = (const slot_of_vertex*)a, *y = (const slot_of_vertex*)b;
    if (x->v != y->v) return x->v < y->v ? -1 : 1;
    return x->j < y->j ? -1 : (x->j > y->j);
}

int ndo_layer_edges(const ndo_graph* g, const int32_t* transits, int32_t n_prev, const int32_t* sampled,
                    int32_t m, int64_t S, int64_t* row_ptr, int32_t* edge_slot, int64_t capacity) {
    if (n_prev < 1 || m < 1 || S < 0) return -1;
    slot_of_vertex* list = (slot_of_vertex*)malloc((size_t)m * sizeof(slot_of_vertex));
    if (!list) return -2;
    int64_t n_edges = 0;
    for (int64_t b = 0; b < S; ++b) {
        /* the sample's new vertices, ordered by (vertex id, slot) */
        int32_t n_list = 0;
        for (int32_t j = 0; j < m; ++j) {
            const int32_t v = sampled[b * m + j];
            if (v == NDO_NULL) continue;
            if (!valid_vertex(g, v)) { free(list); return -3; }
            list[n_list].v = v;
            list[n_list].j = j;
            ++n_list;
        }
        qsort(list, (size_t)n_list, sizeof(slot_of_vertex), by_vertex_then_slot);
        for (int32_t t = 0; t < n_prev; ++t) {
            row_ptr[b * n_prev + t] = n_edges;
            const int32_t tv = transits[b * n_prev + t];
            if (tv == NDO_NULL) continue;
            if (!valid_vertex(g, tv)) { free(list); return -3; }
            /* both lists ascend by vertex id: walk them together */
            int32_t k = 0;
            for (int64_t e = g->off[tv]; e < g->off[tv + 1]; ++e) {
                const int32_t u = g->col[e];
                while (k < n_list && list[k].v < u) ++k;
                for (int32_t kk = k; kk < n_list && list[kk].v == u; ++kk) {
                    if (edge_slot) {
                        if (n_edges >= capacity) { free(list); return -4; }
                        edge_slot[n_edges] = list[kk].j;
                    }
                    ++n_edges;
                }
            }
        }
    }
    row_ptr[S * (int64_t)n_prev] = n_edges;
    free(list);
    return 0;
}
