"""Pins for the oracle's random walks (DeepWalk, PPR, node2vec).

Hand-worked walks, degenerate graphs, brute-force transition probabilities and
reductions between the applications.
"""
import numpy as np
import pytest
from scipy import stats

import oracle
from paper_2009_06693_amd import inputs


def _og(g):
    return oracle.OracleGraph(g.row_offsets, g.col_indices, g.weights)


def test_directed_cycle_is_deterministic():
    n = 9
    g = inputs.from_edges(n, [(i, (i + 1) % n) for i in range(n)])
    for seed in (0, 1, 2 ** 40 + 5):
        out = oracle.deepwalk(_og(g), np.arange(n), 20, seed=seed)
        for i in range(20):
            assert list(out[i]) == [(s + i + 1) % n for s in range(n)]


def test_isolated_vertex_and_dead_end():
    # 0 -> 1 -> 2, vertex 2 has no out-edges, vertex 3 is isolated.
    g = inputs.from_edges(4, [(0, 1), (1, 2)])
    out = oracle.deepwalk(_og(g), [0, 1, 2, 3], 4, seed=5)
    assert out[:, 0].tolist() == [1, 2, -1, -1]
    assert out[:, 1].tolist() == [2, -1, -1, -1]
    assert out[:, 2].tolist() == [-1, -1, -1, -1]
    assert out[:, 3].tolist() == [-1, -1, -1, -1]


def test_out_of_range_root_is_null():
    g = inputs.from_edges(3, [(0, 1), (1, 0)])
    out = oracle.deepwalk(_og(g), [-1, 3, 0], 2, seed=5)
    assert out[:, 0].tolist() == [-1, -1]
    assert out[:, 1].tolist() == [-1, -1]
    assert out[:, 2].tolist() == [1, 0]


def test_self_loop_stays_forever():
    g = inputs.from_edges(2, [(0, 0)])
    out = oracle.deepwalk(_og(g), [0], 50, seed=8)
    assert (out == 0).all()


def test_star_alternates_and_centre_is_uniform():
    leaves = 6
    edges = [(0, i) for i in range(1, leaves + 1)] + [(i, 0) for i in range(1, leaves + 1)]
    g = inputs.from_edges(leaves + 1, edges)
    S = 60000
    out = oracle.deepwalk(_og(g), np.ones(S, dtype=np.int32), 4, seed=21)
    assert (out[0] == 0).all() and (out[2] == 0).all()
    for step in (1, 3):
        counts = np.bincount(out[step], minlength=leaves + 1)[1:]
        assert counts.sum() == S
        assert stats.chisquare(counts).pvalue > 1e-4
    # the two leaf draws of one walk use different counters: not identical
    assert (out[1] != out[3]).mean() > 0.7


def _six_vertex_graph(weighted=False):
    und = [(0, 1), (0, 2), (0, 3), (1, 2), (2, 3), (3, 4), (4, 5), (1, 5), (2, 5)]
    edges = und + [(v, u) for u, v in und]
    w = None
    if weighted:
        base = [1.0, 2.0, 3.5, 1.25, 4.75, 2.0, 1.0, 3.0, 2.5]
        w = base + base
    return inputs.from_edges(6, edges, weights=w)


@pytest.mark.parametrize("weighted", [False, True])
def test_transition_matrix_brute_force(weighted):
    g = _six_vertex_graph(weighted)
    og = _og(g)
    per_root = 40000
    roots = np.repeat(np.arange(6, dtype=np.int32), per_root)
    # two steps: the second step's transition is checked conditionally on the first
    out = oracle.deepwalk(og, roots, 2, seed=77, use_weights=weighted)
    off = g.row_offsets
    for frm, to in ((roots, out[0]), (out[0], out[1])):
        for v in range(6):
            sel = to[frm == v]
            nbrs = g.col_indices[off[v]:off[v + 1]]
            counts = np.array([(sel == u).sum() for u in nbrs])
            assert counts.sum() == sel.shape[0]        # only neighbours are ever drawn
            if weighted:
                w = np.floor(g.weights[off[v]:off[v + 1]].astype(np.float64) * 65536 + 0.5)
                exp = w / w.sum() * sel.shape[0]
            else:
                exp = np.full(len(nbrs), sel.shape[0] / len(nbrs))
            assert stats.chisquare(counts, exp).pvalue > 1e-4


def test_walks_of_different_samples_and_seeds_differ():
    g = _six_vertex_graph()
    og = _og(g)
    a = oracle.deepwalk(og, np.zeros(64, dtype=np.int32), 30, seed=1)
    b = oracle.deepwalk(og, np.zeros(64, dtype=np.int32), 30, seed=2)
    assert (a != b).mean() > 0.3
    assert len({tuple(a[:, s]) for s in range(64)}) > 60


def test_sample_id_base_reproduces_a_slice():
    g = _six_vertex_graph()
    og = _og(g)
    roots = np.arange(600, dtype=np.int32) % 6
    full = oracle.deepwalk(og, roots, 10, seed=4)
    part = oracle.deepwalk(og, roots[100:250], 10, seed=4, sample_id_base=100)
    assert (full[:, 100:250] == part).all()


# ----------------------------------------------------------------------------- PPR

def test_ppr_with_zero_termination_is_deepwalk():
    g = _six_vertex_graph(True)
    og = _og(g)
    roots = np.arange(3000, dtype=np.int32) % 6
    for weighted in (False, True):
        a = oracle.deepwalk(og, roots, 25, seed=31, use_weights=weighted)
        b = oracle.ppr(og, roots, 25, 0.0, seed=31, use_weights=weighted)
        assert (a == b).all()


def test_ppr_prefix_agrees_with_deepwalk_until_termination():
    g = _six_vertex_graph()
    og = _og(g)
    roots = np.arange(6000, dtype=np.int32) % 6
    a = oracle.deepwalk(og, roots, 30, seed=13)
    b = oracle.ppr(og, roots, 30, 0.1, seed=13)
    alive = np.ones(roots.shape[0], dtype=bool)
    for i in range(30):
        alive &= b[i] >= 0
        assert (a[i][alive] == b[i][alive]).all()
        assert (b[i][~alive] == -1).all()


def test_ppr_length_is_truncated_geometric():
    # on a cycle nothing but the coin can end a walk
    n = 5
    g = inputs.from_edges(n, [(i, (i + 1) % n) for i in range(n)])
    prob, cap, S = 0.05, 40, 200000
    out = oracle.ppr(_og(g), np.zeros(S, dtype=np.int32), cap, prob, seed=17)
    length = (out >= 0).sum(axis=0)
    # once NULL always NULL
    assert ((out >= 0).cumprod(axis=0).sum(axis=0) == length).all()
    thr = np.floor(prob * 2.0 ** 32) / 2.0 ** 32
    pmf = np.array([(1 - thr) ** k * thr for k in range(cap)] + [(1 - thr) ** cap])
    counts = np.bincount(length, minlength=cap + 1)
    assert stats.chisquare(counts, pmf * S).pvalue > 1e-4


def test_ppr_coin_is_its_own_word_and_leaves_the_draw_uniform():
    """Section 3, "Random walks": the walk ends with a given probability, whatever it would have
    drawn.  The coin is word R3 of the step's generator call; the neighbour index comes from R0.
    From the centre of a star: a walk survives step 0 exactly when R3 of the call
    (seed, sample, slot 0, step 0) reaches the threshold, and among the survivors the chosen leaf
    is still uniform (a coin taken from the word that also picks the neighbour would empty the
    low-index leaves)."""
    leaves = 10
    edges = [(0, i) for i in range(1, leaves + 1)] + [(i, 0) for i in range(1, leaves + 1)]
    g = inputs.from_edges(leaves + 1, edges)
    prob, S, seed, base = 0.3, 40000, 23, 7
    thr = int(np.floor(prob * 2.0 ** 32))
    out = oracle.ppr(_og(g), np.zeros(S, dtype=np.int32), 2, prob, seed=seed, sample_id_base=base)
    for s in range(300):
        r = oracle.draw(seed, base + s, 0, 0)
        assert (out[0, s] >= 0) == (int(r[3]) >= thr)
        if out[0, s] >= 0:
            assert out[0, s] == 1 + (int(r[0]) * leaves >> 32)
            r1 = oracle.draw(seed, base + s, 0, 1)               # step 1: from the leaf back to 0
            assert (out[1, s] >= 0) == (int(r1[3]) >= thr)
    alive = out[0] >= 0
    assert abs(alive.mean() - (1 - thr / 2.0 ** 32)) < 0.01
    counts = np.bincount(out[0][alive], minlength=leaves + 1)[1:]
    assert counts.min() > 0
    assert stats.chisquare(counts).pvalue > 1e-4


def test_ppr_sample_id_base_reproduces_a_slice():
    g = _six_vertex_graph(True)
    og = _og(g)
    roots = np.arange(900, dtype=np.int32) % 6
    for weighted in (False, True):
        full = oracle.ppr(og, roots, 12, 0.15, seed=9, use_weights=weighted)
        part = oracle.ppr(og, roots[200:420], 12, 0.15, seed=9, use_weights=weighted, sample_id_base=200)
        assert (full[:, 200:420] == part).all()
        shifted = oracle.ppr(og, roots[200:420], 12, 0.15, seed=9, use_weights=weighted, sample_id_base=0)
        assert (full[:, 200:420] != shifted).any()


def test_ppr_certain_termination():
    g = _six_vertex_graph()
    out = oracle.ppr(_og(g), np.arange(6), 5, 1.0, seed=1)
    assert (out == -1).all()


# ----------------------------------------------------------------------------- node2vec

def _n2v_graph(weighted):
    # triangle 0-1-2, pendant 3 on 2, vertex 4 joined to 1 and 3 (a chord path), 5 on 0
    und = [(0, 1), (1, 2), (0, 2), (2, 3), (1, 4), (3, 4), (0, 5)]
    edges = und + [(v, u) for u, v in und]
    w = None
    if weighted:
        base = [1.0, 2.0, 4.5, 1.5, 3.0, 2.25, 1.0]
        w = base + base
    return inputs.from_edges(6, edges, weights=w)


def _n2v_expected(g, t, v, b_ret, b_com, b_far, weighted):
    off = g.row_offsets
    nbrs = g.col_indices[off[v]:off[v + 1]]
    tn = set(g.col_indices[off[t]:off[t + 1]].tolist())
    w = (np.floor(g.weights[off[v]:off[v + 1]].astype(np.float64) * 65536 + 0.5)
         if weighted else np.ones(len(nbrs)))
    bias = np.array([b_ret if u == t else (b_com if u in tn else b_far) for u in nbrs])
    p = w * bias
    return nbrs, p / p.sum()


@pytest.mark.parametrize("weighted", [False, True])
@pytest.mark.parametrize("convention", [0, 1])
@pytest.mark.parametrize("max_attempts", [64, 0, 1])
def test_node2vec_second_order_probabilities(weighted, convention, max_attempts):
    p, q = 2.0, 0.5
    g = _n2v_graph(weighted)
    og = _og(g)
    if convention == 0:
        b = (1 / p, 1.0, 1 / q)
    else:
        b = (p, 1 / q, 1.0)
    per_root = 60000
    roots = np.repeat(np.arange(6, dtype=np.int32), per_root)
    out = oracle.node2vec(og, roots, 2, p, q, seed=1234 + max_attempts, use_weights=weighted,
                          convention=convention, max_attempts=max_attempts)
    off = g.row_offsets
    # first step: bias 1 for every edge -> plain (weighted) neighbour draw
    for t in range(6):
        sel = out[0][roots == t]
        nbrs = g.col_indices[off[t]:off[t + 1]]
        counts = np.array([(sel == u).sum() for u in nbrs])
        assert counts.sum() == sel.shape[0]
        w = (np.floor(g.weights[off[t]:off[t + 1]].astype(np.float64) * 65536 + 0.5)
             if weighted else np.ones(len(nbrs)))
        if len(nbrs) > 1:
            assert stats.chisquare(counts, w / w.sum() * sel.shape[0]).pvalue > 1e-4
    # second step, conditional on (t, v)
    checked = 0
    for t in range(6):
        for v in g.col_indices[off[t]:off[t + 1]]:
            sel = out[1][(roots == t) & (out[0] == v)]
            nbrs, prob = _n2v_expected(g, t, int(v), *b, weighted)
            counts = np.array([(sel == u).sum() for u in nbrs])
            assert counts.sum() == sel.shape[0]
            if len(nbrs) > 1:
                assert stats.chisquare(counts, prob * sel.shape[0]).pvalue > 1e-4
                checked += 1
    assert checked >= 10


def test_node2vec_with_unit_biases_is_uniform_deepwalk():
    # p = q = 1 on an unweighted graph: every proposal is accepted at the first
    # attempt and the proposal index is the uniform index of DeepWalk's draw.
    g = inputs.small_graph(8, 1500, seed=3)
    og = _og(g)
    roots = np.arange(g.V, dtype=np.int32)
    a = oracle.deepwalk(og, roots, 20, seed=9)
    b = oracle.node2vec(og, roots, 20, 1.0, 1.0, seed=9)
    assert (a == b).all()


def test_node2vec_sample_id_base_reproduces_a_slice():
    g = _n2v_graph(True)
    og = _og(g)
    roots = np.arange(700, dtype=np.int32) % g.V
    for weighted, attempts in ((False, 64), (True, 64), (True, 0)):
        kw = dict(p=2.0, q=0.5, seed=14, use_weights=weighted, max_attempts=attempts)
        full = oracle.node2vec(og, roots, 9, **kw)
        part = oracle.node2vec(og, roots[150:380], 9, sample_id_base=150, **kw)
        assert (full[:, 150:380] == part).all()
        shifted = oracle.node2vec(og, roots[150:380], 9, sample_id_base=0, **kw)
        assert (full[:, 150:380] != shifted).any()


def test_node2vec_rejects_bad_parameters():
    g = _n2v_graph(False)
    with pytest.raises(ValueError):
        oracle.node2vec(_og(g), [0], 2, 1e-9, 1.0, seed=1)       # 1/p above 2^8
    with pytest.raises(ValueError):
        oracle.node2vec(_og(g), [0], 2, 2.0, 0.5, seed=1, use_weights=True)  # no weights


def test_node2vec_attempt_budget_changes_draws_not_the_law():
    g = _n2v_graph(True)
    og = _og(g)
    roots = np.zeros(4000, dtype=np.int32)
    a = oracle.node2vec(og, roots, 6, 2.0, 0.5, seed=5, use_weights=True, max_attempts=64)
    b = oracle.node2vec(og, roots, 6, 2.0, 0.5, seed=5, use_weights=True, max_attempts=2)
    assert (a != b).any()
    assert (a[0] == b[0]).mean() > 0.5   # walks accepted within two attempts agree


# ----------------------------------------------------------------------------- multi-dimensional walk

def test_multirw_with_one_root_is_uniform_deepwalk():
    # one root per sample: the pick is always that root and the new vertex replaces it,
    # which is the uniform walk, draw for draw
    g = inputs.small_graph(8, 1500, seed=3)
    og = _og(g)
    roots = np.arange(g.V, dtype=np.int32)
    assert (oracle.multirw(og, roots, 1, 15, seed=9) == oracle.deepwalk(og, roots, 15, seed=9)).all()


def test_multirw_pick_is_uniform_and_replaces_the_picked_root():
    # directed paths a -> a+1 starting at 0, 100, 200, 300: which path advanced says which
    # root was picked, and a path's next vertex says the picked root had been replaced
    n = 400
    g = inputs.from_edges(n, [(v, v + 1) for v in range(n) if v % 100 != 99])
    og = _og(g)
    S, L = 20000, 30
    roots = np.tile(np.array([0, 100, 200, 300], dtype=np.int32), S)
    out = oracle.multirw(og, roots, 4, L, seed=44)
    first = out[0] // 100
    assert stats.chisquare(np.bincount(first, minlength=4)).pvalue > 1e-4
    for s in range(200):
        pos = [0, 100, 200, 300]
        for i in range(L):
            v = int(out[i, s])
            k = v // 100
            assert v == pos[k] + 1          # the picked root is the path's current end
            pos[k] = v
        r2 = int(oracle.draw(44, s, 0, 0)[2])
        assert int(out[0, s]) // 100 == (r2 * 4) >> 32


def test_multirw_dead_pick_adds_null_and_keeps_the_roots():
    # root 1 has no out-edge, root 0 walks a cycle
    g = inputs.from_edges(4, [(0, 2), (2, 3), (3, 0)])
    out = oracle.multirw(_og(g), np.tile(np.array([0, 1], dtype=np.int32), 3000), 2, 12, seed=5)
    nulls = (out == -1)
    assert 0.4 < nulls.mean() < 0.6          # the dead root is picked half of the time, forever
    for s in range(50):
        live = [int(v) for v in out[:, s] if v >= 0]
        assert live == [[2, 3, 0][k % 3] for k in range(len(live))]


def test_multirw_sample_id_base():
    g = inputs.small_graph(8, 1500, seed=3)
    og = _og(g)
    roots = inputs.permutation(g.V, 2)[:50 * 5]
    full = oracle.multirw(og, roots, 5, 20, seed=6)
    part = oracle.multirw(og, roots[10 * 5:30 * 5], 5, 20, seed=6, sample_id_base=10)
    assert (full[:, 10:30] == part).all()
