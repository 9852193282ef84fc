"""Pins for the oracle's k-hop and layer (collective) sampling."""
import numpy as np
import pytest
from scipy import stats

import oracle
from paper_2009_06693_amd import inputs


def _og(g):
    return oracle.OracleGraph(g.row_offsets, g.col_indices, g.weights)


def test_khop_with_unit_fanouts_is_a_uniform_walk():
    g = inputs.small_graph(8, 1500, seed=3)
    og = _og(g)
    roots = np.arange(g.V, dtype=np.int32)
    walk = oracle.deepwalk(og, roots, 6, seed=42)
    hops = oracle.khop(og, roots, [1] * 6, seed=42)
    for i in range(6):
        assert hops[i].shape == (g.V, 1)
        assert (hops[i][:, 0] == walk[i]).all()


def test_khop_shapes_parents_and_nulls():
    # 0 -> {1,2}; 1 -> {0}; 2 has no out-edges; 3 isolated
    g = inputs.from_edges(4, [(0, 1), (0, 2), (1, 0)])
    og = _og(g)
    out = oracle.khop(og, [0, 3, 1], [4, 3], seed=6)
    assert out[0].shape == (3, 4) and out[1].shape == (3, 12)
    assert set(out[0][0].tolist()) <= {1, 2}
    assert (out[0][1] == -1).all() and (out[1][1] == -1).all()   # isolated root
    assert (out[0][2] == 0).all()
    for s in range(3):
        for j in range(12):
            parent = out[0][s, j // 3]
            child = out[1][s, j]
            if parent in (-1, 2):
                assert child == -1                                   # children of NULL / dead end
            elif parent == 1:
                assert child == 0
            else:
                assert child in (1, 2)


def test_khop_single_step_is_one_hop_sampling():
    # one step of fanout m: m independent uniform neighbours of the root (MVS-style 1-hop)
    d, m, S = 5, 8, 30000
    g = inputs.from_edges(d + 1, [(0, i + 1) for i in range(d)])
    out = oracle.khop(_og(g), np.zeros(S, dtype=np.int32), [m], seed=10)[0]
    for j in range(m):
        counts = np.bincount(out[:, j], minlength=d + 1)[1:]
        assert stats.chisquare(counts).pvalue > 1e-4
    # slots of one sample are independent draws: joint of slots 0 and 1 is uniform on d*d
    joint = np.bincount((out[:, 0] - 1) * d + (out[:, 1] - 1), minlength=d * d)
    assert stats.chisquare(joint).pvalue > 1e-4


def test_khop_second_hop_marginals():
    und = [(0, 1), (0, 2), (0, 3), (1, 2), (2, 3), (3, 4), (4, 5), (1, 5), (2, 5)]
    g = inputs.from_edges(6, und + [(v, u) for u, v in und])
    og = _og(g)
    S = 20000
    out = oracle.khop(og, np.zeros(S, dtype=np.int32), [3, 4], seed=2)
    off = g.row_offsets
    parents = np.repeat(out[0], 4, axis=1)        # parent of slot j is slot j // 4
    for v in range(6):
        sel = out[1][parents == v]
        if sel.size == 0:
            continue
        nbrs = g.col_indices[off[v]:off[v + 1]]
        counts = np.array([(sel == u).sum() for u in nbrs])
        assert counts.sum() == sel.size
        assert stats.chisquare(counts).pvalue > 1e-4


def test_khop_counter_uses_the_slot_within_the_sample():
    g = inputs.small_graph(8, 1500, seed=3)
    og = _og(g)
    hub = int(np.argmax(g.degrees()))
    roots = np.array([hub, 9, hub], dtype=np.int32)
    out = oracle.khop(og, roots, [6, 2], seed=8)
    # same root, different sample id: different draws
    assert (out[0][0] != out[0][2]).any()
    # sample_id_base shifts the slice
    part = oracle.khop(og, roots[1:], [6, 2], seed=8, sample_id_base=1)
    assert (part[0] == out[0][1:]).all() and (part[1] == out[1][1:]).all()
    # draws follow the generator: slot j of step 0 of sample 0
    off = g.row_offsets
    d = int(off[hub + 1] - off[hub])
    for j in range(6):
        r0 = int(oracle.draw(8, 0, j, 0)[0])
        assert out[0][0, j] == g.col_indices[off[hub] + (r0 * d >> 32)]


# ----------------------------------------------------------------------------- layer

def _layer_graph():
    # degrees: 0:3, 1:2, 2:4, 3:1, 4:2, 5:0 (directed entries)
    edges = [(0, 1), (0, 2), (0, 4), (1, 2), (1, 3), (2, 0), (2, 1), (2, 3), (2, 5), (3, 4),
             (4, 0), (4, 5)]
    return inputs.from_edges(6, edges)


def _layer_expected(g, transits):
    """P(u) proportional to the sum over transit rows v containing u of floor(2^48/deg(v)^2)."""
    off = g.row_offsets
    mass = np.zeros(g.V)
    for v in transits:
        if v < 0:
            continue
        d = int(off[v + 1] - off[v])
        if d == 0:
            continue
        c = (1 << 48) // (d * d)
        for u in g.col_indices[off[v]:off[v + 1]]:
            mass[u] += c
    return mass / mass.sum()


def test_layer_brute_force_distribution():
    g = _layer_graph()
    og = _og(g)
    rps, m, B = 4, 50, 4000
    batch = np.array([0, 2, 3, 0], dtype=np.int32)         # repeated transit keeps both copies
    roots = np.tile(batch, B)
    out = oracle.layer(og, roots, rps, [m], seed=12)[0]
    assert out.shape == (B, m)
    prob = _layer_expected(g, batch)
    counts = np.bincount(out.reshape(-1), minlength=g.V)
    assert (counts[prob == 0] == 0).all()
    keep = prob > 0
    assert stats.chisquare(counts[keep], prob[keep] * counts.sum()).pvalue > 1e-4
    # hand check of the weights: deg 3 -> c = 2^48/9, deg 4 -> 2^48/16, deg 1 -> 2^48
    c3, c4, c1 = (1 << 48) // 9, (1 << 48) // 16, 1 << 48
    mass = np.zeros(6)
    mass[[1, 2, 4]] += 2 * c3
    mass[[0, 1, 3, 5]] += c4
    mass[4] += c1
    assert np.allclose(prob, mass / mass.sum())


def test_layer_second_step_uses_previous_layer_as_transits():
    g = _layer_graph()
    og = _og(g)
    B = 6000
    roots = np.tile(np.array([3], dtype=np.int32), B)      # 3 -> {4}: the first layer is all 4s
    out = oracle.layer(og, roots, 1, [2, 40], seed=1)
    assert (out[0] == 4).all()
    prob = _layer_expected(g, [4, 4])
    counts = np.bincount(out[1].reshape(-1), minlength=g.V)
    keep = prob > 0
    assert (counts[~keep] == 0).all()
    assert stats.chisquare(counts[keep], prob[keep] * counts.sum()).pvalue > 1e-4


def test_layer_single_transit_is_uniform_over_its_list():
    g = _layer_graph()
    out = oracle.layer(_og(g), np.full(5000, 2, dtype=np.int32), 1, [16], seed=3)[0]
    counts = np.bincount(out.reshape(-1), minlength=6)
    assert counts[[2, 4]].sum() == 0
    assert stats.chisquare(counts[[0, 1, 3, 5]]).pvalue > 1e-4


def test_layer_equal_degrees_give_uniform_over_the_concatenation():
    # 0 -> {2,3}, 1 -> {3,4}: both degree 2, so 3 is twice as likely as 2 or 4
    g = inputs.from_edges(5, [(0, 2), (0, 3), (1, 3), (1, 4)])
    out = oracle.layer(_og(g), np.tile(np.array([0, 1], dtype=np.int32), 4000), 2, [10], seed=4)[0]
    counts = np.bincount(out.reshape(-1), minlength=5)[2:]
    assert stats.chisquare(counts, np.array([0.25, 0.5, 0.25]) * counts.sum()).pvalue > 1e-4


def test_layer_exact_index_arithmetic():
    # One transit of degree 3: total = 3*c, x = floor(r64*total/2^64), index = x // c.
    g = inputs.from_edges(4, [(0, 1), (0, 2), (0, 3)])
    out = oracle.layer(_og(g), np.zeros(50, dtype=np.int32), 1, [7], seed=77)[0]
    c = (1 << 48) // 9
    for b in range(50):
        for j in range(7):
            r = oracle.draw(77, b, j, 0)
            x = ((int(r[0]) << 32 | int(r[1])) * (3 * c)) >> 64
            assert out[b, j] == 1 + x // c


def test_layer_draw_is_monotone_over_the_concatenation():
    # Inverse transform over the concatenated lists: a larger random number can never select an
    # earlier entry of the concatenation (lists in transit order, entries in adjacency order).
    g = inputs.from_edges(7, [(0, 2), (0, 3), (0, 4), (1, 5), (1, 6)])
    B_, m = 300, 16
    out = oracle.layer(_og(g), np.tile(np.array([0, 1], dtype=np.int32), B_), 2, [m], seed=9)[0]
    pos = {2: 0, 3: 1, 4: 2, 5: 3, 6: 4}
    pairs = []
    for b in range(B_):
        for j in range(m):
            r = oracle.draw(9, b, j, 0)
            pairs.append(((int(r[0]) << 32) | int(r[1]), pos[int(out[b, j])]))
    pairs.sort()
    seq = [p for _, p in pairs]
    assert all(a <= b for a, b in zip(seq, seq[1:]))
    assert set(seq) == {0, 1, 2, 3, 4}
    # mass of the first list: 3 * (1/9) against 2 * (1/4)
    first = sum(1 for p in seq if p < 3)
    assert abs(first / len(seq) - (1 / 3) / (1 / 3 + 1 / 2)) < 0.02


def test_layer_step_is_part_of_the_counter():
    """Section 3, "Layer Sampling": every step draws afresh.  A chain 0 -> {1} -> {2, 3, 4}: step 0
    can only add vertex 1, so step 1 has the single transit 1 of degree 3 and its draw j is
    adj(1)[x // c] with x from the generator call (seed, sample, slot j, step 1)."""
    g = inputs.from_edges(5, [(0, 1), (1, 2), (1, 3), (1, 4)])
    seed, base, B_, m = 41, 11, 40, 9
    out = oracle.layer(_og(g), np.zeros(B_, dtype=np.int32), 1, [1, m], seed=seed, sample_id_base=base)
    assert (out[0] == 1).all()
    c = (1 << 48) // 9
    same_as_step0 = 0
    for b in range(B_):
        for j in range(m):
            r = oracle.draw(seed, base + b, j, 1)
            x = ((int(r[0]) << 32 | int(r[1])) * (3 * c)) >> 64
            assert out[1][b, j] == 2 + x // c
            r0 = oracle.draw(seed, base + b, j, 0)
            x0 = ((int(r0[0]) << 32 | int(r0[1])) * (3 * c)) >> 64
            same_as_step0 += int(out[1][b, j] == 2 + x0 // c)
    assert same_as_step0 < 0.5 * B_ * m          # the test can tell the two calls apart


def test_weighted_layer_step_is_part_of_the_counter():
    """The same chain with edge weights: step 1's draw is the weighted-walk draw from vertex 1 with
    the random words of (seed, sample, slot j, step 1)."""
    g = inputs.from_edges(5, [(0, 1), (1, 2), (1, 3), (1, 4)], weights=[1.0, 1.0, 2.5, 4.0])
    og = _og(g)
    seed, base, B_, m = 43, 5, 40, 9
    out = oracle.layer(og, np.zeros(B_, dtype=np.int32), 1, [1, m], seed=seed, sample_id_base=base,
                       use_weights=True)
    assert (out[0] == 1).all()
    differs = 0
    for b in range(B_):
        for j in range(m):
            r = oracle.draw(seed, base + b, j, 1)
            assert out[1][b, j] == 2 + og.weighted_index(1, int(r[0]), int(r[1]))
            r0 = oracle.draw(seed, base + b, j, 0)
            differs += int(out[1][b, j] != 2 + og.weighted_index(1, int(r0[0]), int(r0[1])))
    assert differs > 0.2 * B_ * m


def test_layer_all_dead_transits_give_null():
    g = _layer_graph()
    out = oracle.layer(_og(g), np.array([5, -1, 5, 5], dtype=np.int32), 2, [3, 3], seed=1)
    assert (out[0] == -1).all() and (out[1] == -1).all()


def test_layer_sample_id_base():
    g = inputs.small_graph(8, 1500, seed=3)
    og = _og(g)
    roots = inputs.permutation(g.V, 5)[:8 * 16]
    full = oracle.layer(og, roots, 16, [32, 32], seed=5)
    part = oracle.layer(og, roots[3 * 16:6 * 16], 16, [32, 32], seed=5, sample_id_base=3)
    assert (full[0][3:6] == part[0]).all() and (full[1][3:6] == part[1]).all()


# ----------------------------------------------------------------------------- unique neighbours

def _rows_are_unique_neighbours(g, roots, out, fanout):
    off = g.row_offsets
    parent = np.asarray(roots).reshape(-1, 1)
    for i, m in enumerate(fanout):
        o = out[i]
        for s in range(o.shape[0]):
            live = o[s][o[s] >= 0]
            assert len(set(live.tolist())) == live.size                 # no vertex twice
            for j in range(o.shape[1]):
                p = int(parent[s, j // m])
                if o[s, j] >= 0:
                    assert o[s, j] in g.col_indices[off[p]:off[p + 1]]  # a neighbour of its parent
        parent = o


def test_unique_khop_invariants():
    g = inputs.small_graph(8, 1500, seed=3)
    og = _og(g)
    roots = np.arange(g.V, dtype=np.int32)
    out = oracle.khop(og, roots, [6, 4], seed=12, unique_rounds=4)
    _rows_are_unique_neighbours(g, roots, out, [6, 4])


def test_unique_equals_with_replacement_where_nothing_collides():
    g = inputs.small_graph(8, 1500, seed=3)
    og = _og(g)
    roots = np.arange(g.V, dtype=np.int32)
    plain = oracle.khop(og, roots, [5, 3], seed=13)
    uniq = oracle.khop(og, roots, [5, 3], seed=13, unique_rounds=3)
    same_rows = 0
    for s in range(g.V):
        live0 = plain[0][s][plain[0][s] >= 0]
        live1 = plain[1][s][plain[1][s] >= 0]
        if len(set(live0.tolist())) == live0.size and len(set(live1.tolist())) == live1.size:
            assert (uniq[0][s] == plain[0][s]).all() and (uniq[1][s] == plain[1][s]).all()
            same_rows += 1
    assert same_rows > 20


def test_unique_with_one_round_only_removes_duplicates():
    # no refill: the lowest slot of every repeated vertex keeps it, the others become NULL
    g = inputs.from_edges(5, [(0, 1), (0, 2), (0, 3), (0, 4)])
    og = _og(g)
    roots = np.zeros(3000, dtype=np.int32)
    plain = oracle.khop(og, roots, [4], seed=14)[0]
    uniq = oracle.khop(og, roots, [4], seed=14, unique_rounds=1)[0]
    for s in range(3000):
        seen = set()
        for j in range(4):
            v = int(plain[s, j])
            assert uniq[s, j] == (v if v not in seen else -1)
            seen.add(v)


def test_unique_refill_is_uniform_over_the_remaining_neighbours():
    # two slots from a vertex with five neighbours: ordered pairs of distinct neighbours, all 20 alike
    g = inputs.from_edges(6, [(0, i) for i in range(1, 6)])
    S = 100000
    out = oracle.khop(_og(g), np.zeros(S, dtype=np.int32), [2], seed=15, unique_rounds=12)[0]
    assert (out >= 1).all() and (out[:, 0] != out[:, 1]).all()
    code = (out[:, 0] - 1) * 5 + (out[:, 1] - 1)
    counts = np.bincount(code, minlength=25)
    keep = np.array([a != b for a in range(5) for b in range(5)])
    assert (counts[~keep] == 0).all()
    assert stats.chisquare(counts[keep]).pvalue > 1e-4
    # the refill draw of slot 1 is the generator call with the next attempt number
    off = g.row_offsets
    for s in range(200):
        a = int(out[s, 0])
        for att in range(12):
            r0 = int(oracle.draw(15, s, 1, 0, att)[0])
            cand = int(g.col_indices[off[0] + ((r0 * 5) >> 32)])
            if cand != a:
                assert out[s, 1] == cand
                break


def test_unique_sample_id_base_reproduces_a_slice():
    """Refill draws carry the sample's global id too: a call on roots[a:b] with base a is that
    slice of the call on all roots (small neighbourhoods, so that many slots do draw again)."""
    g = inputs.small_graph(7, 700, seed=4)
    og = _og(g)
    roots = np.arange(120, dtype=np.int32) % g.V
    full = oracle.khop(og, roots, [6, 4], seed=19, unique_rounds=5)
    plain = oracle.khop(og, roots, [6, 4], seed=19)
    assert (full[0] != plain[0]).any()           # the refill really ran
    part = oracle.khop(og, roots[30:90], [6, 4], seed=19, unique_rounds=5, sample_id_base=30)
    assert (full[0][30:90] == part[0]).all() and (full[1][30:90] == part[1]).all()
    shifted = oracle.khop(og, roots[30:90], [6, 4], seed=19, unique_rounds=5, sample_id_base=0)
    assert (full[0][30:90] != shifted[0]).any()


def test_unique_exhausts_small_neighbourhoods():
    # four slots from a vertex with two neighbours: both appear once, two slots stay NULL
    g = inputs.from_edges(3, [(0, 1), (0, 2)])
    out = oracle.khop(_og(g), np.zeros(500, dtype=np.int32), [4, 2], seed=16, unique_rounds=16)
    for s in range(500):
        live = sorted(int(v) for v in out[0][s] if v >= 0)
        assert live == [1, 2]
        assert (out[1][s] == -1).all()          # 1 and 2 have no out-edges; NULL parents give NULL


# ----------------------------------------------------------------------------- layer over edge weights
def _weighted_layer_graph():
    # directed, weights chosen by hand; vertex 4 is a dead end, vertex 5 is nobody's transit below
    edges = [(0, 1), (0, 2), (0, 5), (1, 0), (1, 3), (2, 1), (2, 3), (2, 4), (2, 5), (3, 2), (5, 0)]
    w = [1.0, 2.5, 4.0, 1.5, 1.5, 3.0, 1.0, 2.0, 1.25, 4.5, 2.0]
    return inputs.from_edges(6, edges, weights=w)


def test_weighted_layer_with_one_transit_is_the_weighted_walk_draw():
    """One transit per sample: the combined neighbourhood is that vertex's list, so the draw is the
    inverse-transform draw of the weighted walk (pinned on its own) with the same random words."""
    g = inputs.small_graph(8, 2000, seed=9, weighted=True)
    og = _og(g)
    roots = np.arange(g.V, dtype=np.int32)
    m = 6
    out = oracle.layer(og, roots, 1, [m], seed=77, sample_id_base=5, use_weights=True)[0]
    deg = np.diff(g.row_offsets)
    for b in range(g.V):
        for j in range(m):
            if deg[b] == 0:
                assert out[b, j] == -1
                continue
            r = oracle.draw(77, 5 + b, j, 0)
            e = og.weighted_index(b, int(r[0]), int(r[1]))
            assert out[b, j] == g.col_indices[g.row_offsets[b] + e]


def test_weighted_layer_brute_force_distribution():
    g = _weighted_layer_graph()
    og = _og(g)
    batch = np.array([0, 2, -1, 2, 4, 1], dtype=np.int32)   # a repeat, a NULL and a dead end
    m = 300000
    out = oracle.layer(og, batch, batch.size, [m], seed=31, use_weights=True)[0].reshape(-1)
    wq = np.floor(g.weights.astype(np.float64) * 65536.0 + 0.5)
    mass = np.zeros(g.V)
    for t in batch:
        if t < 0:
            continue
        for e in range(g.row_offsets[t], g.row_offsets[t + 1]):
            mass[g.col_indices[e]] += wq[e]
    prob = mass / mass.sum()
    counts = np.bincount(out, minlength=g.V)
    assert (counts[prob == 0] == 0).all() and (out >= 0).all()
    keep = prob > 0
    assert stats.chisquare(counts[keep], prob[keep] * counts.sum()).pvalue > 1e-4
    # by hand: transits 0, 2, 2, 1 contribute; vertex 3 gets 1.0 twice (from 2) and 1.5 (from 1)
    assert np.isclose(prob[3], (2 * 1.0 + 1.5) / (7.5 + 2 * 7.25 + 3.0))


def test_weighted_layer_walks_down_the_concatenation():
    """Sorted by the random number, the draws of one sample walk through the transits' lists in slot
    order and through every list from front to back."""
    g = _weighted_layer_graph()
    og = _og(g)
    batch = np.array([2, 0, 1], dtype=np.int32)
    m = 4000
    out = oracle.layer(og, batch, 3, [m], seed=8, use_weights=True)[0].reshape(-1)
    r64 = np.array([(int(oracle.draw(8, 0, j, 0)[0]) << 32) | int(oracle.draw(8, 0, j, 0)[1]) for j in range(m)],
                   dtype=np.uint64)
    seq = out[np.argsort(r64, kind="stable")]
    concat = np.concatenate([g.col_indices[g.row_offsets[t]:g.row_offsets[t + 1]] for t in batch])
    # the sorted draws, with repeats squeezed out, spell the concatenation
    squeezed = seq[np.concatenate([[True], seq[1:] != seq[:-1]])]
    assert squeezed.tolist() == concat.tolist()


def test_weighted_layer_needs_weights():
    g = inputs.small_graph(6, 200, seed=1)
    with pytest.raises(Exception):
        oracle.layer(_og(g), np.arange(8, dtype=np.int32), 4, [3], seed=1, use_weights=True)


def test_weighted_layer_boundaries_with_tiny_integer_weights():
    """Weights of 1, 2 and 1 quanta: x takes the values 0..3 with equal probability, so the three
    neighbours must come up with probabilities 1/4, 1/2, 1/4 - a draw that lands on a running sum
    belongs to the next entry."""
    q = 1.0 / 65536.0
    g = inputs.from_edges(4, [(0, 1), (0, 2), (0, 3)], weights=[q, 2 * q, q])
    og = _og(g)
    m = 200000
    out = oracle.layer(og, np.zeros(1, dtype=np.int32), 1, [m], seed=5, use_weights=True)[0].reshape(-1)
    counts = np.bincount(out, minlength=4)[1:]
    assert stats.chisquare(counts, np.array([0.25, 0.5, 0.25]) * m).pvalue > 1e-4
