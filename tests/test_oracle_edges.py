"""Pins for the oracle's layer-to-layer edges (Section 4.2, "Importance Sampling":
each sample records the edges between a step's transits and the vertices the step
added).  Expected values come from a hand-worked example, from a dense adjacency
matrix built independently in numpy, and from the reduction to reading a CSR row."""
import numpy as np
import pytest

import oracle
from paper_2009_06693_amd import inputs


def _directed_graph(V, n_edges, seed):
    rng = np.random.default_rng(seed)
    pairs = {(int(u), int(v)) for u, v in rng.integers(0, V, (n_edges, 2))}
    g = inputs.from_edges(V, sorted(pairs))
    dense = np.zeros((V, V), dtype=bool)
    for u, v in pairs:
        dense[u, v] = True
    return g, dense


def test_hand_worked_example():
    # 0 -> {1, 3}, 1 -> {2}, 2 -> {}, 3 -> {0, 1}; the graph is directed on purpose
    g = inputs.from_edges(4, [(0, 1), (0, 3), (1, 2), (3, 0), (3, 1)])
    og = oracle.OracleGraph(g.row_offsets, g.col_indices)
    transits = [[0, 3, -1, 2]]
    sampled = [[1, 1, 0, 3, -1, 2]]
    row_ptr, slots = oracle.layer_edges(og, transits, sampled)
    # row of vertex 0: neighbour 1 sits in slots 0 and 1, neighbour 3 in slot 3
    # row of vertex 3: neighbour 0 sits in slot 2, neighbour 1 in slots 0 and 1
    # a NULL transit and the sink vertex 2 have empty rows; vertex 2 in slot 5 is nobody's neighbour here
    assert row_ptr.tolist() == [0, 3, 6, 6, 6]
    assert slots.tolist() == [0, 1, 3, 2, 0, 1]


def test_against_a_dense_adjacency_matrix():
    V = 37
    g, dense = _directed_graph(V, 300, seed=5)
    og = oracle.OracleGraph(g.row_offsets, g.col_indices)
    rng = np.random.default_rng(6)
    S, n_prev, m = 5, 9, 23
    transits = rng.integers(-1, V, (S, n_prev)).astype(np.int32)
    sampled = rng.integers(-1, V, (S, m)).astype(np.int32)     # many repeats: m slots, few vertices
    sampled[:, :4] = sampled[:, 4:8]                           # and forced ones
    row_ptr, slots = oracle.layer_edges(og, transits, sampled)
    pos = 0
    for b in range(S):
        for t in range(n_prev):
            assert row_ptr[b * n_prev + t] == pos
            tv = transits[b, t]
            want = []
            if tv >= 0:
                for u in range(V):                 # ascending vertex id
                    if dense[tv, u]:
                        want += [j for j in range(m) if sampled[b, j] == u]
            assert slots[pos:pos + len(want)].tolist() == want, (b, t)
            pos += len(want)
    assert row_ptr[-1] == pos == slots.size
    # the number of recorded edges is the number of ones the dense matrix holds at (transit, sampled) positions
    live_t, live_s = transits >= 0, sampled >= 0
    total = sum(int(dense[transits[b][live_t[b]]][:, sampled[b][live_s[b]]].sum()) for b in range(S))
    assert total == pos


def test_every_vertex_sampled_once_reads_back_the_adjacency_rows():
    g = inputs.small_graph(scale=8, edges=3000, seed=3)
    og = oracle.OracleGraph(g.row_offsets, g.col_indices)
    V = g.V
    transits = np.arange(V, dtype=np.int32).reshape(1, V)
    sampled = np.arange(V, dtype=np.int32).reshape(1, V)       # slot j holds vertex j
    row_ptr, slots = oracle.layer_edges(og, transits, sampled)
    assert np.array_equal(row_ptr, g.row_offsets.astype(np.int64))
    assert np.array_equal(slots, g.col_indices)


def test_slot_order_is_by_vertex_then_slot_and_samples_do_not_mix():
    g = inputs.from_edges(6, [(0, 2), (0, 4), (0, 5), (1, 4)])
    og = oracle.OracleGraph(g.row_offsets, g.col_indices)
    transits = [[0], [1]]
    sampled = [[5, 4, 2, 4, 5, 2], [5, 4, 2, 4, 5, 2]]
    row_ptr, slots = oracle.layer_edges(og, transits, sampled)
    assert row_ptr.tolist() == [0, 6, 8]
    assert slots.tolist() == [2, 5, 1, 3, 0, 4, 1, 3]


def test_out_of_range_vertices_are_refused():
    g = inputs.from_edges(3, [(0, 1)])
    og = oracle.OracleGraph(g.row_offsets, g.col_indices)
    with pytest.raises(Exception):
        oracle.layer_edges(og, [[3]], [[0]])
    with pytest.raises(Exception):
        oracle.layer_edges(og, [[0]], [[-2]])
