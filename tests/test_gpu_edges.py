"""GPU parity for the edges between consecutive layers (Section 4.2, importance
sampling): the C ABI's count + fill against the oracle, entry by entry."""
import numpy as np
import pytest
import torch

import oracle
from paper_2009_06693_amd import binding as B
from paper_2009_06693_amd import inputs

from gpu_util import device_graph

pytestmark = pytest.mark.gpu


def _compare(g, transits, sampled):
    dg, og = device_graph(g)
    t = torch.as_tensor(np.ascontiguousarray(transits, dtype=np.int32), device="cuda:0")
    v = torch.as_tensor(np.ascontiguousarray(sampled, dtype=np.int32), device="cuda:0")
    print(f"[edges] S={t.shape[0]} n_prev={t.shape[1]} m={v.shape[1]}", flush=True)
    row_ptr, slots = B.layer_edges(dg, t, v)
    torch.cuda.synchronize()
    want_ptr, want_slots = oracle.layer_edges(og, transits, sampled)
    assert np.array_equal(row_ptr.cpu().numpy(), want_ptr)
    assert np.array_equal(slots.cpu().numpy(), want_slots)
    return want_ptr


_small = inputs.small_graph()
_small64 = inputs.small_graph(scale=9, edges=9000, seed=17, int64_offsets=True)


@pytest.mark.parametrize("n_prev,m,S", [(1, 1, 1), (64, 64, 7), (64, 2048, 5), (2048, 2048, 3), (100, 777, 9),
                                        (3, 65, 300), (513, 1, 4),
                                        (2049, 2048, 2), (4200, 64, 2)])   # more than one chunk of transit slots
def test_edges_between_random_layers(n_prev, m, S):
    g = _small
    rng = np.random.default_rng(n_prev * 7919 + m)
    transits = rng.integers(-1, g.V, (S, n_prev)).astype(np.int32)
    # new vertices drawn from the transits' neighbourhoods so that edges are plentiful, with repeats
    deg = np.diff(g.row_offsets)
    pool = g.col_indices[: max(1, g.E // 3)]
    sampled = pool[rng.integers(0, pool.size, (S, m))].astype(np.int32)
    sampled[rng.random((S, m)) < 0.05] = -1
    ptr = _compare(g, transits, sampled)
    if n_prev >= 64 and m >= 64:
        assert ptr[-1] > 0


def test_edges_of_a_sampled_layer_call_with_int64_offsets():
    g = _small64
    dg, og = device_graph(g)
    S, R = 6, 16
    roots = inputs.permutation(g.V, 3)[:S * R].copy()
    p = B.nd_params_init(num_steps=2, fanout=[300, 500], roots_per_sample=R)
    r = torch.as_tensor(roots, device="cuda:0")
    s = B.Sampler(dg, B.ND_LAYER, p, S * R)
    out = s.run(r, 9)
    torch.cuda.synchronize()
    layers = [roots.reshape(S, R), out[0].cpu().numpy().reshape(S, 300), out[1].cpu().numpy().reshape(S, 500)]
    for i in range(2):
        ptr = _compare(g, layers[i], layers[i + 1])
        assert ptr[-1] >= layers[i + 1].shape[1] * S   # every drawn vertex is some transit's neighbour


def test_every_vertex_once_reads_back_the_adjacency_rows():
    g = inputs.small_graph(scale=8, edges=2500, seed=4)
    dg, _ = device_graph(g)
    V = g.V
    ids = torch.arange(V, dtype=torch.int32, device="cuda:0").reshape(1, V)
    row_ptr, slots = B.layer_edges(dg, ids, ids.clone())
    assert np.array_equal(row_ptr.cpu().numpy(), g.row_offsets.astype(np.int64))
    assert np.array_equal(slots.cpu().numpy(), g.col_indices)


@pytest.mark.parametrize("copies", [2, 9, 70, 2048])
def test_a_vertex_held_by_many_slots_gives_one_edge_per_slot(copies):
    """Runs of equal vertices of every length class: written lane by lane up to 8, by the search over
    running sums above, and more than one 64-wide group of outputs per queue drain at 70 and 2,048."""
    g = _small
    deg = np.diff(g.row_offsets)
    hub = int(np.argmax(deg))
    nbrs = g.col_indices[g.row_offsets[hub]:g.row_offsets[hub + 1]]
    m = 2048
    rng = np.random.default_rng(copies)
    sampled = rng.integers(0, g.V, (2, m)).astype(np.int32)
    sampled[0, rng.choice(m, copies, replace=False)] = nbrs[0]          # one neighbour of the hub, many times
    sampled[1, :] = nbrs[rng.integers(0, nbrs.size, m)] if copies == 2048 else sampled[1]
    transits = np.full((2, 40), hub, dtype=np.int32)
    transits[:, 1::2] = rng.integers(0, g.V, (2, 20))
    ptr = _compare(g, transits, sampled)
    assert ptr[1] - ptr[0] >= copies


@pytest.mark.parametrize("int64_offsets", [False, True])
def test_adjacency_lists_that_end_at_and_around_the_kernels_step_sizes(int64_offsets):
    """A wavefront streams a list in steps of 256 or 512 entries, 64 at a time: lists one short of,
    equal to and one past the multiples, with the vertices looked for at their very ends."""
    lengths = [1, 63, 64, 65, 255, 256, 257, 511, 512, 513, 767, 768, 1023, 1024, 1025, 1536, 2047, 2048, 2049, 4097]
    V = 5000
    rng = np.random.default_rng(77)
    edges = []
    for u, n in enumerate(lengths):
        edges += [(u, int(v)) for v in np.sort(rng.choice(V, n, replace=False))]
    g = inputs.from_edges(V, edges, int64_offsets=int64_offsets)
    transits = np.array([np.arange(len(lengths)), np.arange(len(lengths))[::-1]], dtype=np.int32)
    ends = [int(g.col_indices[g.row_offsets[u + 1] - 1]) for u in range(len(lengths))]   # the last entry of each list
    firsts = [int(g.col_indices[g.row_offsets[u]]) for u in range(len(lengths))]
    sampled = np.array([ends + firsts, rng.integers(0, V, 2 * len(lengths)).tolist()], dtype=np.int32)
    ptr = _compare(g, transits, sampled)
    assert ptr[len(lengths)] >= 2 * len(lengths) - 1     # every list holds its own first and last entry


def test_empty_and_error_cases():
    g = _small
    dg, _ = device_graph(g)
    e = torch.empty((0, 5), dtype=torch.int32, device="cuda:0")
    row_ptr, slots = B.layer_edges(dg, e, torch.empty((0, 9), dtype=torch.int32, device="cuda:0"))
    assert row_ptr.cpu().tolist() == [0] and slots.numel() == 0
    t = torch.zeros((2, 4), dtype=torch.int32, device="cuda:0")
    with pytest.raises(B.NdError) as err:
        B.layer_edges(dg, t, torch.zeros((2, B.ND_MAX_EDGE_SLOTS + 1), dtype=torch.int32, device="cuda:0"))
    assert err.value.code == B.ND_ERR_TOO_LARGE
    bad = torch.full((2, 4), g.V, dtype=torch.int32, device="cuda:0")
    with pytest.raises(B.NdError) as err:
        B.layer_edges(dg, bad, t)
    assert err.value.code == B.ND_ERR_BAD_ROOT
    # a short edge buffer is filled up to its capacity and not beyond
    rng = np.random.default_rng(1)
    tr = torch.as_tensor(rng.integers(0, g.V, (3, 50)).astype(np.int32), device="cuda:0")
    sv = torch.as_tensor(g.col_indices[rng.integers(0, g.E, (3, 400))].astype(np.int32), device="cuda:0")
    row_ptr, full = B.layer_edges(dg, tr, sv)
    assert full.numel() > 10
    short = torch.full((full.numel(),), -7, dtype=torch.int32, device="cuda:0")
    B.nd_layer_edges_fill(dg, tr, sv, row_ptr, short[: full.numel() // 2])
    torch.cuda.synchronize()
    half = full.numel() // 2
    assert torch.equal(short[:half], full[:half]) and bool((short[half:] == -7).all())


def test_edges_among_the_vertices_of_one_step():
    """Cluster-style use (Section 4.2, "Cluster Sampling": an edge is recorded when it joins two
    transits of the same step): the same array on both sides."""
    g = _small
    rng = np.random.default_rng(77)
    hubs = np.argsort(-np.diff(g.row_offsets))[:400].astype(np.int32)
    members = hubs[rng.integers(0, hubs.size, (6, 300))]
    members[rng.random(members.shape) < 0.03] = -1
    ptr = _compare(g, members, members)
    assert ptr[-1] > 0
