"""nd_sample allocates nothing and never waits for the device, so a call can be recorded into a
HIP graph and replayed, and calls with their own workspaces can run side by side on two streams.
Every replay is checked against the eager result, with eager work between the replays."""
import numpy as np
import pytest
import torch

import oracle
from paper_2009_06693_amd import binding as B
from paper_2009_06693_amd import inputs

from gpu_util import device_graph

pytestmark = pytest.mark.gpu

_small = inputs.small_graph()


@pytest.mark.parametrize("app,kw", [(B.ND_KHOP, dict(num_steps=2, fanout=[6, 5])),
                                    (B.ND_DEEPWALK, dict(num_steps=15)),                  # windows in LDS
                                    (B.ND_DEEPWALK, dict(num_steps=15, sched_window=-1)),  # GPU-wide grouping
                                    (B.ND_KHOP, dict(num_steps=2, fanout=[6, 5], sched_group_bits=6))])
def test_graph_replay_matches_eager(app, kw):
    g = _small
    dg, og = device_graph(g)
    roots_np = np.arange(g.V, dtype=np.int32)
    roots = torch.as_tensor(roots_np, device="cuda:0")
    p = B.nd_params_init(**kw)
    s = B.Sampler(dg, app, p, g.V)
    s.run(roots, 77)
    torch.cuda.synchronize()
    s.status()
    eager = [o.clone() for o in s.out]
    if app == B.ND_KHOP:
        want = [w.reshape(-1) for w in oracle.khop(og, roots_np, kw["fanout"], seed=77)]
    else:
        want = list(oracle.deepwalk(og, roots_np, kw["num_steps"], seed=77))
    for a, b in zip(eager, want):
        assert np.array_equal(a.cpu().numpy(), b)
    print(f"[graph] capturing app={app} {kw}", flush=True)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        s.run(roots, 77)
    for rep in range(3):
        for o in s.out:
            o.fill_(-9)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(eager, s.out):
            assert torch.equal(a, b), f"replay {rep} differs from the eager run"
        # eager work of the program itself between replays
        s.run(roots, 78 + rep)
        torch.cuda.synchronize()


def test_graph_replay_layer_with_large_lds():
    """A layer step with 4,096 transit slots per sample needs 96 KB of dynamic LDS; allowing that
    is done when the graph is created, so the call itself only launches and can be captured."""
    g = _small
    dg, og = device_graph(g)
    R, fan = 64, [4096, 512]                       # step 1 has n_prev = 4,096
    roots_np = inputs.permutation(g.V, 5)[:R * 6].copy()
    roots = torch.as_tensor(roots_np, device="cuda:0")
    p = B.nd_params_init(num_steps=2, fanout=fan, roots_per_sample=R)
    s = B.Sampler(dg, B.ND_LAYER, p, roots_np.size)
    print("[graph] capturing a layer call with n_prev = 4096", flush=True)
    graph = torch.cuda.CUDAGraph()            # captured before any eager layer call of this shape
    with torch.cuda.graph(graph):
        s.run(roots, 31)
    want = oracle.layer(og, roots_np, R, fan, 31)
    for rep in range(3):
        for o in s.out:
            o.fill_(-9)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for i, (o, w) in enumerate(zip(s.out, want)):
            assert np.array_equal(o.cpu().numpy(), np.asarray(w).reshape(-1)), f"replay {rep}, step {i}"
        s.run(roots, 40 + rep)
        torch.cuda.synchronize()


def test_two_streams_side_by_side():
    g = _small
    dg, og = device_graph(g)
    roots_np = np.arange(g.V, dtype=np.int32)
    roots = torch.as_tensor(roots_np, device="cuda:0")
    pa = B.nd_params_init(num_steps=2, fanout=[9, 4])
    pb = B.nd_params_init(num_steps=25)
    sa = B.Sampler(dg, B.ND_KHOP, pa, g.V)
    sb = B.Sampler(dg, B.ND_DEEPWALK, pb, g.V)
    st_a, st_b = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    for rep in range(3):
        sa.run(roots, 5 + rep, stream=st_a)
        sb.run(roots, 50 + rep, stream=st_b)
    torch.cuda.synchronize()
    want_a = oracle.khop(og, roots_np, [9, 4], seed=7)
    want_b = oracle.deepwalk(og, roots_np, 25, seed=52)
    for o, w in zip(sa.out, want_a):
        assert np.array_equal(o.cpu().numpy(), w.reshape(-1))
    for o, w in zip(sb.out, want_b):
        assert np.array_equal(o.cpu().numpy(), w)
