"""nd_sample_static (the entry point that allocates nothing: its scratch is an array inside the
library) against nd_sample, through the C ABI: two calls in a row on the shared array, the
second with a smaller input, for a k-hop, a walk and a layer call; limits and errors."""
import numpy as np
import pytest
import torch

from paper_2009_06693_amd import binding as B
from paper_2009_06693_amd import inputs

pytestmark = pytest.mark.gpu


def _both(dg, app, roots_np, seed, **params):
    """Outputs of nd_sample (caller's workspace) and of nd_sample_static on the same inputs."""
    p = B.nd_params_init(**params)
    roots = torch.as_tensor(np.ascontiguousarray(roots_np, dtype=np.int32), device="cuda:0")
    s = B.Sampler(dg, app, p, int(roots.numel()))
    assert s.workspace_bytes <= B.ND_STATIC_SCRATCH_BYTES
    want = [o.clone() for o in s.run(roots, seed)]
    torch.cuda.synchronize()
    got = [torch.full_like(o, -7) for o in want]
    status = torch.full((1,), 99, dtype=torch.int32, device="cuda:0")
    print(f"[no_alloc] app={app} roots={roots.numel()} seed={seed} params={params}", flush=True)
    B.nd_sample_static(dg, app, p, roots, seed, got, status)
    torch.cuda.synchronize()
    return want, got, int(status.item())


def test_static_scratch_matches_workspace_call_twice_second_smaller():
    g = inputs.small_graph(12, 60000, seed=21)
    dg = B.nd_graph_create(g.row_offsets, g.col_indices)
    roots = inputs.permutation(g.V, 3)
    # first call: 3,000 roots, second: 700 (its data sits in the front part of what the first left)
    for n, seed in ((3000, 5), (700, 6)):
        want, got, status = _both(dg, B.ND_KHOP, roots[:n], seed, num_steps=2, fanout=[25, 10])
        assert status == 0
        for i, (a, b) in enumerate(zip(want, got)):
            assert torch.equal(a, b), f"k-hop, {n} roots, step {i}"
    for n, seed in ((4000, 7), (900, 8)):
        want, got, status = _both(dg, B.ND_DEEPWALK, roots[:n], seed, num_steps=12)
        assert status == 0
        for i, (a, b) in enumerate(zip(want, got)):
            assert torch.equal(a, b), f"walk, {n} roots, step {i}"
    for n, seed in ((64 * 40, 9), (64 * 3, 10)):
        want, got, status = _both(dg, B.ND_LAYER, roots[:n], seed, num_steps=2, fanout=[256, 256],
                                  roots_per_sample=64)
        assert status == 0
        for i, (a, b) in enumerate(zip(want, got)):
            assert torch.equal(a, b), f"layer, {n} roots, step {i}"


def test_static_scratch_reports_bad_roots_and_sample_id_base():
    g = inputs.small_graph(10, 12000, seed=11)
    dg = B.nd_graph_create(g.row_offsets, g.col_indices)
    roots = np.arange(500, dtype=np.int32)
    roots[17] = g.V + 5                                   # out of range: NULL and reported
    want, got, status = _both(dg, B.ND_KHOP, roots, 3, num_steps=2, fanout=[4, 3], sample_id_base=1000)
    assert status == 1
    for a, b in zip(want, got):
        assert torch.equal(a, b)
    assert bool((got[0][17 * 4:18 * 4] == -1).all())


def test_static_scratch_rejects_what_does_not_fit():
    g = inputs.small_graph(10, 12000, seed=11)
    dg = B.nd_graph_create(g.row_offsets, g.col_indices)
    p = B.nd_params_init(num_steps=2, fanout=[25, 10])
    n = 200_000                                           # k-hop needs about 900 B of scratch per root
    lens, wsb = B.nd_sample_query(dg, B.ND_KHOP, p, n)
    assert wsb > B.ND_STATIC_SCRATCH_BYTES
    roots = torch.zeros(n, dtype=torch.int32, device="cuda:0")
    outs = [torch.empty(1, dtype=torch.int32, device="cuda:0") for _ in lens]   # never touched
    with pytest.raises(B.NdError) as e:
        B.nd_sample_static(dg, B.ND_KHOP, p, roots, 1, outs)
    assert e.value.code == B.ND_ERR_TOO_LARGE and "ND_STATIC_SCRATCH_BYTES" in str(e.value)
    with pytest.raises(B.NdError) as e:
        B.lib().nd_sample_static.argtypes  # noqa: B018  (bound)
        B._check(B.lib().nd_sample_static(None, 0, None, None, 0, 0, None, None, None))
    assert e.value.code == B.ND_ERR_NULL_POINTER
