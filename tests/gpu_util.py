"""Helpers for the GPU parity tests: run one application through the C ABI and
through the oracle on the same seeded inputs."""
from __future__ import annotations

import numpy as np
import torch

import oracle
from paper_2009_06693_amd import binding as B

_graph_cache = {}


def device_graph(g):
    key = id(g)
    if key not in _graph_cache:
        _graph_cache[key] = (g, B.nd_graph_create(g.row_offsets, g.col_indices, g.weights),
                             oracle.OracleGraph(g.row_offsets, g.col_indices, g.weights))
    return _graph_cache[key][1], _graph_cache[key][2]


def gpu_sample(dg, app, roots, seed, check_status=True, **params):
    """Returns a list of numpy arrays, one per step (flat, in the ABI's layout)."""
    p = B.nd_params_init(**params)
    r = torch.as_tensor(np.ascontiguousarray(roots, dtype=np.int32), device="cuda:0")
    s = B.Sampler(dg, app, p, int(r.numel()))
    print(f"[gpu_sample] app={app} roots={r.numel()} seed={seed} params={params}", flush=True)
    out = s.run(r, seed)
    torch.cuda.synchronize()
    if check_status:
        s.status()
    res = [o.cpu().numpy().copy() for o in out]
    stats = s.stats() if p.mode == B.ND_MODE_TRANSIT_PARALLEL and app != B.ND_LAYER else None
    del s
    return res, stats


def assert_steps_equal(gpu_steps, oracle_steps, what=""):
    assert len(gpu_steps) == len(oracle_steps)
    for i, (a, b) in enumerate(zip(gpu_steps, oracle_steps)):
        b = np.asarray(b).reshape(-1)
        assert a.shape == b.shape, f"{what} step {i}: shape {a.shape} vs {b.shape}"
        if not np.array_equal(a, b):
            bad = np.flatnonzero(a != b)
            raise AssertionError(f"{what} step {i}: {bad.size} of {a.size} entries differ; first at "
                                 f"{bad[0]}: gpu {a[bad[0]]} oracle {b[bad[0]]}")
