"""GPU parity for the per-sample record format (Section 4.1, "Output format", format 1)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2009_06693_amd import binding as B
from paper_2009_06693_amd import inputs

from gpu_util import device_graph, gpu_sample

pytestmark = pytest.mark.gpu

_small = inputs.small_graph()


def _steps_on_gpu(arrays):
    return [torch.as_tensor(np.ascontiguousarray(a, dtype=np.int32).reshape(-1), device="cuda:0") for a in arrays]


@pytest.mark.parametrize("L,S", [(1, 1), (31, 63), (32, 64), (33, 65), (100, 4096), (64, 1000), (97, 12345)])
def test_walk_records(L, S):
    rng = np.random.default_rng(L * 1000 + S)
    steps = rng.integers(-1, 1 << 30, (L, S)).astype(np.int32)
    print(f"[pack] walk L={L} S={S}", flush=True)
    got = B.nd_samples_pack(_steps_on_gpu(steps), S)
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy(), oracle.pack_samples(steps))


@pytest.mark.parametrize("widths,S", [([25, 250], 777), ([2, 1, 1, 3, 1], 1001), ([64, 2048, 2048], 9),
                                      ([1] * 40 + [5] + [1] * 3, 130)])
def test_records_of_mixed_widths(widths, S):
    rng = np.random.default_rng(sum(widths) + S)
    steps = [rng.integers(-1, 1 << 30, (S, w)).astype(np.int32) for w in widths]
    print(f"[pack] widths={widths[:6]} S={S}", flush=True)
    got = B.nd_samples_pack(_steps_on_gpu(steps), S)
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy(), oracle.pack_samples(steps))


def test_records_of_sampled_walks_and_khop():
    dg, og = device_graph(_small)
    roots = np.arange(_small.V, dtype=np.int32)
    p = B.nd_params_init(num_steps=20)
    r = torch.as_tensor(roots, device="cuda:0")
    s = B.Sampler(dg, B.ND_DEEPWALK, p, roots.size)
    out = s.run(r, 3)
    rec = B.nd_samples_pack(out, roots.size)
    torch.cuda.synchronize()
    assert np.array_equal(rec.cpu().numpy(), oracle.pack_samples(oracle.deepwalk(og, roots, 20, seed=3)))
    # every record is a path of the graph: consecutive vertices are joined by an edge
    path = rec.cpu().numpy()
    for w in (0, 5, roots.size - 1):
        prev = roots[w]
        for v in path[w]:
            if v < 0:
                break
            row = _small.col_indices[_small.row_offsets[prev]:_small.row_offsets[prev + 1]]
            assert v in row
            prev = v
    p = B.nd_params_init(num_steps=2, fanout=[5, 3])
    s = B.Sampler(dg, B.ND_KHOP, p, roots.size)
    out = s.run(r, 4)
    rec = B.nd_samples_pack(out, roots.size)
    torch.cuda.synchronize()
    assert np.array_equal(rec.cpu().numpy(), oracle.pack_samples(oracle.khop(og, roots, [5, 3], seed=4)))


def test_pack_empty_and_errors():
    e = [torch.empty(0, dtype=torch.int32, device="cuda:0")]
    assert B.nd_samples_pack(e, 0).numel() == 0
    x = [torch.zeros(10, dtype=torch.int32, device="cuda:0")]
    with pytest.raises(B.NdError) as err:
        B.nd_samples_pack(x, 3, samples=torch.zeros(30, dtype=torch.int32, device="cuda:0"))
    assert err.value.code == B.ND_ERR_BAD_ARGUMENT
