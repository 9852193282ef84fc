"""Random walks with the grouping by transit done per window of samples inside a workgroup's
LDS (nd_params.sched_window), against the oracle: both window sizes, the GPU-wide grouping and
the sample-parallel kernel give the same bits; forced classes, the heavy-transit threshold, all
LDS staging policies, walks longer than one launch covers, ragged last windows, dead walks."""
import numpy as np
import pytest
import torch

import oracle
from paper_2009_06693_amd import binding as B
from paper_2009_06693_amd import inputs

from gpu_util import assert_steps_equal, device_graph, gpu_sample

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def small_w():
    return inputs.small_graph(10, 12000, seed=12, weighted=True)


@pytest.fixture(scope="module")
def small64():
    return inputs.small_graph(11, 30000, seed=13, int64_offsets=True)


def _roots(g, n, seed):
    r = np.random.default_rng(seed).integers(0, g.V, size=n, dtype=np.int32)
    r[::53] = -1                                           # walks that never start
    return r


@pytest.mark.parametrize("window", [256, 1024, 2048, -1])
@pytest.mark.parametrize("n", [1, 1023, 2049, 7001])
def test_windows_deepwalk_and_ppr(small_w, window, n):
    dg, og = device_graph(small_w)
    roots = _roots(small_w, n, 1)
    for weighted in (0, 1):
        want = oracle.deepwalk(og, roots, 9, seed=5, use_weights=bool(weighted))
        got, stats = gpu_sample(dg, B.ND_DEEPWALK, roots, 5, num_steps=9, use_weights=weighted, sched_window=window)
        assert_steps_equal(got, list(want), f"deepwalk window={window} n={n} weighted={weighted}")
        live = np.array([(roots >= 0).sum()] + [(w >= 0).sum() for w in want[:-1]])
        assert (stats[:, 0] == live).all()                  # live pairs of every step, summed over the windows
        assert (stats[:, 1] <= stats[:, 0]).all() and (stats[:, 1] > 0).all() == (live > 0).all()
        want = oracle.ppr(og, roots, 30, 0.08, seed=6, use_weights=bool(weighted))
        got, _ = gpu_sample(dg, B.ND_PPR, roots, 6, num_steps=30, term_prob=0.08, use_weights=weighted,
                            sched_window=window)
        assert_steps_equal(got, list(want), f"ppr window={window} n={n} weighted={weighted}")


@pytest.mark.parametrize("window", [256, 1024, 2048])
@pytest.mark.parametrize("weighted,convention,attempts", [(0, 0, 64), (1, 0, 64), (1, 1, 64), (1, 0, 0), (0, 1, 1)])
def test_windows_node2vec(small_w, window, weighted, convention, attempts):
    dg, og = device_graph(small_w)
    roots = _roots(small_w, 5000, 2)
    want = oracle.node2vec(og, roots, 8, 2.0, 0.5, seed=41, use_weights=bool(weighted), convention=convention,
                           max_attempts=attempts)
    got, _ = gpu_sample(dg, B.ND_NODE2VEC, roots, 41, num_steps=8, p=2.0, q=0.5, use_weights=weighted,
                        bias_convention=convention, n2v_max_attempts=attempts, sched_window=window)
    assert_steps_equal(got, list(want), "node2vec in windows")


@pytest.mark.parametrize("window", [256, 1024, 2048])
@pytest.mark.parametrize("R,S", [(1, 3000), (4, 2500), (100, 300)])
def test_windows_multirw(small64, window, R, S):
    dg, og = device_graph(small64)
    roots = np.random.default_rng(3).integers(0, small64.V, size=R * S, dtype=np.int32)
    roots[::97] = -1
    want = oracle.multirw(og, roots, R, 20, seed=77, sample_id_base=11)
    got, _ = gpu_sample(dg, B.ND_MULTIRW, roots, 77, num_steps=20, roots_per_sample=R, sample_id_base=11,
                        sched_window=window)
    assert_steps_equal(got, list(want), f"multirw R={R} in windows")


def test_windows_default_is_taken_and_matches_the_other_paths(small64):
    """Without scheduling overrides a walk takes the window path; GPU-wide grouping, the
    sample-parallel kernel and the oracle all agree with it."""
    dg, og = device_graph(small64)
    roots = _roots(small64, 9000, 4)
    want = oracle.deepwalk(og, roots, 11, seed=8, sample_id_base=500)
    outs = {}
    for name, kw in (("default", {}), ("global", dict(sched_window=-1)),
                     ("sp", dict(mode=B.ND_MODE_SAMPLE_PARALLEL))):
        outs[name], _ = gpu_sample(dg, B.ND_DEEPWALK, roots, 8, num_steps=11, sample_id_base=500, **kw)
        assert_steps_equal(outs[name], list(want), name)
    p = B.nd_params_init(num_steps=11)
    _, ws_default = B.nd_sample_query(dg, B.ND_DEEPWALK, p, 9000)
    p = B.nd_params_init(num_steps=11, sched_window=-1)
    _, ws_global = B.nd_sample_query(dg, B.ND_DEEPWALK, p, 9000)
    assert ws_default < ws_global                          # no pair arrays, histograms or group table


@pytest.mark.parametrize("force", [B.ND_CLASS_SUBWAVE, B.ND_CLASS_WORKGROUP])
def test_windows_forced_classes(small_w, force):
    dg, og = device_graph(small_w)
    roots = _roots(small_w, 1500, 5)
    want = oracle.deepwalk(og, roots, 5, seed=9, use_weights=True)
    for policy in (0, 1, 2):
        got, stats = gpu_sample(dg, B.ND_DEEPWALK, roots, 9, num_steps=5, use_weights=1, sched_window=1024,
                                sched_force_class=force, lds_stage_policy=policy)
        assert_steps_equal(got, list(want), f"forced class {force} policy {policy}")
        if force == B.ND_CLASS_WORKGROUP:
            assert (stats[:, 3] == stats[:, 1]).all()      # every transit served by the workgroup
            assert (stats[:, 6] > 0).all() == (policy == 2)
        else:
            assert (stats[:, 3] == 0).all()


def test_windows_heavy_transits_and_staging():
    """A hub that most walks visit: star of 1,500 leaves plus a ring over the leaves.  Walks from the
    hub form one group of thousands of pairs per window; its list fits the 2,048-entry LDS copy of a
    2,048-sample window but not the 1,024-entry one."""
    n = 1500
    edges = [(0, i) for i in range(1, n + 1)] + [(i, 0) for i in range(1, n + 1)]
    edges += [(i, i % n + 1) for i in range(1, n + 1)]
    g = inputs.from_edges(n + 1, edges)
    dg, og = device_graph(g)
    roots = np.zeros(6000, dtype=np.int32)
    roots[1::3] = np.arange(1, 2001, dtype=np.int32)[:roots[1::3].size] % n + 1
    want = oracle.deepwalk(og, roots, 6, seed=13)
    for window, staged in ((2048, True), (1024, False)):
        got, stats = gpu_sample(dg, B.ND_DEEPWALK, roots, 13, num_steps=6, sched_window=window)
        assert_steps_equal(got, list(want), f"hub, window {window}")
        assert stats[0, 3] > 0 and stats[0, 7] >= 4000     # step 0: the hub's groups went to the workgroup class
        assert (stats[0, 6] > 0) == staged and (staged or (stats[:, 6] == 0).all())
    # threshold 1: every transit with two or more pairs in a window is served by the workgroup
    got, stats = gpu_sample(dg, B.ND_DEEPWALK, roots, 13, num_steps=6, sched_window=1024, sched_sub_max=1)
    assert_steps_equal(got, list(want), "hub, threshold 1")
    assert (stats[:, 3] > 0).all() and (stats[:, 2] > 0).any()
    want = oracle.node2vec(og, roots, 6, 0.5, 2.0, seed=14)
    got, _ = gpu_sample(dg, B.ND_NODE2VEC, roots, 14, num_steps=6, p=0.5, q=2.0, sched_window=2048)
    assert_steps_equal(got, list(want), "hub, node2vec")


def test_windows_walks_longer_than_one_launch(small_w):
    """One launch covers 128 steps: longer walks continue from the previous outputs."""
    dg, og = device_graph(small_w)
    roots = _roots(small_w, 2500, 6)
    want = oracle.deepwalk(og, roots, 300, seed=15)
    got, _ = gpu_sample(dg, B.ND_DEEPWALK, roots, 15, num_steps=300)
    assert_steps_equal(got, list(want), "300 steps")
    for L in (129, 130, 257):                               # the previous transit comes from the roots, step 127, ...
        want = oracle.node2vec(og, roots, L, 2.0, 0.5, seed=16, use_weights=True)
        got, _ = gpu_sample(dg, B.ND_NODE2VEC, roots, 16, num_steps=L, p=2.0, q=0.5, use_weights=1)
        assert_steps_equal(got, list(want), f"node2vec {L} steps")
    R = 6
    r = np.random.default_rng(7).integers(0, small_w.V, size=R * 900, dtype=np.int32)
    want = oracle.multirw(og, r, R, 200, seed=17)
    got, _ = gpu_sample(dg, B.ND_MULTIRW, r, 17, num_steps=200, roots_per_sample=R)
    assert_steps_equal(got, list(want), "multirw 200 steps")
    want = oracle.ppr(og, roots, 260, 0.01, seed=18)
    got, _ = gpu_sample(dg, B.ND_PPR, roots, 18, num_steps=260, term_prob=0.01)
    assert_steps_equal(got, list(want), "ppr 260 steps")


def test_windows_bad_roots_and_rejected_combinations(small64):
    dg, og = device_graph(small64)
    roots = _roots(small64, 3000, 8)
    roots[77] = small64.V + 9
    want = oracle.deepwalk(og, roots, 4, seed=19)
    got, _ = gpu_sample(dg, B.ND_DEEPWALK, roots, 19, check_status=False, num_steps=4, sched_window=1024)
    assert_steps_equal(got, list(want), "bad root is NULL")
    p = B.nd_params_init(num_steps=4, sched_window=1024)
    s = B.Sampler(dg, B.ND_DEEPWALK, p, roots.size)
    s.run(torch.as_tensor(roots, device="cuda:0"), 19)
    with pytest.raises(B.NdError) as e:
        s.status()
    assert e.value.code == B.ND_ERR_BAD_ROOT
    for kw in (dict(sched_window=512), dict(sched_window=1024, sched_force_class=B.ND_CLASS_GRID),
               dict(sched_window=1024, sched_group_bits=4)):
        with pytest.raises(B.NdError) as e:
            B.nd_sample_query(dg, B.ND_DEEPWALK, B.nd_params_init(num_steps=4, **kw), 100)
        assert e.value.code == B.ND_ERR_BAD_ARGUMENT
    with pytest.raises(B.NdError):
        B.nd_sample_query(dg, B.ND_KHOP, B.nd_params_init(num_steps=1, fanout=[3], sched_window=1024), 100)
