"""Seeded random configurations against the oracle: graphs of varied shape (dead ends, self
loops, one very long row, int32 / int64 offsets, with and without weights), every application,
both modes, scheduling thresholds low enough to put transits into all three classes, prefix
grouping, split calls.  Every case prints what it is before it runs."""
import numpy as np
import pytest
import torch

import oracle
from paper_2009_06693_amd import binding as B
from paper_2009_06693_amd import inputs

from gpu_util import assert_steps_equal, gpu_sample

pytestmark = pytest.mark.gpu


def _random_graph(rng, case):
    V = int(rng.integers(2, 3000))
    n_edges = int(rng.integers(0, 20 * V))
    src = rng.integers(0, V, n_edges)
    # skewed destinations: squares concentrate on low ids
    dst = (rng.random(n_edges) ** 2 * V).astype(np.int64)
    pairs = set(zip(src.tolist(), dst.tolist()))
    if case % 3 == 0 and V > 50:                      # one row holding nearly every vertex
        hub = int(rng.integers(0, V))
        pairs |= {(hub, int(v)) for v in range(0, V, 1 + case % 2)}
        pairs |= {(int(v), hub) for v in rng.integers(0, V, 5 * V)}   # and many walkers reaching it
    if case % 4 == 1:
        pairs |= {(int(v), int(v)) for v in rng.integers(0, V, 10)}    # self loops
    weights = None
    pairs = sorted(pairs)
    if case % 2 == 0 and pairs:
        weights = (1.0 + 4.0 * rng.random(len(pairs))).astype(np.float32)
    g = inputs.from_edges(V, pairs, weights=weights, int64_offsets=bool(case % 5 == 2))
    return g


@pytest.mark.parametrize("case", range(84))
def test_random_configuration(case):
    rng = np.random.default_rng(1000 + case)
    g = _random_graph(rng, case)
    dg = B.nd_graph_create(g.row_offsets, g.col_indices, g.weights)
    og = oracle.OracleGraph(g.row_offsets, g.col_indices, g.weights)
    S = int(rng.integers(1, 6000))
    roots = rng.integers(-1, g.V, S).astype(np.int32)
    seed = int(rng.integers(0, 2**63))
    base = int(rng.integers(0, 2**31))
    sched = {}
    mode = B.ND_MODE_SAMPLE_PARALLEL if case % 6 == 5 else B.ND_MODE_TRANSIT_PARALLEL
    if mode == B.ND_MODE_TRANSIT_PARALLEL:
        if case % 3 == 1:
            sched = dict(sched_group_bits=int(rng.integers(1, 12)))
        else:
            sub = int(rng.integers(1, 200))
            sched = dict(sched_sub_max=sub, sched_wg_max=sub + int(rng.integers(0, 2000)),
                         lds_stage_policy=int(rng.integers(0, 3)))
    weighted = g.weights is not None and bool(rng.integers(0, 2))
    app = ["deepwalk", "ppr", "node2vec", "khop", "multirw", "layer", "khop_unique"][case % 7]
    print(f"[random] case={case} app={app} V={g.V} E={g.E} S={S} mode={mode} sched={sched} "
          f"weighted={weighted} base={base}", flush=True)
    common = dict(mode=mode, sample_id_base=base, **sched)
    if app == "deepwalk":
        L = int(rng.integers(1, 30))
        want = list(oracle.deepwalk(og, roots, L, seed, use_weights=weighted, sample_id_base=base))
        got, _ = gpu_sample(dg, B.ND_DEEPWALK, roots, seed, check_status=False, num_steps=L,
                            use_weights=int(weighted), **common)
    elif app == "ppr":
        L = int(rng.integers(1, 30))
        tp = float(rng.choice([0.0, 0.01, 0.3, 0.999]))
        want = list(oracle.ppr(og, roots, L, tp, seed, use_weights=weighted, sample_id_base=base))
        got, _ = gpu_sample(dg, B.ND_PPR, roots, seed, check_status=False, num_steps=L, term_prob=tp,
                            use_weights=int(weighted), **common)
    elif app == "node2vec":
        L = int(rng.integers(1, 15))
        p, q = float(rng.choice([0.25, 1.0, 2.0, 4.0])), float(rng.choice([0.25, 0.5, 1.0, 4.0]))
        conv, att = int(rng.integers(0, 2)), int(rng.choice([64, 1, 3]))
        want = list(oracle.node2vec(og, roots, L, p, q, seed, use_weights=weighted, convention=conv,
                                    max_attempts=att, sample_id_base=base))
        got, _ = gpu_sample(dg, B.ND_NODE2VEC, roots, seed, check_status=False, num_steps=L, p=p, q=q,
                            use_weights=int(weighted), bias_convention=conv, n2v_max_attempts=att, **common)
    elif app in ("khop", "khop_unique"):
        k = int(rng.integers(1, 4))
        fan = [int(rng.integers(1, 9)) for _ in range(k)]
        S = min(S, 1500)
        roots = roots[:S]
        ur = int(rng.integers(1, 5)) if app == "khop_unique" else 0
        want = [w.reshape(-1) for w in oracle.khop(og, roots, fan, seed, sample_id_base=base, unique_rounds=ur)]
        got, _ = gpu_sample(dg, B.ND_KHOP, roots, seed, check_status=False, num_steps=k, fanout=fan,
                            unique_rounds=ur, **common)
    elif app == "multirw":
        R = int(rng.integers(1, 12))
        S = max(R, S - S % R)
        roots = rng.integers(-1, g.V, S).astype(np.int32)
        L = int(rng.integers(1, 25))
        want = list(oracle.multirw(og, roots, R, L, seed, sample_id_base=base))
        got, _ = gpu_sample(dg, B.ND_MULTIRW, roots, seed, check_status=False, num_steps=L,
                            roots_per_sample=R, **common)
    else:
        R = int(rng.integers(1, 40))
        S = max(R, S - S % R)
        roots = rng.integers(-1, g.V, S).astype(np.int32)
        fan = [int(rng.integers(1, 300)) for _ in range(int(rng.integers(1, 4)))]
        want = [w.reshape(-1) for w in oracle.layer(og, roots, R, fan, seed, sample_id_base=base,
                                                    use_weights=weighted)]
        got, _ = gpu_sample(dg, B.ND_LAYER, roots, seed, check_status=False, num_steps=len(fan), fanout=fan,
                            roots_per_sample=R, sample_id_base=base, use_weights=int(weighted))
    assert_steps_equal(got, want, f"random case {case} ({app})")
