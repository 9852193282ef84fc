"""Pins for the oracle's primitives: generator, index draws, weight quantisation.

Each check compares the oracle with something fixed outside it: published
known-answer vectors, Python's exact integers, or a closed form.
"""
import math
import os

import numpy as np
import pytest
from scipy import stats

import oracle
from paper_2009_06693_amd import inputs

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _kat_rows():
    rows = []
    with open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            h = [int(x, 16) for x in line.split()]
            rows.append((h[0:4], h[4:6], h[6:10]))
    return rows


def test_philox_known_answers():
    rows = _kat_rows()
    assert len(rows) == 3
    for ctr, key, want in rows:
        assert list(oracle.philox4x32_10(ctr, key)) == want


def test_philox_is_a_bijection_of_the_counter_on_a_sample():
    # Philox is a keyed permutation of the 128-bit counter: distinct counters
    # can never collide.
    seen = set()
    for c0 in range(64):
        for c1 in range(8):
            for c2 in range(8):
                seen.add(tuple(oracle.philox4x32_10([c0, c1, c2, 0], [7, 9])))
    assert len(seen) == 64 * 8 * 8


def test_draw_counter_and_key_layout():
    # draw(seed, sample, slot, step, attempt) is the generator at counter
    # (sample, slot, step, attempt) with key (seed low, seed high).
    seed = 0x299f31d0a4093822
    got = oracle.draw(seed, 0x243f6a88, 0x85a308d3, 0x13198a2e, 0x03707344)
    assert [int(x) for x in got] == [0xd16cfe09, 0x94fdcceb, 0x5001e420, 0x24126ea1]


def test_philox_words_look_uniform():
    words = np.array([oracle.draw(1234, s, 0, 0) for s in range(20000)], dtype=np.uint64)
    for k in range(4):
        counts = np.bincount((words[:, k] >> 28).astype(np.int64), minlength=16)
        assert stats.chisquare(counts).pvalue > 1e-4
    # bits balanced
    for bit in (0, 7, 16, 31):
        ones = int(((words[:, 0] >> bit) & 1).sum())
        assert abs(ones - 10000) < 5 * math.sqrt(20000 * 0.25)


def test_mulhi64_against_exact_integers():
    rng = np.random.default_rng(5)
    vals = [0, 1, 2 ** 32, 2 ** 63, 2 ** 64 - 1] + [int(x) for x in rng.integers(0, 2 ** 63, 50)]
    for a in vals:
        for b in vals[:12]:
            assert oracle.mulhi64(a, b) == (a * b) >> 64


@pytest.mark.parametrize("d", [1, 2, 3, 7, 64, 1000, 20000, 2 ** 31 - 1])
def test_uniform_index_closed_form(d):
    # floor(r*d/2^32) takes value j exactly for r in [ceil(j*2^32/d), ceil((j+1)*2^32/d)).
    two32 = 2 ** 32
    js = sorted(j for j in {0, 1, d // 3, d // 2, d - 2, d - 1} if 0 <= j < d)
    for j in js:
        first = -((-j * two32) // d)
        last = -((-(j + 1) * two32) // d) - 1
        assert oracle.uniform_index(first, d) == j
        assert oracle.uniform_index(last, d) == j
        if first > 0:
            assert oracle.uniform_index(first - 1, d) == j - 1
    assert oracle.uniform_index(two32 - 1, d) == d - 1
    assert oracle.uniform_index(0, d) == 0


def test_q16_rounding():
    assert oracle.q16(1.0) == 65536
    assert oracle.q16(0.5) == 32768
    assert oracle.q16(2.0) == 131072
    assert oracle.q16(1.0 / 3.0) == 21845          # 21845.33 rounds down
    assert oracle.q16(2.0 / 3.0) == 43691          # 43690.67 rounds up
    assert oracle.q16(256.0) == 2 ** 24
    assert oracle.q16(256.01) == 0                  # out of range
    assert oracle.q16(1e-6) == 0                    # rounds below 1


def _weighted_star(weights):
    n = len(weights)
    edges = [(0, i + 1) for i in range(n)]
    return inputs.from_edges(n + 1, edges, weights=list(weights))


def test_weight_quantisation_and_inverse_transform_boundaries():
    # 1 + 2^-17 is exactly representable in float32 and sits on a rounding tie.
    ws = [1.0, 2.5, 1.0 + 2.0 ** -17, 4.999]
    g = _weighted_star(ws)
    og = oracle.OracleGraph(g.row_offsets, g.col_indices, g.weights)
    wq = [int(math.floor(float(np.float32(w)) * 65536.0 + 0.5)) for w in ws]
    assert wq[0] == 65536 and wq[1] == 163840 and wq[2] == 65537
    total = sum(wq)
    cum = np.cumsum(wq)
    # x = floor(r64 * total / 2^64); index j <=> cum[j-1] <= x < cum[j].
    # Smallest r64 with x >= c is ceil(c * 2^64 / total).
    for j in range(len(ws)):
        lo_x = int(cum[j - 1]) if j else 0
        r_first = -((-lo_x * 2 ** 64) // total)
        r_last = -((-int(cum[j]) * 2 ** 64) // total) - 1
        for r64, want in ((r_first, j), (r_last, j)):
            assert og.weighted_index(0, r64 >> 32, r64 & 0xFFFFFFFF) == want
        if j:
            r = r_first - 1
            assert og.weighted_index(0, r >> 32, r & 0xFFFFFFFF) == j - 1


def test_weighted_draw_matches_weights_chi_square():
    ws = [1.0, 4.0, 2.0, 3.0, 1.5]
    g = _weighted_star(ws)
    og = oracle.OracleGraph(g.row_offsets, g.col_indices, g.weights)
    S = 200000
    out = oracle.deepwalk(og, np.zeros(S, dtype=np.int32), 1, seed=99, use_weights=True)[0]
    counts = np.bincount(out, minlength=len(ws) + 1)[1:]
    expected = np.array(ws) / sum(ws) * S
    assert stats.chisquare(counts, expected).pvalue > 1e-4


def test_equal_weights_behave_like_uniform():
    g = _weighted_star([2.0] * 7)
    og = oracle.OracleGraph(g.row_offsets, g.col_indices, g.weights)
    S = 140000
    out = oracle.deepwalk(og, np.zeros(S, dtype=np.int32), 1, seed=3, use_weights=True)[0]
    counts = np.bincount(out, minlength=8)[1:]
    assert stats.chisquare(counts).pvalue > 1e-4


@pytest.mark.parametrize("d", [1, 2, 3, 7, 64, 1000])
def test_uniform_draw_chi_square(d):
    # One million draws from a star's centre against the exact pmf of floor(r*d/2^32).
    g = inputs.from_edges(d + 1, [(0, i + 1) for i in range(d)])
    og = oracle.OracleGraph(g.row_offsets, g.col_indices)
    S = 1_000_000
    out = oracle.deepwalk(og, np.zeros(S, dtype=np.int32), 1, seed=d)[0]
    counts = np.bincount(out, minlength=d + 1)[1:]
    assert counts.sum() == S
    if d == 1:
        assert counts[0] == S
        return
    two32 = 2 ** 32
    pmf = np.array([(-((-(j + 1) * two32) // d)) - (-((-j * two32) // d)) for j in range(d)],
                   dtype=np.float64) / two32
    assert abs(pmf.sum() - 1.0) < 1e-12
    assert stats.chisquare(counts, pmf * S).pvalue > 1e-4
