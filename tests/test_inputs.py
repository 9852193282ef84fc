"""The seeded input generators: structure and reproducibility."""
import numpy as np

from paper_2009_06693_amd import inputs


def _check_structure(g):
    off = g.row_offsets.astype(np.int64)
    assert off[0] == 0 and off[-1] == g.E and (np.diff(off) >= 0).all()
    src = np.repeat(np.arange(g.V, dtype=np.int64), np.diff(off))
    dst = g.col_indices.astype(np.int64)
    assert ((dst >= 0) & (dst < g.V)).all()
    assert (src != dst).all()                                   # no self loops
    key = src * g.V + dst
    assert (np.diff(key) > 0).all()                             # rows ascending, no duplicates
    rev = np.sort(dst * g.V + src)
    assert (rev == key).all()                                   # symmetric


def test_rmat_structure_and_determinism():
    a = inputs.config1_graph()
    b = inputs.config1_graph()
    _check_structure(a)
    assert a.V == 4096 and a.row_offsets.dtype == np.int32
    assert (a.row_offsets == b.row_offsets).all() and (a.col_indices == b.col_indices).all()
    c = inputs.rmat(12, 65536, 0.57, 0.19, 0.19, seed=2)
    assert c.E != a.E or (c.col_indices != a.col_indices).any()
    d = a.degrees()
    assert d.max() > 20 * d.mean()                              # skewed


def test_chung_lu_structure_weights_and_offsets_width():
    g = inputs.config2_graph()
    _check_structure(g)
    assert g.V == 57000 and abs(g.E - 1_640_000) < 50_000
    w = g.weights
    assert w.dtype == np.float32 and (w >= 1.0).all() and (w < 5.0).all()
    assert abs(float(w.mean()) - 3.0) < 0.01
    # both directions of an edge carry the same weight
    off = g.row_offsets.astype(np.int64)
    src = np.repeat(np.arange(g.V, dtype=np.int64), np.diff(off))
    dst = g.col_indices.astype(np.int64)
    order = np.argsort(dst * g.V + src, kind="stable")
    assert (w[order] == w).all()
    h = inputs.small_graph(9, 4000, seed=5, int64_offsets=True)
    assert h.row_offsets.dtype == np.int64
    _check_structure(h)


def test_permutation():
    p = inputs.permutation(1000, 3)
    assert sorted(p.tolist()) == list(range(1000))
    assert (p == inputs.permutation(1000, 3)).all()
    assert (p != inputs.permutation(1000, 4)).any()
