"""Pin for the oracle's per-sample records (Section 4.1, "Output format", format 1):
hand-written expectations."""
import numpy as np

import oracle


def test_walk_records_are_the_paths():
    steps = np.array([[1, 2, 3], [4, -1, 6]], dtype=np.int32)          # [L = 2, S = 3]
    assert oracle.pack_samples(steps).tolist() == [[1, 4], [2, -1], [3, 6]]


def test_khop_records_list_hop_after_hop():
    hop1 = np.array([[10, 11], [20, 21]], dtype=np.int32)               # S = 2, fanout 2
    hop2 = np.array([[100, 101, 110, 111, 112, 113], [200, 201, 210, 211, 212, 213]], dtype=np.int32)
    got = oracle.pack_samples([hop1, hop2])
    assert got.tolist() == [[10, 11, 100, 101, 110, 111, 112, 113], [20, 21, 200, 201, 210, 211, 212, 213]]
