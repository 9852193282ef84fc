"""Seeded synthetic inputs: graphs, edge weights and roots for the five workloads.

This module is input plumbing only.  It is the one piece shared by the CPU
oracle's tests and the GPU library's tests; it contains none of the sampling
method's arithmetic and imports neither of them.

The graphs stand in for the SNAP graphs of the paper's evaluation (Section 8,
table of graphs), which cannot be downloaded here.  Shapes follow the
workload list: R-MAT scale 12 (small DeepWalk case), a 57 K-vertex power-law
graph with weights in [1, 5) (PPI-like; node2vec and PPR), a dense 233 K-vertex
power-law graph (Reddit-like; GraphSAGE 2-hop), a 3 M-vertex power-law graph
(Orkut-like; layer sampling) and R-MAT scale 22 (LiveJournal-like).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "graphgen.cpp")
# ND_GRAPHGEN_LIB lets a test point the module at a build with sanitizers
_LIB = os.environ.get("ND_GRAPHGEN_LIB", os.path.join(_HERE, "libgraphgen.so"))
_lib = None


def compile_generator(lib: str, sanitize: bool = False) -> None:
    """sanitize: AddressSanitizer + UndefinedBehaviorSanitizer build (host code only)."""
    opt = (["-O1", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
            "-fno-omit-frame-pointer", "-g"] if sanitize else ["-O3"])
    subprocess.run(["g++", *opt, "-std=c++17", "-fopenmp", "-shared", "-fPIC", _SRC, "-o", lib], check=True)


def build(force: bool = False) -> str:
    """Compiles the generator (host code only) next to its source."""
    if "ND_GRAPHGEN_LIB" in os.environ:
        return _LIB
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        compile_generator(_LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            build()
        L = ctypes.CDLL(_LIB)
        L.gg_rmat.restype = ctypes.c_void_p
        L.gg_rmat.argtypes = [ctypes.c_int, ctypes.c_int64, ctypes.c_double, ctypes.c_double,
                              ctypes.c_double, ctypes.c_uint64]
        L.gg_chung_lu.restype = ctypes.c_void_p
        L.gg_chung_lu.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_double, ctypes.c_double,
                                  ctypes.c_uint64]
        L.gg_num_vertices.restype = ctypes.c_int64
        L.gg_num_vertices.argtypes = [ctypes.c_void_p]
        L.gg_num_entries.restype = ctypes.c_int64
        L.gg_num_entries.argtypes = [ctypes.c_void_p]
        L.gg_copy.restype = None
        L.gg_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p]
        L.gg_free.restype = None
        L.gg_free.argtypes = [ctypes.c_void_p]
        L.gg_weights.restype = None
        L.gg_weights.argtypes = [ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_double,
                                 ctypes.c_double, ctypes.c_uint64, ctypes.c_void_p]
        L.gg_permutation.restype = None
        L.gg_permutation.argtypes = [ctypes.c_int64, ctypes.c_uint64, ctypes.c_void_p]
        _lib = L
    return _lib


@dataclass
class Graph:
    """Host CSR.  `row_offsets` is int32 or int64 (V+1), `col_indices` int32 (E),
    rows ascending and duplicate-free, `weights` float32 (E) or None."""
    row_offsets: np.ndarray
    col_indices: np.ndarray
    weights: Optional[np.ndarray] = None
    name: str = ""

    @property
    def V(self) -> int:
        return int(self.row_offsets.shape[0] - 1)

    @property
    def E(self) -> int:
        return int(self.col_indices.shape[0])

    def degrees(self) -> np.ndarray:
        return np.diff(self.row_offsets.astype(np.int64))

    def describe(self) -> str:
        d = self.degrees()
        return (f"{self.name}: V={self.V} E={self.E} mean_deg={d.mean():.2f} max_deg={int(d.max())} "
                f"isolated={int((d == 0).sum())} offsets={self.row_offsets.dtype} "
                f"weights={'f32' if self.weights is not None else 'none'}")


def _finish(h, int64_offsets: bool, name: str) -> Graph:
    L = _load()
    if not h:
        raise ValueError("generator rejected its arguments")
    try:
        V, E = L.gg_num_vertices(h), L.gg_num_entries(h)
        if not int64_offsets and E >= 2 ** 31:
            raise ValueError("graph needs int64 offsets")
        off = np.empty(V + 1, dtype=np.int64 if int64_offsets else np.int32)
        col = np.empty(E, dtype=np.int32)
        L.gg_copy(h, off.ctypes.data, 1 if int64_offsets else 0, col.ctypes.data)
    finally:
        L.gg_free(h)
    return Graph(off, col, None, name)


def rmat(scale: int, num_edges: int, a: float, b: float, c: float, seed: int,
         int64_offsets: bool = False, name: str = "rmat") -> Graph:
    """R-MAT: `num_edges` generated edges, self loops dropped, symmetrised, deduplicated,
    vertices relabelled at random."""
    h = _load().gg_rmat(scale, num_edges, a, b, c, seed)
    return _finish(h, int64_offsets, name)


def chung_lu(V: int, num_undirected: int, gamma: float, max_expected_degree: float, seed: int,
             int64_offsets: bool = False, name: str = "chung_lu") -> Graph:
    """Chung-Lu power-law graph with degree exponent `gamma`; `num_undirected` edges are
    drawn before self loops and duplicates are removed."""
    h = _load().gg_chung_lu(V, num_undirected, gamma, max_expected_degree, seed)
    return _finish(h, int64_offsets, name)


def add_weights(g: Graph, lo: float = 1.0, hi: float = 5.0, seed: int = 0) -> Graph:
    """Float32 weights uniform in [lo, hi), equal in both directions of an edge."""
    off64 = np.ascontiguousarray(g.row_offsets, dtype=np.int64)
    w = np.empty(g.E, dtype=np.float32)
    _load().gg_weights(g.V, off64.ctypes.data, g.col_indices.ctypes.data, lo, hi, seed, w.ctypes.data)
    g.weights = w
    return g


def permutation(n: int, seed: int) -> np.ndarray:
    out = np.empty(n, dtype=np.int32)
    _load().gg_permutation(n, seed, out.ctypes.data)
    return out


def from_edges(V: int, edges, weights=None, int64_offsets: bool = False, name: str = "tiny") -> Graph:
    """Builds a CSR from directed (u, v) entries given by hand (tests): rows are sorted by
    destination; duplicates are the caller's business."""
    edges = sorted((int(u), int(v), i) for i, (u, v) in enumerate(edges))
    off = np.zeros(V + 1, dtype=np.int64)
    for u, _, _ in edges:
        off[u + 1] += 1
    off = np.cumsum(off)
    col = np.array([v for _, v, _ in edges], dtype=np.int32).reshape(-1)
    w = None
    if weights is not None:
        w = np.array([weights[i] for _, _, i in edges], dtype=np.float32).reshape(-1)
    return Graph(off.astype(np.int64 if int64_offsets else np.int32), col, w, name)


# ---------------------------------------------------------------------------
# The five workloads.  Generated-edge counts were tuned once so that the entry
# counts after deduplication land near the stated sizes; the actual sizes are
# whatever `Graph.describe()` prints.
# ---------------------------------------------------------------------------

def config1_graph() -> Graph:
    """R-MAT scale 12, 65,536 generated edges, (0.57, 0.19, 0.19), unweighted, int32 offsets."""
    return rmat(12, 65536, 0.57, 0.19, 0.19, seed=1, name="C1 rmat12")


def config2_graph() -> Graph:
    """57,000 vertices, about 820 K undirected edges, degree exponent 2.3, weights U[1,5)."""
    g = chung_lu(57000, 826_000, 2.3, max_expected_degree=1280.0, seed=2, name="C2 chunglu57k")
    return add_weights(g, 1.0, 5.0, seed=2)


def config3_graph() -> Graph:
    """233,000 vertices, about 114 M directed entries, mean degree about 490, max about 20 K."""
    return chung_lu(233000, 59_600_000, 2.1, max_expected_degree=26000.0, seed=3, name="C3 dense233k")


def config4_graph() -> Graph:
    """3.0 M vertices, about 117 M directed entries, degree exponent 2.1."""
    return chung_lu(3_000_000, 58_800_000, 2.1, max_expected_degree=10800.0, seed=4,
                    name="C4 chunglu3m")


def config5_graph() -> Graph:
    """R-MAT scale 22, (0.6, 0.15, 0.15), about 69 M entries after symmetrising; int64 offsets."""
    return rmat(22, 35_800_000, 0.6, 0.15, 0.15, seed=5, int64_offsets=True, name="C5 rmat22")


def all_vertices_roots(g: Graph) -> np.ndarray:
    return np.arange(g.V, dtype=np.int32)


def small_graph(scale: int = 10, edges: int = 12000, seed: int = 11, weighted: bool = False,
                int64_offsets: bool = False) -> Graph:
    """A small skewed graph for element-by-element parity tests."""
    g = rmat(scale, edges, 0.57, 0.19, 0.19, seed=seed, int64_offsets=int64_offsets,
             name=f"rmat{scale}")
    if weighted:
        add_weights(g, 1.0, 5.0, seed=seed)
    return g
