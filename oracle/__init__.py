"""ctypes front end of the CPU oracle (nd_oracle.c).

TEST INFRASTRUCTURE, NOT THE PRODUCT: only tests, the smoke check and the
benchmark's CPU-baseline leg may import this package.  It shares no code with
the GPU library and never imports it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "nd_oracle.c")
# ND_ORACLE_LIB lets the mutation test point the pins at a deliberately broken build
_LIB = os.environ.get("ND_ORACLE_LIB", os.path.join(_HERE, "libnd_oracle.so"))
_lib = None

NULL = -1


SANITIZE_FLAGS = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                  "-fno-omit-frame-pointer", "-g"]


def compile_oracle(src: str, lib: str, sanitize: bool = False) -> None:
    """sanitize: build with AddressSanitizer and UndefinedBehaviorSanitizer (host code only; the
    process that loads such a build needs the sanitizer runtime first in LD_PRELOAD)."""
    opt = ["-O1", *SANITIZE_FLAGS] if sanitize else ["-O2"]
    subprocess.run(["gcc", *opt, "-std=c11", "-Wall", "-Wextra", "-shared", "-fPIC", src, "-o", lib,
                    "-lm"], check=True)


def build(force: bool = False) -> str:
    if "ND_ORACLE_LIB" in os.environ:
        return _LIB
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        compile_oracle(_SRC, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            build()
        L = ctypes.CDLL(_LIB)
        vp, i32, i64, u32, u64, dbl = (ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64,
                                       ctypes.c_uint32, ctypes.c_uint64, ctypes.c_double)
        L.ndo_philox4x32_10.restype = None
        L.ndo_philox4x32_10.argtypes = [vp, vp, vp]
        L.ndo_mulhi64.restype = u64
        L.ndo_mulhi64.argtypes = [u64, u64]
        L.ndo_uniform_index.restype = u32
        L.ndo_uniform_index.argtypes = [u32, u32]
        L.ndo_q16.restype = u32
        L.ndo_q16.argtypes = [dbl]
        L.ndo_graph_create.restype = vp
        L.ndo_graph_create.argtypes = [i64, i64, vp, vp, vp]
        L.ndo_graph_destroy.restype = None
        L.ndo_graph_destroy.argtypes = [vp]
        L.ndo_weighted_index.restype = i64
        L.ndo_weighted_index.argtypes = [vp, i32, u32, u32]
        L.ndo_deepwalk.restype = ctypes.c_int
        L.ndo_deepwalk.argtypes = [vp, ctypes.c_int, vp, i64, u64, u64, i32, vp]
        L.ndo_ppr.restype = ctypes.c_int
        L.ndo_ppr.argtypes = [vp, ctypes.c_int, dbl, vp, i64, u64, u64, i32, vp]
        L.ndo_node2vec.restype = ctypes.c_int
        L.ndo_node2vec.argtypes = [vp, ctypes.c_int, dbl, dbl, ctypes.c_int, i32, vp, i64, u64, u64,
                                   i32, vp]
        L.ndo_multirw.restype = ctypes.c_int
        L.ndo_multirw.argtypes = [vp, i32, vp, i64, u64, u64, i32, vp]
        L.ndo_khop.restype = ctypes.c_int
        L.ndo_khop.argtypes = [vp, vp, i32, vp, i64, u64, u64, vp]
        L.ndo_khop_unique.restype = ctypes.c_int
        L.ndo_khop_unique.argtypes = [vp, vp, i32, i32, vp, i64, u64, u64, vp]
        L.ndo_layer.restype = ctypes.c_int
        L.ndo_layer.argtypes = [vp, i32, vp, i32, vp, i64, u64, u64, vp]
        L.ndo_layer_weighted.restype = ctypes.c_int
        L.ndo_layer_weighted.argtypes = [vp, i32, vp, i32, vp, i64, u64, u64, vp]
        L.ndo_layer_edges.restype = ctypes.c_int
        L.ndo_layer_edges.argtypes = [vp, vp, i32, vp, i32, i64, vp, vp, i64]
        _lib = L
    return _lib


def philox4x32_10(ctr, key):
    c = np.asarray(ctr, dtype=np.uint32).copy()
    k = np.asarray(key, dtype=np.uint32).copy()
    o = np.zeros(4, dtype=np.uint32)
    _load().ndo_philox4x32_10(c.ctypes.data, k.ctypes.data, o.ctypes.data)
    return o


def draw(seed: int, sample_id: int, slot: int, step: int, attempt: int = 0):
    """The four words of the generator call the samplers make for this counter."""
    return philox4x32_10([sample_id, slot, step, attempt], [seed & 0xFFFFFFFF, seed >> 32])


def mulhi64(a: int, b: int) -> int:
    return int(_load().ndo_mulhi64(a, b))


def uniform_index(r: int, d: int) -> int:
    return int(_load().ndo_uniform_index(r, d))


def q16(x: float) -> int:
    return int(_load().ndo_q16(x))


class OracleGraph:
    """Host CSR handed to the oracle (it keeps its own copy, with int64 offsets)."""

    def __init__(self, row_offsets, col_indices, weights=None):
        off = np.ascontiguousarray(row_offsets, dtype=np.int64)
        col = np.ascontiguousarray(col_indices, dtype=np.int32)
        w = None if weights is None else np.ascontiguousarray(weights, dtype=np.float32)
        self.V = int(off.shape[0] - 1)
        self.E = int(col.shape[0])
        self.weighted = w is not None
        self._h = _load().ndo_graph_create(self.V, self.E, off.ctypes.data, col.ctypes.data,
                                           None if w is None else w.ctypes.data)
        if not self._h:
            raise MemoryError("ndo_graph_create failed")

    def __del__(self):
        if getattr(self, "_h", None):
            _load().ndo_graph_destroy(self._h)
            self._h = None

    def weighted_index(self, v: int, r0: int, r1: int) -> int:
        return int(_load().ndo_weighted_index(self._h, v, r0, r1))


def _roots(roots):
    return np.ascontiguousarray(roots, dtype=np.int32)


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"oracle {what} failed with code {rc}")


def deepwalk(g: OracleGraph, roots, length: int, seed: int, use_weights: bool = False,
             sample_id_base: int = 0) -> np.ndarray:
    """Returns int32 [length, S]: row i is the vertex every walk adds at step i."""
    r = _roots(roots)
    out = np.empty((length, r.shape[0]), dtype=np.int32)
    _check(_load().ndo_deepwalk(g._h, int(use_weights), r.ctypes.data, r.shape[0], sample_id_base,
                                seed, length, out.ctypes.data), "deepwalk")
    return out


def ppr(g: OracleGraph, roots, max_length: int, term_prob: float, seed: int,
        use_weights: bool = False, sample_id_base: int = 0) -> np.ndarray:
    r = _roots(roots)
    out = np.empty((max_length, r.shape[0]), dtype=np.int32)
    _check(_load().ndo_ppr(g._h, int(use_weights), term_prob, r.ctypes.data, r.shape[0],
                           sample_id_base, seed, max_length, out.ctypes.data), "ppr")
    return out


def node2vec(g: OracleGraph, roots, length: int, p: float, q: float, seed: int,
             use_weights: bool = False, convention: int = 0, max_attempts: int = 64,
             sample_id_base: int = 0) -> np.ndarray:
    r = _roots(roots)
    out = np.empty((length, r.shape[0]), dtype=np.int32)
    _check(_load().ndo_node2vec(g._h, int(use_weights), p, q, convention, max_attempts,
                                r.ctypes.data, r.shape[0], sample_id_base, seed, length,
                                out.ctypes.data), "node2vec")
    return out


def multirw(g: OracleGraph, roots, roots_per_sample: int, length: int, seed: int,
            sample_id_base: int = 0) -> np.ndarray:
    """`roots` holds S * roots_per_sample vertices; returns int32 [length, S]."""
    r = _roots(roots)
    if r.shape[0] % roots_per_sample:
        raise ValueError("roots must be a whole number of samples")
    S = r.shape[0] // roots_per_sample
    out = np.empty((length, S), dtype=np.int32)
    _check(_load().ndo_multirw(g._h, roots_per_sample, r.ctypes.data, S, sample_id_base, seed, length,
                               out.ctypes.data), "multirw")
    return out


def khop(g: OracleGraph, roots, fanout, seed: int, sample_id_base: int = 0, unique_rounds: int = 0):
    """Returns a list with one int32 [S, W_i] array per step.  unique_rounds > 0: no vertex
    twice within a sample and step (that many draw rounds per slot)."""
    r = _roots(roots)
    f = np.ascontiguousarray(fanout, dtype=np.int32)
    S = r.shape[0]
    widths = np.cumprod(f.astype(np.int64))
    out = np.empty(int(S * widths.sum()), dtype=np.int32)
    if unique_rounds > 0:
        _check(_load().ndo_khop_unique(g._h, f.ctypes.data, f.shape[0], unique_rounds, r.ctypes.data, S,
                                       sample_id_base, seed, out.ctypes.data), "khop_unique")
    else:
        _check(_load().ndo_khop(g._h, f.ctypes.data, f.shape[0], r.ctypes.data, S, sample_id_base,
                                seed, out.ctypes.data), "khop")
    res, base = [], 0
    for W in widths:
        res.append(out[base:base + S * int(W)].reshape(S, int(W)))
        base += S * int(W)
    return res


def layer(g: OracleGraph, roots, roots_per_sample: int, fanout, seed: int, sample_id_base: int = 0,
          use_weights: bool = False):
    """`roots` holds num_samples * roots_per_sample vertices; returns one int32
    [num_samples, fanout[i]] array per step.  use_weights: draw in proportion to the graph's edge
    weights instead of 1 / deg(transit)^2."""
    r = _roots(roots)
    f = np.ascontiguousarray(fanout, dtype=np.int32)
    if r.shape[0] % roots_per_sample:
        raise ValueError("roots must be a whole number of samples")
    B = r.shape[0] // roots_per_sample
    out = np.empty(int(B * f.astype(np.int64).sum()), dtype=np.int32)
    fn = _load().ndo_layer_weighted if use_weights else _load().ndo_layer
    _check(fn(g._h, roots_per_sample, f.ctypes.data, f.shape[0], r.ctypes.data, B,
              sample_id_base, seed, out.ctypes.data), "layer")
    res, base = [], 0
    for m in f:
        res.append(out[base:base + B * int(m)].reshape(B, int(m)))
        base += B * int(m)
    return res


def layer_edges(g: OracleGraph, transits, sampled):
    """Edges between the transits [S, n_prev] of a step and the vertices [S, m] it added.
    Returns (row_ptr int64[S * n_prev + 1], edge_slot int32[row_ptr[-1]])."""
    t = np.ascontiguousarray(transits, dtype=np.int32)
    v = np.ascontiguousarray(sampled, dtype=np.int32)
    if t.ndim != 2 or v.ndim != 2 or t.shape[0] != v.shape[0]:
        raise ValueError("transits and sampled must be [S, n_prev] and [S, m]")
    S, n_prev, m = t.shape[0], t.shape[1], v.shape[1]
    row_ptr = np.empty(S * n_prev + 1, dtype=np.int64)
    _check(_load().ndo_layer_edges(g._h, t.ctypes.data, n_prev, v.ctypes.data, m, S, row_ptr.ctypes.data,
                                   None, 0), "layer_edges (count)")
    edges = np.empty(int(row_ptr[-1]), dtype=np.int32)
    _check(_load().ndo_layer_edges(g._h, t.ctypes.data, n_prev, v.ctypes.data, m, S, row_ptr.ctypes.data,
                                   edges.ctypes.data, edges.shape[0]), "layer_edges")
    return row_ptr, edges


def pack_samples(steps):
    """Output format 1 of Section 4.1: one record per sample holding what it gained at every
    step, in step order.  `steps` is a list of [S, w_i] arrays (a walk's [L, S] array is a list of
    L arrays of S entries); returns int32 [S, sum of w_i]."""
    cols = [np.asarray(x, dtype=np.int32).reshape(len(x), -1) for x in steps]
    return np.concatenate(cols, axis=1)
