"""Thin ctypes binding of libnd.so: same names as include/nd.h, argument
marshalling only.  PyTorch supplies device memory and the current stream;
every step of the sampling path runs inside the library's HIP kernels.

There is no CPU fallback: if the shared library is missing, loading fails.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("ND_LIB", os.path.join(_HERE, "libnd.so"))

ND_MAX_FANOUT_STEPS = 8
ND_MAX_WALK_STEPS = 4096
ND_NULL_VERTEX = -1
ND_MAX_EDGE_SLOTS = 2048

ND_DEEPWALK, ND_PPR, ND_NODE2VEC, ND_KHOP, ND_LAYER, ND_MULTIRW = range(6)
ND_MODE_TRANSIT_PARALLEL, ND_MODE_SAMPLE_PARALLEL = 0, 1
ND_CLASS_AUTO, ND_CLASS_SUBWAVE, ND_CLASS_WORKGROUP, ND_CLASS_GRID = -1, 0, 1, 2

ND_OK = 0
ND_ERR_NULL_POINTER, ND_ERR_BAD_ARGUMENT, ND_ERR_BAD_GRAPH, ND_ERR_BAD_WEIGHT = -1, -2, -3, -4
ND_ERR_NO_WEIGHTS, ND_ERR_WORKSPACE, ND_ERR_HIP, ND_ERR_BAD_ROOT, ND_ERR_TOO_LARGE = -5, -6, -7, -8, -9

EXPORTS = ["nd_params_init", "nd_graph_create", "nd_graph_destroy", "nd_graph_info", "nd_sample_query",
           "nd_sample", "nd_sample_static", "nd_sample_status", "nd_sample_stats", "nd_group_workspace_bytes",
           "nd_group_by_transit", "nd_layer_edges_workspace_bytes", "nd_layer_edges_count",
           "nd_layer_edges_fill", "nd_layer_edges_status", "nd_samples_pack", "nd_probe_store_runs", "nd_profile_enable", "nd_profile_read", "nd_last_error", "nd_version"]

ND_PHASES = ["init", "sort", "group", "sample_sub", "sample_wg", "sample_sp", "layer", "unique", "walk_window"]


class nd_params(ctypes.Structure):
    _fields_ = [
        ("struct_size", ctypes.c_uint32),
        ("num_steps", ctypes.c_int32),
        ("fanout", ctypes.c_int32 * ND_MAX_FANOUT_STEPS),
        ("use_weights", ctypes.c_int32),
        ("bias_convention", ctypes.c_int32),
        ("p", ctypes.c_double),
        ("q", ctypes.c_double),
        ("term_prob", ctypes.c_double),
        ("roots_per_sample", ctypes.c_int32),
        ("n2v_max_attempts", ctypes.c_int32),
        ("sample_id_base", ctypes.c_uint64),
        ("mode", ctypes.c_int32),
        ("sched_force_class", ctypes.c_int32),
        ("sched_sub_max", ctypes.c_int32),
        ("sched_wg_max", ctypes.c_int32),
        ("lds_stage_policy", ctypes.c_int32),
        ("unique_rounds", ctypes.c_int32),
        ("sched_group_bits", ctypes.c_int32),
        ("sched_window", ctypes.c_int32),
        ("reserved", ctypes.c_int32 * 2),
    ]


class NdError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"nd error {code}: {message}")
        self.code = code


_lib = None


def lib() -> ctypes.CDLL:
    """Loads libnd.so (built in-tree by paper_2009_06693_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: run `python -m paper_2009_06693_amd.build` "
                "(there is no CPU fallback)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, u64, sz = (ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_uint64,
                                 ctypes.c_size_t)
        L.nd_params_init.restype = None
        L.nd_params_init.argtypes = [ctypes.POINTER(nd_params)]
        L.nd_graph_create.restype = ctypes.c_int
        L.nd_graph_create.argtypes = [ctypes.POINTER(vp), i64, i64, vp, ctypes.c_int, vp, vp,
                                      ctypes.c_int, vp]
        L.nd_graph_destroy.restype = ctypes.c_int
        L.nd_graph_destroy.argtypes = [vp]
        L.nd_graph_info.restype = ctypes.c_int
        L.nd_graph_info.argtypes = [vp, ctypes.POINTER(i64), ctypes.POINTER(i64),
                                    ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int)]
        L.nd_sample_query.restype = ctypes.c_int
        L.nd_sample_query.argtypes = [vp, ctypes.c_int, ctypes.POINTER(nd_params), i64,
                                      ctypes.POINTER(i32), ctypes.POINTER(i64), ctypes.POINTER(sz)]
        L.nd_sample.restype = ctypes.c_int
        L.nd_sample.argtypes = [vp, ctypes.c_int, ctypes.POINTER(nd_params), vp, i64, u64,
                                ctypes.POINTER(vp), vp, sz, vp]
        L.nd_sample_static.restype = ctypes.c_int
        L.nd_sample_static.argtypes = [vp, ctypes.c_int, ctypes.POINTER(nd_params), vp, i64, u64,
                                       ctypes.POINTER(vp), vp, vp]
        L.nd_sample_status.restype = ctypes.c_int
        L.nd_sample_status.argtypes = [vp, vp]
        L.nd_sample_stats.restype = ctypes.c_int
        L.nd_sample_stats.argtypes = [vp, vp, i32, ctypes.POINTER(i64)]
        L.nd_group_workspace_bytes.restype = sz
        L.nd_group_workspace_bytes.argtypes = [i64, i64]
        L.nd_group_by_transit.restype = ctypes.c_int
        L.nd_group_by_transit.argtypes = [vp, i64, i64, vp, vp, vp, vp, vp, vp, sz, vp]
        L.nd_layer_edges_workspace_bytes.restype = sz
        L.nd_layer_edges_workspace_bytes.argtypes = [i64, i32]
        L.nd_layer_edges_count.restype = ctypes.c_int
        L.nd_layer_edges_count.argtypes = [vp, vp, i32, vp, i32, i64, vp, vp, sz, vp]
        L.nd_layer_edges_fill.restype = ctypes.c_int
        L.nd_layer_edges_fill.argtypes = [vp, vp, i32, vp, i32, i64, vp, vp, i64, vp]
        L.nd_layer_edges_status.restype = ctypes.c_int
        L.nd_layer_edges_status.argtypes = [vp, vp]
        L.nd_samples_pack.restype = ctypes.c_int
        L.nd_samples_pack.argtypes = [vp, i32, ctypes.POINTER(i64), i64, vp, vp]
        L.nd_probe_store_runs.restype = ctypes.c_int
        L.nd_probe_store_runs.argtypes = [vp, i64, i32, ctypes.c_int, vp]
        L.nd_profile_enable.restype = ctypes.c_int
        L.nd_profile_enable.argtypes = [ctypes.c_int]
        L.nd_profile_read.restype = ctypes.c_int
        L.nd_profile_read.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i64)]
        L.nd_last_error.restype = ctypes.c_char_p
        L.nd_last_error.argtypes = []
        L.nd_version.restype = ctypes.c_int
        L.nd_version.argtypes = []
        _lib = L
    return _lib


def _check(rc: int):
    if rc != ND_OK:
        raise NdError(rc, lib().nd_last_error().decode())


def nd_version() -> int:
    return lib().nd_version()


def nd_params_init(**overrides) -> nd_params:
    """Returns an nd_params with the library's defaults, then applies keyword overrides
    (fanout may be given as a sequence)."""
    p = nd_params()
    lib().nd_params_init(ctypes.byref(p))
    for k, v in overrides.items():
        if k == "fanout":
            for i, f in enumerate(v):
                p.fanout[i] = int(f)
        else:
            if not hasattr(p, k):
                raise AttributeError(k)
            setattr(p, k, v)
    return p


def _stream_ptr(stream: Optional[torch.cuda.Stream]) -> int:
    s = stream if stream is not None else torch.cuda.current_stream()
    return s.cuda_stream


class Graph:
    """Owner of an nd_graph handle."""

    def __init__(self, handle: int, V: int, E: int, weighted: bool):
        self._h = handle
        self.V, self.E, self.weighted = V, E, weighted

    def destroy(self):
        if self._h:
            lib().nd_graph_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def nd_graph_create(row_offsets, col_indices, weights=None, stream=None) -> Graph:
    """row_offsets / col_indices / weights: numpy arrays (host) or CUDA tensors (device);
    offsets int32 or int64, columns int32, weights float32."""
    L = lib()
    on_device = isinstance(row_offsets, torch.Tensor)
    if on_device:
        if not (row_offsets.is_cuda and col_indices.is_cuda and (weights is None or weights.is_cuda)):
            raise ValueError("all graph tensors must be CUDA tensors")
        off, col = row_offsets.contiguous(), col_indices.contiguous()
        w = None if weights is None else weights.contiguous()
        if col.dtype != torch.int32 or off.dtype not in (torch.int32, torch.int64):
            raise TypeError("offsets must be int32/int64 and columns int32")
        if w is not None and w.dtype != torch.float32:
            raise TypeError("weights must be float32")
        is64 = off.dtype == torch.int64
        V, E = off.numel() - 1, col.numel()
        ptrs = (off.data_ptr(), col.data_ptr(), None if w is None else w.data_ptr())
    else:
        off = np.ascontiguousarray(row_offsets)
        col = np.ascontiguousarray(col_indices)
        w = None if weights is None else np.ascontiguousarray(weights)
        if col.dtype != np.int32 or off.dtype not in (np.int32, np.int64):
            raise TypeError("offsets must be int32/int64 and columns int32")
        if w is not None and w.dtype != np.float32:
            raise TypeError("weights must be float32")
        is64 = off.dtype == np.int64
        V, E = off.shape[0] - 1, col.shape[0]
        ptrs = (off.ctypes.data, col.ctypes.data, None if w is None else w.ctypes.data)
        torch.cuda.init()
    h = ctypes.c_void_p()
    _check(L.nd_graph_create(ctypes.byref(h), V, E, ptrs[0], int(is64), ptrs[1], ptrs[2],
                             int(on_device), _stream_ptr(stream)))
    return Graph(h.value, V, E, weights is not None)


def nd_graph_destroy(g: Graph):
    g.destroy()


def nd_sample_query(g: Graph, app: int, params: nd_params, num_roots: int):
    """Returns (step_len list, workspace_bytes)."""
    n = ctypes.c_int32()
    lens = (ctypes.c_int64 * ND_MAX_WALK_STEPS)()
    ws = ctypes.c_size_t()
    _check(lib().nd_sample_query(g._h, app, ctypes.byref(params), num_roots, ctypes.byref(n), lens,
                                 ctypes.byref(ws)))
    return [int(lens[i]) for i in range(n.value)], int(ws.value)


def nd_sample(g: Graph, app: int, params: nd_params, roots: torch.Tensor, seed: int,
              step_out: Sequence[torch.Tensor], workspace: torch.Tensor, stream=None):
    """Asynchronous on the stream; step_out[i] are caller-allocated int32 CUDA tensors."""
    if roots.dtype != torch.int32 or not roots.is_cuda or not roots.is_contiguous():
        raise TypeError("roots must be a contiguous int32 CUDA tensor")
    for t in step_out:
        if t.dtype != torch.int32 or not t.is_cuda or not t.is_contiguous():
            raise TypeError("outputs must be contiguous int32 CUDA tensors")
    arr = (ctypes.c_void_p * len(step_out))(*[t.data_ptr() for t in step_out])
    _check(lib().nd_sample(g._h, app, ctypes.byref(params), roots.data_ptr(), roots.numel(), seed, arr,
                           workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                           _stream_ptr(stream)))


ND_STATIC_SCRATCH_BYTES = 32 << 20


def nd_sample_static(g: Graph, app: int, params: nd_params, roots: torch.Tensor, seed: int,
                     step_out: Sequence[torch.Tensor], status: Optional[torch.Tensor] = None, stream=None):
    """nd_sample on the library's own scratch array (no workspace, nothing allocated);
    status: optional int32/uint32 CUDA tensor of one element that receives the status word."""
    if roots.dtype != torch.int32 or not roots.is_cuda or not roots.is_contiguous():
        raise TypeError("roots must be a contiguous int32 CUDA tensor")
    for t in step_out:
        if t.dtype != torch.int32 or not t.is_cuda or not t.is_contiguous():
            raise TypeError("outputs must be contiguous int32 CUDA tensors")
    arr = (ctypes.c_void_p * len(step_out))(*[t.data_ptr() for t in step_out])
    _check(lib().nd_sample_static(g._h, app, ctypes.byref(params), roots.data_ptr(), roots.numel(), seed,
                                  arr, None if status is None else status.data_ptr(),
                                  _stream_ptr(stream)))


def nd_sample_status(workspace: torch.Tensor, stream=None):
    _check(lib().nd_sample_status(workspace.data_ptr(), _stream_ptr(stream)))


def nd_sample_stats(workspace: torch.Tensor, num_steps: int, stream=None) -> np.ndarray:
    """int64 [num_steps, 8]: live pairs, distinct transits, sub-wavefront / workgroup / grid
    transits, grid chunks, work items staged in LDS, reserved."""
    out = (ctypes.c_int64 * (8 * num_steps))()
    _check(lib().nd_sample_stats(workspace.data_ptr(), _stream_ptr(stream), num_steps, out))
    return np.array(out, dtype=np.int64).reshape(num_steps, 8)


def nd_profile_enable(on: bool):
    _check(lib().nd_profile_enable(int(on)))


def nd_profile_read():
    """Returns {phase: (milliseconds, intervals)} accumulated since the previous read."""
    n = len(ND_PHASES)
    ms = (ctypes.c_double * n)()
    cnt = (ctypes.c_int64 * n)()
    _check(lib().nd_profile_read(ms, cnt))
    return {ND_PHASES[i]: (float(ms[i]), int(cnt[i])) for i in range(n)}


def nd_group_by_transit(transits: torch.Tensor, V: int, stream=None):
    """Returns (sorted_transits, sorted_slots, group_transit, group_start, num_pairs, num_groups)."""
    if transits.dtype != torch.int32 or not transits.is_cuda:
        raise TypeError("transits must be an int32 CUDA tensor")
    n = transits.numel()
    dev = transits.device
    sk = torch.empty(max(n, 1), dtype=torch.int32, device=dev)
    sv = torch.empty(max(n, 1), dtype=torch.int32, device=dev)
    gk = torch.empty(max(n, 1), dtype=torch.int32, device=dev)
    gs = torch.empty(n + 1, dtype=torch.int32, device=dev)
    counts = torch.zeros(2, dtype=torch.int64, device=dev)
    wsb = lib().nd_group_workspace_bytes(n, V)
    ws = torch.empty(wsb, dtype=torch.uint8, device=dev)
    _check(lib().nd_group_by_transit(transits.contiguous().data_ptr(), n, V, sk.data_ptr(),
                                     sv.data_ptr(), gk.data_ptr(), gs.data_ptr(), counts.data_ptr(),
                                     ws.data_ptr(), wsb, _stream_ptr(stream)))
    c = counts.cpu()
    P, U = int(c[0]), int(c[1])
    return sk[:P], sv[:P], gk[:U], gs[:U + 1], P, U


def nd_samples_pack(step_out: Sequence[torch.Tensor], num_samples: int, samples: Optional[torch.Tensor] = None,
                    stream=None) -> torch.Tensor:
    """Gathers the per-step arrays of an nd_sample call into one record per sample
    (int32 [num_samples, record])."""
    k = len(step_out)
    for o in step_out:
        if o.dtype != torch.int32 or not o.is_cuda or not o.is_contiguous():
            raise TypeError("step arrays must be contiguous int32 CUDA tensors")
    lens = (ctypes.c_int64 * k)(*[int(o.numel()) for o in step_out])
    ptrs = (ctypes.c_void_p * k)(*[o.data_ptr() for o in step_out])
    record = sum(int(o.numel()) // num_samples for o in step_out) if num_samples else 0
    if samples is None:
        samples = torch.empty((num_samples, record), dtype=torch.int32, device=step_out[0].device)
    elif samples.dtype != torch.int32 or samples.numel() < num_samples * record or not samples.is_contiguous():
        raise TypeError("samples must be a contiguous int32 tensor of num_samples * record entries")
    _check(lib().nd_samples_pack(ptrs, k, lens, num_samples, samples.data_ptr() if samples.numel() else None,
                                 _stream_ptr(stream)))
    return samples


def nd_probe_store_runs(out: torch.Tensor, n_runs: int, run_len: int, scattered: bool, stream=None):
    """Measurement: writes n_runs runs of run_len int32 into `out` (n_runs * run_len entries)."""
    if out.dtype != torch.int32 or not out.is_cuda or out.numel() < n_runs * run_len:
        raise TypeError("out must be an int32 CUDA tensor of n_runs * run_len entries")
    _check(lib().nd_probe_store_runs(out.data_ptr(), n_runs, run_len, int(scattered), _stream_ptr(stream)))


def nd_layer_edges_workspace_bytes(num_samples: int, n_prev: int) -> int:
    return lib().nd_layer_edges_workspace_bytes(num_samples, n_prev)


def nd_layer_edges_count(g: Graph, transits: torch.Tensor, sampled: torch.Tensor, row_ptr: torch.Tensor,
                         workspace: torch.Tensor, stream=None):
    """transits [S, n_prev] and sampled [S, m], int32 on the GPU; row_ptr int64 [S * n_prev + 1]."""
    S, n_prev, m = _edge_shapes(transits, sampled)
    if row_ptr.dtype != torch.int64 or row_ptr.numel() < S * n_prev + 1:
        raise TypeError("row_ptr must be int64 with S * n_prev + 1 entries")
    _check(lib().nd_layer_edges_count(g._h, transits.data_ptr() if S else None, n_prev,
                                      sampled.data_ptr() if S else None, m, S, row_ptr.data_ptr(),
                                      workspace.data_ptr(), workspace.numel(), _stream_ptr(stream)))


def nd_layer_edges_fill(g: Graph, transits: torch.Tensor, sampled: torch.Tensor, row_ptr: torch.Tensor,
                        edge_slot: torch.Tensor, stream=None):
    S, n_prev, m = _edge_shapes(transits, sampled)
    if edge_slot.dtype != torch.int32:
        raise TypeError("edge_slot must be int32")
    _check(lib().nd_layer_edges_fill(g._h, transits.data_ptr() if S else None, n_prev,
                                     sampled.data_ptr() if S else None, m, S, row_ptr.data_ptr(),
                                     edge_slot.data_ptr() if edge_slot.numel() else None,
                                     edge_slot.numel(), _stream_ptr(stream)))


def nd_layer_edges_status(workspace: torch.Tensor, stream=None):
    _check(lib().nd_layer_edges_status(workspace.data_ptr(), _stream_ptr(stream)))


def _edge_shapes(transits, sampled):
    for x in (transits, sampled):
        if x.dtype != torch.int32 or not x.is_cuda or x.dim() != 2 or not x.is_contiguous():
            raise TypeError("transits and sampled must be contiguous 2-D int32 CUDA tensors")
    if transits.shape[0] != sampled.shape[0]:
        raise ValueError("transits and sampled must hold the same number of samples")
    return int(transits.shape[0]), int(transits.shape[1]), int(sampled.shape[1])


def layer_edges(g: Graph, transits: torch.Tensor, sampled: torch.Tensor, stream=None):
    """Count, size, fill: returns (row_ptr int64 [S * n_prev + 1], edge_slot int32 [row_ptr[-1]])."""
    S, n_prev, _ = _edge_shapes(transits, sampled)
    dev = transits.device
    wsb = nd_layer_edges_workspace_bytes(S, n_prev)
    ws = torch.empty(max(wsb, 256), dtype=torch.uint8, device=dev)
    row_ptr = torch.empty(S * n_prev + 1, dtype=torch.int64, device=dev)
    nd_layer_edges_count(g, transits, sampled, row_ptr, ws, stream)
    nd_layer_edges_status(ws, stream)
    total = int(row_ptr[-1].item())
    edge_slot = torch.empty(total, dtype=torch.int32, device=dev)
    nd_layer_edges_fill(g, transits, sampled, row_ptr, edge_slot, stream)
    return row_ptr, edge_slot


# ---------------------------------------------------------------------------
# Convenience wrapper used by tests, smoke and the benchmark: allocates the
# outputs and workspace with torch and calls nd_sample.
# ---------------------------------------------------------------------------

class Sampler:
    def __init__(self, g: Graph, app: int, params: nd_params, num_roots: int, device="cuda:0"):
        self.g, self.app, self.params, self.num_roots = g, app, params, num_roots
        self.step_len, self.workspace_bytes = nd_sample_query(g, app, params, num_roots)
        self.device = torch.device(device)
        self.workspace = torch.empty(max(self.workspace_bytes, 256), dtype=torch.uint8,
                                     device=self.device)
        starts, total = [], 0
        for n in self.step_len:                      # every step starts on a 256-byte boundary
            starts.append(total)
            total += (n + 63) // 64 * 64
        self._flat = torch.empty(max(total, 1), dtype=torch.int32, device=self.device)
        self.out: List[torch.Tensor] = [self._flat[b:b + n] for b, n in zip(starts, self.step_len)]

    def run(self, roots: torch.Tensor, seed: int, stream=None) -> List[torch.Tensor]:
        nd_sample(self.g, self.app, self.params, roots, seed, self.out, self.workspace, stream)
        return self.out

    def status(self):
        nd_sample_status(self.workspace)

    def stats(self) -> np.ndarray:
        return nd_sample_stats(self.workspace, len(self.step_len))
