"""The C-ABI library loads and exports every symbol include/nd.h declares
(no compute calls: this runs without a GPU)."""
import ctypes
import os
import re

from paper_2009_06693_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "nd.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = set(re.findall(r"\b(nd_[a-z_0-9]+)\s*\(", text))
    return names


def test_every_declared_symbol_is_exported():
    L = B.lib()
    names = _declared()
    assert {"nd_graph_create", "nd_sample", "nd_sample_query", "nd_graph_destroy"} <= names
    for n in names:
        assert hasattr(L, n), f"{n} declared in nd.h but not exported"
    assert set(B.EXPORTS) == names


def test_version_and_params_defaults():
    assert B.nd_version() == 100
    p = B.nd_params_init()
    assert p.struct_size == ctypes.sizeof(B.nd_params) == 128
    assert p.n2v_max_attempts == 64 and p.sched_force_class == B.ND_CLASS_AUTO
    assert p.mode == B.ND_MODE_TRANSIT_PARALLEL and p.p == 1.0 and p.q == 1.0


def test_null_arguments_are_errors_not_crashes():
    L = B.lib()
    assert L.nd_graph_destroy(None) == 0
    assert L.nd_sample_query(None, 0, None, 0, None, None, None) == B.ND_ERR_NULL_POINTER
    assert b"NULL" in L.nd_last_error()
    h = ctypes.c_void_p()
    assert L.nd_graph_create(ctypes.byref(h), 4, 0, None, 0, None, None, 0, None) == B.ND_ERR_NULL_POINTER
    assert L.nd_graph_create(None, 4, 0, None, 0, None, None, 0, None) == B.ND_ERR_NULL_POINTER
    assert L.nd_group_workspace_bytes(1000, 50) > 0
