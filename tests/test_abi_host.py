"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, and rejects bad arguments before touching the device."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2603_27156_amd as gsr

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "gsr.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gsr_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert len(names) >= 15
    lib = gsr.lib()
    for name in names:
        assert hasattr(lib, name), name
    assert sorted(gsr.EXPORTED) == names          # the binding covers exactly the header
    assert "gfx950" in gsr.gsr_version()


def test_graph_create_rejects_malformed_csr_before_any_device_work():
    rp = np.array([0, 2, 1], dtype=np.int64)
    ci = np.array([0, 1], dtype=np.int32)
    with pytest.raises(gsr.GsrError) as e:
        gsr.gsr_graph_create(rp, ci, nnz=1)
    assert e.value.status == gsr.GSR_ERR_BAD_CSR
    with pytest.raises(gsr.GsrError) as e:
        gsr.gsr_graph_create(np.array([0, 1], dtype=np.int32), np.array([7], dtype=np.int32))
    assert e.value.status == gsr.GSR_ERR_BAD_CSR and "out of range" in str(e.value)
    with pytest.raises(gsr.GsrError) as e:
        gsr.gsr_graph_create(np.array([0, 1], dtype=np.int32), np.array([0], dtype=np.int32),
                             vals=np.ones(1, np.float32), flags=gsr.GSR_GRAPH_GCN_NORM)
    assert e.value.status == gsr.GSR_ERR_INVALID_ARG


def test_operator_argument_validation():
    lib = gsr.lib()
    st = lib.gsr_group_sparse(None, C.c_int64(4), C.c_int32(64), C.c_int64(64), C.c_int32(65), C.c_int32(0),
                              C.c_int32(0), C.c_float(1e-5), None, None, None)
    assert st == gsr.GSR_ERR_UNSUPPORTED
    st = lib.gsr_group_sparse(None, C.c_int64(4), C.c_int32(257), C.c_int64(257), C.c_int32(1), C.c_int32(0),
                              C.c_int32(0), C.c_float(1e-5), None, None, None)
    assert st == gsr.GSR_ERR_UNSUPPORTED
    st = lib.gsr_group_sparse(None, C.c_int64(4), C.c_int32(64), C.c_int64(64), C.c_int32(4), C.c_int32(0),
                              C.c_int32(0), C.c_float(1e-5), None, None, None)
    assert st == gsr.GSR_ERR_INVALID_ARG and b"null" in lib.gsr_last_error()
    assert lib.gsr_group_sparse(None, C.c_int64(0), C.c_int32(64), C.c_int64(64), C.c_int32(4), C.c_int32(0),
                                C.c_int32(0), C.c_float(1e-5), None, None, None) == gsr.GSR_OK     # empty input
    assert lib.gsr_spmm(None, None, C.c_int64(1), C.c_int32(1), None, C.c_int64(1), C.c_int32(0), None) == gsr.GSR_ERR_INVALID_ARG
    cfg = gsr.Config(n=10, d=64, c=2, k=8).c_struct()
    assert lib.gsr_layer_forward(None, C.byref(cfg), None, None, None, C.c_size_t(0), None) == gsr.GSR_ERR_INVALID_ARG
    assert lib.gsr_step(None, C.byref(cfg), *([None] * 15), C.c_size_t(0), None) == gsr.GSR_ERR_INVALID_ARG


def test_options_are_validated():
    with pytest.raises(gsr.GsrError):
        gsr.gsr_set_option("no_such_option", 1)
    with pytest.raises(gsr.GsrError):
        gsr.gsr_set_option("max_workgroups", 12)
    with pytest.raises(gsr.GsrError):
        gsr.gsr_set_option("hub_threshold", -1)
    gsr.gsr_set_option("hub_threshold", 0)        # 0: chosen per graph
    gsr.gsr_set_option("hub_chunk", 0)
    gsr.gsr_set_option("max_workgroups", 0)
