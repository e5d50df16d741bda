"""The C ABI library loads and exports every symbol include/gad.h declares; host-side argument
validation returns error codes without touching a GPU.  No compute is launched here."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2110_02987_amd import gad
    if not os.path.exists(gad.LIB_PATH):
        from paper_2110_02987_amd.build import build_native
        build_native(verbose=False)
    return gad.lib()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "gad.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gad_[a-z_0-9]+)\s*\(", text)))


def test_header_symbols_exported(lib):
    from paper_2110_02987_amd import gad
    names = declared_symbols()
    assert len(names) >= 10
    assert sorted(gad.SYMBOLS) == names
    for n in names:
        assert hasattr(lib, n), n


def test_host_side_validation(lib):
    err = lambda: lib.gad_last_error().decode()
    out = C.c_void_p()
    assert lib.gad_build_subgraph(None, None, C.c_int64(0), C.c_int64(4), None, C.c_int64(0), None, C.c_int64(0), None,
                                  C.byref(out)) == -2 and "no nodes" in err()
    assert lib.gad_build_subgraph(None, None, C.c_int64(3), C.c_int64(4), None, C.c_int64(2), None, C.c_int64(0), None,
                                  C.byref(out)) == -1
    assert lib.gad_build_subgraph(None, None, C.c_int64(-1), C.c_int64(4), None, C.c_int64(2), None, C.c_int64(0), None,
                                  C.byref(out)) == -2
    assert lib.gad_build_subgraph(None, None, C.c_int64(1 << 30), C.c_int64(4), None, C.c_int64(2), None, C.c_int64(0),
                                  None, C.byref(out)) == -2
    assert lib.gad_build_subgraph(None, None, C.c_int64(0), C.c_int64(4), None, C.c_int64(2), None, C.c_int64(0), None,
                                  None) == -1
    b = C.c_size_t()
    dims = (C.c_int32 * 3)(8, 4, 2)
    assert lib.gad_gcn_workspace_bytes(None, C.c_int(2), dims, C.c_int(0), C.byref(b)) == -1
    assert lib.gad_graph_info(None, None, None, None, None, None, None, None) == -1
    assert lib.gad_graph_destroy(None) == 0
    z = (C.c_double * 2)(1.0, -1.0)
    bufs = (C.c_void_p * 2)(16, 16)          # never dereferenced: validation fails first
    assert lib.gad_weighted_consensus(bufs, C.c_int(2), z, C.c_int64(4), C.c_void_p(16), None) == -6
    z = (C.c_double * 2)(0.0, 0.0)
    assert lib.gad_weighted_consensus(bufs, C.c_int(2), z, C.c_int64(4), C.c_void_p(16), None) == -6
    assert lib.gad_weighted_consensus(bufs, C.c_int(0), z, C.c_int64(4), C.c_void_p(16), None) == -2
    assert lib.gad_weighted_consensus(None, C.c_int(2), z, C.c_int64(4), C.c_void_p(16), None) == -1
    assert lib.gad_spmm(None, None, C.c_int64(4), None, C.c_int64(4), C.c_int32(4), C.c_int(0), None) == -1
    assert lib.gad_subgraph_variance(None, None, C.c_int32(4), C.c_int(0), C.c_double(1.0), None, None, None) == -1
    # entry points added around the per-iteration step: the host checks come before any launch
    assert lib.gad_gemm_workspace_bytes(C.c_int64(8), C.c_int32(0), C.c_int32(8), C.byref(b)) == -2
    assert lib.gad_gemm_workspace_bytes(C.c_int64(8), C.c_int32(8), C.c_int32(8), None) == -1
    assert lib.gad_spmm_workspace_bytes(None, C.c_int32(8), C.byref(b)) == -1
    assert lib.gad_pair_importance_workspace_bytes(None, C.c_int32(8), C.byref(b)) == -1
    assert lib.gad_pair_importance(None, None, C.c_int32(4), C.c_int(0), C.c_double(1.0), None, None, C.c_size_t(0), None) == -1
    assert lib.gad_graph_concat(None, C.c_int(2), None, C.byref(out)) == -1
    assert lib.gad_graph_concat(bufs, C.c_int(0), None, C.byref(out)) == -2
    nh = C.c_int64()
    assert lib.gad_augment_subgraph(None, None, C.c_int64(1), C.c_int32(2), C.c_int64(1), C.c_uint64(0), C.c_int64(10),
                                    None, C.byref(nh), None, None) == -1
    assert lib.gad_consensus_update(bufs, C.c_int(2), z, C.c_int64(4), C.c_float(0.1), None, None, None) == -1
