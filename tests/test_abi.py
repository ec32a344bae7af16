"""Host-side checks that need no GPU: the C-ABI library loads, exports every symbol the header
declares, and turns bad arguments into error codes before any GPU work."""
import ctypes as C
import os
import re

import pytest

from paper_2311_06837_amd import binding as B
from paper_2311_06837_amd import build as build_mod

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        build_mod.build_library()
    return B.lib()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "gnnhot.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(gnn_[a-z0-9_]+)\s*\(", header))
    assert {"gnn_build_active_sets", "gnn_masked_spmm_fwd", "gnn_masked_spmm_bwd", "gnn_linear_fwd", "gnn_linear_bwd",
            "gnn_sample_boundary"} <= declared
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_version(lib):
    assert lib.gnn_version() >= 100


def _csr(n_rows=4, n_cols=4, nnz=0, rp=1, ci=None):
    return B.gnn_csr(n_rows, n_cols, nnz, rp, ci)


def test_bad_arguments_return_codes_without_touching_the_gpu(lib):
    need = C.c_size_t(0)
    # NULL graph
    assert lib.gnn_build_active_sets(None, None, None, 0, 2, None, None, None, None, None, C.byref(need), None) == 1
    assert b"NULL" in lib.gnn_last_error()
    g = _csr()
    # L < 1
    assert lib.gnn_build_active_sets(C.byref(g), None, None, 0, 0, None, None, None, None, None, C.byref(need), None) == 1
    # non-square graph
    g2 = _csr(n_rows=4, n_cols=5)
    assert lib.gnn_build_active_sets(C.byref(g2), None, None, 0, 2, None, None, None, None, None, C.byref(need), None) == 2
    # nnz >= 2^31
    g3 = _csr(nnz=2**31, ci=1)
    assert lib.gnn_masked_spmm_fwd(C.byref(g3), None, 0, None, C.c_int64(4), None, C.c_int64(4), 4, 0, None, None, None, None, None) == 4
    # ws_bytes NULL
    assert lib.gnn_build_active_sets(C.byref(g), None, None, 0, 2, None, None, None, None, None, None, None) == 1
    # leading dimension smaller than F
    assert lib.gnn_masked_spmm_fwd(C.byref(g), None, 0, None, C.c_int64(3), None, C.c_int64(4), 4, 0, None, None, None, None, None) == 2
    # unknown dtype
    assert lib.gnn_masked_spmm_fwd(C.byref(g), None, 0, None, C.c_int64(4), None, C.c_int64(4), 4, 7, None, None, None, None, None) == 4
    # aggregation: the size query of a call the column-blocked route does not apply to reports 0 bytes
    need.value = 77
    assert lib.gnn_masked_spmm_fwd(C.byref(g), None, 4, None, C.c_int64(4), None, C.c_int64(4), 4, 0, None, None, None,
                                   C.byref(need), None) == 0 and need.value == 0
    # linear: K = 0, X_self without W_self, dims over the limit
    assert lib.gnn_linear_fwd(None, 0, None, None, C.c_int64(4), 0, None, None, None, 4, None, C.c_int64(4), 0, 0, None,
                              C.byref(need), None) == 1
    assert lib.gnn_linear_fwd(None, 0, None, C.c_void_p(256), C.c_int64(4), 4, None, None, None, 4, None, C.c_int64(4), 0, 0,
                              None, C.byref(need), None) == 1
    assert lib.gnn_linear_fwd(None, 0, None, None, C.c_int64(5000), 5000, None, None, None, 4, None, C.c_int64(4), 0, 0, None,
                              C.byref(need), None) == 4
    # the forward transform without a workspace: weights beyond what the library's static array holds
    assert lib.gnn_linear_fwd_static(None, 0, None, None, C.c_int64(2048), 2048, None, None, None, 1024, None, C.c_int64(1024), 0, 0,
                                     None) == 4
    assert b"static array" in lib.gnn_last_error()
    # sampling: negative fanout, hops != 1
    assert lib.gnn_sample_boundary(C.byref(g), None, None, 0, -1, 1, C.c_uint64(0), None, None, C.c_int64(0), None, None, None,
                                   C.byref(need), None) == 1
    assert lib.gnn_sample_boundary(C.byref(g), None, None, 0, 5, 2, C.c_uint64(0), None, None, C.c_int64(0), None, None, None,
                                   C.byref(need), None) == 4
    # softmax: too many classes
    assert lib.gnn_softmax_ce(None, 0, None, C.c_int64(5000), 5000, None, None, C.c_int64(0), 0, None, None, C.byref(need),
                              None) == 4


def test_workspace_query_and_too_small_workspace(lib):
    g = _csr(n_rows=1000, n_cols=1000)
    need = C.c_size_t(0)
    assert lib.gnn_build_active_sets(C.byref(g), None, None, 0, 3, None, None, None, None, None, C.byref(need), None) == 0
    assert need.value >= 1000 * 4 and need.value % 256 == 0
    small = C.c_size_t(256)
    assert lib.gnn_build_active_sets(C.byref(g), None, None, 0, 3, None, None, None, None, C.c_void_p(4096), C.byref(small), None) == 3
    assert b"workspace too small" in lib.gnn_last_error()
    # misaligned workspace
    big = C.c_size_t(1 << 30)
    assert lib.gnn_build_active_sets(C.byref(g), None, None, 0, 3, None, None, None, None, C.c_void_p(4100), C.byref(big), None) == 1
    need2 = C.c_size_t(0)
    assert lib.gnn_linear_bwd(None, 100000, None, None, C.c_int64(256), 1, None, None, C.c_int64(608), 602, None, None, 256, None,
                              None, None, None, None, C.c_int64(0), 0, None, C.byref(need2), None) == 0
    assert need2.value > 100000 * 256 * 4


def test_product_package_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2311_06837_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text and "liboracle" not in text, f
