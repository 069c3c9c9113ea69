"""CPU-side checks of the boundary: the C-ABI library loads and exports every symbol that
include/gcn.h declares, and host-side argument validation works without a GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "gcn.h")
LIB = os.path.join(ROOT, "paper_2212_05009_amd", "libgcn.so")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        import __graft_entry__
        __graft_entry__.build()
    import torch  # noqa: F401  (loads the HIP runtime the library binds to)
    return ctypes.CDLL(LIB)


def declared_functions():
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    return sorted(set(re.findall(r"\b(gcn_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_documented_entry_points():
    names = declared_functions()
    for need in ["gcn_csr_build", "gcn_spmm", "gcn_spmm_t", "gcn_halo_gather", "gcn_layer_fwd", "gcn_layer_bwd",
                 "gcn_softmax_xent", "gcn_csr_free", "gcn_csr_info", "gcn_csr_arrays", "gcn_last_error"]:
        assert need in names


def test_library_exports_every_declared_symbol(lib):
    for name in declared_functions():
        assert hasattr(lib, name), f"libgcn.so does not export {name}"


def test_argument_validation_without_gpu(lib):
    lib.gcn_last_error.restype = ctypes.c_char_p
    out = ctypes.c_void_p()
    i64 = ctypes.c_int64
    # n_global < 1
    rc = lib.gcn_csr_build(None, None, i64(0), i64(0), i64(0), i64(0), None, 0, None, ctypes.byref(out))
    assert rc == -1 and b"n_global" in lib.gcn_last_error() and not out.value
    # block without global degrees
    rc = lib.gcn_csr_build(None, None, i64(0), i64(10), i64(2), i64(5), None, 0, None, ctypes.byref(out))
    assert rc == -1 and b"d_deg_global" in lib.gcn_last_error()
    # NULL handle
    assert lib.gcn_spmm(None, None, i64(1), 1, 0, None, i64(1), 0, None, None, i64(0), None) == -1
    assert lib.gcn_csr_info(None, None, None, None) == -1
    assert lib.gcn_csr_free(None) == 0
    # gather: ld < d
    assert lib.gcn_halo_gather(None, i64(2), i64(4), 3, 0, None, i64(1), None, i64(3), None) == -1
    assert b"ld" in lib.gcn_last_error()
    # softmax: C < 1
    assert lib.gcn_softmax_xent(None, i64(1), i64(0), 0, 0, None, ctypes.c_float(1.0), None, None, i64(1), None) == -1


def test_tuning_setter_and_feature_pitch_without_gpu(lib):
    lib.gcn_last_error.restype = ctypes.c_char_p
    lib.gcn_feature_ld.restype = ctypes.c_int64
    assert lib.gcn_debug_set_tuning(b"GCN_NO_SUCH_RULE", 1) == -1 and b"unknown name" in lib.gcn_last_error()
    assert lib.gcn_debug_set_tuning(b"GCN_SPMM_SLICES", 9) == -1
    assert lib.gcn_debug_set_tuning(b"GCN_SPMM_SLICES", 4) == 0
    assert lib.gcn_debug_set_tuning(b"GCN_SPMM_SLICES", -2147483648) == 0        # back to the default
    assert lib.gcn_debug_set_tuning(None, 0) == -1
    # rows start on a 128-byte line and the pitch is an odd number of lines; rows within one line keep their width
    assert [lib.gcn_feature_ld(d, 0) for d in (16, 32, 47, 100, 128, 256, 602)] == [16, 32, 96, 160, 160, 288, 608]
    assert [lib.gcn_feature_ld(d, 1) for d in (47, 64, 100, 256)] == [47, 64, 192, 320]
    assert lib.gcn_feature_ld(0, 0) == -1 and lib.gcn_feature_ld(8, 7) == -1


def test_binding_refuses_cpu_tensors(lib):
    import torch
    import paper_2212_05009_amd as gcn
    with pytest.raises(TypeError):
        gcn.gcn_csr_build(torch.zeros(3, dtype=torch.int32), torch.zeros(3, dtype=torch.int32), 4)
