"""Host-side checks that need no GPU: the library loads, exports every symbol the
header declares, and rejects malformed CSR input before touching the device."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2004_13940_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2004_13940_amd import build
        build.build()
    return binding.load()


def test_every_declared_symbol_is_exported(lib):
    from paper_2004_13940_amd import binding
    header = open(os.path.join(ROOT, "include", "fm.h")).read()
    declared = set(re.findall(r"\b(fm_[a-z0-9_]+)\s*\(", header))
    assert declared, "no declarations found"
    for name in sorted(declared):
        assert hasattr(lib, name), f"{name} declared in fm.h but not exported"
    assert declared == set(binding.EXPORTS)


def test_params_struct_layout_matches_header():
    from paper_2004_13940_amd import binding
    assert ctypes.sizeof(binding.fm_params) == 11 * 4
    assert [f[0] for f in binding.fm_params._fields_] == [
        "K", "loss", "lambda_w", "lambda_v", "eta", "loss_scale", "update_w0", "reg_full_per_cell",
        "refresh_all_rows", "stale_aux", "half_gather"]


def test_enumerators_of_the_binding_match_the_header():
    """Every FM_* enumerator the header defines has the same value in the binding."""
    from paper_2004_13940_amd import binding
    header = open(os.path.join(ROOT, "include", "fm.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    found = dict(re.findall(r"\b(FM_[A-Z0-9_]+)\s*=\s*(-?\d+)", header))
    assert {"FM_OK", "FM_LOSS_LOGISTIC", "FM_OPT_GRAPH", "FM_OPT_DENSE_ROWS"} <= set(found)
    for name, value in found.items():
        assert getattr(binding, name) == int(value), name


def _try_build(lib, N, D, rowptr, col, val):
    rowptr = np.asarray(rowptr, np.int64)
    col = np.asarray(col, np.int32)
    val = np.asarray(val, np.float32)
    h = ctypes.c_void_p(None)
    rc = lib.fm_build_csr(ctypes.c_int64(N), ctypes.c_int64(D), ctypes.c_int64(len(col)),
                          ctypes.c_void_p(rowptr.ctypes.data), ctypes.c_void_p(col.ctypes.data),
                          ctypes.c_void_p(val.ctypes.data), ctypes.c_void_p(None), ctypes.byref(h))
    return rc, (lib.fm_last_error(None) or b"").decode(), h


@pytest.mark.parametrize("rowptr,col,code", [
    ([0, 2, 1, 3], [0, 1, 2], -3),      # rowptr not monotone
    ([1, 2, 3, 3], [0, 1, 2], -3),      # rowptr[0] != 0
    ([0, 1, 2, 2], [0, 1, 2], -3),      # rowptr[N] != nnz
    ([0, 2, 3, 3], [1, 0, 2], -3),      # columns descending inside a row
    ([0, 2, 3, 3], [1, 1, 2], -3),      # duplicate column inside a row
    ([0, 2, 3, 3], [0, 4, 2], -4),      # column outside [0, D)
    ([0, 2, 3, 3], [-1, 1, 2], -4),     # negative column
])
def test_malformed_csr_is_rejected_on_the_host(lib, rowptr, col, code):
    rc, msg, h = _try_build(lib, 3, 4, rowptr, col, [1.0, 2.0, 3.0])
    assert rc == code and msg and not h.value


def test_null_and_oversized_arguments(lib):
    h = ctypes.c_void_p(None)
    rc = lib.fm_build_csr(ctypes.c_int64(1), ctypes.c_int64(1), ctypes.c_int64(0), ctypes.c_void_p(None),
                          ctypes.c_void_p(None), ctypes.c_void_p(None), ctypes.c_void_p(None), ctypes.byref(h))
    assert rc == -1
    rp = np.zeros(2, np.int64)
    rc = lib.fm_build_csr(ctypes.c_int64(1), ctypes.c_int64(1 << 31), ctypes.c_int64(0),
                          ctypes.c_void_p(rp.ctypes.data), ctypes.c_void_p(None), ctypes.c_void_p(None),
                          ctypes.c_void_p(None), ctypes.byref(h))
    assert rc == -4
    assert lib.fm_destroy(ctypes.c_void_p(None)) == 0
    assert lib.fm_profile_kernels() == 8


def test_binding_refuses_to_run_without_a_gpu():
    import torch
    if torch.cuda.is_available():
        pytest.skip("GPU present")
    from paper_2004_13940_amd import binding
    with pytest.raises(RuntimeError):
        binding.Matrix(1, 1, np.array([0, 0]), np.array([], np.int32), np.array([], np.float32))
