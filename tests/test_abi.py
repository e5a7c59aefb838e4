"""The C-ABI library loads and exports every function the public header declares (no GPU needed)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    src = open(os.path.join(ROOT, "include", "capgnn.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(capgnn_[a-z0-9_]+)\s*\(", src)))


def test_header_declares_the_named_entry_points():
    names = declared_functions()
    for must in ["capgnn_cache_build", "capgnn_halo_gather", "capgnn_spmm_fwd", "capgnn_spmm_bwd",
                 "capgnn_layer_fwd", "capgnn_layer_bwd", "capgnn_epoch"]:
        assert must in names


def test_library_exports_every_declared_symbol():
    from paper_2508_13716_amd import binding
    if not os.path.exists(binding.SO_PATH):
        pytest.fail("libcapgnn.so has not been built: run `python -m paper_2508_13716_amd.build`")
    lib = ctypes.CDLL(binding.SO_PATH)
    missing = [n for n in declared_functions() if not hasattr(lib, n)]
    assert not missing, missing
    # and the binding declares a signature for each of them
    assert sorted(binding.SIGNATURES) == declared_functions()


def test_host_only_entry_points_work_without_a_gpu():
    import numpy as np
    from paper_2508_13716_amd import binding as B
    assert B.version() >= 100
    assert B.cal_capacity(24, 1024, [602, 256, 256], 10**9) == 5542204
    assert B.cal_capacity(0.5, 512, [128, 64], 1000) == 0
    gb, hb, sb = B.cache_sizes(1000, 300, [602, 256], B.F32)
    assert gb >= 300 * (2416 + 1024) and hb >= 700 * (2416 + 1024) and sb == hb
    rowptr = np.array([0, 2, 2, 5], np.int64)
    r, c = B.norm_scales(B.NORM_SYM, 3, 2, rowptr, np.array([4, 0], np.int64))
    np.testing.assert_allclose(r, [2 ** -0.5, 1.0, 3 ** -0.5], rtol=1e-7)
    np.testing.assert_allclose(c, [2 ** -0.5, 1.0, 3 ** -0.5, 0.5, 1.0], rtol=1e-7)
    r, c = B.norm_scales(B.NORM_MEAN, 3, 2, rowptr, None)
    np.testing.assert_allclose(r, [0.5, 0.0, 1 / 3], rtol=1e-7)
    assert (c == 1).all()
    with pytest.raises(B.CapgnnError):
        B.cal_capacity(1, 0, [0], 10)
