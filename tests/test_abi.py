"""The C-ABI library loads and exports every symbol include/tri.h declares (no compute calls here)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "tri.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tri_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_four_primitives():
    names = declared_symbols()
    for n in ("tri_build_centers", "tri_score", "tri_select_topk", "tri_compact"):
        assert n in names


def test_library_exports_every_declared_symbol():
    from paper_2604_04921_amd import binding
    assert os.path.exists(binding.LIB_PATH), "libtri.so is not built"
    lib = ctypes.CDLL(binding.LIB_PATH)
    for n in declared_symbols():
        assert hasattr(lib, n), n
    assert sorted(binding.EXPORTS) == declared_symbols()


def test_host_validation_rejects_bad_arguments():
    """Argument checks run on the host before any HIP call, so they can be exercised without a GPU."""
    import numpy as np
    from paper_2604_04921_amd import binding as T
    L = T.lib()
    offs = np.array([1, 2, 4], dtype=np.int64)
    m = T.TriModel(1, 4, 1, 64, 1e6, 0, 3, offs.ctypes.data_as(ctypes.c_void_p))       # head_dim 64: not built
    assert L.tri_build_centers(ctypes.byref(m), None, 0, 1, None, None) == T.TRI_ERR_UNSUPPORTED
    m = T.TriModel(1, 4, 3, 128, 1e6, 0, 3, offs.ctypes.data_as(ctypes.c_void_p))      # 4 % 3 != 0
    assert L.tri_build_centers(ctypes.byref(m), None, 0, 1, None, None) == T.TRI_ERR_INVALID_ARG
    m = T.TriModel(1, 4, 1, 128, 1e6, 0, 3, offs.ctypes.data_as(ctypes.c_void_p))
    assert L.tri_build_centers(ctypes.byref(m), None, 0, 1, None, None) == T.TRI_ERR_INVALID_ARG   # NULL pointers
    assert b"q_samples" in L.tri_last_error()
    assert L.tri_workspace_size(ctypes.byref(m), None, 16) == 0
    c = T.TriCache()
    assert L.tri_score(ctypes.byref(m), None, ctypes.byref(c), None, None, None, 0, None) == T.TRI_ERR_INVALID_ARG
    assert L.tri_timing_attach(None, 4) == T.TRI_ERR_INVALID_ARG
    assert L.tri_timing_detach() == 0
    # entry points added around the four primitives
    m = T.TriModel(1, 4, 1, 128, 1e6, 0, 3, offs.ctypes.data_as(ctypes.c_void_p), 7)   # unknown score variant
    assert L.tri_build_centers(ctypes.byref(m), None, 0, 1, None, None) == T.TRI_ERR_INVALID_ARG
    assert b"variant" in L.tri_last_error()
    m = T.TriModel(1, 4, 1, 128, 1e6, 0, 3, offs.ctypes.data_as(ctypes.c_void_p), 0)
    assert L.tri_centers_accumulate(ctypes.byref(m), None, 0, 1, None, 1, None) == T.TRI_ERR_INVALID_ARG
    assert L.tri_centers_finalize(ctypes.byref(m), None, 0, None, None) == T.TRI_ERR_INVALID_ARG
    assert L.tri_band_diagnostics(ctypes.byref(m), None, None, None, None, 0, None, None) == T.TRI_ERR_INVALID_ARG
    assert L.tri_compact_fill(ctypes.byref(m), ctypes.byref(c), 16, None, None, None, None) == T.TRI_ERR_INVALID_ARG
    assert L.tri_compress_step(ctypes.byref(m), None, ctypes.byref(c), None, 16, None, None, None, None, 0, None) \
        == T.TRI_ERR_INVALID_ARG
