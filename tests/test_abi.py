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


def _fake_cache(T, n_seqs=2, max_seq_len=4096, block_size=0, base=0x10000000):
    """A descriptor over made-up device addresses: enough for the host-side checks, which never dereference them."""
    d = 128
    c = T.TriCache()
    c.k, c.v, c.pos = base, base + (1 << 30), base + (2 << 30)
    c.dtype, c.n_seqs = T.TRI_BF16, n_seqs
    c.seq_len, c.cur_pos = base + (3 << 30), base + (3 << 30) + 4096
    c.max_seq_len, c.block_size = max_seq_len, block_size
    c.block_table, c.max_blocks_per_seq = (base + (3 << 30) + 8192, max_seq_len // block_size) if block_size else (0, 0)
    c.stride_slot, c.stride_head = d, max_seq_len * d
    c.stride_seq_or_block, c.stride_layer = 8 * max_seq_len * d, n_seqs * 8 * max_seq_len * d
    c.pos_stride_head, c.pos_stride_seq_or_block, c.pos_stride_layer = max_seq_len, 8 * max_seq_len, n_seqs * 8 * max_seq_len
    return c


def test_limits_and_in_place_rules_are_checked_before_anything_is_enqueued():
    import numpy as np
    from paper_2604_04921_amd import binding as T
    L = T.lib()
    offs = np.array([1, 2, 4], dtype=np.int64)
    op = offs.ctypes.data_as(ctypes.c_void_p)
    m = T.TriModel(2, 32, 8, 128, 1e6, 0, 3, op, 0)
    src = _fake_cache(T)
    idx, cnt = 0x70000000, 0x70100000
    # in place, but the second descriptor maps slots differently: refused, whichever entry point is used
    dst = _fake_cache(T)
    dst.stride_head *= 2
    assert L.tri_compact(ctypes.byref(m), ctypes.byref(src), ctypes.byref(dst), 512, idx, cnt, None, None) == T.TRI_ERR_INVALID_ARG
    assert b"maps slots differently" in L.tri_last_error()
    assert L.tri_compress_step(ctypes.byref(m), 0x60000000, ctypes.byref(src), ctypes.byref(dst), 512, idx, cnt, None,
                               0x50000000, 1 << 40, None) == T.TRI_ERR_INVALID_ARG
    # a separate paged destination sized for the budget only is accepted by the checks (none of this reaches a launch:
    # the next check, the workspace, fails on purpose)
    dst = _fake_cache(T, max_seq_len=512, block_size=16, base=0x200000000)
    assert L.tri_compress_step(ctypes.byref(m), 0x60000000, ctypes.byref(src), ctypes.byref(dst), 512, idx, cnt, None,
                               None, 0, None) == T.TRI_ERR_WORKSPACE
    dst.max_blocks_per_seq = 512 // 16 - 1   # one block short of the budget
    assert L.tri_compress_step(ctypes.byref(m), 0x60000000, ctypes.byref(src), ctypes.byref(dst), 512, idx, cnt, None,
                               None, 0, None) == T.TRI_ERR_INVALID_ARG
    # grid limits
    big = T.TriModel(70000, 32, 8, 128, 1e6, 0, 3, op, 0)
    assert L.tri_compress_step(ctypes.byref(big), 0x60000000, ctypes.byref(src), None, 512, idx, cnt, None, None, 0, None) \
        == T.TRI_ERR_UNSUPPORTED
    wide = _fake_cache(T, n_seqs=9000)
    assert L.tri_score(ctypes.byref(m), 0x60000000, ctypes.byref(wide), 0x61000000, None, 0x50000000, 1 << 45, None) \
        == T.TRI_ERR_UNSUPPORTED
    # the minimal-move eviction's budget limit is part of the up-front checks of the fused step
    assert L.tri_compress_step(ctypes.byref(m), 0x60000000, ctypes.byref(src), None, 1 << 17, idx, cnt, None, None, 0, None) \
        == T.TRI_ERR_UNSUPPORTED


def test_static_scratch_entry_point_validates_like_the_fused_step():
    import numpy as np
    from paper_2604_04921_amd import binding as T
    L = T.lib()
    assert T.tri_static_scratch_size() == 64 << 20
    offs = np.array([1, 2, 4], dtype=np.int64)
    m = T.TriModel(2, 32, 8, 128, 1e6, 0, 3, offs.ctypes.data_as(ctypes.c_void_p), 0)
    c = T.TriCache()
    assert L.tri_compress_step_static(ctypes.byref(m), None, ctypes.byref(c), None, 16, None, None, None, None) \
        == T.TRI_ERR_INVALID_ARG
    src = _fake_cache(T, n_seqs=64, max_seq_len=65536)   # far more scratch than the array holds
    assert L.tri_compress_step_static(ctypes.byref(m), 0x60000000, ctypes.byref(src), None, 2048, 0x70000000, 0x70100000,
                                      None, None) == T.TRI_ERR_WORKSPACE
    assert b"scratch" in L.tri_last_error()
