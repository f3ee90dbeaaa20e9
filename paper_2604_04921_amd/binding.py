"""ctypes binding of libtri.so: same entry points as include/tri.h, argument marshalling only.

torch owns the device memory and the stream; every step of the path runs inside the library.
"""
import ctypes
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtri.so")

TRI_OK = 0
TRI_ERR_INVALID_ARG, TRI_ERR_UNSUPPORTED, TRI_ERR_WORKSPACE, TRI_ERR_HIP = -1, -2, -3, -4
TRI_F32, TRI_BF16 = 0, 1
TRI_PAIR_INTERLEAVED, TRI_PAIR_HALF = 0, 1
TRI_SCORE_FULL, TRI_SCORE_TRIG_ONLY, TRI_SCORE_NORM_ONLY, TRI_SCORE_NORM_UNWEIGHTED = 0, 1, 2, 3

EXPORTS = ["tri_last_error", "tri_build_centers", "tri_centers_accumulate", "tri_centers_finalize", "tri_band_diagnostics", "tri_workspace_size", "tri_score", "tri_select_topk",
           "tri_compact", "tri_compact_fill", "tri_compress_step", "tri_static_scratch_size", "tri_compress_step_static",
           "tri_timing_attach", "tri_timing_detach"]


class TriModel(ctypes.Structure):
    _fields_ = [("n_layers", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("rope_theta", ctypes.c_double), ("pairs", ctypes.c_int32),
                ("n_offsets", ctypes.c_int32), ("offsets", ctypes.c_void_p), ("score_variant", ctypes.c_int32),
                ("head_budgets", ctypes.c_void_p)]


class TriCache(ctypes.Structure):
    _fields_ = [("k", ctypes.c_void_p), ("v", ctypes.c_void_p), ("pos", ctypes.c_void_p),
                ("dtype", ctypes.c_int32), ("n_seqs", ctypes.c_int32),
                ("seq_len", ctypes.c_void_p), ("cur_pos", ctypes.c_void_p),
                ("max_seq_len", ctypes.c_int32), ("block_size", ctypes.c_int32),
                ("block_table", ctypes.c_void_p), ("max_blocks_per_seq", ctypes.c_int32),
                ("stride_layer", ctypes.c_int64), ("stride_seq_or_block", ctypes.c_int64),
                ("stride_head", ctypes.c_int64), ("stride_slot", ctypes.c_int64),
                ("pos_stride_layer", ctypes.c_int64), ("pos_stride_seq_or_block", ctypes.c_int64),
                ("pos_stride_head", ctypes.c_int64), ("k_rotated", ctypes.c_int32)]


class TriError(RuntimeError):
    def __init__(self, status, msg):
        super().__init__("tri status %d: %s" % (status, msg))
        self.status = status


_lib = None


def lib():
    """Load libtri.so.  torch is imported first so that the HIP runtime it ships is the one in use."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libtri.so is not built (run paper_2604_04921_amd/build.py); there is no fallback")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
        L.tri_last_error.restype = ctypes.c_char_p
        L.tri_last_error.argtypes = []
        L.tri_build_centers.restype = i32
        L.tri_build_centers.argtypes = [ctypes.POINTER(TriModel), vp, i32, i64, vp, vp]
        L.tri_centers_accumulate.restype = i32
        L.tri_centers_accumulate.argtypes = [ctypes.POINTER(TriModel), vp, i32, i64, vp, i32, vp]
        L.tri_centers_finalize.restype = i32
        L.tri_centers_finalize.argtypes = [ctypes.POINTER(TriModel), vp, i64, vp, vp]
        L.tri_band_diagnostics.restype = i32
        L.tri_band_diagnostics.argtypes = [ctypes.POINTER(TriModel), vp, vp, vp, vp, i32, vp, vp]
        L.tri_workspace_size.restype = ctypes.c_size_t
        L.tri_workspace_size.argtypes = [ctypes.POINTER(TriModel), ctypes.POINTER(TriCache), i32]
        L.tri_score.restype = i32
        L.tri_score.argtypes = [ctypes.POINTER(TriModel), vp, ctypes.POINTER(TriCache), vp, vp, vp, ctypes.c_size_t, vp]
        L.tri_select_topk.restype = i32
        L.tri_select_topk.argtypes = [ctypes.POINTER(TriModel), vp, ctypes.POINTER(TriCache), i32, vp, vp, vp,
                                      ctypes.c_size_t, vp]
        L.tri_compact.restype = i32
        L.tri_compact.argtypes = [ctypes.POINTER(TriModel), ctypes.POINTER(TriCache), ctypes.POINTER(TriCache), i32,
                                  vp, vp, vp, vp]
        L.tri_compact_fill.restype = i32
        L.tri_compact_fill.argtypes = [ctypes.POINTER(TriModel), ctypes.POINTER(TriCache), i32, vp, vp, vp, vp]
        L.tri_compress_step.restype = i32
        L.tri_compress_step.argtypes = [ctypes.POINTER(TriModel), vp, ctypes.POINTER(TriCache),
                                        ctypes.POINTER(TriCache), i32, vp, vp, vp, vp, ctypes.c_size_t, vp]
        L.tri_static_scratch_size.restype = ctypes.c_size_t
        L.tri_static_scratch_size.argtypes = []
        L.tri_compress_step_static.restype = i32
        L.tri_compress_step_static.argtypes = [ctypes.POINTER(TriModel), vp, ctypes.POINTER(TriCache),
                                               ctypes.POINTER(TriCache), i32, vp, vp, vp, vp]
        L.tri_timing_attach.restype = i32
        L.tri_timing_attach.argtypes = [vp, i32]
        L.tri_timing_detach.restype = i32
        L.tri_timing_detach.argtypes = []
        _lib = L
    return _lib


def _check(rc):
    if rc != TRI_OK:
        raise TriError(rc, lib().tri_last_error().decode())


def _p(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _dtype(t):
    if t.dtype == torch.bfloat16:
        return TRI_BF16
    if t.dtype == torch.float32:
        return TRI_F32
    raise TypeError("float32 or bfloat16 tensors only, got %s" % t.dtype)


class Model:
    """Host-side tri_model; keeps the offsets array alive."""

    def __init__(self, n_layers, n_q_heads, n_kv_heads, head_dim, rope_theta, offsets, pairs=TRI_PAIR_INTERLEAVED,
                 score_variant=TRI_SCORE_FULL, head_budgets=None):
        self._offsets = np.ascontiguousarray(offsets, dtype=np.int64)
        self._head_budgets = head_budgets   # device int32 [n_layers][n_kv_heads] or None; kept alive here
        if head_budgets is not None:
            assert head_budgets.dtype == torch.int32 and head_budgets.is_contiguous()
            assert tuple(head_budgets.shape) == (n_layers, n_kv_heads)
        self.c = TriModel(n_layers, n_q_heads, n_kv_heads, head_dim, float(rope_theta), pairs, len(self._offsets),
                          self._offsets.ctypes.data_as(ctypes.c_void_p), int(score_variant),
                          None if head_budgets is None else head_budgets.data_ptr())

    @property
    def ref(self):
        return ctypes.byref(self.c)


class Cache:
    """tri_cache over torch tensors.

    contiguous: k, v [L][S][Hkv][N][d], pos [L][S][Hkv][N]
    paged:      k, v [L][n_blocks][Hkv][block][d], pos [L][n_blocks][Hkv][block], block_table [S][max_blocks]
    Strides are taken from the tensors; the last dimension must be dense."""

    def __init__(self, k, v, pos, seq_len, cur_pos, max_seq_len, block_table=None, k_rotated=False):
        assert k.dim() == 5 and pos.dim() == 4 and k.stride(4) == 1 and pos.stride(3) == 1
        assert v is None or (v.stride() == k.stride() and v.dtype == k.dtype)
        assert pos.dtype == torch.int32 and seq_len.dtype == torch.int32 and cur_pos.dtype == torch.int32
        self.tensors = (k, v, pos, seq_len, cur_pos, block_table)
        bs = 0 if block_table is None else k.shape[3]
        self.c = TriCache(k.data_ptr(), 0 if v is None else v.data_ptr(), pos.data_ptr(), _dtype(k),
                          seq_len.numel(), seq_len.data_ptr(), cur_pos.data_ptr(), int(max_seq_len), bs,
                          0 if block_table is None else block_table.data_ptr(),
                          0 if block_table is None else block_table.shape[1],
                          k.stride(0), k.stride(1), k.stride(2), k.stride(3),
                          pos.stride(0), pos.stride(1), pos.stride(2), int(bool(k_rotated)))
        if block_table is not None:
            assert block_table.dtype == torch.int32 and block_table.is_contiguous()

    @property
    def ref(self):
        return ctypes.byref(self.c)


def tri_build_centers(model, q_samples, centers_out, stream=None):
    """q_samples [T][L][Hq][d] (contiguous) -> centers_out [L][Hq][F][3] float32."""
    assert q_samples.is_contiguous() and centers_out.is_contiguous() and centers_out.dtype == torch.float32
    _check(lib().tri_build_centers(model.ref, _p(q_samples), _dtype(q_samples), q_samples.shape[0], _p(centers_out),
                                   _stream(stream)))


def tri_centers_accumulate(model, q_samples, sums, first, stream=None):
    """Adds the sums of one chunk q_samples [T][L][Hq][d] to sums [L][Hq][F][3] float64 (first: overwrite)."""
    assert q_samples.is_contiguous() and sums.is_contiguous() and sums.dtype == torch.float64
    _check(lib().tri_centers_accumulate(model.ref, _p(q_samples), _dtype(q_samples), q_samples.shape[0], _p(sums),
                                        int(bool(first)), _stream(stream)))


def tri_centers_finalize(model, sums, total_tokens, centers_out, stream=None):
    assert sums.is_contiguous() and sums.dtype == torch.float64 and centers_out.dtype == torch.float32
    _check(lib().tri_centers_finalize(model.ref, _p(sums), int(total_tokens), _p(centers_out), _stream(stream)))


def tri_band_diagnostics(model, q_centers, k_centers, mrl_out, contrib_out=None, top_k=0, top_bands_out=None, stream=None):
    _check(lib().tri_band_diagnostics(model.ref, _p(q_centers), _p(k_centers), _p(mrl_out), _p(contrib_out), int(top_k),
                                      _p(top_bands_out), _stream(stream)))


def tri_workspace_size(model, cache, budget):
    return int(lib().tri_workspace_size(model.ref, cache.ref, int(budget)))


def tri_score(model, centers, cache, final_out, raw_out, workspace, stream=None):
    _check(lib().tri_score(model.ref, _p(centers), cache.ref, _p(final_out), _p(raw_out), _p(workspace),
                           workspace.numel() * workspace.element_size(), _stream(stream)))


def tri_select_topk(model, final_scores, cache, budget, kept_idx, kept_cnt, workspace=None, stream=None):
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().tri_select_topk(model.ref, _p(final_scores), cache.ref, int(budget), _p(kept_idx), _p(kept_cnt),
                                 _p(workspace), ws_bytes, _stream(stream)))


def tri_compact(model, src, dst, budget, kept_idx, kept_cnt, new_seq_len=None, stream=None):
    _check(lib().tri_compact(model.ref, src.ref, dst.ref, int(budget), _p(kept_idx), _p(kept_cnt), _p(new_seq_len),
                             _stream(stream)))


def tri_compact_fill(model, cache, budget, kept_idx, kept_cnt, new_seq_len=None, stream=None):
    _check(lib().tri_compact_fill(model.ref, cache.ref, int(budget), _p(kept_idx), _p(kept_cnt), _p(new_seq_len),
                                  _stream(stream)))


def tri_compress_step(model, centers, src, dst, budget, kept_idx, kept_cnt, new_seq_len, workspace, stream=None):
    _check(lib().tri_compress_step(model.ref, _p(centers), src.ref, dst.ref if dst is not None else None, int(budget), _p(kept_idx), _p(kept_cnt),
                                   _p(new_seq_len), _p(workspace), workspace.numel() * workspace.element_size(),
                                   _stream(stream)))


def tri_static_scratch_size():
    return int(lib().tri_static_scratch_size())


def tri_compress_step_static(model, centers, src, dst, budget, kept_idx, kept_cnt, new_seq_len, stream=None):
    """tri_compress_step on the library's own scratch array: no workspace argument, no allocation."""
    _check(lib().tri_compress_step_static(model.ref, _p(centers), src.ref, dst.ref if dst is not None else None, int(budget),
                                          _p(kept_idx), _p(kept_cnt), _p(new_seq_len), _stream(stream)))


def tri_timing_attach(events):
    """events: list of torch.cuda.Event (timing enabled, each recorded once before so that its handle exists),
    laid out start0, stop0, start1, stop1, ...  Returns the ctypes array that must be kept alive until detach."""
    arr = (ctypes.c_void_p * len(events))(*[e.cuda_event for e in events])
    _check(lib().tri_timing_attach(arr, len(events) // 2))
    return arr


def tri_timing_detach():
    return int(lib().tri_timing_detach())
