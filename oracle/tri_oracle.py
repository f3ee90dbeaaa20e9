"""ctypes wrapper around the CPU oracle (tri_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  It imports nothing from the HIP package and the
HIP package imports nothing from here.

Arrays are numpy; bf16 data is passed as uint16 bit patterns and widened
exactly inside the C code.
"""
import ctypes
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tri_oracle.c")
_LIB = os.path.join(_HERE, "libtri_oracle.so")

F32, BF16 = 0, 1
PAIR_INTERLEAVED, PAIR_HALF = 0, 1


def build(force=False):
    """Compile tri_oracle.c with gcc (no fast-math: libm cos/atan2/hypot as they are)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        vp, i32, i64, dbl = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_double
        L.tri_oracle_omega.restype = dbl
        L.tri_oracle_omega.argtypes = [dbl, i32, i32]
        L.tri_oracle_centers.restype = i32
        L.tri_oracle_centers.argtypes = [vp, i32, i64, i32, i32, i32, i32, vp]
        L.tri_oracle_mrl.restype = i32
        L.tri_oracle_mrl.argtypes = [vp, i64, i32, vp]
        L.tri_oracle_band_contrib.restype = i32
        L.tri_oracle_band_contrib.argtypes = [vp, vp, i32, i32, i32, i32, i32, vp, vp]
        L.tri_oracle_s_trig.restype = dbl
        L.tri_oracle_s_trig.argtypes = [vp, vp, i32, i64, i32, i32, dbl, i64]
        for name in ("tri_oracle_s_norm", "tri_oracle_s_norm_mrl", "tri_oracle_s_norm0"):
            fn = getattr(L, name)
            fn.restype = dbl
            fn.argtypes = [vp, vp, i32, i64, i32, i32]
        L.tri_oracle_score_avg.restype = dbl
        L.tri_oracle_score_avg.argtypes = [vp, vp, i32, i64, i32, i32, dbl, i64, i64, vp, i32]
        L.tri_oracle_raw_scores.restype = i32
        L.tri_oracle_raw_scores.argtypes = [vp, i32, vp, i32, i64, vp, i64, i64, i32, i32, dbl, vp, i32, vp]
        L.tri_oracle_raw_scores_ex.restype = i32
        L.tri_oracle_raw_scores_ex.argtypes = [vp, i32, vp, i32, i64, vp, i64, i64, i32, i32, dbl, vp, i32, i32, i32, vp]
        L.tri_oracle_unrotate_key.restype = None
        L.tri_oracle_unrotate_key.argtypes = [vp, i32, i64, i32, i32, dbl, i64, vp]
        L.tri_oracle_gqa_final.restype = i32
        L.tri_oracle_gqa_final.argtypes = [vp, i32, i64, vp, vp, vp]
        L.tri_oracle_topk.restype = i32
        L.tri_oracle_topk.argtypes = [vp, i64, i64, vp, vp]
        L.tri_oracle_compact_rows.restype = i32
        L.tri_oracle_compact_rows.argtypes = [vp, i64, i64, vp, i32, vp, i64]
        L.tri_oracle_compact_fill.restype = i32
        L.tri_oracle_compact_fill.argtypes = [vp, i64, i64, vp, i32]
        L.tri_oracle_paged_gather.restype = i32
        L.tri_oracle_paged_gather.argtypes = [vp, i64, i64, vp, i32, i32, i64, i64, i64, i64, i32, i32, i32, i64, vp]
        L.tri_oracle_paged_compact.restype = i32
        L.tri_oracle_paged_compact.argtypes = [vp, i64, i64, vp, i32, i32, i64, i64, i64, i64, i32, i32, i32, vp, i32]
        _lib = L
    return _lib


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _dtype_code(a):
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    raise TypeError("oracle takes float32 or bf16-as-uint16 arrays, got %s" % a.dtype)


def _c(a, dtype=None):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def omega(theta, d, f):
    return lib().tri_oracle_omega(float(theta), int(d), int(f))


def centers(q, pairs=PAIR_INTERLEAVED):
    """q [T][L][Hq][d] float32 or bf16(uint16) -> stats [L][Hq][F][3] float32."""
    q = _c(q)
    T, L, Hq, d = q.shape
    out = np.empty((L, Hq, d // 2, 3), dtype=np.float32)
    rc = lib().tri_oracle_centers(_ptr(q), _dtype_code(q), T, L, Hq, d, pairs, _ptr(out))
    assert rc == 0
    return out


def mrl(stats):
    """stats [..., F, 3] -> R_f [..., F] float64 (Appendix B.5)."""
    stats = _c(stats, np.float32)
    F = stats.shape[-2]
    out = np.empty(stats.shape[:-1], dtype=np.float64)
    rc = lib().tri_oracle_mrl(_ptr(stats), stats.size // (3 * F), F, _ptr(out))
    assert rc == 0
    return out


def band_contrib(qstats, kstats, top_k):
    """qstats [L][Hq][F][3], kstats [L][Hkv][F][3] -> (C_f [L][Hq][F] float64, dominant bands [L][Hq][top_k] int32)."""
    qstats, kstats = _c(qstats, np.float32), _c(kstats, np.float32)
    L, Hq, F, _ = qstats.shape
    contrib = np.empty((L, Hq, F), dtype=np.float64)
    top = np.empty((L, Hq, top_k), dtype=np.int32)
    rc = lib().tri_oracle_band_contrib(_ptr(qstats), _ptr(kstats), L, Hq, kstats.shape[1], F, top_k, _ptr(contrib), _ptr(top))
    assert rc == 0
    return contrib, top


def s_trig(stats, key, theta, dist, pairs=PAIR_INTERLEAVED):
    stats = _c(stats, np.float32)
    key = _c(key)
    return lib().tri_oracle_s_trig(_ptr(stats), _ptr(key), _dtype_code(key), 0, key.shape[-1], pairs,
                                   float(theta), int(dist))


def s_norm(stats, key, pairs=PAIR_INTERLEAVED, mrl_form=False):
    stats = _c(stats, np.float32)
    key = _c(key)
    fn = lib().tri_oracle_s_norm_mrl if mrl_form else lib().tri_oracle_s_norm
    return fn(_ptr(stats), _ptr(key), _dtype_code(key), 0, key.shape[-1], pairs)


def score_avg(stats, key, theta, p_q, p_k, offsets, pairs=PAIR_INTERLEAVED):
    stats = _c(stats, np.float32)
    key = _c(key)
    off = _c(offsets, np.int64)
    return lib().tri_oracle_score_avg(_ptr(stats), _ptr(key), _dtype_code(key), 0, key.shape[-1], pairs,
                                      float(theta), int(p_q), int(p_k), _ptr(off), len(off))


VARIANT_FULL, VARIANT_TRIG_ONLY, VARIANT_NORM_ONLY, VARIANT_NORM_UNWEIGHTED = 0, 1, 2, 3


def s_norm0(stats, key, pairs=PAIR_INTERLEAVED):
    stats = _c(stats, np.float32)
    key = _c(key)
    return lib().tri_oracle_s_norm0(_ptr(stats), _ptr(key), _dtype_code(key), 0, key.shape[-1], pairs)


def unrotate_key(key, theta, p_k, pairs=PAIR_INTERLEAVED):
    """A stored post-RoPE key [d] -> the pre-RoPE key, float64 [d]."""
    key = _c(key)
    out = np.empty(key.shape[-1], dtype=np.float64)
    lib().tri_oracle_unrotate_key(_ptr(key), _dtype_code(key), 0, key.shape[-1], pairs, float(theta), int(p_k), _ptr(out))
    return out


def raw_scores(stats, K, pos, cur_pos, theta, offsets, pairs=PAIR_INTERLEAVED, threads=1, variant=VARIANT_FULL,
               rotated=False):
    """stats [G][F][3], K [N][d], pos [N] -> raw [G][N] float64.

    variant: one of the VARIANT_* scoring variants; rotated: K holds post-RoPE keys.

    threads > 1 only splits the keys into row ranges handed to a thread pool; every key is
    still scored by the same C routine, independently of the others."""
    stats = _c(stats, np.float32)
    K = _c(K)
    pos = _c(pos, np.int32)
    off = _c(offsets, np.int64)
    G = stats.shape[0]
    N, d = K.shape
    L = lib()

    def run(n0, n1):
        part = np.empty((G, n1 - n0), dtype=np.float64)
        Kc, pc = K[n0:n1], pos[n0:n1]
        if variant == VARIANT_FULL and not rotated:
            rc = L.tri_oracle_raw_scores(_ptr(stats), G, _ptr(Kc), _dtype_code(K), d, _ptr(pc), n1 - n0,
                                         int(cur_pos), d, pairs, float(theta), _ptr(off), len(off), _ptr(part))
        else:
            rc = L.tri_oracle_raw_scores_ex(_ptr(stats), G, _ptr(Kc), _dtype_code(K), d, _ptr(pc), n1 - n0,
                                            int(cur_pos), d, pairs, float(theta), _ptr(off), len(off), int(variant),
                                            int(bool(rotated)), _ptr(part))
        assert rc == 0
        return part

    threads = max(1, min(int(threads), max(1, N // 64)))
    if threads == 1 or N == 0:
        return run(0, N)
    step = -(-N // (threads * 4))
    bounds = [(a, min(N, a + step)) for a in range(0, N, step)]
    with ThreadPoolExecutor(max_workers=threads) as ex:
        parts = list(ex.map(lambda b: run(*b), bounds))
    return np.concatenate(parts, axis=1)


def gqa_final(raw):
    """raw [G][N] float64 -> (mu [G], sigma [G], final [N])."""
    raw = _c(raw, np.float64)
    G, N = raw.shape
    mu = np.empty(G)
    sigma = np.empty(G)
    final = np.empty(N)
    rc = lib().tri_oracle_gqa_final(_ptr(raw), G, N, _ptr(mu), _ptr(sigma), _ptr(final))
    assert rc == 0
    return mu, sigma, final


def topk(final, B):
    """final [N] -> ascending kept indices (min(N, B) of them), ties to the lower index."""
    final = _c(final, np.float64)
    N = final.shape[0]
    idx = np.empty(max(min(N, B), 1), dtype=np.int32)
    cnt = ctypes.c_int32(0)
    rc = lib().tri_oracle_topk(_ptr(final), N, int(B), _ptr(idx), ctypes.byref(cnt))
    assert rc == 0
    return idx[: cnt.value].copy()


def compact_rows(src, idx, out=None):
    """Row j of the result is row idx[j] of src (2-D, any dtype); out may be src itself."""
    assert src.ndim == 2 and src.flags.c_contiguous
    idx = _c(idx, np.int32)
    if out is None:
        out = np.zeros((len(idx), src.shape[1]), dtype=src.dtype)
    rb = src.shape[1] * src.itemsize
    rc = lib().tri_oracle_compact_rows(_ptr(src), src.strides[0], rb, _ptr(idx), len(idx), _ptr(out),
                                       out.strides[0])
    assert rc == 0
    return out


def compact_fill(rows, idx):
    """In place on a 2-D C-contiguous array: the kept rows at or beyond len(idx) fill the free slots below it."""
    assert rows.ndim == 2 and rows.flags.c_contiguous
    idx = _c(idx, np.int32)
    rc = lib().tri_oracle_compact_fill(_ptr(rows), rows.strides[0], rows.shape[1] * rows.itemsize, _ptr(idx), len(idx))
    assert rc == 0
    return rows


def paged_gather(pool, row_elems, block_table, block_size, strides, layer, seq, head, N):
    """Rows 0..N-1 of one head-instance from a paged pool; strides = (layer, block, head, slot) in elements."""
    bt = _c(block_table, np.int32)
    out = np.empty((N, row_elems), dtype=pool.dtype)
    rc = lib().tri_oracle_paged_gather(_ptr(pool), pool.itemsize, row_elems, _ptr(bt), bt.shape[1], block_size,
                                       *[int(s) for s in strides], layer, seq, head, N, _ptr(out))
    assert rc == 0
    return out


def paged_compact(pool, row_elems, block_table, block_size, strides, layer, seq, head, idx):
    bt = _c(block_table, np.int32)
    idx = _c(idx, np.int32)
    assert pool.flags.c_contiguous
    rc = lib().tri_oracle_paged_compact(_ptr(pool), pool.itemsize, row_elems, _ptr(bt), bt.shape[1], block_size,
                                        *[int(s) for s in strides], layer, seq, head, _ptr(idx), len(idx))
    assert rc == 0


def head_instance(stats, K, pos, cur_pos, theta, offsets, B, pairs=PAIR_INTERLEAVED, threads=1, variant=VARIANT_FULL,
                  rotated=False):
    """The whole step for one head-instance: raw scores, final scores, kept indices."""
    raw = raw_scores(stats, K, pos, cur_pos, theta, offsets, pairs, threads=threads, variant=variant, rotated=rotated)
    mu, sigma, final = gqa_final(raw)
    idx = topk(final, B)
    return dict(raw=raw, mu=mu, sigma=sigma, final=final, idx=idx)
