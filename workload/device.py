"""Device-side generator: the recipe of workload.recipe at full size, written straight into HBM.

Centres, sequence lengths and block tables come from the host recipe (same seeds, so the same
centres as the CPU generator); the bulk tensors (keys, values, calibration queries) are filled by
the HIP kernels of gen.hip, and positions by torch.  Inputs only -- no scoring arithmetic."""
import ctypes
import os
import subprocess

import numpy as np
import torch

from . import recipe

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gen.hip")
LIB_PATH = os.path.join(_HERE, "libtri_workload.so")


PROBE_SRC = os.path.join(_HERE, "inst_probe.hip")
PROBE_PATH = os.path.join(_HERE, "inst_probe")


def build(verbose=False):
    """The generator's library and the instruction-rate probe (a stand-alone program)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = ["--offload-arch=gfx950", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
    for cmd in ([hipcc, *flags, "-O3", "-fPIC", "-shared", _SRC, "-o", LIB_PATH],
                [hipcc, *flags, "-O2", PROBE_SRC, "-o", PROBE_PATH]):
        res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if res.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + res.stdout)
    return LIB_PATH


def inst_probe():
    """Runs the instruction-rate probe on the current GPU (as a child process) and returns its table."""
    if not os.path.exists(PROBE_PATH):
        raise RuntimeError("workload/inst_probe is not built (workload.device.build())")
    res = subprocess.run([PROBE_PATH], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    if res.returncode != 0:
        raise RuntimeError("inst_probe failed:\n" + res.stdout)
    return res.stdout


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libtri_workload.so is not built (workload.device.build())")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, u64, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_uint64, ctypes.c_float
        L.wl_fill_samples.restype = i32
        L.wl_fill_samples.argtypes = [vp, i32, vp, i64, i64, i64, i64, f32, f32, f32, u64, u64, vp]
        L.wl_fill_normal.restype = i32
        L.wl_fill_normal.argtypes = [vp, i32, i64, u64, u64, vp]
        L.wl_stream_probe.restype = i64
        L.wl_stream_probe.argtypes = [vp, i64, vp, i32, i32, vp]
        _lib = L
    return _lib


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _centres_tensor(c):
    """complex [n][F] -> float32 [n][F][2] on the device."""
    a = np.stack([c.real, c.imag], axis=-1).astype(np.float32)
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def fill_samples(out, centres, B, C, Dn, noise, outlier_p, outlier_scale, seed, tag):
    assert out.is_contiguous() and out.shape[-1] == 128
    rows = out.numel() // 128
    rc = lib().wl_fill_samples(out.data_ptr(), int(out.dtype == torch.bfloat16), centres.data_ptr(), rows, B, C, Dn,
                               noise, outlier_p, outlier_scale, seed, tag, _stream())
    assert rc == 0


def fill_normal(out, seed, tag):
    assert out.is_contiguous()
    rc = lib().wl_fill_normal(out.data_ptr(), int(out.dtype == torch.bfloat16), out.numel(), seed, tag, _stream())
    assert rc == 0


def generate(cfg, positions=None, layers=None, layer0=0):
    """The workload of `cfg` on cuda:0 as torch tensors.

    positions overrides cfg.positions ("dense"; "sparse" / "sparse16": sorted unique draws from [0, 2N) / [0, 16N);
    "scattered": the draws of "sparse16" left in random slot order); layers overrides cfg.n_layers (layer slabs
    for configurations that do not fit in HBM at once) and layer0 is the slab's first layer: the slab holds layers
    layer0 .. layer0 + layers - 1 of the configuration, each with its own centres and noise).  Returns a dict with q_samples, k, v, pos,
    seq_len, cur_pos and, for paged configurations, block_table (k, v, pos are then block pools)."""
    L = cfg.n_layers if layers is None else layers
    S, Hq, Hkv, F, N = cfg.n_seqs, cfg.n_q_heads, cfg.n_kv_heads, cfg.n_bands, cfg.seq_len
    dt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    mode = positions or cfg.positions
    assert 0 <= layer0 and layer0 + L <= max(cfg.n_layers, L)
    qc = recipe.draw_centres(recipe._rng(cfg.seed, 1), (max(cfg.n_layers, layer0 + L), Hq), F)[layer0:layer0 + L]
    kc = recipe.draw_centres(recipe._rng(cfg.seed, 2), (max(cfg.n_layers, layer0 + L), Hkv), F)[layer0:layer0 + L]
    tag0 = 1000 * layer0   # a slab's noise differs from the other slabs'

    qc_t, kc_t = _centres_tensor(qc.reshape(-1, F)), _centres_tensor(kc.reshape(-1, F))
    out = {}
    q = torch.empty((cfg.n_calib, L, Hq, 2 * F), dtype=dt, device="cuda")
    fill_samples(q, qc_t, cfg.n_calib, L * Hq, 1, cfg.noise, 0.0, 1.0, cfg.seed, 3 + tag0)
    out["q_samples"] = q
    lens = recipe.seq_lens(cfg)
    out["seq_len"] = torch.from_numpy(lens).cuda()
    spread = {"dense": 1, "sparse": 2, "sparse16": 16, "scattered": 16}[mode]
    cur = spread * lens
    out["cur_pos"] = torch.from_numpy(cur.astype(np.int32)).cuda()
    if cfg.block_size:
        bs = cfg.block_size
        bt, nb = recipe.paged_layout(cfg, lens)
        out["block_table"] = torch.from_numpy(bt).cuda()
        k = torch.empty((L, nb, Hkv, bs, 2 * F), dtype=dt, device="cuda")
        fill_samples(k, kc_t, nb, Hkv, bs, cfg.noise, cfg.outlier_p, cfg.outlier_scale, cfg.seed, 4 + tag0)
        v = torch.empty_like(k)
        fill_normal(v, cfg.seed, 5 + tag0)
        # slot n of sequence s holds position n: scatter the arange through the block table
        pos = torch.zeros((L, nb, Hkv, bs), dtype=torch.int32, device="cuda")
        btd = out["block_table"]
        for s in range(S):
            nblk = -(-int(lens[s]) // bs)
            p = torch.arange(nblk * bs, dtype=torch.int32, device="cuda").view(nblk, 1, bs)
            pos[:, btd[s, :nblk].long()] = p.expand(nblk, Hkv, bs)
        assert mode == "dense"
    else:
        k = torch.empty((L, S, Hkv, N, 2 * F), dtype=dt, device="cuda")
        fill_samples(k, kc_t, S, Hkv, N, cfg.noise, cfg.outlier_p, cfg.outlier_scale, cfg.seed, 4 + tag0)
        v = torch.empty_like(k)
        fill_normal(v, cfg.seed, 5 + tag0)
        if mode == "dense":
            pos = torch.arange(N, dtype=torch.int32, device="cuda").expand(L, S, Hkv, N).contiguous()
        else:
            g = torch.Generator(device="cuda")
            g.manual_seed(cfg.seed + 6)
            pos = torch.empty((L, S, Hkv, N), dtype=torch.int32, device="cuda")
            for l in range(L):      # unique draws from [0, spread * N) per head-instance
                r = torch.rand((S * Hkv, spread * N), generator=g, device="cuda")
                sel = r.argsort(dim=1)[:, :N]
                if mode != "scattered":   # "scattered": slot order unrelated to position (after minimal-move evictions)
                    sel = sel.sort(dim=1).values
                pos[l] = sel.to(torch.int32).view(S, Hkv, N)
                del r, sel
    out["k"], out["v"], out["pos"] = k, v, pos
    torch.cuda.synchronize()
    return out


def hbm_probe(gib=16, reps=5):
    """Streaming-read rate of this GPU, alone and with a thin write stream mixed in (1 write byte per 16 / 64 /
    256 read bytes), with plain loads and with loads that carry the non-temporal hint.  Returns {label: GB/s of
    reads}."""
    n = gib << 30
    src = torch.empty(n, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty(n // 16 + 64, dtype=torch.uint8, device="cuda")
    out = {}
    for nt in (0, 1):
        for label, every in (("read_only", 0), ("read_with_1/16_writes", 1), ("read_with_1/64_writes", 4),
                             ("read_with_1/256_writes", 16)):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            got = lib().wl_stream_probe(src.data_ptr(), n, dst.data_ptr(), every, nt, _stream())
            assert got > 0
            e0.record()
            for _ in range(reps):
                lib().wl_stream_probe(src.data_ptr(), n, dst.data_ptr(), every, nt, _stream())
            e1.record()
            torch.cuda.synchronize()
            out[label + ("/nt_loads" if nt else "")] = round(got * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1)
    return out
