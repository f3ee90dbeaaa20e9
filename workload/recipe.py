"""Seeded synthetic KV caches for the compression step: the configurations and the CPU generator.

This module holds input generation only -- no scoring, selection or compaction arithmetic --
and is the one piece the oracle-side tests and the HIP-side tests both use.

Recipe (all draws from numpy's Philox stream keyed by the seed and a tensor tag):
  * centre of a head in band f: magnitude LogNormal(mu=0, sigma=1), phase U[0, 2pi)
  * sample = centre + complex Gaussian noise with E|noise|^2 = (noise * |centre_f|)^2
    (each real component N(0, (noise*|centre_f|)^2 / 2)); noise = 0.3 gives a per-band Mean
    Resultant Length of about 0.978, the concentration the paper measures on Qwen3-8B
  * keys: with probability outlier_p the whole key vector is multiplied by outlier_scale
  * values: unit Gaussian
  * queries for calibration: n_calib samples per (layer, query head) drawn like the keys,
    without outliers; the statistics table comes from running them through the centre build
  * band f occupies elements (2f, 2f+1) of a head vector (interleaved pairs)
  * storage dtype bf16 (round to nearest even) or float32
"""
from dataclasses import dataclass, field, replace
from typing import Optional, Tuple

import numpy as np

SEED_BASE = 0x7A1A77


@dataclass(frozen=True)
class Config:
    name: str
    n_layers: int
    n_seqs: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    rope_theta: float
    seq_len: int                 # N for every sequence, or the maximum when ragged
    budget: int
    n_offsets: int               # D = {2^0 .. 2^(n_offsets-1)}
    dtype: str                   # "bf16" or "f32"
    positions: str               # "dense": 0..N-1, cur_pos = N; "sparse": sorted unique draws from [0, 2N)
    outlier_p: float = 0.01
    outlier_scale: float = 5.0
    noise: float = 0.3
    n_calib: int = 4096
    min_seq_len: Optional[int] = None   # ragged: lengths uniform in [min_seq_len, seq_len]
    block_size: int = 0                 # 0 contiguous, 16 paged
    seed: int = SEED_BASE
    offset_list: Optional[tuple] = None # an explicit offset set (e.g. linear spacing) instead of the powers of two

    @property
    def group(self):
        return self.n_q_heads // self.n_kv_heads

    @property
    def n_bands(self):
        return self.head_dim // 2

    @property
    def offsets(self):
        if self.offset_list is not None:
            return np.array(self.offset_list, dtype=np.int64)
        return np.array([1 << j for j in range(self.n_offsets)], dtype=np.int64)


# The five workloads: Qwen3-8B geometry (32 query / 8 KV heads, d = 128, theta = 1e6), 32K-token
# caches and budget 2048 stand in for the paper's AIME / MATH-500 generation runs.
CONFIGS = {
    "c1_tiny": Config("c1_tiny", 1, 1, 4, 1, 128, 1e6, 4096, 512, 16, "f32", "dense", seed=SEED_BASE + 1),
    "c2_layer": Config("c2_layer", 1, 1, 32, 8, 128, 1e6, 32768, 2048, 16, "bf16", "sparse", seed=SEED_BASE + 2),
    "c3_model": Config("c3_model", 36, 16, 32, 8, 128, 1e6, 32768, 2048, 16, "bf16", "dense", seed=SEED_BASE + 3),
    "c4_paged": Config("c4_paged", 36, 64, 32, 8, 128, 1e6, 65536, 2048, 16, "bf16", "dense",
                       min_seq_len=4096, block_size=16, seed=SEED_BASE + 4),
    "c5_long": Config("c5_long", 64, 1, 64, 8, 128, 1e6, 131072, 4096, 32, "bf16", "dense",
                      outlier_p=0.05, outlier_scale=10.0, seed=SEED_BASE + 5),
    # Steady state of the paper's policy (Section 4.3): budget + one window of 128 new tokens per head-instance,
    # survivors at scattered positions; many short head-instances instead of few long ones.
    "steady_state": Config("steady_state", 36, 64, 32, 8, 128, 1e6, 2176, 2048, 16, "bf16", "sparse",
                           seed=SEED_BASE + 6),
}


def scaled(cfg: Config, **kw) -> Config:
    """A smaller copy of a configuration for CPU-sized tests."""
    return replace(cfg, **kw)


def _rng(seed, tag):
    return np.random.Generator(np.random.Philox(key=[seed & 0xFFFFFFFFFFFFFFFF, tag]))


def to_bf16_bits(x):
    """float32 -> bf16 bit patterns (uint16), round to nearest even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + r) >> 16).astype(np.uint16)


def bf16_bits_to_f32(b):
    return (b.astype(np.uint32) << 16).view(np.float32)


def store(x, dtype):
    """Round a float array to the storage dtype: uint16 bit patterns for bf16, float32 otherwise."""
    return to_bf16_bits(x) if dtype == "bf16" else np.ascontiguousarray(x, dtype=np.float32)


def draw_centres(rng, shape_heads, n_bands):
    """Complex centres [*shape_heads][F]."""
    mag = rng.lognormal(0.0, 1.0, size=shape_heads + (n_bands,))
    ph = rng.uniform(0.0, 2 * np.pi, size=shape_heads + (n_bands,))
    return mag * np.exp(1j * ph)


def draw_samples(rng, centres, n, noise, outlier_p=0.0, outlier_scale=1.0):
    """n samples around each centre: complex [*heads][n][F]."""
    sh = centres.shape[:-1] + (n, centres.shape[-1])
    sd = noise * np.abs(centres)[..., None, :] / np.sqrt(2.0)
    z = centres[..., None, :] + sd * (rng.standard_normal(sh) + 1j * rng.standard_normal(sh))
    if outlier_p > 0:
        out = rng.random(sh[:-1]) < outlier_p
        z = z * np.where(out, outlier_scale, 1.0)[..., None]
    return z


def interleave(z):
    """complex [...][F] -> float32 [...][2F] with band f at (2f, 2f+1)."""
    out = np.empty(z.shape[:-1] + (2 * z.shape[-1],), dtype=np.float32)
    out[..., 0::2] = z.real
    out[..., 1::2] = z.imag
    return out


def seq_lens(cfg: Config):
    if cfg.min_seq_len is None:
        return np.full(cfg.n_seqs, cfg.seq_len, dtype=np.int32)
    return _rng(cfg.seed, 7).integers(cfg.min_seq_len, cfg.seq_len + 1, size=cfg.n_seqs).astype(np.int32)


def generate(cfg: Config):
    """The whole workload on the host (for configurations small enough for it).

    Returns a dict:
      q_samples [T][L][Hq][d]           storage dtype
      k, v      [L][S][Hkv][N][d]       storage dtype (contiguous layout)
      pos       [L][S][Hkv][N] int32    (per head: heads keep different tokens once compacted)
      seq_len   [S] int32, cur_pos [S] int32
    """
    L, S, Hq, Hkv, F, N = cfg.n_layers, cfg.n_seqs, cfg.n_q_heads, cfg.n_kv_heads, cfg.n_bands, cfg.seq_len
    qc = draw_centres(_rng(cfg.seed, 1), (L, Hq), F)
    kc = draw_centres(_rng(cfg.seed, 2), (L, Hkv), F)
    q = draw_samples(_rng(cfg.seed, 3), qc, cfg.n_calib, cfg.noise)          # [L][Hq][T][F]
    q = np.ascontiguousarray(np.transpose(interleave(q), (2, 0, 1, 3)))       # [T][L][Hq][d]
    rk = _rng(cfg.seed, 4)
    k = np.empty((L, S, Hkv, N, 2 * F), dtype=np.float32)
    for s in range(S):
        k[:, s] = interleave(draw_samples(rk, kc, N, cfg.noise, cfg.outlier_p, cfg.outlier_scale))
    v = _rng(cfg.seed, 5).standard_normal((L, S, Hkv, N, 2 * F)).astype(np.float32)
    lens = seq_lens(cfg)
    pos = np.zeros((L, S, Hkv, N), dtype=np.int32)
    cur = np.zeros(S, dtype=np.int32)
    rp = _rng(cfg.seed, 6)
    for s in range(S):
        n = int(lens[s])
        if cfg.positions == "dense":
            pos[:, s, :, :n] = np.arange(n, dtype=np.int32)
            cur[s] = n
        else:
            for l in range(L):
                for h in range(Hkv):
                    pos[l, s, h, :n] = np.sort(rp.choice(2 * n, size=n, replace=False)).astype(np.int32)
            cur[s] = 2 * n
    return dict(q_samples=store(q, cfg.dtype), k=store(k, cfg.dtype), v=store(v, cfg.dtype), pos=pos,
                seq_len=lens, cur_pos=cur, q_centres=qc, k_centres=kc)


def paged_layout(cfg: Config, lens, seed_tag=8):
    """Block table for a paged pool: every sequence gets ceil(N_s / block) blocks, scattered by a
    seeded permutation over the pool.  Returns (block_table [S][max_blocks] int32, n_blocks)."""
    bs = cfg.block_size
    need = [-(-int(n) // bs) for n in lens]
    n_blocks = int(sum(need))
    perm = _rng(cfg.seed, seed_tag).permutation(n_blocks).astype(np.int32)
    mb = max(max(need), -(-int(cfg.seq_len) // bs))   # the table spans the configured maximum length
    bt = np.zeros((len(lens), mb), dtype=np.int32)
    o = 0
    for s, nb in enumerate(need):
        bt[s, :nb] = perm[o:o + nb]
        o += nb
    return bt, n_blocks


def to_paged(x, lens, bt, n_blocks, bs):
    """contiguous [L][S][Hkv][N][w] -> paged pool [L][n_blocks][Hkv][bs][w] following the block table."""
    L, S, H, N, w = x.shape
    pool = np.zeros((L, n_blocks, H, bs, w), dtype=x.dtype)
    for s in range(S):
        n = int(lens[s])
        for b in range(-(-n // bs)):
            m = min(bs, n - b * bs)
            pool[:, bt[s, b], :, :m] = x[:, s, :, b * bs:b * bs + m]
    return pool

