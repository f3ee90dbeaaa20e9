"""Seeded sweep over combinations of the options (group size, storage type, pair layout, paged / contiguous,
pre- / post-RoPE keys, score variant, in-place or not, offsets, sequence lengths around tile and group edges):
every combination runs the whole path against the oracle."""
import numpy as np
import pytest

from workload import recipe

import tri_harness as H
from test_gpu_parity import run_and_check

pytestmark = pytest.mark.gpu


def _cases(n=28, seed=20260409):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        group = int(rng.integers(1, 9))
        kv = int(rng.integers(1, 4))
        dtype = "bf16" if rng.random() < 0.7 else "f32"
        paged = bool(rng.random() < 0.4)
        block = int(rng.choice([4, 8, 16, 32, 64])) if paged else 0
        seq_len = int(rng.choice([15, 16, 17, 63, 64, 65, 255, 256, 257, 300, 511, 777, 1025, 1300]))
        out.append(dict(
            id="%02d-G%d-%s-%s" % (i, group, dtype, "paged%d" % block if paged else "contig"),
            group=group, kv=kv, dtype=dtype, paged=paged, block=block, seq_len=seq_len,
            min_len=int(rng.integers(0, seq_len + 1)), budget=int(rng.integers(1, seq_len + 40)),
            pairs=int(rng.integers(0, 2)), rotated=bool(rng.random() < 0.4), variant=int(rng.integers(0, 4)),
            inplace=bool(rng.random() < 0.5), n_seqs=int(rng.integers(1, 4)), n_layers=int(rng.integers(1, 3)),
            sparse=bool(rng.random() < 0.5), n_off=int(rng.choice([1, 3, 16, 31])), seed=1000 + i))
    return out


@pytest.mark.parametrize("case", _cases(), ids=lambda c: c["id"])
def test_option_combination(oracle, case):
    c = case
    base = recipe.CONFIGS["c4_paged" if c["paged"] else "c2_layer"]
    cfg = recipe.scaled(base, n_layers=c["n_layers"], n_seqs=c["n_seqs"], n_q_heads=c["group"] * c["kv"],
                        n_kv_heads=c["kv"], seq_len=c["seq_len"], min_seq_len=c["min_len"], budget=c["budget"],
                        n_calib=64, dtype=c["dtype"], block_size=c["block"], n_offsets=c["n_off"],
                        positions="dense" if c["paged"] or not c["sparse"] else "sparse", seed=c["seed"])

    def mutate(w):
        if c["pairs"]:
            for name in ("k", "q_samples"):
                x = w[name]
                w[name] = np.ascontiguousarray(np.concatenate([x[..., 0::2], x[..., 1::2]], axis=-1))
        if c["rotated"]:
            w["k"] = H.to_post_rope(w["k"], w["pos"], cfg.rope_theta, c["pairs"], cfg.dtype)

    run_and_check(oracle, cfg, paged=c["paged"], inplace=c["inplace"] or c["paged"], pairs=c["pairs"], mutate=mutate,
                  variant=c["variant"], rotated=c["rotated"])
