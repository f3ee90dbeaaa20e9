"""tri_compact_fill (minimal-move in-place eviction, Section 4.3) against the oracle's compact_fill, bit for bit.

The kept sets are crafted here (any ascending subset is a legal input), so the cases cover what the selection
step rarely produces: nothing to move, everything to move, a single hole, budgets that are not a multiple of 32,
and the steady-state shape (a budget of keys plus one window of 128 new ones).
"""
import numpy as np
import pytest
import torch

from workload import recipe
from tri_harness import GpuRun, to_numpy

pytestmark = pytest.mark.gpu


def kept_sets(cfg, lens, kind, rng):
    """[L][S][Hkv][B] ascending kept indices (-1 beyond the count) and the counts."""
    L, S, H, B = cfg.n_layers, cfg.n_seqs, cfg.n_kv_heads, cfg.budget
    idx = np.full((L, S, H, B), -1, dtype=np.int32)
    cnt = np.zeros((L, S, H), dtype=np.int32)
    for l in range(L):
        for s in range(S):
            n = int(lens[s])
            c = min(n, B)
            for h in range(H):
                if kind == "random":
                    sel = np.sort(rng.choice(n, size=c, replace=False))
                elif kind == "prefix":        # nothing moves
                    sel = np.arange(c)
                elif kind == "suffix":        # every kept key lies as far back as possible
                    sel = np.arange(n - c, n)
                elif kind == "one_hole":      # a single free slot takes the last key
                    sel = np.arange(c)
                    if n > c:
                        sel = np.concatenate([np.delete(sel, (l + s + h) % c), [n - 1]])
                else:
                    raise ValueError(kind)
                idx[l, s, h, :c] = sel
                cnt[l, s, h] = c
    return idx, cnt


def run_fill(oracle, cfg, kind, paged=False):
    w = recipe.generate(cfg)
    lens = w["seq_len"]
    rng = np.random.default_rng(cfg.seed + 17)
    idx, cnt = kept_sets(cfg, lens, kind, rng)
    run = GpuRun(cfg, w, paged=paged)
    run.kept_idx.copy_(torch.from_numpy(idx))
    run.kept_cnt.copy_(torch.from_numpy(cnt))
    run.B.tri_compact_fill(run.model, run.cache, cfg.budget, run.kept_idx, run.kept_cnt, run.new_len)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(run.new_len.cpu().numpy(), np.minimum(lens, cfg.budget))
    got = {"k": to_numpy(run.k), "v": to_numpy(run.v), "pos": run.pos.cpu().numpy()}
    bs = cfg.block_size
    for l in range(cfg.n_layers):
        for s in range(cfg.n_seqs):
            n = int(lens[s])
            for h in range(cfg.n_kv_heads):
                c = int(cnt[l, s, h])
                for name in ("k", "v", "pos"):
                    ref = np.ascontiguousarray(w[name][l, s, h, :n]).reshape(n, -1).copy()
                    oracle.compact_fill(ref, idx[l, s, h, :c])
                    if paged:
                        blocks = run.bt_np[s, : -(-n // bs)]
                        g = got[name][l, blocks, h].reshape(len(blocks) * bs, -1)[:n]
                    else:
                        g = got[name][l, s, h, :n].reshape(n, -1)
                    np.testing.assert_array_equal(g, ref, err_msg="%s l=%d s=%d h=%d" % (name, l, s, h))
    if not paged:   # nothing beyond the sequences' own slots was touched
        for name in ("k", "v", "pos"):
            for s in range(cfg.n_seqs):
                np.testing.assert_array_equal(got[name][:, s, :, int(lens[s]):], w[name][:, s, :, int(lens[s]):])


@pytest.mark.parametrize("kind", ["random", "prefix", "suffix", "one_hole"])
def test_fill_contiguous_bf16(oracle, kind):
    cfg = recipe.scaled(recipe.CONFIGS["c2_layer"], n_layers=2, n_seqs=3, n_q_heads=8, n_kv_heads=2, seq_len=777,
                        min_seq_len=90, budget=203, n_calib=128)
    run_fill(oracle, cfg, kind)


def test_fill_fp32(oracle):
    cfg = recipe.scaled(recipe.CONFIGS["c1_tiny"], n_layers=1, n_seqs=2, seq_len=300, budget=64)
    run_fill(oracle, cfg, "random")


@pytest.mark.parametrize("kind", ["random", "suffix"])
def test_fill_paged(oracle, kind):
    cfg = recipe.scaled(recipe.CONFIGS["c4_paged"], n_layers=2, n_seqs=3, n_q_heads=8, n_kv_heads=2, seq_len=900,
                        min_seq_len=100, budget=160, n_calib=128)
    run_fill(oracle, cfg, kind, paged=True)


def test_fill_steady_state_shape(oracle):
    """Budget 2048 plus one window of 128 new tokens: at most 128 moves per head-instance."""
    cfg = recipe.scaled(recipe.CONFIGS["steady_state"], n_layers=1, n_seqs=2, n_q_heads=8, n_kv_heads=2, n_calib=128)
    run_fill(oracle, cfg, "random")


def test_fill_large_budget(oracle):
    """More than 256 bitmap words (the free-slot scan takes several passes) and a budget-sized move list."""
    cfg = recipe.scaled(recipe.CONFIGS["c2_layer"], n_layers=1, n_seqs=1, n_q_heads=8, n_kv_heads=2, seq_len=20000,
                        budget=9001, n_calib=128)
    run_fill(oracle, cfg, "suffix")
    run_fill(oracle, cfg, "random")
