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


def fused_fill_against_the_three_calls(cfg, paged=False, head_budgets=None, mutate=None):
    """tri_compress_step with dst = NULL (eviction in place, fewest moves) against tri_score + tri_select_topk +
    tri_compact_fill on a second copy of the same cache: kept slots, counts, new lengths and every byte of K, V and
    the positions must agree (the selection on final scores and the one inside the fused step share their z-score,
    so the kept sets are the same bits)."""
    w = recipe.generate(cfg)
    if mutate is not None:
        mutate(w)
    a = GpuRun(cfg, w, paged=paged, head_budgets=head_budgets)
    b = GpuRun(cfg, w, paged=paged, head_budgets=head_budgets)
    a.build_centers()
    b.centers.copy_(a.centers)
    a.score()
    a.select()
    a.B.tri_compact_fill(a.model, a.cache, cfg.budget, a.kept_idx, a.kept_cnt, a.new_len)
    b.B.tri_compress_step(b.model, b.centers, b.cache, None, cfg.budget, b.kept_idx, b.kept_cnt, b.new_len, b.ws)
    torch.cuda.synchronize()
    cnt = a.kept_cnt.cpu().numpy()
    np.testing.assert_array_equal(b.kept_cnt.cpu().numpy(), cnt)
    np.testing.assert_array_equal(b.new_len.cpu().numpy(), a.new_len.cpu().numpy())
    ia, ib = a.kept_idx.cpu().numpy(), b.kept_idx.cpu().numpy()
    for l in range(cfg.n_layers):
        for s in range(cfg.n_seqs):
            for h in range(cfg.n_kv_heads):
                c = int(cnt[l, s, h])
                np.testing.assert_array_equal(ib[l, s, h, :c], ia[l, s, h, :c])
    for name in ("k", "v"):
        np.testing.assert_array_equal(to_numpy(getattr(b, name)), to_numpy(getattr(a, name)), err_msg=name)
    np.testing.assert_array_equal(b.pos.cpu().numpy(), a.pos.cpu().numpy())
    return cnt


def test_fused_fill_ragged_lengths():
    """Lengths below, at and above the budget, an empty sequence, one of a single key: the selection's workgroups do
    the eviction themselves (sequences of at most 4096 keys, budget at most 2048)."""
    cfg = recipe.scaled(recipe.CONFIGS["c2_layer"], n_layers=2, n_seqs=8, n_q_heads=8, n_kv_heads=2, seq_len=3000,
                        min_seq_len=3000, budget=300, n_calib=128)

    def lens(w):
        w["seq_len"][:] = np.array([3000, 0, 1, 299, 300, 301, 428, 2999], dtype=np.int32)
    cnt = fused_fill_against_the_three_calls(cfg, mutate=lens)
    assert cnt[0, :, 0].tolist() == [300, 0, 1, 299, 300, 300, 300, 300]


def test_fused_fill_head_budgets():
    cfg = recipe.scaled(recipe.CONFIGS["c2_layer"], n_layers=2, n_seqs=3, n_q_heads=8, n_kv_heads=2, seq_len=900,
                        min_seq_len=200, budget=300, n_calib=128)
    fused_fill_against_the_three_calls(cfg, head_budgets=np.array([[300, 37], [0, 5000]], dtype=np.int32))


def test_fused_fill_paged():
    cfg = recipe.scaled(recipe.CONFIGS["c4_paged"], n_layers=2, n_seqs=3, n_q_heads=8, n_kv_heads=2, seq_len=900,
                        min_seq_len=100, budget=160, n_calib=128)
    fused_fill_against_the_three_calls(cfg, paged=True)


def test_fused_fill_fp32():
    cfg = recipe.scaled(recipe.CONFIGS["c1_tiny"], n_layers=1, n_seqs=2, seq_len=300, budget=64)
    fused_fill_against_the_three_calls(cfg)


@pytest.mark.parametrize("seq_len,budget", [(4096, 2048), (4097, 2048), (4096, 2049), (9000, 700)])
def test_fused_fill_at_the_limits_of_the_short_kernel(seq_len, budget):
    """4096 keys and a budget of 2048 are the most the selection's own eviction takes; one more of either and the step
    launches tri_compact_fill's kernel after the selection, as it does for longer sequences."""
    cfg = recipe.scaled(recipe.CONFIGS["c2_layer"], n_layers=1, n_seqs=2, n_q_heads=8, n_kv_heads=2, seq_len=seq_len,
                        min_seq_len=seq_len, budget=budget, n_calib=128)
    fused_fill_against_the_three_calls(cfg)
