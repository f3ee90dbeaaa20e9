"""The entry point that allocates nothing (tri_compress_step_static, the library's own scratch array) against
tri_compress_step with a caller's workspace: identical kept slots, counts, lengths and compacted K / V / positions,
on two calls in a row, the second on a smaller input (the array keeps the first call's contents)."""
import numpy as np
import pytest
import torch

from workload import recipe

import tri_harness as H

pytestmark = pytest.mark.gpu


def _step(run, cfg, static):
    """One in-place step on a fresh copy of the cache; returns what the step wrote."""
    B = run.B
    k, v, pos = run.k.clone(), run.v.clone(), run.pos.clone()
    cache = B.Cache(k, v, pos, run.seq_len, run.cur_pos, run.nmax, run.block_table)
    idx = torch.full_like(run.kept_idx, -1)
    cnt = torch.full_like(run.kept_cnt, -1)
    new_len = torch.full_like(run.new_len, -1)
    if static:
        B.tri_compress_step_static(run.model, run.centers, cache, cache, cfg.budget, idx, cnt, new_len)
    else:
        ws = torch.empty_like(run.ws)
        B.tri_compress_step(run.model, run.centers, cache, cache, cfg.budget, idx, cnt, new_len, ws)
    torch.cuda.synchronize()
    return [t.cpu().numpy() for t in (idx, cnt, new_len, k.view(torch.int16) if k.dtype == torch.bfloat16 else k,
                                      v.view(torch.int16) if v.dtype == torch.bfloat16 else v, pos)]


def _compare(cfg, paged):
    w = recipe.generate(cfg)
    run = H.GpuRun(cfg, w, paged=paged)
    run.build_centers()
    from paper_2604_04921_amd import binding as B
    assert B.tri_workspace_size(run.model, run.cache, cfg.budget) <= B.tri_static_scratch_size()
    ref = _step(run, cfg, static=False)
    got = _step(run, cfg, static=True)
    cnt = ref[1]
    assert np.array_equal(got[1], cnt) and np.array_equal(got[2], ref[2])
    keep = np.arange(cfg.budget)[None, None, None, :] < cnt[..., None]
    assert np.array_equal(got[0][keep], ref[0][keep])   # entries past the count are not written
    for a, b in zip(got[3:], ref[3:]):
        assert np.array_equal(a, b)                      # whole caches, bit for bit
    assert int(cnt.min()) >= 0 and int(cnt.max()) == min(cfg.budget, int(w["seq_len"].max()))


def test_static_scratch_twice_second_call_smaller():
    big = recipe.scaled(recipe.CONFIGS["c2_layer"], n_layers=2, n_seqs=3, seq_len=20000, min_seq_len=9000, budget=1024,
                        n_calib=128)
    small = recipe.scaled(recipe.CONFIGS["c2_layer"], n_layers=1, n_seqs=2, seq_len=3000, min_seq_len=500, budget=700, block_size=16,
                          n_calib=128)
    _compare(big, paged=False)
    _compare(small, paged=True)


def test_static_scratch_refuses_what_does_not_fit():
    from paper_2604_04921_amd import binding as B
    cfg = recipe.scaled(recipe.CONFIGS["c2_layer"], n_layers=1, n_seqs=1, seq_len=256, min_seq_len=256, budget=64, n_calib=64)
    w = recipe.generate(cfg)
    run = H.GpuRun(cfg, w)
    run.build_centers()
    # the same buffers described as a cache far larger than the array (nothing may be enqueued, so nothing is read)
    huge = B.Cache(run.k, run.v, run.pos, run.seq_len, run.cur_pos, 1 << 24)
    assert B.tri_workspace_size(run.model, huge, cfg.budget) > B.tri_static_scratch_size()
    with pytest.raises(B.TriError) as e:
        B.tri_compress_step_static(run.model, run.centers, huge, huge, cfg.budget, run.kept_idx, run.kept_cnt, run.new_len)
    assert e.value.status == B.TRI_ERR_WORKSPACE and "scratch" in str(e.value)
    torch.cuda.synchronize()
