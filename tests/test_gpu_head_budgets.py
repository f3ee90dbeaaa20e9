"""Head-specific budgets (named as future work in Appendix A): every (layer, KV head) keeps its own number of keys."""
import numpy as np
import pytest
import torch

from workload import recipe
import tri_harness as H

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("seq_len", [700, 9000])   # 256-thread and 1024-thread selection kernels
def test_head_budgets(oracle, seq_len):
    cfg = recipe.scaled(recipe.CONFIGS["c2_layer"], n_layers=2, n_seqs=2, n_q_heads=8, n_kv_heads=2, seq_len=seq_len,
                        min_seq_len=seq_len // 3, budget=300, n_calib=128)
    budgets = np.array([[300, 37], [0, 5000]], dtype=np.int32)     # 5000 is read as the common budget, 300
    eff = np.minimum(budgets, cfg.budget)
    w = recipe.generate(cfg)
    run = H.GpuRun(cfg, w, head_budgets=budgets)
    stats = oracle.centers(w["q_samples"])
    run.centers.copy_(torch.from_numpy(stats))
    final, raw = run.score()
    G = cfg.group
    for fused in (False, True):
        run.kept_idx.fill_(-1)
        run.kept_cnt.fill_(-1)
        if fused:
            kd, vd, pd = torch.zeros_like(run.k), torch.zeros_like(run.v), torch.zeros_like(run.pos)
            dst = run.B.Cache(kd, vd, pd, run.seq_len, run.cur_pos, run.nmax)
            run.B.tri_compress_step(run.model, run.centers, run.cache, dst, cfg.budget, run.kept_idx, run.kept_cnt,
                                    run.new_len, run.ws)
            torch.cuda.synchronize()
            idx, cnt = run.kept_idx.cpu().numpy(), run.kept_cnt.cpu().numpy()
        else:
            idx, cnt = run.select()
        for l in range(cfg.n_layers):
            for s in range(cfg.n_seqs):
                n = int(w["seq_len"][s])
                for h in range(cfg.n_kv_heads):
                    b = int(eff[l, h])
                    assert cnt[l, s, h] == min(n, b)
                    ref32 = oracle.topk(final[l, s, h, :n].astype(np.float64), b) if b else np.zeros(0, np.int32)
                    if not fused:   # integer work on the same fp32 scores: identical
                        np.testing.assert_array_equal(idx[l, s, h, :len(ref32)], ref32)
                    else:
                        ref = oracle.head_instance(stats[l, h * G:(h + 1) * G], w["k"][l, s, h, :n], w["pos"][l, s, h, :n],
                                                   int(w["cur_pos"][s]), cfg.rope_theta, cfg.offsets, max(b, 1), threads=8)
                        if b:
                            H.check_kept(idx[l, s, h], int(cnt[l, s, h]), ref["final"], ref["idx"], n, b)
                        c = int(cnt[l, s, h])
                        sel = idx[l, s, h, :c]
                        np.testing.assert_array_equal(H.to_numpy(kd)[l, s, h, :c], w["k"][l, s, h][sel])
                        np.testing.assert_array_equal(H.to_numpy(vd)[l, s, h, :c], w["v"][l, s, h][sel])
                        np.testing.assert_array_equal(pd.cpu().numpy()[l, s, h, :c], w["pos"][l, s, h][sel])
                    assert np.all(idx[l, s, h, int(cnt[l, s, h]):] == -1)   # entries past the count are not written
