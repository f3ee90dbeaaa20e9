"""The fused step enqueues kernels only (no allocation, no memset, no synchronisation), so a caller may record it into a
HIP graph: every replay must give what the eager call gives."""
from dataclasses import replace

import pytest
import torch

from workload import device, recipe

pytestmark = pytest.mark.gpu


def test_fused_step_replayed_from_a_graph():
    from paper_2604_04921_amd import binding as B
    cfg = replace(recipe.CONFIGS["steady_state"], n_seqs=2, n_layers=3)
    L, S, Hq, Hkv, Bk, d = cfg.n_layers, cfg.n_seqs, cfg.n_q_heads, cfg.n_kv_heads, cfg.budget, cfg.head_dim
    w = device.generate(cfg, positions=cfg.positions, layers=L)
    model = B.Model(L, Hq, Hkv, d, cfg.rope_theta, cfg.offsets)
    centers = torch.empty((L, Hq, d // 2, 3), dtype=torch.float32, device="cuda")
    B.tri_build_centers(model, w["q_samples"], centers)
    src = B.Cache(w["k"], w["v"], w["pos"], w["seq_len"], w["cur_pos"], cfg.seq_len, None)
    kd = torch.zeros((L, S, Hkv, Bk, d), dtype=w["k"].dtype, device="cuda")
    vd, pd = torch.zeros_like(kd), torch.zeros((L, S, Hkv, Bk), dtype=torch.int32, device="cuda")
    dst = B.Cache(kd, vd, pd, w["seq_len"], w["cur_pos"], Bk)
    kept_idx = torch.empty((L, S, Hkv, Bk), dtype=torch.int32, device="cuda")
    kept_cnt = torch.empty((L, S, Hkv), dtype=torch.int32, device="cuda")
    new_len = torch.empty((S,), dtype=torch.int32, device="cuda")
    ws = torch.empty(B.tri_workspace_size(model, src, Bk), dtype=torch.uint8, device="cuda")

    def step():
        B.tri_compress_step(model, centers, src, dst, Bk, kept_idx, kept_cnt, new_len, ws)

    def clear():
        for t in (kept_idx, kept_cnt, new_len, pd):
            t.fill_(-1)
        kd.zero_()
        vd.zero_()

    clear()
    step()
    torch.cuda.synchronize()
    ref = [t.clone() for t in (kept_idx, kept_cnt, new_len, pd, kd.view(torch.int16), vd.view(torch.int16))]
    assert int(kept_cnt.min()) == Bk

    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        step()   # everything the library sets up once per device happens outside the capture
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=stream, capture_error_mode="thread_local"):
            step()
    torch.cuda.synchronize()
    for rep in range(4):
        clear()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = (kept_idx, kept_cnt, new_len, pd, kd.view(torch.int16), vd.view(torch.int16))
        for a, b in zip(ref, got):
            assert torch.equal(a, b), "replay %d differs from the eager call" % rep
        # the program's own eager work and a synchronisation between the replays
        step()
        torch.cuda.synchronize()
