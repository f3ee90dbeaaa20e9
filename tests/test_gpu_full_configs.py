"""The five benchmark configurations at full size on the GPU, in the launch configuration bench.py times
(tri_compress_step on a device-generated workload).  The oracle checks a few whole head-instances copied
back from the device; every head-instance is checked with properties that hold at any size: kept count,
ascending unique in-range indices, and bit-exact compacted K / V / positions."""
import numpy as np
import pytest
import torch

from workload import device, recipe

import tri_harness as H

pytestmark = pytest.mark.gpu


def instance_from_device(cfg, w, l, s, h):
    """K rows and positions of one head-instance as numpy, read through the block table when paged."""
    n = int(w["seq_len"][s])
    if "block_table" in w:
        bs = cfg.block_size
        bt = w["block_table"][s, : -(-n // bs)].long()
        k = w["k"][l, bt, h].reshape(-1, cfg.head_dim)[:n]
        p = w["pos"][l, bt, h].reshape(-1)[:n]
    else:
        k, p = w["k"][l, s, h, :n], w["pos"][l, s, h, :n]
    return H.to_numpy(k.contiguous()), p.cpu().numpy()


def run_full(oracle, cfg, picks, layers=None, positions=None):
    from paper_2604_04921_amd import binding as T
    L = layers or cfg.n_layers
    w = device.generate(cfg, positions=positions, layers=L)
    S, Hq, Hkv, B, d, G = cfg.n_seqs, cfg.n_q_heads, cfg.n_kv_heads, cfg.budget, cfg.head_dim, cfg.group
    dev = "cuda"
    model = T.Model(L, Hq, Hkv, d, cfg.rope_theta, cfg.offsets)
    paged = "block_table" in w
    src = T.Cache(w["k"], w["v"], w["pos"], w["seq_len"], w["cur_pos"], cfg.seq_len, w.get("block_table"))
    centers = torch.empty((L, Hq, d // 2, 3), dtype=torch.float32, device=dev)
    T.tri_build_centers(model, w["q_samples"], centers)
    kept_idx = torch.full((L, S, Hkv, B), -1, dtype=torch.int32, device=dev)
    kept_cnt = torch.full((L, S, Hkv), -1, dtype=torch.int32, device=dev)
    new_len = torch.full((S,), -1, dtype=torch.int32, device=dev)
    ws = torch.empty(T.tri_workspace_size(model, src, B), dtype=torch.uint8, device=dev)
    # references for the compaction check, taken before an in-place run overwrites the sources
    stats = centers.cpu().numpy()
    lens = w["seq_len"].cpu().numpy()
    ref_inst = {p: instance_from_device(cfg, w, *p) for p in picks}
    if paged:
        dst = src
        v_before = {p: None for p in picks}
        for (l, s, h) in picks:
            n = int(lens[s])
            bt = w["block_table"][s, : -(-n // cfg.block_size)].long()
            v_before[(l, s, h)] = H.to_numpy(w["v"][l, bt, h].reshape(-1, d)[:n].contiguous())
    else:
        kd = torch.zeros((L, S, Hkv, B, d), dtype=w["k"].dtype, device=dev)
        vd = torch.zeros_like(kd)
        pd = torch.zeros((L, S, Hkv, B), dtype=torch.int32, device=dev)
        dst = T.Cache(kd, vd, pd, w["seq_len"], w["cur_pos"], B)
    T.tri_compress_step(model, centers, src, dst, B, kept_idx, kept_cnt, new_len, ws)
    torch.cuda.synchronize()

    # ---- every head-instance: count, order, range
    keep = torch.minimum(w["seq_len"], torch.tensor(B, dtype=torch.int32, device=dev))
    assert torch.equal(new_len, keep)
    assert torch.equal(kept_cnt, keep.view(1, S, 1).expand(L, S, Hkv))
    col = torch.arange(B, device=dev).view(1, 1, 1, B)
    live = col < kept_cnt.unsqueeze(-1)
    idx = kept_idx
    assert bool(((idx >= 0) | ~live).all())
    assert bool(((idx < w["seq_len"].view(1, S, 1, 1)) | ~live).all())
    inc = (idx[..., 1:] > idx[..., :-1]) | ~live[..., 1:]
    assert bool(inc.all())
    # ---- every head-instance, contiguous layout: compacted rows are the selected rows, bit for bit
    if not paged:
        for l in range(L):
            gi = idx[l].clamp(min=0).long()
            m = live[l].unsqueeze(-1)
            for src_t, dst_t in ((w["k"], kd), (w["v"], vd)):
                got = dst_t[l].view(torch.int16)
                want = torch.gather(src_t[l].view(torch.int16), 2, gi.unsqueeze(-1).expand(-1, -1, -1, d))
                assert bool(((got == want) | ~m).all())
            wantp = torch.gather(w["pos"][l], 2, gi)
            assert bool(((pd[l] == wantp) | ~live[l]).all())

    # ---- sampled head-instances against the oracle
    same = 0
    for (l, s, h) in picks:
        kn, pn = ref_inst[(l, s, h)]
        n = int(lens[s])
        ref = oracle.head_instance(stats[l, h * G:(h + 1) * G], kn, pn, int(w["cur_pos"][s]), cfg.rope_theta,
                                   cfg.offsets, B, threads=16)
        c = int(kept_cnt[l, s, h])
        got = kept_idx[l, s, h, :c].cpu().numpy()
        same += H.check_kept(np.concatenate([got, np.zeros(B - c, np.int32)]), c, ref["final"], ref["idx"], n, B)
        if paged:   # in place: the sequence's first blocks now hold the survivors
            bt = w["block_table"][s, : -(-c // cfg.block_size)].long()
            k_after = H.to_numpy(w["k"][l, bt, h].reshape(-1, d)[:c].contiguous())
            v_after = H.to_numpy(w["v"][l, bt, h].reshape(-1, d)[:c].contiguous())
            p_after = w["pos"][l, bt, h].reshape(-1)[:c].cpu().numpy()
            np.testing.assert_array_equal(k_after, kn[got])
            np.testing.assert_array_equal(v_after, v_before[(l, s, h)][got])
            np.testing.assert_array_equal(p_after, pn[got])
    print("\n[%s] %d layers, %d head-instances checked by property, %d by the oracle (%d identical index sets)"
          % (cfg.name, L, L * S * Hkv, len(picks), same), flush=True)
    del w, ws
    torch.cuda.empty_cache()


def test_c2_layer_full(oracle):
    """Config 2: 32 query / 8 KV heads, N = 32768 at sparse positions in [0, 65536), B = 2048 -- all 8 instances."""
    cfg = recipe.CONFIGS["c2_layer"]
    run_full(oracle, cfg, [(0, 0, h) for h in range(8)])


@pytest.mark.parametrize("positions", ["dense", "sparse"])
def test_c3_model_full(oracle, positions):
    """Config 3: 36 layers x 16 sequences x 8 KV heads x 32768 keys, the benchmark workload."""
    cfg = recipe.CONFIGS["c3_model"]
    run_full(oracle, cfg, [(0, 0, 0), (17, 5, 3), (35, 15, 7)], positions=positions)


def test_c4_paged_slab(oracle):
    """Config 4: ragged paged batch, 64 sequences, block 16, compaction in place.  The full 36 layers need more
    than the 288 GB of HBM, so the step is run on a slab of 4 layers (head-instances are independent)."""
    cfg = recipe.CONFIGS["c4_paged"]
    lens = recipe.seq_lens(cfg)
    s_short, s_long = int(np.argmin(lens)), int(np.argmax(lens))
    run_full(oracle, cfg, [(0, s_short, 1), (3, s_long, 6)], layers=4)


def test_c5_long(oracle):
    """Config 5: 64 layers, G = 8, N = 131072, B = 4096, 32 offsets (up to 2^31), 5 % x10 outliers."""
    cfg = recipe.CONFIGS["c5_long"]
    run_full(oracle, cfg, [(41, 0, 5)])
