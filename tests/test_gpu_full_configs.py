"""The five benchmark configurations at full size on the GPU, in the launch configuration bench.py times
(tri_compress_step on a device-generated workload).  The oracle checks a few whole head-instances copied
back from the device; every head-instance is checked with properties that hold at any size: kept count,
ascending unique in-range indices, and bit-exact compacted K / V / positions (directly for the contiguous layout,
through the block table with per-row checksums taken before the step for the paged one).  At these sizes the
oracle comparison is on the kept sets; raw and final scores are compared element by element in test_gpu_parity.py
on inputs of up to 16 901 keys."""
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


def row_checksums(t, lo, hi):
    """One int64 per row of t[lo:hi] (last dimension = the row, bf16 or fp32 viewed as 16-bit words): a weighted
    sum with odd multipliers, enough to tell any two rows of these caches apart.  Done layer by layer to bound
    the temporaries."""
    words = t.view(torch.int16)
    wts = (torch.arange(words.shape[-1], device=t.device, dtype=torch.int64) * 2654435761 + 12345) | 1
    return torch.stack([(words[l].to(torch.int64) * wts).sum(-1) for l in range(lo, hi)])


def run_full(oracle, cfg, picks, layers=None, positions=None, layer0=0):
    """One fused step on `layers` layers of cfg starting at layer0.  picks: (l, s, h) with l relative to the slab."""
    from paper_2604_04921_amd import binding as T
    L = layers or cfg.n_layers
    w = device.generate(cfg, positions=positions, layers=L, layer0=layer0)
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
        # every slot of the pools: checksums of its K row and V row, and its position, before the step
        ck_before, cv_before = row_checksums(w["k"], 0, L), row_checksums(w["v"], 0, L)   # [L][n_blocks][Hkv][bs]
        pos_before = w["pos"].clone()
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
    # ---- every head-instance: compacted rows are the selected rows, bit for bit
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
    else:
        # in place through the block table: slot j of (l, s, h) must now hold what slot kept_idx[j] held before
        # (row checksums of K and V, the position itself), for every head-instance of the slab
        bs = cfg.block_size
        btd = w["block_table"].long()                                   # [S][max_blocks]
        ck_after, cv_after = row_checksums(w["k"], 0, L), row_checksums(w["v"], 0, L)
        hh = torch.arange(Hkv, device=dev).view(1, Hkv, 1).expand(S, Hkv, B)
        jj = torch.arange(B, device=dev).view(1, 1, B).expand(S, Hkv, B)
        dst_blk = torch.gather(btd, 1, (jj[:, 0] // bs).clamp(max=btd.shape[1] - 1)).view(S, 1, B).expand(S, Hkv, B)
        for l in range(L):
            n_src = idx[l].clamp(min=0).long()                           # [S][Hkv][B]
            src_blk = torch.gather(btd.view(S, 1, -1).expand(S, Hkv, -1), 2, n_src // bs)
            for before, after in ((ck_before, ck_after), (cv_before, cv_after), (pos_before, w["pos"])):
                want = before[l][src_blk, hh, n_src % bs]
                got = after[l][dst_blk, hh, jj % bs]
                assert bool(((got == want) | ~live[l]).all())
        del ck_before, cv_before, ck_after, cv_after, pos_before

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
    print("\n[%s] layers %d..%d, %d head-instances checked by property, %d by the oracle (%d identical index sets)"
          % (cfg.name, layer0, layer0 + L - 1, L * S * Hkv, len(picks), same), flush=True)
    del w, ws
    torch.cuda.empty_cache()
    return same


def test_c2_layer_full(oracle):
    """Config 2: 32 query / 8 KV heads, N = 32768 at sparse positions in [0, 65536), B = 2048 -- all 8 instances."""
    cfg = recipe.CONFIGS["c2_layer"]
    run_full(oracle, cfg, [(0, 0, h) for h in range(8)])


@pytest.mark.parametrize("positions", ["dense", "sparse"])
def test_c3_model_full(oracle, positions):
    """Config 3: 36 layers x 16 sequences x 8 KV heads x 32768 keys, the benchmark workload."""
    cfg = recipe.CONFIGS["c3_model"]
    n = 16 if positions == "dense" else 8   # head-instances through the oracle, spread over layers, sequences, heads
    picks = [(0, 0, 0), (35, 15, 7)] + [((7 * i + 3) % 36, (5 * i + 1) % 16, (3 * i + 2) % 8) for i in range(n - 2)]
    run_full(oracle, cfg, picks, positions=positions)


@pytest.mark.parametrize("slab", [0, 1, 2])
def test_c4_paged_slabs(oracle, slab):
    """Config 4: ragged paged batch, 64 sequences, block 16, compaction in place.  The full 36 layers need more
    than the 288 GB of HBM, so the step is run as three slabs of 12 layers (head-instances are independent) that
    together cover every layer.  Six head-instances per slab go through the oracle (shortest and longest
    sequence among them); every head-instance of every slab is checked through the block table."""
    cfg = recipe.CONFIGS["c4_paged"]
    lens = recipe.seq_lens(cfg)
    order = np.argsort(lens)
    seqs = [int(order[0]), int(order[-1]), int(order[len(order) // 2]), int(order[len(order) // 4]),
            int(order[3 * len(order) // 4]), int(order[1])]
    picks = [((5 * i + 2 * slab) % 12, seqs[(i + slab) % 6], (3 * i + slab) % 8) for i in range(6)]
    run_full(oracle, cfg, picks, layers=12, layer0=12 * slab)


def test_c5_long(oracle):
    """Config 5: 64 layers, G = 8, N = 131072, B = 4096, 32 offsets (up to 2^31), 5 % x10 outliers: eight
    head-instances spread over the layers and KV heads go through the oracle."""
    cfg = recipe.CONFIGS["c5_long"]
    run_full(oracle, cfg, [(9 * i, 0, (5 * i + 3) % 8) for i in range(8)])


def test_steady_state_ordered(oracle):
    """The steady-state cadence (Section 4.3): 36 x 64 x 8 head-instances of B + 128 = 2176 keys, ordered compaction."""
    cfg = recipe.CONFIGS["steady_state"]
    run_full(oracle, cfg, [(0, 0, 0), (20, 33, 5), (35, 63, 7)])


def test_steady_state_minimal_move(oracle):
    """The same workload evicted in place with the fewest moves (tri_compress_step with dst = NULL): every
    head-instance is checked by property (the first B slots hold exactly the kept keys, each with its own V row and
    position; nothing at or beyond slot B changed), sampled ones against the oracle's compact_fill bit for bit."""
    from paper_2604_04921_amd import binding as T
    cfg = recipe.CONFIGS["steady_state"]
    L, S, Hq, Hkv, B, d, G, N = (cfg.n_layers, cfg.n_seqs, cfg.n_q_heads, cfg.n_kv_heads, cfg.budget, cfg.head_dim,
                                 cfg.group, cfg.seq_len)
    w = device.generate(cfg)
    dev = "cuda"
    model = T.Model(L, Hq, Hkv, d, cfg.rope_theta, cfg.offsets)
    cache = T.Cache(w["k"], w["v"], w["pos"], w["seq_len"], w["cur_pos"], N)
    centers = torch.empty((L, Hq, d // 2, 3), dtype=torch.float32, device=dev)
    T.tri_build_centers(model, w["q_samples"], centers)
    kept_idx = torch.full((L, S, Hkv, B), -1, dtype=torch.int32, device=dev)
    kept_cnt = torch.full((L, S, Hkv), -1, dtype=torch.int32, device=dev)
    new_len = torch.full((S,), -1, dtype=torch.int32, device=dev)
    ws = torch.empty(T.tri_workspace_size(model, cache, B), dtype=torch.uint8, device=dev)
    k0, v0, p0 = w["k"].clone(), w["v"].clone(), w["pos"].clone()
    assert bool((w["seq_len"] == N).all())
    T.tri_compress_step(model, centers, cache, None, B, kept_idx, kept_cnt, new_len, ws)
    torch.cuda.synchronize()
    assert bool((kept_cnt == B).all()) and bool((new_len == B).all())
    # nothing at or beyond slot B was written
    assert torch.equal(w["k"][..., B:, :].view(torch.int16), k0[..., B:, :].view(torch.int16))
    assert torch.equal(w["v"][..., B:, :].view(torch.int16), v0[..., B:, :].view(torch.int16))
    assert torch.equal(w["pos"][..., B:], p0[..., B:])
    moved = 0
    for l in range(L):   # positions are unique within a head-instance: they identify the keys
        gi = kept_idx[l].long()
        want_pos = torch.gather(p0[l], 2, gi)
        got_pos = w["pos"][l, :, :, :B]
        oa, ob = torch.argsort(got_pos, dim=2), torch.argsort(want_pos, dim=2)
        assert torch.equal(torch.gather(got_pos, 2, oa), torch.gather(want_pos, 2, ob))
        for now, before in ((w["k"], k0), (w["v"], v0)):
            got = torch.gather(now[l, :, :, :B].view(torch.int16), 2, oa.unsqueeze(-1).expand(-1, -1, -1, d))
            src_slot = torch.gather(gi, 2, ob)
            want = torch.gather(before[l].view(torch.int16), 2, src_slot.unsqueeze(-1).expand(-1, -1, -1, d))
            assert torch.equal(got, want)
        moved += int((got_pos != p0[l, :, :, :B]).sum())
    assert moved <= L * S * Hkv * (N - B)      # at most one move per evicted slot below B
    stats = centers.cpu().numpy()
    same = 0
    for (l, s, h) in [(0, 0, 0), (20, 33, 5), (35, 63, 7)]:
        kn, vn, pn = H.to_numpy(k0[l, s, h]), H.to_numpy(v0[l, s, h]), p0[l, s, h].cpu().numpy()
        ref = oracle.head_instance(stats[l, h * G:(h + 1) * G], kn, pn, int(w["cur_pos"][s]), cfg.rope_theta, cfg.offsets,
                                   B, threads=16)
        got = kept_idx[l, s, h].cpu().numpy()
        same += H.check_kept(got, B, ref["final"], ref["idx"], N, B)
        for now, before in ((w["k"], kn), (w["v"], vn), (w["pos"], pn.reshape(N, 1))):
            exp = np.ascontiguousarray(before).copy()
            oracle.compact_fill(exp, got)
            np.testing.assert_array_equal(H.to_numpy(now[l, s, h]).reshape(exp.shape), exp)
    print("\n[steady_state, minimal-move] %d head-instances checked by property, %d slots moved (%.1f per instance), "
          "3 by the oracle (%d identical index sets)" % (L * S * Hkv, moved, moved / (L * S * Hkv), same), flush=True)
    del w, ws, k0, v0, p0
    torch.cuda.empty_cache()
