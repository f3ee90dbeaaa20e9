"""GPU parity: the HIP path through the C ABI against the CPU oracle, element by element."""
import numpy as np
import pytest
import torch

from workload import recipe

import tri_harness as H

pytestmark = pytest.mark.gpu


def oracle_instance(oracle, cfg, w, stats, l, s, h, threads=8, pairs=0, variant=0, rotated=False):
    G = cfg.group
    n = int(w["seq_len"][s])
    return oracle.head_instance(stats[l, h * G:(h + 1) * G], w["k"][l, s, h, :n], w["pos"][l, s, h, :n],
                                int(w["cur_pos"][s]), cfg.rope_theta, cfg.offsets, cfg.budget, pairs=pairs,
                                threads=threads, variant=variant, rotated=rotated)


def run_and_check(oracle, cfg, instances=None, paged=False, inplace=False, pairs=0, mutate=None, variant=0,
                  rotated=False):
    w = recipe.generate(cfg)
    if mutate is not None:
        mutate(w)
    run = H.GpuRun(cfg, w, paged=paged, pairs=pairs, variant=variant, rotated=rotated)
    stats_gpu = run.build_centers()
    stats = oracle.centers(w["q_samples"], pairs=pairs)
    np.testing.assert_allclose(stats_gpu, stats, rtol=3e-7, atol=1e-30)
    # score with the oracle's table so that the two sides read identical bytes
    run.centers.copy_(torch.from_numpy(stats))
    final, raw = run.score()
    idx, cnt = run.select()
    L, S, Hkv, G = cfg.n_layers, cfg.n_seqs, cfg.n_kv_heads, cfg.group
    if instances is None:
        instances = [(l, s, h) for l in range(L) for s in range(S) for h in range(Hkv)]
    exact = 0
    worst_raw = worst_final = 0.0
    for (l, s, h) in instances:
        n = int(w["seq_len"][s])
        if n == 0:
            assert cnt[l, s, h] == 0
            continue
        ref = oracle_instance(oracle, cfg, w, stats, l, s, h, pairs=pairs, variant=variant, rotated=rotated)
        worst_raw = max(worst_raw, H.check_raw(raw[l, s, h * G:(h + 1) * G, :n], ref["raw"]))
        worst_final = max(worst_final, H.check_final(final[l, s, h, :n], ref["final"]))
        exact += H.check_kept(idx[l, s, h], int(cnt[l, s, h]), ref["final"], ref["idx"], n, cfg.budget)
        # selection proper is integer work: on the GPU's own fp32 scores it must match the oracle bit for bit
        ref_idx32 = oracle.topk(final[l, s, h, :n].astype(np.float64), cfg.budget)
        np.testing.assert_array_equal(idx[l, s, h, :len(ref_idx32)], ref_idx32)
    # compaction: bit-exact rows, out of place or in place
    if inplace:
        new_len = run.compact()
        k_out, v_out, p_out = H.to_numpy(run.k), H.to_numpy(run.v), run.pos.cpu().numpy()
    else:
        kd, vd, pd = torch.zeros_like(run.k), torch.zeros_like(run.v), torch.zeros_like(run.pos)
        dst = run.B.Cache(kd, vd, pd, run.seq_len, run.cur_pos, run.nmax, run.block_table)
        new_len = run.compact(dst)
        k_out, v_out, p_out = H.to_numpy(kd), H.to_numpy(vd), pd.cpu().numpy()
    np.testing.assert_array_equal(new_len, np.minimum(w["seq_len"], cfg.budget))
    for (l, s, h) in instances:
        c = int(cnt[l, s, h])
        sel = idx[l, s, h, :c]
        if paged:
            bs = cfg.block_size
            strides = (run.k.stride(0), run.k.stride(1), run.k.stride(2), run.k.stride(3))
            pstr = (run.pos.stride(0), run.pos.stride(1), run.pos.stride(2), 1)
            got_k = oracle.paged_gather(k_out, cfg.head_dim, run.bt_np, bs, strides, l, s, h, c)
            got_v = oracle.paged_gather(v_out, cfg.head_dim, run.bt_np, bs, strides, l, s, h, c)
            got_p = oracle.paged_gather(p_out, 1, run.bt_np, bs, pstr, l, s, h, c)[:, 0]
        else:
            got_k, got_v, got_p = k_out[l, s, h, :c], v_out[l, s, h, :c], p_out[l, s, h, :c]
        np.testing.assert_array_equal(got_k, oracle.compact_rows(w["k"][l, s, h], sel))
        np.testing.assert_array_equal(got_v, oracle.compact_rows(w["v"][l, s, h], sel))
        np.testing.assert_array_equal(got_p, w["pos"][l, s, h][sel])
    print("\n[%s] instances %d, identical index sets %d, worst raw err %.2e (rel), worst final err %.2e"
          % (cfg.name, len(instances), exact, worst_raw, worst_final), flush=True)
    return exact, len(instances)


def test_c1_tiny_fp32(oracle):
    """Config 1 in full: 1 KV head, 4 query heads, N = 4096 dense positions, B = 512, fp32."""
    run_and_check(oracle, recipe.CONFIGS["c1_tiny"])


def test_small_bf16_ragged_sparse(oracle):
    """Qwen3-shaped heads at small N: several tiles and a ragged tail, sparse positions, two layers,
    three sequences of different lengths (one shorter than the budget, one empty)."""
    cfg = recipe.scaled(recipe.CONFIGS["c2_layer"], n_layers=2, n_seqs=3, n_q_heads=8, n_kv_heads=2, seq_len=1000,
                        min_seq_len=0, budget=200, n_calib=256)
    w_len = recipe.seq_lens(cfg)
    assert len(set(w_len.tolist())) == 3
    run_and_check(oracle, cfg)


def test_small_inplace(oracle):
    cfg = recipe.scaled(recipe.CONFIGS["c2_layer"], n_layers=1, n_seqs=2, n_q_heads=8, n_kv_heads=2, seq_len=777,
                        min_seq_len=300, budget=128, n_calib=128)
    run_and_check(oracle, cfg, inplace=True)


@pytest.mark.parametrize("inplace", [False, True])
def test_small_paged(oracle, inplace):
    cfg = recipe.scaled(recipe.CONFIGS["c4_paged"], n_layers=2, n_seqs=3, n_q_heads=8, n_kv_heads=2, seq_len=900,
                        min_seq_len=100, budget=160, n_calib=128)
    run_and_check(oracle, cfg, paged=True, inplace=inplace)


def test_group_of_eight(oracle):
    cfg = recipe.scaled(recipe.CONFIGS["c5_long"], n_layers=1, n_seqs=1, n_q_heads=16, n_kv_heads=2, seq_len=600,
                        budget=100, n_calib=128)
    run_and_check(oracle, cfg)


def test_wild_positions(oracle):
    """Positions that defeat the relative-position table: unsorted, gaps of up to 2^28, one sequence
    with long runs of equal positions.  Exercises the direct path and the base moves of the MFMA kernel."""
    cfg = recipe.scaled(recipe.CONFIGS["c2_layer"], n_layers=1, n_seqs=3, n_q_heads=8, n_kv_heads=2, seq_len=700,
                        budget=100, n_calib=128)

    def mutate(w):
        rng = np.random.default_rng(5)
        n = cfg.seq_len
        w["pos"][:, 0] = rng.integers(0, 1 << 28, size=(1, 2, n)).astype(np.int32)             # unsorted, huge
        mixed = np.sort(rng.integers(0, 5000, size=(1, 2, n)), axis=-1)
        mixed[..., 300:] += 1 << 20                                                              # one big jump
        w["pos"][:, 1] = mixed.astype(np.int32)
        w["pos"][:, 2] = (np.arange(n) // 37 * 3).astype(np.int32)                              # repeated positions
        w["cur_pos"][:] = np.array([1 << 28, (1 << 20) + 5000, 100], dtype=np.int32)

    run_and_check(oracle, cfg, mutate=mutate)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_half_split_pairs(oracle, dtype):
    """Band f = (x[f], x[f + d/2]): the same workload with every head vector permuted to that layout
    (bf16: MFMA kernel; fp32: generic kernel)."""
    cfg = recipe.scaled(recipe.CONFIGS["c2_layer"], n_layers=1, n_seqs=1, n_q_heads=8, n_kv_heads=2, seq_len=500,
                        budget=64, n_calib=128, dtype=dtype)

    def mutate(w):
        for name in ("k", "q_samples"):
            x = w[name]
            w[name] = np.ascontiguousarray(np.concatenate([x[..., 0::2], x[..., 1::2]], axis=-1))

    run_and_check(oracle, cfg, pairs=1, mutate=mutate)


@pytest.mark.parametrize("variant", [1, 2, 3])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_score_variants(oracle, variant, dtype):
    """The ablation variants (trig only, norm only, un-weighted norm) on the MFMA kernel (bf16) and the generic one."""
    cfg = recipe.scaled(recipe.CONFIGS["c2_layer"], n_layers=1, n_seqs=2, n_q_heads=8, n_kv_heads=2, seq_len=700,
                        min_seq_len=300, budget=96, n_calib=128, dtype=dtype)
    run_and_check(oracle, cfg, variant=variant)


@pytest.mark.parametrize("dtype,pairs,paged", [("bf16", 0, False), ("bf16", 0, True), ("bf16", 1, False), ("f32", 0, False)])
def test_post_rope_cache(oracle, dtype, pairs, paged):
    """A cache of post-RoPE keys (every key rotated by its own position before it was stored)."""
    base = recipe.CONFIGS["c4_paged" if paged else "c2_layer"]
    cfg = recipe.scaled(base, n_layers=2, n_seqs=2, n_q_heads=8, n_kv_heads=2, seq_len=800, min_seq_len=200,
                        budget=128, n_calib=128, dtype=dtype)

    def mutate(w):
        if pairs:
            for name in ("k", "q_samples"):
                x = w[name]
                w[name] = np.ascontiguousarray(np.concatenate([x[..., 0::2], x[..., 1::2]], axis=-1))
        w["k"] = H.to_post_rope(w["k"], w["pos"], cfg.rope_theta, pairs, cfg.dtype)

    run_and_check(oracle, cfg, paged=paged, pairs=pairs, mutate=mutate, rotated=True)


@pytest.mark.parametrize("pairs", [0, 1])
def test_paged_blocks_of_eight(oracle, pairs):
    """Blocks shorter than a 16-key group: the generic kernel scores bf16 keys (both pair layouts)."""
    cfg = recipe.scaled(recipe.CONFIGS["c4_paged"], n_layers=1, n_seqs=2, n_q_heads=8, n_kv_heads=2, seq_len=600,
                        min_seq_len=150, budget=100, n_calib=128, block_size=8)

    def mutate(w):
        if pairs:
            for name in ("k", "q_samples"):
                x = w[name]
                w[name] = np.ascontiguousarray(np.concatenate([x[..., 0::2], x[..., 1::2]], axis=-1))

    run_and_check(oracle, cfg, paged=True, inplace=True, pairs=pairs, mutate=mutate)


@pytest.mark.parametrize("group", [3, 5, 6, 7])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_group_sizes_that_are_not_powers_of_two(oracle, group, dtype):
    """G = 3, 5, 6, 7 query heads per KV head (for instance 28 query heads over 4 KV heads)."""
    cfg = recipe.scaled(recipe.CONFIGS["c2_layer"], n_layers=1, n_seqs=2, n_q_heads=2 * group, n_kv_heads=2, seq_len=520,
                        min_seq_len=200, budget=77, n_calib=128, dtype=dtype)
    run_and_check(oracle, cfg)


def test_sequence_lengths_outside_the_host_bound_are_clamped():
    """seq_len lives in device memory, so the host cannot check it: an entry above max_seq_len is read as max_seq_len
    and a negative one as 0 (nothing is indexed beyond what the host sized)."""
    cfg = recipe.scaled(recipe.CONFIGS["c2_layer"], n_layers=1, n_seqs=2, n_q_heads=8, n_kv_heads=2, seq_len=600,
                        min_seq_len=600, budget=100, n_calib=128)
    w = recipe.generate(cfg)
    outs = []
    for lens in ([600, 0], [600 + 4321, -7]):
        w2 = dict(w)
        w2["seq_len"] = np.array(lens, dtype=np.int32)
        run = H.GpuRun(cfg, w2)
        run.build_centers()
        run.B.tri_compress_step(run.model, run.centers, run.cache, run.cache, cfg.budget, run.kept_idx, run.kept_cnt,
                                run.new_len, run.ws)
        torch.cuda.synchronize()
        outs.append([t.clone() for t in (run.kept_idx, run.kept_cnt, run.new_len, run.k.view(torch.int16),
                                         run.v.view(torch.int16), run.pos)])
    for a, b in zip(*outs):
        assert torch.equal(a, b)
    assert outs[0][2].tolist() == [100, 0]


@pytest.mark.parametrize("seq_len,min_len,budget,ties", [(5000, 900, 333, False), (40000, 20000, 2048, False),
                                                         (70000, 33000, 3000, False), (40000, 20000, 2048, True),
                                                         (70000, 33000, 3000, True)])
def test_fused_step_agrees_with_the_three_calls(seq_len, min_len, budget, ties):
    """tri_compress_step forms the final scores inside the selection; tri_score writes them out for tri_select_topk.
    Both go through the same z-score arithmetic, so the kept sets are identical, not merely within the tie band.
    Beyond 32768 keys the fused selection keeps its integer keys in LDS (sequences up to 32768 keys) or in the
    workspace (longer ones); the ragged lengths here exercise both.  ties: stretches of the cache hold copies of one
    key at one position, i.e. hundreds of equal final scores, some of them around the budget's threshold."""
    cfg = recipe.scaled(recipe.CONFIGS["c2_layer"], n_layers=1 if seq_len > 5000 else 2, n_seqs=3, n_q_heads=8,
                        n_kv_heads=2, seq_len=seq_len, min_seq_len=min_len, budget=budget, n_calib=128)
    w = recipe.generate(cfg)
    if ties:
        for start, count in ((1000, 700), (9000, 1500), (15000, 2600)):
            w["k"][..., start:start + count, :] = w["k"][..., start - 1:start, :]
            w["pos"][..., start:start + count] = w["pos"][..., start - 1:start]
    run = H.GpuRun(cfg, w)
    run.build_centers()
    final, _ = run.score(want_raw=False)
    idx_a, cnt_a = run.select()
    if ties:   # most copies tie bit for bit (a wave that scores them against another table base may differ in the
        # last bit); count the head-instances whose threshold falls among equal scores
        stretch = final[0, 0, 0, 1000:1700]
        assert np.mean(stretch == np.median(stretch)) > 0.5
        at_threshold = 0
        for l in range(cfg.n_layers):
            for s_ in range(cfg.n_seqs):
                for h in range(cfg.n_kv_heads):
                    n = int(w["seq_len"][s_])
                    f = np.sort(final[l, s_, h, :n])[::-1]
                    at_threshold += int(f[budget - 1] == f[budget])
        print("\n[ties] head-instances whose threshold lies among equal scores: %d" % at_threshold)
    run.kept_idx.fill_(-1)
    run.kept_cnt.fill_(-1)
    kd = torch.zeros((cfg.n_layers, cfg.n_seqs, cfg.n_kv_heads, budget, cfg.head_dim), dtype=run.k.dtype, device="cuda")
    vd, pd = torch.zeros_like(kd), torch.zeros(kd.shape[:-1], dtype=torch.int32, device="cuda")
    dst = run.B.Cache(kd, vd, pd, run.seq_len, run.cur_pos, budget)
    run.B.tri_compress_step(run.model, run.centers, run.cache, dst, cfg.budget, run.kept_idx, run.kept_cnt,
                            run.new_len, run.ws)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(run.kept_cnt.cpu().numpy(), cnt_a)
    np.testing.assert_array_equal(run.kept_idx.cpu().numpy(), idx_a)
    # and the selection itself is the oracle's on the same fp32 scores (ties to the lower slot)
    from oracle import tri_oracle as O
    for s_ in range(cfg.n_seqs):
        n = int(w["seq_len"][s_])
        ref = O.topk(final[0, s_, 1, :n].astype(np.float64), budget)
        np.testing.assert_array_equal(idx_a[0, s_, 1, :len(ref)], ref)


def test_head_without_statistics_and_constant_scores(oracle):
    """Section 4.3 with sigma = 0 (a head whose scores are all equal contributes 0 to the maximum).
    (a) One query head of each group has an all-zero statistics row: its raw scores are exactly 0 on both sides and
    it drops out of the maximum.  (b) A head-instance whose keys are all copies of one key at one position: every
    head's scores are constant, every final score is 0, and the budget goes to the lowest slots."""
    cfg = recipe.scaled(recipe.CONFIGS["c2_layer"], n_layers=1, n_seqs=2, n_q_heads=8, n_kv_heads=2, seq_len=3000,
                        min_seq_len=3000, budget=500, n_calib=128)
    w = recipe.generate(cfg)
    # (b): sequence 1, KV head 1
    w["k"][0, 1, 1, :, :] = w["k"][0, 1, 1, 77:78, :]
    w["pos"][0, 1, 1, :] = w["pos"][0, 1, 1, 77]
    run = H.GpuRun(cfg, w)
    run.build_centers()
    stats = oracle.centers(w["q_samples"])
    stats[0, 2] = 0.0      # (a): query head 2 of KV head 0 and query head 5 of KV head 1
    stats[0, 5] = 0.0
    run.centers.copy_(torch.from_numpy(stats))
    final, raw = run.score()
    idx, cnt = run.select()
    G = cfg.group
    assert np.all(raw[0, :, 2, :] == 0.0) and np.all(raw[0, :, 5, :] == 0.0)
    for s_ in range(cfg.n_seqs):
        for h in range(cfg.n_kv_heads):
            n = int(w["seq_len"][s_])
            ref = oracle_instance(oracle, cfg, w, stats, 0, s_, h)
            live = [g for g in range(G) if h * G + g not in (2, 5)]
            if (s_, h) == (1, 1):
                assert np.all(ref["final"] == 0.0) and np.all(final[0, s_, h, :n] == 0.0)
                np.testing.assert_array_equal(idx[0, s_, h, :cfg.budget], np.arange(cfg.budget))
                np.testing.assert_array_equal(ref["idx"], np.arange(cfg.budget))
                continue
            H.check_raw(raw[0, s_, h * G:(h + 1) * G, :n][live], ref["raw"][live])
            H.check_final(final[0, s_, h, :n], ref["final"])
            H.check_kept(idx[0, s_, h], int(cnt[0, s_, h]), ref["final"], ref["idx"], n, cfg.budget)
    # the fused step takes the same decisions
    run.kept_idx.fill_(-1)
    run.B.tri_compress_step(run.model, run.centers, run.cache, run.cache, cfg.budget, run.kept_idx, run.kept_cnt,
                            run.new_len, run.ws)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(run.kept_idx.cpu().numpy(), idx)


@pytest.mark.parametrize("kind", ["linear17", "geometric13", "single", "sixty_four"])
def test_offset_sets(oracle, kind):
    """Offset sets other than the sixteen powers of two: the linear spacing and the shorter geometric range of the
    offset ablation (Appendix G), a single offset, and the largest set the library takes (64 offsets)."""
    sets = {"linear17": tuple(int(x) for x in np.linspace(1, 65536, 17)),
            "geometric13": tuple(1 << j for j in range(13)),
            "single": (4096,),
            "sixty_four": tuple(3 * j + 1 for j in range(64))}
    cfg = recipe.scaled(recipe.CONFIGS["c2_layer"], n_layers=1, n_seqs=2, n_q_heads=8, n_kv_heads=2, seq_len=600,
                        min_seq_len=250, budget=90, n_calib=128, offset_list=sets[kind])
    run_and_check(oracle, cfg)


def test_many_short_sequences(oracle):
    """More sequences than the work-list builder has threads (each thread then lists several sequences), lengths from
    0 to a few groups: the score kernel's items are one per existing (sequence, chunk) pair, empty sequences have none."""
    cfg = recipe.scaled(recipe.CONFIGS["c2_layer"], n_layers=1, n_seqs=300, n_q_heads=8, n_kv_heads=2, seq_len=70,
                        min_seq_len=0, budget=20, n_calib=128)
    def lens(w):
        w["seq_len"][::7] = 0
    run_and_check(oracle, cfg, mutate=lens)


def test_chunk_boundaries(oracle):
    """Sequence lengths around the work items of the score kernel.  A batch this small is cut into items of one round
    of the kernel's waves (768 keys): one key short of an item, exactly one, one more; and lengths around 8192 keys and
    two of them plus a ragged tail."""
    cfg = recipe.scaled(recipe.CONFIGS["c2_layer"], n_layers=1, n_seqs=7, n_q_heads=8, n_kv_heads=1, seq_len=16901,
                        min_seq_len=16901, budget=500, n_calib=128)
    def lens(w):
        w["seq_len"][:] = np.array([767, 768, 769, 8191, 8192, 8193, 16901], dtype=np.int32)
    run_and_check(oracle, cfg, mutate=lens)


def test_work_items_of_two_rounds(oracle):
    """A batch large enough for work items of two rounds (1536 keys) and small enough not to reach the full 8192:
    2 layers x 16 sequences x 8 KV heads of up to 6200 keys, lengths around the item size; a dozen head-instances go
    through the oracle, all of them through the compaction check's index rules."""
    cfg = recipe.scaled(recipe.CONFIGS["c2_layer"], n_layers=2, n_seqs=16, n_q_heads=32, n_kv_heads=8, seq_len=6200,
                        min_seq_len=6200, budget=300, n_calib=128)
    def lens(w):
        w["seq_len"][:] = np.array([1535, 1536, 1537, 3071, 3072, 3073, 4608, 6200, 6144, 100, 0, 1600, 5000, 2999, 64, 6199],
                                   dtype=np.int32)
    picks = [(l, s, (3 * s + l) % 8) for l in range(2) for s in (0, 1, 2, 5, 7, 8)]
    run_and_check(oracle, cfg, mutate=lens, instances=picks)


def test_all_sequences_empty():
    """No keys anywhere: the score kernel's work list is empty, every count is zero and nothing is written."""
    cfg = recipe.scaled(recipe.CONFIGS["c2_layer"], n_layers=2, n_seqs=3, n_q_heads=8, n_kv_heads=2, seq_len=300,
                        min_seq_len=300, budget=50, n_calib=128)
    w = recipe.generate(cfg)
    w["seq_len"] = np.zeros(3, dtype=np.int32)
    run = H.GpuRun(cfg, w)
    run.build_centers()
    k0 = run.k.clone()
    run.kept_cnt.fill_(-1)
    run.B.tri_compress_step(run.model, run.centers, run.cache, run.cache, cfg.budget, run.kept_idx, run.kept_cnt,
                            run.new_len, run.ws)
    torch.cuda.synchronize()
    assert run.kept_cnt.cpu().numpy().tolist() == [[[0, 0]] * 3] * 2
    assert run.new_len.cpu().numpy().tolist() == [0, 0, 0]
    assert torch.equal(run.k.view(torch.int16), k0.view(torch.int16))


def test_repeated_calls_give_the_same_bits():
    """Work items reach the workgroups through a shared counter, in an order that differs from launch to launch; the
    raw and final scores, the moments behind them and the kept sets must not depend on it.  4 x 16 x 8 head-instances
    of ragged lengths up to 20000 keys generated on the device (work items of 8192 keys and shorter last ones, about six
    per workgroup the GPU holds), five calls of tri_score and of the fused step compared bit for bit."""
    from paper_2604_04921_amd import binding as B
    from workload import device
    cfg = recipe.scaled(recipe.CONFIGS["c2_layer"], n_layers=4, n_seqs=16, n_q_heads=32, n_kv_heads=8, seq_len=20000,
                        min_seq_len=3000, budget=1024, n_calib=128)
    w = device.generate(cfg, positions="sparse", layers=cfg.n_layers)
    L, S, Hq, Hkv, d, Bk = cfg.n_layers, cfg.n_seqs, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.budget
    model = B.Model(L, Hq, Hkv, d, cfg.rope_theta, cfg.offsets)
    src = B.Cache(w["k"], w["v"], w["pos"], w["seq_len"], w["cur_pos"], cfg.seq_len, None)
    centers = torch.empty((L, Hq, d // 2, 3), dtype=torch.float32, device="cuda")
    B.tri_build_centers(model, w["q_samples"], centers)
    kd = torch.zeros((L, S, Hkv, Bk, d), dtype=w["k"].dtype, device="cuda")
    vd, pd = torch.zeros_like(kd), torch.zeros((L, S, Hkv, Bk), dtype=torch.int32, device="cuda")
    dst = B.Cache(kd, vd, pd, w["seq_len"], w["cur_pos"], Bk)
    final = torch.empty((L, S, Hkv, cfg.seq_len), dtype=torch.float32, device="cuda")
    raw = torch.empty((L, S, Hq, cfg.seq_len), dtype=torch.float32, device="cuda")
    kept_idx = torch.empty((L, S, Hkv, Bk), dtype=torch.int32, device="cuda")
    kept_cnt = torch.empty((L, S, Hkv), dtype=torch.int32, device="cuda")
    new_len = torch.empty((S,), dtype=torch.int32, device="cuda")
    ws = torch.empty(B.tri_workspace_size(model, src, Bk), dtype=torch.uint8, device="cuda")
    first = None
    for rep in range(5):
        final.fill_(float("nan"))
        raw.fill_(float("nan"))
        kept_idx.fill_(-1)
        B.tri_score(model, centers, src, final, raw, ws)
        B.tri_compress_step(model, centers, src, dst, Bk, kept_idx, kept_cnt, new_len, ws)
        torch.cuda.synchronize()
        got = [final.clone().view(torch.int32), raw.clone().view(torch.int32), kept_idx.clone(), kept_cnt.clone(),
               kd.clone().view(torch.int16)]
        if first is None:
            first = got
            assert int(kept_cnt.min()) == Bk and int(kept_cnt.max()) == Bk
            assert not bool(torch.isnan(raw[0, 0, 0, :3000]).any())
        else:
            for a, b in zip(first, got):
                assert torch.equal(a, b), "call %d differs from the first" % rep
