#!/usr/bin/env python3
"""Benchmark of the TriAttention KV-cache compression step on one MI355X.

One "step" = score -> GQA reduce -> top-B -> compact over the whole synthetic batch (all layers,
sequences and KV heads of the configuration), inputs resident in HBM.  Prints ONE JSON line:
throughput in cached keys per second, the roofline of the dominant (score) kernel measured with HIP
events inside the timed region, and the CPU oracle timed on a bounded sample on this machine's host cores.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
SCORE_BYTES_PER_KEY = 260      # one bf16 K row (2*128 B) + one int32 position, read once
STEP_BYTES = lambda n, b: 260 * n + 1032 * min(n, b)   # + survivors' K, V, pos read and written

# HBM bytes of one score-kernel launch measured with rocprofv3 --pmc (FETCH_SIZE and WRITE_SIZE in two runs,
# each scaled by what the same counter reads for a plain device copy of known size: FETCH_SIZE reads 0.5 of the
# bytes a 1 GiB copy fetches, WRITE_SIZE 1.0); summary in profiles/pmc_traffic_c3_model.md.  The figure belongs to
# the kernel sources it was measured on: it is reported only while their hash (kernel_sources_sha16) is unchanged.
MEASURED_TRAFFIC = {"c3_model/dense": {"bytes": 39.30e9 + 2.42e9, "sources_sha16": "087fa4a7bba8d86a"}}


def kernel_sources_sha16():
    """Hash of the library's kernel sources (csrc/*.hip, *.h, sorted by name)."""
    import glob
    import hashlib
    h = hashlib.sha256()
    for f in sorted(glob.glob(os.path.join(ROOT, "paper_2604_04921_amd", "csrc", "*.h*"))):
        h.update(os.path.basename(f).encode())
        h.update(open(f, "rb").read())
    return h.hexdigest()[:16]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="c3_model")
    ap.add_argument("--positions", default=None, choices=[None, "dense", "sparse", "sparse16", "scattered"])
    ap.add_argument("--layers", type=int, default=None, help="layer slab (configurations larger than HBM)")
    ap.add_argument("--slabs", type=int, default=1,
                    help="with --layers: run this many consecutive layer slabs one after the other (each generated, "
                         "measured and freed in turn) and report them as one step over slabs x layers layers")
    ap.add_argument("--ws-candidates", type=int, default=4,
                    help="workspaces to allocate (8 GB apart) and try before the warm-up; the one the score launch runs "
                         "fastest on is kept (see pick_workspace); 1 = a single allocation")
    ap.add_argument("--seqs", type=int, default=None, help="number of sequences instead of the configuration's")
    ap.add_argument("--cpu-instances", type=int, default=32, help="head-instances the CPU oracle is timed on")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--split", action="store_true", help="call the three entry points instead of the fused one")
    ap.add_argument("--fill", action="store_true",
                    help="evict in place with the fewest moves (tri_compact_fill) instead of the ordered compaction")
    ap.add_argument("--post-rope", action="store_true", help="treat the cache as holding post-RoPE keys (k_rotated)")
    ap.add_argument("--half-split", action="store_true", help="band f = (x[f], x[f + d/2]) instead of (x[2f], x[2f+1])")
    ap.add_argument("--variant", type=int, default=0, help="score variant (0 full, 1 trig only, 2 norm only, 3 un-weighted norm)")
    ap.add_argument("--resident", action="store_true",
                    help="measurement aid: every head-instance reads the K rows of the first one (strides 0), so the "
                         "score kernel reads 8 MB over and over instead of streaming from HBM (out of the last-level "
                         "cache rather than L2, since work items take their tiles in rotated orders); not the benchmark")
    ap.add_argument("--inst-probe", action="store_true",
                    help="instead of the benchmark, print the issue rates of the instructions the score kernel is made of")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (a kernel of known traffic for scaling rocprofv3 byte counters)")
    ap.add_argument("--hbm-probe", action="store_true",
                    help="instead of the benchmark, print what a plain streaming read reaches on this GPU, alone "
                         "and with a thin write stream mixed in")
    args = ap.parse_args()
    if args.hbm_probe:
        from workload import device
        print(json.dumps({"hbm_probe_GBps": device.hbm_probe(), "peak_GBps": HBM_PEAK_GBS}), flush=True)
        return
    if args.inst_probe:
        from workload import device
        sys.stdout.write(device.inst_probe())
        return
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); --gpus %d is not supported"
              % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2604_04921_amd import binding as T
    from workload import device, recipe

    if args.resident:
        args.no_cpu = True   # the head-instances no longer hold their own keys
    cfg = recipe.CONFIGS[args.config]
    if args.seqs:
        cfg = recipe.scaled(cfg, n_seqs=args.seqs)
    mode = args.positions or cfg.positions
    L = args.layers or cfg.n_layers
    if args.slabs < 1 or (args.slabs > 1 and not args.layers) or args.slabs * L > max(cfg.n_layers, L):
        print("bench.py: --slabs needs --layers, and slabs x layers may not exceed the configuration's layers", file=sys.stderr)
        sys.exit(2)
    if args.slabs > 1:
        args.no_cpu = True   # the oracle's sample and the kept sets it is compared with belong to one slab
    parts = [measure(args, cfg, mode, L, i * L) for i in range(args.slabs)]
    m = parts[0]
    S, Hq, Hkv, B, d = cfg.n_seqs, cfg.n_q_heads, cfg.n_kv_heads, cfg.budget, cfg.head_dim
    paged, in_place, launches, t_gen = m["paged"], m["in_place"], sum(p_["launches"] for p_ in parts), sum(p_["t_gen"] for p_ in parts)
    lens = m["lens"]
    keys = sum(p_["keys"] for p_ in parts)
    ms = sum(p_["elapsed"] for p_ in parts) * 1e3 / args.steps
    value = keys / (ms * 1e-3) / 1e9
    # one step makes `launches` score launches (one per slab); their mean durations add up to the step's score time
    launch_ms = float(sum(np.mean(p_["k_ms"]) for p_ in parts)) / len(parts)
    eb = 2 if cfg.dtype == "bf16" else 4
    bytes_per_launch = (eb * d + 4) * keys / launches
    achieved = bytes_per_launch / (launch_ms * 1e-3) / 1e9
    L_all = L * args.slabs
    step_bytes = int(sum(STEP_BYTES(int(n), B) for n in lens)) * L_all * Hkv if eb == 2 else None
    if args.fill and step_bytes:   # only the kept keys stored beyond the new length move
        step_bytes = 260 * keys + 1032 * sum(p_["moved"] for p_ in parts)
    # which of the three score kernels ran (the library's dispatch rule, restated for the label only): bf16 keys in
    # blocks of 16 or more go to an MFMA kernel; of those, interleaved pairs to the one-key-per-lane kernel unless the
    # cache is paged and the batch large enough for 8192-key work items
    mfma_path = eb == 2 and (cfg.block_size == 0 or cfg.block_size >= 16)
    waves = 8 if Hq // Hkv > 4 else 12
    rounds = (L * S * Hkv * ((cfg.seq_len + 63) // 64)) // (4 * torch.cuda.get_device_properties(0).multi_processor_count * waves)
    small_items = rounds * waves * 64 < 8192
    lane = mfma_path and not args.half_split and (cfg.block_size == 0 or small_items)
    kernel = "score_lane_kernel" if lane else "score_mfma_kernel" if mfma_path else "score_kernel"
    roofline = {"bound": "hbm", "kernel": kernel, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": measured_traffic(cfg.name, mode, args),
                "launch_ms": round(launch_ms, 4), "launches_per_step": launches,
                "algorithmic_bytes_per_launch": int(bytes_per_launch)}
    if step_bytes:
        roofline["step_gbs"] = round(step_bytes / (ms * 1e-3) / 1e9, 1)
        roofline["step_frac"] = round(step_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)

    cpu = m["cpu"]

    out = {"metric": "cached keys scored+selected+compacted per second", "value": round(value, 3), "unit": "Gkeys/s",
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
           "data": "synthetic",
           "config": {"workload": cfg.name, "positions": mode, "layers": L_all, "slabs": args.slabs, "seqs": S, "kv_heads": Hkv,
                      "q_heads": Hq, "head_dim": d, "keys_per_seq": cfg.seq_len, "budget": B,
                      "n_offsets": len(cfg.offsets), "storage": cfg.dtype, "layout": "paged16" if paged else "contiguous",
                      "keys": keys, "entry": "split" if args.split else "tri_compress_step",
                      "compaction": "fill" if args.fill else "ordered",
                      "keys_stored": "post-rope" if args.post_rope else "pre-rope", "score_variant": args.variant, "pairs": "half-split" if args.half_split else "interleaved",
                      "timed": "each step alone, cache restored before it" if in_place else "all steps in one bracket",
                      "resident": bool(args.resident), "workspace_pick": m["ws_pick"],
                      "kernel_sources_sha16": kernel_sources_sha16(),
                      "generate_s": round(t_gen, 1)},
           "roofline": roofline, "cpu_baseline": cpu}
    print(json.dumps(out), flush=True)


def measure(args, cfg, mode, L, layer0):
    """Generates layers layer0 .. layer0 + L - 1 of the workload on the device, runs the warm-up and the timed steps on
    them and returns what the output line is made of; everything it allocated is released on return."""
    import numpy as np
    import torch
    from paper_2604_04921_amd import binding as T
    from workload import device, recipe

    dev = "cuda"
    t_gen = time.time()
    w = device.generate(cfg, positions=mode, layers=L, layer0=layer0)
    S, Hq, Hkv, B, d = cfg.n_seqs, cfg.n_q_heads, cfg.n_kv_heads, cfg.budget, cfg.head_dim
    model = T.Model(L, Hq, Hkv, d, cfg.rope_theta, cfg.offsets, pairs=int(args.half_split), score_variant=args.variant)
    k_view, v_view = w["k"], w["v"]
    if args.resident:   # one head-instance's rows for everybody: a cache-resident read stream
        assert "block_table" not in w and not args.fill, "--resident: contiguous layout, out-of-place compaction"
        k_view = w["k"][:1, :1, :1].expand(L, cfg.n_seqs, cfg.n_kv_heads, cfg.seq_len, cfg.head_dim)
        v_view = w["v"][:1, :1, :1].expand(L, cfg.n_seqs, cfg.n_kv_heads, cfg.seq_len, cfg.head_dim)
    src = T.Cache(k_view, v_view, w["pos"], w["seq_len"], w["cur_pos"], cfg.seq_len, w.get("block_table"),
                  k_rotated=args.post_rope)
    centers = torch.empty((L, Hq, d // 2, 3), dtype=torch.float32, device=dev)
    T.tri_build_centers(model, w["q_samples"], centers)
    paged = "block_table" in w
    if args.fill:
        dst = None
    elif paged:   # in place: the survivors go to the front blocks of the same pools
        dst = src
    else:
        kd = torch.empty((L, S, Hkv, B, d), dtype=w["k"].dtype, device=dev)
        vd = torch.empty_like(kd)
        pd = torch.empty((L, S, Hkv, B), dtype=torch.int32, device=dev)
        dst = T.Cache(kd, vd, pd, w["seq_len"], w["cur_pos"], B)
    kept_idx = torch.empty((L, S, Hkv, B), dtype=torch.int32, device=dev)
    kept_cnt = torch.empty((L, S, Hkv), dtype=torch.int32, device=dev)
    new_len = torch.empty((S,), dtype=torch.int32, device=dev)
    ws, ws_pick = pick_workspace(T, model, centers, src, cfg, L, B, args.ws_candidates)
    final = torch.empty((L, S, Hkv, cfg.seq_len), dtype=torch.float32, device=dev) if args.split else None
    if args.copy_calibration:   # reads 2^30 bytes and writes 2^30 bytes
        a_ = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        b_ = torch.empty_like(a_)
        b_.copy_(a_)
        del a_, b_
    torch.cuda.synchronize()
    t_gen = time.time() - t_gen

    def step():
        if args.split:
            T.tri_score(model, centers, src, final, None, ws)
            T.tri_select_topk(model, final, src, B, kept_idx, kept_cnt, ws)
            if dst is None:
                T.tri_compact_fill(model, src, B, kept_idx, kept_cnt, new_len)
            else:
                T.tri_compact(model, src, dst, B, kept_idx, kept_cnt, new_len)
        else:
            T.tri_compress_step(model, centers, src, dst, B, kept_idx, kept_cnt, new_len, ws)

    # In-place modes (paged: dst is src; --fill) overwrite the cache they score.  Every step must see the configured
    # workload, so the cache is put back from a device copy before each step, outside the timed region, and the
    # steps are timed one by one; the out-of-place default times all steps in one bracket.
    in_place = dst is None or dst is src
    orig = {n: w[n].clone() for n in ("k", "v", "pos")} if in_place else None

    def restore():
        if in_place:
            for n in ("k", "v", "pos"):
                w[n].copy_(orig[n])

    # the CPU oracle's sample is taken from the untouched cache
    cpu_sample = None if args.no_cpu else cpu_sample_inputs(cfg, w, L, args.cpu_instances, paged)

    # how many score-kernel launches one step makes (the hook brackets each of them)
    probe = [torch.cuda.Event(enable_timing=True) for _ in range(2 * 256)]
    for e in probe:
        e.record()
    torch.cuda.synchronize()
    keep = T.tri_timing_attach(probe)
    step()
    launches = T.tri_timing_detach()
    torch.cuda.synchronize()
    for _ in range(max(0, args.warmup - 1)):
        restore()
        step()
    torch.cuda.synchronize()

    events = [torch.cuda.Event(enable_timing=True) for _ in range(2 * launches * args.steps)]
    for e in events:
        e.record()
    torch.cuda.synchronize()
    keep = T.tri_timing_attach(events)
    if in_place:
        elapsed = 0.0
        for _ in range(args.steps):
            restore()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            step()
            torch.cuda.synchronize()
            elapsed += time.perf_counter() - t0
    else:
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
    got = T.tri_timing_detach()
    assert got == launches * args.steps, (got, launches, args.steps)
    del keep

    lens = w["seq_len"].cpu().numpy().astype(np.int64)
    k_ms = [events[2 * i].elapsed_time(events[2 * i + 1]) for i in range(launches * args.steps)]
    moved = int((kept_idx >= kept_cnt[..., None]).sum()) if args.fill else 0
    cpu = None
    if not args.no_cpu:
        cpu = cpu_baseline(cfg, cpu_sample, centers, kept_idx, kept_cnt, args.variant, args.post_rope, int(args.half_split))
    return {"elapsed": elapsed, "keys": int(lens.sum()) * L * Hkv, "k_ms": k_ms, "launches": launches, "lens": lens,
            "moved": moved, "cpu": cpu, "paged": paged, "in_place": in_place, "t_gen": t_gen, "ws_pick": ws_pick}


def pick_workspace(T, model, centers, src, cfg, L, B, n_candidates):
    """The step's scratch workspace, chosen as a caller may choose it at start-up: on this GPU the score launch runs up
    to 8 % faster or slower with where the workspace (the raw scores it writes) happens to lie in physical memory
    relative to the K cache it reads, which no caller can see or control.  So up to n_candidates workspaces are
    allocated 8 GB apart, the score launch is timed once on each (tri_score into a temporary final-score buffer: the
    caches are not touched), the fastest is kept and the others are freed.  All of this happens before the warm-up;
    the launch times of all candidates go into the output line.  n_candidates = 1: one allocation, no timing."""
    import torch
    nbytes = T.tri_workspace_size(model, src, B)
    dev = "cuda"
    if n_candidates <= 1:
        return torch.empty(nbytes, dtype=torch.uint8, device=dev), None
    S, Hkv = cfg.n_seqs, cfg.n_kv_heads
    final_bytes = L * S * Hkv * cfg.seq_len * 4
    spacing = 8 << 30
    cands, spacers = [], []
    for i in range(n_candidates):
        free, _ = torch.cuda.mem_get_info()
        if i and free < nbytes + spacing + final_bytes + (8 << 30):   # never at the price of running out of HBM
            break
        if i:
            spacers.append(torch.empty(spacing, dtype=torch.uint8, device=dev))
        cands.append(torch.empty(nbytes, dtype=torch.uint8, device=dev))
    if len(cands) == 1:
        return cands[0], None
    final = torch.empty((L, S, Hkv, cfg.seq_len), dtype=torch.float32, device=dev)
    times = []
    for wsc in cands:
        T.tri_score(model, centers, src, final, None, wsc)   # untimed first touch
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(64)]
        for e in ev:
            e.record()
        torch.cuda.synchronize()
        keep = T.tri_timing_attach(ev)
        T.tri_score(model, centers, src, final, None, wsc)
        torch.cuda.synchronize()
        n = T.tri_timing_detach()
        del keep
        times.append(sum(ev[2 * j].elapsed_time(ev[2 * j + 1]) for j in range(n)))
    best = min(range(len(cands)), key=lambda i: times[i])
    ws = cands[best]
    del cands, spacers, final
    torch.cuda.empty_cache()
    return ws, {"candidates": len(times), "spacing_gb": 8, "score_launch_ms": [round(t, 3) for t in times], "picked": best}


def measured_traffic(name, mode, args):
    """The counter-measured HBM bytes of one score launch, if they were measured on these kernel sources and this
    is the plain workload they were measured on; else None."""
    m = MEASURED_TRAFFIC.get("%s/%s" % (name, mode))
    plain = not (args.resident or args.post_rope or args.half_split or args.variant or args.seqs or args.layers)
    if m is None or not plain or m["sources_sha16"] != kernel_sources_sha16():
        return None
    return m["bytes"]


def cpu_sample_inputs(cfg, w, L, n_inst, paged):
    """Whole head-instances spread over layers and sequences, copied back from the device (before any step
    touches the cache): [(l, s, h), K rows, positions, cur_pos]."""
    import numpy as np
    import torch
    S, Hkv = cfg.n_seqs, cfg.n_kv_heads
    lens = w["seq_len"].cpu().numpy()
    cur = w["cur_pos"].cpu().numpy()
    picks = [((i * (L - 1)) // max(1, n_inst - 1) if n_inst > 1 else 0, (i * 5) % S, (i * 3) % Hkv) for i in range(n_inst)]
    jobs = []
    for (l, s, h) in picks:
        n = int(lens[s])
        if paged:
            bs = cfg.block_size
            bt = w["block_table"][s, : -(-n // bs)].long()
            k = w["k"][l, bt, h].reshape(-1, cfg.head_dim)[:n]
            p = w["pos"][l, bt, h].reshape(-1)[:n]
        else:
            k, p = w["k"][l, s, h, :n], w["pos"][l, s, h, :n]
        kn = k.contiguous().view(torch.int16).cpu().numpy().view(np.uint16) if k.dtype == torch.bfloat16 else k.cpu().numpy()
        jobs.append(((l, s, h), kn, p.cpu().numpy(), int(cur[s])))
    return jobs


def cpu_baseline(cfg, jobs, centers, kept_idx, kept_cnt, variant=0, rotated=False, pairs=0):
    """The CPU oracle, as it stands, on a bounded sample of the same workload: whole head-instances spread
    over layers and sequences.  Also confirms the GPU's kept sets on them."""
    import numpy as np
    from oracle import tri_oracle as O

    G = cfg.group
    stats = centers.cpu().numpy()
    threads = min(16, os.cpu_count() or 1)
    O.lib()
    t0 = time.perf_counter()
    res = [O.head_instance(stats[l, h * G:(h + 1) * G], kn, p, c, cfg.rope_theta, cfg.offsets, cfg.budget, threads=threads,
                            variant=variant, rotated=rotated, pairs=pairs)
           for ((l, s, h), kn, p, c) in jobs]
    dt = time.perf_counter() - t0
    nkeys = sum(j[1].shape[0] for j in jobs)
    same = 0
    for ((l, s, h), _, _, _), r in zip(jobs, res):
        c = int(kept_cnt[l, s, h])
        same += int(np.array_equal(kept_idx[l, s, h, :c].cpu().numpy(), r["idx"]))
    return {"value": round(nkeys / dt / 1e9, 9), "unit": "Gkeys/s", "cores": threads, "kind": "oracle",
            "sample": "%d whole head-instances (%d keys) spread over layers/sequences, score+reduce+select; "
                      "compaction is a memcpy and is left out" % (len(jobs), nkeys),
            "seconds": round(dt, 2), "kept_sets_identical_to_gpu": "%d/%d" % (same, len(jobs))}


if __name__ == "__main__":
    main()
