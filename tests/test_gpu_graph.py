"""tri_compress_step recorded into a HIP graph: the library allocates nothing and only enqueues kernels, so a caller
may capture it.  Every replay is checked against the eager result; between replays the inputs change and ordinary
eager work and synchronisations run, as they would in a serving loop."""
import numpy as np
import pytest
import torch

from workload import recipe
from tri_harness import GpuRun, to_torch

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("fill", [False, True])
def test_compress_step_in_a_graph(oracle, fill):
    cfg = recipe.scaled(recipe.CONFIGS["steady_state"], n_layers=2, n_seqs=3, n_q_heads=8, n_kv_heads=2, seq_len=700,
                        budget=600, n_calib=128)
    w = recipe.generate(cfg)
    run = GpuRun(cfg, w)
    run.build_centers()
    B = run.B
    k0, v0, p0 = run.k.clone(), run.v.clone(), run.pos.clone()
    dst = None
    if not fill:
        kd, vd, pd = torch.zeros_like(run.k), torch.zeros_like(run.v), torch.zeros_like(run.pos)
        dst = B.Cache(kd, vd, pd, run.seq_len, run.cur_pos, run.nmax)

    def step(stream=None):
        B.tri_compress_step(run.model, run.centers, run.cache, dst, cfg.budget, run.kept_idx, run.kept_cnt, run.new_len,
                            run.ws, stream=stream)

    def outputs():
        torch.cuda.synchronize()
        cache_out = (run.k, run.v, run.pos) if fill else (kd, vd, pd)
        return [t.clone() for t in (run.kept_idx, run.kept_cnt, run.new_len) + cache_out]

    def set_inputs(shift):
        # another workload each time: keys rolled along the slot axis, the query moved on
        run.k.copy_(torch.roll(k0, shifts=shift, dims=3))
        run.v.copy_(v0)
        run.pos.copy_(p0)
        run.cur_pos.copy_(torch.from_numpy(w["cur_pos"] + shift).cuda())
        for t in (run.kept_idx, run.kept_cnt, run.new_len):
            t.fill_(-1)

    shifts = [0, 5, 111]
    eager = []
    for sh in shifts:                      # eager reference (also sets the kernels' attributes before any capture)
        set_inputs(sh)
        step()
        eager.append(outputs())

    g = torch.cuda.CUDAGraph()
    set_inputs(0)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(g, stream=s):
        step(stream=torch.cuda.current_stream())
    torch.cuda.synchronize()
    for rep, sh in enumerate(shifts + shifts):
        set_inputs(sh)
        scratch = torch.randn(1 << 16, device="cuda").sum().item()   # unrelated eager work and a synchronisation
        assert np.isfinite(scratch)
        g.replay()
        got = outputs()
        for a, b in zip(got, eager[shifts.index(sh)]):
            assert torch.equal(a, b), "replay %d (shift %d) differs from the eager result" % (rep, sh)


def test_two_calls_on_two_streams():
    """Two tri_compress_step calls in flight at once on two streams, each with its own workspace (the score kernel's
    item counter and work list live there): both give what they give one after the other."""
    cfgs = [recipe.scaled(recipe.CONFIGS["c2_layer"], n_layers=2, n_seqs=3, n_q_heads=8, n_kv_heads=2, seq_len=20000,
                          min_seq_len=3000, budget=512, n_calib=128, seed=recipe.SEED_BASE + 40 + i) for i in range(2)]
    runs = []
    for cfg in cfgs:
        run = GpuRun(cfg, recipe.generate(cfg))
        run.build_centers()
        kd, vd, pd = torch.zeros_like(run.k), torch.zeros_like(run.v), torch.zeros_like(run.pos)
        run.dst_tensors = (kd, vd, pd)
        run.dst = run.B.Cache(kd, vd, pd, run.seq_len, run.cur_pos, run.nmax)
        runs.append(run)

    def launch(run, stream=None):
        run.B.tri_compress_step(run.model, run.centers, run.cache, run.dst, run.cfg.budget, run.kept_idx, run.kept_cnt,
                                run.new_len, run.ws, stream=stream)

    def outputs(run):
        return [t.clone() for t in (run.kept_idx, run.kept_cnt, run.new_len) + run.dst_tensors]

    serial = []
    for run in runs:
        launch(run)
        torch.cuda.synchronize()
        serial.append(outputs(run))
        for t in (run.kept_idx, run.kept_cnt, run.new_len) + run.dst_tensors:
            t.fill_(0)
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    for s in streams:
        s.wait_stream(torch.cuda.current_stream())
    for rep in range(3):
        for run, s in zip(runs, streams):
            launch(run, stream=s)
    torch.cuda.synchronize()
    for run, ref in zip(runs, serial):
        for a, b in zip(outputs(run), ref):
            assert torch.equal(a, b)
