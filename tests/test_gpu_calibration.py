"""Calibration at scale and the diagnostics of the statistics table, against the oracle (Section 4.1,
Appendix B.5, B.7, H): centres accumulated over chunks, Mean Resultant Length, band contributions, dominant bands."""
import numpy as np
import pytest
import torch

from workload import recipe
from tri_harness import to_torch

pytestmark = pytest.mark.gpu


def _samples(rng, T, L, H, d, dtype):
    centre = rng.standard_normal((1, L, H, d)) * rng.uniform(0.1, 4.0, size=(1, L, H, d))
    x = (centre + 0.5 * rng.standard_normal((T, L, H, d))).astype(np.float32)
    return recipe.store(x, dtype)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("pairs", [0, 1])
def test_centres_from_chunks(oracle, dtype, pairs):
    """Chunks of different sizes (one of a single token) accumulate to the centres of the whole sample."""
    from paper_2604_04921_amd import binding as B
    rng = np.random.default_rng(11 + pairs)
    T, L, Hq, d = 1000, 2, 4, 128
    q = _samples(rng, T, L, Hq, d, dtype)
    ref = oracle.centers(q, pairs=pairs)
    model = B.Model(L, Hq, 2, d, 1e6, [1, 2, 4], pairs)
    sums = torch.full((L, Hq, d // 2, 3), float("nan"), dtype=torch.float64, device="cuda")   # first=1 must overwrite
    out = torch.empty((L, Hq, d // 2, 3), dtype=torch.float32, device="cuda")
    bounds = [0, 333, 334, 900, 1000]
    for i in range(len(bounds) - 1):
        chunk = to_torch(q[bounds[i]:bounds[i + 1]], dtype)
        B.tri_centers_accumulate(model, chunk, sums, first=(i == 0))
    B.tri_centers_finalize(model, sums, T, out)
    torch.cuda.synchronize()
    np.testing.assert_allclose(out.cpu().numpy(), ref, rtol=3e-7, atol=1e-30)
    # and the one-shot entry point agrees with the chunked one to the same bar
    one = torch.empty_like(out)
    B.tri_build_centers(model, to_torch(q, dtype), one)
    torch.cuda.synchronize()
    np.testing.assert_allclose(one.cpu().numpy(), ref, rtol=3e-7, atol=1e-30)


def test_band_diagnostics(oracle):
    from paper_2604_04921_amd import binding as B
    rng = np.random.default_rng(12)
    T, L, Hq, Hkv, d, K = 300, 3, 8, 2, 128, 5
    q = _samples(rng, T, L, Hq, d, "bf16")
    k = _samples(rng, T, L, Hkv, d, "bf16")
    qs, ks = oracle.centers(q), oracle.centers(k)
    qs[0, 0, 7] = 0.0                         # an all-zero band: R = 0 by convention
    ks[1, 1, 3:6, 2] = ks[1, 1, 3, 2]         # equal key moduli in three bands
    qs[1, 4:8, 3:6, 2] = qs[1, 4, 3, 2]       # ... and equal query moduli for heads 4..7 (they pair with KV head 1): tied contributions
    ref_mrl = oracle.mrl(qs)
    ref_c, ref_top = oracle.band_contrib(qs, ks, K)
    model = B.Model(L, Hq, Hkv, d, 1e6, [1, 2, 4])
    qd, kd = torch.from_numpy(qs).cuda(), torch.from_numpy(ks).cuda()
    mrl = torch.empty((L, Hq, d // 2), dtype=torch.float32, device="cuda")
    con = torch.empty_like(mrl)
    top = torch.full((L, Hq, K), -1, dtype=torch.int32, device="cuda")
    B.tri_band_diagnostics(model, qd, kd, mrl, con, K, top)
    torch.cuda.synchronize()
    np.testing.assert_allclose(mrl.cpu().numpy(), ref_mrl, rtol=2e-7, atol=1e-30)
    np.testing.assert_allclose(con.cpu().numpy(), ref_c, rtol=2e-7)
    got = top.cpu().numpy()
    # ranking is integer work on fp32 contributions: the same decision in the same precision
    c32 = con.cpu().numpy()
    for l in range(L):
        for h in range(Hq):
            np.testing.assert_array_equal(got[l, h], np.argsort(-c32[l, h], kind="stable")[:K])
    # where the oracle's contributions are well separated (or exactly tied), its bands are the same
    same = sum(int(np.array_equal(got[l, h], ref_top[l, h])) for l in range(L) for h in range(Hq))
    assert same >= L * Hq - 1
    np.testing.assert_array_equal(got[1, 4:8], ref_top[1, 4:8])
    # MRL alone needs no key table
    mrl2 = torch.empty_like(mrl)
    B.tri_band_diagnostics(model, qd, None, mrl2)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(mrl2.cpu().numpy(), mrl.cpu().numpy())
    with pytest.raises(B.TriError):
        B.tri_band_diagnostics(model, qd, None, mrl2, con, K, top)
