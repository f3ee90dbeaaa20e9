"""Pins for the CPU oracle: each test holds one oracle routine against something the paper or the
mathematics fixes independently of the oracle's own formula (a different definition, a closed form,
an invariant, brute force).  A dropped term, a wrong sign or index, or swapped operands in
tri_oracle.c fails at least one of them."""
import math
import os

import numpy as np
import pytest
from scipy import special

from workload import recipe

HERE = os.path.dirname(os.path.abspath(__file__))


def rope_rotate(x, p, theta):
    """Section 2.1 Eq. 1: rotate every (x[2f], x[2f+1]) pair of a real d-vector by omega_f * p."""
    d = x.shape[-1]
    y = np.empty_like(x, dtype=np.float64)
    for f in range(d // 2):
        w = theta ** (-2.0 * f / d)
        c, s = math.cos(w * p), math.sin(w * p)
        y[2 * f] = c * x[2 * f] - s * x[2 * f + 1]
        y[2 * f + 1] = s * x[2 * f] + c * x[2 * f + 1]
    return y


def random_case(rng, d, absmean_slack=True):
    F = d // 2
    stats = np.zeros((F, 3), dtype=np.float32)
    stats[:, 0:2] = rng.standard_normal((F, 2)).astype(np.float32) * 2
    A = np.hypot(stats[:, 0].astype(np.float64), stats[:, 1].astype(np.float64))
    stats[:, 2] = (A * (1.0 + (rng.random(F) if absmean_slack else 0.0))).astype(np.float32)
    key = rng.standard_normal(d).astype(np.float32) * 3
    return stats, key


# ---- S_trig -----------------------------------------------------------------------------------

@pytest.mark.parametrize("d", [2, 8, 32, 128])
@pytest.mark.parametrize("theta", [1e4, 1e6])
def test_s_trig_equals_rotated_dot_product(oracle, d, theta):
    """P1: S_trig(k, p_q - p_k) is the plain real dot product of the centre rotated to p_q with the
    key rotated to p_k (Section 2.1 Eq. 1 applied to both; Appendix B.2)."""
    rng = np.random.default_rng(100 + d)
    for _ in range(20):
        stats, key = random_case(rng, d)
        centre = stats[:, 0:2].reshape(-1).astype(np.float64)   # interleaved (re, im)
        p_q, p_k = int(rng.integers(0, 5000)), int(rng.integers(0, 5000))
        brute = float(np.dot(rope_rotate(centre, p_q, theta), rope_rotate(key.astype(np.float64), p_k, theta)))
        got = oracle.s_trig(stats, key, theta, p_q - p_k)
        assert got == pytest.approx(brute, rel=1e-11, abs=1e-10)


def test_score_avg_equals_brute_force_over_offsets(oracle):
    """P1 for the averaged score: mean over offsets of rotated dot products plus the norm term
    written with plain square roots."""
    rng = np.random.default_rng(7)
    d, theta = 16, 1e4
    offs = np.array([1, 2, 4, 8, 16, 32], dtype=np.int64)
    for _ in range(20):
        stats, key = random_case(rng, d)
        centre = stats[:, 0:2].reshape(-1).astype(np.float64)
        p_q, p_k = int(rng.integers(100, 200)), int(rng.integers(0, 100))
        k64 = key.astype(np.float64)
        trig = np.mean([np.dot(rope_rotate(centre, p_q + int(o), theta), rope_rotate(k64, p_k, theta)) for o in offs])
        norm = 0.0
        for f in range(d // 2):
            A = math.sqrt(float(stats[f, 0]) ** 2 + float(stats[f, 1]) ** 2)
            m = math.sqrt(k64[2 * f] ** 2 + k64[2 * f + 1] ** 2)
            norm += (float(stats[f, 2]) - A) * m
        got = oracle.score_avg(stats, key, theta, p_q, p_k, offs)
        assert got == pytest.approx(trig + norm, rel=1e-11, abs=1e-10)


def test_shift_invariance(oracle):
    """P2: the score depends on positions through p_q - p_k only (Section 3.2 Eq. 2)."""
    rng = np.random.default_rng(11)
    d, theta = 128, 1e6
    offs = recipe.CONFIGS["c1_tiny"].offsets
    stats, key = random_case(rng, d)
    base = oracle.score_avg(stats, key, theta, 4096, 17, offs)
    for s in (1, 1000, 123457):
        assert oracle.score_avg(stats, key, theta, 4096 + s, 17 + s, offs) == base
    assert oracle.score_avg(stats, key, theta, 4097, 17, offs) != base


def test_single_band_closed_form(oracle):
    """P3: with one non-zero band the series is A m cos(omega_f x + phi)."""
    d, theta = 16, 1e4
    for f in (0, 3, 7):
        stats = np.zeros((d // 2, 3), dtype=np.float32)
        stats[f] = (1.5, -2.0, 2.5)
        key = np.zeros(d, dtype=np.float32)
        key[2 * f], key[2 * f + 1] = -0.75, 1.25
        x = 37
        w = theta ** (-2.0 * f / d)
        A, m = math.hypot(1.5, -2.0), math.hypot(-0.75, 1.25)
        phi = math.atan2(-2.0, 1.5) - math.atan2(1.25, -0.75)
        assert oracle.s_trig(stats, key, theta, x) == pytest.approx(A * m * math.cos(w * x + phi), rel=1e-13)
        # a key whose only energy is in another band scores zero
        key2 = np.zeros(d, dtype=np.float32)
        key2[(2 * f + 2) % d] = 1.0
        assert oracle.s_trig(stats, key2, theta, x) == pytest.approx(0.0, abs=1e-15)


def test_zero_distance_is_plain_dot_product(oracle):
    """P4: at distance 0 nothing rotates, so S_trig is the real dot product of centre and key."""
    rng = np.random.default_rng(5)
    stats, key = random_case(rng, 64)
    centre = stats[:, 0:2].reshape(-1).astype(np.float64)
    assert oracle.s_trig(stats, key, 1e6, 0) == pytest.approx(float(np.dot(centre, key.astype(np.float64))), rel=1e-12)


def test_ab_form(oracle):
    """P5: Appendix B.3: sum_f a_f cos(omega_f x) + b_f sin(omega_f x) with a_f = A m cos(phi_f),
    b_f = -A m sin(phi_f), written here from the complex product q conj(k)."""
    rng = np.random.default_rng(9)
    d, theta = 32, 1e4
    stats, key = random_case(rng, d)
    q = stats[:, 0].astype(np.float64) + 1j * stats[:, 1].astype(np.float64)
    k = key[0::2].astype(np.float64) + 1j * key[1::2].astype(np.float64)
    z = q * np.conj(k)        # |z| = A m, arg z = phi
    for x in (1, 50, 4097):
        w = theta ** (-2.0 * np.arange(d // 2) / d)
        ab = np.sum(z.real * np.cos(w * x) - z.imag * np.sin(w * x))
        assert oracle.s_trig(stats, key, theta, x) == pytest.approx(float(ab), rel=1e-11, abs=1e-11)


def test_sign_of_distance_matters(oracle):
    """A swapped Delta = p_k - p_q (or phi = arg k - arg q) changes the value: guards the sign pins."""
    rng = np.random.default_rng(3)
    stats, key = random_case(rng, 8)
    assert abs(oracle.s_trig(stats, key, 1e4, 5) - oracle.s_trig(stats, key, 1e4, -5)) > 1e-3


def test_golden_closed_forms(oracle):
    """Hand-derived closed forms in tests/golden/closed_forms.txt (Sections 4.1-4.2)."""
    n = 0
    for line in open(os.path.join(HERE, "golden", "closed_forms.txt")):
        if line.startswith("#") or not line.strip():
            continue
        head, st, ky, pp, of, ex = [s.split() for s in line.split("|")]
        d, theta = int(head[1]), float(head[2])
        stats = np.array(st, dtype=np.float32).reshape(d // 2, 3)
        key = np.array(ky, dtype=np.float32)
        got = oracle.score_avg(stats, key, theta, int(pp[0]), int(pp[1]), np.array(of, dtype=np.int64))
        assert got == pytest.approx(float(ex[0]), rel=1e-12)
        n += 1
    assert n == 3


def test_half_split_pairing(oracle):
    """The half-split layout scores a permuted vector exactly like the interleaved layout scores the original."""
    rng = np.random.default_rng(21)
    d = 16
    stats, key = random_case(rng, d)
    perm = np.concatenate([key[0::2], key[1::2]])
    assert oracle.s_trig(stats, perm, 1e4, 9, pairs=oracle.PAIR_HALF) == oracle.s_trig(stats, key, 1e4, 9)
    assert oracle.s_norm(stats, perm, pairs=oracle.PAIR_HALF) == oracle.s_norm(stats, key)


# ---- S_norm -----------------------------------------------------------------------------------

def test_s_norm_two_forms_and_limits(oracle):
    """P6: the (1 - R_f) form equals the difference form; R_f = 1 gives 0; the weight is never negative."""
    rng = np.random.default_rng(13)
    stats, key = random_case(rng, 64)
    a = oracle.s_norm(stats, key)
    b = oracle.s_norm(stats, key, mrl_form=True)
    assert a == pytest.approx(b, rel=1e-12)
    assert a > 0
    k = key[0::2].astype(np.float64) + 1j * key[1::2].astype(np.float64)
    A = np.abs(stats[:, 0].astype(np.float64) + 1j * stats[:, 1].astype(np.float64))
    assert a == pytest.approx(float(np.sum((stats[:, 2].astype(np.float64) - A) * np.abs(k))), rel=1e-12)
    tight, key2 = random_case(rng, 64, absmean_slack=False)
    assert abs(oracle.s_norm(tight, key2)) < 1e-5 * np.abs(key2).sum()   # fp32 rounding of E|q| only


def test_single_offset_reduces_to_one_evaluation(oracle):
    """P7: |D| = 1."""
    rng = np.random.default_rng(17)
    stats, key = random_case(rng, 32)
    got = oracle.score_avg(stats, key, 1e4, 100, 40, np.array([8], dtype=np.int64))
    assert got == pytest.approx(oracle.s_trig(stats, key, 1e4, 68) + oracle.s_norm(stats, key), rel=1e-14)


def test_offset_fold_identity(oracle):
    """P8: mean over offsets of Re(z e^{i w (x + delta)}) = Re(z E e^{i w x}), E = mean_delta e^{i w delta}.
    This is the algebra the HIP kernel relies on, checked here against the literal oracle."""
    rng = np.random.default_rng(19)
    d, theta = 128, 1e6
    offs = recipe.CONFIGS["c1_tiny"].offsets
    stats, key = random_case(rng, d)
    q = stats[:, 0].astype(np.float64) + 1j * stats[:, 1].astype(np.float64)
    k = key[0::2].astype(np.float64) + 1j * key[1::2].astype(np.float64)
    w = theta ** (-2.0 * np.arange(d // 2) / d)
    E = np.exp(1j * np.outer(w, offs)).mean(axis=1)
    p_q, p_k = 4096, 1234
    folded = np.sum((q * E * np.exp(1j * w * p_q) * np.conj(k * np.exp(1j * w * p_k))).real)
    c = stats[:, 2].astype(np.float64) - np.abs(q)
    folded += np.sum(c * np.abs(k))
    assert oracle.score_avg(stats, key, theta, p_q, p_k, offs) == pytest.approx(float(folded), rel=1e-11)


# ---- GQA normalise + max ----------------------------------------------------------------------

def test_zscore_moments_and_max(oracle):
    """P9: after normalisation each head has mean 0 and population std 1; S_final is the row-wise max."""
    rng = np.random.default_rng(23)
    raw = rng.standard_normal((4, 1000)) * np.array([[1.0], [10.0], [0.1], [3.0]]) + np.array([[5.0], [-2.0], [0.0], [100.0]])
    mu, sigma, final = oracle.gqa_final(raw)
    np.testing.assert_allclose(mu, raw.mean(axis=1), rtol=1e-13)
    np.testing.assert_allclose(sigma, raw.std(axis=1, ddof=0), rtol=1e-12)
    z = (raw - mu[:, None]) / sigma[:, None]
    np.testing.assert_allclose(z.mean(axis=1), 0, atol=1e-12)
    np.testing.assert_allclose(z.std(axis=1), 1, rtol=1e-12)
    np.testing.assert_allclose(final, z.max(axis=0), rtol=1e-12, atol=1e-12)
    # the maximum really is taken over heads: each head wins somewhere
    assert len(set(np.argmax(z, axis=0))) == 4


def test_zscore_degenerate(oracle):
    """sigma = 0 for a head makes that head contribute 0 everywhere; N = 1 gives 0."""
    raw = np.array([[2.0, 2.0, 2.0, 2.0], [1.0, 2.0, 3.0, 4.0]])
    mu, sigma, final = oracle.gqa_final(raw)
    assert sigma[0] == 0
    z1 = (raw[1] - 2.5) / np.std(raw[1])
    np.testing.assert_allclose(final, np.maximum(0.0, z1), rtol=1e-13)
    _, _, f1 = oracle.gqa_final(np.array([[3.0]]))
    assert f1[0] == 0
    # equal scores whose mean is not exact in binary (3000 x 0.1: sum / N differs from 0.1 in the last bit) still
    # have sigma = 0: the head contributes 0, not +-1
    raw = np.vstack([np.full(3000, 0.1), np.linspace(-1.0, 1.0, 3000)])
    assert np.sum(raw[0]) / 3000 != 0.1
    mu, sigma, final = oracle.gqa_final(raw)
    assert sigma[0] == 0
    np.testing.assert_allclose(final, np.maximum(0.0, (raw[1] - raw[1].mean()) / raw[1].std()), rtol=1e-12, atol=1e-15)


def test_head_scale_invariance(oracle):
    """P10: multiplying one head's statistics by a positive constant leaves its normalised scores unchanged."""
    cfg = recipe.scaled(recipe.CONFIGS["c1_tiny"], seq_len=96, n_calib=64)
    w = recipe.generate(cfg)
    stats = oracle.centers(w["q_samples"])[0]
    K, pos = w["k"][0, 0, 0], w["pos"][0, 0, 0]
    r1 = oracle.raw_scores(stats, K, pos, int(w["cur_pos"][0]), cfg.rope_theta, cfg.offsets)
    st2 = stats.copy()
    st2[1] *= 8.0     # power of two: exact in fp32
    r2 = oracle.raw_scores(st2, K, pos, int(w["cur_pos"][0]), cfg.rope_theta, cfg.offsets)
    np.testing.assert_allclose(r2[1], 8.0 * r1[1], rtol=1e-13)
    _, _, f1 = oracle.gqa_final(r1)
    _, _, f2 = oracle.gqa_final(r2)
    np.testing.assert_allclose(f1, f2, rtol=1e-10, atol=1e-12)


def test_single_head_topk_matches_raw(oracle):
    """P11: with G = 1 the z-score is monotone, so top-B of S_final equals top-B of the raw score."""
    rng = np.random.default_rng(29)
    raw = rng.standard_normal((1, 500))
    _, _, final = oracle.gqa_final(raw)
    np.testing.assert_array_equal(oracle.topk(final, 50), oracle.topk(raw[0], 50))


# ---- top-B ------------------------------------------------------------------------------------

def brute_topk(s, B):
    """Definition by rank counting: key i is kept iff fewer than B keys beat it, where j beats i when
    s_j > s_i, or s_j == s_i and j < i."""
    n = len(s)
    keep = []
    for i in range(n):
        rank = sum(1 for j in range(n) if s[j] > s[i] or (s[j] == s[i] and j < i))
        if rank < B:
            keep.append(i)
    return np.array(keep, dtype=np.int32)


def test_topk_matches_rank_counting(oracle):
    """P12 with heavy ties."""
    rng = np.random.default_rng(31)
    for n, B in [(1, 1), (7, 3), (64, 64), (200, 17), (300, 299), (50, 80)]:
        s = rng.integers(0, 6, size=n).astype(np.float64)   # many equal scores
        np.testing.assert_array_equal(oracle.topk(s, B), brute_topk(s, B))
    s = np.array([0.0, -0.0, 1.0, -0.0, 0.0, -1.0])
    np.testing.assert_array_equal(oracle.topk(s, 3), [0, 1, 2])       # -0.0 ties with +0.0, lower index wins
    assert len(oracle.topk(np.zeros(0), 4)) == 0


def test_topk_matches_stable_sort_large(oracle):
    rng = np.random.default_rng(37)
    s = np.round(rng.standard_normal(20000), 2)
    B = 2048
    order = np.argsort(-s, kind="stable")
    np.testing.assert_array_equal(oracle.topk(s, B), np.sort(order[:B]))
    np.testing.assert_array_equal(oracle.topk(s, 30000), np.arange(20000))   # B >= N keeps everything


def test_topk_all_equal_keeps_prefix(oracle):
    np.testing.assert_array_equal(oracle.topk(np.full(100, 3.5), 10), np.arange(10))


# ---- compaction -------------------------------------------------------------------------------

def test_compact_rows(oracle):
    """P13: row j of the result is row idx[j] of the source; in place equals out of place; prefix is idempotent."""
    rng = np.random.default_rng(41)
    src = rng.integers(0, 65535, size=(300, 128)).astype(np.uint16)
    idx = np.sort(rng.choice(300, size=77, replace=False)).astype(np.int32)
    out = oracle.compact_rows(src, idx)
    np.testing.assert_array_equal(out, src[idx])
    inplace = src.copy()
    oracle.compact_rows(inplace, idx, out=inplace)
    np.testing.assert_array_equal(inplace[:77], src[idx])
    np.testing.assert_array_equal(inplace[77 + 1:][idx[-1]:], src[77 + 1:][idx[-1]:])   # rows past the last source untouched
    same = src.copy()
    oracle.compact_rows(same, np.arange(50, dtype=np.int32), out=same)
    np.testing.assert_array_equal(same, src)


def test_paged_gather_and_compact(oracle):
    cfg = recipe.scaled(recipe.CONFIGS["c4_paged"], n_layers=2, n_seqs=3, n_kv_heads=2, n_q_heads=8, seq_len=100,
                        min_seq_len=20, head_dim=8, n_calib=4)
    lens = recipe.seq_lens(cfg)
    bt, nb = recipe.paged_layout(cfg, lens)
    rng = np.random.default_rng(43)
    x = rng.integers(0, 65535, size=(2, 3, 2, 100, 8)).astype(np.uint16)
    pool = recipe.to_paged(x, lens, bt, nb, 16)
    H, bs, w = 2, 16, 8
    strides = (nb * H * bs * w, H * bs * w, bs * w, w)
    for (l, s, h) in [(0, 0, 0), (1, 2, 1), (1, 1, 0)]:
        n = int(lens[s])
        got = oracle.paged_gather(pool, w, bt, bs, strides, l, s, h, n)
        np.testing.assert_array_equal(got, x[l, s, h, :n])
        idx = np.sort(rng.choice(n, size=n // 3, replace=False)).astype(np.int32)
        p2 = pool.copy()
        oracle.paged_compact(p2, w, bt, bs, strides, l, s, h, idx)
        after = oracle.paged_gather(p2, w, bt, bs, strides, l, s, h, len(idx))
        np.testing.assert_array_equal(after, x[l, s, h, idx])
        # other head-instances are untouched
        other = oracle.paged_gather(p2, w, bt, bs, strides, 1 - l, s, h, n)
        np.testing.assert_array_equal(other, x[1 - l, s, h, :n])


# ---- centres ----------------------------------------------------------------------------------

def test_centres_match_numpy_means(oracle):
    """P14: complex mean and mean modulus per (layer, head, band), in double, rounded once."""
    cfg = recipe.scaled(recipe.CONFIGS["c2_layer"], n_q_heads=4, n_kv_heads=2, seq_len=8, n_calib=500)
    w = recipe.generate(cfg)
    q = recipe.bf16_bits_to_f32(w["q_samples"]).astype(np.float64)        # [T][L][Hq][d]
    z = q[..., 0::2] + 1j * q[..., 1::2]
    st = oracle.centers(w["q_samples"])
    np.testing.assert_array_equal(st[..., 0], z.real.mean(axis=0).astype(np.float32))
    np.testing.assert_array_equal(st[..., 1], z.imag.mean(axis=0).astype(np.float32))
    np.testing.assert_allclose(st[..., 2], np.abs(z).mean(axis=0), rtol=2e-7)
    A = np.hypot(st[..., 0].astype(np.float64), st[..., 1].astype(np.float64))
    assert np.all(st[..., 2] >= A * (1 - 1e-6))       # triangle inequality: R_f <= 1


def test_generator_concentration_matches_rice_mean(oracle):
    """The generator's Mean Resultant Length has the closed form of the Rice distribution:
    E|c + n| = s sqrt(pi/2) L_{1/2}(-|c|^2 / (2 s^2)), s^2 the per-component variance.  At noise 0.3 this
    gives R = 0.978, the value the paper measures on Qwen3-8B (Section 3.3)."""
    cfg = recipe.scaled(recipe.CONFIGS["c1_tiny"], seq_len=8, n_calib=20000)
    w = recipe.generate(cfg)
    st = oracle.centers(w["q_samples"]).astype(np.float64)
    R = np.hypot(st[..., 0], st[..., 1]) / st[..., 2]
    s2 = 0.3 ** 2 / 2
    x = -1.0 / (2 * s2)
    rice_mean = math.sqrt(s2) * math.sqrt(math.pi / 2) * special.hyp1f1(-0.5, 1.0, x)
    assert 1.0 / rice_mean == pytest.approx(0.978, abs=1e-3)
    assert R.mean() == pytest.approx(1.0 / rice_mean, abs=2e-3)
    assert 0.97 < R.min() and R.max() < 0.99


def test_compact_fill_moves_only_into_holes(oracle):
    """Minimal-move compaction: afterwards slots [0, cnt) hold exactly the kept rows (as a set), kept rows that
    were already below cnt have not moved, and the number of rows that changed equals the number of holes."""
    rng = np.random.default_rng(47)
    for n, cnt in [(50, 20), (300, 256), (64, 64), (10, 1), (40, 39)]:
        src = rng.integers(1, 65535, size=(n, 16)).astype(np.uint16)
        src[:, 0] = np.arange(n)                      # every row distinct
        idx = np.sort(rng.choice(n, size=cnt, replace=False)).astype(np.int32)
        out = oracle.compact_fill(src.copy(), idx)
        assert sorted(out[:cnt, 0].tolist()) == sorted(idx.tolist())
        stay = idx[idx < cnt]
        np.testing.assert_array_equal(out[stay], src[stay])
        holes = cnt - len(stay)
        assert int(np.any(out[:cnt] != src[:cnt], axis=1).sum()) == holes
        np.testing.assert_array_equal(out[cnt:], src[cnt:])     # nothing beyond cnt is written
        # pairing rule: i-th hole (ascending) <- i-th tail survivor (ascending)
        hole_slots = np.setdiff1d(np.arange(cnt), stay)
        np.testing.assert_array_equal(out[hole_slots], src[idx[idx >= cnt]])


# ---- scoring variants of the ablation study, post-RoPE caches -----------------------------------

def test_unweighted_norm_score(oracle):
    """P16: S_norm^(0) = sum_f E|q_f| |k_f| (Section 4.1).  For a key that coincides with the query centre,
    S_trig at distance 0 is sum_f |E q_f|^2 (a plain dot product of the centre with itself), and that is exactly
    what the concentration weighting removes: S_norm^(0) - S_norm = sum_f |E q_f| |k_f|."""
    rng = np.random.default_rng(41)
    stats, key = random_case(rng, 64)
    k = key[0::2].astype(np.float64) + 1j * key[1::2].astype(np.float64)
    assert oracle.s_norm0(stats, key) == pytest.approx(float(np.sum(stats[:, 2].astype(np.float64) * np.abs(k))), rel=1e-12)
    centre_key = stats[:, 0:2].reshape(-1).copy()
    dot = float(np.dot(centre_key.astype(np.float64), centre_key.astype(np.float64)))
    assert oracle.s_trig(stats, centre_key, 1e4, 0) == pytest.approx(dot, rel=1e-12)
    assert oracle.s_norm0(stats, centre_key) - oracle.s_norm(stats, centre_key) == pytest.approx(dot, rel=1e-9)
    # half-split layout reads the same numbers from other places
    perm = np.concatenate([key[0::2], key[1::2]])
    assert oracle.s_norm0(stats, perm, pairs=oracle.PAIR_HALF) == oracle.s_norm0(stats, key)


def test_variants_are_the_sums_of_their_parts(oracle):
    """P17: the ablation variants (Section 5): trig-only + norm-only = full; "w/o R" exceeds the full score by
    S_norm^(0) - S_norm; norm-only does not depend on positions or offsets; trig-only of a single offset is one
    evaluation of the series."""
    rng = np.random.default_rng(42)
    G, N, d = 3, 40, 32
    stats = np.stack([random_case(rng, d)[0] for _ in range(G)])
    K = (rng.standard_normal((N, d)) * 2).astype(np.float32)
    pos = np.sort(rng.choice(500, size=N, replace=False)).astype(np.int32)
    offs = [1, 2, 4, 8, 16]
    full = oracle.raw_scores(stats, K, pos, 600, 1e4, offs)
    trig = oracle.raw_scores(stats, K, pos, 600, 1e4, offs, variant=oracle.VARIANT_TRIG_ONLY)
    norm = oracle.raw_scores(stats, K, pos, 600, 1e4, offs, variant=oracle.VARIANT_NORM_ONLY)
    unw = oracle.raw_scores(stats, K, pos, 600, 1e4, offs, variant=oracle.VARIANT_NORM_UNWEIGHTED)
    np.testing.assert_allclose(trig + norm, full, rtol=1e-12, atol=1e-12)
    for g in range(G):
        for n in range(N):
            assert norm[g, n] == pytest.approx(oracle.s_norm(stats[g], K[n]), rel=1e-13)
            extra = oracle.s_norm0(stats[g], K[n]) - oracle.s_norm(stats[g], K[n])
            assert unw[g, n] - full[g, n] == pytest.approx(extra, rel=1e-9, abs=1e-9)
    norm2 = oracle.raw_scores(stats, K, pos[::-1].copy(), 99999, 1e4, [3], variant=oracle.VARIANT_NORM_ONLY)
    np.testing.assert_allclose(norm2, norm, rtol=1e-13)
    one = oracle.raw_scores(stats, K, pos, 600, 1e4, [7], variant=oracle.VARIANT_TRIG_ONLY)
    for n in range(0, N, 7):
        assert one[1, n] == pytest.approx(oracle.s_trig(stats[1], K[n], 1e4, 600 - int(pos[n]) + 7), rel=1e-12, abs=1e-12)


@pytest.mark.parametrize("pairs", [0, 1])
def test_post_rope_cache(oracle, pairs):
    """P18: a cache that stores R(p_k) k (Section 2.1 Eq. 1).  Un-rotating what the 2x2 matrices produced gives the
    key back; the scores of the rotated cache equal those of the pre-RoPE cache; and S_trig is then the plain dot
    product of the stored key with the centre rotated to the query position (the post-RoPE attention logit)."""
    rng = np.random.default_rng(43 + pairs)
    G, N, d, theta = 2, 25, 64, 1e4
    stats = np.stack([random_case(rng, d)[0] for _ in range(G)])
    K = (rng.standard_normal((N, d)) * 2).astype(np.float64)      # interleaved pre-RoPE keys
    pos = rng.integers(0, 3000, size=N).astype(np.int32)
    Krot = np.stack([rope_rotate(K[n], int(pos[n]), theta) for n in range(N)])

    def store(x):   # interleaved -> the layout under test, rounded to the float32 storage type
        x = np.concatenate([x[..., 0::2], x[..., 1::2]], axis=-1) if pairs else x
        return np.ascontiguousarray(x.astype(np.float32))

    K32, Krot32 = store(K), store(Krot)
    for n in range(0, N, 6):
        back = oracle.unrotate_key(Krot32[n], theta, int(pos[n]), pairs=pairs)
        np.testing.assert_allclose(back, K32[n].astype(np.float64), atol=2e-6)
    offs = [1, 4, 16]
    a = oracle.raw_scores(stats, K32, pos, 3100, theta, offs, pairs=pairs)
    b = oracle.raw_scores(stats, Krot32, pos, 3100, theta, offs, pairs=pairs, rotated=True)
    np.testing.assert_allclose(b, a, rtol=0, atol=1e-4)   # float32 rounding of the stored rotated key
    assert np.abs(a).max() > 1.0
    # un-rotation matters: reading the rotated cache as if it were pre-RoPE gives other scores
    c = oracle.raw_scores(stats, Krot32, pos, 3100, theta, offs, pairs=pairs)
    assert np.abs(c - a).max() > 0.1
    # single offset 0, trig only: the logit of the rotated centre with the stored key
    t = oracle.raw_scores(stats, Krot32, pos, 3100, theta, [0], pairs=pairs, rotated=True, variant=oracle.VARIANT_TRIG_ONLY)
    for n in range(0, N, 5):
        centre = stats[0][:, 0:2].reshape(-1).astype(np.float64)
        stored = Krot32[n].astype(np.float64)
        if pairs:
            stored = np.stack([stored[: d // 2], stored[d // 2:]], axis=-1).reshape(-1)
        brute = float(np.dot(rope_rotate(centre, 3100, theta), stored))
        assert t[0, n] == pytest.approx(brute, rel=1e-9, abs=1e-9)


# ---- concentration and dominant-band diagnostics (Appendix B.5, B.7) -----------------------------

def test_mrl_of_unit_vectors_and_limits(oracle):
    """P19: for unit vectors R is the length of their mean (first equation of Appendix B.5): n equally spaced
    directions give 0, one repeated direction gives 1, two directions at angle a give cos(a/2); scaling every
    sample by a common factor changes nothing."""
    n, F = 12, 4
    q = np.zeros((n, 1, 1, 2 * F), dtype=np.float32)
    ang = 2 * np.pi * np.arange(n) / n
    q[:, 0, 0, 0], q[:, 0, 0, 1] = np.cos(ang), np.sin(ang)                  # band 0: uniform on the circle
    q[:, 0, 0, 2], q[:, 0, 0, 3] = np.cos(0.7), np.sin(0.7)                  # band 1: one direction
    a = 1.1
    half = np.where(np.arange(n) % 2 == 0, 0.0, a)
    q[:, 0, 0, 4], q[:, 0, 0, 5] = np.cos(half), np.sin(half)                # band 2: two directions
    rng = np.random.default_rng(5)
    u = rng.uniform(0, 2 * np.pi, n)
    q[:, 0, 0, 6], q[:, 0, 0, 7] = np.cos(u), np.sin(u)                      # band 3: random unit vectors
    R = oracle.mrl(oracle.centers(q))[0, 0]
    assert R[0] == pytest.approx(0.0, abs=1e-6)
    assert R[1] == pytest.approx(1.0, abs=1e-6)
    assert R[2] == pytest.approx(math.cos(a / 2), abs=1e-6)
    assert R[3] == pytest.approx(abs(np.mean(np.exp(1j * u))), abs=1e-6)
    R5 = oracle.mrl(oracle.centers(q * np.float32(5.0)))[0, 0]
    np.testing.assert_allclose(R5, R, atol=1e-6)
    assert np.all(R <= 1.0 + 1e-6) and np.all(R >= 0.0)
    assert oracle.mrl(np.zeros((1, 3), dtype=np.float32))[0] == 0.0


def test_band_contribution_and_dominant_bands(oracle):
    """P20: C_f = E|q_f| E|k_f| (Appendix B.7) against numpy means of moduli; the dominant bands are a stable
    descending argsort; query head h pairs with KV head h // G."""
    rng = np.random.default_rng(6)
    T, L, Hq, Hkv, d = 50, 2, 4, 2, 16
    q = rng.standard_normal((T, L, Hq, d)).astype(np.float32) * rng.uniform(0.2, 3.0, size=(1, L, Hq, d)).astype(np.float32)
    k = rng.standard_normal((T, L, Hkv, d)).astype(np.float32) * rng.uniform(0.2, 3.0, size=(1, L, Hkv, d)).astype(np.float32)
    qs, ks = oracle.centers(q), oracle.centers(k)
    C, top = oracle.band_contrib(qs, ks, 3)
    qm = np.abs(q[..., 0::2].astype(np.float64) + 1j * q[..., 1::2]).mean(axis=0)
    km = np.abs(k[..., 0::2].astype(np.float64) + 1j * k[..., 1::2]).mean(axis=0)
    for l in range(L):
        for h in range(Hq):
            ref = qm[l, h] * km[l, h // (Hq // Hkv)]
            np.testing.assert_allclose(C[l, h], ref, rtol=1e-6)
            order = np.argsort(-C[l, h], kind="stable")[:3]
            np.testing.assert_array_equal(top[l, h], order)
    # ties: equal contributions keep the lower band first
    flat = np.ones((1, 1, 8, 3), dtype=np.float32)
    _, t = oracle.band_contrib(flat, flat, 4)
    np.testing.assert_array_equal(t[0, 0], [0, 1, 2, 3])
