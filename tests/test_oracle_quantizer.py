"""Pins for the oracle's norms, random draws and quantizer against what the paper fixes.

Nothing here compares the oracle with itself: expectations are the paper's level
set (Sec. 3.1), its rounding probabilities (App. B eqs. h_case1/h_case2) in exact
rational arithmetic, unbiasedness and the variance identities (Thm 1, Lemma 2,
eq. var_reform), the sparsity lemma (Lemma 4) and special vectors whose
quantization is known in closed form.
"""
from fractions import Fraction
import math

import numpy as np
import pytest

import oracle

F = Fraction
TWO24 = 1 << 24


def paper_levels(s):
    # Sec. 3.1: (0, 1/2^s, ..., 2^(s-1)/2^s, 1)
    return [F(0)] + [F(2 ** k, 2 ** s) for k in range(0, s + 1)]


def paper_bin_and_p(r: Fraction, s: int):
    """App. B: bin and probability of the upper level, exact.
    case 1: r in [0, 2^-s]: p1 = 2^s r (levels 0 and 2^-s)
    case 2: r in [2^(j-s), 2^(j+1-s)], j = 0..s-1: p2 = 2^(s-j) r - 1."""
    if r < F(1, 2 ** s):
        return 0, F(2 ** s) * r
    for j in range(s):
        if F(2 ** j, 2 ** s) <= r < F(2 ** (j + 1), 2 ** s):
            return j + 1, F(2 ** (s - j)) * r - 1
    return s + 1, F(0)          # r >= 1


def exact_ratio(a: float, n: float) -> Fraction:
    return F(float(np.float32(abs(a)))) / F(float(np.float32(n)))


# ------------------------------------------------------------------ level set

def test_level_set_s3_is_the_papers():
    assert oracle.levels(3) == [F(0), F(1, 8), F(1, 4), F(1, 2), F(1)]


@pytest.mark.parametrize("s", range(1, 15))
def test_level_set_all_s(s):
    assert oracle.levels(s) == paper_levels(s)
    # a coordinate sitting exactly on a level is reproduced for every draw
    norm = 3.0
    for j, l in enumerate(paper_levels(s)):
        v = float(l) * norm
        for u in (0, 1, 12345, TWO24 - 1):
            assert oracle.quantize_coord(v, norm, s, u) == j
            assert oracle.quantize_coord(-v, norm, s, u) == j


def test_figure1_example():
    # Fig. 1: s = 3, a point between 1/8 and 1/4, nearer 1/4: goes to one of the two,
    # more often to 1/4.
    hist = oracle.level_histogram(0.21, 1.0, 3)
    assert hist[1] + hist[2] == TWO24 and hist[2] > hist[1] > 0
    assert hist.sum() == TWO24


# ------------------------------------------------------- rounding probabilities

CASES = [
    # (v_i, norm, s)
    (0.001, 1.0, 3), (0.1, 1.0, 3), (0.125, 1.0, 3), (0.2, 1.0, 3), (0.3, 1.0, 3), (0.75, 1.0, 3), (0.999, 1.0, 3),
    (-0.4, 1.7, 1), (0.013, 0.11, 4), (5e-4, 0.9, 7), (0.0123, 1.3, 7), (-3.3e-5, 2.2e-3, 14),
    (1e-30, 3e-28, 3), (1e-41, 1e-38, 2),      # tiny norm, subnormal coordinate
    (2.5e30, 7e30, 5),
]


@pytest.mark.parametrize("vi,norm,s", CASES)
def test_exhaustive_draws_match_paper_probability(vi, norm, s):
    """All 2^24 draws: exactly ceil(p * 2^24) of them round up, p from App. B."""
    r = exact_ratio(vi, norm)
    j_lo, p = paper_bin_and_p(r, s)
    hist = oracle.level_histogram(vi, norm, s)
    assert hist.sum() == TWO24
    ups = math.ceil(p * TWO24)
    if j_lo == s + 1:
        assert hist[s + 1] == TWO24
        return
    assert int(hist[j_lo + 1]) == ups
    assert int(hist[j_lo]) == TWO24 - ups
    # E[h] = r up to the 2^-24 granularity of the draw (Thm 1: unbiased)
    L = paper_levels(s)
    mean = (L[j_lo] * int(hist[j_lo]) + L[j_lo + 1] * int(hist[j_lo + 1])) / TWO24
    assert 0 <= mean - r <= (L[j_lo + 1] - L[j_lo]) / TWO24


def test_ratio_at_or_above_one_maps_to_top_level():
    for s in (1, 3, 7):
        for u in (0, 77, TWO24 - 1):
            assert oracle.quantize_coord(1.0, 1.0, s, u) == s + 1
            assert oracle.quantize_coord(1.0000001, 1.0, s, u) == s + 1


def test_zero_maps_to_zero():
    # App. B: Q_s(0) = 0
    for u in (0, 1, TWO24 - 1):
        assert oracle.quantize_coord(0.0, 1.0, 3, u) == 0
        assert oracle.quantize_coord(-0.0, 1.0, 3, u) == 0
        assert oracle.quantize_coord(0.0, 0.0, 3, u) == 0
    q = oracle.quantize(np.zeros(40, np.float32), 16, 3, 5, np.zeros(3, np.float32))
    assert not q.any()


# -------------------------------------------- four-element vectors, brute force

@pytest.mark.parametrize("vec,s", [
    ([0.3, -0.1, 0.05, 0.9], 3),
    ([1.0, 1.0, 1.0, 1.0], 2),          # r = 1/2 on a level
    ([0.02, 0.5, -0.49, 0.01], 1),
    ([1e-3, -2e-3, 4e-3, 1.0], 7),
])
def test_four_vector_law_mean_and_variance(vec, s):
    """Per-coordinate outcome counts over all draws give the exact law of Q_s(v);
    its mean is v (Thm 1) and E||Q-v||^2 equals Lemma 2's closed form, both up to
    the 2^-24 draw granularity.  Coordinates are independent (Def. 1), so the joint
    law over the 16 outcome pairs is the product and the sums below are exact."""
    v = np.array(vec, dtype=np.float32)
    norm = np.float32(oracle.bucket_norms(v, 4)[0])
    L = paper_levels(s)
    total_var = F(0)
    closed_var = F(0)
    for vi in v:
        r = exact_ratio(vi, norm)
        hist = oracle.level_histogram(float(vi), float(norm), s)
        probs = {j: F(int(c), TWO24) for j, c in enumerate(hist) if c}
        assert len(probs) <= 2 and sum(probs.values()) == 1
        mean = sum(L[j] * p for j, p in probs.items())
        j_lo, p = paper_bin_and_p(r, s)
        tau = L[min(j_lo + 1, s + 1)] - L[min(j_lo, s + 1)]
        assert abs(mean - min(r, F(1))) <= tau / TWO24
        total_var += sum((L[j] - r) ** 2 * pr for j, pr in probs.items())
        if j_lo <= s:
            closed_var += (L[j_lo + 1] - r) * (r - L[j_lo])     # eq. var_norm_coor
    assert abs(total_var - closed_var) <= F(4, TWO24)
    # Thm 1 bound (in units of ||v||^2)
    d = 4
    eps = F(1, 8) + F(d, 2 ** (2 * s + 2)) if d < 2 ** (2 * s + 1) else F(math.sqrt(d)) / 2 ** s - F(7, 8)
    assert total_var <= eps + F(1, 10 ** 9)


def test_constant_vector_special_cases():
    # Thm 5 / Thm 4's proof: v = c*[1..1], r_i = 1/sqrt(d).
    # d = 4: r = 1/2, d = 16: r = 1/4 -> on a level, Q(v) = v for every seed.
    for d, s in ((4, 1), (4, 3), (16, 2), (16, 5)):
        v = np.full(d, 0.75, np.float32)
        nrm = oracle.bucket_norms(v, d).astype(np.float32)
        for seed in range(20):
            q = oracle.quantize(v, d, s, seed, nrm)
            np.testing.assert_array_equal(oracle.dequantize(q, d, s, nrm), v.astype(np.float64))
    # d = 9, s >= 2: r = 1/3 in [1/4, 1/2]; variance = 9 (1/2-1/3)(1/3-1/4) = 1/8 of ||v||^2
    for s in (2, 3, 6):
        hist = oracle.level_histogram(1.0, 3.0, s)
        L = paper_levels(s)
        r = F(1, 3)
        var = sum((L[j] - r) ** 2 * F(int(c), TWO24) for j, c in enumerate(hist) if c) * 9
        assert abs(var - F(1, 8)) <= F(1, 2 ** 22)


def test_single_spike_is_reproduced():
    v = np.zeros(64, np.float32)
    v[17] = -3.25
    nrm = oracle.bucket_norms(v, 64).astype(np.float32)
    for s in (1, 3, 9):
        q = oracle.quantize(v, 64, s, 11, nrm)
        np.testing.assert_array_equal(oracle.dequantize(q, 64, s, nrm), v.astype(np.float64))
        assert q[17] == (0x80 | (s + 1))


# --------------------------------------------------------------------- norms

def test_norms_against_numpy_and_closed_forms():
    rng = np.random.default_rng(0)
    v = rng.standard_normal(1000).astype(np.float32)
    got = oracle.bucket_norms(v, 128)
    assert got.shape == (8,)
    for b in range(8):
        seg = v[b * 128:(b + 1) * 128].astype(np.float64)
        assert got[b] == pytest.approx(np.linalg.norm(seg), rel=1e-14)
    assert oracle.bucket_norms(np.array([3, 4], np.float32), 2)[0] == 5.0
    assert oracle.bucket_norms(np.array([3, 4, 12], np.float32), 2).tolist() == [5.0, 12.0]


# ------------------------------------------------------------ the counter RNG

def chi2(counts, expected):
    return float(((counts - expected) ** 2 / expected).sum())


def test_rng_uniformity_and_independence():
    """The paper only requires independent uniform draws (Def. 1); check the generator
    the format fixes: byte histograms, lag-1 pairs inside a bucket, same index across
    buckets and across seeds.  255 d.o.f.: chi2 > 400 has probability < 1e-8."""
    d, bucket = 1 << 21, 8192
    u = oracle.rng_fill(7, d, bucket)
    assert u.max() < TWO24
    for shift in (16, 8, 0):
        c = np.bincount((u >> shift) & 0xFF, minlength=256)
        assert chi2(c, d / 256) < 400
    pair = ((u[:-1] >> 20) << 4) | (u[1:] >> 20)
    assert chi2(np.bincount(pair, minlength=256), (d - 1) / 256) < 400
    ub = u.reshape(-1, bucket)
    pair = ((ub[:-1, :64] >> 20) << 4) | (ub[1:, :64] >> 20)
    assert chi2(np.bincount(pair.ravel(), minlength=256), pair.size / 256) < 400
    u2 = oracle.rng_fill(8, d, bucket)
    pair = ((u >> 20) << 4) | (u2 >> 20)
    assert chi2(np.bincount(pair, minlength=256), d / 256) < 400
    assert abs(np.corrcoef(u.astype(np.float64), u2.astype(np.float64))[0, 1]) < 5e-3
    # small buckets: many keys, few indices each
    u3 = oracle.rng_fill(123456789012345, 1 << 20, 16)
    c = np.bincount(u3 >> 16, minlength=256)
    assert chi2(c, u3.size / 256) < 400


def test_rng_streams_differ_between_buckets_and_seeds():
    a = oracle.rng_fill(1, 4096, 512).reshape(8, 512)
    assert len({row.tobytes() for row in a}) == 8
    b = oracle.rng_fill(2, 4096, 512).reshape(8, 512)
    assert (a != b).mean() > 0.99


# ------------------------------------------- Monte Carlo over the counter RNG

@pytest.mark.parametrize("s", [1, 3, 4])
def test_monte_carlo_unbiased_with_counter_rng(s):
    """E[Q_s(v)] = v (Thm 1): average over many buckets holding the same 16-vector
    (each bucket has its own key) stays within 5 standard errors, the per-coordinate
    variance taken from eq. var_norm_coor."""
    rng = np.random.default_rng(3)
    base = (rng.standard_normal(16) * np.array([1, 1, 1, 1, .1, .1, .1, .1, .01, .01, .01, .01, 3, 0, 1e-4, .5])).astype(np.float32)
    reps = 200_000
    v = np.tile(base, reps)
    nrm1 = oracle.bucket_norms(base, 16).astype(np.float32)
    norms = np.repeat(nrm1, reps)
    q = oracle.quantize(v, 16, s, 99, norms)
    deq = oracle.dequantize(q, 16, s, norms).reshape(reps, 16)
    mean = deq.mean(axis=0)
    L = paper_levels(s)
    for i in range(16):
        r = exact_ratio(base[i], nrm1[0])
        j, _ = paper_bin_and_p(r, s)
        var = float((L[j + 1] - r) * (r - L[j])) * float(nrm1[0]) ** 2 if j <= s else 0.0
        se = math.sqrt(var / reps)
        assert abs(mean[i] - float(base[i])) <= 5 * se + 1e-7 * abs(float(base[i]))
    # empirical total variance against Lemma 2
    emp = ((deq - base.astype(np.float64)) ** 2).sum(axis=1).mean()
    closed = 0.0
    for i in range(16):
        r = exact_ratio(base[i], nrm1[0])
        j, _ = paper_bin_and_p(r, s)
        if j <= s:
            closed += float((L[j + 1] - r) * (r - L[j])) * float(nrm1[0]) ** 2
    assert emp == pytest.approx(closed, rel=0.02)


@pytest.mark.parametrize("d,s", [(8192, 3), (512, 3), (8192, 4), (4096, 7)])
def test_sparsity_lemma_and_variance_bound_on_gaussian_buckets(d, s):
    """Lemma 4: E||Q||_0 = (d - d_0) + sum_{S_0} 2^s r_i <= 2^(2s) + 2^s sqrt(d);
    Thm 1: E||Q - v||^2 <= eps_Q ||v||^2.  Averages over 300 seeds."""
    rng = np.random.default_rng(d + s)
    v = rng.standard_normal(d).astype(np.float32)
    nrm = oracle.bucket_norms(v, d).astype(np.float32)
    r = np.abs(v.astype(np.float64)) / float(nrm[0])
    in0 = r < 2.0 ** -s
    expect_nnz = (~in0).sum() + (2.0 ** s * r[in0]).sum()
    assert (~in0).sum() <= 2 ** (2 * s)
    assert expect_nnz <= 2 ** (2 * s) + 2 ** s * math.sqrt(d)
    nnz, err = [], []
    for seed in range(300):
        q = oracle.quantize(v, d, s, seed, nrm)
        nnz.append(np.count_nonzero(q & 0x7F))
        err.append(((oracle.dequantize(q, d, s, nrm) - v) ** 2).sum())
    assert np.mean(nnz) == pytest.approx(expect_nnz, rel=0.01)
    # exact variance, eq. var_reform
    lv = np.array([float(x) for x in paper_levels(s)])
    j = np.searchsorted(lv, r, side="right") - 1
    j = np.minimum(j, s)
    closed = ((lv[j + 1] - r) * (r - lv[j])).sum() * float(nrm[0]) ** 2
    assert np.mean(err) == pytest.approx(closed, rel=0.02)
    eps = (1 / 8 + 2.0 ** (-2 * s - 2) * d) if d < 2 ** (2 * s + 1) else (2.0 ** -s * math.sqrt(d) - 7 / 8)
    assert closed <= eps * float(nrm[0]) ** 2


def test_sign_and_byte_layout():
    v = np.array([0.5, -0.5, 0.0, -0.0, 1e-9, -1.0], np.float32)
    nrm = np.array([1.0], np.float32)
    u = np.array([0, 0, 0, 0, TWO24 - 1, 5], np.uint32)
    q = oracle.quantize_given_u(v, 6, 3, nrm, u)
    # 0.5 is level index 3 for s = 3; zeros carry no sign; a draw of 2^24-1 keeps 1e-9 at 0
    assert q.tolist() == [3, 0x83, 0, 0, 0, 0x84]
