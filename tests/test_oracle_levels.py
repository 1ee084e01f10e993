"""Pins for the oracle's level-table quantizer (arbitrary level sequences, Euclidean or maximum norm).

Expectations come from the paper, not from the oracle: Def. 1 for an arbitrary sequence 0 = l_0 < ... < l_{s+1} = 1
and the two cases of Sec. 4.1 (generally spaced levels) in exact rational arithmetic; the reduction to the
already pinned routine on the table (0, 2^-s, ..., 1/2, 1); E[h] = r and Var[h] = (l_{j+1} - r)(r - l_j)
(the two-point law of Def. 1); the exponential family of Sec. 4.1 with tau_0 = p^s, tau_j = (1 - p) p^(s-j);
uniform levels (QSGD) and the maximum norm (QSGDinf), and the paper's statement that QSGD's variance is the
largest of the three.
"""
from fractions import Fraction
import math

import numpy as np
import pytest

import oracle
import workloads

F = Fraction
TWO24 = 1 << 24


def frac(x) -> Fraction:
    return F(float(np.float32(x)))


def bin_and_p(r: Fraction, lev):
    """Sec. 4.1: r in [l_j, l_{j+1}) goes up with p = (r - l_j) / tau_j; r >= 1 is the top level."""
    L = [frac(x) for x in lev]
    if r >= 1:
        return len(L) - 1, F(0)
    j = max(t for t in range(len(L) - 1) if L[t] <= r)
    return j, (r - L[j]) / (L[j + 1] - L[j])


TABLES = [("uniform", 3, None), ("uniform", 7, None), ("exp", 4, 0.3), ("exp", 3, 0.7), ("exp", 14, 0.5),
          ("exp", 6, 0.45)]


# ------------------------------------------------------------ the input helper

def test_level_table_helper_matches_the_papers_families():
    for s, p in ((3, 0.5), (5, 0.3), (8, 0.62)):
        lev = workloads.level_table("exp", s, p)
        assert lev[0] == 0.0 and lev[-1] == 1.0 and len(lev) == s + 2
        tau = np.diff(np.array(lev, dtype=np.float64))
        assert tau[0] == pytest.approx(p ** s, rel=1e-6)                       # tau_0 = p^s
        for j in range(1, s + 1):
            assert tau[j] == pytest.approx((1 - p) * p ** (s - j), rel=1e-5)   # tau_j = (1 - p) p^(s - j)
    assert workloads.level_table("exp", 3, 0.5) == [0.0, 0.125, 0.25, 0.5, 1.0]
    lev = workloads.level_table("uniform", 4)
    assert np.allclose(np.diff(lev), 0.2, rtol=1e-6)


# ---------------------------------------------- reduction to the pinned routine

@pytest.mark.parametrize("s", [1, 2, 3, 4, 7, 10, 14])
def test_power_of_two_table_reproduces_the_main_scheme(s):
    """On (0, 2^-s, ..., 1/2, 1) every operation of the table rule is exact, so it must give the levels of the
    routine pinned in test_oracle_quantizer.py, draw for draw."""
    rng = np.random.default_rng(s)
    d, bucket = 30_000, 1000
    v = rng.standard_normal(d) * np.repeat(10.0 ** rng.uniform(-6, 2, size=d // 100), 100)
    v[rng.random(d) < 0.05] = 0.0
    v[::997] *= 50.0
    v = v.astype(np.float32)
    norms = oracle.bucket_norms(v, bucket).astype(np.float32)
    norms[3] = np.float32(norms[3] * 0.5)          # a norm that is too small: ratios above one
    lev = workloads.level_table("exp", s, 0.5)
    want = oracle.quantize(v, bucket, s, 1234 + s, norms)
    got = oracle.quantize_table(v, bucket, lev, 1234 + s, norms)
    np.testing.assert_array_equal(got, want)
    assert (want & 0x7F).max() == s + 1


# ------------------------------------------------ probabilities, draw by draw

@pytest.mark.parametrize("kind,s,p", TABLES[:4])
def test_exhaustive_draws_match_the_probability_of_the_upper_level(kind, s, p):
    """All 2^24 draws for a few coordinates: the number that round up is exactly ceil(p(r) 2^24) for the strict
    test u / 2^24 < p(r), p(r) in rationals."""
    lev = workloads.level_table(kind, s, p if p else 0.5)
    rng = np.random.default_rng(s * 7)
    norm = np.float32(2.7182817)
    for _ in range(4):
        r_target = rng.random() ** 2
        vi = np.float32(r_target * float(norm)) * (1 if rng.random() < 0.5 else -1)
        r = frac(abs(vi)) / frac(norm)
        j, prob = bin_and_p(r, lev)
        hist = oracle.level_histogram_table(vi, norm, lev)
        assert int(hist.sum()) == TWO24
        assert int(hist[j] + hist[j + 1]) == TWO24          # only the two neighbours of r
        want_up = math.ceil(prob * TWO24)
        assert int(hist[j + 1]) == want_up, (r, j, prob)


def near_ties():
    import os
    rows = []
    for line in open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "table_near_ties.txt")):
        if line.startswith("#") or not line.strip():
            continue
        f = [x.strip() for x in line.split("|")]
        rows.append(([float.fromhex(x) for x in f[0].split()], float.fromhex(f[1]), float.fromhex(f[2]), int(f[3]),
                     int(f[4])))
    return rows


def test_near_ties_are_decided_over_the_reals():
    """tests/golden/table_near_ties.txt: draws at which u tau and (|v_i| - l_j ||v||) 2^24 differ by less than one
    rounding of fp64.  The rule of Def. 1 / Sec. 4.1 in rationals says up; a chain of rounded fp64 operations would
    say down (shown here with numpy, to keep the examples honest)."""
    for lev, norm, a, u, up in near_ties():
        r = F(a) / F(norm)
        j, prob = bin_and_p(r, lev)
        assert (F(u, TWO24) < prob) == bool(up)
        assert oracle.quantize_coord_table(a, norm, lev, u) == j + up
        assert oracle.quantize_coord_table(-a, norm, lev, u) == j + up
        # the neighbours of the draw are far from the tie
        assert oracle.quantize_coord_table(a, norm, lev, u - 1) == j + 1
        assert oracle.quantize_coord_table(a, norm, lev, u + 1) == j
        n = np.float64(np.float32(norm))
        lo_n, hi_n = np.float64(np.float32(lev[j])) * n, np.float64(np.float32(lev[j + 1])) * n
        rounded_up = np.float64(u) * (hi_n - lo_n) < (np.float64(a) - lo_n) * np.float64(TWO24)
        assert bool(rounded_up) != bool(up)


@pytest.mark.parametrize("kind,s,p", TABLES)
def test_threshold_draw_of_random_coordinates(kind, s, p):
    """For random coordinates the first draw that does not go up is exactly ceil(p(r) 2^24), p(r) in rationals;
    also for ratios built to make p(r) 2^24 a whole number (an exact tie stays down: the test is strict)."""
    lev = workloads.level_table(kind, s, p if p else 0.5)
    rng = np.random.default_rng(s * 13 + 1)
    cases = []
    for _ in range(300):
        norm = np.float32(10.0 ** rng.uniform(-20, 20))
        cases.append((np.float32(rng.random() ** 3 * float(norm)), norm))
    for _ in range(100):                                  # exact ties: norm a power of two, r = l_j + u tau / 2^24
        j = int(rng.integers(0, s + 1))
        u = int(rng.integers(1, TWO24))
        norm = np.float32(2.0 ** int(rng.integers(-30, 30)))
        r = frac(lev[j]) + F(u, TWO24) * (frac(lev[j + 1]) - frac(lev[j]))
        a = np.float32(float(r) * float(norm))
        cases.append((a, norm))
    ties = 0
    for a, norm in cases:
        if a == 0:
            continue
        r = frac(a) / frac(norm)
        j, prob = bin_and_p(r, lev)
        if j == len(lev) - 1:
            continue
        first_down = math.ceil(prob * TWO24)              # smallest u with u / 2^24 >= p
        ties += (prob * TWO24).denominator == 1
        if first_down > 0:
            assert oracle.quantize_coord_table(a, norm, lev, first_down - 1) == j + 1
        if first_down < TWO24:
            assert oracle.quantize_coord_table(a, norm, lev, first_down) == j
    assert ties >= 5 or kind == "exp"


@pytest.mark.parametrize("kind,s,p", TABLES)
def test_levels_and_boundaries(kind, s, p):
    """A coordinate on a level stays there for every draw; zero stays zero; r >= 1 is the top level; just below
    a level it can only be that level or the one under it."""
    lev = workloads.level_table(kind, s, p if p else 0.5)
    norm = np.float32(1.0)                                   # l_j * 1 is l_j itself
    for j, l in enumerate(lev):
        for u in (0, 1, 99999, TWO24 - 1):
            assert oracle.quantize_coord_table(l, norm, lev, u) == j
            assert oracle.quantize_coord_table(-l, norm, lev, u) == j
    for u in (0, TWO24 - 1):
        assert oracle.quantize_coord_table(1.5, norm, lev, u) == s + 1
        assert oracle.quantize_coord_table(0.0, norm, lev, u) == 0
        assert oracle.quantize_coord_table(3.0, np.float32(0.0), lev, u) == 0
    for j in range(1, s + 2):
        below = np.nextafter(np.float32(lev[j]), np.float32(0.0))
        assert oracle.quantize_coord_table(below, norm, lev, 0) == j             # u = 0 rounds up unless p = 0
        assert oracle.quantize_coord_table(below, norm, lev, TWO24 - 1) == j - 1


# ------------------------------------------------ unbiasedness and variance

@pytest.mark.parametrize("kind,s,p", [("uniform", 3, None), ("exp", 4, 0.3), ("exp", 3, 0.7)])
def test_monte_carlo_mean_and_variance(kind, s, p):
    """E[Q(v)] = v and Var[Q(v_i)] = ||v||^2 (l_{j+1} - r_i)(r_i - l_j) (two-point law of Def. 1), over many
    buckets that hold the same 16-vector under their own keys."""
    lev = workloads.level_table(kind, s, p if p else 0.5)
    L = [frac(x) for x in lev]
    rng = np.random.default_rng(11)
    base = (rng.standard_normal(16) * np.array([1, 1, 1, 1, .3, .3, .3, .3, .05, .05, .05, .05, 3, 0, 1e-3, .7])).astype(np.float32)
    reps = 200_000
    v = np.tile(base, reps)
    nrm = oracle.bucket_norms(base, 16).astype(np.float32)
    norms = np.repeat(nrm, reps)
    q = oracle.quantize_table(v, 16, lev, 4242, norms)
    deq = oracle.dequantize_table(q, 16, lev, norms).reshape(reps, 16)
    mean = deq.mean(axis=0)
    total = 0.0
    for i in range(16):
        r = frac(abs(base[i])) / frac(nrm[0])
        j, _ = bin_and_p(r, lev)
        var = float((L[j + 1] - r) * (r - L[j])) * float(nrm[0]) ** 2 if j <= s else 0.0
        total += var
        assert abs(mean[i] - float(base[i])) <= 5 * math.sqrt(var / reps) + 1e-7 * abs(float(base[i]))
    emp = ((deq - base.astype(np.float64)) ** 2).sum(axis=1).mean()
    assert emp == pytest.approx(total, rel=0.02)


# ------------------------------------------------------- maximum norm (QSGDinf)

def test_maximum_norm_and_its_top_coordinate():
    rng = np.random.default_rng(3)
    d, bucket, s = 10_000, 512, 3
    v = (rng.standard_normal(d) * 10.0 ** rng.uniform(-4, 1, size=d)).astype(np.float32)
    v[1024:1536] = 0.0
    norms = oracle.bucket_norms_linf(v, bucket)
    pad = np.zeros(-d % bucket, dtype=np.float32)
    want = np.abs(np.concatenate([v, pad])).reshape(-1, bucket).max(axis=1).astype(np.float64)
    np.testing.assert_array_equal(norms, want)                 # a maximum has no rounding
    lev = workloads.level_table("uniform", s)
    q = oracle.quantize_table(v, bucket, lev, 9, norms.astype(np.float32))
    for b in range(norms.size):
        sl = slice(b * bucket, min(d, (b + 1) * bucket))
        if norms[b] == 0:
            assert not q[sl].any()
            continue
        top = np.argmax(np.abs(v[sl]))
        assert (q[sl][top] & 0x7F) == s + 1                    # r = 1 exactly: the top level, whatever the draw
        assert bool(q[sl][top] & 0x80) == bool(v[sl][top] < 0)


def expected_variance(v, norms, bucket, lev):
    """sum_i ||v||^2 (l_{j+1} - r_i)(r_i - l_j) in fp64 (the exact law, evaluated densely)."""
    L = np.array(lev, dtype=np.float64)
    n = np.repeat(np.asarray(norms, dtype=np.float64), bucket)[: v.size]
    r = np.minimum(np.abs(v.astype(np.float64)) / n, 1.0)
    j = np.clip(np.searchsorted(L, r, side="right") - 1, 0, len(L) - 2)
    return float((n * n * (L[j + 1] - r) * (r - L[j])).sum())


def test_variance_ordering_of_the_three_schemes_on_gaussian_buckets():
    """Sec. 1 / Sec. 5: with the same number of levels QSGD (uniform levels, Euclidean norm) has by far the
    largest variance; nonuniform levels (Euclidean norm) and QSGDinf (uniform levels, maximum norm) are both
    below it.  The oracle's empirical variance agrees with the closed form for each scheme."""
    rng = np.random.default_rng(5)
    d, bucket, s = 8 * 8192, 8192, 3
    v = rng.standard_normal(d).astype(np.float32)
    l2 = oracle.bucket_norms(v, bucket).astype(np.float32)
    linf = oracle.bucket_norms_linf(v, bucket).astype(np.float32)
    schemes = {"qsgd": (workloads.level_table("uniform", s), l2),
               "nuqsgd": (workloads.level_table("exp", s, 0.5), l2),
               "qsgdinf": (workloads.level_table("uniform", s), linf)}
    closed, empirical = {}, {}
    for name, (lev, norms) in schemes.items():
        closed[name] = expected_variance(v, norms, bucket, lev)
        acc = 0.0
        for seed in range(20):
            q = oracle.quantize_table(v, bucket, lev, seed, norms)
            acc += float(((oracle.dequantize_table(q, bucket, lev, norms) - v) ** 2).sum())
        empirical[name] = acc / 20
        assert empirical[name] == pytest.approx(closed[name], rel=0.03)
    # the ordering only (the paper prints no number for these vectors); here QSGD is about twice the nonuniform
    # scheme and several times QSGDinf
    assert closed["qsgd"] > 1.5 * closed["nuqsgd"]
    assert closed["qsgd"] > 1.5 * closed["qsgdinf"]


# ------------------------------------------------------------ decode + average

def test_decode_average_with_a_table_is_the_dense_sum():
    rng = np.random.default_rng(8)
    d, bucket, s, K = 7_000, 1000, 4, 3
    lev = workloads.level_table("exp", s, 0.35)
    norms_list, bo_list, w_list, dense = [], [], [], np.zeros(d)
    for k in range(K):
        q = np.where(rng.random(d) < 0.2, rng.integers(1, s + 2, d), 0).astype(np.uint8)
        q |= np.where((q > 0) & (rng.random(d) < 0.5), 0x80, 0).astype(np.uint8)
        norms = (10.0 ** rng.uniform(-2, 2, size=oracle.num_buckets(d, bucket))).astype(np.float32)
        bo, words, _ = oracle.encode(q, bucket, s)
        norms_list.append(norms); bo_list.append(bo); w_list.append(words)
        lv = np.array(lev, dtype=np.float64)[q & 0x7F]
        dense += np.repeat(norms.astype(np.float64), bucket)[:d] * np.where(q & 0x80, -1.0, 1.0) * lv
    out = oracle.decode_average_table(norms_list, bo_list, w_list, d, bucket, lev, 1.0 / K)
    np.testing.assert_allclose(out, dense / K, rtol=1e-15, atol=0)
    prior = rng.standard_normal(d)
    out2 = oracle.decode_average_table(norms_list, bo_list, w_list, d, bucket, lev, 0.5, prior=prior)
    np.testing.assert_allclose(out2, prior + 0.5 * dense, rtol=1e-14, atol=1e-300)
