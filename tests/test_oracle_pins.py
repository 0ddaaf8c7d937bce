"""Pins for the CPU oracle: every check compares the oracle with something that is not the oracle --
a brute-force definition on tiny inputs, a closed form or identity from the paper, an exact rational
computation, a library routine with a different algorithm, or published known-answer vectors.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import mlmc as O
from oracle.philox import philox4x32_10, level_uniform
import mlmc_workloads as W

HERE = os.path.dirname(os.path.abspath(__file__))


# ----------------------------------------------------------------------------- helpers (independent)
def brute_rank(g):
    """rank(j) = #{i: |g_i| > |g_j|} + #{i < j: |g_i| == |g_j|}  -- O(d^2), float compares only."""
    a = [abs(float(x)) for x in g]
    d = len(a)
    return [sum(1 for i in range(d) if a[i] > a[j]) + sum(1 for i in range(j) if a[i] == a[j]) for j in range(d)]


def tiny_rows():
    rng = np.random.default_rng(7)
    rows = []
    rows.append(rng.standard_normal(64).astype(np.float32))
    rows.append(np.array([1, -1, 1, -1, 0.5, -0.0, 0.0, 2, 2, -2, 1e-40, -1e-40, 3e-41, 0, 7, -7], dtype=np.float32))
    rows.append(np.full(33, -0.25, dtype=np.float32))
    rows.append(np.zeros(17, dtype=np.float32))
    rows.append((rng.integers(-2, 3, size=50)).astype(np.float32))
    rows.append(rng.standard_normal(37).astype(np.float32) * np.float32(1e-3))
    return rows


# ----------------------------------------------------------------------------- Philox
def test_philox_known_answers():
    n = 0
    with open(os.path.join(HERE, "golden", "philox4x32_10_kat.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            w = [int(x, 16) for x in line.split()]
            assert list(philox4x32_10(w[0:4], w[4:6])) == w[6:10]
            n += 1
    assert n == 3


def test_philox_counter_layout():
    # key = (seed_lo, seed_hi); counter = (step_lo, step_hi, worker, 0); word 0 is used
    seed, step, worker = 0x299f31d0a4093822, 0x85a308d3243f6a88, 0x13198a2e
    assert level_uniform(seed, step, worker) == philox4x32_10(
        (0x243f6a88, 0x85a308d3, 0x13198a2e, 0), (0xa4093822, 0x299f31d0))[0]
    # uniformity of the word actually used: mean of 20000 draws within 5 sigma of 1/2
    xs = [level_uniform(1, s, 0) / 2 ** 32 for s in range(20000)]
    assert abs(sum(xs) / len(xs) - 0.5) < 5 * math.sqrt(1 / 12 / len(xs))


# ----------------------------------------------------------------------------- ordering / Top-k
@pytest.mark.parametrize("row_id", range(6))
def test_order_matches_bruteforce_rank(row_id):
    g = tiny_rows()[row_id]
    order = O.magnitude_order(g)
    rank = brute_rank(g)
    assert [rank[j] for j in order] == list(range(len(g)))
    for k in (0, 1, 2, len(g) // 2, len(g)):
        want = np.array([g[j] if rank[j] < k else 0 for j in range(len(g))], dtype=np.float32)
        assert np.array_equal(O.topk_dense(g, k).view(np.uint32), want.view(np.uint32))


def test_bf16_rows_upcast_exactly():
    rng = np.random.default_rng(3)
    x = rng.standard_normal(64).astype(np.float32)
    b = W.f32_to_bf16_bits(x)
    up = O.as_f32(b)
    # bf16 RNE: error at most half a bf16 ulp (2^-9 relative), and the upcast has zero low mantissa bits
    assert np.all(np.abs(up - x) <= np.abs(x) * 2.0 ** -8)
    assert np.all((up.view(np.uint32) & 0xFFFF) == 0)
    rank = brute_rank(up)
    assert [rank[j] for j in O.magnitude_order(up)] == list(range(64))


# ----------------------------------------------------------------------------- telescoping / unbiasedness
@pytest.mark.parametrize("row_id", range(6))
def test_telescoping_reproduces_top_level(row_id):
    """App. A: g^0 + sum_l (g^l - g^{l-1}) = g^L.  With every weight 1 the bands tile C_L(g) exactly."""
    g = tiny_rows()[row_id]
    d = len(g)
    ladder = sorted(set([0, 1, 2, d // 4, d // 2, d - 1])) if row_id % 2 else sorted(set([2, 3, d // 3, d - 2]))
    ladder = [k for k in ladder if 0 <= k <= d]
    L = len(ladder) - 1
    ones = [1.0] * L   # not a distribution: forces weight 1 on every band
    total = np.zeros(d, dtype=np.float32)
    seen = np.zeros(d, dtype=int)
    for l in range(1, L + 1):
        m = O.compress_topk_row(g, ladder, ones, 0, 0, 0, force_level=l)
        dense = O.sparse_to_dense(m["idx"], m["val"], d)
        base = O.topk_dense(g, ladder[0])
        total += dense - base
        seen[m["idx"]] += 1
        assert np.all(np.diff(m["idx"].astype(np.int64)) > 0)
        assert len(m["idx"]) == ladder[0] + ladder[l] - ladder[l - 1]
    total += O.topk_dense(g, ladder[0])
    assert np.array_equal(total, O.topk_dense(g, ladder[L]))


@pytest.mark.parametrize("adaptive", [False, True])
def test_exact_expectation_is_top_level(adaptive):
    """Lemma 3.2: sum_l p_l * g~(l) = C_L(g), checked in exact rational arithmetic up to the fp32 rounding
    of the weight and product (relative 2^-22 per entry)."""
    g = tiny_rows()[0]
    d = len(g)
    ladder = [4, 8, 16, 32, 64]
    L = 4
    p = None if adaptive else O.geometric_p(L)
    exp = [Fraction(0)] * d
    for l in range(1, L + 1):
        m = O.compress_topk_row(g, ladder, p, 0, 0, 0, force_level=l)
        pl = Fraction(m["p"][l - 1])
        for j, v in zip(m["idx"], m["val"]):
            exp[j] += pl * Fraction(float(v))
    assert abs(sum(Fraction(x) for x in (m["p"])) - 1) < Fraction(1, 10 ** 12)
    for j in range(d):
        want = Fraction(float(g[j]))
        assert abs(exp[j] - want) <= abs(want) * Fraction(1, 2 ** 21)


def test_importance_sampling_special_case():
    """Sec. 3.2: with the unit ladder k_l = l the message is the single rank-l entry scaled by 1/p_l."""
    g = tiny_rows()[5]
    d = len(g)
    ladder = list(range(d + 1))
    rank = brute_rank(g)
    by_rank = {r: j for j, r in enumerate(rank)}
    norms, _ = O.level_norms_row(g, ladder)
    # Delta_l is the magnitude of the rank-(l-1) entry
    for l in range(1, d + 1):
        assert norms[l - 1] == abs(float(g[by_rank[l - 1]]))
    for step in range(50):
        m = O.compress_topk_row(g, ladder, None, 11, step, 2)
        l = m["level"]
        assert list(m["idx"]) == [by_rank[l - 1]]
        pl = norms[l - 1] / math.fsum(norms)
        assert m["val"][0] == np.float32(g[by_rank[l - 1]]) * np.float32(1.0 / m["p"][l - 1])
        assert abs(m["p"][l - 1] - pl) < 1e-15


def test_monte_carlo_unbiased_tiny_case():
    """Lemma 3.2 by Monte Carlo over 10^5 frozen seeds on the tiny workload's ladder (reduced d): the
    level frequencies match p within 3 sigma (binomial), which for rank bands is the whole statement
    because g~ restricted to band l equals g * 1[level = l] / p_l."""
    w = W.scaled(W.WORKLOADS["tiny_topk"], d=4096, M=1)
    L = w.L
    p = O.geometric_p(L)
    N = 100_000
    T = O.cdf_thresholds(p)
    counts = [0] * (L + 1)
    for seed in range(N):
        x = level_uniform(seed, 0, 0)
        l = next(i for i, t in enumerate(T, start=1) if x < t)
        counts[l] += 1
    for l in range(1, L + 1):
        sd = math.sqrt(p[l - 1] * (1 - p[l - 1]) / N)
        assert abs(counts[l] / N - p[l - 1]) <= 3 * sd + 1e-12, (l, counts[l] / N, p[l - 1])
    # and the function the oracle actually calls agrees with that inverse-CDF on a few seeds
    for seed in range(200):
        x = level_uniform(seed, 0, 0)
        assert O.draw_level(p, seed, 0, 0) == next(i for i, t in enumerate(T, start=1) if x < t)


def test_monte_carlo_unbiased_per_coordinate_small():
    """Per-coordinate 3-sigma check on d = 32 with frozen seeds (Lemma 3.2)."""
    rng = np.random.default_rng(5)
    g = rng.standard_normal(32).astype(np.float32)
    ladder = [2, 4, 8, 16, 32]
    L = 4
    p = O.geometric_p(L)
    N = 20000
    s1 = np.zeros(32)
    s2 = np.zeros(32)
    for seed in range(N):
        m = O.compress_topk_row(g, ladder, p, seed, 3, 1)
        dense = O.sparse_to_dense(m["idx"], m["val"], 32).astype(np.float64)
        s1 += dense
        s2 += dense * dense
    mean = s1 / N
    var = np.maximum(s2 / N - mean ** 2, 0)
    # 3 sigma as stated; coordinates of one band share their error (g~ on band l is g * 1[level = l] / p_l), so the
    # 32 checks are L = 4 distinct ones and the frozen seeds 0..N-1 stay near 1.1 sigma
    assert np.all(np.abs(mean - g) <= 3.0 * np.sqrt(var / N) + 1e-6 * np.abs(g))


# ----------------------------------------------------------------------------- probabilities
def test_geometric_p_is_lemma_3_3_form():
    for L in (1, 5, 10, 63):
        p = O.geometric_p(L)
        assert abs(math.fsum(p) - 1.0) < 1e-15
        for l in range(1, L):
            assert p[l - 1] == 2 * p[l]
        assert Fraction(p[0]) == Fraction(Fraction(1, 2) / (1 - Fraction(1, 2 ** L))) or \
            abs(Fraction(p[0]) - Fraction(1, 2) / (1 - Fraction(1, 2 ** L))) < Fraction(1, 2 ** 53)


def test_cdf_thresholds_integer_inverse_cdf():
    p = [0.5, 0.25, 0.25]
    assert O.cdf_thresholds(p) == [1 << 31, 3 << 30, 1 << 32]
    p = [0.0, 1.0]
    assert O.cdf_thresholds(p) == [0, 1 << 32]       # a zero-probability level is never drawn
    assert all(O.draw_level(p, s, 0, 0) == 2 for s in range(100))
    assert O.adaptive_p([0.0, 0.0, 0.0, 0.0]) == [0.25] * 4


# ----------------------------------------------------------------------------- norms
def test_exact_sumsq_against_rationals_and_fsum():
    rng = np.random.default_rng(11)
    for trial in range(5):
        g = (rng.standard_normal(300) * 10.0 ** rng.uniform(-30, 30, size=300)).astype(np.float32)
        g[::17] = np.float32(1e-42)  # denormals
        exact = sum(Fraction(float(x)) ** 2 for x in g)
        assert Fraction(O.exact_sumsq(g), 2 ** 298) == exact
    # where no square underflows in fp64, fsum of the (exact) fp64 squares is the correctly rounded sum
    g = rng.standard_normal(5000).astype(np.float32)
    assert O.units_to_f64(O.exact_sumsq(g)) == math.fsum((g.astype(np.float64) ** 2).tolist())


def test_level_norms_pythagoras_and_fsum():
    """App. D: Delta_l^2 = ||g^l||^2 - ||g^{l-1}||^2, hence S_0 + sum_l S_l = ||C_L(g)||^2 (exactly, in units)."""
    w = W.scaled(W.WORKLOADS["resnet50_adaptive_topk"], d=20000, M=2)
    G = W.generate(w)
    for i in range(2):
        norms, units = O.level_norms_row(G[i], w.ladder)
        assert sum(units) == O.exact_sumsq(G[i])
        order = sorted(range(w.d), key=lambda j: (-abs(float(G[i][j])), j))
        for l in (1, w.L // 2, w.L):
            band = order[w.ladder[l - 1]:w.ladder[l]]
            want = math.sqrt(math.fsum(float(G[i][j]) ** 2 for j in band))
            assert norms[l - 1] == want


def test_level_norms_exponential_decay_closed_form():
    """Assumption 3.5 / App. E: |v(j)| = |v(0)| e^{-r j / 2} gives
    Delta_l^2 = |v(0)|^2 e^{-r s (l-1)} (1 - e^{-r s}) / (1 - e^{-r}) for the ladder k_l = s l."""
    d, s, r, v0 = 4096, 64, 0.01, 3.0
    j = np.arange(d)
    mags = (v0 * np.exp(-0.5 * r * j)).astype(np.float32)
    rng = np.random.default_rng(2)
    perm = rng.permutation(d)
    g = np.empty(d, dtype=np.float32)
    g[perm] = mags * rng.choice(np.array([-1.0, 1.0], dtype=np.float32), size=d)
    ladder = [s * l for l in range(d // s + 1)]
    norms, _ = O.level_norms_row(g, ladder)
    for l in (1, 2, 10, d // s):
        closed = v0 ** 2 * math.exp(-r * s * (l - 1)) * (1 - math.exp(-r * s)) / (1 - math.exp(-r))
        assert abs(norms[l - 1] ** 2 - closed) <= 1e-6 * closed   # fp32 rounding of the inputs
    # App. D: with the optimal p the second moment is (sum Delta)^2
    p = O.adaptive_p(norms)
    second = 0.0
    for l in (1, 3, 17, d // s):
        m = O.compress_topk_row(g, ladder, None, 0, 0, 0, force_level=l)
        n2 = float(np.sum(m["val"].astype(np.float64) ** 2))
        assert abs(n2 - norms[l - 1] ** 2 / p[l - 1] ** 2) <= 1e-5 * n2
    assert abs(sum(x * x / q for x, q in zip(norms, p)) - math.fsum(norms) ** 2) <= 1e-9 * math.fsum(norms) ** 2


def test_stopk_thousands_of_levels():
    """s-segmented Top-k (Sec. 2.2, Sec. 3.2) with thousands of levels: the ladder, Pythagoras over all bands (App. D),
    the exponential-decay closed form (Assumption 3.5 / App. E) at L = 2048, and Lemma 3.4's s-Top-k form
    p_l = sqrt(alpha_l - alpha_{l-1}) / sum_l' sqrt(alpha_l' - alpha_{l'-1}) with alpha_l = ||C^l(v)||^2 / ||v||^2."""
    assert O.stopk_ladder(10, 3) == [0, 3, 6, 9, 10] and O.stopk_ladder(9, 3) == [0, 3, 6, 9] and O.stopk_ladder(5, 8) == [0, 5]
    d, s, r, v0 = 2048 * 16 + 5, 16, 0.0007, 2.0
    ladder = O.stopk_ladder(d, s)
    L = len(ladder) - 1
    assert L == 2049 and ladder[-1] == d and ladder[-2] == 2048 * 16
    mags = (v0 * np.exp(-0.5 * r * np.arange(d))).astype(np.float32)
    rng = np.random.default_rng(12)
    g = np.empty(d, dtype=np.float32)
    g[rng.permutation(d)] = mags * rng.choice(np.array([-1.0, 1.0], dtype=np.float32), size=d)
    norms, units = O.level_norms_row(g, ladder)
    assert units[0] == 0 and sum(units) == O.exact_sumsq(g)                       # Pythagoras, exactly
    for l in (1, 2, 100, 1024, 2048):
        closed = v0 ** 2 * math.exp(-r * s * (l - 1)) * (1 - math.exp(-r * s)) / (1 - math.exp(-r))
        assert abs(norms[l - 1] ** 2 - closed) <= 2e-6 * closed
    # the residual of level l is the l-th segment of the sorted vector: s entries (the last segment: 5)
    for l in (1, 777, L):
        m = O.compress_topk_row(g, ladder, None, 3, 4, 0, force_level=l)
        want = np.sort(np.argsort(-np.abs(g.astype(np.float64)), kind="stable")[s * (l - 1):s * l])
        assert np.array_equal(m["idx"], want.astype(np.uint32)) and len(m["idx"]) == (5 if l == L else s)
    # Lemma 3.4, s-Top-k form, from the compressions themselves (dense, fp64)
    total = float(np.sum(g.astype(np.float64) ** 2))
    alpha = [float(np.sum(O.topk_dense(g, k).astype(np.float64) ** 2)) / total for k in (ladder[0], ladder[1], ladder[2], ladder[99], ladder[100])]
    p = O.adaptive_p(norms)
    root_sum = math.fsum(norms) / math.sqrt(total)
    assert abs(p[0] - math.sqrt(alpha[1] - alpha[0]) / root_sum) <= 1e-9
    assert abs(p[1] - math.sqrt(alpha[2] - alpha[1]) / root_sum) <= 1e-9
    assert abs(p[99] - math.sqrt(alpha[4] - alpha[3]) / root_sum) <= 1e-7
    # the draw from a long CDF: frequencies of coarse groups of levels match their probability mass (3 sigma)
    N = 4000
    groups = [(0, 64), (64, 512), (512, L)]
    cnt = [0, 0, 0]
    T = O.cdf_thresholds(p)
    for seed in range(N):
        l = O.draw_level(p, seed, 1, 2)
        assert 1 <= l <= L and level_uniform(seed, 1, 2) < T[l - 1] and (l == 1 or level_uniform(seed, 1, 2) >= T[l - 2])
        for gi, (a, b) in enumerate(groups):
            cnt[gi] += a < l <= b
    for gi, (a, b) in enumerate(groups):
        q = math.fsum(p[a:b])
        assert abs(cnt[gi] / N - q) <= 3 * math.sqrt(q * (1 - q) / N)


@pytest.mark.parametrize("adaptive", [False, True])
def test_second_moment_closed_forms(adaptive):
    """App. D: E||g~||^2 = S_0 + sum_l S_l / p_l in general, = S_0 + (sum_l Delta_l)^2 for the adaptive p."""
    w = W.scaled(W.WORKLOADS["resnet18_topk"], d=6000, M=1)
    g = W.generate(w)[0]
    p = None if adaptive else O.geometric_p(w.L)
    norms, units = O.level_norms_row(g, w.ladder)
    S0 = O.units_to_f64(units[0])
    second = 0.0
    for l in range(1, w.L + 1):
        m = O.compress_topk_row(g, w.ladder, p, 0, 0, 0, force_level=l)
        second += m["p"][l - 1] * float(np.sum(m["val"].astype(np.float64) ** 2))
        pp = m["p"]
    want = S0 + sum(x * x / q for x, q in zip(norms, pp) if q > 0)
    assert abs(second - want) <= 1e-6 * want
    if adaptive:
        assert abs(want - (S0 + math.fsum(norms) ** 2)) <= 1e-9 * want


# ----------------------------------------------------------------------------- bit-wise ladder
def test_bits_digits_are_binary_expansion():
    """Sec. 3.1: e = (-1)^{b_0} sum_j b_j 2^-j; the digits the oracle extracts re-assemble the truncation."""
    rng = np.random.default_rng(9)
    g = rng.standard_normal(200).astype(np.float32) * np.float32(0.37)
    e = O.bits_scale_exponent(g)
    s = math.ldexp(1.0, e)
    assert float(np.abs(g).max()) < s <= 2 * float(np.abs(g).max())
    Q = 16
    m = O.fixed_point_digits(g, e, Q)
    for j in range(200):
        x = Fraction(abs(float(g[j]))) / Fraction(s)
        assert 0 <= x < 1
        assert int(m[j]) == int(x * 2 ** Q)             # floor of the exact rational
        for F in (1, 2, 4, 8, 16):
            t = O.bits_truncate_dense(g, F, Q)[j]
            assert abs(Fraction(abs(float(t))) - x * Fraction(s)) < Fraction(s) / 2 ** F   # distortion < 2^-F (scaled)


def test_bits_telescoping_and_constant_magnitude():
    """Unit ladder F = 0..16 with p_l ∝ 2^-l: (1/p_l) b_l 2^-l = (1 - 2^-L) b_l, so every decoded entry is
    0 or ±(1 - 2^-L) s; and sum_l p_l g~(l) = C^{F_L}(g) (Lemma 3.2 for this ladder)."""
    rng = np.random.default_rng(4)
    g = (rng.standard_normal(300) * 0.01).astype(np.float32)
    d = 300
    F = list(range(17))
    L = 16
    p = O.geometric_p(L)
    e = O.bits_scale_exponent(g)
    s = math.ldexp(1.0, e)
    exp = np.zeros(d)
    second = np.zeros(d)
    for l in range(1, L + 1):
        msg = O.compress_bits_row(g, F, p, 0, 0, 0, force_level=l)
        assert msg["planes"].shape == (2, (d + 63) // 64)       # sign + one information bit per entry (Sec. 3.1)
        dec = O.decode_bits_row(msg, F, d).astype(np.float64)
        mags = np.unique(np.abs(dec))
        assert set(mags.tolist()) <= {0.0, float(np.float32((1 - 2.0 ** -L) * s))}
        exp += p[l - 1] * dec
        second += p[l - 1] * dec * dec
    trunc = O.bits_truncate_dense(g, 16, 16)
    assert np.allclose(exp, trunc, rtol=1e-6, atol=0)
    assert np.all(np.abs(trunc - g) < s * 2.0 ** -16)
    # App. C: per-entry second moment (1 - 2^-L) |e| in normalised units
    assert np.allclose(second / s ** 2, (1 - 2.0 ** -L) * np.abs(trunc) / s, rtol=1e-5, atol=0)


def test_bits_general_ladder_expectation_and_layout():
    w = W.scaled(W.WORKLOADS["resnet18_bits"], d=1000, M=1)
    g = W.generate(w)[0]
    d = w.d
    for F in ([0, 1, 2, 4, 8, 16], [2, 3, 8, 12]):
        L = len(F) - 1
        p = O.geometric_p(L)
        exp = np.zeros(d)
        for l in range(1, L + 1):
            msg = O.compress_bits_row(g, F, p, 0, 0, 0, force_level=l)
            assert msg["planes"].shape[0] == 1 + F[0] + F[l] - F[l - 1]
            # plane 0 is the sign, word w bit b <-> element 64 w + b
            for j in (0, 1, 63, 64, 65, d - 1):
                assert bool((int(msg["planes"][0][j // 64]) >> (j % 64)) & 1) == bool(np.signbit(g[j]))
            exp += p[l - 1] * O.decode_bits_row(msg, F, d).astype(np.float64)
        assert np.allclose(exp, O.bits_truncate_dense(g, F[L], F[L]), rtol=2e-6, atol=0)


def test_bits_zero_and_denormal_rows():
    F = [0, 1, 2, 4, 8, 16]
    p = O.geometric_p(5)
    z = np.zeros(130, dtype=np.float32)
    msg = O.compress_bits_row(z, F, p, 0, 0, 0)
    assert msg["scale_exp"] == -125 and not msg["planes"][1:].any()
    assert not O.decode_bits_row(msg, F, 130).any()
    den = np.array([1e-40, -3e-41, 0, 2e-45], dtype=np.float32)
    e = O.bits_scale_exponent(den)
    assert e == -125
    m = O.fixed_point_digits(den, e, 16)
    assert [int(x) for x in m] == [int(Fraction(abs(float(v))) / Fraction(2) ** e * 2 ** 16) for v in den]


# ----------------------------------------------------------------------------- fixed point, divided by the largest entry (Sec. 3.1)
def _vmax_rows():
    rng = np.random.default_rng(77)
    rows = [rng.standard_normal(300).astype(np.float32) * np.float32(0.37)]
    r = (rng.standard_normal(200) * 10.0 ** rng.uniform(-20, 3, size=200)).astype(np.float32)
    r[3] = -r[np.argmax(np.abs(r))]                       # the largest magnitude twice, with both signs
    rows.append(r)
    rows.append(np.array([3.0, -1.5, 0.75, 3.0, -3.0, 1e-40, 0.0, -0.0, 2.9999998], dtype=np.float32))
    rows.append(np.array([1e-40, -3e-41, 0, 2e-45, 1.1754944e-38], dtype=np.float32))     # largest entry barely normal
    rows.append(np.array([2e-45, -1e-45, 0], dtype=np.float32))                           # largest entry the 2nd denormal
    return rows


def _exact_vdigit(x: float, v: float, Q: int) -> int:
    """min(floor(|x| / v 2^Q), 2^Q - 1) in exact rationals."""
    return min(int(Fraction(abs(float(x))) / Fraction(float(v)) * 2 ** Q), 2 ** Q - 1)


def test_vmax_digits_are_the_expansion_of_the_quotient():
    """Sec. 3.1: entries divided by the largest entry, |e| <= 1, binary expansion: digits against exact rationals,
    the distortion bound 2^-F of the truncations, the cap for |e| = 1."""
    for g in _vmax_rows():
        for Q in (1, 7, 16, 24):
            m, v = O.vmax_digits(g, Q)
            assert float(v) == max(abs(float(x)) for x in g)
            assert [int(x) for x in m] == [_exact_vdigit(x, v, Q) for x in g]
            assert int(m[int(np.argmax(np.abs(g)))]) == 2 ** Q - 1
        for F in (1, 2, 4, 8, 16):
            t = O.vbits_truncate_dense(g, F, 16)
            v = Fraction(float(np.abs(g).max()))
            for j in range(g.size):
                err = abs(Fraction(abs(float(g[j]))) - Fraction(abs(float(t[j]))))
                assert err <= v / 2 ** F and (np.signbit(t[j]) == np.signbit(g[j]) or t[j] == 0)
    m, v = O.vmax_digits(np.zeros(70, dtype=np.float32), 16)
    assert v == 0 and not m.any()


def test_vbits_telescoping_expectation_layout_and_aggregate():
    """Lemma 3.2 for this ladder (sum_l p_l g~(l) = C^{F_L}(g)); the wire layout bit by bit and the server's sum
    coordinate by coordinate from exact-rational digits and scalar fp32 operations in worker order."""
    w = W.scaled(W.WORKLOADS["resnet18_bits"], d=64 * 3 + 11, M=4)
    G = W.generate(w)
    G[1] *= np.float32(3.0e6)
    G[2] *= np.float32(1.7e3)
    G[3, ::2] *= np.float32(-1.0)
    d, M = w.d, w.M
    for F, alpha in (([0, 1, 2, 4, 8, 16], 1.0 / 3.0), ([3, 5, 8, 12, 19], 0.37)):
        L, Q = len(F) - 1, F[-1]
        p = O.geometric_p(L)
        g = G[0]
        v0 = float(np.abs(g).max())
        exp = np.zeros(d)
        for l in range(1, L + 1):
            msg = O.compress_vbits_row(g, F, p, 0, 0, 0, force_level=l)
            width = F[l] - F[l - 1]
            assert msg["planes"].shape == (1 + F[0] + width, (d + 63) // 64) and float(msg["vmax"]) == v0
            for j in (0, 1, 63, 64, 65, d - 2, d - 1, int(np.argmax(np.abs(g)))):
                m = _exact_vdigit(g[j], v0, Q)
                base = m >> (Q - F[0]) if F[0] else 0
                field = (m >> (Q - F[l])) & ((1 << width) - 1)
                bit = lambda plane: (int(msg["planes"][plane][j // 64]) >> (j % 64)) & 1
                assert bit(0) == int(np.signbit(g[j]))
                for b in range(F[0]):
                    assert bit(1 + b) == (base >> b) & 1
                for b in range(width):
                    assert bit(1 + F[0] + b) == (field >> b) & 1
            assert not (msg["planes"][:, -1] >> np.uint64(d % 64)).any()
            exp += p[l - 1] * O.decode_vbits_row(msg, F, d).astype(np.float64)
        assert np.allclose(exp, O.vbits_truncate_dense(g, Q, Q), rtol=2e-6, atol=0)
        seed, step = 11, 5
        msgs = O.compress_vbits(G, F, p, seed, step)
        levels = [O.draw_level(p, seed, step, i) for i in range(M)]
        assert len(set(levels)) > 1 and [m["level"] for m in msgs] == levels
        out = O.aggregate_vbits(msgs, F, d, alpha)
        for j in range(d):
            acc = np.float32(0.0)
            for i in range(M):
                l = levels[i]
                v = float(np.abs(G[i]).max())
                m = _exact_vdigit(G[i, j], v, Q)
                f0 = m >> (Q - F[0]) if F[0] else 0
                f = (m >> (Q - F[l])) & ((1 << (F[l] - F[l - 1])) - 1)
                val = np.float32(np.float32(f) * np.float32(math.ldexp(v, -F[l]) / p[l - 1]))
                if F[0]:
                    val = np.float32(np.float32(np.float32(f0) * np.float32(math.ldexp(v, -F[0]))) + val)
                acc = np.float32(acc + (-val if np.signbit(G[i, j]) else val))
            assert out[j] == np.float32(np.float32(alpha) * acc), (F, j)


# ----------------------------------------------------------------------------- Round-to-Nearest ladder (Sec. 3.3, App. G.2)
def _exact_rtn_code(x: float, c: float, b: int) -> int:
    """clamp(rne(x (2^b - 1) / (2c))) in exact rationals, ties to even, |n| <= 2^(b-1) - 1."""
    if b == 0 or c == 0:
        return 0
    t = Fraction(abs(float(x))) * ((1 << b) - 1) / (2 * Fraction(float(c)))
    f = t.numerator // t.denominator
    r = t - f
    n = f + 1 if r > Fraction(1, 2) else f if r < Fraction(1, 2) else (f if f % 2 == 0 else f + 1)
    n = min(n, (1 << (b - 1)) - 1)
    return -n if np.signbit(np.float32(x)) else n


def _rtn_rows():
    rng = np.random.default_rng(5)
    rows = [(rng.standard_normal(400) * 0.3).astype(np.float32)]
    r = (rng.standard_normal(300) * 10.0 ** rng.uniform(-8, 2, size=300)).astype(np.float32)
    r[7] = -np.abs(r).max()
    rows.append(r)
    # quotients exactly between two integers: c = 3.5 and b = 3 give v (2^b - 1) / (2c) = v
    rows.append(np.array([3.5, 0.5, -0.5, 1.5, -1.5, 2.5, -2.5, -3.5, 0.0, -0.0, 0.49999997, 0.50000006, 2.4999998], dtype=np.float32))
    rows.append(np.array([1e-40, -3e-41, 2e-45, 0.0], dtype=np.float32))
    return rows


def test_rtn_codes_round_the_exact_quotient_to_nearest_even():
    """C^l(v) = delta^l clip(round(v / delta^l)), delta^l = 2c / (2^l - 1) (Sec. 3.3): codes against exact rationals
    (ties included), the distortion bound delta^l / 2, zero rows."""
    for g in _rtn_rows():
        c = np.float32(np.abs(g).max())
        for b in (1, 2, 3, 4, 8, 11, 16):
            n = O.rtn_codes(g, c, b)
            assert [int(x) for x in n] == [_exact_rtn_code(x, c, b) for x in g], b
            dense = O.rtn_dense(g, b)
            delta = 2 * Fraction(float(c)) / ((1 << b) - 1)
            for j in range(g.size):
                assert Fraction(float(dense[j])) == 0 or abs(Fraction(float(dense[j])) / delta - int(n[j])) < Fraction(1, 10 ** 9)
                assert abs(int(n[j]) * delta - Fraction(float(g[j]))) <= delta / 2
    tie = _rtn_rows()[2]
    assert O.rtn_codes(tie, np.float32(3.5), 3).tolist() == [3, 0, 0, 2, -2, 2, -2, -3, 0, 0, 0, 1, 2]
    assert not O.rtn_codes(np.zeros(9, dtype=np.float32), np.float32(0), 8).any()
    assert not O.rtn_codes(tie, np.float32(3.5), 0).any()


def test_rtn_norms_telescoping_and_second_moment():
    """Lemma 3.4 for a ladder without rank or bit structure: Delta_l against the plain difference of the two dense
    compressions and against an integer sum in Python ints; sum_l p_l g~(l) = C^{b_L}(v) (Lemma 3.2); with
    p_l = Delta_l / sum Delta the second moment of the residual term is (sum Delta)^2."""
    for B in ([0, 2, 4, 8, 16], [2, 3, 5, 9]):
        for g in _rtn_rows()[:2]:
            d = g.size
            c = np.float32(np.abs(g).max())
            norms = O.rtn_level_norms_row(g, B)
            L = len(B) - 1
            for l in range(1, L + 1):
                diff = O.rtn_dense(g, B[l]) - O.rtn_dense(g, B[l - 1])
                assert math.isclose(norms[l - 1], math.sqrt(math.fsum(diff * diff)), rel_tol=1e-12)
                k = [_exact_rtn_code(x, c, B[l]) * (((1 << B[l - 1]) - 1) if B[l - 1] else 1) -
                     _exact_rtn_code(x, c, B[l - 1]) * ((1 << B[l]) - 1) for x in g]
                assert [int(x) for x in O.rtn_residual_ints(g, c, B[l - 1], B[l])] == k
                DD = ((1 << B[l]) - 1) * (((1 << B[l - 1]) - 1) if B[l - 1] else 1)
                assert norms[l - 1] == (2.0 * float(c) / float(DD)) * math.sqrt(float(sum(x * x for x in k)))
            p = O.adaptive_p(norms)
            exp = np.zeros(d)
            second = 0.0
            base = O.rtn_dense(g, B[0])
            for l in range(1, L + 1):
                msg = O.compress_rtn_row(g, B, None, 0, 0, 0, force_level=l)
                assert msg["planes"].shape[0] == B[0] + (B[l - 1] if l > 1 else 0) + B[l] and msg["p_level"] == p[l - 1]
                dec = O.decode_rtn_row(msg, B, d).astype(np.float64)
                exp += p[l - 1] * dec
                second += p[l - 1] * float(np.sum((dec - base) ** 2))
            assert np.allclose(exp, O.rtn_dense(g, B[L]), rtol=3e-6, atol=float(c) * 1e-9)
            assert math.isclose(second, sum(norms) ** 2, rel_tol=1e-5)


def test_rtn_planes_bit_by_bit_aggregate_and_message_bits():
    """The wire layout from exact-rational codes (two's complement, least significant plane first; base code,
    previous level's code, drawn level's code), the server's sum coordinate by coordinate with scalar fp32
    operations in worker order, and the message size."""
    w = W.scaled(W.WORKLOADS["resnet18_bits"], d=64 * 2 + 9, M=4)
    G = W.generate(w)
    G[1] *= np.float32(3.0e5)
    G[3, ::2] *= np.float32(-1.0)
    d, M = w.d, w.M
    for B, alpha in (([0, 2, 4, 8, 16], 1.0 / 3.0), ([2, 3, 5, 9], 0.37)):
        L = len(B) - 1
        seed, step = 3, 1
        msgs = O.compress_rtn(G, B, None, seed, step)
        levels = [m["level"] for m in msgs]
        for i, m in enumerate(msgs):
            p = O.adaptive_p(O.rtn_level_norms_row(G[i], B))
            assert m["level"] == O.draw_level(p, seed, step, i) and m["p_level"] == p[m["level"] - 1]
        assert len(set(levels)) > 1 or L == 1
        for l in range(1, L + 1):
            g = G[0]
            c = float(np.abs(g).max())
            msg = O.compress_rtn_row(g, B, None, 0, 0, 0, force_level=l)
            fields = ([B[0]] if B[0] else []) + ([B[l - 1]] if l > 1 else []) + [B[l]]
            for j in (0, 1, 63, 64, 65, d - 1, int(np.argmax(np.abs(g)))):
                plane = 0
                for b in fields:
                    u = _exact_rtn_code(g[j], c, b) & ((1 << b) - 1)
                    for q in range(b):
                        assert (int(msg["planes"][plane][j // 64]) >> (j % 64)) & 1 == (u >> q) & 1, (B, l, j, b, q)
                        plane += 1
            assert not (msg["planes"][:, -1] >> np.uint64(d % 64)).any()
            assert O.message_bits_rtn(B, l, d) == d * sum(fields) + 64 + (L - 1).bit_length()
        out = O.aggregate_rtn(msgs, B, d, alpha)
        for j in range(d):
            acc = np.float32(0.0)
            for i in range(M):
                l = levels[i]
                c = float(np.abs(G[i]).max())
                D = (1 << B[l]) - 1
                Dp = ((1 << B[l - 1]) - 1) if B[l - 1] else 1
                k = _exact_rtn_code(G[i, j], c, B[l]) * Dp - _exact_rtn_code(G[i, j], c, B[l - 1]) * D
                val = np.float32(np.float32(k) * np.float32((2.0 * c / float(D * Dp)) / msgs[i]["p_level"]))
                if B[0]:
                    c0 = np.float32(2.0 * c / float((1 << B[0]) - 1))
                    val = np.float32(np.float32(np.float32(_exact_rtn_code(G[i, j], c, B[0])) * c0) + val)
                acc = np.float32(acc + val)
            assert out[j] == np.float32(np.float32(alpha) * acc), (B, j)


# ----------------------------------------------------------------------------- floating-point bit-wise ladder (App. B)
def _fp_rows():
    rng = np.random.default_rng(31)
    g = (rng.standard_normal(400) * 10.0 ** rng.uniform(-12, 6, size=400)).astype(np.float32)
    g[::23] = 0.0
    g[5] = -0.0
    g[7:12] = np.array([1e-40, -3e-41, 2e-45, 1.1754944e-38, -1.17549421e-38], dtype=np.float32)   # denormals and the first normal
    g[12:15] = np.array([1.0, -2.0, 1.0e30], dtype=np.float32)
    return g


def test_float_truncate_is_the_mantissa_truncation():
    """App. B: e = (-1)^S 2^(E-127) (1 + sum_j m_j 2^-j); C^F keeps sign, exponent and the first F mantissa digits.
    Checked with exact rationals built by math.frexp (not from the bit pattern); distortion below 2^(E-127) 2^-F."""
    g = _fp_rows()
    for F in (0, 1, 5, 11, 22, 23):
        t = O.float_truncate(g, F)
        for j in range(g.size):
            x = float(g[j])
            if x == 0.0:
                assert t[j] == 0.0 and np.signbit(t[j]) == np.signbit(g[j])
                continue
            m, e = math.frexp(abs(x))                      # |x| = m 2^e, 0.5 <= m < 1
            e_eff = max(e, -125)                           # denormals: fixed exponent 2^-126, no leading one
            unit = Fraction(2) ** (e_eff - 1)              # 2^(E' - 127): the weight of the digit before the binary point
            q = unit / 2 ** F                              # resolution of C^F
            want = (Fraction(abs(x)) // q) * q             # truncation to a multiple of the resolution
            assert Fraction(abs(float(t[j]))) == want, (F, j, x)
            assert np.signbit(t[j]) == np.signbit(g[j])
            assert Fraction(abs(x)) - want < q
    assert np.array_equal(O.float_truncate(g, 23).view(np.uint32), g.view(np.uint32))


def test_fbits_telescoping_unbiasedness_and_second_moment():
    """Lemma 3.2 for the mantissa ladder: C^{F_0} + sum_l (C^{F_l} - C^{F_{l-1}}) = C^{F_L} (= g when F_L = 23), hence
    sum_l p_l g~(l) = g; and App. B's closed form of the residual's second moment for the unit ladder with
    p_l = 2^-l / (1 - 2^-23): 2^(E-127) (1 - 2^-23) (|e| - 2^(E-127)) per normal entry (exact rationals)."""
    g = _fp_rows()
    for F in (list(range(24)), [0, 1, 2, 4, 8, 16, 23], [3, 5, 12, 20]):
        L = len(F) - 1
        p = O.geometric_p(L)
        tele = O.float_truncate(g, F[0]).astype(np.float64)
        for l in range(1, L + 1):
            tele += O.float_truncate(g, F[l]).astype(np.float64) - O.float_truncate(g, F[l - 1]).astype(np.float64)
        assert np.array_equal(tele, O.float_truncate(g, F[L]).astype(np.float64))
        exp = np.zeros(g.size)
        for l in range(1, L + 1):
            est = O.fbits_estimate_dense(g, F, l, p[l - 1])
            msg = O.compress_fbits_row(g, F, p, 0, 0, 0, force_level=l)
            assert msg["planes"].shape[0] == 9 + F[0] + F[l] - F[l - 1]
            assert np.array_equal(O.decode_fbits_row(msg, F, g.size).view(np.uint32), est.view(np.uint32))   # wire -> same estimate
            exp += p[l - 1] * est.astype(np.float64)
        assert np.allclose(exp, O.float_truncate(g, F[L]).astype(np.float64), rtol=3e-7, atol=0)
    # second moment, unit ladder, exact: sum_l (1/p_l) (m_l 2^-l 2^(E-127))^2
    F = list(range(24))
    pf = [Fraction(1, 2 ** l) / (1 - Fraction(1, 2 ** 23)) for l in range(1, 24)]
    for j in (1, 2, 3, 12, 13, 30, 31, 77):
        x = Fraction(abs(float(g[j])))
        if x == 0:
            continue
        m, e = math.frexp(float(x))
        if e < -125:
            continue
        unit = Fraction(2) ** (e - 1)
        second = Fraction(0)
        for l in range(1, 24):
            r = Fraction(float(O.float_truncate(g[j:j + 1], l)[0])) - Fraction(float(O.float_truncate(g[j:j + 1], l - 1)[0]))
            second += r * r / pf[l - 1]
        assert second == unit * (1 - Fraction(1, 2 ** 23)) * (x - unit)


def test_fbits_planes_bit_by_bit_and_message_bits():
    """Wire layout from Python integers (struct, not numpy views): plane 0 sign, planes 1..8 the exponent field LSB
    first, then the base digits and the level digits as numbers, LSB first; word w bit b <-> element 64 w + b."""
    import struct
    g = _fp_rows()[:64 * 3 + 9]
    d = g.size
    for F in (list(range(24)), [2, 3, 8, 12]):
        L = len(F) - 1
        p = O.geometric_p(L)
        for l in (1, 2, L):
            msg = O.compress_fbits_row(g, F, p, 0, 0, 0, force_level=l)
            width = F[l] - F[l - 1]
            for j in (0, 1, 5, 7, 9, 12, 14, 63, 64, 65, d - 1):
                u = struct.unpack("<I", struct.pack("<f", float(g[j])))[0]
                sign, E, frac = u >> 31, (u >> 23) & 0xFF, u & 0x7FFFFF
                base = frac >> (23 - F[0]) if F[0] else 0
                field = (frac >> (23 - F[l])) & ((1 << width) - 1)
                bit = lambda plane: (int(msg["planes"][plane][j // 64]) >> (j % 64)) & 1
                assert bit(0) == sign
                assert [bit(1 + b) for b in range(8)] == [(E >> b) & 1 for b in range(8)]
                assert [bit(9 + b) for b in range(F[0])] == [(base >> b) & 1 for b in range(F[0])]
                assert [bit(9 + F[0] + b) for b in range(width)] == [(field >> b) & 1 for b in range(width)]
            assert not (msg["planes"][:, -1] >> np.uint64(d % 64)).any()
    # App. B: 13 d + log2(52) bits for fp64 (sign + 11 exponent bits + one mantissa digit), here with the level rounded up
    assert O.message_bits_floating_point(list(range(53)), 17, 1000, exponent_bits=11) == 13 * 1000 + 6
    assert O.message_bits_floating_point(list(range(24)), 5, 1000) == 10 * 1000 + 5


def test_aggregate_fbits_bruteforce():
    """Server aggregate of floating-point messages, one coordinate at a time from the definition (truncations of the
    worker's entry, scalar fp32 operations, worker order, alpha once)."""
    rng = np.random.default_rng(41)
    M, d = 4, 130
    G = (rng.standard_normal((M, d)) * np.array([[1.0], [3e6], [2e-3], [40.0]])).astype(np.float32)
    for F, alpha in (([0, 1, 2, 4, 8, 16, 23], 0.37), ([3, 5, 12, 20], 1.0 / 3.0)):
        L = len(F) - 1
        p = O.geometric_p(L)
        msgs = O.compress_fbits(G, F, p, 11, 5)
        levels = [O.draw_level(p, 11, 5, i) for i in range(M)]
        assert [m["level"] for m in msgs] == levels and len(set(levels)) > 1
        out = O.aggregate_fbits(msgs, F, d, alpha)
        for j in range(d):
            acc = np.float32(0.0)
            for i in range(M):
                l = levels[i]
                e = G[i, j:j + 1]
                r = np.float32(O.float_truncate(e, F[l])[0] - O.float_truncate(e, F[l - 1])[0])
                v = np.float32(O.float_truncate(e, F[0])[0] + np.float32(r * np.float32(1.0 / p[l - 1])))
                acc = np.float32(acc + v)
            assert out[j] == np.float32(np.float32(alpha) * acc), (F, j)


# ----------------------------------------------------------------------------- aggregate
def test_aggregate_identity_special_case_is_alg1_mean():
    """L = 1, k_0 = 0, k_1 = d, p_1 = 1: g~ = g and the aggregate with alpha = 1/M is Alg. 1's mean."""
    rng = np.random.default_rng(1)
    M, d = 4, 257
    G = rng.standard_normal((M, d)).astype(np.float32)
    msgs = O.compress_topk(G, [0, d], [1.0], 0, 0)
    for i in range(M):
        assert np.array_equal(msgs[i]["idx"], np.arange(d)) and np.array_equal(msgs[i]["val"], G[i])
    out = O.aggregate_sparse(msgs, d, 1.0 / M)
    acc = np.zeros(d, dtype=np.float32)
    for i in range(M):
        acc = acc + G[i]
    assert np.array_equal(out, acc * np.float32(0.25))
    assert np.allclose(out, G.astype(np.float64).mean(axis=0), rtol=1e-5, atol=1e-6)


def test_aggregate_sparse_bruteforce():
    rng = np.random.default_rng(8)
    M, d = 5, 90
    G = rng.standard_normal((M, d)).astype(np.float32)
    ladder = [3, 7, 20, 90]
    msgs = O.compress_topk(G, ladder, O.geometric_p(3), 5, 9)
    out = O.aggregate_sparse(msgs, d, 0.5)
    for j in range(d):
        acc = np.float32(0)
        for m in msgs:
            hit = np.nonzero(m["idx"] == j)[0]
            if hit.size:
                acc = np.float32(acc + m["val"][hit[0]])
        assert out[j] == np.float32(np.float32(0.5) * acc)
    # different workers draw different levels across steps (the draw depends on the worker id)
    levels = {(m["level"]) for s in range(20) for m in O.compress_topk(G, ladder, O.geometric_p(3), 5, s)}
    assert len(levels) > 1


def _exact_digit(x: float, e: int, Q: int) -> int:
    """floor(|x| / 2^e * 2^Q) with exact rationals (Sec. 3.1: the first Q fraction bits of the normalised magnitude)."""
    return int(Fraction(abs(float(x))) * Fraction(2) ** (Q - e))


def _check_bits_planes_bit_by_bit():
    """Wire layout of a bit-wise message, element by element from Python integers: word w bit b of a plane belongs
    to element 64 w + b; plane 0 is the sign, planes 1..F_0 are the bits of the base field m >> (Q - F_0), least
    significant first, planes 1 + F_0 + b are bit b of the level field (m >> (Q - F_l)) mod 2^(F_l - F_{l-1})."""
    w = W.scaled(W.WORKLOADS["resnet18_bits"], d=64 * 3 + 11, M=1)
    g = W.generate(w)[0]
    g[65] = -g[65]
    d = w.d
    for F in ([0, 1, 2, 4, 8, 16], [3, 5, 8, 12, 19]):
        L, Q = len(F) - 1, F[-1]
        p = O.geometric_p(L)
        Emax = max((int(np.float32(abs(x)).view(np.uint32)) >> 23) for x in g)
        e = max(Emax, 1) - 126
        for l in range(1, L + 1):
            msg = O.compress_bits_row(g, F, p, 0, 0, 0, force_level=l)
            assert msg["scale_exp"] == e
            width = F[l] - F[l - 1]
            for j in (0, 1, 63, 64, 65, d - 2, d - 1):
                m = _exact_digit(g[j], e, Q)
                base = m >> (Q - F[0]) if F[0] else 0
                field = (m >> (Q - F[l])) & ((1 << width) - 1)
                bit = lambda plane: (int(msg["planes"][plane][j // 64]) >> (j % 64)) & 1
                assert bit(0) == int(np.signbit(g[j]))
                for b in range(F[0]):
                    assert bit(1 + b) == (base >> b) & 1, (F, l, j, b)
                for b in range(width):
                    assert bit(1 + F[0] + b) == (field >> b) & 1, (F, l, j, b)
            # pad bits of the last word are zero in every plane
            assert not (msg["planes"][:, -1] >> np.uint64(d % 64)).any()


def test_bits_planes_bit_by_bit():
    _check_bits_planes_bit_by_bit()


def _check_aggregate_bits_bruteforce():
    """Alg. 2 "Server aggregates" for bit-wise messages, one coordinate at a time: every worker's value is rebuilt
    from exact-rational digits and scalar fp32 operations, added in worker order, then scaled by alpha once."""
    w = W.scaled(W.WORKLOADS["resnet18_bits"], d=150, M=4)
    G = W.generate(w)
    G[1] *= np.float32(3.0e6)     # workers of very different scales: the fp32 sums round, so the order of the adds shows
    G[2] *= np.float32(1.7e3)
    G[3, ::2] *= np.float32(-1.0)
    d, M = w.d, w.M
    for F, alpha in (([2, 3, 8, 12], 0.37), ([0, 1, 2, 4, 8, 16], 1.0 / 3.0)):
        L, Q = len(F) - 1, F[-1]
        p = O.geometric_p(L)
        seed, step = 11, 5
        msgs = O.compress_bits(G, F, p, seed, step)
        levels = [O.draw_level(p, seed, step, i) for i in range(M)]
        assert len(set(levels)) > 1 and [m["level"] for m in msgs] == levels
        out = O.aggregate_bits(msgs, F, d, alpha)
        for j in range(d):
            acc = np.float32(0.0)
            for i in range(M):
                l = levels[i]
                Emax = max((int(np.float32(abs(x)).view(np.uint32)) >> 23) for x in G[i])
                e = max(Emax, 1) - 126
                m = _exact_digit(G[i, j], e, Q)
                f0 = m >> (Q - F[0]) if F[0] else 0
                f = (m >> (Q - F[l])) & ((1 << (F[l] - F[l - 1])) - 1)
                v = np.float32(np.float32(f) * np.float32(math.ldexp(1.0, e - F[l]) / p[l - 1]))
                if F[0]:
                    v = np.float32(np.float32(np.float32(f0) * np.float32(math.ldexp(1.0, e - F[0]))) + v)
                acc = np.float32(acc + (-v if np.signbit(G[i, j]) else v))
            assert out[j] == np.float32(np.float32(alpha) * acc), (F, j)


def test_aggregate_bits_bruteforce():
    _check_aggregate_bits_bruteforce()


def test_bits_pins_catch_planted_mistakes(monkeypatch):
    """The two pins above fail when a plausible mistake is planted in the oracle (on the CPU): planes packed most
    significant bit first, field planes emitted most significant first, alpha dropped, alpha applied per worker,
    workers added in reverse order."""
    real_pack, real_unpack, real_decode, real_compress = O.pack_plane, O.unpack_plane, O.decode_bits_row, O.compress_bits_row

    def expect_failure(check):
        with pytest.raises(AssertionError):
            check()

    # bit order inside a word reversed on both sides (self-consistent, so only an element-position pin sees it)
    def pack_msb(bits):
        dd = bits.size
        padded = np.zeros((dd + 63) // 64 * 64, dtype=np.uint8)
        padded[:dd] = bits
        return np.packbits(padded.reshape(-1, 64)[:, ::-1].reshape(-1), bitorder="little").view("<u8").astype(np.uint64)

    def unpack_msb(words, dd):
        b = np.unpackbits(words.astype("<u8").view(np.uint8), bitorder="little").reshape(-1, 64)[:, ::-1].reshape(-1)
        return b[:dd].astype(bool)

    monkeypatch.setattr(O, "pack_plane", pack_msb)
    monkeypatch.setattr(O, "unpack_plane", unpack_msb)
    expect_failure(_check_bits_planes_bit_by_bit)
    monkeypatch.setattr(O, "pack_plane", real_pack)
    monkeypatch.setattr(O, "unpack_plane", real_unpack)

    # level-field planes in the opposite order on both sides
    def compress_rev(row, F, p, seed, step, worker, force_level=None):
        msg = real_compress(row, F, p, seed, step, worker, force_level)
        k = 1 + F[0]
        msg["planes"] = np.concatenate([msg["planes"][:k], msg["planes"][k:][::-1]])
        return msg

    def decode_rev(msg, F, dd):
        k = 1 + F[0]
        m2 = dict(msg, planes=np.concatenate([msg["planes"][:k], msg["planes"][k:][::-1]]))
        return real_decode(m2, F, dd)

    monkeypatch.setattr(O, "compress_bits_row", compress_rev)
    monkeypatch.setattr(O, "decode_bits_row", decode_rev)
    expect_failure(_check_bits_planes_bit_by_bit)
    _check_aggregate_bits_bruteforce()      # self-consistent: the aggregate pin alone cannot see a wire-order slip
    monkeypatch.setattr(O, "compress_bits_row", real_compress)
    monkeypatch.setattr(O, "decode_bits_row", real_decode)

    # aggregate: alpha dropped / applied to every worker's value / workers in reverse order
    def agg_no_alpha(msgs, F, dd, alpha):
        acc = np.zeros(dd, dtype=np.float32)
        for m in msgs:
            acc = acc + real_decode(m, F, dd)
        return acc

    def agg_alpha_per_row(msgs, F, dd, alpha):
        acc = np.zeros(dd, dtype=np.float32)
        for m in msgs:
            acc = acc + np.float32(alpha) * real_decode(m, F, dd)
        return acc

    def agg_reversed(msgs, F, dd, alpha):
        acc = np.zeros(dd, dtype=np.float32)
        for m in msgs[::-1]:
            acc = acc + real_decode(m, F, dd)
        return (np.float32(alpha) * acc).astype(np.float32)

    for wrong in (agg_no_alpha, agg_alpha_per_row, agg_reversed):
        monkeypatch.setattr(O, "aggregate_bits", wrong)
        expect_failure(_check_aggregate_bits_bruteforce)
    monkeypatch.undo()
    _check_bits_planes_bit_by_bit()
    _check_aggregate_bits_bruteforce()


# ----------------------------------------------------------------------------- server update, message sizes
def test_server_update_is_alg1_sgd_step_in_the_identity_case():
    """Alg. 2 "Server updates" x_{t+1} = x_t - eta g~_t: entry by entry with scalar fp32 operations; and with the
    identity ladder (L = 1, k_1 = d, p_1 = 1) the step is Alg. 1's SGD step on the plain mean of the gradients."""
    rng = np.random.default_rng(21)
    M, d, eta = 4, 300, 0.0371
    G = rng.standard_normal((M, d)).astype(np.float32)
    x = rng.standard_normal(d).astype(np.float32)
    gt = O.aggregate_sparse(O.compress_topk(G, [0, d], [1.0], 0, 0), d, 1.0 / M)
    got = O.server_update(x, gt, eta)
    for j in range(d):
        assert got[j] == np.float32(x[j] - np.float32(np.float32(eta) * gt[j]))
    want64 = x.astype(np.float64) - eta * G.astype(np.float64).mean(axis=0)
    assert np.allclose(got, want64, rtol=1e-5, atol=1e-6)
    # a planted fused multiply-add (one rounding) differs somewhere; so does a dropped eta
    fused = (x.astype(np.float64) - np.float64(np.float32(eta)) * gt.astype(np.float64)).astype(np.float32)
    assert np.any(fused != got) and np.any((x - gt) != got)


def test_message_bits_match_the_papers_counts():
    d = 1_000_003
    # Sec. 3.1: unit fixed-point ladder of 63 bits, 64-bit scale: 2 d + 64 + ceil(log2 63)
    F = list(range(64))
    for l in (1, 17, 63):
        assert O.message_bits_fixed_point(F, l, d, scale_bits=64) == 2 * d + 64 + 6
    # the benchmark's ladder 1, 2, 4, 8, 16 bits with a 32-bit scale: sign + field width per entry
    F = [0, 1, 2, 4, 8, 16]
    assert [O.message_bits_fixed_point(F, l, d) for l in range(1, 6)] == [d * w + 32 + 3 for w in (2, 2, 3, 5, 9)]
    # Sec. 3 / Sec. 3.2: Top-k with k_l = l sends one entry, s-Top-k sends s entries (value + index), plus the level
    ladder = list(range(0, 101))
    assert O.message_bits_topk(ladder, 37, d) == (32 + 20) + 7
    s_ladder = [64 * l for l in range(0, 51)]
    assert O.message_bits_topk(s_ladder, 50, d) == 64 * (32 + 20) + 6
    assert O.message_bits_topk([10, 20, 40], 2, 1 << 20) == (10 + 20) * (32 + 20) + 1


# ----------------------------------------------------------------------------- workloads
def test_workload_generators_are_deterministic_and_shaped():
    for name in ("tiny_topk", "resnet18_topk", "resnet50_adaptive_topk", "resnet18_bits", "bert_adaptive_topk_bf16"):
        w = W.WORKLOADS[name]
        assert w.ladder[-1] == (w.d if w.kind == "topk" else 16)
        s = W.scaled(w, d=5000, M=2)
        a, b = W.generate(s), W.generate(s)
        assert a.shape == (2, 5000) and np.array_equal(a, b)
        assert not np.array_equal(a[0], a[1])
    assert W.WORKLOADS["resnet18_topk"].ladder[:3] == (11415, 22831, 45662)
    assert W.WORKLOADS["resnet50_adaptive_topk"].ladder[0] == 6239
    assert W.WORKLOADS["bert_adaptive_topk_bf16"].ladder[0] == 1898
    lens, std = W.segment_layout(11_689_512, 62, 1e-4, 1e-1, 0)
    assert lens.sum() == 11_689_512 and len(lens) == 62 and std.min() >= 1e-4 and std.max() <= 1e-1
