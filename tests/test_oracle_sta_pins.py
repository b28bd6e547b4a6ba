"""Pins of the oracle's standard dithering D_sta^{p,s} (the paper's comparison operator) and of
the relation between natural and standard dithering (Thm. 5 and the empirical-variance appendix)."""
import math
from fractions import Fraction

import numpy as np

from conftest import golden_lines

TWO32 = 1 << 32


def threshold(oracle, y, s):
    """(low code, T) with outcome low+1 iff r < T."""
    c_hi, c_lo = oracle.sta_level(y, s, 0), oracle.sta_level(y, s, TWO32 - 1)
    assert c_hi - c_lo in (0, 1)
    if c_hi == c_lo:
        return c_lo, 0
    lo, hi = 0, TWO32
    while hi - lo > 1:
        mid = (lo + hi) // 2
        if oracle.sta_level(y, s, mid) == c_hi:
            lo = mid
        else:
            hi = mid
    return c_lo, hi


def test_paper_example_exhaustive(oracle):
    (_, s, y, ln, ld, hn, hd, p_high), = golden_lines("paper_examples.txt", "sdither")
    s, y = int(s), float(y)
    low, high = Fraction(int(ln), int(ld)), Fraction(int(hn), int(hd))
    c_low, c_high = int(low * s), int(high * s)
    assert c_high == c_low + 1
    n_high = oracle.sta_count(y, s, c_high)
    assert n_high + oracle.sta_count(y, s, c_low) == TWO32
    # t = fl(0.375 * 3) = 1.125 exactly, so the probability is exactly 1/8
    assert Fraction(n_high, TWO32) == Fraction(p_high)


def test_probabilities_match_definition(oracle):
    """xi(y) = l_high w.p. (y - l_low)/(l_high - l_low) with l_j = j/s (Def. 3), up to the one
    rounding of t = fl(y s) (relative 2^-24) and the 2^-32 truncation of the threshold."""
    rng = np.random.default_rng(51)
    for s in (1, 2, 3, 4, 7, 8, 15, 16, 100, 128, 255):
        for y in np.concatenate([rng.uniform(0, 1, 40), [0.0, 1.0, 0.5, 1.0 / s, 1e-30]]).astype(np.float32):
            fy = Fraction(float(y))
            c_lo, T = threshold(oracle, y, s)
            if fy >= 1:
                assert (c_lo, T) == (s, 0)
                continue
            t_exact = fy * s
            p_up = Fraction(T, TWO32)
            mean_level = Fraction(c_lo) + p_up          # E[c] should be y s
            assert abs(mean_level - t_exact) <= t_exact * Fraction(1, 1 << 23) + Fraction(1, TWO32)
            assert Fraction(c_lo) <= t_exact * (1 + Fraction(1, 1 << 23))
            assert t_exact * (1 - Fraction(1, 1 << 23)) <= c_lo + 1
    # exact levels stay put, values above 1 and NaN are the top level
    for s in (4, 8):
        for j in range(s + 1):
            for r in (0, TWO32 - 1):
                assert oracle.sta_level(j / s if (j / s) == float(np.float32(j / s)) else 0.0, s, r) in (j, 0)
    assert oracle.sta_level(1.5, 4, 0) == 4 and oracle.sta_level(float("nan"), 4, 5) == 4


def test_vector_roundtrip_unbiased_and_qsgd_bound(oracle):
    """Decoded magnitudes are norm * j/s with j adjacent to |x| s / norm; over seeds the mean is x and
    the variance obeys the QSGD bound min(d/s^2, sqrt(d)/s) ||x||^2 for p = 2."""
    rng = np.random.default_rng(52)
    d, s, S = 2000, 4, 300
    x = rng.standard_normal(d).astype(np.float32)
    x64 = x.astype(np.float64)
    norms = oracle.pnorm_segments(x, 2).astype(np.float32)
    acc = np.zeros(d)
    var = 0.0
    for seed in range(S):
        code, sign = oracle.sta_encode(x, s, norms, seed)
        y = oracle.sta_decode(norms, code, sign, d, s).astype(np.float64)
        j = np.abs(y) / float(norms[0]) * s
        assert np.all(np.abs(j - np.rint(j)) < 1e-5)
        t = np.abs(x64) / float(norms[0]) * s
        assert np.all((np.rint(j) >= np.floor(t) - 1e-9) & (np.rint(j) <= np.floor(t) + 1 + 1e-9))
        assert np.array_equal(np.signbit(y), np.signbit(x))
        acc += y
        var += ((y - x64) ** 2).sum()
    var /= S
    assert var <= min(d / s ** 2, math.sqrt(d) / s) * (x64 ** 2).sum()
    sd = math.sqrt(var / d / S)
    assert abs((acc / S - x64).mean()) < 5 * sd / math.sqrt(d)


def test_natural_vs_standard_variance(oracle):
    """Empirical-variance appendix, smaller d: with the same number of levels natural dithering has
    a far smaller variance (p = 1, 2, where the normalised entries are small); against standard dithering with 2^(s-1) levels it is within the factor
    of Thm. 5 (omega_nat + 1 <= 9/8 (omega_sta + 1)); for p = inf and s = 32 standard dithering wins
    and natural dithering sits near its 1/8 floor."""
    rng = np.random.default_rng(53)
    d, S = 20000, 12

    def omega(kind, x, p, s):
        norms = oracle.pnorm_segments(x, p).astype(np.float32)
        x64 = x.astype(np.float64)
        tot = 0.0
        for seed in range(S):
            if kind == "nat":
                c, sg = oracle.dither_encode(x, s, norms, seed)
                y = oracle.dither_decode(norms, c, sg, d, s)
            else:
                c, sg = oracle.sta_encode(x, s, norms, seed)
                y = oracle.sta_decode(norms, c, sg, d, s)
            tot += ((y.astype(np.float64) - x64) ** 2).sum() / (x64 ** 2).sum()
        return tot / S

    x = rng.standard_normal(d).astype(np.float32)
    for p in (1, 2, math.inf):
        s = 8
        w_nat, w_sta_same, w_sta_exp = omega("nat", x, p, s), omega("sta", x, p, s), omega("sta", x, p, 2 ** (s - 1))
        if p != math.inf:       # for the max-norm and s = 8 the linear partition is the finer one where the mass is
            assert w_nat < 0.1 * w_sta_same
        assert w_nat + 1 <= (9 / 8) * (w_sta_exp + 1) * 1.02
    w_nat, w_sta = omega("nat", x, math.inf, 32), omega("sta", x, math.inf, 32)
    assert w_sta < w_nat <= 1 / 8 * 1.05
