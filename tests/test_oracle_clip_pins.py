"""Pins of the oracle's clipped 8-bit format and integer aggregation (the aggregation prototype of
the experimental setup and the appendix on fast aggregation): bytes that follow from the text for
powers of two, the clip applied to the (separately pinned) C_nat planes, integer sums against
Python's exact integers, and the compression of the integer sum against closed-form thresholds and
against the binary32 master path on sums binary32 holds exactly."""
import math

import numpy as np

from conftest import golden_lines

TWO32 = 1 << 32
DOMAIN_MASTER = 3


def test_bytes_of_powers_of_two(oracle):
    rows = golden_lines("clip8_examples.txt", "clip")
    x = np.array([(-1.0 if r[1] == "1" else 1.0) * (0.0 if r[2] == "zero" else math.ldexp(1.0, int(r[2])))
                  for r in rows], np.float32)
    want = np.array([int(r[3], 16) for r in rows], np.uint8)
    for seed in (0, 1, 2**40 + 7):
        for off in (0, 5):
            assert np.array_equal(oracle.clip_encode(x, seed, worker=3, index_offset=off), want)


def test_units_of_a_byte(oracle):
    rows = golden_lines("clip8_examples.txt", "units")
    code = np.array([[int(r[1], 16) for r in rows]], np.uint8)
    total, _, _ = oracle.clip_aggregate(code, code.shape[1], seed=0)
    assert [int(v) for v in total] == [int(r[2]) for r in rows]
    # and the decoded binary32 value is that integer times 2^-50
    dec = oracle.clip_decode(code[0])
    assert [math.ldexp(float(v), 50) for v in dec] == [float(int(r[2])) for r in rows]


def test_equals_clipped_natural_compression(oracle):
    """Byte stream == C_nat planes (pinned elsewhere) with the exponent clamped in numpy."""
    rng = np.random.default_rng(5)
    d = 50_000
    x = (rng.laplace(0, 1, d) * np.exp2(rng.uniform(-70, 25, d))).astype(np.float32)
    x[::97] = 0.0
    x[1::197] = -0.0
    seed, worker, off = 77, 2, 12
    e, s = oracle.nat_encode(x, seed, worker, off)
    q = oracle.nat_decode(e, s, d).astype(np.float64)
    clipped = np.where(q == 0, q, np.copysign(np.clip(np.abs(q), 2.0**-50, 2.0**10), q))
    got = oracle.clip_decode(oracle.clip_encode(x, seed, worker, off)).astype(np.float64)
    assert np.array_equal(got, clipped)
    assert np.array_equal(np.signbit(got), np.signbit(clipped))
    # the clip really is exercised on both sides
    assert (np.abs(q[q != 0]) < 2.0**-50).any() and (np.abs(q) > 2.0**10).any()


def test_integer_sum_is_exact(oracle):
    rng = np.random.default_rng(6)
    n, d = 7, 20_000
    code = rng.integers(0, 61, size=(n, d)).astype(np.uint8)
    code |= (rng.integers(0, 2, size=(n, d)) << 7).astype(np.uint8)
    zero = rng.random((n, d)) < 0.1
    code[zero] = (code[zero] & 0x80) | 0x40
    code[:, 0] = 60          # seven times the largest magnitude: 7 * 2^60 < 2^63
    code[:, 1] = 60 | 0x80
    total, _, _ = oracle.clip_aggregate(code, d, seed=1)
    dec = np.stack([oracle.clip_decode(code[w]) for w in range(n)])
    for i in list(range(64)) + list(rng.integers(0, d, 500)):
        exact = sum(int(math.ldexp(float(dec[w, i]), 50)) for w in range(n))   # Python integers
        assert int(total[i]) == exact
    assert int(total[0]) == 7 << 60 and int(total[1]) == -(7 << 60)


def _codes_for(values_units):
    """One worker per non-zero bit of each integer (all positive here)."""
    nbits = max(bin(v).count("1") for v in values_units)
    code = np.full((nbits, len(values_units)), 0x40, np.uint8)
    for i, v in enumerate(values_units):
        bits = [b for b in range(64) if (v >> b) & 1]
        for w, b in enumerate(bits):
            code[w, i] = b
    return code


def test_rounding_thresholds_closed_form(oracle):
    """S = 5 * 2^j has (|S| - 2^k) / 2^k = 1/4; S = 3 * 2^j has 1/2; a power of two never moves;
    2^45 + 2^44 + 2^3 has 1/2 + 2^-42, which 32 bits see as 1/2."""
    d, seed, master, off = 4096, 99, 4, 8
    r = np.array([oracle.random_word(seed, master, DOMAIN_MASTER, off + i) for i in range(d)], np.uint64)
    for units, k, threshold in [(5 << 7, 9, 1 << 30), (3 << 20, 21, 1 << 31), (1 << 33, 33, 0),
                                ((1 << 45) + (1 << 44) + (1 << 3), 45, 1 << 31), (7, 2, 3 << 30),
                                ((1 << 60) + (1 << 28), 60, 1), ((1 << 60) + (1 << 27), 60, 0)]:
        code = np.repeat(_codes_for([units]), d, axis=1)
        total, e, s = oracle.clip_aggregate(code, d, seed, master, off)
        assert (total == units).all() and not s.any()
        want = (k - 50 + 127) + (r < threshold).astype(np.int64)
        assert np.array_equal(e.astype(np.int64), want)
        if 0 < threshold < TWO32:
            p = threshold / TWO32
            assert abs((r < threshold).mean() - p) < 5 * math.sqrt(p * (1 - p) / d)


def test_negative_sums_and_zero(oracle):
    code = np.array([[50, 50 | 0x80, 0x40, 52 | 0x80, 0xC0],
                     [50 | 0x80, 50 | 0x80, 0x40, 50, 0xC0]], np.uint8)
    total, e, s = oracle.clip_aggregate(code, 5, seed=3)
    assert [int(v) for v in total] == [0, -(2 << 50), 0, -(3 << 50), 0]
    assert e[0] == 0 and e[2] == 0 and e[4] == 0            # integer zero: byte 0, no sign
    assert e[1] == 128 and e[3] in (128, 129)               # -2 exactly; -3 goes to -2 or -4
    assert s[0] == 0b01010


def test_matches_binary32_master_on_exact_sums(oracle):
    """Fields 39..59 and 8 workers: every partial sum is a multiple of 2^39 below 2^63, at most 24
    significant bits, so the binary32 sum is exact and C_nat of it draws the same comparison."""
    rng = np.random.default_rng(8)
    n, d = 8, 30_000
    field = rng.integers(39, 60, size=(n, d)).astype(np.uint8)
    sign = rng.integers(0, 2, size=(n, d)).astype(np.uint8)
    zero = rng.random((n, d)) < 0.15
    code = np.where(zero, 0x40, field | (sign << 7)).astype(np.uint8)
    exp_plane = np.where(zero, 0, field.astype(np.int64) - 50 + 127).astype(np.uint8)
    sign_plane = np.stack([np.packbits(np.where(zero[w], 0, sign[w]), bitorder="little") for w in range(n)])
    seed, master, off = 31, 1, 4
    sum32, e32, s32 = oracle.master_nat(exp_plane, sign_plane, d, seed, master, off)
    total, e, s = oracle.clip_aggregate(code, d, seed, master, off)
    assert np.array_equal(np.ldexp(total.astype(np.float64), -50), sum32.astype(np.float64))
    nz = total != 0
    assert np.array_equal(e[nz], e32[nz]) and (e[~nz] == 0).all() and (e32[~nz] == 0).all()
    assert np.array_equal(s, s32)
    assert nz.sum() > d // 2 and (e != (np.floor(np.log2(np.abs(total) + (total == 0))) + 77))[nz].any()


def test_rounding_counts_exhaustive(oracle):
    """All 2^32 words: 5 * 2^57 goes up for exactly 2^30 of them and 2^60 + 2^28 for exactly one
    (r = 0); for other sums the two words next to the threshold decide (strict comparison)."""
    assert oracle.clip_count_up(5 << 57) == 1 << 30
    assert oracle.clip_count_up((1 << 60) + (1 << 28)) == 1
    for total, k, threshold in [(5 << 7, 9, 1 << 30), (3 << 40, 41, 1 << 31), (-7, 2, 3 << 30), (-(9 << 20), 23, 1 << 29)]:
        assert oracle.clip_round(total, threshold - 1) == k + 77 + 1
        assert oracle.clip_round(total, threshold) == k + 77         # r = threshold stays
        assert oracle.clip_round(total, 0) == k + 77 + 1 and oracle.clip_round(total, TWO32 - 1) == k + 77
    for r in (0, 1, TWO32 - 1):
        assert oracle.clip_round(1 << 33, r) == 33 + 77 and oracle.clip_round(0, r) == 0


def test_word_equal_to_threshold_stays(oracle):
    """An element whose word r is known and small gets the sum 2^60 + r 2^28, whose threshold is r
    itself: it must stay at 2^60; one more unit of 2^28 and it goes up."""
    seed, master = 123, 2
    g = oracle.find_word_below(seed, master, DOMAIN_MASTER, 0, 1 << 22, 1 << 12)
    assert g >= 0
    r = oracle.random_word(seed, master, DOMAIN_MASTER, g)
    assert 0 < r < (1 << 12)
    for extra, up in [(0, 0), (1, 1)]:
        units = (1 << 60) + ((r + extra) << 28)
        code = _codes_for([units])
        total, e, s = oracle.clip_aggregate(code, 1, seed, master, index_offset=g)
        assert int(total[0]) == units and e[0] == 60 + 77 + up and s[0] == 0
