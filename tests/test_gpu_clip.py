"""GPU parity of the clipped 8-bit representation and the integer aggregator: the HIP library
(through its C ABI) against the CPU oracle, bit for bit (bytes, int64 sums, exponent and sign
planes of the compressed sum)."""
import numpy as np
import pytest
import torch

from gpu_util import Guarded, dev, host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def nc():
    from paper_1905_10988_amd import natcomp
    natcomp.lib()
    assert torch.cuda.is_available()
    return natcomp


@pytest.fixture(scope="module")
def wl():
    from paper_1905_10988_amd import workloads
    return workloads


def wide(rng, d):
    """Laplace values times 2^U(-70, 25): both ends of the clip range are exercised."""
    x = (rng.laplace(0, 1, d) * np.exp2(rng.uniform(-70, 25, d))).astype(np.float32)
    x[::53] = 0.0
    x[7::211] = -0.0
    return x


def random_codes(rng, n, d, max_field=63):
    code = rng.integers(0, max_field + 1, size=(n, d)).astype(np.uint8)
    code |= (rng.integers(0, 2, size=(n, d)) << 7).astype(np.uint8)
    zero = rng.random((n, d)) < 0.1
    code[zero] = (code[zero] & 0x80) | 0x40
    return code


@pytest.mark.parametrize("d", [1, 3, 4, 5, 31, 1023, 1024, 1029, 70_001])
def test_encode_decode_sizes(nc, oracle, wl, d):
    rng = np.random.default_rng(d)
    x = wide(rng, d)
    x[: min(d, 25)] = wl.edge_values()[: min(d, 25)]
    for seed, worker, off in [(0, 0, 0), (2**40 + 3, 5, 8), (9, 1, 2**34 + 4)]:
        buf = Guarded(d)
        nc.nat_clip_encode(dev(x), seed, worker, off, code_out=buf.t)
        torch.cuda.synchronize()
        got = buf.check()
        want = oracle.clip_encode(x, seed, worker, off)
        assert np.array_equal(got, want), f"bytes differ at {np.flatnonzero(got != want)[:8]}"
        out = Guarded(d, torch.float32)
        nc.nat_clip_decode(buf.t, d, out=out.t)
        torch.cuda.synchronize()
        assert np.array_equal(out.check().view(np.uint32), oracle.clip_decode(want).view(np.uint32))


@pytest.mark.parametrize("shift,index_offset", [(1, 0), (3, 4), (0, 1), (0, 6), (2, 2**35 + 3)])
def test_encode_unaligned(nc, oracle, shift, index_offset):
    d = 9001
    rng = np.random.default_rng(77)
    base = wide(rng, d + 8)
    x = base[shift: shift + d].copy()
    xdev = dev(base)[shift: shift + d]
    raw = Guarded(d + 8)
    out = raw.t[shift + 1: shift + 1 + d]          # misaligned destination too
    before = host(raw.t).copy()
    nc.nat_clip_encode(xdev, 5, 2, index_offset, code_out=out)
    torch.cuda.synchronize()
    got = raw.check()
    want = oracle.clip_encode(x, 5, 2, index_offset)
    assert np.array_equal(got[shift + 1: shift + 1 + d], want)
    assert np.array_equal(got[: shift + 1], before[: shift + 1])
    assert np.array_equal(got[shift + 1 + d:], before[shift + 1 + d:])
    dec = Guarded(d + 4, torch.float32)
    nc.nat_clip_decode(out, d, out=dec.t[1: 1 + d])
    torch.cuda.synchronize()
    assert np.array_equal(dec.check()[1: 1 + d].view(np.uint32), oracle.clip_decode(want).view(np.uint32))


def test_encode_batch_and_relation_to_nat_encode(nc, oracle):
    """Three workers in one launch; the byte is the clipped form of nc_nat_encode's planes."""
    n, d, row = 3, 40_003, 40_192
    rng = np.random.default_rng(3)
    x = np.zeros((n, row), np.float32)
    for w in range(n):
        x[w, :d] = wide(rng, d)
    xdev = dev(x)
    code = nc.nat_clip_encode(xdev, 17, first_worker=4, index_offset=12, d=d)
    torch.cuda.synchronize()
    assert code.shape[0] == n and code.shape[1] % 256 == 0
    for w in range(n):
        want = oracle.clip_encode(x[w, :d], 17, 4 + w, 12)
        assert np.array_equal(host(code[w, :d]), want)
        e, s = nc.nat_encode(xdev[w, :d].contiguous(), 17, 4 + w, 12)
        e, s = host(e)[:d].astype(np.int64), np.unpackbits(host(s), bitorder="little")[:d]
        byte = np.where(e == 0, 0x40, np.clip(e, 77, 137) - 77) | (s.astype(np.int64) << 7)
        assert np.array_equal(byte.astype(np.uint8), want)


def test_decode_every_byte(nc, oracle):
    code = np.tile(np.arange(256, dtype=np.uint8), 9)[: 256 * 9 - 3]
    got = host(nc.nat_clip_decode(dev(code), code.size))
    assert np.array_equal(got.view(np.uint32), oracle.clip_decode(code).view(np.uint32))


@pytest.mark.parametrize("n", [1, 2, 3, 7, 8, 9, 17])
def test_aggregate_parity(nc, oracle, n):
    rng = np.random.default_rng(100 + n)
    for d, stride, off in [(20_011, 20_016, 0), (4096, 4096, 8), (2053, 2061, 5), (5, 8, 2**34)]:
        code = np.zeros((n, stride), np.uint8)
        code[:, :d] = random_codes(rng, n, d, max_field=63 if n != 7 else 60)
        sums, e, s = Guarded(d, torch.int64), Guarded(d), Guarded(nc.sign_bytes(d))
        nc.clip_aggregate_int(dev(code), d, 41, master=2, index_offset=off, sum_out=sums.t, exp_out=e.t,
                              sign_out=s.t)
        torch.cuda.synchronize()
        so, eo, sgo = oracle.clip_aggregate(code, d, 41, 2, off)
        assert np.array_equal(sums.check(), so)
        assert np.array_equal(e.check(), eo), f"exponents differ at {np.flatnonzero(e.check() != eo)[:8]}"
        assert np.array_equal(s.check(), sgo)
        # either output alone gives the same bits
        only_sum, none_e, none_s = nc.clip_aggregate_int(dev(code), d, 41, 2, off, want_sum=True, want_planes=False)
        assert none_e is None and none_s is None and np.array_equal(host(only_sum), so)
        _, e2, s2 = nc.clip_aggregate_int(dev(code), d, 41, 2, off)
        assert np.array_equal(host(e2), eo) and np.array_equal(host(s2), sgo)


def test_aggregate_unaligned_views(nc, oracle):
    n, d = 4, 3001
    rng = np.random.default_rng(9)
    code = np.zeros((n, d + 3), np.uint8)
    code[:, :d] = random_codes(rng, n, d)
    base = dev(np.concatenate([np.zeros(1, np.uint8), code.ravel()]))
    view = base[1:].view(n, d + 3)                     # rows start at odd addresses
    e_raw, sum_raw = Guarded(d + 1), Guarded(d + 1, torch.int64)
    s_out = Guarded(nc.sign_bytes(d))
    nc.clip_aggregate_int(view, d, 6, master=0, index_offset=3, sum_out=sum_raw.t[1: 1 + d], exp_out=e_raw.t[1: 1 + d],
                          sign_out=s_out.t)
    torch.cuda.synchronize()
    so, eo, sgo = oracle.clip_aggregate(code, d, 6, 0, 3)
    assert np.array_equal(sum_raw.check()[1: 1 + d], so)
    assert np.array_equal(e_raw.check()[1: 1 + d], eo) and np.array_equal(s_out.check(), sgo)


def test_pipeline_matches_float_master_inside_the_range(nc, oracle, wl):
    """Gradient-like values (all exponents inside -50 .. 10, within 24 bits of each other after
    compression is not required): the integer path's decoded result equals nc_master_nat's when the
    binary32 sum is exact, and is always within one binade of it."""
    n, d = 8, 100_000
    x = np.stack([wl.config1(seed=30 + w)[:d] for w in range(n)])
    code = nc.nat_clip_encode(dev(x), 21)
    _, e, s = nc.clip_aggregate_int(code, d, 22, master=1)
    got = host(nc.nat_decode(e, s, d)).astype(np.float64)
    sums, _, _ = nc.clip_aggregate_int(code, d, 22, master=1, want_sum=True, want_planes=False)
    exact = np.ldexp(host(sums).astype(np.float64), -50)     # |sums| < 2^53 here: conversion is exact
    assert np.abs(host(sums)).max() < 2**53
    nz = exact != 0
    ratio = np.abs(got[nz]) / np.abs(exact[nz])
    assert ((ratio > 0.5) & (ratio <= 2.0)).all() and np.array_equal(np.sign(got[nz]), np.sign(exact[nz]))
    assert (got[~nz] == 0).all()
    # oracle on the same bytes
    so, eo, sgo = oracle.clip_aggregate(host(code), d, 22, 1, 0)
    assert np.array_equal(host(sums), so) and np.array_equal(host(e), eo) and np.array_equal(host(s), sgo)


def test_full_size_config2_shape(nc, oracle, wl):
    """d = 25,557,032, 8 workers (the headline shape): encode of one worker and the integer
    aggregation of all eight, whole vectors against the oracle."""
    d, n = wl.D_RESNET50, 8
    x = torch.empty((n, d), dtype=torch.float32, device="cuda")
    g = torch.Generator(device="cuda")
    g.manual_seed(1234)
    x.normal_(generator=g)
    x *= 1e-3
    code = nc.nat_clip_encode(x, 7)
    torch.cuda.synchronize()
    w = 5
    want = oracle.clip_encode(host(x[w]), 7, w, 0)
    assert np.array_equal(host(code[w, :d]), want)
    sums, e, s = nc.clip_aggregate_int(code, d, 8, master=0, want_sum=True)
    torch.cuda.synchronize()
    so, eo, sgo = oracle.clip_aggregate(host(code), d, 8, 0, 0)
    assert np.array_equal(host(sums), so) and np.array_equal(host(e), eo) and np.array_equal(host(s), sgo)


def test_errors(nc):
    x = torch.zeros(100, dtype=torch.float32, device="cuda")
    code = torch.zeros((2, 100), dtype=torch.uint8, device="cuda")
    with pytest.raises(nc.NatcompError, match="NULL"):
        nc.clip_aggregate_int(code, 100, 0, want_sum=False, want_planes=False)
    with pytest.raises(nc.NatcompError, match="NULL"):
        nc.clip_aggregate_int(code, 100, 0, want_planes=False, exp_out=torch.zeros(100, dtype=torch.uint8, device="cuda"))
    with pytest.raises(nc.NatcompError, match="INVALID"):
        nc._check(nc.lib().nc_clip_aggregate_int(code.data_ptr(), 50, 2, 100, 0, 0, 0, None, code.data_ptr(),
                                                 code.data_ptr(), None))
    assert nc.nat_clip_encode(x[:0], 0).numel() == 0


def test_word_equal_to_threshold_stays_on_gpu(nc, oracle):
    """The comparison in the master's rounding is strict: an element whose random word r is known
    carries the sum 2^60 + r 2^28 (threshold = r) and must stay at 2^60, both in the vector path
    and in the any-alignment path; with one more unit of 2^28 it goes up."""
    seed, master = 123, 2
    g = oracle.find_word_below(seed, master, 3, 0, 1 << 22, 1 << 12)
    r = oracle.random_word(seed, master, 3, g)
    assert g >= 0 and 0 < r < (1 << 12)
    for extra, up in [(0, 0), (1, 1)]:
        units = (1 << 60) + ((r + extra) << 28)
        bits = [b for b in range(64) if (units >> b) & 1]
        for d, pos, off in [(64, g % 4, g - g % 4), (64, 37, g - 37), (5, 2, g - 2)]:
            if off < 0:
                continue
            code = np.full((len(bits), d), 0x40, np.uint8)
            code[:, pos] = bits
            sums, e, s = nc.clip_aggregate_int(dev(code), d, seed, master=master, index_offset=off, want_sum=True)
            so, eo, sgo = oracle.clip_aggregate(code, d, seed, master, off)
            assert np.array_equal(host(sums), so) and np.array_equal(host(e), eo) and np.array_equal(host(s), sgo)
            assert int(host(sums)[pos]) == units and int(host(e)[pos]) == 60 + 77 + up
