"""Differential test over randomly drawn configurations (fixed seed): vector length, segment
description (whole vector, buckets of any size, layer offsets with empty and tiny segments),
norm, level count, alignment of every buffer, index offset and number of workers are drawn
together, so that combinations no hand-written case names still meet the oracle."""
import math

import numpy as np
import pytest
import torch

from gpu_util import dev, host

pytestmark = pytest.mark.gpu
INF = math.inf


@pytest.fixture(scope="module")
def nc():
    from paper_1905_10988_amd import natcomp
    natcomp.lib()
    return natcomp


def draw_segments(rng, d):
    kind = rng.integers(0, 4)
    if kind == 0:
        return None, 0
    if kind == 1:                                        # buckets: any size, often a multiple of 8 or 32
        b = int(rng.integers(1, 5000))
        step = int(rng.choice([1, 8, 32, 32, 256]))
        return None, max(step, b // step * step)
    if kind == 2:                                        # power-of-two buckets
        return None, int(2 ** rng.integers(3, 14))
    cuts = np.sort(rng.integers(0, d + 1, size=int(rng.integers(0, 40))))
    if rng.random() < 0.3:                               # some tiny and empty segments
        extra = cuts[: len(cuts) // 2] + rng.integers(0, 3, size=len(cuts) // 2)
        cuts = np.sort(np.concatenate([cuts, np.minimum(extra, d)]))
    return np.concatenate([[0], cuts, [d]]).astype(np.uint64), 0


def shifted(t, shift, dtype):
    """A device buffer whose first element sits `shift` elements past an aligned address."""
    raw = torch.empty(t + shift + 16, dtype=dtype, device="cuda")
    return raw[shift: shift + t]


@pytest.mark.parametrize("case", range(120))
def test_dither_roundtrip_and_sum(nc, oracle, case):
    rng = np.random.default_rng(7000 + case)
    d = int(rng.choice([rng.integers(1, 300), rng.integers(300, 20_000), rng.integers(20_000, 120_000)]))
    offsets, bucket = draw_segments(rng, d)
    p = [1, 2, INF][rng.integers(0, 3)]
    s = int(rng.choice([1, 2, 3, 4, 7, 8, 15, 16, 31, 100, 127]))
    n = int(rng.choice([1, 1, 2, 3, 8, 9]))
    seed = int(rng.integers(0, 2**62))
    index_offset = int(rng.choice([0, 4, 8, 1, 6, 2**33 + 4, 2**34 + 3]))
    aligned = rng.random() < 0.6
    sh = (lambda: 0) if aligned else (lambda: int(rng.integers(0, 4)))
    scale = np.exp2(rng.uniform(-20, 5, size=d)).astype(np.float32) if rng.random() < 0.5 else np.float32(1e-2)
    offdev = None if offsets is None else dev(offsets)
    nseg = nc.segment_count(d, 0 if offsets is None else offsets.size - 1, bucket, offsets is not None)
    cb, sb = nc.dither_code_bytes(d, s), nc.dither_sign_bytes(d, s)
    pad = 0 if aligned else int(rng.integers(1, 4))
    norms_all = torch.zeros((n, nseg + pad), dtype=torch.float32, device="cuda")
    code_all = torch.zeros((n, nc.plane_stride(cb) + pad), dtype=torch.uint8, device="cuda")
    sign_all = torch.zeros((n, nc.plane_stride(max(sb, 1)) + pad), dtype=torch.uint8, device="cuda")
    xs = []
    for w in range(n):
        x = (rng.laplace(0, 1, d).astype(np.float32) * scale).astype(np.float32)
        if rng.random() < 0.3:
            x[rng.integers(0, d, size=max(d // 50, 1))] = 0.0
        xs.append(x)
        xdev = shifted(d, sh(), torch.float32)
        xdev.copy_(torch.from_numpy(x))
        nc.dither_encode(xdev, p, s, seed, worker=w, index_offset=index_offset, seg_offsets=offdev, bucket=bucket,
                         norms_out=norms_all[w, :nseg], code_out=code_all[w, :cb],
                         sign_out=sign_all[w, :sb] if sb else None)
    torch.cuda.synchronize()
    norms_h, code_h, sign_h = host(norms_all)[:, :nseg].copy(), host(code_all), host(sign_all)
    for w in range(n):
        ref = oracle.pnorm_segments(xs[w], p, offsets=offsets, bucket=bucket)
        assert np.all(np.abs(norms_h[w] - ref) <= 1e-5 * np.abs(ref)), (case, "norms", w)
        co, so = oracle.dither_encode(xs[w], s, norms_h[w], seed, w, index_offset, offsets=offsets, bucket=bucket)
        assert np.array_equal(code_h[w, :cb], co), (case, "codes", w, np.flatnonzero(code_h[w, :cb] != co)[:5])
        if sb:
            assert np.array_equal(sign_h[w, :sb], so), (case, "signs", w)
    out = shifted(d, sh(), torch.float32)
    nc.dither_decode(norms_all[0, :nseg].contiguous(), code_all[0, :cb], sign_all[0, :sb] if sb else None, d, s,
                     seg_offsets=offdev, bucket=bucket, out=out)
    yo = oracle.dither_decode(norms_h[0], code_h[0, :cb].copy(), sign_h[0, :sb].copy() if sb else None, d, s,
                              offsets=offsets, bucket=bucket)
    assert np.array_equal(host(out).view(np.uint32), yo.view(np.uint32)), (case, "decode")
    total = shifted(d, sh(), torch.float32)
    nc.aggregate_sum(nc.NC_KIND_DITHER, d, code_all, sign_all if sb else None, norms_all, s=s, seg_offsets=offdev,
                     bucket=bucket, out=total)
    _, o32, _ = oracle.aggregate_dither(norms_h, code_h, sign_h if sb else None, d, s, offsets=offsets, bucket=bucket)
    assert np.array_equal(host(total).view(np.uint32), o32.view(np.uint32)), (case, "sum")


@pytest.mark.parametrize("case", range(40))
def test_nat_and_clip(nc, oracle, case):
    rng = np.random.default_rng(9000 + case)
    d = int(rng.choice([rng.integers(1, 300), rng.integers(300, 20_000), rng.integers(20_000, 120_000)]))
    n = int(rng.choice([1, 2, 3, 8, 9, 17]))
    seed = int(rng.integers(0, 2**62))
    index_offset = int(rng.choice([0, 4, 1, 6, 2**33 + 4, 2**34 + 3]))
    aligned = rng.random() < 0.6
    pad = 0 if aligned else int(rng.integers(1, 8))
    xs = (rng.laplace(0, 1, (n, d)) * np.exp2(rng.uniform(-60, 20, (n, d)))).astype(np.float32)
    xdev = torch.zeros((n, d + pad), dtype=torch.float32, device="cuda")
    xdev[:, :d] = torch.from_numpy(xs)
    exp = torch.zeros((n, nc.plane_stride(d) + pad), dtype=torch.uint8, device="cuda")
    sign = torch.zeros((n, nc.plane_stride(nc.sign_bytes(d)) + pad), dtype=torch.uint8, device="cuda")
    clip = torch.zeros((n, nc.plane_stride(d) + pad), dtype=torch.uint8, device="cuda")
    nc.nat_encode_batch(xdev, seed, first_worker=2, index_offset=index_offset, exp_out=exp, sign_out=sign, d=d)
    nc.nat_clip_encode(xdev, seed, first_worker=2, index_offset=index_offset, code_out=clip, d=d)
    torch.cuda.synchronize()
    nsb = nc.sign_bytes(d)
    eh, sh_, ch = host(exp), host(sign), host(clip)
    for w in range(n):
        eo, so = oracle.nat_encode(xs[w], seed, 2 + w, index_offset)
        assert np.array_equal(eh[w, :d], eo) and np.array_equal(sh_[w, :nsb], so), (case, w)
        assert np.array_equal(ch[w, :d], oracle.clip_encode(xs[w], seed, 2 + w, index_offset)), (case, w)
    total = nc.aggregate_sum(nc.NC_KIND_NAT, d, exp, sign)
    _, o32, _ = oracle.aggregate_nat(eh, sh_, d)
    assert np.array_equal(host(total).view(np.uint32), o32.view(np.uint32)), (case, "sum")
    me, ms = nc.master_nat(d, exp, sign, seed + 1, master=5, index_offset=index_offset)
    _, meo, mso = oracle.master_nat(eh, sh_, d, seed + 1, 5, index_offset)
    assert np.array_equal(host(me), meo) and np.array_equal(host(ms), mso), (case, "master")
    sums, ce, cs = nc.clip_aggregate_int(clip, d, seed + 2, master=1, index_offset=index_offset, want_sum=True)
    so_, ceo, cso = oracle.clip_aggregate(ch, d, seed + 2, 1, index_offset)
    assert np.array_equal(host(sums), so_) and np.array_equal(host(ce), ceo) and np.array_equal(host(cs), cso), (case, "int")
