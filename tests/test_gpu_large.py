"""GPU parity beyond 2^32 elements: one vector of d = 2^32 + 12,301 fp32 (17 GB) goes through the
C_nat, clipped-byte and bucketed D_nat kernels; slices at the start, across the 2^32 boundary and at
the ragged end are compared bit for bit with the oracle, which can compute any slice on its own
because every random word depends on the element's global index only (index_offset)."""
import math

import numpy as np
import pytest
import torch

from gpu_util import dev, host

pytestmark = pytest.mark.gpu

D = 2**32 + 12_301
BUCKET = 8192
SLICE = 3 * BUCKET                                    # slice length (whole buckets, multiple of 8)


def slice_starts():
    """Start of the vector, a slice that crosses element 2^32, and everything from 2^32 to the ragged end."""
    return [0, 2**32 - 2 * BUCKET, 2**32]


@pytest.fixture(scope="module")
def nc():
    from paper_1905_10988_amd import natcomp
    natcomp.lib()
    assert torch.cuda.is_available()
    return natcomp


@pytest.fixture(scope="module")
def big():
    free, _ = torch.cuda.mem_get_info()
    if free < 100 * 2**30:
        pytest.skip("needs 100 GB of free device memory")
    g = torch.Generator(device="cuda")
    g.manual_seed(99)
    x = torch.empty(D, dtype=torch.float32, device="cuda")
    x.normal_(generator=g)
    x *= 1e-2
    out = torch.empty(D, dtype=torch.float32, device="cuda")
    yield x, out
    del x, out
    torch.cuda.empty_cache()


def test_nat_encode_decode_sum(nc, oracle, big):
    x, out = big
    planes = []
    for w in (0, 1):
        e, s = nc.nat_encode(x, 11, worker=w)
        planes.append((e, s))
    nc.nat_decode(planes[0][0], planes[0][1], D, out=out)
    torch.cuda.synchronize()
    for b in slice_starts():
        n = min(SLICE, D - b)
        xs = host(x[b: b + n])
        for w in (0, 1):
            eo, so = oracle.nat_encode(xs, 11, w, index_offset=b)
            assert np.array_equal(host(planes[w][0][b: b + n]), eo), (b, w)
            assert np.array_equal(host(planes[w][1][b // 8: b // 8 + (n + 7) // 8]), so), (b, w)
        eo, so = oracle.nat_encode(xs, 11, 0, index_offset=b)
        assert np.array_equal(host(out[b: b + n]).view(np.uint32), oracle.nat_decode(eo, so, n).view(np.uint32))
    exp2 = torch.stack([planes[0][0], planes[1][0]])
    sign2 = torch.stack([planes[0][1], planes[1][1]])
    nc.aggregate_sum(nc.NC_KIND_NAT, D, exp2, sign2, out=out)
    torch.cuda.synchronize()
    for b in slice_starts():
        n = min(SLICE, D - b)
        e2 = host(exp2[:, b: b + n])
        s2 = host(sign2[:, b // 8: b // 8 + (n + 7) // 8])
        _, o32, _ = oracle.aggregate_nat(e2, s2, n)
        assert np.array_equal(host(out[b: b + n]).view(np.uint32), o32.view(np.uint32)), b


def test_clip_encode_and_integer_sum(nc, oracle, big):
    x, _ = big
    code = torch.empty((2, nc.plane_stride(D)), dtype=torch.uint8, device="cuda")
    for w in (0, 1):
        nc.nat_clip_encode(x, 12, first_worker=w, code_out=code[w, :D])
    sums, e, s = nc.clip_aggregate_int(code, D, 13, master=0, want_sum=True)
    torch.cuda.synchronize()
    for b in slice_starts():
        n = min(SLICE, D - b)
        xs = host(x[b: b + n])
        want = np.stack([oracle.clip_encode(xs, 12, w, index_offset=b) for w in (0, 1)])
        assert np.array_equal(host(code[:, b: b + n]), want), b
        so, eo, sgo = oracle.clip_aggregate(want, n, 13, 0, index_offset=b)
        assert np.array_equal(host(sums[b: b + n]), so)
        assert np.array_equal(host(e[b: b + n]), eo)
        assert np.array_equal(host(s[b // 8: b // 8 + (n + 7) // 8]), sgo)


@pytest.mark.parametrize("p,s,bucket", [(math.inf, 4, BUCKET), (2, 8, 512)])
def test_dither_buckets(nc, oracle, big, p, s, bucket):
    x, out = big
    nseg = nc.segment_count(D, 0, bucket, False)
    norms = torch.empty(nseg, dtype=torch.float32, device="cuda")
    code = torch.empty(nc.dither_code_bytes(D, s), dtype=torch.uint8, device="cuda")
    sign = torch.empty(max(nc.dither_sign_bytes(D, s), 1), dtype=torch.uint8, device="cuda")
    nc.dither_encode(x, p, s, 14, worker=2, bucket=bucket, norms_out=norms, code_out=code, sign_out=sign)
    nc.dither_decode(norms, code, sign, D, s, bucket=bucket, out=out)
    torch.cuda.synchronize()
    nsign = nc.dither_sign_bytes(D, s)
    for b in slice_starts():
        n = min(SLICE, D - b)
        xs = host(x[b: b + n])
        nb = -(-n // bucket)
        gn = host(norms[b // bucket: b // bucket + nb])
        ref = oracle.pnorm_segments(xs, p, bucket=bucket)
        assert np.all(np.abs(gn - ref) <= 1e-5 * np.abs(ref))
        co, so = oracle.dither_encode(xs, s, gn, 14, 2, index_offset=b, bucket=bucket)
        assert np.array_equal(host(code[b // 2: b // 2 + co.size]), co), b
        if nsign:
            assert np.array_equal(host(sign[b // 8: b // 8 + so.size]), so), b
        yo = oracle.dither_decode(gn, co, so if nsign else None, n, s, bucket=bucket)
        assert np.array_equal(host(out[b: b + n]).view(np.uint32), yo.view(np.uint32)), b


def test_dither_layer_offsets(nc, oracle, big):
    """The two-pass path (segment offsets) on the same vector: a 4.29 G-element segment whose norm
    is finished from half a million partials, segment boundaries next to element 2^32, and a ragged
    last segment."""
    x, out = big
    p, s = 2, 8
    a0, a1, a2 = 2**32 - 2 * BUCKET, 2**32 + BUCKET, D
    off = np.array([0, SLICE, a0, a0 + 1000, 2**32 + 5, a1, a2], np.uint64)
    nseg = off.size - 1
    offdev = dev(off)
    norms = torch.empty(nseg, dtype=torch.float32, device="cuda")
    code = torch.empty(nc.dither_code_bytes(D, s), dtype=torch.uint8, device="cuda")
    sign = torch.empty(nc.dither_sign_bytes(D, s), dtype=torch.uint8, device="cuda")
    nc.dither_encode(x, p, s, 15, worker=1, seg_offsets=offdev, norms_out=norms, code_out=code, sign_out=sign)
    nc.dither_decode(norms, code, sign, D, s, seg_offsets=offdev, out=out)
    torch.cuda.synchronize()
    gn = host(norms)
    big_norm = float(torch.linalg.vector_norm(x[SLICE:a0], dtype=torch.float64))
    assert abs(gn[1] - big_norm) <= 1e-5 * big_norm
    for b, e, first_seg in [(0, SLICE, 0), (a0, a1, 2), (a1, a2, 5)]:
        n = e - b
        xs = host(x[b:e])
        local = (off[(off >= b) & (off <= e)] - np.uint64(b)).astype(np.uint64)
        seg_norms = gn[first_seg: first_seg + local.size - 1]
        ref = oracle.pnorm_segments(xs, p, offsets=local)
        assert np.all(np.abs(seg_norms - ref) <= 1e-5 * np.abs(ref))
        co, so = oracle.dither_encode(xs, s, seg_norms, 15, 1, index_offset=b, offsets=local)
        assert np.array_equal(host(code[b // 2: b // 2 + co.size]), co), b
        assert np.array_equal(host(sign[b // 8: b // 8 + so.size]), so), b
        yo = oracle.dither_decode(seg_norms, co, so, n, s, offsets=local)
        assert np.array_equal(host(out[b:e]).view(np.uint32), yo.view(np.uint32)), b
