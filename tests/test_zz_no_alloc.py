"""The entry point that allocates nothing: nc_dither_encode_static keeps its scratch memory in a
static device array instead of a caller workspace.  Its outputs must equal nc_dither_encode's bit
for bit, on two calls in a row, the second with a smaller input (the array still holds the first
call's contents), and a description that does not fit the array must be refused."""
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
    natcomp.static_scratch_init()     # set-up: the runtime places the static array in device memory here, once
    return natcomp


@pytest.fixture(scope="module")
def wl():
    from paper_1905_10988_amd import workloads
    return workloads


def both_ways(nc, x, p, s, seed, worker, offsets=None, bucket=0):
    """(norms, code, sign) of the workspace entry point and of the static one, as host arrays."""
    d = x.numel()
    offdev = None if offsets is None else dev(offsets)
    count = nc.segment_count(d, 0 if offsets is None else offsets.size - 1, bucket, offsets is not None)
    ref = nc.dither_encode(x, p, s, seed, worker=worker, seg_offsets=offdev, bucket=bucket)
    norms, code = Guarded(count, torch.float32), Guarded(nc.dither_code_bytes(d, s))
    sign = Guarded(nc.dither_sign_bytes(d, s))
    free_before = torch.cuda.mem_get_info()[0]
    nc.dither_encode_static(x, p, s, seed, norms.t, code.t, sign.t if sign.n else None, worker=worker,
                            seg_offsets=offdev, bucket=bucket)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free_before, "the static entry point changed the amount of free device memory"
    got = (norms.check(), code.check(), sign.check() if sign.n else None)
    want = (host(ref[0]), host(ref[1]), None if ref[2] is None else host(ref[2]))
    return got, want


@pytest.mark.parametrize("p,s", [(2, 8), (float("inf"), 4), (1, 20)])
def test_static_scratch_matches_workspace_twice(nc, wl, p, s):
    cases = [(300_007, 23, 11), (70_001, 9, 12)]          # the second call is smaller than the first
    for d, layers, seed in cases:
        off = wl.layer_offsets(d=d, num_layers=layers, lo=64, hi=d // 2, seed=seed)
        x = dev(wl.layered_laplace(3, off, seed=seed))
        got, want = both_ways(nc, x, p, s, seed=5, worker=2, offsets=off)
        for g, w, name in zip(got, want, ("norms", "code", "sign")):
            if w is not None:
                assert np.array_equal(g.view(np.uint8), w.view(np.uint8)), f"{name} differ (d={d}, p={p}, s={s})"


def test_static_scratch_other_segment_descriptions(nc, wl):
    x = dev(wl.config1(d=100_003, seed=4))
    for bucket in (0, 1000, 12345, 512):                   # one segment, buckets on the two-pass path, one-pass buckets
        got, want = both_ways(nc, x, 2, 8, seed=9, worker=1, bucket=bucket)
        for g, w in zip(got, want):
            if w is not None:
                assert np.array_equal(g.view(np.uint8), w.view(np.uint8)), f"bucket={bucket}"


def test_static_scratch_rejects_what_does_not_fit(nc):
    """A description whose workspace exceeds the static array is an error, and nothing runs."""
    limit = nc.static_scratch_bytes()
    d = 64
    nseg = limit // 8                                      # 12 bytes per segment and more: beyond the array
    assert nc.dither_workspace_bytes(d, nseg, 0, True) > limit
    off = torch.zeros(nseg + 1, dtype=torch.int64, device="cuda")
    off[-1] = d
    x = torch.ones(d, dtype=torch.float32, device="cuda")
    norms = torch.full((nseg,), 7.0, dtype=torch.float32, device="cuda")
    code = torch.full((nc.dither_code_bytes(d, 8),), 0xEE, dtype=torch.uint8, device="cuda")
    sign = torch.full((nc.dither_sign_bytes(d, 8),), 0xEE, dtype=torch.uint8, device="cuda")
    with pytest.raises(nc.NatcompError, match="NC_ERR_WORKSPACE"):
        nc.dither_encode_static(x, 2, 8, 0, norms, code, sign, seg_offsets=off)
    torch.cuda.synchronize()
    assert bool((code == 0xEE).all()) and bool((norms == 7.0).all())
