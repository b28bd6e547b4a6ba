"""The entry points inside a captured HIP graph (a serving loop's way of calling them): every launch
goes to the caller's stream and nothing is allocated or cleared with a memset, so a capture of the
calls replays to the same bytes as the eager calls.  Each graph is replayed several times with eager
work and synchronisation in between, on outputs overwritten before every replay, and every replay is
compared with the eager result (itself checked against the oracle)."""
import math

import numpy as np
import pytest
import torch

from gpu_util import dev, host

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


def capture(step, warm=True):
    """Captures step() on a side stream (after one eager run there, which torch asks for)."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        if warm:
            step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    return graph


def replay_and_compare(graph, outputs, expected, rounds=3):
    for r in range(rounds):
        for o in outputs:
            o.fill_(0x5A if o.dtype == torch.uint8 else 123)      # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for o, e in zip(outputs, expected):
            assert torch.equal(o.view(torch.uint8), e.view(torch.uint8)), r


def test_nat_step_in_a_graph(nc, oracle, wl):
    n, d = 8, 300_003
    rows = np.stack([wl.dense_gaussian(w, d=d, seed=3) for w in range(n)])
    x = dev(rows)
    exp_e, sign_e = nc.nat_encode_batch(x, seed=11)
    out_e = nc.aggregate_sum(nc.NC_KIND_NAT, d, exp_e, sign_e)
    torch.cuda.synchronize()
    eo, so = oracle.nat_encode(rows[3], 11, worker=3)
    assert np.array_equal(host(exp_e)[3, :d], eo) and np.array_equal(host(sign_e)[3, : so.size], so)
    exp_g, sign_g, out_g = torch.empty_like(exp_e), torch.empty_like(sign_e), torch.empty_like(out_e)

    def step():
        nc.nat_encode_batch(x, seed=11, exp_out=exp_g, sign_out=sign_g)
        nc.aggregate_sum(nc.NC_KIND_NAT, d, exp_g, sign_g, out=out_g)

    graph = capture(step)
    # the padding between the workers' planes is never written: compare what the planes hold
    replay_and_compare(graph, [out_g], [out_e])
    assert torch.equal(exp_g[:, :d], exp_e[:, :d]) and torch.equal(sign_g[:, : (d + 7) // 8], sign_e[:, : (d + 7) // 8])


def test_layered_dithering_in_a_graph(nc, oracle, wl):
    """The three-launch encoder on the library's own scratch array (the entry point for callers
    that cannot allocate) and the decoder."""
    d = 700_001
    off = wl.layer_offsets(d=d, num_layers=37, lo=64, hi=90_000, seed=4)
    offdev = dev(off.view(np.int64))
    nseg = off.size - 1
    xh = wl.dense_gaussian(0, d=d, seed=9)
    x = dev(xh)
    nc.static_scratch_init()
    mk = lambda nbytes: torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    norms_e, code_e, sign_e = torch.empty(nseg, dtype=torch.float32, device="cuda"), mk(nc.dither_code_bytes(d, 8)), mk(nc.dither_sign_bytes(d, 8))
    nc.dither_encode_static(x, 2, 8, 5, norms_e, code_e, sign_e, seg_offsets=offdev)
    out_e = nc.dither_decode(norms_e, code_e, sign_e, d, 8, seg_offsets=offdev)
    torch.cuda.synchronize()
    co, so = oracle.dither_encode(xh, 8, host(norms_e), 5, 0, 0, offsets=off)
    assert np.array_equal(host(code_e), co) and np.array_equal(host(sign_e), so)
    norms_g, code_g, sign_g, out_g = (torch.empty_like(t) for t in (norms_e, code_e, sign_e, out_e))

    def step():
        nc.dither_encode_static(x, 2, 8, 5, norms_g, code_g, sign_g, seg_offsets=offdev)
        nc.dither_decode(norms_g, code_g, sign_g, d, 8, seg_offsets=offdev, out=out_g)

    graph = capture(step)
    replay_and_compare(graph, [norms_g, code_g, sign_g, out_g], [norms_e, code_e, sign_e, out_e])


def test_partitioned_sparse_sum_in_a_graph(nc, oracle, wl):
    """Seven launches on one workspace, whose contents no launch expects to find cleared."""
    n, d, k = 5, 900_007, 60_000
    rows = np.stack([wl.dense_gaussian(w, d=d, seed=21) for w in range(n)])
    idx, exp, sign = nc.sparse_nat_encode_batch(dev(rows), k, np.float32(d / k), seed=2)
    ws = torch.randint(0, 256, (nc.sparse_aggregate_workspace_bytes(n, k, d),), dtype=torch.uint8, device="cuda")
    out_e = nc.sparse_nat_aggregate(idx, exp, sign, k, d)
    torch.cuda.synchronize()
    o32, _, _ = oracle.sparse_nat_aggregate(host(idx).view(np.uint32), host(exp), host(sign), k, d)
    assert np.array_equal(host(out_e).view(np.uint32), o32.view(np.uint32))
    out_g = torch.empty_like(out_e)

    def step():
        nc.sparse_nat_aggregate_ws(idx, exp, sign, k, d, out=out_g, workspace=ws)

    graph = capture(step)
    for r in range(3):
        ws.random_(0, 256)                      # garbage in the workspace before every replay
        replay_and_compare(graph, [out_g], [out_e], rounds=1)
