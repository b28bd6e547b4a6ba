"""GPU parity of C_nat o S^k and its dense scatter-sum: indices, exponent and sign planes
bit-exact with the oracle; the dense binary32 sum bit-exact with the oracle's worker-ordered
binary32 sum and within 1e-5 * sum|v| of its double sum.  Both forms of the sum (one scatter
per worker; entries partitioned by output tile in a workspace) take every aggregate test."""
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


@pytest.fixture(params=["scatter", "partitioned"])
def aggregate(request, nc):
    """The entry point under test; the partitioned form gets a workspace full of garbage."""
    if request.param == "scatter":
        return nc.sparse_nat_aggregate

    def run(idx, exp, sign, k, d, out=None):
        need = nc.sparse_aggregate_workspace_bytes(idx.shape[0], k, d)
        assert need > 0
        ws = torch.randint(0, 256, (need,), dtype=torch.uint8, device="cuda")
        return nc.sparse_nat_aggregate_ws(idx, exp, sign, k, d, out=out, workspace=ws)
    return run


def check_message(nc, oracle, x, k, scale, seed, worker):
    idx, exp, sign = nc.sparse_nat_encode(dev(x), k, scale, seed, worker)
    torch.cuda.synchronize()
    io, eo, so = oracle.sparse_nat_encode(x, k, scale, seed, worker)
    assert np.array_equal(host(idx).view(np.uint32), io)
    assert np.array_equal(host(exp), eo)
    assert np.array_equal(host(sign), so)
    return idx, exp, sign


@pytest.mark.parametrize("d,k", [(1, 1), (2, 1), (7, 7), (8, 8), (9, 5), (1000, 10), (1000, 1000), (4099, 333),
                                 (65536, 655), (65537, 8193), (1_000_003, 10_001)])
def test_messages_match_oracle(nc, oracle, wl, d, k):
    x = wl.dense_gaussian(0, d=d, seed=d + k)
    for seed, worker in ((0, 0), (12345678901234, 5)):
        check_message(nc, oracle, x, k, np.float32(d / k), seed, worker)


def test_k_equal_d_reproduces_dense_codes(nc, oracle, wl):
    """S^d is the identity: with k = d and scale 1 the sparse message is the dense C_nat code in
    permuted order (same random word per dense position)."""
    d = 20011
    x = wl.config1(d=d, seed=6)
    idx, exp, sign = check_message(nc, oracle, x, d, 1.0, 9, 2)
    e_dense, s_dense = nc.nat_encode(dev(x), 9, worker=2)
    i = host(idx).astype(np.int64)
    assert sorted(i.tolist()) == list(range(d))
    assert np.array_equal(host(exp), host(e_dense)[i])
    sd = np.unpackbits(host(s_dense), bitorder="little")[:d]
    assert np.array_equal(np.unpackbits(host(sign), bitorder="little")[:d], sd[i])


@pytest.mark.parametrize("n", [1, 2, 8, 11])
def test_batch_and_aggregate(nc, oracle, wl, aggregate, n):
    d, k = 50_003, 5_001
    rows = np.stack([wl.dense_gaussian(w, d=d, seed=77) for w in range(n)])
    scale = np.float32(d / k)
    idx, exp, sign = nc.sparse_nat_encode_batch(dev(rows), k, scale, seed=3)
    out = Guarded(d, torch.float32)
    aggregate(idx, exp, sign, k, d, out=out.t)
    torch.cuda.synchronize()
    got = out.check()
    ih, eh, sh = host(idx).view(np.uint32), host(exp), host(sign)
    for w in range(n):
        io, eo, so = oracle.sparse_nat_encode(rows[w], k, scale, 3, w)
        assert np.array_equal(ih[w, :k], io) and np.array_equal(eh[w, :k], eo)
        assert np.array_equal(sh[w, : so.size], so)
    o32, o64, oa = oracle.sparse_nat_aggregate(ih, eh, sh, k, d)
    assert np.array_equal(got.view(np.uint32), o32.view(np.uint32))
    assert np.all(np.abs(got.astype(np.float64) - o64) <= 1e-5 * oa)


@pytest.mark.parametrize("n,d,k", [(3, 8192, 8192), (16, 8191, 4000), (5, 3 * 8192 + 1, 9000), (2, 100_000, 1),
                                   (33, 20_000, 19_999)])
def test_sum_with_many_collisions(nc, oracle, wl, aggregate, n, d, k):
    """k close to d and magnitudes 1e8 apart between workers: almost every output element receives
    several workers' entries and the order of the binary32 additions decides the result."""
    rows = np.stack([wl.dense_gaussian(w, d=d, seed=91) * np.float32(10.0 ** (2 * (w % 5))) for w in range(n)])
    idx, exp, sign = nc.sparse_nat_encode_batch(dev(rows), k, 1.0, seed=4)
    o32, _, _ = oracle.sparse_nat_aggregate(host(idx).view(np.uint32), host(exp), host(sign), k, d)
    out = Guarded(d, torch.float32)
    aggregate(idx, exp, sign, k, d, out=out.t)
    torch.cuda.synchronize()
    assert np.array_equal(out.check().view(np.uint32), o32.view(np.uint32))


def test_unaligned_output_and_tiny_sizes(nc, oracle, wl, aggregate):
    d, k, n = 1001, 77, 3
    rows = np.stack([wl.dense_gaussian(w, d=d, seed=5) for w in range(n)])
    idx, exp, sign = nc.sparse_nat_encode_batch(dev(rows), k, 13.0, seed=8)
    buf = torch.full((d + 3,), 7.0, dtype=torch.float32, device="cuda")
    aggregate(idx, exp, sign, k, d, out=buf[1: d + 1])
    got = host(buf)
    assert got[0] == 7.0 and got[d + 1] == 7.0 and got[d + 2] == 7.0
    o32, _, _ = oracle.sparse_nat_aggregate(host(idx).view(np.uint32), host(exp), host(sign), k, d)
    assert np.array_equal(got[1: d + 1].view(np.uint32), o32.view(np.uint32))


@pytest.mark.parametrize("n,d,k", [(3, 5_000_011, 50_000), (2, 2_097_153, 2_000_000), (8, 1, 1), (1, 8193, 8193)])
def test_sum_over_several_coarse_bins(nc, oracle, wl, aggregate, n, d, k):
    """Vectors longer than 256 tiles (several tiles per coarse bin), a last tile and a last coarse
    bin that are not full, and the smallest sizes."""
    rows = np.stack([wl.dense_gaussian(w, d=d, seed=17) for w in range(n)])
    idx, exp, sign = nc.sparse_nat_encode_batch(dev(rows), k, np.float32(d / k), seed=6)
    out = Guarded(d, torch.float32)
    aggregate(idx, exp, sign, k, d, out=out.t)
    torch.cuda.synchronize()
    o32, _, _ = oracle.sparse_nat_aggregate(host(idx).view(np.uint32), host(exp), host(sign), k, d, only32=True)
    assert np.array_equal(out.check().view(np.uint32), o32.view(np.uint32))


def test_indices_past_the_end_are_ignored(nc, oracle, aggregate):
    """Hand-made messages: some indices >= d (ignored by the definition of the sum), rows longer than k."""
    rng = np.random.default_rng(5)
    n, d, k, row = 4, 30_000, 2_000, 2_048
    ih = np.zeros((n, row), dtype=np.uint32)
    for w in range(n):
        ih[w, :k] = rng.permutation(2 * d)[:k]          # about half of them past the end
    ih[:, k:] = 7                                         # beyond k: not part of the message
    eh = rng.integers(100, 140, (n, row), dtype=np.uint8)
    sh = rng.integers(0, 256, (n, row // 8), dtype=np.uint8)
    out = Guarded(d, torch.float32)
    aggregate(dev(ih.view(np.int32)), dev(eh), dev(sh), k, d, out=out.t)
    torch.cuda.synchronize()
    # the oracle's sum over 2d positions, cut to the first d: entries past d do not touch them
    o32, _, _ = oracle.sparse_nat_aggregate(ih, eh, sh, k, 2 * d)
    assert np.array_equal(out.check().view(np.uint32), o32[:d].view(np.uint32))


@pytest.mark.parametrize("d", [600_000_011, 2 ** 32 - 5])
def test_sum_at_the_largest_sizes(nc, oracle, aggregate, d):
    """d beyond 2^29 (more than 256 tiles per coarse bin) and just below 2^32 (2048 tiles per bin):
    hand-made messages with planted collisions, entries on the first and last positions and on
    tile borders.  The sum at a position depends only on the entries with that index, so the
    oracle runs on the indices renumbered 0, 1, ... in ascending order; every other position of
    the output must hold +0.0."""
    rng = np.random.default_rng(d % 1000)
    n, k = 3, 150_000
    ih = np.zeros((n, k), dtype=np.uint32)
    for w in range(n):
        pool = np.unique(rng.integers(0, d, size=2 * k, dtype=np.int64))
        rng.shuffle(pool)
        ih[w] = pool[:k].astype(np.uint32)
    special = np.array([0, 1, 8191, 8192, 8193, d - 1, d - 2, d - 8193, (d >> 13) << 13], dtype=np.int64)
    for w in range(n):                       # planted: the special positions and 2000 of worker 0's
        row = ih[w].astype(np.int64)
        plant = special if w == 0 else np.concatenate([special, ih[0, 100:2100].astype(np.int64)])
        keep = row[~np.isin(row, plant)]
        ih[w] = np.concatenate([plant, keep])[:k].astype(np.uint32)
        assert np.unique(ih[w]).size == k
    eh = rng.integers(90, 150, (n, k), dtype=np.uint8)
    sh = rng.integers(0, 256, (n, (k + 7) // 8), dtype=np.uint8)
    out = aggregate(dev(ih.view(np.int32)), dev(eh), dev(sh), k, d)
    torch.cuda.synchronize()
    positions, compact = np.unique(ih, return_inverse=True)
    o32, _, _ = oracle.sparse_nat_aggregate(compact.reshape(n, k).astype(np.uint32), eh, sh, k, positions.size)
    got = host(out[torch.from_numpy(positions.astype(np.int64)).cuda()])
    assert np.array_equal(got.view(np.uint32), o32.view(np.uint32))
    nonzero_words = int((out.view(torch.int32) != 0).sum())
    assert nonzero_words == int(np.count_nonzero(o32.view(np.uint32)))


def test_partitioned_sum_reuses_its_workspace(nc, oracle, wl):
    """Two calls in a row on one workspace, the second on a smaller problem."""
    ws = torch.empty(nc.sparse_aggregate_workspace_bytes(5, 40_000, 400_009), dtype=torch.uint8, device="cuda")
    for n, d, k, seed in ((5, 400_009, 40_000, 1), (2, 100_003, 999, 2)):
        rows = np.stack([wl.dense_gaussian(w, d=d, seed=seed) for w in range(n)])
        idx, exp, sign = nc.sparse_nat_encode_batch(dev(rows), k, np.float32(d / k), seed=seed)
        got = nc.sparse_nat_aggregate_ws(idx, exp, sign, k, d, workspace=ws)
        torch.cuda.synchronize()
        o32, _, _ = oracle.sparse_nat_aggregate(host(idx).view(np.uint32), host(exp), host(sign), k, d)
        assert np.array_equal(host(got).view(np.uint32), o32.view(np.uint32))


def test_partitioned_sum_argument_errors(nc):
    idx = torch.zeros((2, 16), dtype=torch.int32, device="cuda")
    exp = torch.zeros((2, 16), dtype=torch.uint8, device="cuda")
    sign = torch.zeros((2, 2), dtype=torch.uint8, device="cuda")
    need = nc.sparse_aggregate_workspace_bytes(2, 16, 100)
    assert need > 0
    with pytest.raises(nc.NatcompError, match="WORKSPACE"):
        nc.sparse_nat_aggregate_ws(idx, exp, sign, 16, 100, workspace=torch.empty(need - 1, dtype=torch.uint8, device="cuda"))
    assert nc.sparse_aggregate_workspace_bytes(65536, 16, 100) == 0      # more workers than the entry point takes
    assert nc.sparse_aggregate_workspace_bytes(8, 2 ** 29, 2 ** 32) == 0   # 2^32 entries
    assert nc.sparse_aggregate_workspace_bytes(2, 101, 100) == 0         # k > d


def test_argument_errors(nc):
    x = torch.zeros(100, dtype=torch.float32, device="cuda")
    with pytest.raises(nc.NatcompError, match="INVALID"):
        nc.sparse_nat_encode(x, 101, 1.0, 0)


def test_config5_full_size_two_workers(nc, oracle, wl, aggregate):
    """Config 5 at its full d = 335,000,000 and k = d/100, two of the eight workers: messages in
    full against the oracle, and the whole dense sum against the oracle's."""
    d = wl.D_BERT_LARGE
    k = d // 100
    n = 2
    scale = np.float32(d / k)
    xdev = torch.empty((n, d), dtype=torch.float32, device="cuda")
    xs = []
    for w in range(n):
        x = wl.dense_gaussian(w)
        xs.append(x)
        xdev[w] = torch.from_numpy(x).cuda()
    idx, exp, sign = nc.sparse_nat_encode_batch(xdev, k, scale, seed=0)
    out = aggregate(idx, exp, sign, k, d)
    torch.cuda.synchronize()
    ih, eh, sh = host(idx).view(np.uint32), host(exp), host(sign)
    for w in range(n):
        io, eo, so = oracle.sparse_nat_encode(xs[w], k, scale, 0, w)
        assert np.array_equal(ih[w, :k], io) and np.array_equal(eh[w, :k], eo)
        assert np.array_equal(sh[w, : so.size], so)
    del xs
    o32, _, _ = oracle.sparse_nat_aggregate(ih, eh, sh, k, d, only32=True)
    got = host(out)
    assert np.array_equal(got.view(np.uint32), o32.view(np.uint32))
    assert np.count_nonzero(got) > 2 * k * 0.98
