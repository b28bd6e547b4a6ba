"""Benchmark of the hot path on one MI355X.

A step is one pass of the headline workload ("config 2"): natural compression of 8 workers'
gradients (d = 25,557,032 fp32 each, 161 layers) in one batched launch, then the fused
decode-and-sum of the 8 code streams.  Inputs are resident in HBM before the timed region.
`value` is fp32 input bytes (8 * 4 * d) per second of step time.

Prints ONE JSON line with the metric, a `roofline` object for the dominant kernel (the
batched encoder), a `roofline_aggregate` object for the fused sum (also on rotated, cold code
sets) and a `cpu_baseline` object (the CPU oracle timed on the host cores).

Timing rules: HIP events on the launch stream around every kernel of every timed step (of
every k-th step when there are more than 64); median, minimum and mean are reported.  Kernels
timed on their own (the cold aggregate, the other configurations) take one event pair per four
consecutive launches, which spreads the 3 to 4 us the markers cost over the group.  Before
the warm-up steps the same step is run for a fixed wall time (`settle_ms`, its step count is
printed as `settle_steps`) so that the clocks have left their idle state; the timed region is
still exactly `--steps` steps after `--warmup` further untimed ones.  Kernels whose working
set would fit the 256 MB last-level cache are timed round-robin over several buffer sets
that together exceed 512 MB.
"""
import argparse
import ctypes
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
ENCODE_BYTES_PER_ELEM = 4 + 1 + 1 / 8            # read fp32, write exponent byte + sign bit
ROTATE_BYTES = 600e6                             # buffer sets of a rotated timing cover at least this much


def aggregate_bytes_per_elem(n):
    return n * (1 + 1 / 8) + 4                    # read n code streams, write fp32


def measured_traffic(name):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary, if there is one."""
    path = os.path.join(ROOT, "profiles", name)
    try:
        m = re.search(r"^traffic_bytes_per_launch:\s*([0-9.eE+]+)", open(path).read(), re.M)
        return float(m.group(1)) if m else None
    except OSError:
        return None


def sets_for(working_set_bytes):
    """How many distinct buffer sets a rotated timing needs for this working set."""
    return max(1, int(-(-ROTATE_BYTES // max(working_set_bytes, 1))))


class Timer:
    """HIP-event timing of launches on torch's current stream."""

    def __init__(self, torch, np, warm_ms=25.0):
        # warm_ms: a kernel is run for this long before it is timed; after a change of workload the clocks
        # take some 10 ms to settle (the first launches are fast, the next few dozen up to 30 % slower)
        self.torch, self.np, self.warm_ms = torch, np, warm_ms

    def stats(self, samples_ms):
        a = self.np.asarray(samples_ms, dtype=self.np.float64)
        return {"median": float(self.np.median(a)), "min": float(a.min()), "mean": float(a.mean()), "samples": int(a.size),
                "raw": [float(v) for v in a]}

    def rotating(self, fns, reps=20, warm=5, group=4):
        """fns[i % len(fns)]() is one launch (or group of launches) on buffer set i.  A sample is the
        time between two events around `group` consecutive calls (on consecutive buffer sets), divided
        by `group`: the cost of the event markers themselves, 3 to 4 us per pair, is spread over the
        group.  Returns the statistics over `reps` samples, in ms per call."""
        torch = self.torch
        t0, i = time.perf_counter(), 0
        while i < max(warm, group) or (time.perf_counter() - t0) * 1e3 < self.warm_ms:   # at least `warm` calls and warm_ms
            for _ in range(4):
                fns[i % len(fns)]()
                i += 1
            torch.cuda.synchronize()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        call = 0
        for a, b in evs:
            a.record()
            for _ in range(group):
                fns[call % len(fns)]()
                call += 1
            b.record()
        torch.cuda.synchronize()
        return self.stats([a.elapsed_time(b) / group for a, b in evs])


def _entry(st, alg_bytes, input_bytes, note, nsets):
    ms = st["median"]
    gbs = alg_bytes / (ms * 1e-3) / 1e9
    return {"ms": round(ms, 5), "min_ms": round(st["min"], 5), "mean_ms": round(st["mean"], 5),
            "algorithmic_GBps": round(gbs, 1), "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4),
            "fp32_input_GBps": round(input_bytes / (ms * 1e-3) / 1e9, 1), "algorithmic_bytes": alg_bytes,
            "buffer_sets": nsets, "note": note}


# ----------------------------------------------------------------------------------------------
# the device's own ceilings (bench-only kernels of libncprobe.so)
class Probe:
    def __init__(self, torch):
        path = os.path.join(ROOT, "paper_1905_10988_amd", "libncprobe.so")
        if not os.path.exists(path):
            raise RuntimeError(f"{path} is missing: run `python -m paper_1905_10988_amd.build` first")
        L = ctypes.CDLL(path)
        vp, u64, u32 = ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint32
        L.ncp_copy.argtypes = [vp, vp, u64, vp]
        L.ncp_read.argtypes = [vp, u64, vp, vp]
        L.ncp_fill.argtypes = [vp, u64, vp]
        L.ncp_mix94.argtypes = [vp, vp, vp, vp, u64, vp]
        L.ncp_philox.argtypes = [vp, u32, u32, vp]
        self.L, self.torch = L, torch

    def _s(self):
        return ctypes.c_void_p(self.torch.cuda.current_stream().cuda_stream)

    def ceilings(self, timer, nbytes=1 << 29):
        """GB/s of a streaming copy / read / fill / 9:4 mix over buffers of `nbytes` (rotated over
        enough sets to move more than 600 MB before one comes round again, far beyond the
        last-level cache), and Philox calls per second."""
        torch, L = self.torch, self.L
        nsets = max(2, -(-600_000_000 // nbytes))
        R = range(nsets)
        a = [torch.zeros(nbytes // 4, dtype=torch.int32, device="cuda") for _ in R]
        b = [torch.ones(nbytes // 4, dtype=torch.int32, device="cuda") for _ in R]
        c = [torch.ones(nbytes // 16, dtype=torch.int32, device="cuda") for _ in R]
        dst = [torch.empty(nbytes // 4, dtype=torch.int32, device="cuda") for _ in R]
        sink = torch.zeros(1024, dtype=torch.int32, device="cuda")

        def ok(rc):
            assert rc == 0, f"probe launch failed: {rc}"

        res = {}
        st = timer.rotating([lambda i=i: ok(L.ncp_copy(a[i].data_ptr(), dst[i].data_ptr(), nbytes, self._s())) for i in R])
        res["copy_kernel_GBps"] = round(2.0 * nbytes / (st["median"] * 1e-3) / 1e9, 1)
        st = timer.rotating([lambda i=i: ok(L.ncp_read(a[i].data_ptr(), nbytes, sink.data_ptr(), self._s())) for i in R])
        res["read_kernel_GBps"] = round(1.0 * nbytes / (st["median"] * 1e-3) / 1e9, 1)
        st = timer.rotating([lambda i=i: ok(L.ncp_fill(dst[i].data_ptr(), nbytes, self._s())) for i in R])
        res["fill_kernel_GBps"] = round(1.0 * nbytes / (st["median"] * 1e-3) / 1e9, 1)
        st = timer.rotating([lambda i=i: ok(L.ncp_mix94(a[i].data_ptr(), b[i].data_ptr(), c[i].data_ptr(), dst[i].data_ptr(),
                                                       nbytes, self._s())) for i in R])
        res["mix_9to4_kernel_GBps"] = round(3.25 * nbytes / (st["median"] * 1e-3) / 1e9, 1)
        if nbytes < 1 << 28:  # fits the last-level cache: what reading the same buffer again is worth
            st = timer.rotating([lambda: ok(L.ncp_read(a[0].data_ptr(), nbytes, sink.data_ptr(), self._s()))])
            res["read_kernel_same_buffer_GBps"] = round(1.0 * nbytes / (st["median"] * 1e-3) / 1e9, 1)
        if nbytes >= 1 << 29:
            st = timer.rotating([lambda: dst[0].copy_(a[0]), lambda: dst[1].copy_(a[1])])
            res["torch_copy_GBps"] = round(2.0 * nbytes / (st["median"] * 1e-3) / 1e9, 1)
            wgs, calls = 256 * 64, 512
            st = timer.rotating([lambda: ok(L.ncp_philox(sink.data_ptr(), wgs, calls, self._s()))], reps=10, warm=2)
            res["philox_Gcalls_per_s"] = round(wgs * 256 * calls / (st["median"] * 1e-3) / 1e9, 1)
        res["probe_bytes"] = nbytes
        return res


# ----------------------------------------------------------------------------------------------
def secondary_kernels(nc, wl, torch, np, timer):
    """The remaining kernels of the path, each on its configuration's shape (not part of `value`).
    Kernels at d = 25.6 M rotate over enough buffer sets to exceed the last-level cache; the
    launches of configurations 4 and 5 move more than 1 GB each and need no rotation."""
    import math
    res = {}
    d = wl.D_RESNET50
    off = wl.layer_offsets()
    offdev = torch.from_numpy(off.view(np.int64)).cuda()
    nseg = off.size - 1
    n = wl.NUM_WORKERS

    # ---- config 1: C_nat encode and decode of one vector of 2^20 elements (5.4 MB, cache-resident).  A
    # launch this short is bound by the host's call path when every launch is a Python call, so 16
    # launches are captured in a HIP graph and the replay is timed: GPU time per launch, back to back.
    d1 = 1 << 20
    x1 = torch.from_numpy(wl.config1()).cuda()
    e1, s1 = nc.nat_encode(x1, 0)
    o1 = torch.empty(d1, dtype=torch.float32, device="cuda")

    def graph_of(fn, launches=16):
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            fn()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            for _ in range(launches):
                fn()
        return g, launches

    for name, fn in (("config1_nat_encode_d1M", lambda: nc.nat_encode(x1, 0, exp_out=e1, sign_out=s1)),
                     ("config1_nat_decode_d1M", lambda: nc.nat_decode(e1, s1, d1, out=o1))):
        st_host = timer.rotating([fn])
        g, launches = graph_of(fn)
        st = timer.rotating([g.replay], group=1)
        st = {k: (v / launches if isinstance(v, float) else v) for k, v in st.items() if k != "raw"}
        res[name] = _entry(st, 5.125 * d1, 4.0 * d1,
                           "GPU time per launch, 16 launches replayed from a HIP graph (cache-resident, bound by the "
                           "launch); through one Python call per launch the host needs %.1f us" % (st_host["median"] * 1e3), 1)

    # ---- C_nat decode of one worker (config 2 shape): 1.125 d read, 4 d written
    R = sets_for(5.125 * d)
    xs = [wl.layered_laplace_device(r, off) for r in range(R)]
    outs = [torch.empty(d, dtype=torch.float32, device="cuda") for _ in range(R)]
    planes = [nc.nat_encode(xs[r], 0) for r in range(R)]
    st = timer.rotating([lambda r=r: nc.nat_decode(planes[r][0], planes[r][1], d, out=outs[r]) for r in range(R)])
    res["nat_decode_d25.6M"] = _entry(st, (1.125 + 4) * d, 4.0 * d, "1.125 B read + 4 B written per element", R)
    del planes

    # ---- config 3: D_nat^{2,8}, norm per layer tensor, encode then decode
    norms = [torch.empty(nseg, dtype=torch.float32, device="cuda") for _ in range(R)]
    code = [torch.empty(nc.dither_code_bytes(d, 8), dtype=torch.uint8, device="cuda") for _ in range(R)]
    sign = [torch.empty(nc.dither_sign_bytes(d, 8), dtype=torch.uint8, device="cuda") for _ in range(R)]
    ws = torch.empty(nc.dither_workspace_bytes(d, nseg, 0, True), dtype=torch.uint8, device="cuda")
    st = timer.rotating([lambda r=r: nc.dither_encode(xs[r], 2, 8, 0, seg_offsets=offdev, norms_out=norms[r],
                                                      code_out=code[r], sign_out=sign[r], workspace=ws) for r in range(R)])
    res["config3_dither_2_8_layer_encode"] = _entry(
        st, 4.625 * d, 4.0 * d, "norm per layer then encode; minimum 4 + 0.625 B per element, a second read of x "
        "that misses the last-level cache makes it 8 + 0.625", R)
    st = timer.rotating([lambda r=r: nc.dither_decode(norms[r], code[r], sign[r], d, 8, seg_offsets=offdev, out=outs[r])
                         for r in range(R)])
    res["config3_dither_2_8_layer_decode"] = _entry(st, 4.625 * d, 4.0 * d, "0.625 B read + 4 B written per element", R)
    del norms, code, sign

    # ---- D_nat^{inf,4} with small buckets (512 elements): one-pass encode of one worker
    b512 = 512
    nb512 = nc.segment_count(d, 0, b512, False)
    cstride = nc.plane_stride(nc.dither_code_bytes(d, 4))
    R3 = sets_for(8 * 0.5 * d + 4 * d)
    norms5 = [torch.empty((n, nb512), dtype=torch.float32, device="cuda") for _ in range(max(R, R3))]
    code5 = [torch.empty((n, cstride), dtype=torch.uint8, device="cuda") for _ in range(max(R, R3))]
    st = timer.rotating([lambda r=r: nc.dither_encode(xs[r], math.inf, 4, 0, bucket=b512, norms_out=norms5[r][0],
                                                      code_out=code5[r][0]) for r in range(R)])
    res["dither_inf_4_bucket512_encode_d25.6M"] = _entry(st, 4.5 * d + 4.0 * nb512, 4.0 * d,
                                                        "one pass, 8 buckets per workgroup; 4 + 0.5 B per element", R)
    # ... and the fused sum of 8 workers
    for r in range(R3):
        for w in range(n):
            nc.dither_encode(xs[(r + w) % R], math.inf, 4, r, worker=w, bucket=b512, norms_out=norms5[r][w], code_out=code5[r][w])
    st = timer.rotating([lambda r=r: nc.aggregate_sum(nc.NC_KIND_DITHER, d, code5[r], None, norms5[r], s=4, bucket=b512,
                                                      out=outs[r]) for r in range(R3)])
    res["dither_inf_4_bucket512_aggregate_n8_d25.6M"] = _entry(st, 8.0 * d + 4.0 * nb512 * n, 4.0 * d * n,
                                                              "per-(worker, bucket) tables; 8 x 0.5 B read + 4 B written", R3)
    del norms5, code5, xs

    # ---- Algorithm 1's master step with C_M = C_nat at the config-2 shape; the 8-bit clipped form
    row = (d + 63) // 64 * 64
    xb = torch.empty((n, row), dtype=torch.float32, device="cuda")
    for w in range(n):
        xb[w, :d] = wl.layered_laplace_device(w, off)
    Rm = sets_for((n * 1.125 + 1.125) * d)
    ebs = [nc.nat_encode_batch(xb, seed=r, d=d) for r in range(Rm)]
    em = [torch.empty(nc.nat_exp_bytes(d), dtype=torch.uint8, device="cuda") for _ in range(Rm)]
    sm = [torch.empty(nc.sign_bytes(d), dtype=torch.uint8, device="cuda") for _ in range(Rm)]
    st = timer.rotating([lambda r=r: nc.master_nat(d, ebs[r][0], ebs[r][1], seed=1, exp_out=em[r], sign_out=sm[r])
                         for r in range(Rm)])
    res["master_nat_n8_d25.6M"] = _entry(st, (n * 1.125 + 1.125) * d, 4.0 * d * n,
                                         "fused decode+sum of 8 streams and C_nat of the sum: 9 B read + 1.125 B written per element", Rm)
    del ebs
    cbs = [torch.empty((n, nc.plane_stride(d)), dtype=torch.uint8, device="cuda") for _ in range(Rm)]
    st = timer.rotating([lambda r=r: nc.nat_clip_encode(xb, r, code_out=cbs[r], d=d) for r in range(Rm)])
    res["clip8_encode_x8_d25.6M"] = _entry(st, 5.0 * d * n, 4.0 * d * n,
                                           "8 workers in one launch; 4 B read + 1 B written per element (818 MB read per launch)", Rm)
    st = timer.rotating([lambda r=r: nc.clip_aggregate_int(cbs[r], d, 1, exp_out=em[r], sign_out=sm[r]) for r in range(Rm)])
    res["clip8_aggregate_int64_n8_d25.6M"] = _entry(
        st, (n + 1.125) * d, 4.0 * d * n,
        "int64 sum of 8 byte streams and C_nat of the sum: 8 B read + 1.125 B written per element", Rm)
    del xb, cbs, em, sm, outs

    # ---- config 4: D_nat^{inf,4}, buckets of 8192, 8 workers, fused decode+sum
    d4, bucket = wl.D_VGG16, wl.BUCKET
    nb = nc.segment_count(d4, 0, bucket, False)
    x4 = torch.empty((n, d4), dtype=torch.float32, device="cuda")
    for w in range(n):
        wl.bucketed_gaussian_device(w, out=x4[w])
    norms4 = torch.empty((n, nb), dtype=torch.float32, device="cuda")
    code4 = torch.empty((n, nc.plane_stride(nc.dither_code_bytes(d4, 4))), dtype=torch.uint8, device="cuda")
    out4 = torch.empty(d4, dtype=torch.float32, device="cuda")

    def encode_all():
        for w in range(n):
            nc.dither_encode(x4[w], math.inf, 4, 0, worker=w, bucket=bucket, norms_out=norms4[w], code_out=code4[w])

    st = timer.rotating([encode_all], reps=20, warm=3, group=1)
    res["config4_dither_inf_4_bucket_encode_x8"] = _entry(st, 4.5 * d4 * n, 4.0 * d4 * n,
                                                         "8 one-pass launches over 4.4 GB of input; 4 + 0.5 B per element", 1)
    st = timer.rotating([lambda: nc.aggregate_sum(nc.NC_KIND_DITHER, d4, code4, None, norms4, s=4, bucket=bucket, out=out4)],
                        reps=20, warm=3)
    res["config4_dither_inf_4_aggregate_n8"] = _entry(st, 8.0 * d4 + 4.0 * nb * n, 4.0 * d4 * n,
                                                     "8 x 0.5 B read + 4 B written per output element, plus norms (1.1 GB per launch)", 1)
    del x4, norms4, code4, out4

    # ---- config 5: C_nat o S^k, d = 335,000,000, k = d/100, 8 workers, dense scatter-sum
    d5, k5 = wl.D_BERT_LARGE, wl.D_BERT_LARGE // 100
    x5 = torch.empty((n, d5), dtype=torch.float32, device="cuda")
    for w in range(n):
        wl.dense_gaussian_device(w, out=x5[w])
    idx = torch.empty((n, nc.plane_stride(4 * k5) // 4), dtype=torch.int32, device="cuda")
    exp5 = torch.empty((n, nc.plane_stride(k5)), dtype=torch.uint8, device="cuda")
    sign5 = torch.empty((n, nc.plane_stride(nc.sign_bytes(k5))), dtype=torch.uint8, device="cuda")
    out5 = torch.empty(d5, dtype=torch.float32, device="cuda")
    scale = float(np.float32(d5 / k5))
    st = timer.rotating([lambda: nc.sparse_nat_encode_batch(x5, k5, scale, 0, idx_out=idx, exp_out=exp5, sign_out=sign5)],
                        reps=20, warm=3)
    res["config5_sparse_nat_encode_x8"] = _entry(
        st, n * k5 * (4 + 4 + 1.125), 4.0 * d5 * n,
        "8 workers in one launch; per kept entry a 4 B gather out of 10.7 GB, 4 B index + 1.125 B code written "
        "(each gather moves a whole cache line)", 1)
    st = timer.rotating([lambda: nc.sparse_nat_aggregate(idx, exp5, sign5, k5, d5, out=out5)], reps=20, warm=3)
    res["config5_sparse_nat_aggregate_n8"] = _entry(
        st, 4.0 * d5 + n * k5 * (4 + 1.125 + 8), 4.0 * d5 * n,
        "dense fp32 sum of 8 sparse messages, one scatter launch per worker: 4 B per coordinate written + per entry "
        "5.125 B read and a 4 B read-modify-write", 1)
    ws5 = torch.empty(nc.sparse_aggregate_workspace_bytes(n, k5, d5), dtype=torch.uint8, device="cuda")
    st = timer.rotating([lambda: nc.sparse_nat_aggregate_ws(idx, exp5, sign5, k5, d5, out=out5, workspace=ws5)], reps=20, warm=3)
    res["config5_sparse_nat_aggregate_ws_n8"] = _entry(
        st, 4.0 * d5 + n * k5 * 5.125, 4.0 * d5 * n,
        "the same sum with the entries partitioned by output tile in a workspace: 4 B per coordinate written + "
        "5.125 B per entry read (the partition's own traffic, about 50 B per entry, is not counted)", 1)
    return res


def pmc_probe(which, nc, wl, torch, np, step):
    """For `rocprofv3 --pmc` / `--kernel-trace` runs: a few launches of one configuration's kernels plus
    1 GiB device copies (the counter calibration), no timing."""
    import math
    src = torch.zeros(1 << 28, dtype=torch.float32, device="cuda")      # 1 GiB read + 1 GiB written per copy
    dst = torch.empty_like(src)
    info = {"pmc_probe": which, "copy_bytes_read": src.numel() * 4, "copy_bytes_written": src.numel() * 4}
    n = wl.NUM_WORKERS
    if which == "headline":
        for i in range(3):
            step(i)
            dst.copy_(src)
        info.update({"d": wl.D_RESNET50, "n_workers": n})
    elif which == "cfg3":
        d = wl.D_RESNET50
        off = wl.layer_offsets()
        offdev = torch.from_numpy(off.view(np.int64)).cuda()
        x = wl.layered_laplace_device(0, off)
        ws = torch.empty(nc.dither_workspace_bytes(d, off.size - 1, 0, True), dtype=torch.uint8, device="cuda")
        out = torch.empty(d, dtype=torch.float32, device="cuda")
        for i in range(3):
            norms, code, sign = nc.dither_encode(x, 2, 8, i, seg_offsets=offdev, workspace=ws)
            dst.copy_(src)
            nc.dither_decode(norms, code, sign, d, 8, seg_offsets=offdev, out=out)
            dst.copy_(src)
        info.update({"d": d, "segments": int(off.size - 1)})
    elif which == "cfg4":
        d4, bucket = wl.D_VGG16, wl.BUCKET
        x4 = torch.empty((n, d4), dtype=torch.float32, device="cuda")
        for w in range(n):
            wl.bucketed_gaussian_device(w, out=x4[w])
        nb = nc.segment_count(d4, 0, bucket, False)
        norms4 = torch.empty((n, nb), dtype=torch.float32, device="cuda")
        code4 = torch.empty((n, nc.plane_stride(nc.dither_code_bytes(d4, 4))), dtype=torch.uint8, device="cuda")
        out4 = torch.empty(d4, dtype=torch.float32, device="cuda")
        for i in range(2):
            for w in range(n):
                nc.dither_encode(x4[w], math.inf, 4, i, worker=w, bucket=bucket, norms_out=norms4[w], code_out=code4[w])
            dst.copy_(src)
            nc.aggregate_sum(nc.NC_KIND_DITHER, d4, code4, None, norms4, s=4, bucket=bucket, out=out4)
            dst.copy_(src)
        info.update({"d": d4, "n_workers": n, "bucket": bucket})
    elif which == "cfg5":
        d5, k5 = wl.D_BERT_LARGE, wl.D_BERT_LARGE // 100
        x5 = torch.empty((n, d5), dtype=torch.float32, device="cuda")
        for w in range(n):
            wl.dense_gaussian_device(w, out=x5[w])
        out5 = torch.empty(d5, dtype=torch.float32, device="cuda")
        for i in range(2):
            idx, e5, s5 = nc.sparse_nat_encode_batch(x5, k5, float(np.float32(d5 / k5)), i)
            dst.copy_(src)
            nc.sparse_nat_aggregate(idx, e5, s5, k5, d5, out=out5)
            dst.copy_(src)
            nc.sparse_nat_aggregate_ws(idx, e5, s5, k5, d5, out=out5)
            dst.copy_(src)
        info.update({"d": d5, "k": k5, "n_workers": n})
    else:
        sys.exit(f"bench.py: unknown --pmc-probe {which}")
    torch.cuda.synchronize()
    print(json.dumps(info))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--settle-ms", type=float, default=400.0,
                    help="wall time of untimed steps run before the warm-up so the clocks leave idle (0: none)")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing")
    ap.add_argument("--no-secondary", action="store_true", help="skip the other kernels (decode, dithering, sparse, clip)")
    ap.add_argument("--quick", action="store_true", help="smaller d (for profiling runs); not a valid result")
    ap.add_argument("--pmc-probe", nargs="?", const="headline", default=None,
                    choices=["headline", "cfg3", "cfg4", "cfg5"],
                    help="for rocprofv3 runs: a few launches of one configuration's kernels plus 1 GiB device "
                         "copies (the counter calibration), no timing")
    ap.add_argument("--ceilings", action="store_true",
                    help="print only the device ceilings (copy / read / fill / 9:4 mix kernels, Philox rate)")
    ap.add_argument("--dump-steps", default=None, help="write the per-step event times of the timed region to this JSON file")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1")

    import numpy as np
    import torch

    from paper_1905_10988_amd import natcomp as nc
    from paper_1905_10988_amd import workloads as wl

    nc.lib()                                       # fails loudly if libnatcomp.so is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    timer = Timer(torch, np)
    if args.ceilings:
        pr = Probe(torch)
        print(json.dumps({"ceilings": pr.ceilings(timer), "ceilings_at_4d_bytes": pr.ceilings(timer, 4 * wl.D_RESNET50 // 16 * 16)}))
        return

    n = wl.NUM_WORKERS
    d = wl.D_RESNET50 if not args.quick else wl.D_RESNET50 // 16
    off = wl.layer_offsets(d=d) if not args.quick else wl.layer_offsets(d=d, hi=d // 8)
    row = (d + 63) // 64 * 64
    xdev = torch.empty((n, row), dtype=torch.float32, device="cuda")
    x_host = []
    for w in range(n):
        xw = wl.layered_gaussian(w, off)
        xdev[w, :d] = torch.from_numpy(xw).cuda()
        x_host.append(xw)
    torch.cuda.synchronize()
    exp = torch.empty((n, nc.plane_stride(nc.nat_exp_bytes(d))), dtype=torch.uint8, device="cuda")
    sign = torch.empty((n, nc.plane_stride(nc.sign_bytes(d))), dtype=torch.uint8, device="cuda")
    out = torch.empty(d, dtype=torch.float32, device="cuda")

    def step(seed):
        nc.nat_encode_batch(xdev, seed=seed, d=d, exp_out=exp, sign_out=sign)
        nc.aggregate_sum(nc.NC_KIND_NAT, d, exp, sign, out=out)

    if args.pmc_probe:
        pmc_probe(args.pmc_probe, nc, wl, torch, np, step)
        return

    # settle: the same step for a fixed wall time, so the timed region does not start on idle clocks
    settle_steps = 0
    t_settle = time.perf_counter()
    while (time.perf_counter() - t_settle) * 1e3 < args.settle_ms:
        for _ in range(16):
            step(settle_steps)
            settle_steps += 1
        torch.cuda.synchronize()
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()

    # timed region: exactly K steps.  Events before the encoder and between the two kernels of every
    # sampled step (every step up to K = 64); the event that opens the next step closes the aggregate.
    K = args.steps
    every = max(1, -(-K // 64))
    sampled = list(range(0, K, every))
    ev = {i: [torch.cuda.Event(enable_timing=True) for _ in range(3 if every > 1 else 2)] for i in sampled}
    ev_end = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(K):
        e = ev.get(i)
        if e is None:
            step(1000 + i)
            continue
        e[0].record()
        nc.nat_encode_batch(xdev, seed=1000 + i, d=d, exp_out=exp, sign_out=sign)
        e[1].record()
        nc.aggregate_sum(nc.NC_KIND_NAT, d, exp, sign, out=out)
        if every > 1:
            e[2].record()
    ev_end.record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / K
    enc_samples = [ev[i][0].elapsed_time(ev[i][1]) for i in sampled]
    if every > 1:
        agg_samples = [ev[i][1].elapsed_time(ev[i][2]) for i in sampled]
        step_samples = [ev[i][0].elapsed_time(ev[i][2]) for i in sampled]
    else:
        closing = [ev[i + 1][0] if i + 1 < K else ev_end for i in sampled]
        agg_samples = [ev[i][1].elapsed_time(c) for i, c in zip(sampled, closing)]
        step_samples = [ev[i][0].elapsed_time(c) for i, c in zip(sampled, closing)]
    enc_st, agg_st, step_st = timer.stats(enc_samples), timer.stats(agg_samples), timer.stats(step_samples)

    # the fused sum on cold code sets: several sets of 8 streams (more than 512 MB in all), summed round-robin
    Rc = sets_for(n * 1.125 * d + 4.0 * d) + 1
    cold_sets = [nc.nat_encode_batch(xdev, seed=77 + r, d=d) for r in range(Rc)]
    cold_out = [torch.empty(d, dtype=torch.float32, device="cuda") for _ in range(Rc)]
    cold_st = timer.rotating([lambda r=r: nc.aggregate_sum(nc.NC_KIND_NAT, d, cold_sets[r][0], cold_sets[r][1], out=cold_out[r])
                              for r in range(Rc)], reps=max(20, min(K, 64)), warm=5)
    # the encoder writing to rotated code sets (its 818 MB of input per launch never fit a cache)
    enc_rot_st = timer.rotating([lambda r=r: nc.nat_encode_batch(xdev, seed=5 + r, d=d, exp_out=cold_sets[r][0],
                                                                 sign_out=cold_sets[r][1]) for r in range(Rc)],
                                reps=max(20, min(K, 64)), warm=5)
    del cold_sets, cold_out
    if args.dump_steps:
        with open(args.dump_steps, "w") as f:
            json.dump({"encode_ms": enc_samples, "aggregate_ms": agg_samples, "step_ms": step_samples,
                       "settle_steps": settle_steps, "wall_ms_per_step": ms_per_step,
                       "cold_aggregate_ms": cold_st["raw"], "rotated_encode_ms": enc_rot_st["raw"]}, f)

    probe = Probe(torch)
    ceil = probe.ceilings(timer)
    # the same kernels on buffers the size of one config-2/3 vector (102 MB): what a launch of
    # that size can reach, start and drain included
    ceil_small = probe.ceilings(timer, 4 * d // 16 * 16)

    input_bytes = 4.0 * d * n
    value = input_bytes / (ms_per_step * 1e-3) / 1e9
    enc_alg = ENCODE_BYTES_PER_ELEM * d * n
    agg_alg = aggregate_bytes_per_elem(n) * d

    def gbs(alg, ms):
        return alg / (ms * 1e-3) / 1e9

    enc_gbs, agg_gbs = gbs(enc_alg, enc_st["mean"]), gbs(agg_alg, agg_st["mean"])
    result = {
        "metric": "GB/s fp32 input encoded (C_nat) and decoded+summed (n=8)",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": args.warmup,
        "settle_steps": settle_steps,
        "settle_ms": args.settle_ms,
        "ms_per_step": round(ms_per_step, 5),
        "ms_per_step_median": round(step_st["median"], 5),
        "ms_per_step_min": round(step_st["min"], 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u32/f32",
        "data": "synthetic",
        "config": {
            "workload": "config 2: C_nat encode of 8 workers x d=25,557,032 fp32 (161 layers, N(0, sigma_l^2)), "
                        "then fused decode+sum n=8" + (" [QUICK, reduced d: not a valid result]" if args.quick else ""),
            "d": d, "n_workers": n, "launches_per_step": 2,
        },
        "roofline": {
            "kernel": "nat_encode_kernel (8 workers in one launch)",
            "bound": "hbm",
            "achieved": round(enc_gbs, 1),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(enc_gbs / HBM_PEAK_GBS, 4),
            "traffic": measured_traffic("nat_encode_config2_pmc.txt"),
            "algorithmic_bytes_per_launch": enc_alg,
            "avg_launch_ms": round(enc_st["mean"], 5),
            "median_launch_ms": round(enc_st["median"], 5),
            "min_launch_ms": round(enc_st["min"], 5),
            "event_samples": enc_st["samples"],
            "frac_median": round(gbs(enc_alg, enc_st["median"]) / HBM_PEAK_GBS, 4),
            "rotated_outputs_median_ms": round(enc_rot_st["median"], 5),
            "rotated_outputs_frac": round(gbs(enc_alg, enc_rot_st["median"]) / HBM_PEAK_GBS, 4),
            "device_copy_kernel_GBps": ceil["copy_kernel_GBps"],
            "frac_of_device_copy_kernel": round(enc_gbs / ceil["copy_kernel_GBps"], 4),
        },
        "roofline_aggregate": {
            "kernel": "nat_aggregate_kernel (n=8)",
            "bound": "hbm",
            "achieved": round(agg_gbs, 1),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(agg_gbs / HBM_PEAK_GBS, 4),
            "traffic": measured_traffic("nat_aggregate_config2_pmc.txt"),
            "algorithmic_bytes_per_launch": agg_alg,
            "avg_launch_ms": round(agg_st["mean"], 5),
            "median_launch_ms": round(agg_st["median"], 5),
            "min_launch_ms": round(agg_st["min"], 5),
            "event_samples": agg_st["samples"],
            "frac_median": round(gbs(agg_alg, agg_st["median"]) / HBM_PEAK_GBS, 4),
            "cold_buffer_sets": Rc,
            "cold_median_ms": round(cold_st["median"], 5),
            "cold_min_ms": round(cold_st["min"], 5),
            "cold_mean_ms": round(cold_st["mean"], 5),
            "cold_frac": round(gbs(agg_alg, cold_st["median"]) / HBM_PEAK_GBS, 4),
            "device_mix_9to4_kernel_GBps": ceil["mix_9to4_kernel_GBps"],
            "frac_of_device_mix_kernel": round(agg_gbs / ceil["mix_9to4_kernel_GBps"], 4),
        },
        "device_ceilings": ceil,
        "device_ceilings_at_4d_bytes": ceil_small,
    }

    if not args.no_secondary and not args.quick:
        result["other_kernels"] = secondary_kernels(nc, wl, torch, np, timer)

    if not args.no_cpu_baseline:
        import oracle
        # the same step on the host: all 8 workers encoded by the oracle, then decoded and summed
        # (it is short enough to run whole); rate per fp32 input byte, like `value`
        exp_h = np.zeros((n, d), np.uint8)
        sign_h = np.zeros((n, (d + 7) // 8), np.uint8)
        reps, t0 = 0, time.perf_counter()
        while reps < 8 and (reps == 0 or time.perf_counter() - t0 < 1.0):   # about 10-30 s of CPU work on 16 cores
            for w in range(n):
                exp_h[w], sign_h[w] = oracle.nat_encode(x_host[w], 1000 + reps, w)
            oracle.aggregate_nat(exp_h, sign_h, d)
            reps += 1
        dt = (time.perf_counter() - t0) / reps
        # the same oracle on one core: one worker's encode and a one-stream decode
        cores = oracle.threads()
        oracle.set_threads(1)
        t1 = time.perf_counter()
        e1, s1 = oracle.nat_encode(x_host[0], 1000, 0)
        oracle.nat_decode(e1, s1, d)
        dt1 = time.perf_counter() - t1
        oracle.set_threads(cores)
        result["cpu_baseline"] = {
            "value": round(n * 4.0 * d / dt / 1e9, 3),
            "unit": "GB/s",
            "cores": cores,
            "kind": "oracle",
            "single_core_value": round(4.0 * d / dt1 / 1e9, 3),
            "single_core_sample": f"one worker (d={d}) encoded and decoded on one thread, {dt1:.2f} s",
            "sample": f"{reps} whole steps (8 workers x d={d} encoded, 8 streams decoded+summed each), "
                      f"{dt:.2f} s of wall time per step",
        }
        # cross-check the GPU result of the last timed step on a window while we are here
        a, b = 0, 4096
        step(1000 + K - 1)
        torch.cuda.synchronize()
        eo, so = oracle.nat_encode(x_host[0][a:b], 1000 + K - 1, 0, index_offset=a)
        assert np.array_equal(exp[0, a:b].cpu().numpy(), eo), "GPU codes differ from the oracle"

    print(json.dumps(result))


if __name__ == "__main__":
    main()
