"""Benchmark of the hot path on one MI355X.

A step is one pass of the headline workload ("config 2"): natural compression of 8 workers'
gradients (d = 25,557,032 fp32 each, 161 layers) in one batched launch, then the fused
decode-and-sum of the 8 code streams.  Inputs are resident in HBM before the timed region.
`value` is fp32 input bytes (8 * 4 * d) per second of step time.

Prints ONE JSON line with the metric, a `roofline` object for the dominant kernel (the
batched encoder) and a `cpu_baseline` object (the CPU oracle timed on the host cores).
"""
import argparse
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


def _time_ms(torch, np, fn, reps=20, warm=3):
    """Average HIP-event time of fn() on the current stream."""
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    for a, b in evs:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    return float(np.mean([a.elapsed_time(b) for a, b in evs]))


def _entry(ms, alg_bytes, input_bytes, note):
    gbs = alg_bytes / (ms * 1e-3) / 1e9
    return {"ms": round(ms, 5), "algorithmic_GBps": round(gbs, 1), "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4),
            "fp32_input_GBps": round(input_bytes / (ms * 1e-3) / 1e9, 1), "algorithmic_bytes": alg_bytes, "note": note}


def secondary_kernels(nc, wl, torch, np):
    """The remaining kernels of the path, each on its configuration's shape (not part of `value`)."""
    import math
    res = {}
    d = wl.D_RESNET50
    off = wl.layer_offsets()
    offdev = torch.from_numpy(off.view(np.int64)).cuda()
    nseg = off.size - 1
    x = wl.layered_laplace_device(0, off)
    out = torch.empty(d, dtype=torch.float32, device="cuda")
    # C_nat decode of one worker (config 2 shape)
    e, sg = nc.nat_encode(x, 0)
    ms = _time_ms(torch, np, lambda: nc.nat_decode(e, sg, d, out=out))
    res["nat_decode_d25.6M"] = _entry(ms, (1.125 + 4) * d, 4.0 * d, "1.125 B read + 4 B written per element")
    # Algorithm 1's master step with C_M = C_nat at the config-2 shape: sum of 8 streams, re-compressed
    xb = torch.empty((wl.NUM_WORKERS, (d + 63) // 64 * 64), dtype=torch.float32, device="cuda")
    for w in range(wl.NUM_WORKERS):
        xb[w, :d] = wl.layered_laplace_device(w, off)
    eb, sb = nc.nat_encode_batch(xb, seed=0, d=d)
    em = torch.empty(nc.nat_exp_bytes(d), dtype=torch.uint8, device="cuda")
    sm = torch.empty(nc.sign_bytes(d), dtype=torch.uint8, device="cuda")
    ms = _time_ms(torch, np, lambda: nc.master_nat(d, eb, sb, seed=1, exp_out=em, sign_out=sm))
    res["master_nat_n8_d25.6M"] = _entry(ms, (wl.NUM_WORKERS * 1.125 + 1.125) * d, 4.0 * d * wl.NUM_WORKERS,
                                         "fused decode+sum of 8 streams and C_nat of the sum: 9 B read + 1.125 B written per element")
    # the 8-bit clipped representation and the int64 aggregator with master-side C_nat, same shape
    cb = torch.empty((wl.NUM_WORKERS, nc.plane_stride(d)), dtype=torch.uint8, device="cuda")
    ms = _time_ms(torch, np, lambda: nc.nat_clip_encode(xb, 0, code_out=cb, d=d))
    res["clip8_encode_x8_d25.6M"] = _entry(ms, 5.0 * d * wl.NUM_WORKERS, 4.0 * d * wl.NUM_WORKERS,
                                           "8 workers in one launch; 4 B read + 1 B written per element")
    ms = _time_ms(torch, np, lambda: nc.clip_aggregate_int(cb, d, 1, exp_out=em, sign_out=sm))
    res["clip8_aggregate_int64_n8_d25.6M"] = _entry(
        ms, (wl.NUM_WORKERS + 1.125) * d, 4.0 * d * wl.NUM_WORKERS,
        "int64 sum of 8 byte streams and C_nat of the sum: 8 B read + 1.125 B written per element "
        "(bound by the 64-bit integer arithmetic, not by HBM)")
    del xb, eb, sb, cb
    # config 3: D_nat^{2,8}, norm per layer tensor, encode then decode
    norms = torch.empty(nseg, dtype=torch.float32, device="cuda")
    code = torch.empty(nc.dither_code_bytes(d, 8), dtype=torch.uint8, device="cuda")
    sign = torch.empty(nc.dither_sign_bytes(d, 8), dtype=torch.uint8, device="cuda")
    ws = torch.empty(nc.dither_workspace_bytes(d, nseg, 0, True), dtype=torch.uint8, device="cuda")
    ms = _time_ms(torch, np, lambda: nc.dither_encode(x, 2, 8, 0, seg_offsets=offdev, norms_out=norms, code_out=code,
                                                      sign_out=sign, workspace=ws))
    res["config3_dither_2_8_layer_encode"] = _entry(
        ms, 4.625 * d, 4.0 * d, "3 launches (partial norms, finish, encode); minimum 4 + 0.625 B per element, "
        "this two-pass path moves 8 + 0.625 unless the second read hits the last-level cache")
    ms = _time_ms(torch, np, lambda: nc.dither_decode(norms, code, sign, d, 8, seg_offsets=offdev, out=out))
    res["config3_dither_2_8_layer_decode"] = _entry(ms, 4.625 * d, 4.0 * d, "0.625 B read + 4 B written per element")
    # D_nat^{inf,4} with small buckets (512 elements, the usual choice of QSGD-style bucketing): one-pass encode
    # of one worker and the fused sum of 8 workers, d = 25.6 M
    nw, b512 = wl.NUM_WORKERS, 512
    nb512 = nc.segment_count(d, 0, b512, False)
    norms5 = torch.empty((nw, nb512), dtype=torch.float32, device="cuda")
    code5 = torch.empty((nw, nc.plane_stride(nc.dither_code_bytes(d, 4))), dtype=torch.uint8, device="cuda")
    for w in range(nw):
        nc.dither_encode(x, math.inf, 4, 0, worker=w, bucket=b512, norms_out=norms5[w], code_out=code5[w])
    ms = _time_ms(torch, np, lambda: nc.dither_encode(x, math.inf, 4, 0, bucket=b512, norms_out=norms5[0],
                                                      code_out=code5[0]))
    res["dither_inf_4_bucket512_encode_d25.6M"] = _entry(ms, 4.5 * d + 4.0 * nb512, 4.0 * d,
                                                        "one pass, 8 buckets per workgroup; 4 + 0.5 B per element")
    ms = _time_ms(torch, np, lambda: nc.aggregate_sum(nc.NC_KIND_DITHER, d, code5, None, norms5, s=4, bucket=b512,
                                                      out=out))
    res["dither_inf_4_bucket512_aggregate_n8_d25.6M"] = _entry(ms, 8.0 * d + 4.0 * nb512 * nw, 4.0 * d * nw,
                                                              "per-(worker, bucket) tables; 8 x 0.5 B read + 4 B written")
    del x, out, code, sign, e, sg, norms5, code5
    # config 4: D_nat^{inf,4}, buckets of 8192, 8 workers, fused decode+sum
    d4, n, bucket = wl.D_VGG16, wl.NUM_WORKERS, wl.BUCKET
    nb = nc.segment_count(d4, 0, bucket, False)
    xs = torch.empty((n, d4), dtype=torch.float32, device="cuda")
    for w in range(n):
        wl.bucketed_gaussian_device(w, out=xs[w])
    norms4 = torch.empty((n, nb), dtype=torch.float32, device="cuda")
    code4 = torch.empty((n, nc.plane_stride(nc.dither_code_bytes(d4, 4))), dtype=torch.uint8, device="cuda")
    out4 = torch.empty(d4, dtype=torch.float32, device="cuda")

    def encode_all():
        for w in range(n):
            nc.dither_encode(xs[w], math.inf, 4, 0, worker=w, bucket=bucket, norms_out=norms4[w], code_out=code4[w])

    ms = _time_ms(torch, np, encode_all, reps=10)
    res["config4_dither_inf_4_bucket_encode_x8"] = _entry(ms, 4.5 * d4 * n, 4.0 * d4 * n,
                                                         "8 one-pass launches; 4 + 0.5 B per element")
    ms = _time_ms(torch, np, lambda: nc.aggregate_sum(nc.NC_KIND_DITHER, d4, code4, None, norms4, s=4, bucket=bucket,
                                                      out=out4), reps=10)
    res["config4_dither_inf_4_aggregate_n8"] = _entry(ms, 8.0 * d4 + 4.0 * nb * n, 4.0 * d4 * n,
                                                     "8 x 0.5 B read + 4 B written per output element, plus norms")
    del xs, norms4, code4, out4
    # config 5: C_nat o S^k, d = 335,000,000, k = d/100, 8 workers, dense scatter-sum
    d5, k5 = wl.D_BERT_LARGE, wl.D_BERT_LARGE // 100
    x5 = torch.empty((n, d5), dtype=torch.float32, device="cuda")
    for w in range(n):
        wl.dense_gaussian_device(w, out=x5[w])
    idx = torch.empty((n, nc.plane_stride(4 * k5) // 4), dtype=torch.int32, device="cuda")
    exp5 = torch.empty((n, nc.plane_stride(k5)), dtype=torch.uint8, device="cuda")
    sign5 = torch.empty((n, nc.plane_stride(nc.sign_bytes(k5))), dtype=torch.uint8, device="cuda")
    out5 = torch.empty(d5, dtype=torch.float32, device="cuda")
    scale = float(np.float32(d5 / k5))
    ms = _time_ms(torch, np, lambda: nc.sparse_nat_encode_batch(x5, k5, scale, 0, idx_out=idx, exp_out=exp5,
                                                                sign_out=sign5), reps=10)
    res["config5_sparse_nat_encode_x8"] = _entry(
        ms, n * k5 * (4 + 4 + 1.125), 4.0 * d5 * n,
        "8 workers in one launch; per kept entry a 4 B gather, 4 B index + 1.125 B code written "
        "(the gather really moves a 32-64 B sector per entry)")
    ms = _time_ms(torch, np, lambda: nc.sparse_nat_aggregate(idx, exp5, sign5, k5, d5, out=out5), reps=10)
    res["config5_sparse_nat_aggregate_n8"] = _entry(
        ms, 4.0 * d5 + n * k5 * (4 + 1.125 + 8), 4.0 * d5 * n,
        "zero-fill of the dense vector (4 B per coordinate) + 8 launches of k random 4 B read-modify-writes")
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing")
    ap.add_argument("--no-secondary", action="store_true", help="skip the other kernels (decode, dithering configs 3 and 4)")
    ap.add_argument("--quick", action="store_true", help="smaller d (for profiling runs); not a valid result")
    ap.add_argument("--pmc-probe", action="store_true",
                    help="for `rocprofv3 --pmc` runs: a few steps plus 1 GiB device copies (the counter calibration), no timing")
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
    exp = torch.empty((n, nc.plane_stride(nc.nat_exp_bytes(d))), dtype=torch.uint8, device="cuda")
    sign = torch.empty((n, nc.plane_stride(nc.sign_bytes(d))), dtype=torch.uint8, device="cuda")
    out = torch.empty(d, dtype=torch.float32, device="cuda")

    def step(seed):
        nc.nat_encode_batch(xdev, seed=seed, d=d, exp_out=exp, sign_out=sign)
        nc.aggregate_sum(nc.NC_KIND_NAT, d, exp, sign, out=out)

    if args.pmc_probe:
        src = torch.zeros(1 << 28, dtype=torch.float32, device="cuda")      # 1 GiB read + 1 GiB written per copy
        dst = torch.empty_like(src)
        for i in range(3):
            step(i)
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"pmc_probe": True, "copy_bytes_read": src.numel() * 4, "copy_bytes_written": src.numel() * 4,
                          "d": d, "n_workers": n}))
        return

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()

    # timed region: exactly K steps; HIP events on the launch stream bracket each kernel of every
    # 8th step (three event records cost about 12 us, 5 % of a step, so not every step carries them)
    K = args.steps
    every = 8 if K >= 16 else 1
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range((K + every - 1) // every)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(K):
        if i % every == 0:
            e3 = ev[i // every]
            e3[0].record()
            nc.nat_encode_batch(xdev, seed=1000 + i, d=d, exp_out=exp, sign_out=sign)
            e3[1].record()
            nc.aggregate_sum(nc.NC_KIND_NAT, d, exp, sign, out=out)
            e3[2].record()
        else:
            step(1000 + i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / K
    enc_ms = float(np.mean([e[0].elapsed_time(e[1]) for e in ev]))
    agg_ms = float(np.mean([e[1].elapsed_time(e[2]) for e in ev]))

    # reference: a plain device-to-device copy of 1 GiB (bytes read + bytes written per second)
    src = torch.zeros(1 << 28, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    copy_ms = _time_ms(torch, np, lambda: dst.copy_(src), reps=10)
    copy_gbs = 2.0 * src.numel() * 4 / (copy_ms * 1e-3) / 1e9
    del src, dst

    input_bytes = 4.0 * d * n
    value = input_bytes / (ms_per_step * 1e-3) / 1e9
    enc_alg = ENCODE_BYTES_PER_ELEM * d * n
    agg_alg = aggregate_bytes_per_elem(n) * d
    enc_gbs = enc_alg / (enc_ms * 1e-3) / 1e9
    agg_gbs = agg_alg / (agg_ms * 1e-3) / 1e9

    result = {
        "metric": "GB/s fp32 input encoded (C_nat) and decoded+summed (n=8)",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
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
            "avg_launch_ms": round(enc_ms, 5),
            "device_copy_GBps": round(copy_gbs, 1),
            "frac_of_device_copy": round(enc_gbs / copy_gbs, 4),
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
            "avg_launch_ms": round(agg_ms, 5),
            "frac_of_device_copy": round(agg_gbs / copy_gbs, 4),
        },
    }

    if not args.no_secondary and not args.quick:
        result["other_kernels"] = secondary_kernels(nc, wl, torch, np)

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
        # cross-check the GPU result of the last step on a window while we are here
        a, b = 0, 4096
        eo, so = oracle.nat_encode(x_host[0][a:b], 1000 + K - 1, 0, index_offset=a)
        assert np.array_equal(exp[0, a:b].cpu().numpy(), eo), "GPU codes differ from the oracle"

    print(json.dumps(result))


if __name__ == "__main__":
    main()
