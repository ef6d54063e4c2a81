#!/usr/bin/env python3
"""Benchmark of the DQSG/NDQSG hot path on one MI355X.

One "step" is one pass of the whole path over one batch of synthetic gradients
already resident in HBM: every worker's encode (scale, dither, quantize, pack),
then the server's decode chain with side information and running-sum
aggregation.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 5] [--no-cpu]
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

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published peak


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", type=int, default=5, help="configuration number (5 = the metric's)")
    ap.add_argument("--n", type=int, default=0, help="override elements per worker (debugging)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--cpu-sample", type=int, default=1 << 27,
                    help="elements per worker the oracle is timed on")
    ap.add_argument("--kernel-reps", type=int, default=20)
    ap.add_argument("--schedule", choices=["serial", "overlap", "fused"], default="serial",
                    help="serial: one library call per worker and direction, one stream; "
                         "overlap: the same calls, encoders and decoders on two streams; "
                         "fused: all encodes, then the whole server loop in one call")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch a plain copy of 2^28 floats (ndq_aggregate with W=1, "
                         "scale=1: 1 GiB read + 1 GiB written) so that a counter run has a "
                         "kernel of known traffic to scale FETCH_SIZE / WRITE_SIZE by")
    return ap.parse_args()


def algorithmic_bytes(kind, n, bits, K, s_in):
    """Bytes the method itself must move per launch (inputs once, outputs once)."""
    packed = (n * bits + 7) // 8
    if kind == "encode":
        return n * s_in + packed + 4 * K
    if kind == "dq_decode_store":
        return packed + 4 * K + 4 * n
    if kind == "dq_decode_accumulate":
        return packed + 4 * K + 8 * n
    if kind == "nested_decode":          # read side (= running sum), write it back
        return packed + 4 * K + 8 * n
    raise ValueError(kind)


def measured_traffic(kernel_key):
    """HBM bytes per launch from the committed rocprofv3 counter summary, if any."""
    path = os.path.join(ROOT, "profiles", "cfg5_hbm_traffic_pmc.txt")
    if not os.path.exists(path):
        return None
    pat = re.compile(r"^%s\s+traffic_bytes_per_launch\s*=\s*([0-9.eE+]+)" % re.escape(kernel_key))
    for line in open(path):
        m = pat.match(line.strip())
        if m:
            return float(m.group(1))
    return None


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (workers are simulated as buffers on it); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_1904_01197_amd import ndq, pipeline, workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    ndq.lib()   # fail loudly if the HIP library is missing

    wl = workloads.CONFIGS[args.workload]
    n = args.n or wl.n
    s_in = 2 if wl.dtype == "bf16" else 4
    K = ndq.ndq_num_buckets(n, wl.bucket)

    t0 = time.time()
    host = workloads.gradients(wl, n, threads=16)
    dev = pipeline.to_device(wl, host)
    bufs = pipeline.allocate(wl, n)
    ds = pipeline.dithers(wl)
    preset = 0.0
    if wl.shared_step:   # the shared step is a preset (read back once, outside the timed region)
        preset = pipeline.encode_all(wl, dev, bufs, ds)
    torch.cuda.synchronize()
    gen_s = time.time() - t0

    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            ndq.ndq_aggregate([src], 1.0, dst)
        torch.cuda.synchronize()
        del src, dst

    # ---- whole path: W warm-up steps, then exactly K timed steps ----------------
    if args.schedule == "overlap":
        ts = pipeline.TwoStreams(wl.W)
        one_step = lambda: pipeline.step_overlapped(wl, dev, bufs, ds, ts, preset)
    elif args.schedule == "fused":
        one_step = lambda: pipeline.step_fused(wl, dev, bufs, ds, preset)
    else:
        one_step = lambda: pipeline.step(wl, dev, bufs, ds, preset)
    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for _ in range(args.steps):
        one_step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    ms_per_step = elapsed * 1e3 / args.steps
    grad_bytes = wl.W * n * s_in
    value = grad_bytes / (ms_per_step * 1e-3) / 1e9

    # ---- per-kernel durations with events on the launch stream ------------------
    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps   # ms

    kernels = []
    seen = {}
    count = 0
    for w, (kind, arg) in enumerate(wl.plan):
        bits = ndq.ndq_code_bits(arg)
        if kind == "dq":
            enc_key, enc = "dq_encode_%s_b%d" % (wl.dtype, bits), (
                lambda w=w, arg=arg: ndq.ndq_dq_encode(dev[w], preset, arg, wl.bucket, ds[w],
                                                       bufs.codes[w], bufs.steps[w]))
            dkind = "dq_decode_accumulate" if count > 0 else "dq_decode_store"
            dec_key, dec = "%s_b%d" % (dkind, bits), (
                lambda w=w, arg=arg, c=count: ndq.ndq_dq_decode(
                    bufs.codes[w], n, arg, wl.bucket, bufs.steps[w], ds[w], bufs.total, c > 0))
        else:
            enc_key, enc = "nested_encode_%s_b%d" % (wl.dtype, bits), (
                lambda w=w, arg=arg: ndq.ndq_nested_encode(dev[w], preset, wl.fine_levels, arg,
                                                           wl.bucket, ds[w], bufs.codes[w],
                                                           bufs.steps[w]))
            dkind = "nested_decode"
            dec_key, dec = "nested_decode_inplace_b%d" % bits, (
                lambda w=w, arg=arg, c=count: ndq.ndq_nested_decode(
                    bufs.codes[w], n, arg, wl.bucket, bufs.steps[w], ds[w], bufs.total, 1.0 / c,
                    bufs.total, True))
        count += 1
        for key, fn, akind in ((enc_key, enc, "encode"), (dec_key, dec, dkind)):
            if key in seen:
                seen[key]["launches_per_step"] += 1
                continue
            ms = timed(fn, args.kernel_reps)
            nbytes = algorithmic_bytes(akind, n, bits, K, s_in)
            rec = {"kernel": key, "launches_per_step": 1, "avg_ms": round(ms, 5),
                   "algorithmic_bytes": nbytes, "GBps": round(nbytes / (ms * 1e-3) / 1e9, 1)}
            seen[key] = rec
            kernels.append(rec)
    if wl.out_scale != 1.0:
        ms = timed(lambda: ndq.ndq_aggregate([bufs.total], wl.out_scale, bufs.total),
                   args.kernel_reps)
        kernels.append({"kernel": "aggregate_scale", "launches_per_step": 1, "avg_ms": round(ms, 5),
                        "algorithmic_bytes": 8 * n, "GBps": round(8 * n / (ms * 1e-3) / 1e9, 1)})
    dominant = max(kernels, key=lambda r: r["avg_ms"] * r["launches_per_step"])
    achieved = dominant["algorithmic_bytes"] / (dominant["avg_ms"] * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": dominant["kernel"], "achieved": round(achieved, 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": measured_traffic(dominant["kernel"]),
                "algorithmic_bytes_per_launch": dominant["algorithmic_bytes"],
                "avg_launch_ms": dominant["avg_ms"]}
    step_bytes = sum(r["algorithmic_bytes"] * r["launches_per_step"] for r in kernels)

    # ---- CPU baseline: the oracle, as it stands, on a bounded sample ------------
    cpu = None
    if not args.no_cpu:
        import oracle
        from oracle import pipeline as opipe
        ns = min(n, args.cpu_sample) // max(wl.bucket, 64) * max(wl.bucket, 64) or n
        sl = [h[:ns] for h in host]
        seeds = [workloads.dither_seed(wl, w) for w in range(wl.W)]
        ds_o = opipe.dithers(wl.W, seeds)
        oracle.lib()
        c0 = time.perf_counter()
        codes, steps, _ = opipe.encode_all(wl.plan, wl.fine_levels, wl.bucket, wl.shared_step, sl,
                                           ds_o, preset)
        ref = opipe.decode_chain(wl.plan, wl.bucket, ns, codes, steps, ds_o, wl.out_scale)
        cpu_s = time.perf_counter() - c0
        cpu = {"value": round(wl.W * ns * s_in / cpu_s / 1e9, 5), "unit": "GB/s", "cores": 1,
               "kind": "oracle",
               "sample": "first %d elements per worker of the same %d-worker workload "
                         "(encode all + decode chain), %.1f s single-thread C oracle on a "
                         "%d-core host" % (ns, wl.W, cpu_s, os.cpu_count() or 0)}

    out = {
        "metric": "encode+decode+aggregate GB/s of gradient (and % of MI355X HBM peak) at n=2^27",
        "value": round(value, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": wl.name, "W": wl.W, "n_per_worker": n, "input_dtype": wl.dtype,
                   "bucket": wl.bucket, "schedule": args.schedule, "plan": ["%s%d" % p for p in wl.plan],
                   "launches_per_step": sum(r["launches_per_step"] for r in kernels)},
        "gelem_per_s": round(wl.W * n / (ms_per_step * 1e-3) / 1e9, 3),
        "step_algorithmic_bytes": step_bytes,
        "step_hbm_frac_of_peak": round(step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
        "roofline": roofline,
        "cpu_baseline": cpu,
        "kernels": kernels,
        "input_generation_s": round(gen_s, 1),
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
