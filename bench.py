#!/usr/bin/env python3
"""Benchmark of the DQSG/NDQSG hot path on one MI355X.

One "step" is one pass of the whole path over one batch of synthetic gradients
already resident in HBM: every worker's encode (scale, dither, quantize, pack),
then the server's decode chain with side information and running-sum
aggregation.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 5] [--no-cpu] [--prewarm-ms T]
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
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", type=int, default=5, help="configuration number (5 = the metric's)")
    ap.add_argument("--n", type=int, default=0, help="override elements per worker (debugging)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--cpu-sample", type=int, default=1 << 27,
                    help="elements per worker the oracle is timed on")
    ap.add_argument("--kernel-reps", type=int, default=50)
    ap.add_argument("--schedule", choices=["serial", "fused"], default="fused",
                    help="serial: one library call per worker and direction; "
                         "fused: all encodes, then the whole server loop in one call")
    ap.add_argument("--prewarm-ms", type=float, default=300.0,
                    help="untimed steps run for this long before the warm-up steps: the chip's clocks "
                         "settle only some tens of milliseconds after load begins (reported as prewarm_ms)")
    ap.add_argument("--cpu-threads", type=int, default=0,
                    help="threads of the all-cores oracle leg (default: min(16, host cores))")
    ap.add_argument("--graph", action="store_true",
                    help="record the step into a HIP graph once and replay it for the timed steps")
    ap.add_argument("--extras", action="store_true",
                    help="also time the kernels beyond the headline path (half-dithered decode, "
                         "shrinkage alpha<1, index entropy, dense base-L stream, sigma_z estimate) "
                         "on worker 0/1 of the same workload; reported under \"extras\"")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch a plain copy of 2^28 floats (ndq_aggregate with W=1, "
                         "scale=1: 1 GiB read + 1 GiB written) so that a counter run has a "
                         "kernel of known traffic to scale FETCH_SIZE / WRITE_SIZE by")
    return ap.parse_args()


# VALU roof: 256 CUs x 4 SIMDs x 32 lanes x 2.4 GHz = 78.6 T lane-operations/s for the
# instructions a SIMD retires at full rate (fp32 add/mul/fma, integer add, logic) --
# the published 157.3 TFLOP/s fp32 vector figure at 2 flops per fma.  Conversions,
# left shifts and bit-fields, min/max/med3, rounding and integer multiplies retire at
# half that rate (profiles/gfx950_valu_issue_rates.txt has the measurement).
VALU_PEAK_TOPS = 256 * 4 * 32 * 2.4e9 / 1e12

# Algorithmic lane-operations per element: the arithmetic the header states on a
# machine with a 32x32->64 multiply, a three-input logic op and fma; work that is
# uniform across a wave (key schedule, step, 1/step) is not counted.  Each entry is
# (operations counted once each, the same in full-rate equivalents: a half-rate
# operation counts 2).  roofline.frac uses the first; the second is reported as
# frac_weighted and credits nothing but says how busy the issue ports are.
OPS_PHILOX = (40 / 8.0, (20 * 2 + 20 * 1) / 8.0)   # 10 rounds x (2 multiplies + 2 xor3) per 8 elements
OPS_DITHER = (2.0, 3.0)                            # convert the 16-bit half (half rate), fma


def _ops_encode(bf16, nested_pow2_own_step):
    widen = (1.0, 1.5) if bf16 else (0.0, 0.0)      # low half: shift (half rate), high half: mask
    absmax = (1.0, 1.5) if bf16 else (2.0, 3.0)     # bf16: and + packed 16-bit max per 2 elements; fp32: |.|, max
    if nested_pow2_own_step:                        # fma, magic-constant add, funnel shift (half rate)
        quant = (3.0, 4.0)
    else:                                           # fma, rint, clip (both half rate), pack fma, convert per 4 codes
        quant = (4.25, 6.5)
    return tuple(OPS_PHILOX[i] + OPS_DITHER[i] + widen[i] + absmax[i] + quant[i] for i in (0, 1))


def _plus(base, once, weighted):
    return (base[0][0] + base[1][0] + once, base[0][1] + base[1][1] + weighted)


OPS = {
    "dq_encode": lambda bf16: _ops_encode(bf16, False),
    "nested_encode": lambda bf16: _ops_encode(bf16, True),
    # code -> float (mask, fma), subtract dither, scale (+ add when accumulating)
    "dq_decode_store": lambda bf16: _plus((OPS_PHILOX, OPS_DITHER), 4, 4),
    "dq_decode_accumulate": lambda bf16: _plus((OPS_PHILOX, OPS_DITHER), 5, 5),
    # code -> m/M (mask, fma), side scale, fma, fma, rint (half rate), add, fma, scale, add to the sum
    "nested_decode": lambda bf16: _plus((OPS_PHILOX, OPS_DITHER), 10, 11),
}


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


def kernel_source_hash():
    """sha256 over the kernel sources: a counter summary under profiles/ names the hash it
    was taken with, and its traffic figure is only passed on while the sources still match."""
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_1904_01197_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        if name.startswith("ndq_") and name.endswith((".hip", ".hpp")):
            h.update(name.encode())
            h.update(open(os.path.join(csrc, name), "rb").read())
    return h.hexdigest()[:16]


def measured_traffic(kernel_key):
    """(HBM bytes per launch from the committed rocprofv3 counter summary, its provenance) --
    (None, reason) when there is none or it was taken with other kernel sources."""
    path = os.path.join(ROOT, "profiles", "cfg5_hbm_traffic_pmc.txt")
    if not os.path.exists(path):
        return None, "no counter summary committed"
    text = open(path).read()
    m = re.search(r"^kernel_source_sha256_16\s*=\s*([0-9a-f]+)", text, re.M)
    if not m or m.group(1) != kernel_source_hash():
        return None, "profiles/cfg5_hbm_traffic_pmc.txt was taken with other kernel sources"
    m2 = re.search(r"^%s\s+traffic_bytes_per_launch\s*=\s*([0-9.eE+]+)" % re.escape(kernel_key), text, re.M)
    if not m2:
        return None, "kernel not in profiles/cfg5_hbm_traffic_pmc.txt"
    return float(m2.group(1)), "profiles/cfg5_hbm_traffic_pmc.txt (sources %s)" % m.group(1)


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
    from paper_1904_01197_amd.build import ensure_built
    ensure_built()   # compiles only when no built library is there
    ndq.lib()        # fail loudly if the HIP library cannot be loaded

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
        pipeline.encode_all(wl, dev, bufs, ds)
        preset = float(bufs.steps[0][0].item())
    torch.cuda.synchronize()
    gen_s = time.time() - t0

    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            ndq.ndq_aggregate([src], 1.0, dst)
        torch.cuda.synchronize()
        del src, dst

    # ---- whole path: time-based pre-warm, W warm-up steps, then exactly K timed steps ----
    if args.schedule == "fused":
        one_step = lambda: pipeline.step_fused(wl, dev, bufs, ds, preset)
    else:
        one_step = lambda: pipeline.step(wl, dev, bufs, ds, preset)
    if args.graph:
        eager_step = one_step
        cap = torch.cuda.Stream()
        cap.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(cap):
            eager_step()
        torch.cuda.current_stream().wait_stream(cap)
        torch.cuda.synchronize()
        hip_graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(hip_graph, stream=cap):
            eager_step()
        one_step = hip_graph.replay
    # The first few milliseconds after idle run at boost clocks, the next tens of
    # milliseconds well below the settled rate: a short timed region right after idle
    # measures the power controller, not the kernels.
    t_pre = time.perf_counter()
    prewarm_steps = 0
    while (time.perf_counter() - t_pre) * 1e3 < args.prewarm_ms:
        for _ in range(8):
            one_step()
        torch.cuda.synchronize()
        prewarm_steps += 8
    prewarm_ms = (time.perf_counter() - t_pre) * 1e3
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
    # the same steps once more with an event on the launch stream around each: the median
    step_marks = [torch.cuda.Event(enable_timing=True) for _ in range(max(args.steps, 20) + 1)]
    step_marks[0].record()
    for i in range(1, len(step_marks)):
        one_step()
        step_marks[i].record()
    torch.cuda.synchronize()
    step_ms = sorted(step_marks[i].elapsed_time(step_marks[i + 1]) for i in range(len(step_marks) - 1))
    ms_per_step_event_median = step_ms[len(step_ms) // 2]

    # ---- per-kernel durations, in place: events on the launch stream around
    # every library call of the step, averaged over --kernel-reps further steps ----
    bf16 = wl.dtype == "bf16"
    calls = []   # (kernel key, function, algorithmic bytes, algorithmic lane-ops)
    count = 0
    chain_bytes, chain_ops = 4 * n, (0.0, 0.0)
    decs = []
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
                                                           1.0, wl.bucket, ds[w], bufs.codes[w],
                                                           bufs.steps[w]))
            dkind = "nested_decode"
            dec_key, dec = "nested_decode_inplace_b%d" % bits, (
                lambda w=w, arg=arg, c=count: ndq.ndq_nested_decode(
                    bufs.codes[w], n, arg, 1.0, wl.bucket, bufs.steps[w], ds[w], bufs.total, 1.0 / c,
                    bufs.total, True))
        count += 1
        chain_bytes += (n * bits + 7) // 8 + 4 * K
        dec_ops = tuple(n * x for x in OPS[dkind](bf16))
        chain_ops = (chain_ops[0] + dec_ops[0], chain_ops[1] + dec_ops[1])
        own_step = wl.bucket != 0 or preset == 0.0
        enc_ops = tuple(n * x for x in OPS["nested_encode" if (kind != "dq" and arg & (arg - 1) == 0 and own_step)
                                           else "dq_encode"](bf16))
        calls.append((enc_key, enc, algorithmic_bytes("encode", n, bits, K, s_in), enc_ops))
        decs.append((dec_key, dec, algorithmic_bytes(dkind, n, bits, K, s_in), dec_ops))
    enc_bytes = sum(c[2] for c in calls)
    serial_bytes = enc_bytes + sum(d[2] for d in decs) + (8 * n if wl.out_scale != 1.0 else 0)
    fused_bytes = enc_bytes + chain_bytes
    if args.schedule == "fused":
        calls.append(("decode_chain_w%d" % wl.W,
                      lambda: pipeline.decode_chain_fused(wl, n, bufs, ds), chain_bytes, chain_ops))
    else:
        calls += decs
        if wl.out_scale != 1.0:
            calls.append(("aggregate_scale",
                          lambda: ndq.ndq_aggregate([bufs.total], wl.out_scale, bufs.total),
                          8 * n, (float(n), float(n))))
    reps = args.kernel_reps
    marks = [[torch.cuda.Event(enable_timing=True) for _ in range(len(calls) + 1)]
             for _ in range(reps)]
    torch.cuda.synchronize()
    for r in range(reps):
        for i, (_, fn, _, _) in enumerate(calls):
            marks[r][i].record()
            fn()
        marks[r][len(calls)].record()
    torch.cuda.synchronize()
    kernels, seen = [], {}
    for i, (key, _, nbytes, nops) in enumerate(calls):
        ms = sum(marks[r][i].elapsed_time(marks[r][i + 1]) for r in range(reps)) / reps
        if key in seen:
            rec = seen[key]
            rec["_ms_sum"] += ms
            rec["launches_per_step"] += 1
        else:
            rec = {"kernel": key, "launches_per_step": 1, "_ms_sum": ms,
                   "algorithmic_bytes": nbytes, "algorithmic_lane_ops": nops[0],
                   "algorithmic_lane_ops_weighted": nops[1]}
            seen[key] = rec
            kernels.append(rec)
    for rec in kernels:
        ms = rec.pop("_ms_sum") / rec["launches_per_step"]
        rec["avg_ms"] = round(ms, 5)
        rec["GBps"] = round(rec["algorithmic_bytes"] / (ms * 1e-3) / 1e9, 1)
        rec["Tops"] = round(rec["algorithmic_lane_ops"] / (ms * 1e-3) / 1e12, 2)
        rec["hbm_frac"] = round(rec["algorithmic_bytes"] / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
        rec["alu_frac"] = round(rec["algorithmic_lane_ops"] / (ms * 1e-3) / 1e12 / VALU_PEAK_TOPS, 4)

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

    # The brackets above put an event before and after every call; the event itself costs a few
    # microseconds between two kernels, which a 50 us encoder shows and a 200 us decoder hides.
    # Second figure per kernel: the same call launched back to back inside ONE pair of events,
    # an encoder reading another worker's vector every time (no input is still in a cache) and
    # writing to buffers of its own.
    alone_reps = max(4, min(args.kernel_reps, 24))
    for rec in kernels:
        group = [c for c in calls if c[0] == rec["kernel"]]
        if rec["kernel"].startswith(("dq_encode", "nested_encode")):
            w0 = next(w for w, c in enumerate(calls[:wl.W]) if c[0] == rec["kernel"])
            arg = wl.plan[w0][1]
            out_c, out_s = torch.empty_like(bufs.codes[w0]), torch.empty_like(bufs.steps[w0])
            if wl.plan[w0][0] == "dq":
                fns = [lambda w=w: ndq.ndq_dq_encode(dev[w], preset, arg, wl.bucket, ds[w0], out_c, out_s)
                       for w in range(wl.W)]
            else:
                fns = [lambda w=w: ndq.ndq_nested_encode(dev[w], preset, wl.fine_levels, arg, 1.0, wl.bucket,
                                                         ds[w0], out_c, out_s) for w in range(wl.W)]
        else:
            fns = [c[1] for c in group]
        turn = [0]

        def rotate(fns=fns, turn=turn):
            fns[turn[0] % len(fns)]()
            turn[0] += 1
        ms = timed(rotate, alone_reps)
        rec["alone_ms"] = round(ms, 5)
        rec["alone_GBps"] = round(rec["algorithmic_bytes"] / (ms * 1e-3) / 1e9, 1)
    one_step()     # the in-place decoders above have run out of turn: leave the buffers as a step leaves them
    torch.cuda.synchronize()

    dominant = max(kernels, key=lambda r: r["avg_ms"] * r["launches_per_step"])
    sec = dominant["avg_ms"] * 1e-3
    hbm_frac = dominant["algorithmic_bytes"] / sec / 1e9 / HBM_PEAK_GBS
    alu_frac = dominant["algorithmic_lane_ops"] / sec / 1e12 / VALU_PEAK_TOPS
    alu_frac_weighted = dominant["algorithmic_lane_ops_weighted"] / sec / 1e12 / VALU_PEAK_TOPS
    traffic, traffic_from = measured_traffic(dominant["kernel"])
    if hbm_frac >= alu_frac:
        roofline = {"bound": "hbm", "kernel": dominant["kernel"],
                    "achieved": round(hbm_frac * HBM_PEAK_GBS, 1), "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": round(hbm_frac, 4)}
    else:
        roofline = {"bound": "alu", "kernel": dominant["kernel"],
                    "achieved": round(alu_frac * VALU_PEAK_TOPS, 2),
                    "peak": round(VALU_PEAK_TOPS, 2), "unit": "Tlane-op/s (each operation of the method counted once)",
                    "frac": round(alu_frac, 4)}
    roofline.update({"traffic": traffic, "traffic_from": traffic_from,
                     "algorithmic_bytes_per_launch": dominant["algorithmic_bytes"],
                     "algorithmic_lane_ops_per_launch": dominant["algorithmic_lane_ops"],
                     "hbm_frac": round(hbm_frac, 4), "alu_frac": round(alu_frac, 4),
                     "alu_frac_weighted": round(alu_frac_weighted, 4),
                     "alu_frac_weighted_note": "half-rate instructions counted as 2 full-rate ones: how busy the "
                                               "issue ports are, not a credit",
                     "avg_launch_ms": dominant["avg_ms"]})
    step_bytes = sum(r["algorithmic_bytes"] * r["launches_per_step"] for r in kernels)

    # the other schedule, for context (same inputs, same outputs)
    other = "serial" if args.schedule == "fused" else "fused"
    other_fn = (lambda: pipeline.step(wl, dev, bufs, ds, preset)) if other == "serial" else (
        lambda: pipeline.step_fused(wl, dev, bufs, ds, preset))
    other_ms = timed(other_fn, max(3, args.steps // 3))

    extras = None
    if args.extras:
        extras = []

        def extra(name, fn, nbytes, note):
            ms = timed(fn, 10)
            extras.append({"kernel": name, "avg_ms": round(ms, 5), "algorithmic_bytes": nbytes,
                           "GBps": round(nbytes / (ms * 1e-3) / 1e9, 1),
                           "hbm_frac": round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4), "note": note})

        kind0, arg0 = wl.plan[0]
        b0 = ndq.ndq_code_bits(arg0)
        pk0 = (n * b0 + 7) // 8
        scratch = torch.empty(n, dtype=torch.float32, device="cuda")
        pipeline.encode_all(wl, dev, bufs, ds, preset)
        extra("dq_decode_half_b%d" % b0,
              lambda: ndq.ndq_dq_decode_half(bufs.codes[0], n, arg0, wl.bucket, bufs.steps[0], scratch),
              pk0 + 4 * K + 4 * n, "no dither regenerated; write-bound")
        hist = torch.empty(1 << b0, dtype=torch.int64, device="cuda")
        ent = torch.empty(1, dtype=torch.float64, device="cuda")
        extra("code_entropy_b%d" % b0, lambda: ndq.ndq_code_entropy(bufs.codes[0], n, b0, hist, ent),
              pk0, "histogram + entropy of worker 0's index stream")
        entropy0 = float(ent.item())
        # the same call on streams long enough to stream: the 4n bytes of `scratch` read as 2-bit
        # and as 8-bit codes (any byte is a valid group of such codes)
        raw = scratch.view(torch.uint8)
        hist2 = torch.empty(4, dtype=torch.int64, device="cuda")
        hist8 = torch.empty(256, dtype=torch.int64, device="cuda")
        ent8 = torch.empty(1, dtype=torch.float64, device="cuda")
        extra("code_entropy_b2_long", lambda: ndq.ndq_code_entropy(raw, 16 * n, 2, hist2, ent8), 4 * n,
              "a 2-bit stream of 16 n codes (4n bytes)")
        extra("code_entropy_b8_long", lambda: ndq.ndq_code_entropy(raw, 4 * n, 8, hist8, ent8), 4 * n,
              "an 8-bit stream of 4 n codes (4n bytes)")
        # bits per gradient element that each worker sends (Sec. 4, the kind of number in
        # Table 2, here on the synthetic workload): fixed-width codes, and what an ideal
        # entropy coder would leave of them; both with the 32-bit step of every bucket
        sent = []
        for w, (kind_w, arg_w) in enumerate(wl.plan):
            b_w = ndq.ndq_code_bits(arg_w)
            hist_w = torch.empty(1 << b_w, dtype=torch.int64, device="cuda")
            ndq.ndq_code_entropy(bufs.codes[w], n, b_w, hist_w, ent)
            sent.append({"worker": w, "kind": kind_w, "fixed_width_bits": round(b_w + 32.0 * K / n, 4),
                         "entropy_bits": round(float(ent.item()) + 32.0 * K / n, 4)})
        lv = 3
        c3, s3 = ndq.ndq_dq_encode(dev[0], 0.0, lv, wl.bucket, ds[0])
        dense = torch.empty(ndq.ndq_dense_bytes(n, lv), dtype=torch.uint8, device="cuda")
        back = torch.empty_like(c3)
        extra("dense_pack_L3", lambda: ndq.ndq_dense_pack(c3, n, lv, dense),
              c3.numel() + dense.numel(), "2-bit stream -> 1.6 bits per index")
        extra("dense_unpack_L3", lambda: ndq.ndq_dense_unpack(dense, n, lv, back),
              c3.numel() + dense.numel(), "")
        # the same transcoders on streams long enough to stream: the 4n bytes of `scratch` read as
        # n dense words (any word expands to twenty valid three-level codes), expanded and packed again
        n_long = 20 * n
        fixed_long = torch.empty(ndq.ndq_packed_bytes(n_long, 2), dtype=torch.uint8, device="cuda")
        dense_long = torch.empty(ndq.ndq_dense_bytes(n_long, lv), dtype=torch.uint8, device="cuda")
        extra("dense_unpack_L3_long", lambda: ndq.ndq_dense_unpack(raw, n_long, lv, fixed_long),
              raw.numel() + fixed_long.numel(), "20 n codes: 4n bytes dense -> 5n bytes at fixed width")
        extra("dense_pack_L3_long", lambda: ndq.ndq_dense_pack(fixed_long, n_long, lv, dense_long),
              fixed_long.numel() + dense_long.numel(), "")
        del fixed_long, dense_long
        ws = torch.empty(ndq.ndq_sqdiff_workspace() // 8, dtype=torch.float64, device="cuda")
        sq = torch.empty(1, dtype=torch.float64, device="cuda")
        other_f32 = torch.empty(n, dtype=torch.float32, device="cuda").normal_()
        extra("sqdiff", lambda: ndq.ndq_sqdiff(scratch, other_f32, ws, sq), 8 * n,
              "sigma_z^2 estimate, binary64, fixed order")
        if wl.W > 1 and wl.plan[1][0] == "nested":
            M1 = wl.plan[1][1]
            b1 = ndq.ndq_code_bits(M1)
            pk1 = (n * b1 + 7) // 8
            ca, sa = ndq.ndq_nested_encode(dev[1], preset, wl.fine_levels, M1, 0.9, wl.bucket, ds[1])
            extra("nested_encode_alpha0.9_%s_b%d" % (wl.dtype, b1),
                  lambda: ndq.ndq_nested_encode(dev[1], preset, wl.fine_levels, M1, 0.9, wl.bucket,
                                                ds[1], ca, sa),
                  n * s_in + pk1 + 4 * K, "shrinkage alpha = 0.9")
            extra("nested_decode_alpha0.9_inplace_b%d" % b1,
                  lambda: ndq.ndq_nested_decode(ca, n, M1, 0.9, wl.bucket, sa, ds[1], scratch, 1.0,
                                                scratch, True),
                  pk1 + 4 * K + 8 * n, "shrinkage alpha = 0.9, running sum updated in place")
        parts = [torch.empty(n, dtype=torch.float32, device="cuda").normal_() for _ in range(4)]
        extra("aggregate_w4", lambda: ndq.ndq_aggregate(parts, 0.25, scratch), 20 * n,
              "mean of four separately decoded gradients")
        del parts
        extras.append({"index_entropy_bits_worker0": round(entropy0, 4), "fixed_width_bits": b0})
        extras.append({"bits_per_element_sent": sent,
                       "mean_fixed_width_bits": round(sum(x["fixed_width_bits"] for x in sent) / wl.W, 4),
                       "mean_entropy_bits": round(sum(x["entropy_bits"] for x in sent) / wl.W, 4),
                       "uncompressed_bits": 32})
        del scratch, other_f32

    # ---- practical memory roof: a plain copy (ndq_aggregate, one input, scale 1) ----
    m = min(n, 1 << 27)
    spare = torch.empty(m, dtype=torch.float32, device="cuda")
    copy_ms = timed(lambda: ndq.ndq_aggregate([bufs.total[:m]], 1.0, spare), 10)
    copy_gbps = 8.0 * m / (copy_ms * 1e-3) / 1e9
    del spare

    # ---- CPU baseline: the oracle, as it stands -- and the whole step checked against it ----
    cpu, parity, diagnostics = None, None, None
    if not args.no_cpu:
        import oracle
        from oracle import pipeline as opipe
        ns = min(n, args.cpu_sample) // max(wl.bucket, 64) * max(wl.bucket, 64) or n
        sl = [h[:ns] for h in host]
        seeds = [workloads.dither_seed(wl, w) for w in range(wl.W)]
        ds_o = opipe.dithers(wl.W, seeds)
        oracle.lib()
        # what the GPU path leaves after one more step of the timed schedule
        one_step()
        torch.cuda.synchronize()
        got_out = bufs.total.cpu().numpy()
        got_codes = [c.cpu().numpy() for c in bufs.codes]
        got_steps = [x.cpu().numpy() for x in bufs.steps]
        # (i) one thread, one call per worker and direction over the sample
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
        ref_codes, ref_steps, ref_out, n_cmp = codes, steps, ref, ns
        # (ii) the same oracle on bucket-aligned slices, as many at a time as the host has cores for
        if wl.bucket > 0 and not wl.shared_step:
            threads = args.cpu_threads or min(16, os.cpu_count() or 1)
            c0 = time.perf_counter()
            ref_codes, ref_steps, ref_out = opipe.step_sliced(wl.plan, wl.fine_levels, wl.bucket, host, seeds,
                                                              wl.out_scale, threads=threads)
            all_s = time.perf_counter() - c0
            n_cmp = n
            cpu["all_cores"] = {"value": round(grad_bytes / all_s / 1e9, 5), "unit": "GB/s", "cores": threads,
                                "host_cores": os.cpu_count() or 0,
                                "sample": "all %d elements per worker, %.1f s, %d threads on bucket-aligned "
                                          "slices (the same C functions; they release the interpreter lock)"
                                          % (n, all_s, threads)}
            same = all(a[:x.size].tobytes() == x.tobytes() for a, x in zip(ref_codes, codes)) and \
                np.array_equal(ref_out[:ns], ref)
            cpu["all_cores"]["equals_single_thread_result_on_its_sample"] = bool(same)
            _, _, _, diagnostics = opipe.step_sliced(wl.plan, wl.fine_levels, wl.bucket, host, seeds, wl.out_scale,
                                                     threads=threads, diagnostics=True)
        # whole-step parity: every code byte, every step, every output of the n_cmp elements compared
        codes_ok = all(g[:(n_cmp * ndq.ndq_code_bits(arg) + 7) // 8].tobytes() ==
                       r[:(n_cmp * ndq.ndq_code_bits(arg) + 7) // 8].tobytes()
                       for g, r, (_, arg) in zip(got_codes, ref_codes, wl.plan))
        kb = ndq.ndq_num_buckets(n_cmp, wl.bucket)
        steps_ok = all(np.array_equal(g[:kb], r[:kb]) for g, r in zip(got_steps, ref_steps))
        diff = np.abs(got_out[:n_cmp].astype(np.float64) - ref_out[:n_cmp].astype(np.float64))
        step_sum = sum(r[:kb].astype(np.float64) for r in ref_steps)
        tol = (np.repeat(step_sum, wl.bucket)[:n_cmp] if wl.bucket else step_sum[0]) * 2.0 ** -20
        parity = {"parity_checked": True, "elements_compared_per_worker": int(n_cmp),
                  "codes_bit_exact": bool(codes_ok), "steps_bit_exact": bool(steps_ok),
                  "max_abs_diff_over_step": float(diff.max()) if n_cmp else 0.0,
                  "outputs_within_2^-20_step": bool(np.all(diff <= tol)),
                  "outputs_bit_exact": bool(np.array_equal(got_out[:n_cmp], ref_out[:n_cmp]))}
        if not (codes_ok and steps_ok and parity["outputs_within_2^-20_step"]):
            print("bench.py: the GPU path disagrees with the oracle: %r" % parity, file=sys.stderr)
            sys.exit(3)

    out = {
        "metric": "encode+decode+aggregate GB/s of gradient (and % of MI355X HBM peak) at n=2^27",
        "value": round(value, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "ms_per_step_event_median": round(ms_per_step_event_median, 4),
        "prewarm_ms": round(prewarm_ms, 1), "prewarm_steps": prewarm_steps, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": wl.name, "W": wl.W, "n_per_worker": n, "input_dtype": wl.dtype,
                   "bucket": wl.bucket, "schedule": args.schedule, "hip_graph": bool(args.graph), "plan": ["%s%d" % p for p in wl.plan],
                   "launches_per_step": sum(r["launches_per_step"] for r in kernels)},
        "gelem_per_s": round(wl.W * n / (ms_per_step * 1e-3) / 1e9, 3),
        "step_algorithmic_bytes": step_bytes,
        "step_hbm_frac_of_peak": round(step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
        "device_copy_GBps": round(copy_gbps, 1),
        "step_frac_of_device_copy": round(step_bytes / (ms_per_step * 1e-3) / 1e9 / copy_gbps, 4),
        "roofline": roofline,
        "cpu_baseline": cpu,
        "parity": parity,
        "clip_fraction": diagnostics["clip_fraction"] if diagnostics else None,
        "coset_error_fraction": diagnostics["coset_error_fraction"] if diagnostics else None,
        "kernels": kernels,
        "kernel_ms_sum_per_step": round(sum(r["avg_ms"] * r["launches_per_step"] for r in kernels), 4),
        "kernels_note": "avg_ms: an event before and after every call inside whole steps (carries about 3 us of event "
                        "handling per call); alone_ms: the call launched back to back inside one pair of events, "
                        "encoders reading another worker's vector each time",
        "other_schedule": {
            "schedule": other, "ms_per_step": round(other_ms, 4),
            "value": round(grad_bytes / (other_ms * 1e-3) / 1e9, 2),
            "step_algorithmic_bytes": serial_bytes if other == "serial" else fused_bytes,
            "step_hbm_frac_of_peak": round((serial_bytes if other == "serial" else fused_bytes)
                                           / (other_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)},
        "input_generation_s": round(gen_s, 1),
        "extras": extras,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
