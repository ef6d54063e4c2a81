"""One training iteration's communication path for a workload, on the GPU.

Workers (Algorithm 1 / Algorithm 2, "Workers"): every worker encodes its
gradient -- DQSG workers (group P1) with ndq_dq_encode, nested workers (group
P2) with ndq_nested_encode.  Server (Algorithm 2, "Server"): the P1 workers are
decoded into a running sum S; every P2 worker is then decoded against the
running mean S/count and added to S.  The result is scale * S.

Only library calls and buffer management happen here; all arithmetic runs in
the kernels of libndq.
"""
from dataclasses import dataclass, field
from typing import List, Optional

import torch

from . import ndq
from .workloads import Workload, dither_seed


@dataclass
class Buffers:
    """Device memory for one iteration of a workload, allocated once."""
    codes: List[torch.Tensor]
    steps: List[torch.Tensor]
    total: torch.Tensor                      # running sum S, then the result
    decoded: Optional[List[torch.Tensor]] = None   # per-worker g~ (separate-decode form)


def dithers(wl: Workload, step: int = 0, offset: int = 0):
    return [ndq.ndq_dither(dither_seed(wl, w), step, w, offset) for w in range(wl.W)]


def allocate(wl: Workload, n: int, device="cuda", separate=False) -> Buffers:
    codes, steps = [], []
    for kind, arg in wl.plan:
        bits = ndq.ndq_code_bits(arg)
        codes.append(torch.empty(ndq.ndq_packed_bytes(n, bits), dtype=torch.uint8, device=device))
        steps.append(torch.empty(ndq.ndq_num_buckets(n, wl.bucket), dtype=torch.float32,
                                 device=device))
    total = torch.empty(n, dtype=torch.float32, device=device)
    decoded = None
    if separate:
        decoded = [torch.empty(n, dtype=torch.float32, device=device) for _ in range(wl.W)]
    return Buffers(codes, steps, total, decoded)


def encode_all(wl: Workload, grads, bufs: Buffers, ds, preset_step: float = 0.0):
    """Worker side.  With wl.shared_step and no preset, worker 0 chooses the step and
    the other workers read it from worker 0's steps in device memory (Algorithm 1,
    initialisation: one Delta for all): no host round trip between the calls."""
    for w, (kind, arg) in enumerate(wl.plan):
        shared = wl.shared_step and w > 0 and preset_step == 0.0
        if kind == "dq" and shared:
            ndq.ndq_dq_encode_with_step(grads[w], bufs.steps[0], arg, ds[w], bufs.codes[w], bufs.steps[w])
        elif kind == "dq":
            ndq.ndq_dq_encode(grads[w], preset_step, arg, wl.bucket, ds[w], bufs.codes[w], bufs.steps[w])
        elif shared:
            ndq.ndq_nested_encode_with_step(grads[w], bufs.steps[0], arg, 1.0, ds[w], bufs.codes[w],
                                            bufs.steps[w])
        else:
            ndq.ndq_nested_encode(grads[w], preset_step, wl.fine_levels, arg, 1.0, wl.bucket, ds[w],
                                  bufs.codes[w], bufs.steps[w])


def decode_chain(wl: Workload, n: int, bufs: Buffers, ds):
    """Server side with a running sum: DQSG workers first, then the nested
    workers one after the other against the running mean."""
    count = 0
    S = bufs.total
    for w, (kind, arg) in enumerate(wl.plan):
        if kind == "dq":
            ndq.ndq_dq_decode(bufs.codes[w], n, arg, wl.bucket, bufs.steps[w], ds[w], S,
                              accumulate=count > 0)
        else:
            ndq.ndq_nested_decode(bufs.codes[w], n, arg, 1.0, wl.bucket, bufs.steps[w], ds[w], S,
                                  1.0 / count, S, accumulate=True)
        count += 1
    if wl.out_scale != 1.0:
        ndq.ndq_aggregate([S], wl.out_scale, S)
    return S


def decode_chain_fused(wl: Workload, n: int, bufs: Buffers, ds):
    """The same server loop as decode_chain() in ONE library call: the running
    sum stays in registers, codes are read once, the result is written once."""
    workers = [(bufs.codes[w], bufs.steps[w],
                ndq.NDQ_WORKER_DQ if kind == "dq" else ndq.NDQ_WORKER_NESTED, arg, ds[w])
               for w, (kind, arg) in enumerate(wl.plan)]
    return ndq.ndq_decode_chain(workers, n, wl.bucket, wl.out_scale, bufs.total)


def decode_separately(wl: Workload, n: int, bufs: Buffers, ds):
    """Server side of Algorithm 1 as printed: reconstruct every worker's gradient,
    then average them (all-DQSG workloads only)."""
    for w, (kind, arg) in enumerate(wl.plan):
        assert kind == "dq"
        ndq.ndq_dq_decode(bufs.codes[w], n, arg, wl.bucket, bufs.steps[w], ds[w], bufs.decoded[w])
    return ndq.ndq_aggregate(bufs.decoded, wl.out_scale, bufs.total)


def step(wl: Workload, grads, bufs: Buffers, ds, preset_step: float = 0.0):
    """One pass of the whole hot path: all encodes, all decodes, aggregation."""
    n = grads[0].numel()
    encode_all(wl, grads, bufs, ds, preset_step)
    return decode_chain(wl, n, bufs, ds)


def step_fused(wl: Workload, grads, bufs: Buffers, ds, preset_step: float = 0.0):
    """All encodes, then the fused server loop."""
    n = grads[0].numel()
    encode_all(wl, grads, bufs, ds, preset_step)
    return decode_chain_fused(wl, n, bufs, ds)


def to_device(wl: Workload, host_grads, device="cuda"):
    out = []
    for g in host_grads:
        t = torch.from_numpy(g)
        if wl.dtype == "bf16":
            t = t.view(torch.bfloat16)
        out.append(t.to(device))
    return out
