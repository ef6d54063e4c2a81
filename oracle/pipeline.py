"""The same iteration as the GPU pipeline, spelled with oracle calls (test
infrastructure).  Workers encode; the server decodes the DQSG workers into a
running sum and each nested worker against the running mean (Algorithm 2)."""
import numpy as np

import oracle


def dithers(plan_len, seeds, step=0, offset=0):
    return [oracle.dither(seeds[w], step, w, offset) for w in range(plan_len)]


def encode_all(plan, fine_levels, bucket, shared_step, grads, ds, preset_step=0.0):
    codes, steps = [], []
    delta = preset_step
    for w, (kind, arg) in enumerate(plan):
        if kind == "dq":
            c, s = oracle.dq_encode(grads[w], delta, arg, bucket, ds[w])
        else:
            c, s = oracle.nested_encode(grads[w], delta, fine_levels, arg, bucket, ds[w])
        codes.append(c)
        steps.append(s)
        if shared_step and w == 0 and delta == 0.0:
            delta = float(s[0])
    return codes, steps, delta


def decode_chain(plan, bucket, n, codes, steps, ds, out_scale, want_indices=False):
    S = None
    count = 0
    indices = []
    for w, (kind, arg) in enumerate(plan):
        if kind == "dq":
            S = oracle.dq_decode(codes[w], n, arg, bucket, steps[w], ds[w], out=S)
            indices.append(None)
        else:
            scale = np.float32(1.0 / count)
            if want_indices:
                indices.append(oracle.coset_indices(codes[w], n, arg, bucket, steps[w], ds[w], S,
                                                    scale))
            S = oracle.nested_decode(codes[w], n, arg, bucket, steps[w], ds[w], S, scale, out=S)
        count += 1
    if out_scale != 1.0:
        S = oracle.aggregate([S], out_scale)
    return (S, indices) if want_indices else S


def decode_separately(plan, bucket, n, codes, steps, ds, out_scale):
    outs = [oracle.dq_decode(codes[w], n, arg, bucket, steps[w], ds[w])
            for w, (kind, arg) in enumerate(plan)]
    return oracle.aggregate(outs, out_scale), outs
