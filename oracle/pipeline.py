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


def step_sliced(plan, fine_levels, bucket, grads, seeds, out_scale, threads=1, slice_buckets=256,
                diagnostics=False, step=0):
    """One whole iteration (encode every worker, decode chain) of a bucketed workload
    with the oracle as it stands, on bucket-aligned slices of the vectors: every step
    of the path is elementwise apart from the per-bucket max-norm and the dither
    depends on the element index only (the `offset` field), so the slices are
    independent and `threads` of them run side by side (the C functions release the
    interpreter lock).  Returns (codes, steps, out[, diagnostics]) for the whole
    vectors -- the same bytes as one call over everything.

    diagnostics: {"clip_fraction": [...per DQSG worker...], "coset_error_fraction":
    [...per nested worker...]} -- how many DQSG indices saturated, and how many
    coarse bins the nested decoder resolved wrongly (Thm 4's event)."""
    from concurrent.futures import ThreadPoolExecutor

    assert bucket > 0, "a shared step needs the whole vector's max-norm first"
    W, n = len(plan), grads[0].size
    bits = [oracle.code_bits(arg) for _, arg in plan]
    codes = [np.zeros(oracle.packed_bytes(n, b), dtype=np.uint8) for b in bits]
    steps = [np.empty(oracle.num_buckets(n, bucket), dtype=np.float32) for _ in plan]
    out = np.empty(n, dtype=np.float32)
    span = slice_buckets * bucket
    clipped = np.zeros(W, dtype=np.int64)
    wrong = np.zeros(W, dtype=np.int64)

    def work(lo):
        hi = min(lo + span, n)
        m = hi - lo
        ds = dithers(W, seeds, step=step, offset=lo)
        sl = [g[lo:hi] for g in grads]
        c, s, _ = encode_all(plan, fine_levels, bucket, False, sl, ds)
        for w in range(W):
            nb = (m * bits[w] + 7) // 8
            codes[w][lo * bits[w] // 8:lo * bits[w] // 8 + nb] = c[w][:nb]
            steps[w][lo // bucket:lo // bucket + s[w].size] = s[w]
        if diagnostics:
            ref, idx = decode_chain(plan, bucket, m, c, s, ds, out_scale, True)
            cl, wr = np.zeros(W, dtype=np.int64), np.zeros(W, dtype=np.int64)
            for w, (kind, arg) in enumerate(plan):
                q = oracle.fine_indices(sl[w], bucket, s[w], ds[w])
                if kind == "dq":
                    cl[w] = np.count_nonzero((q < -(arg // 2)) | (q > -(arg // 2) + arg - 1))
                else:
                    wr[w] = np.count_nonzero(idx[w] != q)
            out[lo:hi] = ref
            return cl, wr
        out[lo:hi] = decode_chain(plan, bucket, m, c, s, ds, out_scale)
        return None

    starts = list(range(0, n, span))
    if threads > 1:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            results = list(ex.map(work, starts))
    else:
        results = [work(lo) for lo in starts]
    if not diagnostics:
        return codes, steps, out
    for cl, wr in results:
        clipped += cl
        wrong += wr
    diag = {"clip_fraction": [float(clipped[w]) / n for w, (k, _) in enumerate(plan) if k == "dq"],
            "coset_error_fraction": [float(wrong[w]) / n for w, (k, _) in enumerate(plan) if k != "dq"]}
    return codes, steps, out, diag
