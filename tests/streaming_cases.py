"""Cases for the persistent ("streaming") encoder and chain-decoder kernels, run in
a process of its own by test_gpu_streaming.py with

    NDQ_STREAM_MIN_TILES_PER_WAVE=0  NDQ_STREAM_MAX_BLOCKS=3

so that vectors of a few hundred thousand elements -- small enough for the oracle
-- go through the persistent kernels on twelve waves: several tiles per wave (the
next tile's rows loaded into the registers of the rows just consumed, even and odd
tile counts), waves with one tile fewer, and a ragged last tile.  Everything is
compared with the oracle bit for bit.  (The persistent encoder serves bfloat16 input;
binary32 input takes the one-tile-per-wave encoder whatever the environment says, and
its cases here run through that.)
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import torch  # noqa: E402

import oracle  # noqa: E402
from oracle import pipeline as opipe  # noqa: E402
from paper_1904_01197_amd import ndq, workloads  # noqa: E402

F = np.float32


def make(n, dtype, seed, scale=0.01):
    rng = np.random.default_rng(seed)
    x = (rng.standard_t(3.0, n) * scale).astype(F)
    return workloads.f32_to_bf16_bits(x) if dtype == "bf16" else x


def to_dev(g):
    t = torch.from_numpy(g)
    if g.dtype == np.uint16:
        t = t.view(torch.bfloat16)
    return t.cuda()


def encoder_cases():
    count = 0
    for dtype in ("f32", "bf16"):
        tile = 2048 if dtype == "f32" else 4096
        for tiles, tail in ((12, 0), (37, 100), (50, tile - 8), (121, 64), (3, 8)):
            n = tiles * tile + tail
            g = make(n, dtype, seed=n)
            gf = workloads.bf16_bits_to_f32(g) if dtype == "bf16" else g
            g_d = to_dev(g)
            for offset in (0, 8 * tile):
                d_o, d_g = oracle.dither(11, 3, 2, offset), ndq.ndq_dither(11, 3, 2, offset)
                # max-norm found in registers (bucket == tile), one step for the whole vector found
                # by the max-norm pass (bucket 0, delta 0), and a preset step (bucket 0, delta > 0)
                for levels in (2, 3, 4, 16):
                    preset = float(F(2 * np.abs(gf).max() / (levels - 1)))
                    for bucket, delta in ((tile, 0.0), (0, 0.0), (0, preset)):
                        print("dq encode", dtype, n, offset, levels, bucket, delta, flush=True)
                        c_ref, s_ref = oracle.dq_encode(g, delta, levels, bucket, d_o)
                        codes, steps = ndq.ndq_dq_encode(g_d, delta, levels, bucket, d_g)
                        assert np.array_equal(steps.cpu().numpy(), s_ref)
                        assert codes.cpu().numpy().tobytes() == c_ref.tobytes()
                        count += 1
                    # the same preset step, handed over in device memory
                    print("dq encode with step", dtype, n, offset, levels, flush=True)
                    step_d = torch.tensor([preset], dtype=torch.float32, device="cuda")
                    codes, steps = ndq.ndq_dq_encode_with_step(g_d, step_d, levels, d_g)
                    assert np.array_equal(steps.cpu().numpy(), s_ref)
                    assert codes.cpu().numpy().tobytes() == c_ref.tobytes()
                    count += 1
                for M, levels in ((2, 4), (4, 16), (16, 64), (2, 2)):
                    preset = float(F(2 * np.abs(gf).max() / (levels - 1)))
                    for bucket, delta in ((tile, 0.0), (0, 0.0), (0, preset)):
                        print("nested encode", dtype, n, offset, M, levels, bucket, delta, flush=True)
                        c_ref, s_ref = oracle.nested_encode(g, delta, levels, M, bucket, d_o)
                        codes, steps = ndq.ndq_nested_encode(g_d, delta, levels, M, 1.0, bucket, d_g)
                        assert np.array_equal(steps.cpu().numpy(), s_ref)
                        assert codes.cpu().numpy().tobytes() == c_ref.tobytes()
                        count += 1
                    print("nested encode with step", dtype, n, offset, M, flush=True)
                    step_d = torch.tensor([preset], dtype=torch.float32, device="cuda")
                    codes, steps = ndq.ndq_nested_encode_with_step(g_d, step_d, M, 1.0, d_g)
                    assert np.array_equal(steps.cpu().numpy(), s_ref)
                    assert codes.cpu().numpy().tobytes() == c_ref.tobytes()
                    count += 1
    return count


def chain_cases():
    count = 0
    plans = [
        ((("dq", 4), ("nested", 2), ("nested", 2), ("nested", 2)), 4, 4096, 1.0, False),
        ((("dq", 16),) + (("nested", 4),) * 6, 16, 0, 1.0 / 7, True),
        ((("dq", 16),) * 5, 16, 2048, 0.2, False),
        ((("dq", 2), ("nested", 16), ("nested", 16)), 64, 1024, 1.0, False),
        ((("dq", 3),), 3, 0, 1.0, False),
        ((("dq", 4), ("dq", 2)), 4, 3072, 0.5, False),
    ]
    for plan, fine, bucket, scale, shared in plans:
        # whole tiles only (the hand-ordered fold with results staged through LDS: one, several
        # and unequal numbers of tiles per wave), then ragged ends (the plain fold)
        for n in (1024 * 12, 1024 * 40, 1024 * 129, 1024 * 37 + 100, 1024 * 150 + 1023, 1024 * 3 + 8):
            print("chain", plan, bucket, n, flush=True)
            rng = np.random.default_rng(n + len(plan))
            common = rng.standard_normal(n) * 0.01
            host = [(common + rng.standard_normal(n) * 0.002).astype(F) for _ in plan]
            seeds = [7 + w for w in range(len(plan))]
            # the call is a slice of a longer vector: its first element is element `offset` of the dither stream
            offset = 8 * (n % 4099)
            ds_o = opipe.dithers(len(plan), seeds, step=3, offset=offset)
            c_ref, s_ref, _ = opipe.encode_all(plan, fine, bucket, shared, host, ds_o)
            ref = opipe.decode_chain(plan, bucket, n, c_ref, s_ref, ds_o, scale)
            workers = [(torch.from_numpy(c_ref[w]).cuda(), torch.from_numpy(s_ref[w]).cuda(),
                        ndq.NDQ_WORKER_DQ if kind == "dq" else ndq.NDQ_WORKER_NESTED, arg,
                        ndq.ndq_dither(seeds[w], 3, w, offset)) for w, (kind, arg) in enumerate(plan)]
            out = ndq.ndq_decode_chain(workers, n, bucket, scale)
            assert np.array_equal(out.cpu().numpy(), ref), (plan, n)
            count += 1
    return count


if __name__ == "__main__":
    assert os.environ.get("NDQ_STREAM_MIN_TILES_PER_WAVE") == "0"
    assert torch.cuda.is_available()
    torch.cuda.set_device(0)
    e = encoder_cases()
    c = chain_cases()
    print("STREAMING_CASES_OK encoder=%d chain=%d" % (e, c), flush=True)
