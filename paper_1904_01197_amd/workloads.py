"""Seeded synthetic gradient workloads.

The paper's experiments quantize training gradients of small image models; those
datasets are not available here, so the inputs follow the paper's own gradient
model instead (Sec. 3.1 Lemma 2 and Sec. 3.2: every worker's stochastic gradient
is a common vector plus independent zero-mean noise) and stand in for them.

This module only draws random inputs.  It holds none of the quantizer's
arithmetic and is the one piece of code the GPU path's tests and the CPU oracle's
tests both use, so that both sides see the same bytes.

Vectors are generated in independent chunks of 2**20 elements, each from its own
seed (config, stream, chunk), so any slice of a very long vector can be
regenerated without producing the rest.
"""
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import List, Tuple

import numpy as np

CHUNK = 1 << 20


@dataclass(frozen=True)
class Workload:
    """One benchmark configuration.

    ``plan`` has one entry per worker, in decoding order:
    ("dq", levels) for a DQSG worker (group P1) or ("nested", M) for an NDQSG
    worker (group P2); ``fine_levels`` fixes the step of every worker
    (step = 2*kappa/(fine_levels-1)).
    """
    name: str
    cfg: int
    W: int
    n: int
    dtype: str              # "f32" | "bf16"
    dist: str               # "normal" | "student_t3"
    common_scale: float     # std (or t3 scale) of the shared component
    indep_scale: float      # std (or t3 scale) of the per-worker component
    bucket: int             # 0 = one step for the whole vector
    fine_levels: int
    plan: Tuple[Tuple[str, int], ...]
    out_scale: float        # 1 = sum, 1/W = mean
    shared_step: bool = False   # all workers use worker 0's step (no buckets)
    seed_per_worker: bool = False  # dither seed = worker id (else 0)
    mix: Tuple[float, float] = (1.0, 1.0)  # g_w = mix[0]*common + mix[1]*indep_w


def _cfgs():
    c = {}
    c[1] = Workload("cfg1_dqsg_roundtrip", 1, 1, 65536, "f32", "normal", 0.01, 0.0, 0, 3,
                    (("dq", 3),), 1.0)
    # g2 = 0.9*g1 + sqrt(1-0.81)*N(0,0.01^2): worker 0 is the common part itself
    c[2] = Workload("cfg2_ndqsg_pair", 2, 2, 1 << 20, "f32", "normal", 0.01, 0.01, 0, 8,
                    (("dq", 8), ("nested", 4)), 1.0, shared_step=True)
    c[3] = Workload("cfg3_dqsg_w8", 3, 8, 25557032, "f32", "normal", 0.01, 0.005, 2048, 16,
                    tuple(("dq", 16) for _ in range(8)), 1.0 / 8, seed_per_worker=True)
    c[4] = Workload("cfg4_ndqsg_chain_w16", 4, 16, 11173962, "f32", "normal", 0.01, 0.003, 0,
                    16, (("dq", 16),) + tuple(("nested", 4) for _ in range(15)), 1.0 / 16,
                    shared_step=True)
    c[5] = Workload("cfg5_heavy_tail_bf16_w4", 5, 4, 1 << 27, "bf16", "student_t3", 1e-3, 1e-3,
                    4096, 4, (("dq", 4),) + tuple(("nested", 2) for _ in range(3)), 1.0,
                    mix=(0.8 ** 0.5, 0.2 ** 0.5))
    return c


CONFIGS = _cfgs()


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round to nearest even."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(
        np.float32)


def _draw(wl: Workload, stream: int, chunk: int, m: int, scale: float) -> np.ndarray:
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([wl.cfg, stream, chunk])))
    if wl.dist == "normal":
        x = rng.standard_normal(m, dtype=np.float32)
    else:
        x = rng.standard_t(3.0, m).astype(np.float32)
    return x * np.float32(scale)


def gradient_chunk(wl: Workload, worker: int, chunk: int, n: int = None) -> np.ndarray:
    """Elements [chunk*CHUNK, min((chunk+1)*CHUNK, n)) of worker `worker`.

    Returns float32, or uint16 bfloat16 bit patterns for a bf16 workload.
    """
    n = wl.n if n is None else n
    m = min(CHUNK, n - chunk * CHUNK)
    assert m > 0
    common = _draw(wl, 0, chunk, m, wl.common_scale)
    if wl.cfg == 2:
        # worker 0 = g1; worker 1 = 0.9*g1 + sqrt(0.19)*noise
        if worker == 0:
            g = common
        else:
            g = np.float32(0.9) * common + np.float32(0.19 ** 0.5) * _draw(
                wl, 1 + worker, chunk, m, wl.indep_scale)
    elif wl.indep_scale == 0.0:
        g = common
    else:
        g = np.float32(wl.mix[0]) * common + np.float32(wl.mix[1]) * _draw(
            wl, 1 + worker, chunk, m, wl.indep_scale)
    g = np.ascontiguousarray(g, dtype=np.float32)
    return f32_to_bf16_bits(g) if wl.dtype == "bf16" else g


def gradient(wl: Workload, worker: int, n: int = None, threads: int = 8) -> np.ndarray:
    """The first n elements (default: all) of worker `worker`'s gradient."""
    n = wl.n if n is None else n
    nchunks = (n + CHUNK - 1) // CHUNK
    out = np.empty(n, dtype=np.uint16 if wl.dtype == "bf16" else np.float32)

    def fill(c):
        out[c * CHUNK:min((c + 1) * CHUNK, n)] = gradient_chunk(wl, worker, c, n)

    if nchunks == 1:
        fill(0)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(fill, range(nchunks)))
    return out


def gradients(wl: Workload, n: int = None, threads: int = 8) -> List[np.ndarray]:
    return [gradient(wl, w, n, threads) for w in range(wl.W)]


def dither_seed(wl: Workload, worker: int) -> int:
    return worker if wl.seed_per_worker else 0
