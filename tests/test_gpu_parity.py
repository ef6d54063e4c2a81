"""Parity of the HIP path (through the C ABI) against the CPU oracle, element by
element on the same seeded inputs.

Bar: packed codes and steps bit-exact; decoded floats within 2^-20 * Delta of
the oracle's (the arithmetic is one subtraction and one multiplication in
binary32 on values |q - v| <= 8.5 for the level counts used, so either
operation order stays inside that bound; in practice the two agree exactly).
"""
import os

import numpy as np
import pytest
import torch

import oracle
from oracle import pipeline as opipe
from paper_1904_01197_amd import ndq, pipeline, workloads

pytestmark = pytest.mark.gpu

F = np.float32
TOL = 2.0 ** -20


def _gpu():
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible: the gpu-marked tests need an MI355X")
    return torch.device("cuda:0")


def _to_dev(g):
    t = torch.from_numpy(g)
    if g.dtype == np.uint16:
        t = t.view(torch.bfloat16)
    return t.to(_gpu())


def _make(n, dtype, seed, scale=0.01, heavy=False):
    rng = np.random.default_rng(seed)
    x = rng.standard_t(3.0, n) if heavy else rng.standard_normal(n)
    x = (x * scale).astype(F)
    return workloads.f32_to_bf16_bits(x) if dtype == "bf16" else x


def _steps_per_elem(steps, bucket, n):
    if bucket == 0:
        return np.full(n, steps[0], dtype=np.float64)
    return np.repeat(steps.astype(np.float64), bucket)[:n]


def _assert_values_close(got, ref, steps, bucket, n, mult=1.0):
    tol = _steps_per_elem(steps, bucket, n) * TOL * mult
    diff = np.abs(got.astype(np.float64) - ref.astype(np.float64))
    bad = np.nonzero(diff > tol)[0]
    assert bad.size == 0, "first mismatch at %d: %r vs %r" % (bad[0], got[bad[0]], ref[bad[0]])


SIZES = [1, 3, 63, 64, 65, 255, 2047, 2048, 2049, 4096 + 7, 3 * 4096, 5 * 2048 + 1234, 70001]


# --------------------------------------------------------------------------
# a2 + a3 + a4: scale, quantize, pack  /  a6: unpack + reconstruct
# --------------------------------------------------------------------------

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("levels,bucket,preset", [
    (3, 0, False), (3, 0, True), (2, 64, False), (4, 4096, False), (5, 128, False),
    (8, 2048, False), (16, 2048, False), (16, 2112, False), (33, 8192, False), (100, 0, False),
    (256, 1024, False), (255, 12288, False), (4, 512, False), (3, 1024, False), (4, 16384, False),
    (5, 4096, False)])
def test_dq_encode_decode_matches_oracle(dtype, levels, bucket, preset):
    for n in SIZES:
        g = _make(n, dtype, seed=n + levels)
        gf = workloads.bf16_bits_to_f32(g) if dtype == "bf16" else g
        delta = float(F(2 * np.abs(gf).max() / (levels - 1))) if preset else 0.0
        d_o = oracle.dither(5, 7, 2)
        d_g = ndq.ndq_dither(5, 7, 2, 0)
        c_ref, s_ref = oracle.dq_encode(g, delta, levels, bucket, d_o)
        codes, steps = ndq.ndq_dq_encode(_to_dev(g), delta, levels, bucket, d_g)
        assert np.array_equal(steps.cpu().numpy(), s_ref), (n, "steps")
        assert codes.cpu().numpy().tobytes() == c_ref.tobytes(), (n, "codes")
        ref = oracle.dq_decode(c_ref, n, levels, bucket, s_ref, d_o)
        out = ndq.ndq_dq_decode(codes, n, levels, bucket, steps, d_g)
        _assert_values_close(out.cpu().numpy(), ref, s_ref, bucket, n)
        # accumulate adds into an existing buffer
        base = _make(n, "f32", seed=n + 1)
        acc = ndq.ndq_dq_decode(codes, n, levels, bucket, steps, d_g, _to_dev(base), True)
        ref_acc = oracle.dq_decode(c_ref, n, levels, bucket, s_ref, d_o, out=base.copy())
        _assert_values_close(acc.cpu().numpy(), ref_acc, s_ref, bucket, n, mult=2.0)
        assert np.array_equal(out.cpu().numpy(), ref)          # in fact bit-exact
        assert np.array_equal(acc.cpu().numpy(), ref_acc)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_encode_with_a_step_in_device_memory_matches_oracle(dtype):
    """One Delta for all workers (Algorithm 1 / 2, initialisation), handed over as a
    device pointer: the codes are those of the oracle's preset-step encoder; worker 0's
    own steps_out serves as step_in; a zero step gives index 0 everywhere."""
    dev = _gpu()
    for n in SIZES:
        if n == 0:
            continue
        g0, g1 = _make(n, dtype, seed=n + 31), _make(n, dtype, seed=n + 32)
        g1f = workloads.bf16_bits_to_f32(g1) if dtype == "bf16" else g1
        d0_o, d1_o = oracle.dither(9, 4, 0), oracle.dither(9, 4, 1)
        d0_g, d1_g = ndq.ndq_dither(9, 4, 0, 0), ndq.ndq_dither(9, 4, 1, 0)
        for levels, M in ((4, 2), (16, 4), (100, 3), (256, 16)):
            _, s0_ref = oracle.dq_encode(g0, 0.0, levels, 0, d0_o)
            _, steps0 = ndq.ndq_dq_encode(_to_dev(g0), 0.0, levels, 0, d0_g)
            assert np.array_equal(steps0.cpu().numpy(), s0_ref)
            delta = float(s0_ref[0])
            # worker 1 (values partly outside worker 0's range: it saturates / wraps as the oracle does)
            c_ref, s_ref = oracle.dq_encode(g1, delta, levels, 0, d1_o)
            codes, steps = ndq.ndq_dq_encode_with_step(_to_dev(g1), steps0, levels, d1_g)
            assert np.array_equal(steps.cpu().numpy(), s_ref), (n, levels)
            assert codes.cpu().numpy().tobytes() == c_ref.tobytes(), (n, levels)
            for alpha in (1.0, 0.75):
                c_ref, s_ref = oracle.nested_encode(g1, delta, levels, M, 0, d1_o, alpha=alpha)
                codes, steps = ndq.ndq_nested_encode_with_step(_to_dev(g1), steps0, M, alpha, d1_g)
                assert np.array_equal(steps.cpu().numpy(), s_ref), (n, M, alpha)
                assert codes.cpu().numpy().tobytes() == c_ref.tobytes(), (n, M, alpha)
            # step_in and steps_out are the same address
            inout = steps0.clone()
            codes, steps = ndq.ndq_dq_encode_with_step(_to_dev(g1), inout, levels, d1_g, steps_out=inout)
            c_ref, _ = oracle.dq_encode(g1, delta, levels, 0, d1_o)
            assert codes.cpu().numpy().tobytes() == c_ref.tobytes() and float(inout.item()) == delta
        # a zero step (what an all-zero vector's encoder sends): fine index 0 everywhere
        zero = torch.zeros(1, dtype=torch.float32, device=dev)
        codes, steps = ndq.ndq_dq_encode_with_step(_to_dev(g1), zero, 5, d1_g)
        want = oracle.pack(np.full(n, 2, dtype=np.uint32), 3)
        assert codes.cpu().numpy().tobytes() == want.tobytes() and float(steps.item()) == 0.0
        codes, steps = ndq.ndq_nested_encode_with_step(_to_dev(g1), zero, 4, 1.0, d1_g)
        assert not codes.cpu().numpy().any() and float(steps.item()) == 0.0
        assert np.abs(g1f).max() > 0


@pytest.mark.parametrize("levels,bucket", [(3, 0), (5, 2048), (9, 64), (16, 4096), (256, 2112), (7, 0)])
def test_half_dithered_decode_matches_oracle(levels, bucket):
    """Reconstruction without dither subtraction (stochastic / ternary quantizers'
    rule): out = Delta * q, bit-exact."""
    for n in SIZES:
        g = _make(n, "f32", seed=n + levels)
        d_o, d_g = oracle.dither(2, 3, 4), ndq.ndq_dither(2, 3, 4, 0)
        c_ref, s_ref = oracle.dq_encode(g, 0.0, levels, bucket, d_o)
        codes, steps = ndq.ndq_dq_encode(_to_dev(g), 0.0, levels, bucket, d_g)
        ref = oracle.dq_decode_half(c_ref, n, levels, bucket, s_ref)
        out = ndq.ndq_dq_decode_half(codes, n, levels, bucket, steps)
        assert np.array_equal(out.cpu().numpy(), ref), n
        base = _make(n, "f32", seed=n + 9)
        ref_acc = oracle.dq_decode_half(c_ref, n, levels, bucket, s_ref, out=base.copy())
        acc = ndq.ndq_dq_decode_half(codes, n, levels, bucket, steps, _to_dev(base), True)
        assert np.array_equal(acc.cpu().numpy(), ref_acc), n


def test_config1_dqsg_roundtrip():
    """n = 65,536 fp32 N(0, 0.01^2), 3 levels (2-bit codes), Delta = 2 max|g|/(3-1),
    dither (seed 0, step 0): encode -> pack -> unpack -> decode."""
    wl = workloads.CONFIGS[1]
    g = workloads.gradient(wl, 0)
    d_o, d_g = oracle.dither(0, 0, 0), ndq.ndq_dither(0, 0, 0, 0)
    c_ref, s_ref = oracle.dq_encode(g, 0.0, 3, 0, d_o)
    assert s_ref[0] == F(np.abs(g).max())
    codes, steps = ndq.ndq_dq_encode(_to_dev(g), 0.0, 3, 0, d_g)
    assert steps.cpu().numpy()[0] == s_ref[0]
    assert codes.cpu().numpy().tobytes() == c_ref.tobytes()
    assert codes.numel() == 65536 * 2 // 8
    ref = oracle.dq_decode(c_ref, wl.n, 3, 0, s_ref, d_o)
    out = ndq.ndq_dq_decode(codes, wl.n, 3, 0, steps, d_g).cpu().numpy()
    _assert_values_close(out, ref, s_ref, 0, wl.n)
    assert np.abs(out - g).max() <= s_ref[0] * (0.5 + 2.0 ** -18)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_absmax_matches_oracle(dtype):
    for n in SIZES:
        for bucket in (0, 64, 2048, 4096, 6400):
            g = _make(n, dtype, seed=n)
            ref = oracle.absmax(g, bucket)
            got = ndq.ndq_absmax(_to_dev(g), bucket).cpu().numpy()
            assert np.array_equal(got, ref), (n, bucket)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_absmax_of_buckets_that_span_many_tiles(dtype):
    """Whole-vector and very large buckets take the kernel whose workgroups stride over a
    bucket's tiles; the maximum sits in a different place for every bucket, the last
    bucket is short and ragged, and the encoder that reads those steps must agree too."""
    n = 5 * (1 << 18) + 4096 * 3 + 77 * 8
    g = _make(n, dtype, seed=31)
    gf = workloads.bf16_bits_to_f32(g) if dtype == "bf16" else g
    peak = F(np.abs(gf).max() * 3)
    for b, pos in enumerate((5, (1 << 18) + 262143, 2 * (1 << 18) + 131072, 3 * (1 << 18) + 70001,
                             4 * (1 << 18) + 1, n - 1)):
        val = np.array([peak * F(1 + b)], dtype=F)
        g[pos] = workloads.f32_to_bf16_bits(val)[0] if dtype == "bf16" else val[0]
    gd = _to_dev(g)
    d_o, d_g = oracle.dither(2, 0, 1), ndq.ndq_dither(2, 0, 1, 0)
    for bucket in (0, 1 << 18, 1 << 19):
        ref = oracle.absmax(g, bucket)
        assert np.array_equal(ndq.ndq_absmax(gd, bucket).cpu().numpy(), ref), bucket
        c_ref, s_ref = oracle.dq_encode(g, 0.0, 16, bucket, d_o)
        codes, steps = ndq.ndq_dq_encode(gd, 0.0, 16, bucket, d_g)
        assert np.array_equal(steps.cpu().numpy(), s_ref), bucket
        assert codes.cpu().numpy().tobytes() == c_ref.tobytes(), bucket


def test_degenerate_inputs():
    dev = _gpu()
    d_o, d_g = oracle.dither(1, 1, 1), ndq.ndq_dither(1, 1, 1, 0)
    # all-zero and vanishing buckets are sent as step 0 and decode to zero
    n = 4096
    g = np.zeros(n, dtype=F)
    g[2048:] = 1e-38
    g[100] = 0.5
    c_ref, s_ref = oracle.dq_encode(g, 0.0, 4, 1024, d_o)
    codes, steps = ndq.ndq_dq_encode(_to_dev(g), 0.0, 4, 1024, d_g)
    assert np.array_equal(steps.cpu().numpy(), s_ref) and s_ref[1] == 0 and s_ref[2] == 0
    assert codes.cpu().numpy().tobytes() == c_ref.tobytes()
    out = ndq.ndq_dq_decode(codes, n, 4, 1024, steps, d_g).cpu().numpy()
    assert np.array_equal(out, oracle.dq_decode(c_ref, n, 4, 1024, s_ref, d_o))
    assert np.all(out[1024:] == 0)
    # values far outside a preset range saturate
    g = np.array([1e30, -1e30, 3.0, -3.0, 0.1, 0.0, 2.49, -2.51] * 8, dtype=F)
    c_ref, s_ref = oracle.dq_encode(g, 1.0, 5, 0, d_o)
    codes, steps = ndq.ndq_dq_encode(_to_dev(g), 1.0, 5, 0, d_g)
    assert codes.cpu().numpy().tobytes() == c_ref.tobytes()
    # empty input is a no-op
    empty = torch.empty(0, dtype=torch.float32, device=dev)
    codes, steps = ndq.ndq_dq_encode(empty, 1.0, 4, 0, d_g)
    assert codes.numel() == 0
    ndq.ndq_dq_decode(codes, 0, 4, 0, steps, d_g, empty)


def test_slices_with_offset_reproduce_the_whole():
    """A bucket-aligned slice with the matching dither offset gives the bytes of
    the whole vector (how the path shards)."""
    n, bucket, levels = 5 * 4096, 4096, 16
    g = _make(n, "bf16", seed=3)
    gd = _to_dev(g)
    codes, steps = ndq.ndq_dq_encode(gd, 0.0, levels, bucket, ndq.ndq_dither(9, 1, 4, 0))
    lo, hi = 4096, 4 * 4096
    c2, s2 = ndq.ndq_dq_encode(gd[lo:hi], 0.0, levels, bucket, ndq.ndq_dither(9, 1, 4, lo))
    assert torch.equal(c2[:(hi - lo) // 2], codes[lo // 2:hi // 2])
    assert torch.equal(s2, steps[1:4])
    c_ref, _ = oracle.dq_encode(g[lo:hi], 0.0, levels, bucket, oracle.dither(9, 1, 4, lo))
    assert c2.cpu().numpy().tobytes() == c_ref.tobytes()
    # large offsets exercise the high counter word
    big = (1 << 36) + 4096
    c3, _ = ndq.ndq_dq_encode(gd[:8192], 0.0, levels, bucket, ndq.ndq_dither(9, 1, 4, big))
    c_ref, _ = oracle.dq_encode(g[:8192], 0.0, levels, bucket, oracle.dither(9, 1, 4, big))
    assert c3.cpu().numpy().tobytes() == c_ref.tobytes()


def test_argument_errors_are_reported_not_launched():
    dev = _gpu()
    g = torch.zeros(4096, dtype=torch.float32, device=dev)
    d = ndq.ndq_dither(0, 0, 0, 0)
    for bad in (lambda: ndq.ndq_dq_encode(g, 0.0, 1, 0, d),
                lambda: ndq.ndq_dq_encode(g, 0.0, 257, 0, d),
                lambda: ndq.ndq_nested_encode(g, 0.0, 4, 1, 1.0, 0, d),
                lambda: ndq.ndq_nested_encode(g, 0.0, 4, 300, 1.0, 0, d),
                lambda: ndq.ndq_nested_encode(g, 0.0, 4, 4, 1.5, 0, d)):
        with pytest.raises(ndq.NdqError) as e:
            bad()
        assert e.value.rc == ndq.NDQ_EINVAL
    with pytest.raises(ndq.NdqError) as e:
        ndq.ndq_dq_encode(g, 0.0, 4, 100, d)                 # bucket not a multiple of 64
    assert e.value.rc == ndq.NDQ_EALIGN
    with pytest.raises(ndq.NdqError) as e:
        ndq.ndq_dq_encode(g[1:], 0.0, 4, 0, d)               # misaligned gradient
    assert e.value.rc == ndq.NDQ_EALIGN
    with pytest.raises(ndq.NdqError) as e:
        ndq.ndq_dq_encode(g, 0.0, 4, 0, ndq.ndq_dither(0, 0, 0, 2))
    assert e.value.rc == ndq.NDQ_EALIGN
    codes, steps = ndq.ndq_nested_encode(g, 1.0, 4, 4, 1.0, 0, d)
    buf = torch.zeros(4096 + 8, dtype=torch.float32, device=dev)
    with pytest.raises(ndq.NdqError) as e:                   # partially overlapping side / out
        ndq.ndq_nested_decode(codes, 4096, 4, 1.0, 0, steps, d, buf[:4096], 1.0, buf[4:4100], True)
    assert e.value.rc == ndq.NDQ_EINVAL
    torch.cuda.synchronize()


# --------------------------------------------------------------------------
# a5 + a7: nested encode, coset decode with side information
# --------------------------------------------------------------------------

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("M,levels,bucket", [
    (2, 4, 4096), (4, 16, 0), (4, 8, 2048), (3, 7, 0), (8, 64, 512), (5, 16, 2112), (16, 256, 0),
    (256, 256, 64), (7, 9, 8192), (2, 4, 16384), (4, 16, 1024)])
def test_nested_encode_decode_matches_oracle(dtype, M, levels, bucket):
    for n in SIZES:
        g = _make(n, dtype, seed=n + M, heavy=(dtype == "bf16"))
        gf = workloads.bf16_bits_to_f32(g) if dtype == "bf16" else g
        rng = np.random.default_rng(n)
        side = (gf + rng.standard_normal(n).astype(F) * F(0.3 * np.abs(gf).max() / levels)).astype(F)
        d_o, d_g = oracle.dither(3, 2, 9), ndq.ndq_dither(3, 2, 9, 0)
        c_ref, s_ref = oracle.nested_encode(g, 0.0, levels, M, bucket, d_o)
        codes, steps = ndq.ndq_nested_encode(_to_dev(g), 0.0, levels, M, 1.0, bucket, d_g)
        assert np.array_equal(steps.cpu().numpy(), s_ref), (n, "steps")
        assert codes.cpu().numpy().tobytes() == c_ref.tobytes(), (n, "codes")
        side_d = _to_dev(side)
        for scale in (1.0, 0.5, 1.0 / 3.0):
            ref = oracle.nested_decode(c_ref, n, M, bucket, s_ref, d_o, side, scale)
            out = ndq.ndq_nested_decode(codes, n, M, 1.0, bucket, steps, d_g, side_d, scale)
            # the coset representative is an integer decision: it must agree exactly
            assert np.array_equal(out.cpu().numpy(), ref), (n, scale)
        # running-sum forms: separate buffer, and in place (out is side)
        base = _make(n, "f32", seed=n + 2)
        ref_acc = oracle.nested_decode(c_ref, n, M, bucket, s_ref, d_o, side, 0.5, out=base.copy())
        acc = ndq.ndq_nested_decode(codes, n, M, 1.0, bucket, steps, d_g, side_d, 0.5, _to_dev(base), True)
        assert np.array_equal(acc.cpu().numpy(), ref_acc)
        ref_inp = side.copy()
        oracle.nested_decode(c_ref, n, M, bucket, s_ref, d_o, side, 0.5, out=ref_inp)
        s_inp = _to_dev(side)
        ndq.ndq_nested_decode(codes, n, M, 1.0, bucket, steps, d_g, s_inp, 0.5, s_inp, True)
        assert np.array_equal(s_inp.cpu().numpy(), ref_inp)


@pytest.mark.parametrize("bucket", [0, 2048])
def test_exact_rounding_ties_go_to_the_even_index_on_the_gpu_too(bucket):
    """Every element is built so that g/Delta + v is exactly an integer plus one half (the
    step is exactly 1: max|g| = 2 with 5 levels): the encoders must break the tie like
    rint, towards the even index.  Exercises the magic-constant rounding of the nested
    encoder, the DQSG encoder, and the decoders on the codes that result."""
    n = 3 * 2048 + 192
    d_o, d_g = oracle.dither(5, 1, 3), ndq.ndq_dither(5, 1, 3, 0)
    v = oracle.unit_dithers(d_o, n).astype(np.float64)
    rng = np.random.default_rng(8)
    half = rng.choice(np.array([-1.5, -0.5, 0.5, 1.5]), n)
    g = (half - v).astype(F)
    assert np.array_equal(g.astype(np.float64) + v, half)          # exact ties in binary32
    g[::2048] = F(2.0)                                             # pins every bucket's max-norm
    g[-1] = F(-2.0)
    gd = _to_dev(g)
    for levels, M in ((5, 2), (5, 4), (5, 8)):
        c_ref, s_ref = oracle.nested_encode(g, 0.0, levels, M, bucket, d_o)
        assert np.all(s_ref == F(1.0))
        codes, steps = ndq.ndq_nested_encode(gd, 0.0, levels, M, 1.0, bucket, d_g)
        assert np.array_equal(steps.cpu().numpy(), s_ref)
        assert codes.cpu().numpy().tobytes() == c_ref.tobytes(), (levels, M)
        # the tie rule itself: the index is the even neighbour
        q = oracle.fine_indices(g, bucket, s_ref, d_o)
        ties = np.ones(n, bool); ties[::2048] = False; ties[-1] = False
        assert np.all(q[ties] % 2 == 0) and np.array_equal(np.abs(q[ties] - half[ties]), np.full(ties.sum(), 0.5))
        side = (g + F(0.25)).astype(F)
        ref = oracle.nested_decode(c_ref, n, M, bucket, s_ref, d_o, side, 1.0)
        out = ndq.ndq_nested_decode(codes, n, M, 1.0, bucket, steps, d_g, _to_dev(side), 1.0)
        assert np.array_equal(out.cpu().numpy(), ref)
    c_ref, s_ref = oracle.dq_encode(g, 0.0, 5, bucket, d_o)
    codes, steps = ndq.ndq_dq_encode(gd, 0.0, 5, bucket, d_g)
    assert codes.cpu().numpy().tobytes() == c_ref.tobytes()
    assert np.array_equal(ndq.ndq_dq_decode(codes, n, 5, bucket, steps, d_g).cpu().numpy(),
                          oracle.dq_decode(c_ref, n, 5, bucket, s_ref, d_o))
    # DQSG with other odd level counts (max-norm (L-1)/2: step exactly 1; -q_min odd and even),
    # every element a tie, the extreme ones sitting half a step inside the outermost level
    for levels in (3, 7, 9, 33):
        kap = (levels - 1) // 2
        halves = np.arange(-kap, kap) + 0.5
        gl = (rng.choice(halves, n) - v).astype(F)
        assert np.array_equal(gl.astype(np.float64) + v, np.round(gl.astype(np.float64) + v - 0.5) + 0.5)
        gl[::2048] = F(kap)
        gl[-1] = F(-kap)
        c_ref, s_ref = oracle.dq_encode(gl, 0.0, levels, bucket, d_o)
        assert np.all(s_ref == F(1.0))
        codes, steps = ndq.ndq_dq_encode(_to_dev(gl), 0.0, levels, bucket, d_g)
        assert np.array_equal(steps.cpu().numpy(), s_ref)
        assert codes.cpu().numpy().tobytes() == c_ref.tobytes(), levels
        unpacked = oracle.unpack(c_ref, n, oracle.code_bits(levels))
        assert unpacked.min() == 0 and unpacked.max() == levels - 1          # both outermost levels occur
        # a third of the elements at +-max|g| under every dither value, and the same with a
        # max-norm whose step and reciprocal both round (the closest the index comes to overload)
        for kappa in (F(kap), F(kap) * F(1.2345678)):
            gx = (rng.uniform(-1.0, 1.0, n) * float(kappa)).astype(F)
            gx[::3] = kappa
            gx[1::3] = -kappa
            c_ref, s_ref = oracle.dq_encode(gx, 0.0, levels, bucket, d_o)
            codes, steps = ndq.ndq_dq_encode(_to_dev(gx), 0.0, levels, bucket, d_g)
            assert np.array_equal(steps.cpu().numpy(), s_ref)
            assert codes.cpu().numpy().tobytes() == c_ref.tobytes(), (levels, float(kappa))


@pytest.mark.parametrize("M", [3, 5, 6, 7, 12])
def test_coset_decisions_at_and_next_to_exact_ties_for_any_nesting_ratio(M):
    """Side information placed midway between two coset points, or a few units in the last
    place beside it: (y/Delta + v - m)/M is a half-integer or next to one.  The kernels divide
    by M with a rounded reciprocal and must fall back to the true division there.  For every
    element the y (within 16 ulps of the tie) is taken at which the reciprocal product and the
    division round to different integers, where there is one: a kernel without the fallback
    fails on those."""
    n, levels, bucket = 3 * 1024 + 512 + 64, 5, 0
    d_o, d_g = oracle.dither(11, 4, 6), ndq.ndq_dither(11, 4, 6, 0)
    v = oracle.unit_dithers(d_o, n).astype(F)
    rng = np.random.default_rng(M)
    g = (rng.uniform(-1.9, 1.9, n)).astype(F)
    g[0] = F(2.0)                                                   # max-norm 2, 5 levels: step exactly 1
    codes_ref, steps_ref = oracle.nested_encode(g, 0.0, levels, M, bucket, d_o)
    assert steps_ref[0] == F(1.0)
    m = oracle.unpack(codes_ref, n, oracle.code_bits(M)).astype(F)
    j = rng.integers(-100, 101, n).astype(np.float64)
    y = (M * j + M / 2.0 + m.astype(np.float64) - v.astype(np.float64)).astype(F)
    tie_bits, found = y.view(np.int32).copy(), np.zeros(n, bool)
    for off in range(-16, 17):
        cand = (tie_bits + off).view(F)
        c = (cand.astype(np.float64) + v.astype(np.float64)).astype(F)          # fma(y, 1/Delta = 1, v)
        diff = (c - m).astype(F)
        differ = np.rint((diff / F(M)).astype(F)) != np.rint((diff * (F(1.0) / F(M))).astype(F))
        take = differ & ~found
        y[take] = cand[take]
        found |= take
    if M != 5:      # (the product with the rounded 1/5 happens to agree with the quotient near these ties)
        assert found.sum() > 100
    codes, steps = ndq.ndq_nested_encode(_to_dev(g), 0.0, levels, M, 1.0, bucket, d_g)
    assert codes.cpu().numpy().tobytes() == codes_ref.tobytes()
    ref = oracle.nested_decode(codes_ref, n, M, bucket, steps_ref, d_o, y, 1.0)
    out = ndq.ndq_nested_decode(codes, n, M, 1.0, bucket, steps, d_g, _to_dev(y), 1.0)
    assert np.array_equal(out.cpu().numpy(), ref)
    # in place, as the running sum of the server loop
    S = _to_dev(y.copy())
    ndq.ndq_nested_decode(codes, n, M, 1.0, bucket, steps, d_g, S, 1.0, S, True)
    ref_S = y.copy()
    oracle.nested_decode(codes_ref, n, M, bucket, steps_ref, d_o, y, 1.0, out=ref_S)
    assert np.array_equal(S.cpu().numpy(), ref_S)
    # the fused server loop has its own fast pass / repeat logic per row of eight elements.  Side
    # information some 10^5 steps away from the origin widens the doubtful zone around a tie to
    # a few per cent of the unit, so that most rows are repeated with the division
    big = (rng.uniform(-4.0e5, 4.0e5, n)).astype(F)
    dq_ref, dq_steps = oracle.dq_encode(big, 0.0, 16, bucket, d_o)
    first = oracle.dq_decode(dq_ref, n, 16, bucket, dq_steps, d_o)
    approx = (first.astype(np.float64) + v - m) / M
    doubtful = np.abs(np.abs(approx - np.rint(approx)) - 0.5) < 2.0 ** -21 * (np.abs(approx) + 1)
    assert doubtful[: n // 512 * 512].reshape(-1, 512).any(axis=1).sum() >= 2     # a row: 64 lanes x 8 elements
    ref_chain = first.copy()
    oracle.nested_decode(codes_ref, n, M, bucket, steps_ref, d_o, first, 1.0, out=ref_chain)
    dev = _gpu()
    got = ndq.ndq_decode_chain(
        [(torch.from_numpy(dq_ref).to(dev), torch.from_numpy(dq_steps).to(dev), ndq.NDQ_WORKER_DQ, 16, d_g),
         (codes, steps, ndq.NDQ_WORKER_NESTED, M, d_g)], n, bucket, 1.0)
    assert np.array_equal(got.cpu().numpy(), ref_chain)
    # with shrinkage the reciprocal path is the same code
    ref_a = oracle.nested_decode(codes_ref, n, M, bucket, steps_ref, d_o, y, 1.0, alpha=0.75)
    out_a = ndq.ndq_nested_decode(codes, n, M, 0.75, bucket, steps, d_g, _to_dev(y), 1.0)
    assert np.array_equal(out_a.cpu().numpy(), ref_a)


def test_nested_equals_dqsg_inside_guaranteed_region_on_gpu():
    """|g - y| < (M-1) Delta / 2  =>  the nested reconstruction is the DQSG one."""
    n, M, levels = 1 << 18, 4, 64
    rng = np.random.default_rng(17)
    g = (rng.standard_normal(n) * 0.01).astype(F)
    delta = float(F(2 * np.abs(g).max() / (levels - 1)))
    bound = (M - 1) * delta / 2
    y = (g + rng.uniform(-0.999 * bound, 0.999 * bound, n)).astype(F)
    d = ndq.ndq_dither(21, 5, 1, 0)
    gd = _to_dev(g)
    c_dq, s_dq = ndq.ndq_dq_encode(gd, delta, levels + 3, 0, d)
    ref = ndq.ndq_dq_decode(c_dq, n, levels + 3, 0, s_dq, d)
    c_n, s_n = ndq.ndq_nested_encode(gd, delta, levels, M, 1.0, 0, d)
    got = ndq.ndq_nested_decode(c_n, n, M, 1.0, 0, s_n, d, _to_dev(y), 1.0)
    assert torch.equal(got, ref)


# --------------------------------------------------------------------------
# a8: aggregation
# --------------------------------------------------------------------------

@pytest.mark.parametrize("W", [1, 2, 3, 8, 16, 32, 33, 70])
def test_aggregate_matches_oracle(W):
    for n in (1, 5, 1023, 1024, 4096 + 3, 100003):
        rng = np.random.default_rng(W * 1000 + n)
        gs = [(rng.standard_normal(n) * 0.01).astype(F) for _ in range(W)]
        for scale in (1.0, 1.0 / W):
            ref = oracle.aggregate(gs, scale)
            out = ndq.ndq_aggregate([_to_dev(g) for g in gs], scale)
            assert np.array_equal(out.cpu().numpy(), ref), (W, n, scale)
    # in place on the first input
    gd = [_to_dev(g) for g in gs[:8]]
    ref = oracle.aggregate(gs[:8], 0.125)
    ndq.ndq_aggregate(gd, 0.125, gd[0])
    assert np.array_equal(gd[0].cpu().numpy(), ref)


# --------------------------------------------------------------------------
# whole path on the benchmark configurations
# --------------------------------------------------------------------------

def _run_both(wl, n, separate=False):
    host = workloads.gradients(wl, n)
    seeds = [workloads.dither_seed(wl, w) for w in range(wl.W)]
    ds_o = opipe.dithers(wl.W, seeds)
    c_ref, s_ref, delta = opipe.encode_all(wl.plan, wl.fine_levels, wl.bucket, wl.shared_step,
                                           host, ds_o)
    dev = pipeline.to_device(wl, host)
    bufs = pipeline.allocate(wl, n, separate=separate)
    ds_g = pipeline.dithers(wl)
    pipeline.encode_all(wl, dev, bufs, ds_g)       # a shared step stays in device memory
    if wl.shared_step:
        assert float(bufs.steps[0][0].item()) == delta
    for w in range(wl.W):
        assert np.array_equal(bufs.steps[w].cpu().numpy(), s_ref[w]), ("steps", w)
        assert bufs.codes[w].cpu().numpy().tobytes() == c_ref[w].tobytes(), ("codes", w)
    return host, c_ref, s_ref, ds_o, bufs, ds_g


def test_config2_ndqsg_pair():
    """2 workers, correlation 0.9: worker 0 DQSG 8 levels (3-bit codes), worker 1
    nested M = 4 (2-bit) with the same step, decoded against worker 0; sum."""
    wl = workloads.CONFIGS[2]
    host, c_ref, s_ref, ds_o, bufs, ds_g = _run_both(wl, wl.n)
    ref = opipe.decode_chain(wl.plan, wl.bucket, wl.n, c_ref, s_ref, ds_o, wl.out_scale)
    out = pipeline.decode_chain(wl, wl.n, bufs, ds_g).cpu().numpy()
    assert np.array_equal(out, ref)
    assert bufs.codes[0].numel() == (1 << 20) * 3 // 8 and bufs.codes[1].numel() == (1 << 20) // 4


def test_config3_dqsg_eight_workers_full_size():
    """8 workers, n = 25,557,032, 16 levels, 2,048-element buckets (ragged last
    bucket of 40), dither seed = worker id; decode all and average -- both as
    Algorithm 1 prints it (separate reconstructions, then the mean) and with a
    running sum."""
    wl = workloads.CONFIGS[3]
    host, c_ref, s_ref, ds_o, bufs, ds_g = _run_both(wl, wl.n, separate=True)
    assert bufs.steps[0].numel() == 12480
    ref, ref_each = opipe.decode_separately(wl.plan, wl.bucket, wl.n, c_ref, s_ref, ds_o,
                                            wl.out_scale)
    out = pipeline.decode_separately(wl, wl.n, bufs, ds_g).cpu().numpy()
    for w in (0, 7):
        assert np.array_equal(bufs.decoded[w].cpu().numpy(), ref_each[w])
    assert np.array_equal(out, ref)
    ref2 = opipe.decode_chain(wl.plan, wl.bucket, wl.n, c_ref, s_ref, ds_o, wl.out_scale)
    out2 = pipeline.decode_chain(wl, wl.n, bufs, ds_g).cpu().numpy()
    assert np.array_equal(out2, ref2)


def test_config4_ndqsg_chain_full_size():
    """16 workers, n = 11,173,962 (not a multiple of 4): worker 0 DQSG 16 levels,
    workers 1..15 nested M = 4 with the same step, each decoded against the
    running mean of the workers before it; reports the coset decode errors."""
    wl = workloads.CONFIGS[4]
    host, c_ref, s_ref, ds_o, bufs, ds_g = _run_both(wl, wl.n)
    ref, idx = opipe.decode_chain(wl.plan, wl.bucket, wl.n, c_ref, s_ref, ds_o, wl.out_scale, True)
    out = pipeline.decode_chain(wl, wl.n, bufs, ds_g).cpu().numpy()
    assert np.array_equal(out, ref)
    rates = []
    for w in range(1, wl.W):
        q_true = oracle.fine_indices(host[w], wl.bucket, s_ref[w], ds_o[w])
        wrong = idx[w] != q_true
        assert np.all((idx[w] - q_true)[wrong] % 4 == 0)
        rates.append(wrong.mean())
    print("config 4 coset decode error fraction per worker:", ["%.2e" % r for r in rates],
          "overall %.3e" % np.mean(rates))
    assert max(rates) < 0.05 and rates[-1] <= rates[0]


def test_config5_heavy_tail_bf16_reduced_size():
    """Config 5 at n = 2^22 + 4096 + 100 (ragged): bf16 Student-t inputs, 4,096-element
    buckets, worker 0 DQSG 4 levels (2-bit), workers 1-3 nested M = 2 (1-bit)."""
    wl = workloads.CONFIGS[5]
    n = (1 << 22) + 4096 + 100
    host, c_ref, s_ref, ds_o, bufs, ds_g = _run_both(wl, n)
    ref = opipe.decode_chain(wl.plan, wl.bucket, n, c_ref, s_ref, ds_o, wl.out_scale)
    out = pipeline.decode_chain(wl, n, bufs, ds_g).cpu().numpy()
    assert np.array_equal(out, ref)


def test_config5_diagnostics_clip_and_coset_error_fractions():
    """Untimed diagnostics of the benchmark workload on a 2^22-element sample: how
    many DQSG indices saturate (even level count: the positive end clips) and how
    often a nested worker's coarse bin is resolved wrongly (Thm 4's event); wrong
    decodes are off by exact multiples of M fine steps."""
    wl = workloads.CONFIGS[5]
    n = 1 << 22
    host, c_ref, s_ref, ds_o, bufs, ds_g = _run_both(wl, n)
    q0 = oracle.fine_indices(host[0], wl.bucket, s_ref[0], ds_o[0])
    L = wl.plan[0][1]
    clip = np.mean((q0 < -(L // 2)) | (q0 > -(L // 2) + L - 1))
    ref, idx = opipe.decode_chain(wl.plan, wl.bucket, n, c_ref, s_ref, ds_o, wl.out_scale, True)
    rates = []
    for w in range(1, wl.W):
        q_true = oracle.fine_indices(host[w], wl.bucket, s_ref[w], ds_o[w])
        wrong = idx[w] != q_true
        assert np.all((idx[w] - q_true)[wrong] % wl.plan[w][1] == 0)
        rates.append(wrong.mean())
    print("config 5 (n=2^22 sample): clip fraction of worker 0 = %.2e; coset decode error "
          "fraction per nested worker = %s" % (clip, ["%.2e" % r for r in rates]))
    assert clip < 0.01 and max(rates) < 0.05
    out = pipeline.decode_chain_fused(wl, n, bufs, ds_g).cpu().numpy()
    assert np.array_equal(out, ref)


def test_config5_full_size_whole_vectors():
    """Config 5 at its full size (n = 2^27 per worker) in the launch configuration
    the benchmark times (all encodes, then the fused server loop) and in the
    call-by-call one: the GPU processes the whole vectors and so does the oracle
    (on bucket-aligned slices, sixteen at a time); every code byte, every step and
    every one of the 2^27 outputs must agree bit for bit."""
    wl = workloads.CONFIGS[5]
    n = wl.n
    host = workloads.gradients(wl, n, threads=16)
    dev = pipeline.to_device(wl, host)
    bufs = pipeline.allocate(wl, n)
    ds_g = pipeline.dithers(wl)
    out = pipeline.step_fused(wl, dev, bufs, ds_g)
    torch.cuda.synchronize()
    seeds = [workloads.dither_seed(wl, w) for w in range(wl.W)]
    threads = min(16, os.cpu_count() or 1)
    c_ref, s_ref, ref = opipe.step_sliced(wl.plan, wl.fine_levels, wl.bucket, host, seeds, wl.out_scale,
                                          threads=threads)
    for w in range(wl.W):
        assert bufs.codes[w].cpu().numpy().tobytes() == c_ref[w].tobytes(), ("codes", w)
        assert np.array_equal(bufs.steps[w].cpu().numpy(), s_ref[w]), ("steps", w)
    assert np.array_equal(out.cpu().numpy(), ref)
    del c_ref, s_ref, ref
    # properties that hold at any size, checked on all 2^27 elements with device-side
    # tensor arithmetic: the DQSG reconstruction error of worker 0 is within half a
    # step except where the index saturated (about 1e-4 of the elements), has mean 0
    # and variance 1/12 in units of the bucket's step (Thm 1 / Lemma 2)
    assert bool(torch.isfinite(out).all())
    g0 = ndq.ndq_dq_decode(bufs.codes[0], n, wl.plan[0][1], wl.bucket, bufs.steps[0], ds_g[0])
    g0 -= dev[0].float()
    st = bufs.steps[0].repeat_interleave(wl.bucket)[:n]
    ok = st > 0
    e = (g0[ok] / st[ok]).double()
    del g0, st
    inside = e.abs() <= 0.5 + 2.0 ** -12
    clipped = 1.0 - inside.double().mean().item()
    assert clipped < 1e-3, clipped
    e_in = e[inside]
    assert abs(e_in.mean().item()) < 5.0 * (1.0 / 12 / e_in.numel()) ** 0.5 + 1e-4
    assert abs(e_in.var().item() * 12 - 1) < 0.01
    del e, e_in, inside, ok
    fused = out.clone()
    # the call-by-call schedule gives the same 2^27 values
    bufs2 = pipeline.allocate(wl, n)
    out2 = pipeline.step(wl, dev, bufs2, ds_g)
    assert torch.equal(out2, fused)
    for w in range(wl.W):
        assert torch.equal(bufs.codes[w], bufs2.codes[w]) and torch.equal(bufs.steps[w], bufs2.steps[w])
    # the fine index never leaves the range the step allows: |q| <= (L-1)/2 + 1/2 for the
    # worker's own data, so every nested residue is one of M values and the histogram is full
    hist, _ = ndq.ndq_code_entropy(bufs.codes[1], n, 1)
    assert int(hist.sum().item()) == n


@pytest.mark.parametrize("n", [2 * 6144 * 1024 + 5 * 1024 + 517, 3 * 6144 * 1024 + 1, 2 * 4096 * 4096 + 4096 * 3 + 64])
def test_config5_plan_with_a_ragged_end_at_the_persistent_grid_size(n):
    """Config 5's workers on vectors long enough for the persistent kernels on their full
    grids (two to three tiles per wave slot) that do not end on a tile: the encoders'
    ragged last tile and the chain decoder's, which runs through the hand-ordered loop
    with clamped code fetches and a guarded copy-out.  Whole vectors against the oracle
    (on bucket-aligned slices, all host cores), and against the call-by-call schedule."""
    wl = workloads.CONFIGS[5]
    host = workloads.gradients(wl, n, threads=16)
    dev = pipeline.to_device(wl, host)
    bufs = pipeline.allocate(wl, n)
    # guard words behind the result: the ragged tile's copy-out must not reach them
    guarded = torch.full((n + 1024,), 12345.0, dtype=torch.float32, device=dev[0].device)
    bufs.total = guarded[:n]
    ds_g = pipeline.dithers(wl)
    out = pipeline.step_fused(wl, dev, bufs, ds_g)
    torch.cuda.synchronize()
    seeds = [workloads.dither_seed(wl, w) for w in range(wl.W)]
    c_ref, s_ref, ref = opipe.step_sliced(wl.plan, wl.fine_levels, wl.bucket, host, seeds, wl.out_scale,
                                          threads=min(16, os.cpu_count() or 1))
    for w in range(wl.W):
        assert bufs.codes[w].cpu().numpy().tobytes() == c_ref[w].tobytes(), ("codes", w)
        assert np.array_equal(bufs.steps[w].cpu().numpy(), s_ref[w]), ("steps", w)
    assert np.array_equal(out.cpu().numpy(), ref)
    assert bool((guarded[n:] == 12345.0).all())
    bufs2 = pipeline.allocate(wl, n)
    assert torch.equal(pipeline.step(wl, dev, bufs2, ds_g), out)


def test_runs_are_deterministic():
    wl = workloads.CONFIGS[5]
    n = 1 << 20
    dev = pipeline.to_device(wl, workloads.gradients(wl, n))
    ds = pipeline.dithers(wl)
    b1, b2 = pipeline.allocate(wl, n), pipeline.allocate(wl, n)
    o1 = pipeline.step(wl, dev, b1, ds).clone()
    o2 = pipeline.step(wl, dev, b2, ds)
    assert torch.equal(o1, o2)
    for w in range(wl.W):
        assert torch.equal(b1.codes[w], b2.codes[w])
    # a different iteration number draws a different dither
    ds2 = pipeline.dithers(wl, step=1)
    pipeline.step(wl, dev, b2, ds2)
    assert not torch.equal(b1.codes[0], b2.codes[0])


# --------------------------------------------------------------------------
# the whole server loop of Algorithm 2 in one call
# --------------------------------------------------------------------------

def _chain_case(plan, fine_levels, bucket, n, dtype, seed, out_scale, shared_step):
    rng = np.random.default_rng(seed)
    common = rng.standard_normal(n) * 0.01
    host = []
    for w in range(len(plan)):
        x = (common + rng.standard_normal(n) * 0.002).astype(F)
        host.append(workloads.f32_to_bf16_bits(x) if dtype == "bf16" else x)
    seeds = [7 + w for w in range(len(plan))]
    ds_o = opipe.dithers(len(plan), seeds, step=3)
    c_ref, s_ref, _ = opipe.encode_all(plan, fine_levels, bucket, shared_step, host, ds_o)
    ref = opipe.decode_chain(plan, bucket, n, c_ref, s_ref, ds_o, out_scale)
    dev = _gpu()
    workers = []
    for w, (kind, arg) in enumerate(plan):
        workers.append((torch.from_numpy(c_ref[w]).to(dev), torch.from_numpy(s_ref[w]).to(dev),
                        ndq.NDQ_WORKER_DQ if kind == "dq" else ndq.NDQ_WORKER_NESTED, arg,
                        ndq.ndq_dither(seeds[w], 3, w, 0)))
    out = ndq.ndq_decode_chain(workers, n, bucket, out_scale)
    assert np.array_equal(out.cpu().numpy(), ref), (plan, n)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_decode_chain_matches_oracle_loop(dtype):
    plans = [
        ((("dq", 4), ("nested", 2), ("nested", 2), ("nested", 2)), 4, 4096, 1.0, False),
        ((("dq", 16),) + (("nested", 4),) * 15, 16, 0, 1.0 / 16, True),
        ((("dq", 16),) * 8, 16, 2048, 0.125, False),
        ((("dq", 8), ("nested", 3), ("dq", 5), ("nested", 7), ("nested", 256), ("dq", 256)),
         8, 2112, 1.0, False),
        ((("dq", 3),), 3, 0, 1.0, False),
        # buckets of one row of a tile (each row has its own step), and smaller ones
        ((("dq", 4), ("nested", 2), ("nested", 4), ("dq", 9)), 4, 512, 0.25, False),
        ((("dq", 16), ("nested", 4)), 16, 256, 1.0, False),
    ]
    for plan, fine, bucket, scale, shared in plans:
        for n in (1, 255, 1024, 1025, 1536, 4096 * 3 + 77, 70001):
            _chain_case(plan, fine, bucket, n, dtype, seed=n, out_scale=scale, shared_step=shared)


def test_decode_chain_more_workers_than_one_launch_holds():
    plan = (("dq", 16),) + tuple(("nested", 4) if w % 3 else ("dq", 9) for w in range(1, 70))
    _chain_case(plan, 16, 1024, 9000, "f32", seed=5, out_scale=1.0 / 70, shared_step=False)


def test_decode_chain_rejects_a_nested_first_worker():
    dev = _gpu()
    codes = torch.zeros(1024, dtype=torch.uint8, device=dev)
    steps = torch.ones(1, dtype=torch.float32, device=dev)
    with pytest.raises(ndq.NdqError) as e:
        ndq.ndq_decode_chain([(codes, steps, ndq.NDQ_WORKER_NESTED, 4, ndq.ndq_dither(0, 0, 0, 0))],
                             1024, 0)
    assert e.value.rc == ndq.NDQ_EINVAL


def test_fused_step_equals_call_by_call_step_on_the_configs():
    for cfg, n in ((2, None), (3, 1 << 21), (4, (1 << 21) + 2), (5, (1 << 22) + 100)):
        wl = workloads.CONFIGS[cfg]
        n = n or wl.n
        dev = pipeline.to_device(wl, workloads.gradients(wl, n))
        ds = pipeline.dithers(wl)
        b1, b2 = pipeline.allocate(wl, n), pipeline.allocate(wl, n)
        ref = pipeline.step(wl, dev, b1, ds).clone()
        # a shared step read from worker 0's message on the device, then the same step as a host preset
        out = pipeline.step_fused(wl, dev, b2, ds)
        assert torch.equal(out, ref), cfg
        if wl.shared_step:
            b2.total.zero_()
            out = pipeline.step_fused(wl, dev, b2, ds, float(b1.steps[0][0].item()))
            assert torch.equal(out, ref), cfg


# --------------------------------------------------------------------------
# histogram and entropy of the index stream
# --------------------------------------------------------------------------

@pytest.mark.parametrize("bits", [1, 2, 3, 4, 5, 6, 7, 8])
def test_code_histogram_and_entropy_match_oracle(bits):
    dev = _gpu()
    for n in (0, 1, 31, 32, 33, 1000, 8191, 65536 + 17, 3000001):
        rng = np.random.default_rng(n + bits)
        # skewed code distribution, like real index streams
        p = rng.dirichlet(np.full(1 << bits, 0.3))
        codes = rng.choice(1 << bits, size=n, p=p).astype(np.uint32)
        packed = oracle.pack(codes, bits)
        ref_h = oracle.code_histogram(packed, n, bits)
        ref_e = oracle.entropy_bits(ref_h)
        packed_d = torch.from_numpy(packed).to(dev)
        # outputs that hold something else before the call (the call clears them itself)
        hist = torch.full((1 << bits,), 12345, dtype=torch.int64, device=dev)
        ent = torch.full((1,), 7.5, dtype=torch.float64, device=dev)
        ndq.ndq_code_entropy(packed_d, n, bits, hist, ent)
        assert np.array_equal(hist.cpu().numpy().astype(np.uint64), ref_h), (bits, n)
        assert abs(float(ent.item()) - ref_e) <= 1e-9, (bits, n)
        # the histogram alone (null entropy_out), twice in a row into the same buffer
        for _ in range(2):
            hist2, none = ndq.ndq_code_entropy(packed_d, n, bits, hist, want_entropy=False)
            assert none is None
            assert np.array_equal(hist2.cpu().numpy().astype(np.uint64), ref_h), (bits, n)


@pytest.mark.parametrize("bits", [1, 2, 3, 8])
def test_code_histogram_ignores_what_lies_in_the_padding(bits):
    """Bits of the stream beyond code n-1 are not counted, whatever they hold."""
    dev = _gpu()
    for n in (1, 5, 63, 64, 65, 127, 129, 1000, 70001, 1 << 20):
        rng = np.random.default_rng(100 * n + bits)
        codes = rng.integers(0, 1 << bits, size=n, dtype=np.uint32)
        packed = oracle.pack(codes, bits).copy()
        ref_h = oracle.code_histogram(packed, n, bits)
        used = n * bits
        tail = np.unpackbits(packed, bitorder="little")
        tail[used:] = 1
        dirty = np.packbits(tail, bitorder="little")
        hist, _ = ndq.ndq_code_entropy(torch.from_numpy(dirty).to(dev), n, bits)
        assert np.array_equal(hist.cpu().numpy().astype(np.uint64), ref_h), (bits, n)


def test_entropy_of_the_benchmark_code_streams():
    """Entropy of the actual DQSG / nested index streams of config 5 (reduced size):
    GPU histogram against the oracle's, bit-exact."""
    wl = workloads.CONFIGS[5]
    n = (1 << 21) + 123
    host, c_ref, s_ref, ds_o, bufs, ds_g = _run_both(wl, n)
    for w, (kind, arg) in enumerate(wl.plan):
        bits = oracle.code_bits(arg)
        ref_h = oracle.code_histogram(c_ref[w], n, bits)
        hist, ent = ndq.ndq_code_entropy(bufs.codes[w], n, bits)
        assert np.array_equal(hist.cpu().numpy().astype(np.uint64), ref_h)
        assert abs(float(ent.item()) - oracle.entropy_bits(ref_h)) <= 1e-9
        assert float(ent.item()) <= bits


# --------------------------------------------------------------------------
# dense base-L stream
# --------------------------------------------------------------------------

@pytest.mark.parametrize("levels", [2, 3, 4, 5, 6, 7, 9, 16, 17, 100, 255, 256])
def test_dense_stream_matches_oracle(levels):
    dev = _gpu()
    bits = oracle.code_bits(levels)
    k = oracle.dense_group(levels)
    assert ndq.ndq_dense_group(levels) == k
    for n in (1, k - 1, k, k + 1, 8 * k, 8 * k + 1, 1000, 65536 + 5, 1000003):
        rng = np.random.default_rng(n + levels)
        codes = rng.integers(0, levels, n).astype(np.uint32)
        codes[:min(n, k)] = levels - 1
        fixed = oracle.pack(codes, bits)
        ref = oracle.dense_pack(codes, levels)
        assert ndq.ndq_dense_bytes(n, levels) == ref.size
        fixed_d = torch.from_numpy(fixed).to(dev)
        dense = ndq.ndq_dense_pack(fixed_d, n, levels)
        assert dense.cpu().numpy().tobytes() == ref.tobytes(), (levels, n)
        # what lies beyond code n-1 in the fixed-width stream does not reach the dense one
        stream_bits = np.unpackbits(fixed, bitorder="little")
        stream_bits[n * bits:] = 1
        dirty = torch.from_numpy(np.packbits(stream_bits, bitorder="little")).to(dev)
        assert ndq.ndq_dense_pack(dirty, n, levels).cpu().numpy().tobytes() == ref.tobytes(), (levels, n)
        back = torch.full((fixed.size,), 0xAB, dtype=torch.uint8, device=dev)
        ndq.ndq_dense_unpack(dense, n, levels, back)
        assert back.cpu().numpy().tobytes() == fixed.tobytes(), (levels, n)


def test_three_level_gradient_in_dense_form():
    """The paper's three-level DQSG message at 1.6 bits per index: encode, make
    dense, expand, decode -- same reconstruction as without the detour."""
    n = 266610                       # FC-300-100's parameter count (Table 1)
    g = _make(n, "f32", seed=1)
    d = ndq.ndq_dither(1, 0, 0, 0)
    codes, steps = ndq.ndq_dq_encode(_to_dev(g), 0.0, 3, 0, d)
    dense = ndq.ndq_dense_pack(codes, n, 3)
    assert dense.numel() * 8 <= 1.0097 * n * np.log2(3) + 128 and dense.numel() < codes.numel()
    back = ndq.ndq_dense_unpack(dense, n, 3)
    assert torch.equal(back, codes)
    assert torch.equal(ndq.ndq_dq_decode(back, n, 3, 0, steps, d), ndq.ndq_dq_decode(codes, n, 3, 0, steps, d))


# --------------------------------------------------------------------------
# shrinkage factor alpha < 1 (eqs. (7)-(8), Thm 4) and its parameter estimate
# --------------------------------------------------------------------------

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("M,alpha,bucket", [(4, 0.9, 0), (2, 0.75, 4096), (3, 0.5, 2048), (8, 0.97, 2112)])
def test_nested_with_shrinkage_matches_oracle(dtype, M, alpha, bucket):
    levels = 16
    for n in SIZES:
        g = _make(n, dtype, seed=n + M)
        gf = workloads.bf16_bits_to_f32(g) if dtype == "bf16" else g
        rng = np.random.default_rng(n)
        side = (gf + rng.standard_normal(n).astype(F) * F(0.2 * np.abs(gf).max() / levels)).astype(F)
        d_o, d_g = oracle.dither(13, 2, 5), ndq.ndq_dither(13, 2, 5, 0)
        c_ref, s_ref = oracle.nested_encode(g, 0.0, levels, M, bucket, d_o, alpha=alpha)
        codes, steps = ndq.ndq_nested_encode(_to_dev(g), 0.0, levels, M, alpha, bucket, d_g)
        assert np.array_equal(steps.cpu().numpy(), s_ref), n
        assert codes.cpu().numpy().tobytes() == c_ref.tobytes(), n
        ref = oracle.nested_decode(c_ref, n, M, bucket, s_ref, d_o, side, 0.5, alpha=alpha)
        out = ndq.ndq_nested_decode(codes, n, M, alpha, bucket, steps, d_g, _to_dev(side), 0.5)
        assert np.array_equal(out.cpu().numpy(), ref), n
        ref_inp = side.copy()
        oracle.nested_decode(c_ref, n, M, bucket, s_ref, d_o, side, 0.5, out=ref_inp, alpha=alpha)
        s_inp = _to_dev(side)
        ndq.ndq_nested_decode(codes, n, M, alpha, bucket, steps, d_g, s_inp, 0.5, s_inp, True)
        assert np.array_equal(s_inp.cpu().numpy(), ref_inp), n


def test_chain_with_shrinkage_and_parameter_selection():
    """Parameter selection of Thm 4 on the device estimate of sigma_z^2, then the
    fused server loop with per-worker alpha, against the oracle's loop."""
    n, levels, M, bucket = 300001, 16, 4, 0
    rng = np.random.default_rng(77)
    common = (rng.standard_normal(n) * 0.01).astype(F)
    gs = [(common + rng.standard_normal(n) * 0.002).astype(F) for _ in range(4)]
    dev = _gpu()
    gd = [_to_dev(g) for g in gs]
    # sigma_z^2 between two workers, on the device and in the oracle
    sq = ndq.ndq_sqdiff(gd[1], gd[0])
    ref_sq = oracle.sqdiff_sum(gs[1], gs[0])
    assert abs(float(sq.item()) - ref_sq) <= 1e-12 * ref_sq
    assert torch.equal(ndq.ndq_sqdiff(gd[1], gd[0]), sq)              # fixed reduction order
    delta = float(F(2 * np.abs(gs[0]).max() / (levels - 1)))
    alpha = ndq.ndq_alpha_for_equal_variance(delta, ref_sq / n)
    assert 0.5 < alpha < 1.0
    seeds = [0, 0, 0, 0]
    ds_o = [oracle.dither(seeds[w], 9, w) for w in range(4)]
    ds_g = [ndq.ndq_dither(seeds[w], 9, w, 0) for w in range(4)]
    c0, s0 = oracle.dq_encode(gs[0], delta, levels, bucket, ds_o[0])
    S = oracle.dq_decode(c0, n, levels, bucket, s0, ds_o[0])
    workers = [(torch.from_numpy(c0).to(dev), torch.from_numpy(s0).to(dev), ndq.NDQ_WORKER_DQ,
                levels, ds_g[0])]
    for w in range(1, 4):
        a_w = alpha if w != 2 else 1.0                                # mixed per-worker alpha
        c, s = oracle.nested_encode(gs[w], delta, levels, M, bucket, ds_o[w], alpha=a_w)
        cg, sg = ndq.ndq_nested_encode(gd[w], delta, levels, M, a_w, bucket, ds_g[w])
        assert cg.cpu().numpy().tobytes() == c.tobytes()
        S = oracle.nested_decode(c, n, M, bucket, s, ds_o[w], S, F(1.0 / w), out=S, alpha=a_w)
        workers.append((cg, sg, ndq.NDQ_WORKER_NESTED, M, ds_g[w], a_w))
    out = ndq.ndq_decode_chain(workers, n, bucket, 0.25)
    assert np.array_equal(out.cpu().numpy(), oracle.aggregate([S], 0.25))


def test_nesting_ratio_chosen_from_the_device_estimate_keeps_decode_errors_under_the_target():
    """Thm 4 end to end on the device: sigma_z^2 from ndq_sqdiff, the smallest
    nesting ratio whose bound meets the target, then nested encode and decode with
    the other worker's gradient as side information.  The fraction of elements whose
    coarse bin is resolved wrongly stays under the target; right ones are within half
    a fine step of the input and wrong ones off by multiples of M steps."""
    n, delta, target = 1 << 22, 0.002, 1e-3
    rng = np.random.default_rng(2024)
    common = (rng.standard_normal(n) * 0.02).astype(F)
    g = (common + rng.standard_normal(n) * 0.003).astype(F)
    y_d, g_d = _to_dev(common), _to_dev(g)
    var_z = float(ndq.ndq_sqdiff(g_d, y_d).item()) / n
    assert abs(var_z - 9e-6) < 2e-7
    M = ndq.ndq_nesting_ratio_for_error(delta, 1.0, var_z, target)
    assert 2 < M <= 256
    assert ndq.ndq_decode_error_bound(delta, M, 1.0, var_z) <= target
    assert ndq.ndq_decode_error_bound(delta, M - 1, 1.0, var_z) > target
    d = ndq.ndq_dither(5, 1, 1, 0)
    rates = {}
    for ratio in (M, max(2, M // 16)):
        codes, steps = ndq.ndq_nested_encode(g_d, delta, 16, ratio, 1.0, 0, d)
        out = torch.empty(n, dtype=torch.float32, device=y_d.device)
        ndq.ndq_nested_decode(codes, n, ratio, 1.0, 0, steps, d, y_d, 1.0, out, False)
        err = (out.double() - g_d.double()).abs().cpu().numpy() / delta
        wrong = err > 0.75
        assert np.all(err[~wrong] <= 0.5 + 1e-3)
        off = err[wrong] / ratio
        assert np.all(np.abs(off - np.rint(off)) <= 0.5 / ratio + 1e-3) and np.all(np.rint(off) >= 1)
        rates[ratio] = wrong.mean()
    assert rates[M] <= target
    assert rates[max(2, M // 16)] > rates[M]          # a much smaller ratio does fail visibly


@pytest.mark.parametrize("n", [0, 1, 3, 4, 5, 1023, 262144, 1000003])
def test_sqdiff_matches_oracle(n):
    rng = np.random.default_rng(n)
    a = rng.standard_normal(n).astype(F)
    b = rng.standard_normal(n).astype(F)
    ref = oracle.sqdiff_sum(a, b)
    if n == 0:
        dev = _gpu()
        e = torch.empty(0, dtype=torch.float32, device=dev)
        assert float(ndq.ndq_sqdiff(e, e).item()) == 0.0
        return
    got = float(ndq.ndq_sqdiff(_to_dev(a), _to_dev(b)).item())
    assert abs(got - ref) <= 1e-12 * ref


def test_step_can_be_captured_in_a_hip_graph_and_replayed():
    """The library only enqueues kernels on the given stream (no allocation, no
    memset, no synchronisation), so a whole step can be recorded into a HIP graph;
    every replay, with eager work and synchronisation in between, must reproduce
    the eager result."""
    wl = workloads.CONFIGS[5]
    n = (1 << 20) + 4096 + 8
    dev = pipeline.to_device(wl, workloads.gradients(wl, n))
    ds = pipeline.dithers(wl)
    eager = pipeline.allocate(wl, n)
    ref = pipeline.step_fused(wl, dev, eager, ds).clone()
    torch.cuda.synchronize()
    bufs = pipeline.allocate(wl, n)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):              # warm-up on the capture stream
        pipeline.step_fused(wl, dev, bufs, ds)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        pipeline.step_fused(wl, dev, bufs, ds)
    for rep in range(4):
        bufs.total.fill_(float(rep))           # eager work between replays
        for c in bufs.codes:
            c.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(bufs.total, ref), rep
        for w in range(wl.W):
            assert torch.equal(bufs.codes[w], eager.codes[w]), (rep, w)
            assert torch.equal(bufs.steps[w], eager.steps[w]), (rep, w)


def test_tools_can_be_captured_in_a_hip_graph_and_replayed():
    """The calls beyond the headline path in one graph: a two-pass encode (max-norm pass and
    encoder), an encode that reads its step from device memory, the histogram with its
    entropy (cleared by a kernel, closed by the last workgroup's ticket), the dense
    transcoders and the sum of squared differences from the library's own scratch.  Every
    replay, with the outputs overwritten in between, must reproduce the eager results."""
    dev = _gpu()
    n = 3 * 40960 + 12345
    g0, g1 = _to_dev(_make(n, "f32", seed=77)), _to_dev(_make(n, "bf16", seed=78))
    d0, d1 = ndq.ndq_dither(3, 1, 0, 0), ndq.ndq_dither(3, 1, 1, 0)

    def run(o):
        ndq.ndq_dq_encode(g0, 0.0, 3, 0, d0, o["c0"], o["s0"])
        ndq.ndq_nested_encode_with_step(g1, o["s0"], 4, 1.0, d1, o["c1"], o["s1"])
        ndq.ndq_code_entropy(o["c0"], n, 2, o["hist"], o["ent"])
        ndq.ndq_dense_pack(o["c0"], n, 3, o["dense"])
        ndq.ndq_dense_unpack(o["dense"], n, 3, o["back"])
        ndq.ndq_sqdiff_static(g0, o["f"], o["sq"])

    def outputs():
        return {"c0": torch.empty(ndq.ndq_packed_bytes(n, 2), dtype=torch.uint8, device=dev),
                "s0": torch.empty(1, dtype=torch.float32, device=dev),
                "c1": torch.empty(ndq.ndq_packed_bytes(n, 2), dtype=torch.uint8, device=dev),
                "s1": torch.empty(1, dtype=torch.float32, device=dev),
                "hist": torch.empty(4, dtype=torch.int64, device=dev),
                "ent": torch.empty(1, dtype=torch.float64, device=dev),
                "dense": torch.empty(ndq.ndq_dense_bytes(n, 3), dtype=torch.uint8, device=dev),
                "back": torch.empty(ndq.ndq_packed_bytes(n, 2), dtype=torch.uint8, device=dev),
                "f": torch.zeros(n, dtype=torch.float32, device=dev),
                "sq": torch.empty(1, dtype=torch.float64, device=dev)}

    eager = outputs()
    run(eager)
    torch.cuda.synchronize()
    assert torch.equal(eager["back"], eager["c0"]) and int(eager["hist"].sum().item()) == n
    bufs = outputs()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):              # warm-up on the capture stream (first use of the static scratch)
        run(bufs)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        run(bufs)
    for rep in range(4):
        for k, t in bufs.items():              # eager work between replays: the outputs hold something else
            if k != "f":
                t.fill_(rep + 1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k in bufs:
            assert torch.equal(bufs[k], eager[k]), (rep, k)


def test_vector_longer_than_2_pow_32_elements():
    """Largest practical size: n > 2^32 elements per worker (8.6 GB of bf16), so that
    element indices, bit offsets and Philox counters leave 32 bits.  Inputs are
    drawn on the device with torch (inputs are just bytes); the oracle recomputes
    bucket-aligned slices -- the first, the one straddling index 2^32, some beyond
    it, and the ragged end -- from the same bytes."""
    dev = _gpu()
    free, _ = torch.cuda.mem_get_info()
    if free < 70 * (1 << 30):
        pytest.skip("needs about 60 GB of free device memory")
    n = (1 << 32) + (1 << 20) + 8
    bucket, L, M = 4096, 4, 2
    gen = torch.Generator(device=dev).manual_seed(20240607)
    g = [torch.empty(n, dtype=torch.bfloat16, device=dev) for _ in range(2)]
    step = 1 << 28
    for a in range(0, n, step):
        b = min(n, a + step)
        common = torch.randn(b - a, generator=gen, device=dev) * 1e-3
        g[0][a:b] = common.to(torch.bfloat16)
        g[1][a:b] = (0.9 * common + 0.4e-3 * torch.randn(b - a, generator=gen, device=dev)).to(torch.bfloat16)
        del common
    d = [ndq.ndq_dither(11, 5, w, 0) for w in range(2)]
    c0, s0 = ndq.ndq_dq_encode(g[0], 0.0, L, bucket, d[0])
    c1, s1 = ndq.ndq_nested_encode(g[1], 0.0, L, M, 1.0, bucket, d[1])
    out = ndq.ndq_decode_chain([(c0, s0, ndq.NDQ_WORKER_DQ, L, d[0]),
                                (c1, s1, ndq.NDQ_WORKER_NESTED, M, d[1])], n, bucket, 1.0)
    out2 = ndq.ndq_dq_decode(c0, n, L, bucket, s0, d[0])
    ndq.ndq_nested_decode(c1, n, M, 1.0, bucket, s1, d[1], out2, 1.0, out2, True)
    for a in range(0, n, step):
        assert torch.equal(out[a:min(n, a + step)], out2[a:min(n, a + step)]), a
    del out2
    torch.cuda.synchronize()
    span = 4 * bucket
    tail = (n // bucket - 3) * bucket
    starts = [0, (1 << 32) - 2 * bucket, (1 << 32) + 5 * bucket, (1 << 32) + (1 << 19), tail]
    for lo in starts:
        hi = min(n, lo + span)
        m = hi - lo
        h0 = g[0][lo:hi].view(torch.int16).cpu().numpy().view(np.uint16)
        h1 = g[1][lo:hi].view(torch.int16).cpu().numpy().view(np.uint16)
        r0, t0 = oracle.dq_encode(h0, 0.0, L, bucket, oracle.dither(11, 5, 0, lo))
        r1, t1 = oracle.nested_encode(h1, 0.0, L, M, bucket, oracle.dither(11, 5, 1, lo))
        nb = (m + bucket - 1) // bucket
        assert np.array_equal(s0[lo // bucket:lo // bucket + nb].cpu().numpy(), t0), lo
        assert np.array_equal(s1[lo // bucket:lo // bucket + nb].cpu().numpy(), t1), lo
        b0, b1 = (m * 2 + 7) // 8, (m + 7) // 8
        assert c0[lo * 2 // 8:lo * 2 // 8 + b0].cpu().numpy().tobytes() == r0[:b0].tobytes(), lo
        assert c1[lo // 8:lo // 8 + b1].cpu().numpy().tobytes() == r1[:b1].tobytes(), lo
        S = oracle.dq_decode(r0, m, L, bucket, t0, oracle.dither(11, 5, 0, lo))
        S = oracle.nested_decode(r1, m, M, bucket, t1, oracle.dither(11, 5, 1, lo), S, 1.0, out=S)
        assert np.array_equal(out[lo:hi].cpu().numpy(), S), lo
    # padding after the last code is zero and within the buffer
    assert c0.numel() == ndq.ndq_packed_bytes(n, 2) and c1.numel() == ndq.ndq_packed_bytes(n, 1)
    assert int(c1[(n + 7) // 8:].sum().item()) == 0 and int(c0[(2 * n + 7) // 8:].sum().item()) == 0


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_extreme_magnitudes_denormals_and_signed_zeros(dtype):
    """Log-uniform magnitudes over the whole exponent range, denormals, +-0: every
    rounding on the GPU is the oracle's (no flush to zero, correctly rounded
    division, no contraction), including indices that saturate and coset searches
    far outside any sensible range."""
    n = 3 * 4096 + 100
    rng = np.random.default_rng(99)
    expo = rng.uniform(-44, 37, n)
    g32 = (rng.choice([-1.0, 1.0], n) * 10.0 ** expo).astype(F)
    g32[::17] = 0.0
    g32[1::17] = -0.0
    g32[2::17] = F(1e-45)                                # smallest denormal
    g = workloads.f32_to_bf16_bits(g32) if dtype == "bf16" else g32
    gd = _to_dev(g)
    side32 = (rng.choice([-1.0, 1.0], n) * 10.0 ** rng.uniform(-40, 30, n)).astype(F)
    side_d = _to_dev(side32)
    d_o, d_g = oracle.dither(3, 1, 2), ndq.ndq_dither(3, 1, 2, 0)
    for bucket, delta in ((4096, 0.0), (64, 0.0), (0, 0.0), (0, 1e-30), (0, 1e30), (0, 1.0)):
        for levels in (3, 4, 256):
            c_ref, s_ref = oracle.dq_encode(g, delta, levels, bucket, d_o)
            codes, steps = ndq.ndq_dq_encode(gd, delta, levels, bucket, d_g)
            assert np.array_equal(steps.cpu().numpy(), s_ref), (bucket, delta, levels)
            assert codes.cpu().numpy().tobytes() == c_ref.tobytes(), (bucket, delta, levels)
            ref = oracle.dq_decode(c_ref, n, levels, bucket, s_ref, d_o)
            out = ndq.ndq_dq_decode(codes, n, levels, bucket, steps, d_g)
            assert np.array_equal(out.cpu().numpy(), ref, equal_nan=True), (bucket, delta, levels)
        for M, alpha in ((2, 1.0), (4, 1.0), (3, 1.0), (4, 0.75), (256, 1.0)):
            c_ref, s_ref = oracle.nested_encode(g, delta, 16, M, bucket, d_o, alpha=alpha)
            codes, steps = ndq.ndq_nested_encode(gd, delta, 16, M, alpha, bucket, d_g)
            assert np.array_equal(steps.cpu().numpy(), s_ref), (bucket, delta, M)
            assert codes.cpu().numpy().tobytes() == c_ref.tobytes(), (bucket, delta, M)
            ref = oracle.nested_decode(c_ref, n, M, bucket, s_ref, d_o, side32, 0.5, alpha=alpha)
            out = ndq.ndq_nested_decode(codes, n, M, alpha, bucket, steps, d_g, side_d, 0.5)
            assert np.array_equal(out.cpu().numpy(), ref, equal_nan=True), (bucket, delta, M, alpha)


def test_randomized_differential_against_oracle():
    """300 seeded random draws of (n, dtype, bucket, levels, M, alpha, preset, offset,
    accumulate form): every entry point against the oracle, bit for bit.  (NDQ_FUZZ_SEED and
    NDQ_FUZZ_CASES in the environment run other draws, or more of them; NDQ_FUZZ_MAX_N longer
    vectors.)"""
    rng = np.random.default_rng(int(os.environ.get("NDQ_FUZZ_SEED", "20240611")))
    dev = _gpu()
    for case in range(int(os.environ.get("NDQ_FUZZ_CASES", "300"))):
        n = int(rng.choice([rng.integers(1, 300), rng.integers(300, 5000),
                            rng.integers(5000, int(os.environ.get("NDQ_FUZZ_MAX_N", "40000")))]))
        dtype = "bf16" if rng.random() < 0.5 else "f32"
        bucket = int(rng.choice([0, 64, 128, 512, 1024, 2048, 4096, 4160, 8192, 16384]))
        levels = int(rng.choice([2, 3, 4, 5, 7, 8, 15, 16, 17, 64, 100, 255, 256]))
        M = int(rng.choice([2, 3, 4, 5, 6, 7, 8, 12, 16, 31, 65, 256]))
        alpha = float(rng.choice([1.0, 1.0, 0.9, 0.5]))
        offset = int(rng.choice([0, 8, 4096, (1 << 33) + 64])) if bucket == 0 else \
            int(rng.choice([0, 1, 7, 1 << 22])) * bucket
        preset = bucket == 0 and rng.random() < 0.5
        seed, step, worker = int(rng.integers(0, 1 << 62)), int(rng.integers(0, 1 << 31)), int(rng.integers(0, 64))
        g = _make(n, dtype, seed=case, heavy=rng.random() < 0.3)
        gf = workloads.bf16_bits_to_f32(g) if dtype == "bf16" else g
        kappa = float(np.abs(gf).max())
        delta = float(F(2 * kappa / (levels - 1))) if preset and kappa > 0 else 0.0
        d_o, d_g = oracle.dither(seed, step, worker, offset), ndq.ndq_dither(seed, step, worker, offset)
        gd = _to_dev(g)
        tag = (case, n, dtype, bucket, levels, M, alpha, offset, preset)
        # DQSG
        c_ref, s_ref = oracle.dq_encode(g, delta, levels, bucket, d_o)
        codes, steps = ndq.ndq_dq_encode(gd, delta, levels, bucket, d_g)
        assert np.array_equal(steps.cpu().numpy(), s_ref), tag
        assert codes.cpu().numpy().tobytes() == c_ref.tobytes(), tag
        ref = oracle.dq_decode(c_ref, n, levels, bucket, s_ref, d_o)
        assert np.array_equal(ndq.ndq_dq_decode(codes, n, levels, bucket, steps, d_g).cpu().numpy(), ref), tag
        assert np.array_equal(ndq.ndq_dq_decode_half(codes, n, levels, bucket, steps).cpu().numpy(),
                              oracle.dq_decode_half(c_ref, n, levels, bucket, s_ref)), tag
        # nested against the DQSG reconstruction as side information, in place
        m_ref, t_ref = oracle.nested_encode(g, delta, levels, M, bucket, d_o, alpha=alpha)
        mc, ms = ndq.ndq_nested_encode(gd, delta, levels, M, alpha, bucket, d_g)
        assert np.array_equal(ms.cpu().numpy(), t_ref), tag
        assert mc.cpu().numpy().tobytes() == m_ref.tobytes(), tag
        if preset and delta > 0.0:
            # the same preset step handed over in device memory
            step_d = torch.tensor([delta], dtype=torch.float32, device=dev)
            c2, s2 = ndq.ndq_dq_encode_with_step(gd, step_d, levels, d_g)
            assert torch.equal(c2, codes) and torch.equal(s2, steps), tag
            m2, t2 = ndq.ndq_nested_encode_with_step(gd, step_d, M, alpha, d_g)
            assert torch.equal(m2, mc) and torch.equal(t2, ms), tag
        S_ref = ref.copy()
        oracle.nested_decode(m_ref, n, M, bucket, t_ref, d_o, S_ref, 1.0, out=S_ref, alpha=alpha)
        S = torch.from_numpy(ref).to(dev)
        ndq.ndq_nested_decode(mc, n, M, alpha, bucket, ms, d_g, S, 1.0, S, True)
        assert np.array_equal(S.cpu().numpy(), S_ref), tag
        # the same two workers through the fused loop
        out = ndq.ndq_decode_chain([(codes, steps, ndq.NDQ_WORKER_DQ, levels, d_g),
                                    (mc, ms, ndq.NDQ_WORKER_NESTED, M, d_g, alpha)], n, bucket, 1.0)
        assert np.array_equal(out.cpu().numpy(), S_ref), tag
        # entropy and dense form of the index streams
        bits = oracle.code_bits(levels)
        hist, _ = ndq.ndq_code_entropy(codes, n, bits)
        assert np.array_equal(hist.cpu().numpy().astype(np.uint64), oracle.code_histogram(c_ref, n, bits)), tag
        dense = ndq.ndq_dense_pack(codes, n, levels)
        assert dense.cpu().numpy().tobytes() == oracle.dense_pack(oracle.unpack(c_ref, n, bits), levels).tobytes(), tag
