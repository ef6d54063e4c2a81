"""Python face of the CPU oracle (test infrastructure, not the product).

Loads ``libndq_oracle.so`` (plain C, built from ``ndq_oracle.c`` with gcc) through
ctypes and exposes each oracle function on numpy arrays.  Only the tests, the
smoke check and the CPU-baseline leg of the benchmark may import this module;
it imports nothing from the GPU package.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.environ.get("NDQ_ORACLE_LIBRARY", os.path.join(_HERE, "libndq_oracle.so"))   # override: another build
_SRC = os.path.join(_HERE, "ndq_oracle.c")
_HDR = os.path.join(_HERE, "ndq_oracle.h")

F32, BF16 = 0, 1


def build(force=False):
    """Compile the oracle with gcc (no contraction, no fast-math)."""
    if "NDQ_ORACLE_LIBRARY" in os.environ:      # somebody else's build (a sanitizer run): use it as it is
        return _SO
    stale = (not os.path.exists(_SO)) or any(
        os.path.getmtime(p) > os.path.getmtime(_SO) for p in (_SRC, _HDR))
    if force or stale:
        subprocess.check_call([
            "gcc", "-std=c99", "-O2", "-ffp-contract=off", "-fno-fast-math", "-Wall",
            "-Wextra", "-shared", "-fPIC", "-o", _SO, _SRC, "-lm"])
    return _SO


class Dither(C.Structure):
    _fields_ = [("seed", C.c_uint64), ("step", C.c_uint32), ("worker", C.c_uint32),
                ("offset", C.c_uint64)]


def dither(seed=0, step=0, worker=0, offset=0):
    return Dither(seed, step, worker, offset)


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_SO)
        vp, sz, u32, f32, i32 = C.c_void_p, C.c_size_t, C.c_uint32, C.c_float, C.c_int
        L.oracle_philox4x32_10.argtypes = [vp, vp, vp]
        L.oracle_philox4x32_10.restype = None
        L.oracle_unit_dither.argtypes = [C.c_uint64, u32, u32, C.c_uint64]
        L.oracle_unit_dither.restype = f32
        L.oracle_unit_dithers.argtypes = [Dither, sz, vp]
        L.oracle_unit_dithers.restype = None
        L.oracle_code_bits.argtypes = [u32]
        L.oracle_code_bits.restype = u32
        L.oracle_step_from_kappa.argtypes = [f32, u32]
        L.oracle_step_from_kappa.restype = f32
        L.oracle_inv_step.argtypes = [f32]
        L.oracle_inv_step.restype = f32
        L.oracle_dq_code.argtypes = [f32, f32, f32, u32]
        L.oracle_dq_code.restype = u32
        L.oracle_dq_value.argtypes = [u32, f32, f32, u32]
        L.oracle_dq_value.restype = f32
        L.oracle_dq_value_f64.argtypes = [u32, C.c_double, C.c_double, u32]
        L.oracle_dq_value_f64.restype = C.c_double
        L.oracle_fine_index.argtypes = [f32, f32, f32]
        L.oracle_fine_index.restype = C.c_int32
        L.oracle_nested_code.argtypes = [f32, f32, f32, u32]
        L.oracle_nested_code.restype = u32
        L.oracle_coset_index.argtypes = [u32, f32, f32, f32, u32]
        L.oracle_coset_index.restype = C.c_int32
        L.oracle_coset_k.argtypes = [u32, f32, f32, f32, u32]
        L.oracle_coset_k.restype = f32
        L.oracle_coset_value.argtypes = [f32, u32, u32, f32, f32]
        L.oracle_coset_value.restype = f32
        L.oracle_index_value.argtypes = [C.c_int32, f32, f32]
        L.oracle_index_value.restype = f32
        L.oracle_nested_code_alpha.argtypes = [f32, f32, f32, f32, u32]
        L.oracle_nested_code_alpha.restype = u32
        L.oracle_nested_value_alpha.argtypes = [u32, f32, f32, f32, f32, u32]
        L.oracle_nested_value_alpha.restype = f32
        L.oracle_alpha_for_equal_variance.argtypes = [C.c_double, C.c_double]
        L.oracle_alpha_for_equal_variance.restype = C.c_double
        L.oracle_decode_error_bound.argtypes = [C.c_double, u32, C.c_double, C.c_double]
        L.oracle_decode_error_bound.restype = C.c_double
        L.oracle_nesting_ratio_for_error.argtypes = [C.c_double, C.c_double, C.c_double, C.c_double]
        L.oracle_nesting_ratio_for_error.restype = u32
        L.oracle_sqdiff_sum.argtypes = [vp, vp, sz]
        L.oracle_sqdiff_sum.restype = C.c_double
        L.oracle_packed_bytes.argtypes = [sz, u32]
        L.oracle_packed_bytes.restype = sz
        L.oracle_num_buckets.argtypes = [sz, u32]
        L.oracle_num_buckets.restype = sz
        L.oracle_pack.argtypes = [vp, sz, u32, vp]
        L.oracle_pack.restype = None
        L.oracle_unpack.argtypes = [vp, sz, u32, vp]
        L.oracle_unpack.restype = None
        L.oracle_absmax.argtypes = [vp, i32, sz, u32, vp]
        L.oracle_absmax.restype = None
        L.oracle_dq_encode.argtypes = [vp, i32, sz, f32, u32, u32, Dither, vp, vp]
        L.oracle_dq_encode.restype = None
        L.oracle_dq_decode.argtypes = [vp, sz, u32, u32, vp, Dither, vp, i32]
        L.oracle_dq_decode.restype = None
        L.oracle_dq_value_half.argtypes = [u32, f32, u32]
        L.oracle_dq_value_half.restype = f32
        L.oracle_dq_decode_half.argtypes = [vp, sz, u32, u32, vp, vp, i32]
        L.oracle_dq_decode_half.restype = None
        L.oracle_dense_group.argtypes, L.oracle_dense_group.restype = [u32], u32
        L.oracle_dense_bytes.argtypes, L.oracle_dense_bytes.restype = [sz, u32], sz
        L.oracle_dense_pack.argtypes, L.oracle_dense_pack.restype = [vp, sz, u32, vp], None
        L.oracle_dense_unpack.argtypes, L.oracle_dense_unpack.restype = [vp, sz, u32, vp], None
        L.oracle_code_histogram.argtypes = [vp, sz, u32, vp]
        L.oracle_code_histogram.restype = None
        L.oracle_entropy_bits.argtypes = [vp, u32]
        L.oracle_entropy_bits.restype = C.c_double
        L.oracle_nested_encode.argtypes = [vp, i32, sz, f32, u32, u32, f32, u32, Dither, vp, vp]
        L.oracle_nested_encode.restype = None
        L.oracle_nested_decode.argtypes = [vp, sz, u32, f32, u32, vp, Dither, vp, f32, vp, i32]
        L.oracle_nested_decode.restype = None
        L.oracle_aggregate.argtypes = [vp, u32, sz, f32, vp]
        L.oracle_aggregate.restype = None
        L.oracle_fine_indices.argtypes = [vp, i32, sz, u32, vp, Dither, vp]
        L.oracle_fine_indices.restype = None
        L.oracle_coset_indices.argtypes = [vp, sz, u32, u32, vp, Dither, vp, f32, vp]
        L.oracle_coset_indices.restype = None
        _lib = L
    return _lib


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


def _dtype_of(g):
    if g.dtype == np.float32:
        return F32
    if g.dtype == np.uint16:  # bfloat16 bit patterns
        return BF16
    raise TypeError("gradient must be float32 or uint16 (bfloat16 bits)")


# ---- scalar functions -------------------------------------------------------

def philox4x32_10(ctr, key):
    ctr = np.ascontiguousarray(ctr, dtype=np.uint32)
    key = np.ascontiguousarray(key, dtype=np.uint32)
    out = np.empty(4, dtype=np.uint32)
    lib().oracle_philox4x32_10(_p(ctr), _p(key), _p(out))
    return out


def unit_dither(seed, step, worker, i):
    return lib().oracle_unit_dither(seed, step, worker, i)


def unit_dithers(d, n):
    v = np.empty(n, dtype=np.float32)
    lib().oracle_unit_dithers(d, n, _p(v))
    return v


def code_bits(x):
    return lib().oracle_code_bits(x)


def step_from_kappa(kappa, levels):
    return lib().oracle_step_from_kappa(kappa, levels)


def inv_step(delta):
    return lib().oracle_inv_step(delta)


def dq_code(g, inv_delta, v, levels):
    return lib().oracle_dq_code(g, inv_delta, v, levels)


def dq_value(code, delta, v, levels):
    return lib().oracle_dq_value(code, delta, v, levels)


def dq_value_f64(code, delta, v, levels):
    return lib().oracle_dq_value_f64(code, delta, v, levels)


def fine_index(g, inv_delta, v):
    return lib().oracle_fine_index(g, inv_delta, v)


def nested_code(g, inv_delta, v, M):
    return lib().oracle_nested_code(g, inv_delta, v, M)


def coset_index(m, y, inv_delta, v, M):
    return lib().oracle_coset_index(m, y, inv_delta, v, M)


def coset_k(m, y, inv_delta, v, M):
    """k of the coset representative m + M k (a binary32 integer value, unbounded)."""
    return lib().oracle_coset_k(m, y, inv_delta, v, M)


def coset_value(k, m, M, delta, v):
    return lib().oracle_coset_value(k, m, M, delta, v)


def index_value(q, delta, v):
    return lib().oracle_index_value(q, delta, v)


def nested_code_alpha(g, inv_delta, alpha, v, M):
    return lib().oracle_nested_code_alpha(g, inv_delta, alpha, v, M)


def nested_value_alpha(m, y, delta, alpha, v, M):
    return lib().oracle_nested_value_alpha(m, y, delta, alpha, v, M)


def alpha_for_equal_variance(delta1, sigma_z2):
    return lib().oracle_alpha_for_equal_variance(delta1, sigma_z2)


def decode_error_bound(delta1, M, alpha, sigma_z2):
    return lib().oracle_decode_error_bound(delta1, M, alpha, sigma_z2)


def nesting_ratio_for_error(delta1, alpha, sigma_z2, p_max):
    return lib().oracle_nesting_ratio_for_error(delta1, alpha, sigma_z2, p_max)


def sqdiff_sum(a, b):
    a = np.ascontiguousarray(a, dtype=np.float32)
    b = np.ascontiguousarray(b, dtype=np.float32)
    assert a.size == b.size
    return lib().oracle_sqdiff_sum(_p(a), _p(b), a.size)


def packed_bytes(n, bits):
    return lib().oracle_packed_bytes(n, bits)


def num_buckets(n, bucket):
    return lib().oracle_num_buckets(n, bucket)


# ---- vector functions -------------------------------------------------------

def pack(codes, bits):
    codes = np.ascontiguousarray(codes, dtype=np.uint32)
    out = np.empty(packed_bytes(codes.size, bits), dtype=np.uint8)
    lib().oracle_pack(_p(codes), codes.size, bits, _p(out))
    return out


def unpack(packed, n, bits):
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    assert packed.size >= packed_bytes(n, bits)
    codes = np.empty(n, dtype=np.uint32)
    lib().oracle_unpack(_p(packed), n, bits, _p(codes))
    return codes


def absmax(g, bucket=0):
    g = np.ascontiguousarray(g)
    out = np.empty(num_buckets(g.size, bucket), dtype=np.float32)
    lib().oracle_absmax(_p(g), _dtype_of(g), g.size, bucket, _p(out))
    return out


def dq_encode(g, delta, levels, bucket, d):
    """-> (packed codes uint8, steps float32)"""
    g = np.ascontiguousarray(g)
    codes = np.empty(packed_bytes(g.size, code_bits(levels)), dtype=np.uint8)
    steps = np.empty(num_buckets(g.size, bucket), dtype=np.float32)
    lib().oracle_dq_encode(_p(g), _dtype_of(g), g.size, delta, levels, bucket, d,
                           _p(codes), _p(steps))
    return codes, steps


def dq_decode(codes, n, levels, bucket, steps, d, out=None):
    """out given -> accumulate into it; returns the float32 vector."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    steps = np.ascontiguousarray(steps, dtype=np.float32)
    acc = out is not None
    if out is None:
        out = np.empty(n, dtype=np.float32)
    assert out.dtype == np.float32 and out.size == n and out.flags.c_contiguous
    lib().oracle_dq_decode(_p(codes), n, levels, bucket, _p(steps), d, _p(out), int(acc))
    return out


def dq_value_half(code, delta, levels):
    return lib().oracle_dq_value_half(code, delta, levels)


def dq_decode_half(codes, n, levels, bucket, steps, out=None):
    """Half-dithered reconstruction Delta*q (no dither subtraction)."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    steps = np.ascontiguousarray(steps, dtype=np.float32)
    acc = out is not None
    if out is None:
        out = np.empty(n, dtype=np.float32)
    assert out.dtype == np.float32 and out.size == n and out.flags.c_contiguous
    lib().oracle_dq_decode_half(_p(codes), n, levels, bucket, _p(steps), _p(out), int(acc))
    return out


def dense_group(levels):
    return lib().oracle_dense_group(levels)


def dense_bytes(n, levels):
    return lib().oracle_dense_bytes(n, levels)


def dense_pack(codes, levels):
    codes = np.ascontiguousarray(codes, dtype=np.uint32)
    out = np.empty(dense_bytes(codes.size, levels), dtype=np.uint8)
    lib().oracle_dense_pack(_p(codes), codes.size, levels, _p(out))
    return out


def dense_unpack(dense, n, levels):
    dense = np.ascontiguousarray(dense, dtype=np.uint8)
    assert dense.size >= dense_bytes(n, levels)
    codes = np.empty(n, dtype=np.uint32)
    lib().oracle_dense_unpack(_p(dense), n, levels, _p(codes))
    return codes


def code_histogram(codes, n, bits):
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    hist = np.zeros(1 << bits, dtype=np.uint64)
    lib().oracle_code_histogram(_p(codes), n, bits, _p(hist))
    return hist


def entropy_bits(hist):
    hist = np.ascontiguousarray(hist, dtype=np.uint64)
    return lib().oracle_entropy_bits(_p(hist), hist.size)


def nested_encode(g, delta, levels, M, bucket, d, alpha=1.0):
    g = np.ascontiguousarray(g)
    codes = np.empty(packed_bytes(g.size, code_bits(M)), dtype=np.uint8)
    steps = np.empty(num_buckets(g.size, bucket), dtype=np.float32)
    lib().oracle_nested_encode(_p(g), _dtype_of(g), g.size, delta, levels, M, np.float32(alpha),
                               bucket, d, _p(codes), _p(steps))
    return codes, steps


def nested_decode(codes, n, M, bucket, steps, d, side, side_scale=1.0, out=None, alpha=1.0):
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    steps = np.ascontiguousarray(steps, dtype=np.float32)
    side = np.ascontiguousarray(side, dtype=np.float32)
    acc = out is not None
    if out is None:
        out = np.empty(n, dtype=np.float32)
    assert out.dtype == np.float32 and out.size == n and out.flags.c_contiguous
    lib().oracle_nested_decode(_p(codes), n, M, np.float32(alpha), bucket, _p(steps), d, _p(side),
                               np.float32(side_scale), _p(out), int(acc))
    return out


def aggregate(gs, scale=1.0):
    gs = [np.ascontiguousarray(g, dtype=np.float32) for g in gs]
    n = gs[0].size
    ptrs = (C.c_void_p * len(gs))(*[g.ctypes.data for g in gs])
    out = np.empty(n, dtype=np.float32)
    lib().oracle_aggregate(C.cast(ptrs, C.c_void_p), len(gs), n, np.float32(scale), _p(out))
    return out


def fine_indices(g, bucket, steps, d):
    g = np.ascontiguousarray(g)
    steps = np.ascontiguousarray(steps, dtype=np.float32)
    q = np.empty(g.size, dtype=np.int32)
    lib().oracle_fine_indices(_p(g), _dtype_of(g), g.size, bucket, _p(steps), d, _p(q))
    return q


def coset_indices(codes, n, M, bucket, steps, d, side, side_scale=1.0):
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    steps = np.ascontiguousarray(steps, dtype=np.float32)
    side = np.ascontiguousarray(side, dtype=np.float32)
    q = np.empty(n, dtype=np.int32)
    lib().oracle_coset_indices(_p(codes), n, M, bucket, _p(steps), d, _p(side),
                               np.float32(side_scale), _p(q))
    return q
