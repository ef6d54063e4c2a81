"""The exact-arithmetic identities the streaming kernels rely on, checked on the CPU
with rational arithmetic: every operation below is "the exact result, rounded once to
binary32, ties to even", which is what an IEEE add, multiply or fused multiply-add
does.  Nothing here calls the library or the oracle; the GPU parity tests compare the
kernels' results with the oracle's, these tests show why the rearranged forms must
give the same bits as the plain ones (eq. (2), eqs. (7)-(8), Algorithm 1's server step).
"""
from fractions import Fraction
import random
import struct

import numpy as np


def f32(x):
    """A rational rounded once to binary32 (ties to even), as a Fraction."""
    x = Fraction(x)
    if x == 0:
        return Fraction(0)
    sign = -1 if x < 0 else 1
    a = abs(x)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    assert Fraction(2) ** e <= a < Fraction(2) ** (e + 1)
    e = max(e, -126)                       # subnormals share the smallest normal's spacing
    ulp = Fraction(2) ** (e - 23)
    q = a / ulp
    n = q.numerator // q.denominator
    rem = q - n
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and n % 2 == 1):
        n += 1
    return sign * n * ulp


def is_f32(x):
    return f32(x) == Fraction(x)


def fma(a, b, c):
    return f32(Fraction(a) * Fraction(b) + Fraction(c))


def rint(x):
    """Nearest integer, ties to even, of an exact value."""
    x = Fraction(x)
    n = x.numerator // x.denominator
    rem = x - n
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and n % 2 == 1):
        n += 1
    return Fraction(n)


def bits_to_f32(u):
    return Fraction(struct.unpack("<f", struct.pack("<I", u & 0xFFFFFFFF))[0])


C0 = Fraction(-1, 2) + Fraction(1, 2 ** 17)       # centre of cell 0 of the 16-bit dither grid


def unit_dither(cell, centre=C0):
    return fma(cell, Fraction(1, 2 ** 16), centre)


def test_rounding_helper_agrees_with_numpy():
    rng = random.Random(5)
    for _ in range(2000):
        x = Fraction(rng.getrandbits(60) - (1 << 59), 1 << rng.randrange(1, 70))
        assert f32(x) == Fraction(float(np.float32(float(x)))) or abs(x) < Fraction(1, 2 ** 120)
    assert f32(Fraction(1) + Fraction(1, 2 ** 24)) == 1                       # tie to even, down
    assert f32(Fraction(1) + Fraction(3, 2 ** 24)) == 1 + Fraction(1, 2 ** 22)  # tie to even, up


def test_unit_dither_is_exact_and_so_is_its_shift_by_an_index_offset():
    # v = (cell + 1/2) 2^-16 - 1/2 needs 17 bits; v - q_min needs at most 21 for |q_min| <= 8
    for cell in list(range(0, 65536, 257)) + [0, 1, 65534, 65535]:
        v = unit_dither(cell)
        assert v == Fraction(2 * cell + 1, 2 ** 17) - Fraction(1, 2)
        for q_min in range(-8, 1):
            centre = f32(Fraction(-q_min) + C0)
            assert centre == Fraction(-q_min) + C0                      # the constant itself is exact
            assert unit_dither(cell, centre) == v - q_min               # and so is the one fma


def test_dq_index_offset_folded_into_the_dither_gives_the_same_reconstruction():
    # Algorithm 1's server step Delta * ((c + q_min) - v) against Delta * (c - (v - q_min))
    rng = random.Random(11)
    for _ in range(3000):
        cell = rng.randrange(65536)
        levels = rng.choice([2, 3, 4, 5, 8, 16])
        q_min = -(levels // 2)
        c = rng.randrange(levels)
        step = f32(Fraction(rng.getrandbits(24) + 1, 1 << rng.randrange(20, 40)))
        v = unit_dither(cell)
        plain = f32(step * f32(Fraction(c + q_min) - v))
        shifted = f32(step * f32(Fraction(c) - unit_dither(cell, f32(Fraction(-q_min) + C0))))
        assert plain == shifted


def test_code_field_masked_into_a_power_of_two_mantissa():
    # (group & mask_j) | bits(2^(23 - j b - s)) read as a float is 2^(23-jb-s) + c 2^-s exactly;
    # subtracting 2^(23-jb-s) leaves c 2^-s (s = 0: the code; s = b: the code over M = 2^b)
    rng = random.Random(3)
    for b in (1, 2, 4):
        nf = 4 if b == 4 else 8
        for s in (0, b):
            for j in range(nf):
                mask = ((1 << b) - 1) << (j * b)
                base = (150 - j * b - s) << 23
                assert bits_to_f32(base) == Fraction(2) ** (23 - j * b - s)
                for _ in range(50):
                    group = rng.getrandbits(16 if b == 4 else 8 * b)
                    c = (group >> (j * b)) & ((1 << b) - 1)
                    x = bits_to_f32((group & mask) | base)
                    assert x == Fraction(2) ** (23 - j * b - s) + Fraction(c, 2 ** s)
                    assert f32(x - bits_to_f32(base)) == Fraction(c, 2 ** s)


def test_nested_decode_in_ten_float_operations_equals_the_plain_coset_decoder():
    # plain (eq. (8), alpha = 1, M = 2^b): c = fma(y, 1/Delta, v); k = rint((c - m) / M) with the
    # difference and the scaling each rounded; q = fma(k, M, m); S + Delta * (q - v)
    # streaming form: m' = m / M; k = rint(fma(c, 1/M, -m')); q' = k + m'; S + Delta * fma(q', M, -v)
    rng = random.Random(23)
    for _ in range(4000):
        b = rng.choice([1, 2, 4])
        M = 1 << b
        m = rng.randrange(M)
        cell = rng.randrange(65536)
        v = unit_dither(cell)
        step = f32(Fraction(rng.getrandbits(24) + 1, 1 << rng.randrange(24, 36)))
        inv = f32(1 / step)
        S = f32(Fraction(rng.getrandbits(26) - (1 << 25), 1 << rng.randrange(20, 44)))
        side = f32(Fraction(1, rng.choice([1, 2, 3, 5, 7])))
        y = f32(S * side)
        c = fma(y, inv, v)
        # plain
        diff = f32(c - m)
        k_plain = rint(f32(diff * Fraction(1, M)))
        q_plain = fma(k_plain, M, m)
        plain = f32(S + f32(step * f32(q_plain - v)))
        # streaming
        mp = Fraction(m, M)
        k_s = rint(fma(c, Fraction(1, M), -mp))
        qp = f32(k_s + mp)
        stream = f32(S + f32(step * fma(qp, M, -v)))
        assert k_plain == k_s and plain == stream, (b, m, cell, float(step), float(S))


def test_magic_constant_addition_is_round_to_nearest_even():
    # t + 1.5 * 2^23 for |t| < 2^22: the sum's unit in the last place is 1, so the one rounding of
    # the addition is rint(t), and the low mantissa bits hold the index in two's complement
    magic = Fraction(3 * 2 ** 22)
    rng = random.Random(7)
    cases = [Fraction(k, 2) for k in range(-9, 10)]
    cases += [f32(Fraction(rng.getrandbits(30) - (1 << 29), 1 << rng.randrange(8, 30))) for _ in range(3000)]
    for t in cases:
        if abs(t) >= 2 ** 22:
            continue
        s = f32(t + magic)
        assert s - magic == rint(t)
        word = struct.unpack("<I", struct.pack("<f", float(s)))[0]
        for bits in (1, 2, 4):
            assert (word & ((1 << bits) - 1)) == int(rint(t)) % (1 << bits)


def test_base_three_digits_two_at_a_time_with_small_multiplies():
    # the dense base-3 stream (Table 1's log2(3) bits per index): a 32-bit word holds 20 digits;
    # its halves below 3^10 fit 16 bits, where y // 9 == (y * 58255) >> 19 with a product below
    # 2^32 and factors below 2^24, and the two 2-bit codes c0 + 4 c1 of a remainder r = c0 + 3 c1
    # are r + r // 3 with r // 3 == (r * 11) >> 5
    assert 3 ** 20 < 2 ** 32 <= 3 ** 21 and 3 ** 10 < 2 ** 16
    for y in range(1 << 16):
        assert (y * 58255) >> 19 == y // 9 and y * 58255 < 1 << 32
    for r in range(9):
        assert r + ((r * 11) >> 5) == (r % 3) + 4 * (r // 3)
    rng = random.Random(17)
    for _ in range(2000):
        digits = [rng.randrange(3) for _ in range(20)]
        value = sum(c * 3 ** d for d, c in enumerate(digits))
        top = value // 59049
        got = []
        for y in (value - top * 59049, top):
            for _pair in range(5):
                q = (y * 58255) >> 19
                r = y - 9 * q
                pair = r + ((r * 11) >> 5)
                got += [pair & 3, pair >> 2]
                y = q
        assert got == digits


def test_step_rule_is_monotone_so_the_maximum_of_steps_is_the_step_of_the_maximum():
    # Sec. 3.1 eq. (2): Delta = 2 kappa / (L - 1), kappa = max |g|.  The two-pass encoder lets every
    # part of a bucket convert its own max-norm and takes the maximum of the steps; that equals the
    # step of the bucket's max-norm because each operation of the rule (an exact doubling, a correctly
    # rounded division, the threshold below 2^-100) is monotone.
    def step(kappa, levels):
        s = np.float32(np.float32(2.0) * kappa) / np.float32(levels - 1)
        return s if s >= np.float32(2.0 ** -100) else np.float32(0.0)

    rng = np.random.default_rng(41)
    for levels in (2, 3, 4, 5, 7, 16, 100, 255, 256):
        parts = np.abs(rng.standard_normal((400, 9)).astype(np.float32)) * \
            np.float32(10.0) ** rng.integers(-38, 6, size=(400, 1)).astype(np.float32)
        parts[::7, 3] = 0.0
        parts[5] = 0.0
        with np.errstate(over="ignore", under="ignore"):
            for row in parts:
                assert max(step(k, levels) for k in row) == step(row.max(), levels)
            # neighbours in binary32 around the threshold and around a power of two
            for centre in (2.0 ** -101, 2.0 ** -100, 2.0 ** -99, 1.0, 3.0e38):
                k = np.float32(centre)
                for _ in range(200):
                    nxt = np.nextafter(k, np.float32(np.inf))
                    assert step(k, levels) <= step(nxt, levels)
                    k = nxt
