// Device-side building blocks of libndq (gfx950 only): the Philox dither, the
// step rule, the scalar quantizers and the wave-level helpers.
//
// Everything that decides an integer is written as explicit IEEE binary32
// operations (the file is compiled with -ffp-contract=off): one fma and one
// round-to-nearest-even per index, one correctly rounded division per bucket.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ndq {

constexpr int kWave = 64;           // CDNA wavefront
#ifndef NDQ_WAVES_PER_BLOCK
#define NDQ_WAVES_PER_BLOCK 4
#endif
constexpr int kWavesPerBlock = NDQ_WAVES_PER_BLOCK;   // waves of a workgroup work independently
constexpr int kBlock = kWave * kWavesPerBlock;
// Encoder tile: eight 16-byte loads in flight per lane (4096 bfloat16 or 2048
// binary32 elements per wave), the largest bucket whose max-norm one wave reduces.
constexpr int kEncLoads = 8;
#ifndef NDQ_DEC_ROWS_STREAM
#define NDQ_DEC_ROWS_STREAM 4
#endif
#ifndef NDQ_DEC_ROWS_UPDATE
#define NDQ_DEC_ROWS_UPDATE 4
#endif
// 16-byte stores per lane and decoder tile, for decoders that only write values
// (DQSG, no accumulate) and for those that also read values (side information,
// running sum).  Measured at n = 2^27 with streaming accesses: 4 rows (4 KB of
// values per wave) is fastest for both -- 82 us against 106 us with 8 rows for the
// store-only decoder, 167 us against 171 (2 rows), 174 (8) and 176 (1) for the
// in-place nested decoder.  Short tiles keep the reads and writes in flight on
// the chip within a few MB of HBM; very short ones pay per-wave overhead.
constexpr int kDecRowsStream = NDQ_DEC_ROWS_STREAM;
constexpr int kDecRowsUpdate = NDQ_DEC_ROWS_UPDATE;

// ---------------------------------------------------------------------------
// Dither (Sec. 2.1 Remark 1: the receiver regenerates the dither from the same
// generator and seed).  Philox4x32 with 10 rounds, Salmon et al., SC'11: per
// round two 32x32->64 multiplies, the high halves are xor-ed with the other two
// counter words and the round key, the key advances by a Weyl constant.
// ---------------------------------------------------------------------------
struct DitherStream {
    uint32_t key0, key1;   // seed, low and high word
    uint32_t step;         // training iteration
    uint32_t worker;       // worker index p
};

__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c)
{
    // gfx950 three-input bitwise op; truth table 0x96 = a ^ b ^ c
    return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);
}

__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t (&out)[4])
{
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = xor3((uint32_t)(p1 >> 32), c1, k0);
        const uint32_t n2 = xor3((uint32_t)(p0 >> 32), c3, k1);
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// Nothing is scheduled across this point: the instruction order of the source is
// the order of the program.
#define NDQ_PIN() __builtin_amdgcn_sched_barrier(0)

// One Philox block advanced a piece at a time, so that the caller can place other
// work between the pieces: a round is mul0, mul1, mix0, mix1, next_round in that
// order (each mix needs both products' owner words untouched: mul0 before mix0,
// mul1 before mix1).  After ten rounds words() are those of philox4x32_10.
struct PhiloxFlight {
    uint32_t c0, c1, c2, c3, k0, k1;
    uint64_t p0, p1;
    __device__ __forceinline__ void start(const DitherStream& s, uint64_t block)
    {
        c0 = (uint32_t)block; c1 = (uint32_t)(block >> 32); c2 = s.step; c3 = s.worker;
        k0 = s.key0; k1 = s.key1;
    }
    // the 32x32->64 multiply as the one instruction it is (left to the compiler it becomes a
    // high and a low multiply once the two halves are used in different pinned regions)
    static __device__ __forceinline__ uint64_t wide_mul(uint32_t constant, uint32_t x)
    {
        uint64_t p;
        asm("v_mad_u64_u32 %0, vcc, %1, %2, 0" : "=v"(p) : "s"(constant), "v"(x) : "vcc");
        return p;
    }
    __device__ __forceinline__ void mul0() { p0 = wide_mul(0xD2511F53u, c0); }
    __device__ __forceinline__ void mul1() { p1 = wide_mul(0xCD9E8D57u, c2); }
    __device__ __forceinline__ void mix0() { c0 = xor3((uint32_t)(p1 >> 32), c1, k0); c1 = (uint32_t)p1; }
    __device__ __forceinline__ void mix1() { c2 = xor3((uint32_t)(p0 >> 32), c3, k1); c3 = (uint32_t)p0; }
    __device__ __forceinline__ void next_round() { k0 += 0x9E3779B9u; k1 += 0xBB67AE85u; }
    __device__ __forceinline__ void run()
    {
#pragma unroll
        for (int round = 0; round < 10; ++round) { mul0(); mul1(); mix0(); mix1(); next_round(); }
    }
    __device__ __forceinline__ void words(uint32_t (&r)[4]) const { r[0] = c0; r[1] = c1; r[2] = c2; r[3] = c3; }
};

// Mid-point of cell `cell` of 2^16 equal cells of [-1/2, 1/2): exact in binary32.
__device__ __forceinline__ float unit_dither(uint32_t cell)
{
    return __builtin_fmaf((float)cell, 0x1p-16f, -0.5f + 0x1p-17f);
}

// One Philox block serves eight consecutive elements, 16 bits each: element I
// takes half (I mod 2) of word ((I/2) mod 4) of block I/8.

// The eight unit dithers of elements 8*block .. 8*block+7.
__device__ __forceinline__ void dither8(const DitherStream& s, uint64_t block, float (&v)[8])
{
    uint32_t r[4];
    philox4x32_10((uint32_t)block, (uint32_t)(block >> 32), s.step, s.worker, s.key0, s.key1, r);
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        v[2 * w] = unit_dither(r[w] & 0xFFFFu);
        v[2 * w + 1] = unit_dither(r[w] >> 16);
    }
}

// The same plus an integer `shift` with |shift| <= 8: v + shift needs at most 21
// significant bits, so the one fma that forms it is as exact as unit_dither's.
__device__ __forceinline__ float unit_dither_shifted(uint32_t cell, float centre)   // centre = shift - 1/2 + 2^-17
{
    return __builtin_fmaf((float)cell, 0x1p-16f, centre);
}
__device__ __forceinline__ void dither8_shifted(const DitherStream& s, uint64_t block, float shift, float (&v)[8])
{
    uint32_t r[4];
    philox4x32_10((uint32_t)block, (uint32_t)(block >> 32), s.step, s.worker, s.key0, s.key1, r);
    const float centre = shift + (-0.5f + 0x1p-17f);
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        v[2 * w] = unit_dither_shifted(r[w] & 0xFFFFu, centre);
        v[2 * w + 1] = unit_dither_shifted(r[w] >> 16, centre);
    }
}

// The four unit dithers of elements 4*quad .. 4*quad+3 (half a block; used where
// a lane owns four elements and memory, not arithmetic, is the limit).
__device__ __forceinline__ void dither4(const DitherStream& s, uint64_t quad, float (&v)[4])
{
    const uint64_t block = quad >> 1;
    uint32_t r[4];
    philox4x32_10((uint32_t)block, (uint32_t)(block >> 32), s.step, s.worker, s.key0, s.key1, r);
    const bool upper = (quad & 1u) != 0u;
    const uint32_t a = upper ? r[2] : r[0], b = upper ? r[3] : r[1];
    v[0] = unit_dither(a & 0xFFFFu);
    v[1] = unit_dither(a >> 16);
    v[2] = unit_dither(b & 0xFFFFu);
    v[3] = unit_dither(b >> 16);
}

// ---------------------------------------------------------------------------
// Step rule (Sec. 3.1 eq. (2)): kappa = max|g| maps g into [-1,1]; 2M+1 levels
// have normalised step 1/M = 2/(L-1); in absolute units Delta = 2 kappa/(L-1).
// ---------------------------------------------------------------------------
__device__ __forceinline__ float step_from_kappa(float kappa, uint32_t levels)
{
    float step = (2.0f * kappa) / (float)(levels - 1u);
    if (!(step >= 0x1p-100f)) step = 0.0f;
    return step;
}

__device__ __forceinline__ float inv_step(float step)
{
    return (step > 0.0f) ? 1.0f / step : 0.0f;
}

// ---------------------------------------------------------------------------
// Quantizer parameters shared by encoder and decoder.
//   kDq           : DQSG, clipped to `levels` indices            (Algorithm 1)
//   kDqNarrow     : the same for codes of at most 6 bits (encoder packs in float)
//   kDqHalf       : decoder only: half-dithered reconstruction Delta*q, no dither
//                   regenerated (Sec. 2.1, last paragraph; Lemma 1)
//   kNestedPow2   : NDQSG, M a power of two (mask / exact scale); decoder: alpha = 1
//   kNestedPow2Shrink : decoder only: M a power of two, shrinkage factor alpha < 1
//   kNestedAnyM   : NDQSG, any M in [2,256], any shrinkage factor alpha in (0,1]
//   kNestedPow2Bounded : encoder only: M a power of two and the step derived from
//                   the bucket's own max-norm, so |g/Delta + v| <= 128.1 (see
//                   nested_low_bits)
//   kNestedAnyMBounded : encoder only: the same bound, any M up to 64 (see
//                   nested_residue_f)
// ---------------------------------------------------------------------------
enum Mode { kDq = 0, kNestedPow2 = 1, kNestedAnyM = 2, kDqNarrow = 3, kDqHalf = 4, kNestedPow2Shrink = 5,
            kNestedPow2Bounded = 6, kNestedAnyMBounded = 7 };

struct Quant {
    float q_min_f, q_max_f;  // DQSG index range as floats
    int32_t q_min;           // -(levels/2)
    uint32_t levels;         // fixes the step: Delta = 2 kappa/(levels-1)
    uint32_t M;              // nesting ratio Delta_2/Delta_1 (nested modes)
    float M_f, inv_M_f;      // (float)M and 1/M rounded to binary32 (exact for powers of two)
    uint32_t bits;           // code width
    float pack_bias;         // kDqNarrow: -q_min * sum_k 2^(k*bits), k = 0..3 (codes of <= 6 bits)
    float alpha, beta;       // nested: shrinkage factor and 1 - alpha^2 (kNestedAnyM when alpha < 1)
};

// Clipped index of eq. (2) / Algorithm 1, still as a float (an exact small integer).
__device__ __forceinline__ float dq_index_f(float g, float inv, float v, const Quant& qp)
{
    const float r = __builtin_rintf(__builtin_fmaf(g, inv, v));
    return __builtin_amdgcn_fmed3f(r, qp.q_min_f, qp.q_max_f);   // clip: median of (r, lo, hi)
}

// The same as a code in [0, levels).
__device__ __forceinline__ uint32_t dq_code(float g, float inv, float v, const Quant& qp)
{
    return (uint32_t)((int32_t)dq_index_f(g, inv, v, qp) - qp.q_min);
}

// Fine index of eq. (7) reduced modulo M.
template <int MODE>
__device__ __forceinline__ uint32_t nested_code(float g, float inv, float v, const Quant& qp)
{
    float r = __builtin_rintf(__builtin_fmaf(g, inv, v));
    r = __builtin_fminf(__builtin_fmaxf(r, -16777216.0f), 16777216.0f);
    const int32_t q = (int32_t)r;
    if (MODE == kNestedPow2 || MODE == kNestedPow2Shrink) return (uint32_t)q & (qp.M - 1u);
    int32_t m = q % (int32_t)qp.M;
    if (m < 0) m += (int32_t)qp.M;
    return (uint32_t)m;
}

// Fine index of eq. (7) for |t| < 2^22, t = g/Delta + v, as a word whose low 22
// bits are the index in two's complement: adding 1.5 * 2^23 moves t into the
// binade whose unit in the last place is 1, so that one addition rounds it to
// the nearest integer, ties to even (1.5 * 2^23 is even: the parity of the sum is
// the parity of the index) -- exactly rint(t), without convert or mask.  The
// index mod 2^b is then the low b bits.
__device__ __forceinline__ uint32_t nested_low_bits(float g, float inv, float v)
{
    const float t = __builtin_fmaf(g, inv, v);
    return __float_as_uint(t + 12582912.0f);
}

// Fine index of eq. (7) reduced mod M, as a float, for |q| <= 2^8 (a step derived
// from the data) and any M in [2, 256]: k = floor(q/M) is floor(q * (1/M) + 1/(2M)).
// The exact value q/M + 1/(2M) is at least 1/(2M) >= 2^-9 away from every
// integer, the rounded reciprocal and the fma put the computed one within 2^-15
// of it, so the floor is exact; q - k M is then formed exactly by one fma.
__device__ __forceinline__ float nested_residue_f(float g, float inv, float v, const Quant& qp)
{
    const float q = __builtin_rintf(__builtin_fmaf(g, inv, v));
    const float k = __builtin_floorf(__builtin_fmaf(q, qp.inv_M_f, 0.5f * qp.inv_M_f));
    return __builtin_fmaf(-k, qp.M_f, q);
}

template <int MODE>
__device__ __forceinline__ uint32_t encode_one(float g, float inv, float v, const Quant& qp)
{
    if (MODE == kDq || MODE == kDqNarrow) return dq_code(g, inv, v, qp);
    return nested_code<MODE>(g, inv, v, qp);
}

// eq. (8) with a shrinkage factor: y + alpha (r - Q2(r)) = (1 - alpha^2) y + alpha * lattice
template <int MODE>
__device__ __forceinline__ float shrink(float lattice, float y, const Quant& qp)
{
    if (MODE != kNestedAnyM && MODE != kNestedPow2Shrink) return lattice;
    const float scaled = qp.alpha * lattice;
    return __builtin_fmaf(qp.beta, y, scaled);
}

// Reconstruction Delta * (q - v) of Algorithm 1's server step.
__device__ __forceinline__ float index_value(float q, float step, float v)
{
    const float centred = q - v;
    return step * centred;
}

// Field j of a packed group of codes as a float, plus a constant, in two
// full-rate operations instead of extract + add + convert: the field is masked
// in place into the mantissa of 2^23 (the float 2^23 + c 2^(j b), an integer, so
// exact), then one fma scales it down and removes the 2^23 -- every product and
// sum is exactly representable, so the result is c + constant with no rounding.
// Needs (j + 1) b <= 23.
template <int NF>
struct FieldAsFloat {
    uint32_t mask[NF];
    float scale[NF], offset[NF];
    __device__ __forceinline__ FieldAsFloat(uint32_t bits, float constant)
    {
#pragma unroll
        for (uint32_t j = 0; j < (uint32_t)NF; ++j) {
            mask[j] = ((1u << bits) - 1u) << (j * bits);
            scale[j] = __uint_as_float((127u - j * bits) << 23);
            offset[j] = constant - __uint_as_float((150u - j * bits) << 23);
        }
    }
    __device__ __forceinline__ float get(uint32_t group, int j) const
    {
        const uint32_t x = __builtin_amdgcn_bitop3_b32(group, mask[j], 0x4B000000u, 0xEA);  // (group & mask) | 2^23
        return __builtin_fmaf(__uint_as_float(x), scale[j], offset[j]);
    }
};
constexpr uint32_t kFieldAsFloatMaxBits = 5;   // four fields of a group stay inside 23 bits

// The same with the field masked into the mantissa of 2^(23 - j b - s) instead of
// 2^23: that float is 2^(23-jb-s) + c 2^-s exactly, and subtracting a constant
// (2^(23-jb-s) - constant, an exact float) leaves c 2^-s + constant, again with
// no rounding.  The per-field constants are then an operand of the bit operation
// (scalar register) and a literal of the subtraction: none of them occupies a
// vector register, where FieldAsFloat keeps one offset per field.  Used with a
// compile-time width; s = log2 of a power-of-two divisor (0: none).
template <int NF>
struct FieldScaled {
    uint32_t mask[NF], base[NF];
    float minus[NF];
    __device__ __forceinline__ FieldScaled(uint32_t bits, uint32_t s, float constant = 0.0f)
    {
#pragma unroll
        for (uint32_t j = 0; j < (uint32_t)NF; ++j) {
            mask[j] = ((1u << bits) - 1u) << (j * bits);
            base[j] = (150u - j * bits - s) << 23;
            minus[j] = __uint_as_float(base[j]) - constant;
        }
    }
    // the two halves of get(): the masked field inside its power of two, and its value
    __device__ __forceinline__ float raw(uint32_t group, int j) const
    {
        return __uint_as_float(__builtin_amdgcn_bitop3_b32(group, mask[j], base[j], 0xEA));   // (group & mask) | base
    }
    __device__ __forceinline__ float finish(float x, int j) const { return x - minus[j]; }
    __device__ __forceinline__ float get(uint32_t group, int j) const { return finish(raw(group, j), j); }
};

// Coset decoder of eq. (8), alpha = 1: the integer congruent to m (mod M) nearest
// to y/Delta + v, returned as a float.  m + M*k is formed by one fma: exact while
// below 2^24 and otherwise rounded once, exactly like converting the exact
// integer; eq. (8) puts no bound on k and neither does this.
//
// How coset_index_f divides by M.  kDivExact: the correctly rounded quotient, as
// the decoder is defined.  kDivFast: the product with the rounded reciprocal,
// which differs from that quotient by less than 2^-22 |quotient| and therefore
// rounds to the same integer unless it lies that close to a half-integer; the
// caller is told (`near_tie`) and repeats the few affected rows with kDivExact.
// For a power of two M the two coincide and near_tie is never set.
enum Div { kDivExact = 0, kDivFast = 1 };

template <int MODE, int DIV>
__device__ __forceinline__ float coset_index_f(float m_f, float y, float inv, float v,
                                               const Quant& qp, bool& near_tie)
{
    const float c = __builtin_fmaf(y, inv, v);
    const float diff = c - m_f;
    float k;
    if (MODE == kNestedPow2 || MODE == kNestedPow2Shrink) {
        k = __builtin_rintf(diff * qp.inv_M_f);        // exact scaling
    } else if (DIV == kDivFast) {
        const float approx = diff * qp.inv_M_f;
        k = __builtin_rintf(approx);
        const float off = approx - k;                                  // exact, in [-1/2, 1/2]
        const float tol = __builtin_fmaf(__builtin_fabsf(approx), 0x1p-21f, 0x1p-21f);
        near_tie = near_tie || (__builtin_fabsf(off) + tol >= 0.5f);
    } else {
        k = __builtin_rintf(diff / qp.M_f);
    }
    return __builtin_fmaf(k, qp.M_f, m_f);
}

// ---------------------------------------------------------------------------
// Input element types.  A lane owns 8 consecutive elements per row (one Philox
// block): V 16-byte vectors.
// ---------------------------------------------------------------------------
template <int DT> struct Elem;
template <> struct Elem<0> {               // binary32: two 16-byte vectors
    static constexpr int V = 2;
    using scalar = float;
    struct Row { uint4 v[2]; };
    __device__ static __forceinline__ float get(const Row& row, int k)
    {
        const uint4& raw = row.v[k >> 2];
        const int c = k & 3;
        const uint32_t w = (c == 0) ? raw.x : (c == 1) ? raw.y : (c == 2) ? raw.z : raw.w;
        return __uint_as_float(w);
    }
    __device__ static __forceinline__ float scalar_at(const void* p, size_t i)
    {
        return ((const float*)p)[i];
    }
    // running max of |x|; the carrier is a float
    using maxacc = float;
    __device__ static __forceinline__ float max_init() { return 0.0f; }
    __device__ static __forceinline__ float max4(float m, const uint4& raw)
    {
        m = __builtin_fmaxf(m, __builtin_fmaxf(__builtin_fabsf(__uint_as_float(raw.x)),
                                               __builtin_fabsf(__uint_as_float(raw.y))));
        return __builtin_fmaxf(m, __builtin_fmaxf(__builtin_fabsf(__uint_as_float(raw.z)),
                                                  __builtin_fabsf(__uint_as_float(raw.w))));
    }
    __device__ static __forceinline__ float max_update(float m, const Row& row)
    {
        return max4(max4(m, row.v[0]), row.v[1]);
    }
    __device__ static __forceinline__ float max_final(float m) { return m; }
};
template <> struct Elem<1> {               // bfloat16, widened exactly: one 16-byte vector
    static constexpr int V = 1;
    using scalar = uint16_t;
    struct Row { uint4 v[1]; };
    __device__ static __forceinline__ float get(const Row& row, int k)
    {
        const uint4& raw = row.v[0];
        const int wi = k >> 1;
        const uint32_t w = (wi == 0) ? raw.x : (wi == 1) ? raw.y : (wi == 2) ? raw.z : raw.w;
        return __uint_as_float((k & 1) ? (w & 0xFFFF0000u) : (w << 16));
    }
    __device__ static __forceinline__ float scalar_at(const void* p, size_t i)
    {
        return __uint_as_float((uint32_t)((const uint16_t*)p)[i] << 16);
    }
    // |x| of a bfloat16 orders like its low 15 bits, so the running max is kept
    // as two 16-bit integers per word and widened once at the end
    using maxacc = uint32_t;
    __device__ static __forceinline__ uint32_t max_init() { return 0u; }
    __device__ static __forceinline__ uint32_t pk_max(uint32_t a, uint32_t b)
    {
        typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
        const u16x2 x = __builtin_bit_cast(u16x2, a), y = __builtin_bit_cast(u16x2, b);
        return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(x, y));
    }
    __device__ static __forceinline__ uint32_t max_update(uint32_t m, const Row& row)
    {
        const uint4& raw = row.v[0];
        m = pk_max(m, raw.x & 0x7FFF7FFFu);
        m = pk_max(m, raw.y & 0x7FFF7FFFu);
        m = pk_max(m, raw.z & 0x7FFF7FFFu);
        return pk_max(m, raw.w & 0x7FFF7FFFu);
    }
    __device__ static __forceinline__ float max_final(uint32_t m)
    {
        const uint32_t hi = m >> 16, lo = m & 0xFFFFu;
        return __uint_as_float((hi > lo ? hi : lo) << 16);
    }
};
constexpr int kLaneElems = 8;   // elements per lane and row in the encoders

// Gradients are read once and results written once per call, and every vector is
// larger than the caches, so both go through non-temporal (streaming) accesses:
// the lines do not linger in L2 / Infinity Cache, and a kernel's dirty output is
// not written back underneath the next kernel (measured: the encoder that follows
// a decoder runs 35 % faster, in-place decoders 5 % faster).  -DNDQ_NO_STREAMING
// falls back to plain accesses.
__device__ __forceinline__ void store_streaming(float* p, float a, float b, float c, float d)
{
#ifdef NDQ_NO_STREAMING
    *(float4*)p = make_float4(a, b, c, d);
#else
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    f32x4 v = {a, b, c, d};
    __builtin_nontemporal_store(v, (f32x4*)p);
#endif
}

__device__ __forceinline__ float4 load_streaming_f4(const float* p)
{
#if defined(NDQ_NO_STREAMING) || defined(NDQ_NO_STREAMING_RMW_LOADS)
    return *(const float4*)p;
#else
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    const f32x4 t = __builtin_nontemporal_load((const f32x4*)p);
    return make_float4(t.x, t.y, t.z, t.w);
#endif
}

__device__ __forceinline__ uint4 load_streaming(const void* p)
{
#ifdef NDQ_NO_STREAMING
    return *(const uint4*)p;
#else
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 t = __builtin_nontemporal_load((const u32x4*)p);
    return make_uint4(t.x, t.y, t.z, t.w);
#endif
}

// Loads the 8 elements at element offset `o` (a multiple of 8) of a tile with
// `len` valid elements.  FULL: the whole tile is valid, plain 16-byte loads.
// Otherwise elements past the end read as zero.
template <int DT, bool FULL>
__device__ __forceinline__ typename Elem<DT>::Row load_row(const void* tile, uint32_t o, uint32_t len)
{
    using T = Elem<DT>;
    typename T::Row row;
    const typename T::scalar* base = (const typename T::scalar*)tile + o;
#pragma unroll
    for (int j = 0; j < T::V; ++j) {
        constexpr uint32_t per = kLaneElems / T::V;        // elements per vector
        const uint32_t oj = o + j * per;
        if (FULL || oj + per <= len) {
            row.v[j] = load_streaming(base + j * per);
        } else {
            uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
            for (uint32_t k = 0; k < per; ++k)
                if (oj + k < len) {
                    if (DT == 0) w[k & 3] = ((const uint32_t*)tile)[oj + k];
                    else w[k >> 1] |= (uint32_t)((const uint16_t*)tile)[oj + k] << (16 * (k & 1));
                }
            row.v[j] = make_uint4(w[0], w[1], w[2], w[3]);
        }
    }
    return row;
}

// Maximum of a non-negative float over the 64 lanes of a wave, returned in every
// lane.  Non-negative floats order like their bit patterns, so the reduction
// runs on integers: four data-parallel-primitive steps inside each row of 16
// lanes (no LDS traffic), then the four row results are combined on the scalar
// unit.  Every lane of the wave must be active at the call.
__device__ __forceinline__ float wave_max(float x)
{
    int v = (int)__float_as_uint(x);
    int t;
    t = __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xF, 0xF, false);   // quad_perm [1,0,3,2]
    v = v > t ? v : t;
    t = __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xF, 0xF, false);   // quad_perm [2,3,0,1]
    v = v > t ? v : t;
    t = __builtin_amdgcn_update_dpp(0, v, 0x141, 0xF, 0xF, false);  // row_half_mirror
    v = v > t ? v : t;
    t = __builtin_amdgcn_update_dpp(0, v, 0x140, 0xF, 0xF, false);  // row_mirror
    v = v > t ? v : t;
    const int r0 = __builtin_amdgcn_readlane(v, 0), r1 = __builtin_amdgcn_readlane(v, 16);
    const int r2 = __builtin_amdgcn_readlane(v, 32), r3 = __builtin_amdgcn_readlane(v, 48);
    const int m01 = r0 > r1 ? r0 : r1, m23 = r2 > r3 ? r2 : r3;
    return __uint_as_float((uint32_t)(m01 > m23 ? m01 : m23));
}

// Orders a wave's own LDS traffic: what its lanes wrote before is visible to all
// of its lanes after (a wave's LDS instructions execute in order; the fences keep
// the compiler from moving accesses across).
__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Tile geometry.  A vector is cut into buckets (one step each; bucket == 0: the
// whole vector) and every bucket into tiles of at most `tile` elements, so that
// a tile never straddles two steps.  One wave owns one tile.
struct Tiling {
    uint64_t n;            // elements in the call
    uint64_t bucket_len;   // bucket, or n when bucket == 0
    uint32_t tiles_per_bucket;
    uint32_t total_tiles;
};

struct TileRef {
    uint64_t start;   // first element
    uint32_t len;     // valid elements (0: nothing to do)
    uint32_t bucket;  // index of its step
};

__device__ __forceinline__ TileRef locate_tile(const Tiling& tl, uint32_t tile_id, uint32_t tile)
{
    TileRef t;
    t.start = 0; t.len = 0; t.bucket = 0;
    if (tile_id >= tl.total_tiles) return t;
    const uint32_t b = tile_id / tl.tiles_per_bucket;
    const uint32_t j = tile_id - b * tl.tiles_per_bucket;
    const uint64_t in_bucket = (uint64_t)j * tile;
    const uint64_t start = (uint64_t)b * tl.bucket_len + in_bucket;
    if (in_bucket >= tl.bucket_len || start >= tl.n) return t;
    uint64_t len = tl.bucket_len - in_bucket;
    if (len > tile) len = tile;
    if (len > tl.n - start) len = tl.n - start;
    t.start = start; t.len = (uint32_t)len; t.bucket = b;
    return t;
}

}  // namespace ndq
