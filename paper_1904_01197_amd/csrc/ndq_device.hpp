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
constexpr int kWavesPerBlock = 4;   // 256-thread workgroups, waves work independently
constexpr int kBlock = kWave * kWavesPerBlock;
#ifndef NDQ_ENC_ROWS
#define NDQ_ENC_ROWS 8
#endif
#ifndef NDQ_DEC_ROWS
#define NDQ_DEC_ROWS 8
#endif
constexpr int kEncRows = NDQ_ENC_ROWS;   // 16-byte loads in flight per lane and encoder tile
constexpr int kDecRows = NDQ_DEC_ROWS;   // 16-byte stores per lane and decoder tile

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

__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t (&out)[4])
{
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// Mid-point of cell k = word>>8 of 2^24 equal cells of [-1/2, 1/2): exact in binary32.
__device__ __forceinline__ float unit_dither(uint32_t word)
{
    return __builtin_fmaf((float)(word >> 8), 0x1p-24f, -0.5f + 0x1p-25f);
}

// The four unit dithers of elements 4*block .. 4*block+3 of a stream.
__device__ __forceinline__ void dither4(const DitherStream& s, uint64_t block, float (&v)[4])
{
    uint32_t r[4];
    philox4x32_10((uint32_t)block, (uint32_t)(block >> 32), s.step, s.worker, s.key0, s.key1, r);
#pragma unroll
    for (int k = 0; k < 4; ++k) v[k] = unit_dither(r[k]);
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
//   kNestedPow2   : NDQSG, M a power of two (mask / exact scale) (Algorithm 2)
//   kNestedAnyM   : NDQSG, any M in [2,256]
// ---------------------------------------------------------------------------
enum Mode { kDq = 0, kNestedPow2 = 1, kNestedAnyM = 2 };

struct Quant {
    float q_min_f, q_max_f;  // DQSG index range as floats
    int32_t q_min;           // -(levels/2)
    uint32_t levels;         // fixes the step: Delta = 2 kappa/(levels-1)
    uint32_t M;              // nesting ratio Delta_2/Delta_1 (nested modes)
    float M_f, inv_M_f;      // (float)M and, for powers of two, its exact reciprocal
    uint32_t bits;           // code width
};

// Index of eq. (2) / Algorithm 1, as a code in [0, levels).
__device__ __forceinline__ uint32_t dq_code(float g, float inv, float v, const Quant& qp)
{
    float r = __builtin_rintf(__builtin_fmaf(g, inv, v));
    r = __builtin_fminf(__builtin_fmaxf(r, qp.q_min_f), qp.q_max_f);
    return (uint32_t)((int32_t)r - qp.q_min);
}

// Fine index of eq. (7) reduced modulo M.
template <int MODE>
__device__ __forceinline__ uint32_t nested_code(float g, float inv, float v, const Quant& qp)
{
    float r = __builtin_rintf(__builtin_fmaf(g, inv, v));
    r = __builtin_fminf(__builtin_fmaxf(r, -16777216.0f), 16777216.0f);
    const int32_t q = (int32_t)r;
    if (MODE == kNestedPow2) return (uint32_t)q & (qp.M - 1u);
    int32_t m = q % (int32_t)qp.M;
    if (m < 0) m += (int32_t)qp.M;
    return (uint32_t)m;
}

template <int MODE>
__device__ __forceinline__ uint32_t encode_one(float g, float inv, float v, const Quant& qp)
{
    if (MODE == kDq) return dq_code(g, inv, v, qp);
    return nested_code<MODE>(g, inv, v, qp);
}

// Reconstruction Delta * (q - v) of Algorithm 1's server step.
__device__ __forceinline__ float index_value(int32_t q, float step, float v)
{
    const float centred = (float)q - v;
    return step * centred;
}

// Coset decoder of eq. (8), alpha = 1: integer congruent to m nearest to y/Delta + v.
template <int MODE>
__device__ __forceinline__ int32_t coset_index(uint32_t m, float y, float inv, float v,
                                               const Quant& qp)
{
    const float c = __builtin_fmaf(y, inv, v);
    const float diff = c - (float)m;
    float k = (MODE == kNestedPow2) ? diff * qp.inv_M_f : diff / qp.M_f;
    k = __builtin_rintf(k);
    k = __builtin_fminf(__builtin_fmaxf(k, -4194304.0f), 4194304.0f);
    return (int32_t)m + (int32_t)qp.M * (int32_t)k;
}

// ---------------------------------------------------------------------------
// Input element types: 16-byte loads hold E elements.
// ---------------------------------------------------------------------------
template <int DT> struct Elem;
template <> struct Elem<0> {               // binary32
    static constexpr int E = 4;
    using scalar = float;
    __device__ static __forceinline__ float get(const uint4& raw, int k)
    {
        const uint32_t w = (k == 0) ? raw.x : (k == 1) ? raw.y : (k == 2) ? raw.z : raw.w;
        return __uint_as_float(w);
    }
    __device__ static __forceinline__ uint32_t bits_of(const void* p, size_t i)
    {
        return ((const uint32_t*)p)[i];
    }
};
template <> struct Elem<1> {               // bfloat16, widened exactly
    static constexpr int E = 8;
    using scalar = uint16_t;
    __device__ static __forceinline__ float get(const uint4& raw, int k)
    {
        const int wi = k >> 1;
        const uint32_t w = (wi == 0) ? raw.x : (wi == 1) ? raw.y : (wi == 2) ? raw.z : raw.w;
        return __uint_as_float((k & 1) ? (w & 0xFFFF0000u) : (w << 16));
    }
    __device__ static __forceinline__ uint32_t bits_of(const void* p, size_t i)
    {
        return ((const uint16_t*)p)[i];
    }
};

// Loads E elements at element offset `o` of a tile with `len` valid elements.
// FULL: the whole tile is valid, a plain 16-byte load (o % E == 0).  Otherwise
// elements past the end read as zero.
template <int DT, bool FULL>
__device__ __forceinline__ uint4 load_row(const void* tile, uint32_t o, uint32_t len)
{
    using T = Elem<DT>;
    if (FULL) return *(const uint4*)((const typename T::scalar*)tile + o);
    uint4 raw = make_uint4(0u, 0u, 0u, 0u);
    if (o + T::E <= len) {
        raw = *(const uint4*)((const typename T::scalar*)tile + o);
    } else if (o < len) {
        uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
        for (uint32_t k = 0; k < (uint32_t)T::E; ++k)
            if (o + k < len) {
                const uint32_t b = T::bits_of(tile, o + k);
                if (DT == 0) w[k & 3] = b; else w[k >> 1] |= b << (16 * (k & 1));
            }
        raw = make_uint4(w[0], w[1], w[2], w[3]);
    }
    return raw;
}

__device__ __forceinline__ float wave_max(float x)
{
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) x = __builtin_fmaxf(x, __shfl_xor(x, s, kWave));
    return x;
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
