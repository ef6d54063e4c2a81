// libndq kernels and C ABI (gfx950).  See include/ndq.h for the contract.
//
// Every kernel is a streaming pass: one wave owns one tile of a few thousand
// consecutive elements, issues all of its 16-byte loads up front, regenerates
// the dither with Philox in registers and writes 16-byte (values) or 8-byte
// (packed codes) coalesced stores.  Nothing here is a contraction, so no MFMA;
// LDS is used only to transpose the small packed codes into stream order.
#include <hip/hip_runtime.h>

#include <math.h>

#include "ndq.h"
#include "ndq_device.hpp"

namespace ndq {

// ---------------------------------------------------------------------------
// Encoder: Algorithm 1 worker block (DQSG) / Algorithm 2 worker block (NDQSG)
// ---------------------------------------------------------------------------
struct EncodeArgs {
    const void* g;
    unsigned char* codes;
    float* steps;          // written (fused / preset) or read (two-pass)
    Tiling tl;
    uint64_t index0;       // dither offset of element 0
    uint64_t total_bytes;  // size of the packed stream incl. zero padding
    DitherStream ds;
    Quant qp;
    float preset_step;     // > 0: bucket == 0 with a caller-set step
};

template <int DT> struct EncRows { static constexpr int R = kEncLoads / Elem<DT>::V; };
template <int DT> struct EncTile { static constexpr uint32_t N = kWave * kLaneElems * EncRows<DT>::R; };

// One wave encodes one tile: loads it (all 16-byte loads issued back to back),
// finds the step, quantizes, and leaves the packed codes in `stage` in stream
// order.  A lane owns 8 consecutive elements per row: one Philox block, and
// 8 codes = `bits` whole bytes of the stream.  FULL: every element of the tile
// is valid -- no guards anywhere.
template <int DT, int MODE, bool FUSED, bool FULL>
__device__ __forceinline__ void encode_tile(const EncodeArgs& a, const TileRef& t, uint32_t tile_id,
                                            unsigned char* stage, int lane)
{
    using T = Elem<DT>;
    constexpr int ROWS = EncRows<DT>::R;
    const uint32_t bits = a.qp.bits;
    const typename T::scalar* tile = (const typename T::scalar*)a.g + t.start;
    typename T::Row raw[ROWS];
#pragma unroll
    for (int r = 0; r < ROWS; ++r)
        raw[r] = load_row<DT, FULL>(tile, (uint32_t)(r * kWave + lane) * kLaneElems, t.len);

    float step;
    if (FUSED) {
        // the bucket is this tile: kappa = max|g| in registers (Sec. 3.1 eq. (2))
        typename T::maxacc m = T::max_init();
#pragma unroll
        for (int r = 0; r < ROWS; ++r) m = T::max_update(m, raw[r]);
        step = step_from_kappa(wave_max(T::max_final(m)), a.qp.levels);
        if (lane == 0) a.steps[t.bucket] = step;
    } else if (a.preset_step > 0.0f) {
        step = a.preset_step;
        if (tile_id == 0 && lane == 0) a.steps[0] = step;
    } else {
        step = a.steps[t.bucket];
    }
    const float inv = a.qp.alpha * inv_step(step);   // alpha = 1 unless a nested worker shrinks
    const uint64_t block0 = (a.index0 + t.start) >> 3;

#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        const uint32_t o = (uint32_t)(r * kWave + lane) * kLaneElems;
        float v[8];
        dither8(a.ds, block0 + (o >> 3), v);
        uint32_t quad[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            uint32_t chunk = 0;
            if (MODE == kDqNarrow) {
                // codes of <= 6 bits: sum (q_k - q_min) 2^(k b) stays an exact float below 2^24
                float acc = a.qp.pack_bias;
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    float q = dq_index_f(T::get(raw[r], 4 * h + k), inv, v[4 * h + k], a.qp);
                    if (!FULL && o + 4 * h + k >= t.len) q = a.qp.q_min_f;
                    acc = __builtin_fmaf(q, __uint_as_float((127u + k * bits) << 23), acc);
                }
                chunk = (uint32_t)acc;
            } else {
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    uint32_t c = encode_one<MODE>(T::get(raw[r], 4 * h + k), inv, v[4 * h + k], a.qp);
                    if (!FULL && o + 4 * h + k >= t.len) c = 0;
                    chunk |= c << (k * bits);
                }
            }
            quad[h] = chunk;
        }
        // eight consecutive codes -> `bits` bytes at byte (o/8)*bits of the tile's stream
        const uint64_t chunk8 = (uint64_t)quad[0] | ((uint64_t)quad[1] << (4 * bits));
        unsigned char* p = stage + (o >> 3) * bits;
        switch (bits) {
            case 1: *p = (unsigned char)chunk8; break;
            case 2: *(uint16_t*)p = (uint16_t)chunk8; break;
            case 4: *(uint32_t*)p = (uint32_t)chunk8; break;
            case 8: *(uint64_t*)p = chunk8; break;
            default:
                for (uint32_t k = 0; k < bits; ++k) p[k] = (unsigned char)(chunk8 >> (8 * k));
        }
    }
    if (lane == 0) *(uint64_t*)(stage + (size_t)EncTile<DT>::N / 8 * bits) = 0;  // pad unit
}

// FUSED: the bucket fits one tile; its max-norm is reduced in registers and
// the step is written.  Otherwise the step is the preset one or read from
// `steps` (filled by absmax_kernel + steps_from_kappa_kernel).
// Occupancy target.  The bfloat16 encoder is bound by instruction issue with a
// burst of loads at the start of every tile; eight waves per SIMD (64 registers)
// hide that burst better than four (+8 % measured).  The binary32 encoder moves
// twice the bytes per element and measured best with the registers it asks for.
template <int DT> struct EncWaves { static constexpr int W = DT == 1 ? 8 : 4; };
template <int DT, int MODE, bool FUSED>
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(EncWaves<DT>::W)))
void encode_kernel(EncodeArgs a)
{
    constexpr uint32_t TILE = EncTile<DT>::N;
    __shared__ __align__(16) unsigned char stage_all[kWavesPerBlock][TILE + 8];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);   // wave-uniform
    unsigned char* stage = stage_all[wave];

    const uint32_t tile_id = blockIdx.x * kWavesPerBlock + wave;
    const TileRef t = locate_tile(a.tl, tile_id, TILE);
    const uint32_t bits = a.qp.bits;
    if (t.len == TILE) encode_tile<DT, MODE, FUSED, true>(a, t, tile_id, stage, lane);
    else if (t.len != 0) encode_tile<DT, MODE, FUSED, false>(a, t, tile_id, stage, lane);
    __syncthreads();
    if (t.len != 0) {
        const uint64_t byte0 = (t.start >> 3) * bits;                 // tile start is a multiple of 64
        const bool last = t.start + t.len == a.tl.n;
        const uint64_t nbytes = last ? a.total_bytes - byte0 : (uint64_t)(t.len >> 3) * bits;
        const uint32_t units = (uint32_t)(nbytes >> 3);
        uint64_t* dst = (uint64_t*)(a.codes + byte0);
        const uint64_t* src = (const uint64_t*)stage;
        for (uint32_t u = lane; u < units; u += kWave) dst[u] = src[u];
    }
}

// ---------------------------------------------------------------------------
// Max-norm per bucket (two-pass path and ndq_absmax)
// ---------------------------------------------------------------------------
__global__ void fill_zero_kernel(uint32_t* p, uint64_t n)
{
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

template <int DT>
__global__ __launch_bounds__(kBlock) void absmax_kernel(const void* g, Tiling tl, uint32_t* kappa_bits)
{
    using T = Elem<DT>;
    constexpr uint32_t TILE = EncTile<DT>::N;
    const int lane = threadIdx.x & (kWave - 1);
    const uint32_t tile_id =
        blockIdx.x * kWavesPerBlock + __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const TileRef t = locate_tile(tl, tile_id, TILE);
    if (t.len == 0) return;
    const typename T::scalar* tile = (const typename T::scalar*)g + t.start;
    constexpr int ROWS = EncRows<DT>::R;
    typename T::Row raw[ROWS];
    if (t.len == TILE) {
#pragma unroll
        for (int r = 0; r < ROWS; ++r)
            raw[r] = load_row<DT, true>(tile, (uint32_t)(r * kWave + lane) * kLaneElems, t.len);
    } else {
#pragma unroll
        for (int r = 0; r < ROWS; ++r)
            raw[r] = load_row<DT, false>(tile, (uint32_t)(r * kWave + lane) * kLaneElems, t.len);
    }
    typename T::maxacc acc = T::max_init();
#pragma unroll
    for (int r = 0; r < ROWS; ++r) acc = T::max_update(acc, raw[r]);
    const float m = wave_max(T::max_final(acc));
    // non-negative floats order like their bit patterns
    if (lane == 0) atomicMax(kappa_bits + t.bucket, __float_as_uint(m));
}

__global__ void steps_from_kappa_kernel(float* steps, uint64_t K, uint32_t levels)
{
    const uint64_t b = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (b < K) steps[b] = step_from_kappa(steps[b], levels);
}

// ---------------------------------------------------------------------------
// Decoder: Algorithm 1 server block (DQSG) / Algorithm 2 server loop (NDQSG)
// ---------------------------------------------------------------------------
struct DecodeArgs {
    const unsigned char* codes;
    const float* steps;
    const float* side;     // nested modes
    float* out;
    Tiling tl;
    uint64_t index0;
    DitherStream ds;
    Quant qp;
    float side_scale;
};

template <int ROWS> struct DecTile { static constexpr uint32_t N = kWave * 4 * ROWS; };  // outputs per wave
template <int MODE, int ACC> struct DecRows {
    static constexpr int R = ((MODE == kDq || MODE == kDqHalf) && ACC == 0) ? kDecRowsStream : kDecRowsUpdate;
};

enum Acc { kStore = 0, kAccumulate = 1, kAccumulateInPlace = 2 };  // in place: out == side

// One wave decodes one tile.  FULL: every element valid, no guards.  STRADDLE:
// the code width does not divide 8, so four codes may cross a 32-bit word.
template <int MODE, int ACC, bool FULL, bool STRADDLE>
__device__ __forceinline__ void decode_tile(const DecodeArgs& a, const TileRef& t, int lane)
{
    const uint32_t bits = a.qp.bits;
    const uint32_t* codes32 = (const uint32_t*)(a.codes + (t.start >> 3) * bits);
    const float* side = a.side + t.start;
    float* out = a.out + t.start;
    const float step = a.steps[t.bucket];
    const float inv = a.qp.alpha * inv_step(step);
    const uint64_t block0 = (a.index0 + t.start) >> 2;

    constexpr int kDecRows = DecRows<MODE, ACC>::R;
    uint32_t packed[kDecRows];
    float4 y[kDecRows], prev[kDecRows];
#pragma unroll
    for (int r = 0; r < kDecRows; ++r) {
        const uint32_t o = (uint32_t)r * kWave * 4 + (uint32_t)lane * 4;
        packed[r] = 0;
        y[r] = make_float4(0.f, 0.f, 0.f, 0.f);
        prev[r] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (FULL || o < t.len) {
            const uint32_t bit = o * bits;
            const uint32_t w = bit >> 5, sh = bit & 31u;
            if (STRADDLE) {
                // read the next word only if a valid code reaches into it (a ragged
                // tail must not touch memory past the stream)
                const uint32_t ncodes = FULL ? 4u : (t.len - o < 4u ? t.len - o : 4u);
                uint64_t window = codes32[w];
                if (sh + ncodes * bits > 32u) window |= (uint64_t)codes32[w + 1] << 32;
                packed[r] = (uint32_t)(window >> sh);
            } else {
                packed[r] = codes32[w] >> sh;
            }
            if (FULL || o + 4 <= t.len) {
                if (MODE == kNestedPow2 || MODE == kNestedAnyM || MODE == kNestedPow2Shrink)
                    y[r] = load_streaming_f4(side + o);
                if (ACC == kAccumulate) prev[r] = load_streaming_f4(out + o);
            } else {
                float ys[4] = {0.f, 0.f, 0.f, 0.f}, ps[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (uint32_t k = 0; k < 4; ++k)
                    if (o + k < t.len) {
                        if (MODE == kNestedPow2 || MODE == kNestedAnyM || MODE == kNestedPow2Shrink)
                            ys[k] = side[o + k];
                        if (ACC == kAccumulate) ps[k] = out[o + k];
                    }
                y[r] = make_float4(ys[0], ys[1], ys[2], ys[3]);
                prev[r] = make_float4(ps[0], ps[1], ps[2], ps[3]);
            }
        }
    }
#pragma unroll
    for (int r = 0; r < kDecRows; ++r) {
        const uint32_t o = (uint32_t)r * kWave * 4 + (uint32_t)lane * 4;
        if (!FULL && o >= t.len) continue;
        float v[4] = {0.f, 0.f, 0.f, 0.f};
        if (MODE != kDqHalf) dither4(a.ds, block0 + (o >> 2), v);
        const float ys[4] = {y[r].x, y[r].y, y[r].z, y[r].w};
        const float ps[4] = {prev[r].x, prev[r].y, prev[r].z, prev[r].w};
        float res[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const uint32_t c = __builtin_amdgcn_ubfe(packed[r], k * bits, bits);   // bit-field extract
            float q, yk = 0.0f;
            if (MODE == kDq || MODE == kDqHalf) {
                q = (float)((int32_t)c + a.qp.q_min);
            } else {
                yk = ys[k] * a.side_scale;
                q = coset_index_f<MODE>(c, yk, inv, v[k], a.qp);
            }
            const float val = (MODE == kDqHalf) ? step * q
                                                : shrink<MODE>(index_value(q, step, v[k]), yk, a.qp);
            if (ACC == kStore) res[k] = val;
            else if (ACC == kAccumulate) res[k] = ps[k] + val;
            else res[k] = ys[k] + val;
        }
        if (FULL || o + 4 <= t.len) {
            store_streaming(out + o, res[0], res[1], res[2], res[3]);
        } else {
#pragma unroll
            for (uint32_t k = 0; k < 4; ++k)
                if (o + k < t.len) out[o + k] = res[k];
        }
    }
}

template <int MODE, int ACC, bool STRADDLE>
__global__ __launch_bounds__(kBlock) void decode_kernel(DecodeArgs a)
{
    const int lane = threadIdx.x & (kWave - 1);
    const uint32_t tile_id =
        blockIdx.x * kWavesPerBlock + __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    constexpr uint32_t TILE = DecTile<DecRows<MODE, ACC>::R>::N;
    const TileRef t = locate_tile(a.tl, tile_id, TILE);
    if (t.len == TILE) decode_tile<MODE, ACC, true, STRADDLE>(a, t, lane);
    else if (t.len != 0) decode_tile<MODE, ACC, false, STRADDLE>(a, t, lane);
}

// ---------------------------------------------------------------------------
// Chain decoder: the whole server loop of Algorithm 2 in one pass.  The running
// sum of a lane's elements lives in registers while the workers are folded in
// one after the other; the next worker's code words and step are prefetched
// while the current worker's dither is generated.
// ---------------------------------------------------------------------------
constexpr uint32_t kChainMax = 32;    // workers per launch
#ifndef NDQ_CHAIN_ROWS
#define NDQ_CHAIN_ROWS 2
#endif
constexpr int kChainRows = NDQ_CHAIN_ROWS;   // rows of 8 elements per lane and tile
constexpr uint32_t kChainTile = kWave * kLaneElems * kChainRows;

struct ChainWorker {
    const unsigned char* codes;
    const float* steps;
    uint64_t index0;
    DitherStream ds;
    int32_t q_min;
    uint32_t M;
    float M_f, inv_M_f;
    float alpha, beta;    // nested: shrinkage factor and 1 - alpha^2
    float side_scale;     // 1/(workers folded in before this one); 0 for the first
    uint32_t bits;
    uint32_t mode;        // Mode
    uint32_t first;       // S <- value instead of S + value
};

struct ChainArgs {
    ChainWorker w[kChainMax];
    float* out;
    Tiling tl;
    uint32_t W;
    int continue_sum;     // S starts from out (an earlier group of workers)
    int apply_scale;
    float scale;
};

// What is prefetched per worker: the step and, per row, the words holding the
// lane's eight codes (8*bits bits starting at a multiple of 8 bits).
struct ChainFetch {
    uint32_t w0[kChainRows], w1[kChainRows], w2[kChainRows];
    float step;
};

template <bool FULL>
__device__ __forceinline__ void chain_fetch(const ChainWorker& cw, const TileRef& t, int lane,
                                            ChainFetch& f)
{
    const uint32_t bits = cw.bits;
    const uint32_t* codes32 = (const uint32_t*)(cw.codes + (t.start >> 3) * bits);
    f.step = cw.steps[t.bucket];
#pragma unroll
    for (int r = 0; r < kChainRows; ++r) {
        const uint32_t o = (uint32_t)(r * kWave + lane) * kLaneElems;
        f.w0[r] = 0; f.w1[r] = 0; f.w2[r] = 0;
        if (FULL || o < t.len) {
            const uint32_t bit = o * bits;                     // multiple of 8
            const uint32_t w = bit >> 5, sh = bit & 31u;
            // bits used from word w on; a ragged tail only counts its valid codes so
            // that no word past the stream is touched
            const uint32_t ncodes = FULL ? 8u : (t.len - o < 8u ? t.len - o : 8u);
            const uint32_t end = sh + ncodes * bits;
            f.w0[r] = codes32[w];
            if (end > 32u) f.w1[r] = codes32[w + 1];
            if (end > 64u) f.w2[r] = codes32[w + 2];
        }
    }
}

template <int MODE>
__device__ __forceinline__ void chain_fold(const ChainWorker& cw, const ChainFetch& f,
                                           uint64_t block0, int lane, float (&S)[kChainRows][8])
{
    const uint32_t bits = cw.bits;
    const float step = f.step;
    const float inv = cw.alpha * inv_step(step);
    Quant qp;
    qp.M = cw.M; qp.M_f = cw.M_f; qp.inv_M_f = cw.inv_M_f; qp.q_min = cw.q_min;
    qp.alpha = cw.alpha; qp.beta = cw.beta;
#pragma unroll
    for (int r = 0; r < kChainRows; ++r) {
        const uint32_t o = (uint32_t)(r * kWave + lane) * kLaneElems;
        const uint32_t sh = (o * bits) & 31u;
        // the lane's 8*bits code bits, in two halves of four codes
        const uint64_t low = (((uint64_t)f.w1[r] << 32) | f.w0[r]) >> sh;
        const uint64_t high = sh ? ((uint64_t)f.w2[r] << (64u - sh)) : 0u;
        const uint64_t chunk = low | high;
        const uint32_t half[2] = {(uint32_t)chunk, (uint32_t)(chunk >> (4u * bits))};
        float v[8];
        dither8(cw.ds, block0 + (o >> 3), v);
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const uint32_t c = __builtin_amdgcn_ubfe(half[k >> 2], (k & 3) * bits, bits);   // bit-field extract
            float q, yk = 0.0f;
            if (MODE == kDq) {
                q = (float)((int32_t)c + qp.q_min);
            } else {
                yk = S[r][k] * cw.side_scale;
                q = coset_index_f<MODE>(c, yk, inv, v[k], qp);
            }
            const float val = shrink<MODE>(index_value(q, step, v[k]), yk, qp);
            S[r][k] = (MODE == kDq && cw.first) ? val : S[r][k] + val;
        }
    }
}

template <bool FULL>
__device__ __forceinline__ void chain_tile(const ChainArgs& a, const TileRef& t, int lane)
{
    float S[kChainRows][8];
    float* out = a.out + t.start;
#pragma unroll
    for (int r = 0; r < kChainRows; ++r) {
        const uint32_t o = (uint32_t)(r * kWave + lane) * kLaneElems;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            S[r][k] = 0.0f;
            if (a.continue_sum && (FULL || o + k < t.len)) S[r][k] = out[o + k];
        }
    }
    ChainFetch cur;
    chain_fetch<FULL>(a.w[0], t, lane, cur);
    ChainFetch nxt = cur;
    for (uint32_t w = 0; w < a.W; ++w) {
        const ChainWorker& cw = a.w[w];
        if (w + 1 < a.W) chain_fetch<FULL>(a.w[w + 1], t, lane, nxt);
        const uint64_t block0 = (cw.index0 + t.start) >> 3;
        if (cw.mode == kDq) chain_fold<kDq>(cw, cur, block0, lane, S);
        else if (cw.mode == kNestedPow2) chain_fold<kNestedPow2>(cw, cur, block0, lane, S);
        else if (cw.mode == kNestedPow2Shrink) chain_fold<kNestedPow2Shrink>(cw, cur, block0, lane, S);
        else chain_fold<kNestedAnyM>(cw, cur, block0, lane, S);
        cur = nxt;
    }
#pragma unroll
    for (int r = 0; r < kChainRows; ++r) {
        const uint32_t o = (uint32_t)(r * kWave + lane) * kLaneElems;
        float res[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) res[k] = a.apply_scale ? a.scale * S[r][k] : S[r][k];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            if (FULL || o + 4 * j + 4 <= t.len) {
                store_streaming(out + o + 4 * j, res[4 * j], res[4 * j + 1], res[4 * j + 2], res[4 * j + 3]);
            } else {
#pragma unroll
                for (uint32_t k = 0; k < 4; ++k)
                    if (o + 4 * j + k < t.len) out[o + 4 * j + k] = res[4 * j + k];
            }
        }
    }
}

#ifndef NDQ_CHAIN_WAVES_PER_EU
#define NDQ_CHAIN_WAVES_PER_EU 6
#endif
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(NDQ_CHAIN_WAVES_PER_EU)))
void chain_kernel(ChainArgs a)
{
    const int lane = threadIdx.x & (kWave - 1);
    const uint32_t tile_id =
        blockIdx.x * kWavesPerBlock + __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const TileRef t = locate_tile(a.tl, tile_id, kChainTile);
    if (t.len == kChainTile) chain_tile<true>(a, t, lane);
    else if (t.len != 0) chain_tile<false>(a, t, lane);
}

// ---------------------------------------------------------------------------
// Aggregation: Algorithm 1 server, "compute the average"
// ---------------------------------------------------------------------------
constexpr uint32_t kAggMax = 32;
struct AggArgs {
    const float* g[kAggMax];
    float* out;
    uint64_t n;
    uint32_t W;
    int continue_sum;   // start from out (partial sum of an earlier group of workers)
    int finish;         // multiply by scale
    float scale;
};

__global__ __launch_bounds__(kBlock) void aggregate_kernel(AggArgs a)
{
    const uint64_t i4 = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    const uint64_t i = i4 * 4;
    if (i >= a.n) return;
    if (i + 4 <= a.n) {
        float4 acc = a.continue_sum ? *(const float4*)(a.out + i) : make_float4(0.f, 0.f, 0.f, 0.f);
        for (uint32_t w0 = 0; w0 < a.W; w0 += 8) {
            float4 x[8];
#pragma unroll
            for (uint32_t j = 0; j < 8; ++j)
                if (w0 + j < a.W) x[j] = load_streaming_f4(a.g[w0 + j] + i);
#pragma unroll
            for (uint32_t j = 0; j < 8; ++j)
                if (w0 + j < a.W) {
                    acc.x = acc.x + x[j].x; acc.y = acc.y + x[j].y;
                    acc.z = acc.z + x[j].z; acc.w = acc.w + x[j].w;
                }
        }
        if (a.finish) { acc.x = a.scale * acc.x; acc.y = a.scale * acc.y; acc.z = a.scale * acc.z; acc.w = a.scale * acc.w; }
        store_streaming(a.out + i, acc.x, acc.y, acc.z, acc.w);
    } else {
        for (uint64_t e = i; e < a.n; ++e) {
            float acc = a.continue_sum ? a.out[e] : 0.0f;
            for (uint32_t w = 0; w < a.W; ++w) acc = acc + a.g[w][e];
            a.out[e] = a.finish ? a.scale * acc : acc;
        }
    }
}

// ---------------------------------------------------------------------------
// Histogram and entropy of an index stream (Sec. 4: the bit rate after entropy
// coding is reported through the entropy of the transmitted indices).
// A thread reads units of 32 codes (= `bits` consecutive 32-bit words) with a
// small bit reader.  Counting: 1-bit and 2-bit streams by population count in
// registers; up to 16 bins in a private LDS column per thread (no conflicts);
// wider codes with LDS atomics on one histogram per workgroup.
// ---------------------------------------------------------------------------
constexpr int kHistBlock = 256;

__global__ __launch_bounds__(kHistBlock) void histogram_kernel(const uint32_t* __restrict__ words,
                                                               uint64_t n, uint32_t bits,
                                                               unsigned long long* hist)
{
    __shared__ uint32_t cols[16][kHistBlock];   // bits <= 4: one column per thread
    __shared__ uint32_t wide[256];              // bits  > 4: shared, atomic
    const uint32_t tid = threadIdx.x;
    const uint32_t nbins = 1u << bits;
    for (uint32_t b = 0; b < 16; ++b) cols[b][tid] = 0u;
    wide[tid] = 0u;
    __syncthreads();

    const uint64_t units = (n + 31u) >> 5;
    const uint32_t mask = nbins - 1u;
    uint32_t c1 = 0u, c2 = 0u, c3 = 0u, seen = 0u;   // registers for the 1- and 2-bit paths
    for (uint64_t u = (uint64_t)blockIdx.x * kHistBlock + tid; u < units;
         u += (uint64_t)gridDim.x * kHistBlock) {
        const uint32_t valid = (u + 1u == units) ? (uint32_t)(n - (u << 5)) : 32u;
        const uint32_t* p = words + u * bits;
        if (bits == 1u) {
            uint32_t w = p[0];
            if (valid < 32u) w &= (1u << valid) - 1u;
            c1 += __builtin_popcount(w);
            seen += valid;
        } else if (bits == 2u) {
#pragma unroll
            for (uint32_t j = 0; j < 2; ++j) {
                const uint32_t have = valid > 16u * j ? (valid - 16u * j < 16u ? valid - 16u * j : 16u) : 0u;
                uint32_t w = have ? p[j] : 0u;
                uint32_t field = have == 16u ? 0x55555555u : ((1u << (2u * have)) - 1u) & 0x55555555u;
                const uint32_t lo = w & field, hi = (w >> 1) & field;
                c1 += __builtin_popcount(lo & ~hi);
                c2 += __builtin_popcount(hi & ~lo);
                c3 += __builtin_popcount(lo & hi);
                seen += have;
            }
        } else {
            uint64_t buf = 0u;
            uint32_t have = 0u, next = 0u;
            for (uint32_t j = 0; j < valid; ++j) {
                if (have < bits) {
                    buf |= (uint64_t)p[next++] << have;
                    have += 32u;
                }
                const uint32_t code = (uint32_t)buf & mask;
                buf >>= bits;
                have -= bits;
                if (bits <= 4u) cols[code][tid] += 1u;      // private column: no race
                else atomicAdd(&wide[code], 1u);
            }
        }
    }
    if (bits == 1u) {
        cols[1][tid] = c1; cols[0][tid] = seen - c1;
    } else if (bits == 2u) {
        cols[1][tid] = c1; cols[2][tid] = c2; cols[3][tid] = c3; cols[0][tid] = seen - c1 - c2 - c3;
    }
    __syncthreads();
    if (bits <= 4u) {
        // 16 threads per bin add up the bin's 256 columns, then one atomic per bin and block
        const uint32_t bin = tid >> 4, part = tid & 15u;
        uint32_t sum = 0u;
        for (uint32_t k = 0; k < kHistBlock / 16; ++k) sum += cols[bin][part * (kHistBlock / 16) + k];
#pragma unroll
        for (int sft = 8; sft >= 1; sft >>= 1) sum += __shfl_xor(sum, sft, 16);
        if (part == 0u && bin < nbins && sum) atomicAdd(hist + bin, (unsigned long long)sum);
    } else if (tid < nbins && wide[tid]) {
        atomicAdd(hist + tid, (unsigned long long)wide[tid]);
    }
}

__global__ void fill_zero64_kernel(unsigned long long* p, uint32_t count)
{
    if (threadIdx.x < count) p[threadIdx.x] = 0ull;
}

// -sum p log2 p over at most 256 bins, binary64, fixed reduction order
__global__ __launch_bounds__(256) void entropy_kernel(const unsigned long long* hist, uint32_t nbins,
                                                      uint64_t n, double* entropy_out)
{
    __shared__ double term[256];
    const uint32_t tid = threadIdx.x;
    double t = 0.0;
    if (tid < nbins && n) {
        const unsigned long long h = hist[tid];
        if (h) {
            const double p = (double)h / (double)n;
            t = -p * log2(p);
        }
    }
    term[tid] = t;
    __syncthreads();
    for (uint32_t s = 128; s >= 1; s >>= 1) {
        if (tid < s) term[tid] += term[tid + s];
        __syncthreads();
    }
    if (tid == 0) entropy_out[0] = term[0];
}

// ---------------------------------------------------------------------------
// Dense base-L stream (Sec. 4 Table 1 counts log2 L bits per index): k indices
// per 32-bit word as the number sum_j c_j L^j.  Transcoders between the
// fixed-width stream and the dense one.  A thread owns 8 dense words = 8k
// indices = k*bits whole bytes of the fixed-width stream, so no two threads
// touch the same byte.
// ---------------------------------------------------------------------------
struct DenseArgs {
    unsigned char* fixed;     // fixed-width stream (read by pack, written by unpack)
    uint32_t* dense;          // dense stream (written by pack, read by unpack)
    uint64_t n;               // indices
    uint64_t fixed_valid;     // ceil(n*bits/8): bytes of the fixed stream that hold indices
    uint64_t fixed_total;     // its padded size
    uint64_t dense_valid;     // ceil(n/k) words that hold indices
    uint64_t dense_total;     // padded size in words
    uint32_t levels, k, bits;
};

__global__ __launch_bounds__(256) void dense_pack_kernel(DenseArgs a)
{
    const uint64_t t = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const uint64_t w0 = t * 8u;
    if (w0 >= a.dense_total) return;
    uint64_t byte = t * a.k * a.bits;
    const uint32_t mask = (1u << a.bits) - 1u;
    uint32_t buf = 0u, have = 0u;
    for (uint32_t j = 0; j < 8u; ++j) {
        const uint64_t w = w0 + j;
        if (w >= a.dense_total) break;
        uint64_t value = 0u, weight = 1u;
        for (uint32_t d = 0; d < a.k; ++d) {
            if (have < a.bits) {
                const uint32_t b = byte < a.fixed_valid ? a.fixed[byte] : 0u;
                ++byte;
                buf |= b << have;
                have += 8u;
            }
            uint32_t c = buf & mask;
            buf >>= a.bits;
            have -= a.bits;
            if (w * a.k + d >= a.n) c = 0u;
            value += c * weight;
            weight *= a.levels;
        }
        a.dense[w] = (uint32_t)value;
    }
}

__global__ __launch_bounds__(256) void dense_unpack_kernel(DenseArgs a)
{
    const uint64_t t = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    uint64_t byte = t * a.k * a.bits;
    if (byte >= a.fixed_total) return;
    const uint64_t w0 = t * 8u;
    uint32_t buf = 0u, have = 0u;
    for (uint32_t j = 0; j < 8u; ++j) {
        const uint64_t w = w0 + j;
        uint32_t value = w < a.dense_valid ? a.dense[w] : 0u;
        for (uint32_t d = 0; d < a.k; ++d) {
            uint32_t c = value % a.levels;
            value /= a.levels;
            if (w * a.k + d >= a.n) c = 0u;
            buf |= c << have;
            have += a.bits;
            if (have >= 8u) {
                if (byte < a.fixed_total) a.fixed[byte] = (unsigned char)buf;
                ++byte;
                buf >>= 8;
                have -= 8u;
            }
        }
    }
}

// ---------------------------------------------------------------------------
// sum_i (a_i - b_i)^2 in binary64 (the sigma_z^2 estimate behind Thm 4's parameter
// choice).  Two passes over a fixed grid so that the reduction order, and hence
// the result, does not depend on scheduling.
// ---------------------------------------------------------------------------
constexpr uint32_t kSqBlocks = 1024;

__device__ __forceinline__ double block_sum_256(double x, double* sh)
{
    const uint32_t tid = threadIdx.x;
    sh[tid] = x;
    __syncthreads();
    for (uint32_t s = 128; s >= 1; s >>= 1) {
        if (tid < s) sh[tid] += sh[tid + s];
        __syncthreads();
    }
    return sh[0];
}

__global__ __launch_bounds__(256) void sqdiff_partial_kernel(const float* __restrict__ a,
                                                             const float* __restrict__ b, uint64_t n,
                                                             double* partial)
{
    __shared__ double sh[256];
    const uint64_t n4 = n >> 2;
    double acc = 0.0;
    for (uint64_t i = (uint64_t)blockIdx.x * 256u + threadIdx.x; i < n4; i += (uint64_t)kSqBlocks * 256u) {
        const float4 x = ((const float4*)a)[i], y = ((const float4*)b)[i];
        const double d0 = (double)x.x - (double)y.x, d1 = (double)x.y - (double)y.y;
        const double d2 = (double)x.z - (double)y.z, d3 = (double)x.w - (double)y.w;
        acc += d0 * d0; acc += d1 * d1; acc += d2 * d2; acc += d3 * d3;
    }
    if (blockIdx.x == 0 && threadIdx.x < (n & 3u)) {       // the last n mod 4 elements
        const uint64_t i = (n4 << 2) + threadIdx.x;
        const double d = (double)a[i] - (double)b[i];
        acc += d * d;
    }
    const double total = block_sum_256(acc, sh);
    if (threadIdx.x == 0) partial[blockIdx.x] = total;
}

__global__ __launch_bounds__(256) void sqdiff_final_kernel(const double* partial, double* out)
{
    __shared__ double sh[256];
    double acc = 0.0;
    for (uint32_t j = 0; j < kSqBlocks / 256u; ++j) acc += partial[j * 256u + threadIdx.x];
    const double total = block_sum_256(acc, sh);
    if (threadIdx.x == 0) out[0] = total;
}

// ---------------------------------------------------------------------------
// Host side: validation and dispatch
// ---------------------------------------------------------------------------
static uint32_t code_bits(uint32_t x)
{
    if (x < 2u || x > 256u) return 0u;
    uint32_t b = 0u;
    while ((1u << b) < x) ++b;
    return b;
}

static size_t packed_bytes(size_t n, uint32_t bits)
{
    const size_t bytes = (n * (size_t)bits + 7u) / 8u;
    return (bytes + 15u) / 16u * 16u;
}

static bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }
static bool aligned4(const void* p) { return ((uintptr_t)p & 3u) == 0; }
constexpr uint64_t kMaxN = (uint64_t)1 << 40;

static int make_tiling(uint64_t n, uint32_t bucket, uint32_t tile, Tiling* tl)
{
    tl->n = n;
    tl->bucket_len = bucket ? bucket : n;
    const uint64_t K = bucket ? (n + bucket - 1) / bucket : 1;
    const uint64_t tpb = (tl->bucket_len + tile - 1) / tile;
    if (tpb * K >= ((uint64_t)1 << 31) || tpb >= ((uint64_t)1 << 31)) return NDQ_EUNSUPPORTED;
    tl->tiles_per_bucket = (uint32_t)tpb;
    tl->total_tiles = (uint32_t)(tpb * K);
    return NDQ_OK;
}

static int make_quant(uint32_t levels, uint32_t M, bool nested, float alpha, Quant* qp)
{
    if (levels < 2u || levels > 256u) return NDQ_EINVAL;
    if (nested && (M < 2u || M > 256u)) return NDQ_EINVAL;
    if (nested && !(alpha > 0.0f && alpha <= 1.0f)) return NDQ_EINVAL;
    qp->alpha = nested ? alpha : 1.0f;
    qp->beta = (float)(1.0 - (double)qp->alpha * (double)qp->alpha);
    qp->levels = levels;
    qp->q_min = -(int32_t)(levels / 2u);
    qp->q_min_f = (float)qp->q_min;
    qp->q_max_f = (float)(qp->q_min + (int32_t)levels - 1);
    qp->M = nested ? M : 1u;
    qp->M_f = (float)qp->M;
    qp->inv_M_f = 1.0f / qp->M_f;   // exact when M is a power of two, unused otherwise
    qp->bits = code_bits(nested ? M : levels);
    float weights = 0.0f;
    for (uint32_t k = 0; k < 4; ++k) weights += (float)(1u << (k * qp->bits < 31u ? k * qp->bits : 31u));
    qp->pack_bias = -qp->q_min_f * weights;   // exact for bits <= 6, the only user
    return NDQ_OK;
}

static bool is_pow2(uint32_t x) { return (x & (x - 1u)) == 0u; }

static DitherStream make_stream(const ndq_dither* d)
{
    DitherStream s;
    s.key0 = (uint32_t)d->seed;
    s.key1 = (uint32_t)(d->seed >> 32);
    s.step = d->step;
    s.worker = d->worker;
    return s;
}

static int launched() { return hipGetLastError() == hipSuccess ? NDQ_OK : NDQ_ELAUNCH; }

static uint32_t blocks_for(uint32_t tiles) { return (tiles + kWavesPerBlock - 1) / kWavesPerBlock; }

template <int DT>
static int run_absmax(const void* g, const Tiling& tl, uint64_t K, float* kappa, hipStream_t s)
{
    hipLaunchKernelGGL(fill_zero_kernel, dim3((uint32_t)((K + 255) / 256)), dim3(256), 0, s,
                       (uint32_t*)kappa, K);
    if (launched() != NDQ_OK) return NDQ_ELAUNCH;
    hipLaunchKernelGGL(absmax_kernel<DT>, dim3(blocks_for(tl.total_tiles)), dim3(kBlock), 0, s, g, tl,
                       (uint32_t*)kappa);
    return launched();
}

template <int DT, int MODE>
static int run_encode(const EncodeArgs& a, bool fused, hipStream_t s)
{
    const dim3 grid(blocks_for(a.tl.total_tiles)), block(kBlock);
    if (fused) hipLaunchKernelGGL((encode_kernel<DT, MODE, true>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((encode_kernel<DT, MODE, false>), grid, block, 0, s, a);
    return launched();
}

static int encode_common(const void* g, ndq_dtype dt, size_t n, float delta, uint32_t levels,
                         uint32_t M, bool nested, float alpha, uint32_t bucket, const ndq_dither* d,
                         void* codes_out, float* steps_out, void* stream)
{
    EncodeArgs a;
    int rc = make_quant(levels, M, nested, alpha, &a.qp);
    if (rc != NDQ_OK) return rc;
    if (dt != NDQ_F32 && dt != NDQ_BF16) return NDQ_EINVAL;
    if (!d) return NDQ_EINVAL;
    if (n == 0) return NDQ_OK;
    if (!g || !codes_out || !steps_out) return NDQ_EINVAL;
    if (!(delta == delta)) return NDQ_EINVAL;
    if (n >= kMaxN) return NDQ_EUNSUPPORTED;
    if (!aligned16(g) || !aligned16(codes_out) || !aligned4(steps_out)) return NDQ_EALIGN;
    if (bucket % 64u != 0u || (d->offset & 7u) != 0u) return NDQ_EALIGN;

    const uint32_t tile = dt == NDQ_F32 ? EncTile<0>::N : EncTile<1>::N;
    rc = make_tiling(n, bucket, tile, &a.tl);
    if (rc != NDQ_OK) return rc;
    a.g = g;
    a.codes = (unsigned char*)codes_out;
    a.steps = steps_out;
    a.index0 = d->offset;
    a.total_bytes = packed_bytes(n, a.qp.bits);
    a.ds = make_stream(d);
    a.preset_step = (bucket == 0u && delta > 0.0f) ? delta : 0.0f;
    hipStream_t s = (hipStream_t)stream;

    const bool fused = bucket != 0u && bucket <= tile;
    if (!fused && a.preset_step == 0.0f) {
        // two passes: max-norm per bucket, then steps, then the encoder reads them
        const uint64_t K = bucket ? (n + bucket - 1) / bucket : 1;
        rc = dt == NDQ_F32 ? run_absmax<0>(g, a.tl, K, steps_out, s)
                           : run_absmax<1>(g, a.tl, K, steps_out, s);
        if (rc != NDQ_OK) return rc;
        hipLaunchKernelGGL(steps_from_kappa_kernel, dim3((uint32_t)((K + 255) / 256)), dim3(256), 0,
                           s, steps_out, K, levels);
        if (launched() != NDQ_OK) return NDQ_ELAUNCH;
    }
#ifndef NDQ_NARROW_MAX_BITS
#define NDQ_NARROW_MAX_BITS 6u
#endif
    const int mode = !nested ? (a.qp.bits <= NDQ_NARROW_MAX_BITS ? kDqNarrow : kDq)
                             : (is_pow2(M) ? kNestedPow2 : kNestedAnyM);
    if (dt == NDQ_F32) {
        if (mode == kDqNarrow) return run_encode<0, kDqNarrow>(a, fused, s);
        if (mode == kDq) return run_encode<0, kDq>(a, fused, s);
        if (mode == kNestedPow2) return run_encode<0, kNestedPow2>(a, fused, s);
        return run_encode<0, kNestedAnyM>(a, fused, s);
    }
    if (mode == kDqNarrow) return run_encode<1, kDqNarrow>(a, fused, s);
    if (mode == kDq) return run_encode<1, kDq>(a, fused, s);
    if (mode == kNestedPow2) return run_encode<1, kNestedPow2>(a, fused, s);
    return run_encode<1, kNestedAnyM>(a, fused, s);
}

template <int MODE, int ACC, bool STRADDLE>
static int run_decode3(DecodeArgs a, uint64_t n, uint32_t bucket, hipStream_t s)
{
    const int rc = make_tiling(n, bucket, DecTile<DecRows<MODE, ACC>::R>::N, &a.tl);
    if (rc != NDQ_OK) return rc;
    hipLaunchKernelGGL((decode_kernel<MODE, ACC, STRADDLE>), dim3(blocks_for(a.tl.total_tiles)),
                       dim3(kBlock), 0, s, a);
    return launched();
}

template <int MODE, bool STRADDLE>
static int run_decode2(const DecodeArgs& a, uint64_t n, uint32_t bucket, int acc, hipStream_t s)
{
    if (acc == kStore) return run_decode3<MODE, kStore, STRADDLE>(a, n, bucket, s);
    if (acc == kAccumulate) return run_decode3<MODE, kAccumulate, STRADDLE>(a, n, bucket, s);
    return run_decode3<MODE, kAccumulateInPlace, STRADDLE>(a, n, bucket, s);
}

template <int MODE>
static int run_decode(const DecodeArgs& a, uint64_t n, uint32_t bucket, int acc, hipStream_t s)
{
    // four b-bit codes sit inside one 32-bit word exactly when 4b divides 32
    const bool straddle = (32u % (4u * a.qp.bits)) != 0u;
    return straddle ? run_decode2<MODE, true>(a, n, bucket, acc, s)
                    : run_decode2<MODE, false>(a, n, bucket, acc, s);
}

static int decode_common(const void* codes, size_t n, uint32_t levels, uint32_t M, bool nested,
                         bool half, float alpha, uint32_t bucket, const float* steps,
                         const ndq_dither* d,
                         const float* side, float side_scale, float* out, int accumulate,
                         void* stream)
{
    DecodeArgs a;
    int rc = make_quant(levels, M, nested, alpha, &a.qp);
    if (rc != NDQ_OK) return rc;
    if (!d) return NDQ_EINVAL;
    if (n == 0) return NDQ_OK;
    if (!codes || !steps || !out || (nested && !side)) return NDQ_EINVAL;
    if (n >= kMaxN) return NDQ_EUNSUPPORTED;
    if (!aligned16(codes) || !aligned16(out) || !aligned4(steps) || (nested && !aligned16(side)))
        return NDQ_EALIGN;
    if (bucket % 64u != 0u || (d->offset & 7u) != 0u) return NDQ_EALIGN;
    if (nested && side != out) {
        // partial overlap of side and out would race between waves
        const uintptr_t s0 = (uintptr_t)side, o0 = (uintptr_t)out, len = (uintptr_t)n * 4u;
        if (s0 < o0 + len && o0 < s0 + len) return NDQ_EINVAL;
    }
    a.codes = (const unsigned char*)codes;
    a.steps = steps;
    a.side = nested ? side : out;
    a.out = out;
    a.index0 = d->offset;
    a.ds = make_stream(d);
    a.side_scale = side_scale;
    hipStream_t s = (hipStream_t)stream;
    int acc = accumulate ? kAccumulate : kStore;
    if (nested && accumulate && side == out) acc = kAccumulateInPlace;
    if (!nested) return half ? run_decode<kDqHalf>(a, n, bucket, acc, s)
                             : run_decode<kDq>(a, n, bucket, acc, s);
    if (is_pow2(M) && alpha == 1.0f) return run_decode<kNestedPow2>(a, n, bucket, acc, s);
    if (is_pow2(M)) return run_decode<kNestedPow2Shrink>(a, n, bucket, acc, s);
    return run_decode<kNestedAnyM>(a, n, bucket, acc, s);
}

}  // namespace ndq

// ---------------------------------------------------------------------------
// C ABI
// ---------------------------------------------------------------------------
extern "C" {

uint32_t ndq_code_bits(uint32_t levels_or_M) { return ndq::code_bits(levels_or_M); }

size_t ndq_packed_bytes(size_t n, uint32_t bits) { return ndq::packed_bytes(n, bits); }

size_t ndq_num_buckets(size_t n, uint32_t bucket)
{
    return bucket ? (n + bucket - 1u) / bucket : 1u;
}

int ndq_absmax(const void* g, ndq_dtype dt, size_t n, uint32_t bucket, float* kappa_out,
               void* stream)
{
    using namespace ndq;
    if (dt != NDQ_F32 && dt != NDQ_BF16) return NDQ_EINVAL;
    if (!kappa_out) return NDQ_EINVAL;
    if (n >= kMaxN) return NDQ_EUNSUPPORTED;
    if (!aligned4(kappa_out) || bucket % 64u != 0u) return NDQ_EALIGN;
    hipStream_t s = (hipStream_t)stream;
    if (n == 0) {   // one (empty) bucket: its max-norm is 0
        if (bucket != 0u) return NDQ_OK;
        hipLaunchKernelGGL(fill_zero_kernel, dim3(1), dim3(256), 0, s, (uint32_t*)kappa_out, (uint64_t)1);
        return launched();
    }
    if (!g) return NDQ_EINVAL;
    if (!aligned16(g)) return NDQ_EALIGN;
    Tiling tl;
    const uint32_t tile = dt == NDQ_F32 ? EncTile<0>::N : EncTile<1>::N;
    int rc = make_tiling(n, bucket, tile, &tl);
    if (rc != NDQ_OK) return rc;
    const uint64_t K = bucket ? (n + bucket - 1) / bucket : 1;
    return dt == NDQ_F32 ? run_absmax<0>(g, tl, K, kappa_out, s) : run_absmax<1>(g, tl, K, kappa_out, s);
}

int ndq_dq_encode(const void* g, ndq_dtype dt, size_t n, float delta, uint32_t levels,
                  uint32_t bucket, const ndq_dither* d, void* codes_out, float* steps_out,
                  void* stream)
{
    return ndq::encode_common(g, dt, n, delta, levels, 0u, false, 1.0f, bucket, d, codes_out,
                              steps_out, stream);
}

int ndq_nested_encode(const void* g, ndq_dtype dt, size_t n, float delta, uint32_t levels,
                      uint32_t M, float alpha, uint32_t bucket, const ndq_dither* d,
                      void* codes_out, float* steps_out, void* stream)
{
    return ndq::encode_common(g, dt, n, delta, levels, M, true, alpha, bucket, d, codes_out,
                              steps_out, stream);
}

int ndq_dq_decode(const void* codes, size_t n, uint32_t levels, uint32_t bucket,
                  const float* steps, const ndq_dither* d, float* out, int accumulate,
                  void* stream)
{
    return ndq::decode_common(codes, n, levels, 0u, false, false, 1.0f, bucket, steps, d, nullptr,
                              1.0f, out, accumulate, stream);
}

int ndq_dq_decode_half(const void* codes, size_t n, uint32_t levels, uint32_t bucket,
                       const float* steps, float* out, int accumulate, void* stream)
{
    const ndq_dither none = {0u, 0u, 0u, 0u};   // no dither is regenerated
    return ndq::decode_common(codes, n, levels, 0u, false, true, 1.0f, bucket, steps, &none,
                              nullptr, 1.0f, out, accumulate, stream);
}

int ndq_nested_decode(const void* codes, size_t n, uint32_t M, float alpha, uint32_t bucket,
                      const float* steps, const ndq_dither* d, const float* side,
                      float side_scale, float* out, int accumulate, void* stream)
{
    // `levels` plays no part in decoding: the step travels in `steps`
    return ndq::decode_common(codes, n, 2u, M, true, false, alpha, bucket, steps, d, side,
                              side_scale, out, accumulate, stream);
}

int ndq_aggregate(const float* const* gs, uint32_t W, size_t n, float scale, float* out,
                  void* stream)
{
    using namespace ndq;
    if (!gs || W < 1u || W > 1024u) return NDQ_EINVAL;
    if (n == 0) return NDQ_OK;
    if (!out) return NDQ_EINVAL;
    if (n >= kMaxN) return NDQ_EUNSUPPORTED;
    if (!aligned16(out)) return NDQ_EALIGN;
    for (uint32_t w = 0; w < W; ++w) {
        if (!gs[w]) return NDQ_EINVAL;
        if (!aligned16(gs[w])) return NDQ_EALIGN;
        if (W > kAggMax && gs[w] == out) return NDQ_EINVAL;
    }
    const uint64_t threads = (n + 3) / 4;
    const uint64_t blocks = (threads + kBlock - 1) / kBlock;
    if (blocks >= ((uint64_t)1 << 31)) return NDQ_EUNSUPPORTED;
    for (uint32_t w0 = 0; w0 < W; w0 += kAggMax) {
        AggArgs a;
        a.W = (W - w0 < kAggMax) ? W - w0 : kAggMax;
        for (uint32_t j = 0; j < kAggMax; ++j) a.g[j] = j < a.W ? gs[w0 + j] : nullptr;
        a.out = out;
        a.n = n;
        a.continue_sum = w0 != 0u;
        a.finish = w0 + kAggMax >= W;
        a.scale = scale;
        hipLaunchKernelGGL(aggregate_kernel, dim3((uint32_t)blocks), dim3(kBlock), 0,
                           (hipStream_t)stream, a);
        if (launched() != NDQ_OK) return NDQ_ELAUNCH;
    }
    return NDQ_OK;
}

int ndq_decode_chain(const ndq_worker* workers, uint32_t W, size_t n, uint32_t bucket,
                     float scale, float* out, void* stream)
{
    using namespace ndq;
    if (!workers || W < 1u || W > 1024u) return NDQ_EINVAL;
    if (workers[0].kind != NDQ_WORKER_DQ) return NDQ_EINVAL;   // nothing to decode against yet
    for (uint32_t p = 0; p < W; ++p) {
        const ndq_worker& wk = workers[p];
        if (wk.kind != NDQ_WORKER_DQ && wk.kind != NDQ_WORKER_NESTED) return NDQ_EINVAL;
        if (wk.levels_or_M < 2u || wk.levels_or_M > 256u) return NDQ_EINVAL;
        if (wk.kind == NDQ_WORKER_NESTED && !(wk.alpha > 0.0f && wk.alpha <= 1.0f)) return NDQ_EINVAL;
    }
    if (n == 0) return NDQ_OK;
    if (!out) return NDQ_EINVAL;
    if (n >= kMaxN) return NDQ_EUNSUPPORTED;
    if (!aligned16(out) || bucket % 64u != 0u) return NDQ_EALIGN;
    for (uint32_t p = 0; p < W; ++p) {
        const ndq_worker& wk = workers[p];
        if (!wk.codes || !wk.steps) return NDQ_EINVAL;
        if (!aligned16(wk.codes) || !aligned4(wk.steps) || (wk.dither.offset & 7u) != 0u)
            return NDQ_EALIGN;
    }
    ChainArgs a;
    int rc = make_tiling(n, bucket, kChainTile, &a.tl);
    if (rc != NDQ_OK) return rc;
    a.out = out;
    a.scale = scale;
    for (uint32_t p0 = 0; p0 < W; p0 += kChainMax) {
        a.W = (W - p0 < kChainMax) ? W - p0 : kChainMax;
        a.continue_sum = p0 != 0u;
        a.apply_scale = (p0 + kChainMax >= W) && scale != 1.0f;
        for (uint32_t j = 0; j < a.W; ++j) {
            const ndq_worker& wk = workers[p0 + j];
            const bool nested = wk.kind == NDQ_WORKER_NESTED;
            Quant qp;
            make_quant(nested ? 2u : wk.levels_or_M, wk.levels_or_M, nested, wk.alpha, &qp);
            ChainWorker& cw = a.w[j];
            cw.codes = (const unsigned char*)wk.codes;
            cw.steps = wk.steps;
            cw.index0 = wk.dither.offset;
            cw.ds = make_stream(&wk.dither);
            cw.q_min = qp.q_min;
            cw.M = qp.M;
            cw.M_f = qp.M_f;
            cw.inv_M_f = qp.inv_M_f;
            cw.alpha = qp.alpha;
            cw.beta = qp.beta;
            cw.side_scale = (p0 + j) ? 1.0f / (float)(p0 + j) : 0.0f;
            cw.bits = qp.bits;
            cw.mode = !nested ? kDq
                              : (!is_pow2(wk.levels_or_M) ? kNestedAnyM
                                 : (wk.alpha == 1.0f ? kNestedPow2 : kNestedPow2Shrink));
            cw.first = (p0 + j) == 0u;
        }
        hipLaunchKernelGGL(chain_kernel, dim3(blocks_for(a.tl.total_tiles)), dim3(kBlock), 0,
                           (hipStream_t)stream, a);
        if (launched() != NDQ_OK) return NDQ_ELAUNCH;
    }
    return NDQ_OK;
}

int ndq_code_entropy(const void* codes, size_t n, uint32_t bits, uint64_t* hist_out,
                     double* entropy_out, void* stream)
{
    using namespace ndq;
    if (bits < 1u || bits > 8u || !hist_out) return NDQ_EINVAL;
    if (n >= kMaxN) return NDQ_EUNSUPPORTED;
    if (((uintptr_t)hist_out & 7u) != 0u || ((uintptr_t)entropy_out & 7u) != 0u) return NDQ_EALIGN;
    if (n != 0 && !codes) return NDQ_EINVAL;
    if (n != 0 && !aligned16(codes)) return NDQ_EALIGN;
    hipStream_t s = (hipStream_t)stream;
    const uint32_t nbins = 1u << bits;
    hipLaunchKernelGGL(fill_zero64_kernel, dim3(1), dim3(256), 0, s, (unsigned long long*)hist_out, nbins);
    if (launched() != NDQ_OK) return NDQ_ELAUNCH;
    if (n != 0) {
        const uint64_t units = (n + 31u) >> 5;
        uint64_t blocks = (units + kHistBlock - 1) / kHistBlock;
        if (blocks > 4096u) blocks = 4096u;
        hipLaunchKernelGGL(histogram_kernel, dim3((uint32_t)blocks), dim3(kHistBlock), 0, s,
                           (const uint32_t*)codes, (uint64_t)n, bits, (unsigned long long*)hist_out);
        if (launched() != NDQ_OK) return NDQ_ELAUNCH;
    }
    if (entropy_out) {
        hipLaunchKernelGGL(entropy_kernel, dim3(1), dim3(256), 0, s,
                           (const unsigned long long*)hist_out, nbins, (uint64_t)n, entropy_out);
        if (launched() != NDQ_OK) return NDQ_ELAUNCH;
    }
    return NDQ_OK;
}

uint32_t ndq_dense_group(uint32_t levels)
{
    if (levels < 2u || levels > 256u) return 0u;
    uint32_t k = 0u;
    uint64_t power = 1u;
    while (power * levels <= ((uint64_t)1 << 32)) { power *= levels; ++k; }
    return k;
}

size_t ndq_dense_bytes(size_t n, uint32_t levels)
{
    const uint32_t k = ndq_dense_group(levels);
    if (!k) return 0u;
    const size_t words = (n + k - 1u) / k;
    return (words * 4u + 15u) / 16u * 16u;
}

static int dense_common(const void* fixed, const void* dense, size_t n, uint32_t levels, bool pack,
                        void* stream)
{
    using namespace ndq;
    DenseArgs a;
    a.k = ndq_dense_group(levels);
    if (!a.k) return NDQ_EINVAL;
    if (n == 0) return NDQ_OK;
    if (!fixed || !dense) return NDQ_EINVAL;
    if (n >= kMaxN) return NDQ_EUNSUPPORTED;
    if (!aligned16(fixed) || !aligned16(dense)) return NDQ_EALIGN;
    a.fixed = (unsigned char*)fixed;
    a.dense = (uint32_t*)dense;
    a.n = n;
    a.levels = levels;
    a.bits = code_bits(levels);
    a.fixed_valid = ((uint64_t)n * a.bits + 7u) / 8u;
    a.fixed_total = packed_bytes(n, a.bits);
    a.dense_valid = ((uint64_t)n + a.k - 1u) / a.k;
    a.dense_total = ndq_dense_bytes(n, levels) / 4u;
    const uint64_t per_thread_bytes = (uint64_t)a.k * a.bits;
    const uint64_t threads = pack ? (a.dense_total + 7u) / 8u
                                  : (a.fixed_total + per_thread_bytes - 1u) / per_thread_bytes;
    const uint64_t blocks = (threads + 255u) / 256u;
    if (blocks >= ((uint64_t)1 << 31)) return NDQ_EUNSUPPORTED;
    if (pack) hipLaunchKernelGGL(dense_pack_kernel, dim3((uint32_t)blocks), dim3(256), 0, (hipStream_t)stream, a);
    else hipLaunchKernelGGL(dense_unpack_kernel, dim3((uint32_t)blocks), dim3(256), 0, (hipStream_t)stream, a);
    return launched();
}

int ndq_dense_pack(const void* codes, size_t n, uint32_t levels, void* dense_out, void* stream)
{
    return dense_common(codes, dense_out, n, levels, true, stream);
}

int ndq_dense_unpack(const void* dense, size_t n, uint32_t levels, void* codes_out, void* stream)
{
    return dense_common(codes_out, dense, n, levels, false, stream);
}

double ndq_alpha_for_equal_variance(double delta1, double sigma_z2)
{
    const double arg = 1.0 - delta1 * delta1 / (12.0 * sigma_z2);
    return arg > 0.0 ? sqrt(arg) : 0.0;
}

double ndq_decode_error_bound(double delta1, uint32_t M, double alpha, double sigma_z2)
{
    const double delta2 = (double)M * delta1;
    return delta1 * delta1 / (3.0 * delta2 * delta2) + 4.0 * alpha * alpha * sigma_z2 / (delta2 * delta2);
}

size_t ndq_sqdiff_workspace(void) { return ndq::kSqBlocks * sizeof(double); }

int ndq_sqdiff(const float* a, const float* b, size_t n, double* workspace, double* out,
               void* stream)
{
    using namespace ndq;
    if (!workspace || !out) return NDQ_EINVAL;
    if (n != 0 && (!a || !b)) return NDQ_EINVAL;
    if (n >= kMaxN) return NDQ_EUNSUPPORTED;
    if (((uintptr_t)workspace & 7u) || ((uintptr_t)out & 7u)) return NDQ_EALIGN;
    if (n != 0 && (!aligned16(a) || !aligned16(b))) return NDQ_EALIGN;
    hipStream_t s = (hipStream_t)stream;
    hipLaunchKernelGGL(sqdiff_partial_kernel, dim3(kSqBlocks), dim3(256), 0, s, a, b, (uint64_t)n,
                       workspace);
    if (launched() != NDQ_OK) return NDQ_ELAUNCH;
    hipLaunchKernelGGL(sqdiff_final_kernel, dim3(1), dim3(256), 0, s, (const double*)workspace, out);
    return launched();
}

const char* ndq_strerror(int rc)
{
    switch (rc) {
        case NDQ_OK: return "success";
        case NDQ_EINVAL: return "invalid argument (null pointer, levels or M outside [2,256], overlapping buffers, bad W)";
        case NDQ_EALIGN: return "alignment violated (16-byte data pointers, bucket multiple of 64, offset multiple of 8)";
        case NDQ_EUNSUPPORTED: return "vector too long for one call";
        case NDQ_ELAUNCH: return "the HIP runtime refused a kernel launch";
        default: return "unknown ndq status";
    }
}

}  // extern "C"
