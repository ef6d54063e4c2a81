// libndq, server side (gfx950): DQSG / NDQSG decoders, the fused server loop of
// Algorithm 2, aggregation.  See include/ndq.h for the contract.
#include <hip/hip_runtime.h>

#include "ndq.h"
#include "ndq_device.hpp"
#include "ndq_host.hpp"

namespace ndq {

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

// Four elements of a row: res = decoded value (stored, or added to ps / ys).
// Returns whether a fast quotient was too close to a rounding tie (see Div).
template <int MODE, int ACC, int DIV>
__device__ __forceinline__ bool decode_row(const DecodeArgs& a, uint32_t packed, uint32_t bits,
                                           const float (&ys)[4], const float (&ps)[4], const float (&v)[4],
                                           float step, float inv, float (&res)[4])
{
    bool near_tie = false;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const uint32_t c = __builtin_amdgcn_ubfe(packed, k * bits, bits);   // bit-field extract
        float q, yk = 0.0f;
        if (MODE == kDq || MODE == kDqHalf) {
            q = (float)((int32_t)c + a.qp.q_min);
        } else {
            yk = ys[k] * a.side_scale;
            q = coset_index_f<MODE, DIV>((float)c, yk, inv, v[k], a.qp, near_tie);
        }
        const float val = (MODE == kDqHalf) ? step * q
                                            : shrink<MODE>(index_value(q, step, v[k]), yk, a.qp);
        if (ACC == kStore) res[k] = val;
        else if (ACC == kAccumulate) res[k] = ps[k] + val;
        else res[k] = ys[k] + val;
    }
    return near_tie;
}

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
        const bool near_tie = decode_row<MODE, ACC, kDivFast>(a, packed[r], bits, ys, ps, v, step, inv, res);
        // wave-uniform and rare (M not a power of two only): redo the row with the division
        if (MODE == kNestedAnyM && __builtin_amdgcn_ballot_w64(near_tie) != 0)
            decode_row<MODE, ACC, kDivExact>(a, packed[r], bits, ys, ps, v, step, inv, res);
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
    uint32_t row_buckets; // 1: a bucket is one row of a tile (tiling is by tile, a step per row)
    uint32_t num_buckets; // with row_buckets: steps per worker (rows past them decode with step 0)
    uint32_t tile_begin;  // chain_kernel: first tile of this launch; chain_stream_kernel: tiles it owns
};

// What is prefetched per worker: the step and, per row, the words holding the
// lane's eight codes (8*bits bits starting at a multiple of 8 bits).
struct ChainFetch {
    uint32_t w0[kChainRows], w1[kChainRows], w2[kChainRows];
    float step[kChainRows];
};

// Code widths 1, 2 and 4: a lane's eight codes are exactly 1, 2 or 4 bytes at a
// multiple of their size, so in a full tile one narrow load fetches them with
// nothing to shift or join afterwards.
__device__ __forceinline__ bool chain_aligned(uint32_t bits) { return bits == 1u || bits == 2u || bits == 4u; }

// ROWB: a bucket is one row of the tile (the tiling is by tile and every row has
// its own step); otherwise one step serves the tile.
template <bool FULL, bool ROWB>
__device__ __forceinline__ void chain_fetch(const ChainArgs& a, const ChainWorker& cw, const TileRef& t,
                                            int lane, ChainFetch& f)
{
    const uint32_t bits = cw.bits;
    const uint32_t* codes32 = (const uint32_t*)(cw.codes + (t.start >> 3) * bits);
    if (ROWB) {
#pragma unroll
        for (int r = 0; r < kChainRows; ++r) {
            const uint32_t b = t.bucket * kChainRows + r;          // rows past the last bucket get 0
            f.step[r] = b < a.num_buckets ? cw.steps[b] : 0.0f;
        }
    } else {
        f.step[0] = cw.steps[t.bucket];
    }
    if (FULL && chain_aligned(bits)) {
        const unsigned char* mine = (const unsigned char*)codes32 + (uint32_t)lane * bits;
#pragma unroll
        for (int r = 0; r < kChainRows; ++r) {
            const unsigned char* p = mine + (uint32_t)(r * kWave) * bits;
            f.w0[r] = bits == 1u ? (uint32_t)*p : bits == 2u ? (uint32_t)*(const uint16_t*)p : *(const uint32_t*)p;
            f.w1[r] = 0; f.w2[r] = 0;
        }
        return;
    }
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

// One row of eight elements of one worker: next = S + (this worker's decoded
// values), the side information being S scaled.  Returns whether any element's
// fast quotient was too close to a rounding tie to be trusted (see Div).
template <int MODE, bool FIRST, int DIV>
__device__ __forceinline__ bool chain_row(const ChainWorker& cw, const Quant& qp, const float (&c_f)[8],
                                          const float (&v)[8], float step, float inv,
                                          const float (&S)[8], float (&next)[8])
{
    bool near_tie = false;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        float q, yk = 0.0f;
        if (MODE == kDq) {
            q = c_f[k];
        } else {
            yk = S[k] * cw.side_scale;
            q = coset_index_f<MODE, DIV>(c_f[k], yk, inv, v[k], qp, near_tie);
        }
        const float val = shrink<MODE>(index_value(q, step, v[k]), yk, qp);
        next[k] = FIRST ? val : S[k] + val;
    }
    return near_tie;
}

// Folds one worker into the running sum S of a tile.  WIDTH: 1, 2, 4 = that many
// code bits, fetched by chain_fetch's aligned path (full tiles only); -1 = any
// width up to kFieldAsFloatMaxBits; 0 = any width.  All but 0 turn the codes into
// floats with FieldAsFloat.  FIRST: the running sum starts with this worker.
template <int MODE, int WIDTH, bool FIRST, bool ROWB>
__device__ __forceinline__ void chain_fold(const ChainWorker& cw, const ChainFetch& f,
                                           uint64_t block0, int lane, float (&S)[kChainRows][8])
{
    constexpr bool ALIGNED = WIDTH > 0;
    constexpr int NF = (WIDTH == 1 || WIDTH == 2) ? 8 : 4;     // fields taken from one 32-bit group
    const uint32_t bits = ALIGNED ? (uint32_t)WIDTH : cw.bits;
    const FieldAsFloat<NF> field(WIDTH != 0 ? bits : 1u, MODE == kDq ? (float)cw.q_min : 0.0f);
    float inv_row[kChainRows];
#pragma unroll
    for (int r = 0; r < kChainRows; ++r)
        inv_row[r] = (ROWB || r == 0) ? cw.alpha * inv_step(f.step[ROWB ? r : 0]) : inv_row[0];
    Quant qp;
    qp.M = cw.M; qp.M_f = cw.M_f; qp.inv_M_f = cw.inv_M_f; qp.q_min = cw.q_min;
    qp.alpha = cw.alpha; qp.beta = cw.beta;
#pragma unroll
    for (int r = 0; r < kChainRows; ++r) {
        const uint32_t o = (uint32_t)(r * kWave + lane) * kLaneElems;
        const float step = f.step[ROWB ? r : 0], inv = inv_row[r];
        uint32_t half[2];
        if (ALIGNED) {
            half[0] = f.w0[r];
            half[1] = NF == 8 ? f.w0[r] : f.w0[r] >> (4u * bits);
        } else {
            const uint32_t sh = (o * bits) & 31u;
            // the lane's 8*bits code bits, in two halves of four codes
            const uint64_t low = (((uint64_t)f.w1[r] << 32) | f.w0[r]) >> sh;
            const uint64_t high = sh ? ((uint64_t)f.w2[r] << (64u - sh)) : 0u;
            const uint64_t chunk = low | high;
            half[0] = (uint32_t)chunk;
            half[1] = (uint32_t)(chunk >> (4u * bits));
        }
        float v[8];
        dither8(cw.ds, block0 + (o >> 3), v);
        if (MODE == kNestedAnyM) {
            // the eight residues as floats, a fast pass, and -- wave-uniform and rare -- the
            // row again with the true division where a quotient sat too close to a tie
            float c_f[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                if (WIDTH != 0) c_f[k] = NF == 8 ? field.get(half[0], k) : field.get(half[k >> 2], k & 3);
                else c_f[k] = (float)__builtin_amdgcn_ubfe(half[k >> 2], (k & 3) * bits, bits);
            }
            float next[8];
            const bool near_tie = chain_row<MODE, FIRST, kDivFast>(cw, qp, c_f, v, step, inv, S[r], next);
            if (__builtin_amdgcn_ballot_w64(near_tie) != 0)
                chain_row<MODE, FIRST, kDivExact>(cw, qp, c_f, v, step, inv, S[r], next);
#pragma unroll
            for (int k = 0; k < 8; ++k) S[r][k] = next[k];
        } else {
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                // the code as a float: plus q_min for DQSG, as it is for a nested worker
                float c_f;
                if (WIDTH != 0) {
                    c_f = NF == 8 ? field.get(half[0], k) : field.get(half[k >> 2], k & 3);
                } else {
                    const uint32_t c = __builtin_amdgcn_ubfe(half[k >> 2], (k & 3) * bits, bits);
                    c_f = MODE == kDq ? (float)((int32_t)c + qp.q_min) : (float)c;
                }
                float q, yk = 0.0f;
                bool unused = false;
                if (MODE == kDq) {
                    q = c_f;
                } else {
                    yk = S[r][k] * cw.side_scale;
                    q = coset_index_f<MODE, kDivExact>(c_f, yk, inv, v[k], qp, unused);
                }
                const float val = shrink<MODE>(index_value(q, step, v[k]), yk, qp);
                S[r][k] = FIRST ? val : S[r][k] + val;
            }
        }
    }
}

// Picks the instantiation for a worker's code width.
template <int MODE, bool FULL, bool FIRST, bool ROWB>
__device__ __forceinline__ void chain_fold_width(const ChainWorker& cw, const ChainFetch& f,
                                                 uint64_t block0, int lane, float (&S)[kChainRows][8])
{
    const uint32_t bits = cw.bits;
    if (FULL && bits == 1u) chain_fold<MODE, 1, FIRST, ROWB>(cw, f, block0, lane, S);
    else if (FULL && bits == 2u) chain_fold<MODE, 2, FIRST, ROWB>(cw, f, block0, lane, S);
    else if (FULL && bits == 4u) chain_fold<MODE, 4, FIRST, ROWB>(cw, f, block0, lane, S);
    else if (bits <= kFieldAsFloatMaxBits) chain_fold<MODE, -1, FIRST, ROWB>(cw, f, block0, lane, S);
    else chain_fold<MODE, 0, FIRST, ROWB>(cw, f, block0, lane, S);
}

template <bool FULL, bool ROWB, bool ANYM>
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
    chain_fetch<FULL, ROWB>(a, a.w[0], t, lane, cur);
    ChainFetch nxt = cur;
    for (uint32_t w = 0; w < a.W; ++w) {
        const ChainWorker& cw = a.w[w];
        if (w + 1 < a.W) chain_fetch<FULL, ROWB>(a, a.w[w + 1], t, lane, nxt);
        const uint64_t block0 = (cw.index0 + t.start) >> 3;
        if (cw.mode == kDq) {
            if (cw.first) chain_fold_width<kDq, FULL, true, ROWB>(cw, cur, block0, lane, S);
            else chain_fold_width<kDq, FULL, false, ROWB>(cw, cur, block0, lane, S);
        } else if (cw.mode == kNestedPow2) {
            chain_fold_width<kNestedPow2, FULL, false, ROWB>(cw, cur, block0, lane, S);
        } else if (cw.mode == kNestedPow2Shrink) {
            chain_fold_width<kNestedPow2Shrink, FULL, false, ROWB>(cw, cur, block0, lane, S);
        } else if (ANYM) {
            chain_fold_width<kNestedAnyM, FULL, false, ROWB>(cw, cur, block0, lane, S);
        }
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
// ANYM: some worker's nesting ratio is not a power of two.  Those workers take
// the two-pass rows of chain_fold, which need more registers: that instantiation
// runs four waves per SIMD, and the common one does not carry their code at all.
template <bool ROWB, bool ANYM>
__global__ __launch_bounds__(kBlock)
__attribute__((amdgpu_waves_per_eu(ANYM ? 4 : NDQ_CHAIN_WAVES_PER_EU)))
void chain_kernel(ChainArgs a)
{
    const int lane = threadIdx.x & (kWave - 1);
    const uint32_t tile_id =
        a.tile_begin + blockIdx.x * kWavesPerBlock + __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const TileRef t = locate_tile(a.tl, tile_id, kChainTile);
    if (t.len == kChainTile) chain_tile<true, ROWB, ANYM>(a, t, lane);
    else if (t.len != 0) chain_tile<false, ROWB, ANYM>(a, t, lane);
}

// ---------------------------------------------------------------------------
// Streaming chain decoder for the common plans: a first DQSG worker, then
// workers that are all alike -- all DQSG, or all nested with a power-of-two
// nesting ratio and no shrinkage -- with code widths of 1, 2 or 4 bits, and a
// vector cut into whole tiles.  One instantiation of the fold serves every
// worker after the first, so the sixteen running sums of a lane stay in the same
// registers from the first worker to the store (the general kernel dispatches on
// mode and width after every worker and moves them around each time).  Waves are
// persistent: a wave walks over tiles wave, wave + W, ... and fetches the next
// worker's, and at the end the next tile's, code words while it folds the
// current worker in.
//
// Arithmetic per element of a nested worker, bit for bit that of chain_row with
// kNestedPow2 (every scaling below is by a power of two, which commutes with
// rounding; k and m/M + k are exact or rounded exactly like m + M k):
//   m' = m / M (from the packed field, exact)      y = S * side_scale
//   c  = fma(y, 1/Delta, v)                        k = rint(fma(c, 1/M, -m'))
//   q' = k + m'                                    S = S + Delta * fma(q', M, -v)
// ---------------------------------------------------------------------------
#ifndef NDQ_CHAIN_STREAM_WAVES
#define NDQ_CHAIN_STREAM_WAVES 6
#endif
constexpr int kChainStreamWaves = NDQ_CHAIN_STREAM_WAVES;

// per-worker parameters as the kernel reads them: through the constant address
// space, indexed by the loop variable (scalar loads, no copy of the arguments)
typedef const __attribute__((address_space(4))) ChainArgs* ChainArgsPtr;

struct ChainCodes { uint32_t w[kChainRows]; float step; };

// a lane's eight codes of a row: `WIDTH` bytes at a multiple of WIDTH (full tiles).
// `limit`: the largest byte offset inside the tile's codes that may be read (a multiple of
// WIDTH); lanes past it read there instead.  Whole tiles pass 0xFFFFFFFF; for the vector's
// ragged last tile it is the stream's last WIDTH bytes, so that the tile can be fetched and
// folded like a whole one (what lanes past the end compute is never stored).
template <int WIDTH>
__device__ __forceinline__ void stream_fetch(const unsigned char* codes, uint64_t start, int lane, ChainCodes& f,
                                             uint32_t limit = 0xFFFFFFFFu)
{
    const unsigned char* tile = codes + (start >> 3) * WIDTH;
#pragma unroll
    for (int r = 0; r < kChainRows; ++r) {
        uint32_t off = (uint32_t)(r * kWave + lane) * WIDTH;
        off = off < limit ? off : limit;
        const unsigned char* p = tile + off;
        f.w[r] = WIDTH == 1 ? (uint32_t)*p : WIDTH == 2 ? (uint32_t)*(const uint16_t*)p : *(const uint32_t*)p;
    }
    f.step = 0.0f;     // whole tiles take their steps from the step lanes of the kernel
}

// The same for the vector's ragged last tile of `len` elements: a lane fetches its bytes
// only if its first code exists (they then lie inside the stream, whose size is padded to
// a multiple of 16 bytes: (o/8 + 1) * WIDTH <= the padded size of the tile's codes).
template <int WIDTH>
__device__ __forceinline__ void stream_fetch_ragged(const unsigned char* codes, const float* steps, uint64_t start,
                                                    uint32_t len, uint32_t bucket, int lane, ChainCodes& f)
{
    const unsigned char* mine = codes + (start >> 3) * WIDTH + (uint32_t)lane * WIDTH;
#pragma unroll
    for (int r = 0; r < kChainRows; ++r) {
        const unsigned char* p = mine + (uint32_t)(r * kWave) * WIDTH;
        f.w[r] = 0u;
        if ((uint32_t)(r * kWave + lane) * kLaneElems < len)
            f.w[r] = WIDTH == 1 ? (uint32_t)*p : WIDTH == 2 ? (uint32_t)*(const uint16_t*)p : *(const uint32_t*)p;
    }
    f.step = steps[bucket];
}

template <int MODE, int WIDTH, bool FIRST>
__device__ __forceinline__ void stream_fold(const DitherStream& ds, uint64_t block0, float q_min_f,
                                            float side_scale, const ChainCodes& f, float step, float inv,
                                            int lane, float (&S)[kChainRows][8])
{
    constexpr int NF = WIDTH == 4 ? 4 : 8;
    // a power-of-two nesting ratio is 2^(code width): M and 1/M are compile-time constants
    constexpr float M_f = (float)(1u << WIDTH), inv_M_f = 1.0f / M_f;
    // DQSG: the code c itself, the index offset q_min going into the dither instead:
    // (c + q_min) - v and c - (v - q_min) are the same exact value rounded once, and
    // v - q_min is exact for |q_min| <= 8 (code widths up to 4 bits).  Nested: m' = c / M.
    const FieldScaled<NF> field((uint32_t)WIDTH, MODE == kDq ? 0u : (uint32_t)WIDTH);
#pragma unroll
    for (int r = 0; r < kChainRows; ++r) {
        const uint32_t o = (uint32_t)(r * kWave + lane) * kLaneElems;
        float v[8];
        if (MODE == kDq) dither8_shifted(ds, block0 + (o >> 3), -q_min_f, v);
        else dither8(ds, block0 + (o >> 3), v);
        const uint32_t lo = f.w[r], hi = WIDTH == 4 ? f.w[r] >> 16 : f.w[r];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const float c_f = NF == 8 ? field.get(lo, k) : field.get(k < 4 ? lo : hi, k & 3);
            float val;
            if (MODE == kDq) {
                val = index_value(c_f, step, v[k]);
            } else {
                const float y = S[r][k] * side_scale;
                const float c = __builtin_fmaf(y, inv, v[k]);
                const float kk = __builtin_rintf(__builtin_fmaf(c, inv_M_f, -c_f));
                const float qs = kk + c_f;
                const float centred = __builtin_fmaf(qs, M_f, -v[k]);
                val = step * centred;
            }
            S[r][k] = FIRST ? val : S[r][k] + val;
        }
    }
}

// The same fold of one row with its instructions in a fixed order, and one Philox
// block (the dither of a later row) advanced by its ten rounds in between.  On
// gfx950 a binary32 add / multiply / fma issued right after a quarter-rate
// instruction (the 32x32 multiply, the round-to-integer) costs next to nothing,
// and alternating integer and float instructions issue faster than runs of
// either (measured with fixed instruction patterns); the compiler's own order
// has the Philox rounds in one run and the float arithmetic in another.  The
// values are those of stream_fold: the same operations on the same operands,
// only their order in the program differs.  Per element the float stages are
// 0: v = unit dither of the cell (DQSG: minus q_min)   1: code field -> c (DQSG) or m' = m/M (nested)
// DQSG    2: c - v   3: Delta * (...)   4: S + (...)
// nested  2: y = S * (1/count)   3: c = fma(y, 1/Delta, v)   4: fma(c, 1/M, -m')
//         [round to integer]     5: + m'   6: fma(q', M, -v)   7: Delta * (...)   8: S + (...)
template <int MODE, int WIDTH, bool FIRST>
__device__ __forceinline__ void fold_row_piped(const uint32_t (&words)[4], uint32_t code, float step, float inv,
                                               float side_scale, float q_min_f, float (&S)[8], PhiloxFlight& fl)
{
    constexpr int NF = WIDTH == 4 ? 4 : 8;
    constexpr float M_f = (float)(1u << WIDTH), inv_M_f = 1.0f / M_f;
    const FieldScaled<NF> field((uint32_t)WIDTH, MODE == kDq ? 0u : (uint32_t)WIDTH);
    // DQSG: the index offset q_min goes into the dither (see stream_fold)
    const float centre = (MODE == kDq ? -q_min_f : 0.0f) + (-0.5f + 0x1p-17f);
    const uint32_t lo = code, hi = WIDTH == 4 ? code >> 16 : code;
    float v[8], m[8], w[8];
    // float stages of an element, in order; nested: the round-to-integer sits between stages 4 and 5
    constexpr int kStages = MODE == kDq ? (FIRST ? 4 : 5) : 9;
    auto stage = [&](int st, int k) __attribute__((always_inline)) {
        const int j = NF == 8 ? k : (k & 3);
        if (st == 0) { v[k] = __builtin_fmaf(v[k], 0x1p-16f, centre); return; }   // unit_dither (shifted)
        if (st == 1) { m[k] = field.finish(m[k], j); return; }
        if (MODE == kDq) {
            if (st == 2) w[k] = m[k] - v[k];
            if (st == 3) { w[k] = step * w[k]; if (FIRST) S[k] = w[k]; }
            if (st == 4) S[k] = S[k] + w[k];
        } else {
            if (st == 2) w[k] = S[k] * side_scale;
            if (st == 3) w[k] = __builtin_fmaf(w[k], inv, v[k]);
            if (st == 4) w[k] = __builtin_fmaf(w[k], inv_M_f, -m[k]);
            if (st == 5) w[k] = w[k] + m[k];
            if (st == 6) w[k] = __builtin_fmaf(w[k], M_f, -v[k]);
            if (st == 7) w[k] = step * w[k];
            if (st == 8) S[k] = S[k] + w[k];
        }
    };
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const uint32_t word = words[k >> 1];
        v[k] = (float)((k & 1) ? word >> 16 : word & 0xFFFFu);
        m[k] = field.raw(NF == 8 ? lo : (k < 4 ? lo : hi), NF == 8 ? k : (k & 3));
        NDQ_PIN();
    }
    constexpr int kInRounds = (MODE == kDq ? kStages : 5) * 8;
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        const int s0 = 4 * round;
        fl.mul0();
        if (s0 + 0 < kInRounds) stage((s0 + 0) >> 3, (s0 + 0) & 7);
        NDQ_PIN();
        fl.mul1();
        if (s0 + 1 < kInRounds) stage((s0 + 1) >> 3, (s0 + 1) & 7);
        NDQ_PIN();
        fl.mix0();
        if (s0 + 2 < kInRounds) stage((s0 + 2) >> 3, (s0 + 2) & 7);
        NDQ_PIN();
        fl.mix1();
        fl.next_round();
        if (s0 + 3 < kInRounds) stage((s0 + 3) >> 3, (s0 + 3) & 7);
        NDQ_PIN();
    }
    if (MODE != kDq) {
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            w[k] = __builtin_rintf(w[k]);
            if (k > 0) stage(5, k - 1);
            NDQ_PIN();
        }
        stage(5, 7);
#pragma unroll
        for (int st = 6; st < kStages; ++st)
#pragma unroll
            for (int k = 0; k < 8; ++k) stage(st, k);
    }
}

template <int MODE, int WIDTH, bool FIRST>
__device__ __forceinline__ void stream_fold_piped(const DitherStream& ds, uint64_t block0, const DitherStream& ds_next,
                                                  uint64_t block_next, float q_min_f, float side_scale,
                                                  const ChainCodes& f, float step, float inv,
                                                  float (&S)[kChainRows][8], PhiloxFlight& fl)
{
#pragma unroll
    for (int r = 0; r < kChainRows; ++r) {
        uint32_t words[4];
        fl.words(words);
        if (r + 1 < kChainRows) fl.start(ds, block0 + (uint32_t)((r + 1) * kWave));
        else fl.start(ds_next, block_next);
        fold_row_piped<MODE, WIDTH, FIRST>(words, f.w[r], step, inv, side_scale, q_min_f, S[r], fl);
    }
}

// The ragged last tile with the same folds: lanes past the end decode zeros and store nothing.
template <int RMODE, int W0, int WR>
__device__ __forceinline__ void stream_ragged_tile(ChainArgsPtr a, uint64_t start, uint32_t len, uint32_t bucket,
                                                   int lane)
{
    const uint32_t W = a->W;
    float S[kChainRows][8];
    ChainCodes cur, nxt;
    stream_fetch_ragged<W0>(a->w[0].codes, a->w[0].steps, start, len, bucket, lane, cur);
    nxt = cur;
    if (W > 1u) stream_fetch_ragged<WR>(a->w[1].codes, a->w[1].steps, start, len, bucket, lane, nxt);
    {
        const DitherStream ds = {a->w[0].ds.key0, a->w[0].ds.key1, a->w[0].ds.step, a->w[0].ds.worker};
        stream_fold<kDq, W0, true>(ds, (a->w[0].index0 + start) >> 3, (float)a->w[0].q_min, 0.0f, cur, cur.step,
                                   inv_step(cur.step), lane, S);
    }
    cur = nxt;
    for (uint32_t w = 1; w < W; ++w) {
        if (w + 1u < W) stream_fetch_ragged<WR>(a->w[w + 1u].codes, a->w[w + 1u].steps, start, len, bucket, lane, nxt);
        const DitherStream ds = {a->w[w].ds.key0, a->w[w].ds.key1, a->w[w].ds.step, a->w[w].ds.worker};
        stream_fold<RMODE, WR, false>(ds, (a->w[w].index0 + start) >> 3, (float)a->w[w].q_min, a->w[w].side_scale,
                                      cur, cur.step, inv_step(cur.step), lane, S);
        cur = nxt;
    }
    float* out = a->out + start;
    const float scale = a->scale;
    const bool apply_scale = a->apply_scale != 0;
#pragma unroll
    for (int r = 0; r < kChainRows; ++r) {
        const uint32_t o = (uint32_t)(r * kWave + lane) * kLaneElems;
#pragma unroll
        for (uint32_t k = 0; k < 8; ++k)
            if (o + k < len) out[o + k] = apply_scale ? scale * S[r][k] : S[r][k];
    }
}

// RAGGED: the vector ends in a ragged tile.  An instantiation of its own, because the mere
// presence of that code in the kernel measured 6 % on the main loop (config 5, which has
// no ragged tile: 215 against 203 us) although the loop's instructions are the same.
// Without PIPED one wave folds that tile with guarded code of its own (stream_ragged_tile).
// With PIPED it is one more tile of the loop: its codes are fetched with the lane offsets
// clamped to the end of the stream, it is folded like a whole tile, and only its copy-out is
// guarded (a persistent ragged launch in the plain form is 7-9 % slower than one tile per
// wave at two to three tiles per wave slot, where the piped form is 1-5 % faster).
//
// PIPED (persistent launches of whole tiles): two changes that only pay together.
// (1) A lane's eight consecutive results are 32 bytes of the output, so a 16-byte store per
// lane writes every other 16 bytes of a 2 KB span, and such half-written sectors sustain only
// 2.6 TB/s: with the arithmetic taken out the stores alone took as long as the whole kernel
// (206 us at n = 2^27; 105 us when every store writes 1 KB of consecutive bytes).  The tile
// therefore leaves through the wave's 4 KB of LDS as four stores of consecutive bytes.
// (2) stream_fold_piped: the fold's instructions in a fixed order with the next row's Philox
// block advanced in between (7 % fewer issue cycles; hidden behind the stores until (1)).
// It starts one extra Philox block per wave, which only a wave with many tiles amortises,
// and the LDS round trip costs a one-tile wave more than the stores do, so launches of one
// tile per wave keep the plain form.
#ifndef NDQ_CHAIN_PIPED_WAVES
#define NDQ_CHAIN_PIPED_WAVES NDQ_CHAIN_STREAM_WAVES
#endif
template <int RMODE, int W0, int WR, bool RAGGED, bool PIPED>
__global__ __launch_bounds__(kBlock)
__attribute__((amdgpu_waves_per_eu(PIPED ? NDQ_CHAIN_PIPED_WAVES : kChainStreamWaves, PIPED ? NDQ_CHAIN_PIPED_WAVES : kChainStreamWaves)))
void chain_stream_kernel(ChainArgs a_by_value)
{
    constexpr bool TAIL = RAGGED && PIPED;     // the ragged tile runs through the main loop
    const ChainArgsPtr a = (ChainArgsPtr)__builtin_amdgcn_kernarg_segment_ptr();
    const int lane = threadIdx.x & (kWave - 1);
    const uint32_t stride = gridDim.x * kWavesPerBlock;
    const uint32_t wave_in_block = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const uint32_t first = blockIdx.x * kWavesPerBlock + wave_in_block;
    __shared__ __align__(16) float out_stage_all[PIPED ? kWavesPerBlock : 1][PIPED ? kChainTile : 4];
    float* out_stage = out_stage_all[PIPED ? wave_in_block : 0u];
    const uint32_t tiles = a->tile_begin;                  // whole tiles: ids 0 .. tiles-1
    const uint32_t tiles_all = TAIL ? tiles + 1u : tiles;  // TAIL: and the ragged one, id `tiles`
    const uint32_t W = a->W;
    const uint32_t tpb = a->tl.tiles_per_bucket;
    const bool one_bucket = a->tl.bucket_len == a->tl.n;   // bucket == 0
    float* out_base = a->out;
    const float scale = a->scale;
    const bool apply_scale = __builtin_amdgcn_readfirstlane(a->apply_scale) != 0;
    // The ragged last tile goes first, to a wave that has no whole tile if the grid has one
    // (one tile per wave), else to wave 0: at the start every SIMD is full and hides its
    // latencies; as a kernel of its own, or at the end, it would run alone at a fifth of the rate.
    const uint64_t whole = (uint64_t)tiles * kChainTile;
    if (RAGGED && !PIPED && whole < a->tl.n && first == (stride > tiles ? tiles : 0u))
        stream_ragged_tile<RMODE, W0, WR>(a, whole, (uint32_t)(a->tl.n - whole), one_bucket ? 0u : tiles / tpb, lane);
    if (first >= tiles_all) return;
    const uint32_t my_tiles = (tiles_all - first + stride - 1u) / stride;
    // TAIL: elements of the ragged tile, and per code width the last byte offset inside its
    // codes that a lane may read: the stream is padded to a multiple of 16 bytes, the tile
    // starts at one, so at least 16 bytes of it exist
    const uint32_t tail_len = TAIL ? (uint32_t)(a->tl.n - whole) : 0u;
    auto tail_limit = [&](uint32_t width) __attribute__((always_inline)) {
        const uint64_t total = ((((uint64_t)a->tl.n * width + 7u) >> 3) + 15u) & ~(uint64_t)15u;
        return (uint32_t)(total - (whole >> 3) * width) - width;
    };
    const uint32_t limit0 = TAIL ? tail_limit((uint32_t)W0) : 0xFFFFFFFFu;
    const uint32_t limitr = TAIL ? tail_limit((uint32_t)WR) : 0xFFFFFFFFu;
    auto limit_for = [&](uint32_t tile_id, uint32_t tail) __attribute__((always_inline)) {
        return (TAIL && tile_id == tiles) ? tail : 0xFFFFFFFFu;
    };
    uint32_t done = 0;
    if (my_tiles > 1u) __builtin_amdgcn_s_setprio(3);

    ChainCodes cur;
    stream_fetch<W0>(a->w[0].codes, (uint64_t)first * kChainTile, lane, cur, limit_for(first, limit0));
    // PIPED: the dither of the row after the current one is always in flight; here the first row's
    PhiloxFlight fl;
    if (PIPED) {
        const DitherStream ds = {a->w[0].ds.key0, a->w[0].ds.key1, a->w[0].ds.step, a->w[0].ds.worker};
        fl.start(ds, ((a->w[0].index0 + (uint64_t)first * kChainTile) >> 3) + (uint32_t)lane);
        fl.run();
    }
    // Lane w looks after worker w's step: one load and ONE correctly rounded division per tile
    // for all workers (at most 32, one per lane), instead of one per worker in every lane; a
    // worker's step and reciprocal are then read from its lane into scalar registers.
    const uint32_t my_worker = (uint32_t)lane < W ? (uint32_t)lane : W - 1u;
    const float* my_steps = a->w[my_worker].steps;
    float steps_ahead = my_steps[one_bucket ? 0u : first / tpb];
    for (uint32_t tile = first; tile < tiles_all; tile += stride) {
        const uint64_t start = (uint64_t)tile * kChainTile;
        // where the dither after this tile's last row belongs: past the end after the last tile (unused)
        const uint64_t next_start = start + (uint64_t)stride * kChainTile;
        float S[kChainRows][8];
        ChainCodes nxt;
        const float steps_here = steps_ahead;
        {
            const uint32_t nt = tile + stride < tiles_all ? tile + stride : tile;
            steps_ahead = my_steps[one_bucket ? 0u : nt / tpb];
        }
        const float invs_here = inv_step(steps_here);
        auto from_lane = [](float x, uint32_t w) __attribute__((always_inline)) {
            return __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)__float_as_uint(x), (int)w));
        };
        // first worker: DQSG, starts the sum; meanwhile the second worker's codes (or the next tile's)
        if (W > 1u) {
            stream_fetch<WR>(a->w[1].codes, start, lane, nxt, limit_for(tile, limitr));
        } else {
            const uint32_t nt = tile + stride < tiles_all ? tile + stride : tile;
            ChainCodes tmp;
            stream_fetch<W0>(a->w[0].codes, (uint64_t)nt * kChainTile, lane, tmp, limit_for(nt, limit0));
            nxt = tmp;
        }
        {
            const DitherStream ds = {a->w[0].ds.key0, a->w[0].ds.key1, a->w[0].ds.step, a->w[0].ds.worker};
            if (PIPED) {
                const uint32_t wn = W > 1u ? 1u : 0u;
                const DitherStream dn = {a->w[wn].ds.key0, a->w[wn].ds.key1, a->w[wn].ds.step, a->w[wn].ds.worker};
                stream_fold_piped<kDq, W0, true>(ds, ((a->w[0].index0 + start) >> 3) + (uint32_t)lane, dn,
                                                 ((a->w[wn].index0 + (W > 1u ? start : next_start)) >> 3) + (uint32_t)lane,
                                                 (float)a->w[0].q_min, 0.0f, cur, from_lane(steps_here, 0u), 0.0f, S, fl);
            } else {
                stream_fold<kDq, W0, true>(ds, (a->w[0].index0 + start) >> 3, (float)a->w[0].q_min, 0.0f, cur,
                                           from_lane(steps_here, 0u), 0.0f, lane, S);
            }
        }
        cur = nxt;
        for (uint32_t w = 1; w < W; ++w) {
            // the codes of worker w are in `cur`; fetch worker w+1's, or the first worker's of the next tile
            if (w + 1u < W) {
                stream_fetch<WR>(a->w[w + 1u].codes, start, lane, nxt, limit_for(tile, limitr));
            } else {
                const uint32_t nt = tile + stride < tiles_all ? tile + stride : tile;
                ChainCodes tmp;
                stream_fetch<W0>(a->w[0].codes, (uint64_t)nt * kChainTile, lane, tmp, limit_for(nt, limit0));
                nxt = tmp;
            }
            const DitherStream ds = {a->w[w].ds.key0, a->w[w].ds.key1, a->w[w].ds.step, a->w[w].ds.worker};
            if (PIPED) {
                const bool last = w + 1u == W;
                const uint32_t wn = last ? 0u : w + 1u;
                const DitherStream dn = {a->w[wn].ds.key0, a->w[wn].ds.key1, a->w[wn].ds.step, a->w[wn].ds.worker};
                stream_fold_piped<RMODE, WR, false>(ds, ((a->w[w].index0 + start) >> 3) + (uint32_t)lane, dn,
                                                    ((a->w[wn].index0 + (last ? next_start : start)) >> 3) + (uint32_t)lane,
                                                    (float)a->w[w].q_min, a->w[w].side_scale, cur,
                                                    from_lane(steps_here, w), from_lane(invs_here, w), S, fl);
            } else {
                stream_fold<RMODE, WR, false>(ds, (a->w[w].index0 + start) >> 3, (float)a->w[w].q_min,
                                              a->w[w].side_scale, cur, from_lane(steps_here, w),
                                              from_lane(invs_here, w), lane, S);
            }
            cur = nxt;
        }
        float* out = out_base + start;
#pragma unroll
        for (int r = 0; r < kChainRows; ++r) {
            const uint32_t o = (uint32_t)(r * kWave + lane) * kLaneElems;
            if (apply_scale) {       // wave-uniform
#pragma unroll
                for (int k = 0; k < 8; ++k) S[r][k] = scale * S[r][k];
            }
            if (PIPED) {
                *(float4*)(out_stage + o) = make_float4(S[r][0], S[r][1], S[r][2], S[r][3]);
                *(float4*)(out_stage + o + 4) = make_float4(S[r][4], S[r][5], S[r][6], S[r][7]);
            } else {
                store_streaming(out + o, S[r][0], S[r][1], S[r][2], S[r][3]);
                store_streaming(out + o + 4, S[r][4], S[r][5], S[r][6], S[r][7]);
            }
        }
        if (PIPED) {
            wave_lds_sync();
            if (TAIL && tile == tiles) {       // the ragged tile: only the elements that exist
#pragma unroll
                for (int j = 0; j < (int)(kChainTile / (kWave * 4)); ++j) {
                    const uint32_t e = (uint32_t)(j * (kWave * 4) + lane * 4);
                    const float4 x = *(const float4*)(out_stage + e);
                    if (e + 4u <= tail_len) {
                        store_streaming(out + e, x.x, x.y, x.z, x.w);
                    } else {
                        if (e < tail_len) out[e] = x.x;
                        if (e + 1u < tail_len) out[e + 1u] = x.y;
                        if (e + 2u < tail_len) out[e + 2u] = x.z;
                    }
                }
            } else {
#pragma unroll
                for (int j = 0; j < (int)(kChainTile / (kWave * 4)); ++j) {
                    const float4 x = *(const float4*)(out_stage + j * (kWave * 4) + lane * 4);
                    store_streaming(out + j * (kWave * 4) + lane * 4, x.x, x.y, x.z, x.w);
                }
            }
            wave_lds_sync();     // the next tile's writes come after these reads
        }
        // the arbiter serves the oldest wave of a SIMD first: lower a wave's priority as it
        // gets ahead, so that the waves of a SIMD finish together
        ++done;
        const uint32_t quarter = my_tiles > 1u ? 4u * done / my_tiles : 0u;
        if (quarter == 1u) __builtin_amdgcn_s_setprio(2);
        else if (quarter == 2u) __builtin_amdgcn_s_setprio(1);
        else if (quarter >= 3u) __builtin_amdgcn_s_setprio(0);
    }
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
// Host side: dispatch
// ---------------------------------------------------------------------------
template <int MODE, int ACC, bool STRADDLE>
static int run_decode3(DecodeArgs a, uint64_t n, uint32_t bucket, hipStream_t s)
{
    const int rc = make_tiling(n, bucket, DecTile<DecRows<MODE, ACC>::R>::N, &a.tl);
    if (rc != NDQ_OK) return rc;
    return launch((decode_kernel<MODE, ACC, STRADDLE>), dim3(blocks_for(a.tl.total_tiles)), dim3(kBlock), s, a);
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

template <int RMODE, int W0, int WR>
static int launch_chain_stream(const ChainArgs& a, hipStream_t s)
{
    // Long vectors: persistent waves, kChainStreamWaves on every SIMD, every wave with the same
    // number of tiles (give or take one).  Otherwise one tile per wave: with only a few tiles
    // per wave a fixed share would leave SIMDs idle at the end.
    const uint32_t tiles = a.tile_begin, slots = 1024u * kChainStreamWaves;
    const bool ragged = (uint64_t)tiles * kChainTile < a.tl.n;     // one more wave takes the ragged last tile
    // (the more workers a tile folds in, the earlier a persistent wave pays: W = 16 gains 3-4 % at
    // one and a half tiles per wave slot, where W = 4 still loses 4 %)
    const StreamTuning& tuning = stream_tuning();
    const bool persistent = tiles >= tuning.chain_min_tiles_per_wave * slots ||
                            (!tuning.threshold_from_env && a.W >= 8u && 2u * (uint64_t)tiles >= 3u * (uint64_t)slots);
    const uint32_t blocks = persistent ? persistent_blocks(tiles + (ragged ? 1u : 0u), 1024u * NDQ_CHAIN_PIPED_WAVES)
                                       : blocks_for(tiles + (ragged ? 1u : 0u));
    if (persistent && ragged)
        return launch((chain_stream_kernel<RMODE, W0, WR, true, true>), dim3(blocks), dim3(kBlock), s, a);
    if (ragged) return launch((chain_stream_kernel<RMODE, W0, WR, true, false>), dim3(blocks), dim3(kBlock), s, a);
    if (persistent) return launch((chain_stream_kernel<RMODE, W0, WR, false, true>), dim3(blocks), dim3(kBlock), s, a);
    return launch((chain_stream_kernel<RMODE, W0, WR, false, false>), dim3(blocks), dim3(kBlock), s, a);
}

template <int RMODE, int W0>
static int launch_chain_stream_w(const ChainArgs& a, uint32_t wr, hipStream_t s)
{
    if (wr == 1u) return launch_chain_stream<RMODE, W0, 1>(a, s);
    if (wr == 2u) return launch_chain_stream<RMODE, W0, 2>(a, s);
    return launch_chain_stream<RMODE, W0, 4>(a, s);
}

// Runs the streaming kernel when the plan and the tiling allow it; returns 1 when it
// does not apply.
static int try_chain_stream(ChainArgs a, uint32_t bucket, hipStream_t s)
{
    if (a.row_buckets || a.continue_sum) return 1;
    if (!(bucket == 0u || bucket % kChainTile == 0u)) return 1;
    const uint32_t w0 = a.w[0].bits;
    if (a.w[0].mode != kDq || !(w0 == 1u || w0 == 2u || w0 == 4u)) return 1;
    uint32_t rmode = kDq, wr = w0;
    if (a.W > 1u) {
        rmode = a.w[1].mode;
        wr = a.w[1].bits;
        if (rmode != kDq && rmode != kNestedPow2) return 1;
        if (!(wr == 1u || wr == 2u || wr == 4u)) return 1;
        for (uint32_t j = 2; j < a.W; ++j)
            if (a.w[j].mode != rmode || a.w[j].bits != wr) return 1;
    }
    const uint32_t full = (uint32_t)(a.tl.n / kChainTile);
    if (full == 0u) return 1;
    ChainArgs b = a;
    b.tile_begin = full;
    int rc;
    if (rmode == kDq) {
        rc = w0 == 1u ? launch_chain_stream_w<kDq, 1>(b, wr, s) : w0 == 2u ? launch_chain_stream_w<kDq, 2>(b, wr, s)
                                                                            : launch_chain_stream_w<kDq, 4>(b, wr, s);
    } else {
        rc = w0 == 1u ? launch_chain_stream_w<kNestedPow2, 1>(b, wr, s)
                      : w0 == 2u ? launch_chain_stream_w<kNestedPow2, 2>(b, wr, s)
                                 : launch_chain_stream_w<kNestedPow2, 4>(b, wr, s);
    }
    return rc;
}

}  // namespace ndq

extern "C" {

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
        if (launch(aggregate_kernel, dim3((uint32_t)blocks), dim3(kBlock), (hipStream_t)stream, a) != NDQ_OK)
            return NDQ_ELAUNCH;
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
    // buckets of exactly one row share a tile, each row with its own step
    a.row_buckets = (kChainRows > 1 && bucket == kWave * kLaneElems) ? 1u : 0u;
    a.num_buckets = a.row_buckets ? (uint32_t)ndq_num_buckets(n, bucket) : 0u;   // n < 2^40: fits
    int rc = make_tiling(n, a.row_buckets ? kChainTile : bucket, kChainTile, &a.tl);
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
        bool any_m = false;
        for (uint32_t j = 0; j < a.W; ++j) any_m = any_m || a.w[j].mode == kNestedAnyM;
        hipStream_t hs = (hipStream_t)stream;
        a.tile_begin = 0u;
#ifndef NDQ_NO_STREAM_CHAIN
        if (W <= kChainMax) {
            const int rc_stream = try_chain_stream(a, bucket, hs);
            if (rc_stream != 1) return rc_stream;
        }
#endif
        const dim3 grid(blocks_for(a.tl.total_tiles)), block(kBlock);
        int rc_launch;
        if (a.row_buckets && any_m) rc_launch = launch((chain_kernel<true, true>), grid, block, hs, a);
        else if (a.row_buckets) rc_launch = launch((chain_kernel<true, false>), grid, block, hs, a);
        else if (any_m) rc_launch = launch((chain_kernel<false, true>), grid, block, hs, a);
        else rc_launch = launch((chain_kernel<false, false>), grid, block, hs, a);
        if (rc_launch != NDQ_OK) return NDQ_ELAUNCH;
    }
    return NDQ_OK;
}

}  // extern "C"
