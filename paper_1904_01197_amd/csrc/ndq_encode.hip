// libndq, worker side (gfx950): max-norm scale factors, DQSG / NDQSG encoders.
// See include/ndq.h for the contract.
//
// Every kernel of the library is a streaming pass: a wave owns a tile of
// consecutive elements at a time (one tile per wave in the short-vector kernels,
// tile after tile in the persistent ones), loads it with 16-byte loads,
// regenerates the dither with Philox in registers and writes coalesced vectors.
// Nothing is a contraction, so no MFMA; LDS only transposes the small packed
// codes into stream order and, for buckets of two or four tiles, carries the
// tile maxima between the waves of a workgroup.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "ndq.h"
#include "ndq_device.hpp"
#include "ndq_host.hpp"

namespace ndq {

// ---------------------------------------------------------------------------
// Encoder: Algorithm 1 worker block (DQSG) / Algorithm 2 worker block (NDQSG)
// ---------------------------------------------------------------------------
struct EncodeArgs {
    const void* g;
    unsigned char* codes;
    float* steps;          // written (fused / preset) or read (two-pass, or a step handed over in device memory)
    Tiling tl;
    uint64_t index0;       // dither offset of element 0
    uint64_t total_bytes;  // size of the packed stream incl. zero padding
    DitherStream ds;
    Quant qp;
    float preset_step;     // > 0: bucket == 0 with a caller-set step
    uint32_t rows_log2;    // MULTI: a bucket is 2^rows_log2 rows of a tile
    uint32_t num_buckets;  // MULTI: buckets in the call (steps to write)
    uint32_t waves_log2;   // FUSED, not MULTI: a bucket is 2^waves_log2 tiles of one workgroup
};

template <int DT> struct EncRows { static constexpr int R = kEncLoads / Elem<DT>::V; };
template <int DT> struct EncTile { static constexpr uint32_t N = kWave * kLaneElems * EncRows<DT>::R; };

// A tile in registers: a lane owns 8 consecutive elements per row (one Philox
// block, and 8 codes = `bits` whole bytes of the stream).
template <int DT> struct TileRegs { typename Elem<DT>::Row row[EncRows<DT>::R]; };

// Issues all 16-byte loads of a tile back to back.  FULL: every element of the
// tile is valid, no guards; otherwise elements past the end read as zero.
template <int DT, bool FULL>
__device__ __forceinline__ void load_tile(const void* g, const TileRef& t, int lane, TileRegs<DT>& regs)
{
    using T = Elem<DT>;
    const typename T::scalar* tile = (const typename T::scalar*)g + t.start;
#pragma unroll
    for (int r = 0; r < EncRows<DT>::R; ++r)
        regs.row[r] = load_row<DT, FULL>(tile, (uint32_t)(r * kWave + lane) * kLaneElems, t.len);
}

// folds the lane's share of a tile into its running max |g|
template <int DT>
__device__ __forceinline__ typename Elem<DT>::maxacc lane_max(typename Elem<DT>::maxacc m,
                                                               const TileRegs<DT>& regs)
{
#pragma unroll
    for (int r = 0; r < EncRows<DT>::R; ++r) m = Elem<DT>::max_update(m, regs.row[r]);
    return m;
}

// max |g| over the tile a wave holds (Sec. 3.1 eq. (2)), the same in every lane
template <int DT>
__device__ __forceinline__ float tile_max(const TileRegs<DT>& regs)
{
    using T = Elem<DT>;
    return wave_max(T::max_final(lane_max<DT>(T::max_init(), regs)));
}

// One wave encodes the tile it holds: finds the step, quantizes, and leaves the
// packed codes in `stage` in stream order.  FULL: no guards anywhere.  FUSED: the
// step comes from `kappa`, the max-norm of the tile's bucket, found in registers.
// MULTI (with FUSED): the bucket is a whole number of rows and several buckets
// share the tile, each with its own step.
// REFILL: a row's registers are loaded again while the row is processed, with the same row of
// the whole tile at `refill` (lane `refill_lane`'s share), so that one set of registers holds
// the current tile and, by the end, the next one.
template <int DT, int MODE, bool FUSED, bool FULL, bool MULTI, int BITSW = 0, bool REFILL = false>
__device__ __forceinline__ void encode_tile(const EncodeArgs& a, const TileRef& t, uint32_t tile_id,
                                            typename std::conditional<REFILL, TileRegs<DT>, const TileRegs<DT>>::type& regs,
                                            float kappa, bool writes_step, unsigned char* stage, int lane,
                                            const void* refill = nullptr, int refill_lane = 0)
{
    using T = Elem<DT>;
    constexpr int ROWS = EncRows<DT>::R;
    const uint32_t bits = BITSW ? (uint32_t)BITSW : a.qp.bits;   // BITSW: the code width, known at compile time
    auto& raw = regs.row;

    // 1/step per row (alpha/step for a nested worker that shrinks), wave-uniform
    float inv_row[ROWS];
    if (FUSED && MULTI) {
        // max-norm of every row, then of aligned groups of 2 and 4 rows: a bucket is
        // 1, 2 or 4 rows (Sec. 3.1 eq. (2) per bucket)
        float k1[ROWS], k2[ROWS], k4[ROWS];
#pragma unroll
        for (int r = 0; r < ROWS; ++r)
            k1[r] = wave_max(T::max_final(T::max_update(T::max_init(), raw[r])));
#pragma unroll
        for (int r = 0; r < ROWS; ++r) k2[r] = __builtin_fmaxf(k1[r], k1[r ^ 1]);
#pragma unroll
        for (int r = 0; r < ROWS; ++r) k4[r] = __builtin_fmaxf(k2[r], k2[(r ^ 2) % ROWS]);
        const uint32_t rl = a.rows_log2, group_mask = (1u << rl) - 1u;
#pragma unroll
        for (int r = 0; r < ROWS; ++r) {
            if (((uint32_t)r & group_mask) == 0u) {   // first row of a bucket
                const float kappa_r = rl == 0u ? k1[r] : rl == 1u ? k2[r] : k4[r];
                const float step = step_from_kappa(kappa_r, a.qp.levels);
                const uint32_t bucket = t.bucket * ((uint32_t)ROWS >> rl) + ((uint32_t)r >> rl);
                if (lane == 0 && bucket < a.num_buckets) a.steps[bucket] = step;
                inv_row[r] = __uint_as_float(
                    __builtin_amdgcn_readfirstlane(__float_as_uint(a.qp.alpha * inv_step(step))));
            } else {
                inv_row[r] = inv_row[r > 0 ? r - 1 : 0];
            }
        }
    } else {
        float step;
        if (FUSED) {
            step = step_from_kappa(kappa, a.qp.levels);
            if (REFILL) a.steps[t.bucket] = step;     // every lane, the same value: no branch around the store
            else if (lane == 0 && writes_step) a.steps[t.bucket] = step;
        } else if (a.preset_step > 0.0f) {
            step = a.preset_step;
            // (the streaming kernel writes the preset step itself, outside its tile loop)
            if (!REFILL && tile_id == 0 && lane == 0) a.steps[0] = step;
        } else {
            step = a.steps[t.bucket];
        }
        const float inv_all = a.qp.alpha * inv_step(step);   // alpha = 1 unless a nested worker shrinks
#pragma unroll
        for (int r = 0; r < ROWS; ++r) inv_row[r] = inv_all;
    }
    const uint64_t block0 = (a.index0 + t.start) >> 3;

#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        const uint32_t o = (uint32_t)(r * kWave + lane) * kLaneElems;
        const float inv = inv_row[r];
        float v[8];
        dither8(a.ds, block0 + (o >> 3), v);
        // REFILL: the row is widened to binary32 first and its registers are loaded again right
        // here, at one fixed place per row between the dither and the quantizer (measured: 5 %
        // faster than leaving the load's place to the compiler, which batches two rows' loads
        // and issues them later; earlier, before the dither, is slower too).
        float gw[8];
        if constexpr (REFILL) {
#pragma unroll
            for (int k = 0; k < 8; ++k) gw[k] = T::get(raw[r], k);
            asm volatile("" : "+v"(gw[0]), "+v"(gw[1]), "+v"(gw[2]), "+v"(gw[3]), "+v"(gw[4]), "+v"(gw[5]), "+v"(gw[6]), "+v"(gw[7]));
            raw[r] = load_row<DT, true>(refill, (uint32_t)(r * kWave + refill_lane) * kLaneElems, EncTile<DT>::N);
            __builtin_amdgcn_sched_barrier(0);
        }
        auto elem = [&](int i) __attribute__((always_inline)) { return REFILL ? gw[i] : T::get(raw[r], i); };
        uint32_t quad[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            uint32_t chunk = 0;
            if (MODE == kDqNarrow) {
                // codes of <= 6 bits: sum (q_k - q_min) 2^(k b) stays an exact float below 2^24
                float acc = a.qp.pack_bias;
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    float q = dq_index_f(elem(4 * h + k), inv, v[4 * h + k], a.qp);
                    if (!FULL && o + 4 * h + k >= t.len) q = a.qp.q_min_f;
                    acc = __builtin_fmaf(q, __uint_as_float((127u + k * bits) << 23), acc);
                }
                chunk = (uint32_t)acc;
            } else if (MODE == kNestedAnyMBounded) {
                // residues of <= 6 bits packed like the narrow DQSG codes: exact float fma's
                float acc = 0.0f;
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    float m = nested_residue_f(elem(4 * h + k), inv, v[4 * h + k], a.qp);
                    if (!FULL && o + 4 * h + k >= t.len) m = 0.0f;
                    acc = __builtin_fmaf(m, __uint_as_float((127u + k * bits) << 23), acc);
                }
                chunk = (uint32_t)acc;
            } else if (MODE == kNestedPow2Bounded) {
                // each code enters at the top of the word and moves down as the next
                // ones arrive: one funnel shift per code keeps exactly its low `bits` bits
                uint32_t acc = 0;
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    uint32_t low = nested_low_bits(elem(4 * h + k), inv, v[4 * h + k]);
                    if (!FULL && o + 4 * h + k >= t.len) low = 0;
                    acc = __builtin_amdgcn_alignbit(low, acc, bits);
                }
                chunk = acc >> (32u - 4u * bits);
            } else {
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    uint32_t c = encode_one<MODE>(elem(4 * h + k), inv, v[4 * h + k], a.qp);
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

// Copies a tile's packed codes from the wave's stage to the stream, 8 bytes per lane.
__device__ __forceinline__ void stage_to_stream(const EncodeArgs& a, const TileRef& t, uint32_t bits,
                                                const unsigned char* stage, int lane)
{
    const uint64_t byte0 = (t.start >> 3) * bits;                 // tile start is a multiple of 64
    const bool last = t.start + t.len == a.tl.n;
    const uint64_t nbytes = last ? a.total_bytes - byte0 : (uint64_t)(t.len >> 3) * bits;
    const uint32_t units = (uint32_t)(nbytes >> 3);
    uint64_t* dst = (uint64_t*)(a.codes + byte0);
    const uint64_t* src = (const uint64_t*)stage;
    for (uint32_t u = lane; u < units; u += kWave) dst[u] = src[u];
}

// Occupancy target.  The bfloat16 encoder is bound by instruction issue with a
// burst of loads at the start of every tile; eight waves per SIMD (64 registers)
// hide that burst better than four (+8 % measured).  The binary32 encoder moves
// twice the bytes per element and measured best with the registers it asks for.
#ifndef NDQ_ENC_WAVES_BF16
#define NDQ_ENC_WAVES_BF16 8
#endif
template <int DT> struct EncWaves { static constexpr int W = DT == 1 ? NDQ_ENC_WAVES_BF16 : 4; };
// FUSED: the bucket fits one tile.  MULTI: several buckets to a tile.  BLOCK: the
// bucket is 2 or 4 tiles, all held by the waves of one workgroup.  In all three
// the max-norm is found in registers and the step written; otherwise the step is
// the preset one or read from `steps` (written by the max-norm pass, or handed over).
// BITSW: the code width when it is 1, 2 or 4 (the common ones: the packing and the store of a
// row's codes are then straight-line code); 0: any width, read from the arguments.
template <int DT, int MODE, bool FUSED, bool MULTI, bool BLOCK, int BITSW = 0>
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
    const uint32_t bits = BITSW ? (uint32_t)BITSW : a.qp.bits;
    if (BLOCK) {
        // A bucket of 2 or 4 tiles lies inside one workgroup (tile ids are consecutive
        // and buckets start at multiples of their length): the waves exchange their
        // tile maxima through LDS.  Every wave of the workgroup reaches the barrier,
        // also one whose tile is empty.
        __shared__ float part[kWavesPerBlock];
        TileRegs<DT> regs;
        if (t.len == TILE) load_tile<DT, true>(a.g, t, lane, regs);
        else if (t.len != 0) load_tile<DT, false>(a.g, t, lane, regs);
        float kappa = 0.0f;
        if (t.len != 0) kappa = tile_max<DT>(regs);
        if (lane == 0) part[wave] = kappa;
        __syncthreads();
        const uint32_t group = 1u << a.waves_log2, first = (uint32_t)wave & ~(group - 1u);
        kappa = part[first];
        for (uint32_t w = 1; w < group; ++w) kappa = __builtin_fmaxf(kappa, part[first + w]);
        const bool writes_step = (uint32_t)wave == first;
        if (t.len == TILE)
            encode_tile<DT, MODE, true, true, false>(a, t, tile_id, regs, kappa, writes_step, stage, lane);
        else if (t.len != 0)
            encode_tile<DT, MODE, true, false, false>(a, t, tile_id, regs, kappa, writes_step, stage, lane);
    } else if (t.len == TILE) {
        TileRegs<DT> regs;
        load_tile<DT, true>(a.g, t, lane, regs);
        const float kappa = (FUSED && !MULTI) ? tile_max<DT>(regs) : 0.0f;
        encode_tile<DT, MODE, FUSED, true, MULTI, BITSW>(a, t, tile_id, regs, kappa, true, stage, lane);
    } else if (t.len != 0) {
        TileRegs<DT> regs;
        load_tile<DT, false>(a.g, t, lane, regs);
        const float kappa = (FUSED && !MULTI) ? tile_max<DT>(regs) : 0.0f;
        encode_tile<DT, MODE, FUSED, false, MULTI, BITSW>(a, t, tile_id, regs, kappa, true, stage, lane);
    }
    wave_lds_sync();     // a wave copies out only the stage it filled itself
    if (t.len != 0) stage_to_stream(a, t, bits, stage, lane);
}

// The same for a full tile that is not the vector's last, with the code width known
// at compile time: a fixed number of store instructions, so that the compiler can
// count the memory operations in flight between a tile's loads and its use.
template <int DT, int BITSW>
__device__ __forceinline__ void stage_to_stream_full(const EncodeArgs& a, const TileRef& t,
                                                     const unsigned char* stage, int lane)
{
    constexpr uint32_t units = EncTile<DT>::N / 64u * BITSW;       // 8-byte units: a multiple of 64 for bfloat16 tiles
    uint64_t* dst = (uint64_t*)(a.codes + (t.start >> 3) * BITSW);
    const uint64_t* src = (const uint64_t*)stage;
    if constexpr (units % kWave == 0u) {
#pragma unroll
        for (uint32_t u = 0; u < units; u += kWave) dst[u + lane] = src[u + lane];
    } else {
        static_assert(units < (uint32_t)kWave, "a partial store only for less than one unit per lane");
        if ((uint32_t)lane < units) dst[lane] = src[lane];
    }
}

// ---------------------------------------------------------------------------
// Streaming encoder for vectors made of whole tiles (bucket == tile with the
// max-norm found in registers, or one step for the whole vector): every wave
// walks over the tiles wave, wave + W, wave + 2W, ... (W = waves in the grid).
// One set of registers holds the current tile and, by the end of it, the next
// one: as soon as a row is quantized its registers are loaded again with the
// same row of the wave's next tile, so the loads leave one row at a time
// instead of a tile at a time, and a row has the rest of the tile's arithmetic
// (the first) down to the copy-out (the last) to arrive.  Measured against two
// register sets with the whole next tile requested at the start of the current
// one: 49.7 against 52.6 us (1-bit nested) and 57.5 against 59.9 us (2-bit
// DQSG) at 2^27 bfloat16 elements; with the registers this frees, 5, 6 or 8
// waves per SIMD are slower than 4 (55, 55, 54 us), and so are 3 and 2.
// No wave is ever new: the instruction arbiter serves older waves first, so in
// a one-tile-per-wave grid a new wave crawls through its address arithmetic,
// its loads and its max-norm behind busy neighbours, and the SIMD idles
// whenever those neighbours run out at the same time.
// ---------------------------------------------------------------------------
#ifndef NDQ_STREAM_WAVES
#define NDQ_STREAM_WAVES 4
#endif
constexpr int kStreamWaves = NDQ_STREAM_WAVES;   // per SIMD

template <int DT>
__device__ __forceinline__ TileRef stream_tile_ref(const EncodeArgs& a, uint32_t tile_id, bool fused)
{
    TileRef t;
    t.start = (uint64_t)tile_id * EncTile<DT>::N;
    t.len = EncTile<DT>::N;
    t.bucket = fused ? tile_id : 0u;
    return t;
}

template <int DT, int MODE, bool FUSED, int BITSW>
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(kStreamWaves, kStreamWaves)))
void encode_stream_kernel(EncodeArgs a, uint32_t full_tiles)
{
    constexpr uint32_t TILE = EncTile<DT>::N;
    __shared__ __align__(16) unsigned char stage_all[kWavesPerBlock][TILE + 8];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    unsigned char* stage = stage_all[wave];
    const uint32_t stride = gridDim.x * kWavesPerBlock;
    const uint32_t first = blockIdx.x * kWavesPerBlock + wave;
    if (!FUSED && a.preset_step > 0.0f && first == 0u && lane == 0) a.steps[0] = a.preset_step;
    if (first < full_tiles) {
        // Every pass over a tile issues exactly one load per row, also the last one (then of the
        // vector's first 16 bytes per row, all lanes alike: one cache line, no traffic to speak
        // of), and the code width is a compile-time constant, so that the number of memory
        // operations in flight at every wait is known at compile time: they complete in order,
        // and a wait must cover a row's load but not the loads and stores issued after it.
        TileRegs<DT> regs;
        uint32_t cur = first;
        // The arbiter serves the oldest wave of a SIMD first, so left alone the waves of a
        // SIMD finish one after the other and the last one runs alone, at a third of the
        // SIMD's rate.  Lower a wave's priority as it gets ahead: they finish together.
        const uint32_t my_tiles = (full_tiles - first + stride - 1) / stride;
        uint32_t done = 0;
        __builtin_amdgcn_s_setprio(3);
        load_tile<DT, true>(a.g, stream_tile_ref<DT>(a, cur, FUSED), lane, regs);
        for (;;) {
            const uint32_t nxt = cur + stride;
            const bool more = nxt < full_tiles;
            const TileRef t = stream_tile_ref<DT>(a, cur, FUSED);
            const float kappa = FUSED ? tile_max<DT>(regs) : 0.0f;
            wave_lds_sync();     // the previous tile's copy-out has read the stage
            encode_tile<DT, MODE, FUSED, true, false, BITSW, true>(
                a, t, cur, regs, kappa, true, stage, lane,
                (const typename Elem<DT>::scalar*)a.g + (uint64_t)(more ? nxt : 0u) * TILE, more ? lane : 0);
            wave_lds_sync();
            stage_to_stream_full<DT, BITSW>(a, t, stage, lane);
            if (!more) break;
            ++done;
            const uint32_t quarter = 4u * done / my_tiles;
            if (quarter == 1u) __builtin_amdgcn_s_setprio(2);
            else if (quarter == 2u) __builtin_amdgcn_s_setprio(1);
            else if (quarter >= 3u) __builtin_amdgcn_s_setprio(0);
            cur = nxt;
        }
    }
    // the ragged last tile, if there is one, by the wave whose turn it would be
    if (full_tiles < a.tl.total_tiles && full_tiles % stride == first) {
        const TileRef t = locate_tile(a.tl, full_tiles, TILE);
        if (t.len != 0) {
            TileRegs<DT> regs;
            load_tile<DT, false>(a.g, t, lane, regs);
            const float kappa = FUSED ? tile_max<DT>(regs) : 0.0f;
            wave_lds_sync();
            encode_tile<DT, MODE, FUSED, false, false, BITSW>(a, t, full_tiles, regs, kappa, true, stage, lane);
            wave_lds_sync();
            stage_to_stream(a, t, BITSW ? (uint32_t)BITSW : a.qp.bits, stage, lane);
        }
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

// levels != 0: the bucket's step is wanted, not its max-norm.  The step rule is monotone in
// kappa (an exact doubling, one correctly rounded division, a threshold), so the maximum of
// the parts' steps is the step of the maximum: each part converts before its atomic, and no
// pass over the buckets is needed afterwards.
__device__ __forceinline__ uint32_t absmax_word(float m, uint32_t levels)
{
    // non-negative floats order like their bit patterns
    return __float_as_uint(levels ? step_from_kappa(m, levels) : m);
}

template <int DT>
__global__ __launch_bounds__(kBlock) void absmax_kernel(const void* g, Tiling tl, uint32_t* kappa_bits,
                                                       uint32_t levels)
{
    using T = Elem<DT>;
    constexpr uint32_t TILE = EncTile<DT>::N;
    const int lane = threadIdx.x & (kWave - 1);
    const uint32_t tile_id =
        blockIdx.x * kWavesPerBlock + __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const TileRef t = locate_tile(tl, tile_id, TILE);
    if (t.len == 0) return;
    TileRegs<DT> regs;
    if (t.len == TILE) load_tile<DT, true>(g, t, lane, regs);
    else load_tile<DT, false>(g, t, lane, regs);
    const float m = tile_max<DT>(regs);
    if (lane == 0) atomicMax(kappa_bits + t.bucket, absmax_word(m, levels));
}

// The same for buckets of many tiles (a whole vector at the extreme), where one
// atomic per tile would serialize every tile on one address: a workgroup's
// waves stride over the bucket's tiles with the running max in registers, and
// the workgroup issues a single atomic at the end.
template <int DT>
__global__ __launch_bounds__(kBlock) void absmax_span_kernel(const void* g, Tiling tl, uint32_t* kappa_bits,
                                                            uint32_t blocks_per_bucket, uint32_t levels)
{
    using T = Elem<DT>;
    constexpr uint32_t TILE = EncTile<DT>::N;
    constexpr int ROWS = EncRows<DT>::R;
    __shared__ float part[kWavesPerBlock];
    const int lane = threadIdx.x & (kWave - 1);
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const uint32_t bucket = blockIdx.x / blocks_per_bucket;
    const uint32_t first = (blockIdx.x - bucket * blocks_per_bucket) * kWavesPerBlock + wave;
    const uint32_t stride = blocks_per_bucket * kWavesPerBlock;
    typename T::maxacc acc = T::max_init();
    for (uint32_t j = first; j < tl.tiles_per_bucket; j += stride) {
        const TileRef t = locate_tile(tl, bucket * tl.tiles_per_bucket + j, TILE);
        if (t.len == 0) break;   // past the end of the vector: so are this wave's later tiles
        TileRegs<DT> regs;
        if (t.len == TILE) load_tile<DT, true>(g, t, lane, regs);
        else load_tile<DT, false>(g, t, lane, regs);
        acc = lane_max<DT>(acc, regs);
    }
    const float m = wave_max(T::max_final(acc));
    if (lane == 0) part[wave] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        float all = part[0];
#pragma unroll
        for (int w = 1; w < kWavesPerBlock; ++w) all = __builtin_fmaxf(all, part[w]);
        atomicMax(kappa_bits + bucket, absmax_word(all, levels));
    }
}

// A step that already lies in device memory becomes this worker's transmitted step.
__global__ void copy_step_kernel(const float* step_in, float* steps)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) steps[0] = step_in[0];
}

// ---------------------------------------------------------------------------
// Host side: dispatch
// ---------------------------------------------------------------------------
template <int DT>
static int run_absmax(const void* g, const Tiling& tl, uint64_t K, float* kappa, uint32_t levels, hipStream_t s)
{
    if (launch(fill_zero_kernel, dim3((uint32_t)((K + 255) / 256)), dim3(256), s, (uint32_t*)kappa, K) != NDQ_OK)
        return NDQ_ELAUNCH;
    // many tiles per bucket: a few hundred tiles per workgroup, about 4096 workgroups in all
    constexpr uint32_t kSpanMinTiles = 64, kSpanTarget = 4096;
    if (tl.tiles_per_bucket >= kSpanMinTiles && K <= kSpanTarget) {
        uint32_t per_bucket = kSpanTarget / (uint32_t)K;
        const uint32_t most = tl.tiles_per_bucket / (2 * kWavesPerBlock);   // at least two tiles per wave
        if (per_bucket > most) per_bucket = most;
        if (per_bucket < 1) per_bucket = 1;
        return launch(absmax_span_kernel<DT>, dim3((uint32_t)K * per_bucket), dim3(kBlock), s, g, tl,
                      (uint32_t*)kappa, per_bucket, levels);
    }
    return launch(absmax_kernel<DT>, dim3(blocks_for(tl.total_tiles)), dim3(kBlock), s, g, tl, (uint32_t*)kappa,
                  levels);
}

// Waves of the streaming kernel: kStreamWaves on each of the 1,024 SIMDs.
constexpr uint32_t kStreamSlots = 1024u * kStreamWaves;

template <int DT, int MODE, bool FUSED, int BITSW>
static int launch_stream(const EncodeArgs& a, uint32_t full_tiles, hipStream_t s)
{
    const uint32_t blocks = persistent_blocks(full_tiles, kStreamSlots);
    return launch((encode_stream_kernel<DT, MODE, FUSED, BITSW>), dim3(blocks), dim3(kBlock), s, a, full_tiles);
}

// The streaming kernel serves vectors cut into whole tiles (a ragged last one aside):
// bucket == tile (fused max-norm) or one step for the whole vector (preset, or found by
// the max-norm pass), in the quantizer modes and code widths of the common
// configurations.  Returns 1 when it does not apply.
template <int DT, int MODE>
static int try_stream(const EncodeArgs& a, bool fused, bool multi, uint32_t bucket, hipStream_t s)
{
    constexpr uint32_t TILE = EncTile<DT>::N;
    // binary32 input: one tile per wave is faster at every length (2^27 elements: 112 against 120 us,
    // 25.6 M: 22.8 against 23.2; its tile carries half the arithmetic of a bfloat16 tile per byte, so
    // the kernel is nearer to a plain copy, which gains nothing from persistence); bfloat16: the
    // persistent kernel wins from two tiles per wave slot on (3-9 %)
    if constexpr (DT == 0 || (MODE != kDqNarrow && MODE != kNestedPow2Bounded && MODE != kNestedPow2)) {
        return 1;
    } else {
    if (multi || a.waves_log2 != 0u) return 1;
    if (!(bucket == TILE || bucket == 0u)) return 1;
    if (fused != (bucket == TILE)) return 1;
    const uint32_t full_tiles = (uint32_t)(a.tl.n / TILE);
    // shorter vectors: with only a few tiles per wave a fixed share leaves SIMDs idle at the end
    if (full_tiles == 0u || full_tiles < stream_tuning().enc_min_tiles_per_wave * kStreamSlots) return 1;
    const uint32_t bits = a.qp.bits;
    if (bits != 1u && bits != 2u && bits != 4u) return 1;
    if (fused) {
        if constexpr (MODE == kNestedPow2) {
            return 1;      // a preset step comes with bucket == 0
        } else {
            if (bits == 1u) return launch_stream<DT, MODE, true, 1>(a, full_tiles, s);
            if (bits == 2u) return launch_stream<DT, MODE, true, 2>(a, full_tiles, s);
            return launch_stream<DT, MODE, true, 4>(a, full_tiles, s);
        }
    }
    if (bits == 1u) return launch_stream<DT, MODE, false, 1>(a, full_tiles, s);
    if (bits == 2u) return launch_stream<DT, MODE, false, 2>(a, full_tiles, s);
    return launch_stream<DT, MODE, false, 4>(a, full_tiles, s);
    }
}

template <int DT, int MODE>
static int run_encode(const EncodeArgs& a, bool fused, bool multi, uint32_t bucket, hipStream_t s)
{
#ifndef NDQ_NO_STREAM_ENCODER
    const int rc = try_stream<DT, MODE>(a, fused, multi, bucket, s);
    if (rc != 1) return rc;
#endif
    const dim3 grid(blocks_for(a.tl.total_tiles)), block(kBlock);
    if (a.waves_log2 != 0u) return launch((encode_kernel<DT, MODE, true, false, true>), grid, block, s, a);
    if (multi) return launch((encode_kernel<DT, MODE, true, true, false>), grid, block, s, a);
    if constexpr (MODE == kDqNarrow || MODE == kNestedPow2Bounded || MODE == kNestedPow2) {
        const uint32_t bits = a.qp.bits;
        if (fused) {
            if (bits == 1u) return launch((encode_kernel<DT, MODE, true, false, false, 1>), grid, block, s, a);
            if (bits == 2u) return launch((encode_kernel<DT, MODE, true, false, false, 2>), grid, block, s, a);
            if (bits == 4u) return launch((encode_kernel<DT, MODE, true, false, false, 4>), grid, block, s, a);
        } else {
            if (bits == 1u) return launch((encode_kernel<DT, MODE, false, false, false, 1>), grid, block, s, a);
            if (bits == 2u) return launch((encode_kernel<DT, MODE, false, false, false, 2>), grid, block, s, a);
            if (bits == 4u) return launch((encode_kernel<DT, MODE, false, false, false, 4>), grid, block, s, a);
        }
    }
    if (fused) return launch((encode_kernel<DT, MODE, true, false, false>), grid, block, s, a);
    return launch((encode_kernel<DT, MODE, false, false, false>), grid, block, s, a);
}

// step_in != nullptr: one step for the whole vector, read from device memory when the
// kernels run (bucket and delta are then 0, and `levels` is not used to derive a step).
static int encode_common(const void* g, int dt, size_t n, float delta, const float* step_in,
                         uint32_t levels, uint32_t M, bool nested, float alpha, uint32_t bucket,
                         const ndq_dither* d, void* codes_out, float* steps_out, void* stream)
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
    if (step_in && !aligned4(step_in)) return NDQ_EALIGN;
    if (bucket % 64u != 0u || (d->offset & 7u) != 0u) return NDQ_EALIGN;

    const uint32_t tile = dt == NDQ_F32 ? EncTile<0>::N : EncTile<1>::N;
    // buckets of 1, 2 or 4 whole rows (2, 4 or 8 to a tile) share tiles: the tiling is
    // that of tile-sized buckets and the kernel finds a max-norm per group of rows
    constexpr uint32_t row = kWave * kLaneElems;
    const bool multi = bucket != 0u && bucket < tile && tile % bucket == 0u && bucket % row == 0u &&
                       bucket / row <= 4u && (bucket / row & (bucket / row - 1u)) == 0u;
    rc = make_tiling(n, multi ? tile : bucket, tile, &a.tl);
    if (rc != NDQ_OK) return rc;
    a.rows_log2 = multi ? (bucket / row == 1u ? 0u : bucket / row == 2u ? 1u : 2u) : 0u;
    // buckets of 2 or 4 tiles: the waves of one workgroup hold the whole bucket
    const bool block_fused = kWavesPerBlock == 4 && (bucket == 2u * tile || bucket == 4u * tile);
    a.waves_log2 = block_fused ? (bucket == 2u * tile ? 1u : 2u) : 0u;
    a.num_buckets = (uint32_t)((n + (bucket ? bucket : n) - 1) / (bucket ? bucket : n));
    a.g = g;
    a.codes = (unsigned char*)codes_out;
    a.steps = steps_out;
    a.index0 = d->offset;
    a.total_bytes = packed_bytes(n, a.qp.bits);
    a.ds = make_stream(d);
    a.preset_step = (bucket == 0u && delta > 0.0f) ? delta : 0.0f;
    hipStream_t s = (hipStream_t)stream;

    const bool fused = (bucket != 0u && bucket <= tile) || block_fused;   // (multi implies fused)
    if (step_in) {
        // the kernels read steps_out[0], as after the max-norm passes below
        if (step_in != steps_out &&
            launch(copy_step_kernel, dim3(1), dim3(kWave), s, step_in, steps_out) != NDQ_OK)
            return NDQ_ELAUNCH;
    } else if (!fused && a.preset_step == 0.0f) {
        // two passes: the step of every bucket from its max-norm, then the encoder reads them
        const uint64_t K = bucket ? (n + bucket - 1) / bucket : 1;
        rc = dt == NDQ_F32 ? run_absmax<0>(g, a.tl, K, steps_out, levels, s)
                           : run_absmax<1>(g, a.tl, K, steps_out, levels, s);
        if (rc != NDQ_OK) return rc;
    }
#ifndef NDQ_NARROW_MAX_BITS
#define NDQ_NARROW_MAX_BITS 6u
#endif
    // a step derived from the data bounds |g/Delta|; a caller's step (preset, or in device memory) does not
    const bool own_step = a.preset_step == 0.0f && !step_in;
    const int mode = !nested ? (a.qp.bits <= NDQ_NARROW_MAX_BITS ? kDqNarrow : kDq)
                             : (!is_pow2(M) ? ((!own_step || a.qp.bits > 6u) ? kNestedAnyM : kNestedAnyMBounded)
                                            : (!own_step ? kNestedPow2 : kNestedPow2Bounded));
    if (dt == NDQ_F32) {
        if (mode == kDqNarrow) return run_encode<0, kDqNarrow>(a, fused, multi, bucket, s);
        if (mode == kDq) return run_encode<0, kDq>(a, fused, multi, bucket, s);
        if (mode == kNestedPow2) return run_encode<0, kNestedPow2>(a, fused, multi, bucket, s);
        if (mode == kNestedPow2Bounded) return run_encode<0, kNestedPow2Bounded>(a, fused, multi, bucket, s);
        if (mode == kNestedAnyMBounded) return run_encode<0, kNestedAnyMBounded>(a, fused, multi, bucket, s);
        return run_encode<0, kNestedAnyM>(a, fused, multi, bucket, s);
    }
    if (mode == kDqNarrow) return run_encode<1, kDqNarrow>(a, fused, multi, bucket, s);
    if (mode == kDq) return run_encode<1, kDq>(a, fused, multi, bucket, s);
    if (mode == kNestedPow2) return run_encode<1, kNestedPow2>(a, fused, multi, bucket, s);
    if (mode == kNestedPow2Bounded) return run_encode<1, kNestedPow2Bounded>(a, fused, multi, bucket, s);
    if (mode == kNestedAnyMBounded) return run_encode<1, kNestedAnyMBounded>(a, fused, multi, bucket, s);
    return run_encode<1, kNestedAnyM>(a, fused, multi, bucket, s);
}

}  // namespace ndq

extern "C" {

int ndq_absmax(const void* g, int dt, size_t n, uint32_t bucket, float* kappa_out,
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
        return launch(fill_zero_kernel, dim3(1), dim3(256), s, (uint32_t*)kappa_out, (uint64_t)1);
    }
    if (!g) return NDQ_EINVAL;
    if (!aligned16(g)) return NDQ_EALIGN;
    Tiling tl;
    const uint32_t tile = dt == NDQ_F32 ? EncTile<0>::N : EncTile<1>::N;
    int rc = make_tiling(n, bucket, tile, &tl);
    if (rc != NDQ_OK) return rc;
    const uint64_t K = bucket ? (n + bucket - 1) / bucket : 1;
    return dt == NDQ_F32 ? run_absmax<0>(g, tl, K, kappa_out, 0u, s) : run_absmax<1>(g, tl, K, kappa_out, 0u, s);
}

int ndq_dq_encode(const void* g, int dt, size_t n, float delta, uint32_t levels,
                  uint32_t bucket, const ndq_dither* d, void* codes_out, float* steps_out,
                  void* stream)
{
    return ndq::encode_common(g, dt, n, delta, nullptr, levels, 0u, false, 1.0f, bucket, d, codes_out,
                              steps_out, stream);
}

int ndq_dq_encode_with_step(const void* g, int dt, size_t n, const float* step_in, uint32_t levels,
                            const ndq_dither* d, void* codes_out, float* steps_out, void* stream)
{
    if (!step_in && n != 0) return NDQ_EINVAL;
    return ndq::encode_common(g, dt, n, 0.0f, step_in, levels, 0u, false, 1.0f, 0u, d, codes_out,
                              steps_out, stream);
}

int ndq_nested_encode(const void* g, int dt, size_t n, float delta, uint32_t levels,
                      uint32_t M, float alpha, uint32_t bucket, const ndq_dither* d,
                      void* codes_out, float* steps_out, void* stream)
{
    return ndq::encode_common(g, dt, n, delta, nullptr, levels, M, true, alpha, bucket, d, codes_out,
                              steps_out, stream);
}

int ndq_nested_encode_with_step(const void* g, int dt, size_t n, const float* step_in, uint32_t M,
                                float alpha, const ndq_dither* d, void* codes_out, float* steps_out,
                                void* stream)
{
    if (!step_in && n != 0) return NDQ_EINVAL;
    // the number of fine levels only ever served to derive a step: any valid value will do
    return ndq::encode_common(g, dt, n, 0.0f, step_in, 2u, M, true, alpha, 0u, d, codes_out,
                              steps_out, stream);
}

}  // extern "C"
