// Host-side helpers shared by the translation units of libndq: size rules,
// argument checks, tiling and quantizer parameters, launch status.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>

#include <tuple>
#include <utility>

#include "ndq.h"
#include "ndq_device.hpp"

namespace ndq {

inline uint32_t code_bits(uint32_t x)
{
    if (x < 2u || x > 256u) return 0u;
    uint32_t b = 0u;
    while ((1u << b) < x) ++b;
    return b;
}

inline size_t packed_bytes(size_t n, uint32_t bits)
{
    const size_t bytes = (n * (size_t)bits + 7u) / 8u;
    return (bytes + 15u) / 16u * 16u;
}

inline bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }
inline bool aligned4(const void* p) { return ((uintptr_t)p & 3u) == 0; }
constexpr uint64_t kMaxN = (uint64_t)1 << 40;

inline int make_tiling(uint64_t n, uint32_t bucket, uint32_t tile, Tiling* tl)
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

inline int make_quant(uint32_t levels, uint32_t M, bool nested, float alpha, Quant* qp)
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
    qp->inv_M_f = 1.0f / qp->M_f;   // exact when M is a power of two
    qp->bits = code_bits(nested ? M : levels);
    float weights = 0.0f;
    for (uint32_t k = 0; k < 4; ++k) weights += (float)(1u << (k * qp->bits < 31u ? k * qp->bits : 31u));
    qp->pack_bias = -qp->q_min_f * weights;   // exact for bits <= 6, the only user
    return NDQ_OK;
}

inline bool is_pow2(uint32_t x) { return (x & (x - 1u)) == 0u; }

inline DitherStream make_stream(const ndq_dither* d)
{
    DitherStream s;
    s.key0 = (uint32_t)d->seed;
    s.key1 = (uint32_t)(d->seed >> 32);
    s.step = d->step;
    s.worker = d->worker;
    return s;
}

// Launches `kernel` on `stream` and reports the launch call's OWN status.  (The
// thread's last-error slot, hipGetLastError(), is shared with every other user of
// the runtime in the process: reading it could report, and would clear, an error
// that is not ours.)  The arguments are converted to the kernel's parameter types
// first, as a <<<>>> launch would.
template <typename... Params, size_t... I>
inline int launch_with(void (*kernel)(Params...), dim3 grid, dim3 block, hipStream_t stream,
                       std::tuple<Params...>& held, std::index_sequence<I...>)
{
    void* ptrs[sizeof...(Params) ? sizeof...(Params) : 1] = {(void*)&std::get<I>(held)...};
    return hipLaunchKernel((const void*)kernel, grid, block, ptrs, 0, stream) == hipSuccess ? NDQ_OK
                                                                                          : NDQ_ELAUNCH;
}

template <typename... Params, typename... Args>
inline int launch(void (*kernel)(Params...), dim3 grid, dim3 block, hipStream_t stream, Args&&... args)
{
    static_assert(sizeof...(Params) == sizeof...(Args), "one argument per kernel parameter");
    std::tuple<Params...> held(static_cast<Params>(args)...);
    return launch_with(kernel, grid, block, stream, held, std::index_sequence_for<Params...>{});
}

inline uint32_t blocks_for(uint32_t tiles) { return (tiles + kWavesPerBlock - 1) / kWavesPerBlock; }

// When the persistent ("streaming") kernels take over from the one-tile-per-wave
// ones: a vector needs at least `min_tiles_per_wave` tiles for every wave the
// persistent grid would hold, or its fixed shares leave SIMDs idle at the end.
// Two environment variables, read once per process, override the defaults; they
// exist for tuning and so that tests can drive the persistent kernels with short
// vectors:
//   NDQ_STREAM_MIN_TILES_PER_WAVE   threshold for both kernels (0: always persistent)
//   NDQ_STREAM_MAX_BLOCKS           cap on the persistent grid, in workgroups (0: none)
struct StreamTuning {
    uint32_t enc_min_tiles_per_wave, chain_min_tiles_per_wave, max_blocks;
    bool threshold_from_env;
};

inline const StreamTuning& stream_tuning()
{
    static const StreamTuning t = [] {
        // measured over vector lengths, each kernel in both forms in one run: the persistent bfloat16
        // encoders win by 3-9 % from two tiles per wave slot on, the persistent chain decoder by 2-9 %
        // (chains of eight or more workers already from one and a half: see launch_chain_stream)
        StreamTuning v = {2u, 2u, 0u, false};
        if (const char* e = getenv("NDQ_STREAM_MIN_TILES_PER_WAVE")) {
            v.enc_min_tiles_per_wave = v.chain_min_tiles_per_wave = (uint32_t)strtoul(e, nullptr, 10);
            v.threshold_from_env = true;
        }
        if (const char* e = getenv("NDQ_STREAM_MAX_BLOCKS")) v.max_blocks = (uint32_t)strtoul(e, nullptr, 10);
        return v;
    }();
    return t;
}

// Grid of a persistent kernel: `slots` waves, i.e. the same number of workgroups on
// every compute unit (a grid trimmed so that every wave gets exactly the same number
// of tiles leaves some compute units one workgroup short, and the others set the time).
inline uint32_t persistent_blocks(uint32_t tiles, uint32_t slots)
{
    const uint32_t cap = stream_tuning().max_blocks;
    uint32_t blocks = blocks_for(tiles < slots ? tiles : slots);
    if (cap != 0u && blocks > cap) blocks = cap;
    return blocks;
}

}  // namespace ndq
