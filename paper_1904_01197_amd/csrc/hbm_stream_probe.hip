// Streaming-bandwidth probe for gfx950: what the memory system gives a kernel with
// the encoders' traffic -- 8 KB read per tile, a small packed-code write per tile --
// when there is no arithmetic at all.  Stand-alone program, no part of libndq.so;
// the figures are the practical roof the encoders' HBM fractions are read against.
//
// Persistent waves (four per SIMD) walk over tiles wave, wave + W, ...; a tile is
// eight 16-byte non-temporal loads per lane (8 KB per wave) and, per variant, a
// write of 0, 512, 1,024 or 2,048 bytes (one to four 8-byte stores per lane), as a
// 1-, 2- or 4-bit code stream of a bfloat16 tile would be.  Every launch reads a
// different 256 MiB slice of a 3 GiB buffer, so nothing is served from a cache.
//
// build: hipcc -O3 --offload-arch=gfx950 -o hbm_stream_probe hbm_stream_probe.hip
// run:   ./hbm_stream_probe
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>

#define CHECK(x)                                                                          \
    do {                                                                                  \
        hipError_t e_ = (x);                                                              \
        if (e_ != hipSuccess) {                                                           \
            fprintf(stderr, "%s failed: %s (line %d)\n", #x, hipGetErrorString(e_), __LINE__); \
            exit(1);                                                                      \
        }                                                                                 \
    } while (0)

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int CODE_BYTES>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4, 4)))
void stream_kernel(const u32x4* __restrict__ src, uint64_t* codes, uint32_t tiles)
{
    const int lane = threadIdx.x & 63;
    const uint32_t wave = blockIdx.x * 4 + (threadIdx.x >> 6);
    const uint32_t nwaves = gridDim.x * 4;
    constexpr int U = CODE_BYTES / 512;   // 8-byte stores per lane and tile
    uint32_t keep = 0;
    for (uint32_t t = wave; t < tiles; t += nwaves) {
        u32x4 v[8];
#pragma unroll
        for (int r = 0; r < 8; ++r) v[r] = __builtin_nontemporal_load(src + (size_t)t * 512 + lane + r * 64);
        uint32_t acc = 0;
#pragma unroll
        for (int r = 0; r < 8; ++r) acc ^= v[r].x ^ v[r].y ^ v[r].z ^ v[r].w;
        keep ^= acc;
#pragma unroll
        for (int u = 0; u < U; ++u) codes[(size_t)t * (CODE_BYTES / 8) + u * 64 + lane] = ((uint64_t)acc << 32) | (t + u);
    }
    if (CODE_BYTES == 0 && keep == 0x12345678u) codes[wave] = keep;   // keeps the loads alive
}

template <int CODE_BYTES>
static void run(const u32x4* src, uint64_t* codes, size_t bytes, int slices)
{
    const uint32_t tiles = (uint32_t)(bytes / 8192);
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    for (int w = 0; w < 3; ++w)
        hipLaunchKernelGGL(stream_kernel<CODE_BYTES>, dim3(1024), dim3(256), 0, 0, src + (size_t)(w % slices) * (bytes / 16), codes, tiles);
    CHECK(hipDeviceSynchronize());
    const int reps = 20;
    CHECK(hipEventRecord(e0));
    for (int w = 0; w < reps; ++w)
        hipLaunchKernelGGL(stream_kernel<CODE_BYTES>, dim3(1024), dim3(256), 0, 0, src + (size_t)((w + 3) % slices) * (bytes / 16), codes, tiles);
    CHECK(hipEventRecord(e1));
    CHECK(hipEventSynchronize(e1));
    float ms = 0.f;
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    const double sec = ms / reps * 1e-3, wr = (double)tiles * CODE_BYTES;
    printf("8 KB read + %4d B written per tile: %7.2f us per 256 MiB   read %6.0f GB/s   read+write %6.0f GB/s = %.3f of 8 TB/s\n",
           CODE_BYTES, sec * 1e6, bytes / sec / 1e9, (bytes + wr) / sec / 1e9, (bytes + wr) / sec / 8e12);
    CHECK(hipEventDestroy(e0));
    CHECK(hipEventDestroy(e1));
}

int main()
{
    const size_t bytes = (size_t)1 << 28;
    const int slices = 12;
    u32x4* src;
    uint64_t* codes;
    CHECK(hipMalloc(&src, bytes * slices));
    CHECK(hipMalloc(&codes, bytes / 4));
    CHECK(hipMemset(src, 1, bytes * slices));
    // some hundred milliseconds of load first: the clocks settle only after that
    for (int w = 0; w < 300; ++w)
        hipLaunchKernelGGL(stream_kernel<0>, dim3(1024), dim3(256), 0, 0, src + (size_t)(w % slices) * (bytes / 16), codes, (uint32_t)(bytes / 8192));
    CHECK(hipDeviceSynchronize());
    for (int round = 0; round < 2; ++round) {
        run<0>(src, codes, bytes, slices);
        run<512>(src, codes, bytes, slices);
        run<1024>(src, codes, bytes, slices);
        run<2048>(src, codes, bytes, slices);
    }
    CHECK(hipFree(src));
    CHECK(hipFree(codes));
    return 0;
}
