// Issue-rate probe for gfx950 vector-ALU instructions: the measurement behind the
// instruction choices in the libndq kernels and behind the weights of the
// benchmark's "alu" roof.  Stand-alone program, no part of libndq.so.
//
// Every kernel runs one instruction (or a fixed pair) in a loop on eight
// independent register chains per lane, written in inline assembly so that the
// mix is exact; 2,048 workgroups of 256 lanes keep eight waves on every SIMD of
// the 256 compute units.  Reported per instruction: the time per wave64
// instruction per SIMD, in nanoseconds and in shader-clock cycles.  The shader
// clock is measured, not assumed: lane 0 of every wave reads the shader-cycle
// counter (s_memtime) and the constant 100 MHz counter (s_memrealtime) around
// its loop, and the ratio of the two differences is the clock the loop ran at.
//
// build: hipcc -O3 --offload-arch=gfx950 -o valu_issue_probe valu_issue_probe.hip
// run:   ./valu_issue_probe            (prints one line per instruction)
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#define CHECK(x)                                                                          \
    do {                                                                                  \
        hipError_t e_ = (x);                                                              \
        if (e_ != hipSuccess) {                                                           \
            fprintf(stderr, "%s failed: %s (line %d)\n", #x, hipGetErrorString(e_), __LINE__); \
            exit(1);                                                                      \
        }                                                                                 \
    } while (0)

constexpr int kIters = 2048;
constexpr int kChains = 8;
constexpr int kGrid = 2048, kBlockThreads = 256;

struct Clocks { unsigned long long shader, realtime; };

// One instruction per chain and iteration.  OP is a macro taking the chain's
// register (read-write), and two loop-invariant vector operands.
#define PROBE_KERNEL(NAME, ASM, CONSTRAINTS_EXTRA)                                        \
    __global__ void NAME(uint32_t* out, Clocks* clk, uint32_t p, uint32_t q)              \
    {                                                                                     \
        uint32_t a[kChains];                                                              \
        for (int c = 0; c < kChains; ++c) a[c] = (threadIdx.x + 1u) * (2u * c + 3u);      \
        uint32_t vp = p ^ threadIdx.x, vq = q + threadIdx.x;                              \
        const unsigned long long s0 = __builtin_readcyclecounter();                      \
        const unsigned long long r0 = __builtin_amdgcn_s_memrealtime();                  \
        for (int it = 0; it < kIters; ++it) {                                             \
            _Pragma("unroll") for (int c = 0; c < kChains; ++c)                           \
                asm volatile(ASM : "+v"(a[c]) : "v"(vp), "v"(vq) CONSTRAINTS_EXTRA);      \
        }                                                                                 \
        const unsigned long long s1 = __builtin_readcyclecounter();                      \
        const unsigned long long r1 = __builtin_amdgcn_s_memrealtime();                  \
        uint32_t sum = 0;                                                                 \
        for (int c = 0; c < kChains; ++c) sum += a[c];                                    \
        out[blockIdx.x * blockDim.x + threadIdx.x] = sum;                                 \
        if (threadIdx.x == 0 && blockIdx.x == 0) { clk->shader = s1 - s0; clk->realtime = r1 - r0; } \
    }

#define NOCLOB
#define VCC : "vcc"

// full-rate candidates
PROBE_KERNEL(k_mov, "v_mov_b32_e32 %0, %1", NOCLOB)
PROBE_KERNEL(k_add_f32, "v_add_f32_e32 %0, %0, %1", NOCLOB)
PROBE_KERNEL(k_sub_f32, "v_sub_f32_e32 %0, %0, %1", NOCLOB)
PROBE_KERNEL(k_mul_f32, "v_mul_f32_e32 %0, %0, %1", NOCLOB)
PROBE_KERNEL(k_fma_f32, "v_fma_f32 %0, %0, %1, %2", NOCLOB)
PROBE_KERNEL(k_fmac_f32, "v_fmac_f32_e32 %0, %1, %2", NOCLOB)
PROBE_KERNEL(k_add_u32, "v_add_u32_e32 %0, %0, %1", NOCLOB)
PROBE_KERNEL(k_and_b32, "v_and_b32_e32 %0, %0, %1", NOCLOB)
PROBE_KERNEL(k_xor_b32, "v_xor_b32_e32 %0, %0, %1", NOCLOB)
PROBE_KERNEL(k_bitop3, "v_bitop3_b32 %0, %0, %1, %2 bitop3:0x96", NOCLOB)
PROBE_KERNEL(k_and_or, "v_and_or_b32 %0, %0, %1, %2", NOCLOB)
PROBE_KERNEL(k_or3, "v_or3_b32 %0, %0, %1, %2", NOCLOB)
PROBE_KERNEL(k_bfi, "v_bfi_b32 %0, %1, %0, %2", NOCLOB)
PROBE_KERNEL(k_mul_u32_u24, "v_mul_u32_u24_e32 %0, %0, %1", NOCLOB)
PROBE_KERNEL(k_mad_u32_u24, "v_mad_u32_u24 %0, %0, %1, %2", NOCLOB)
PROBE_KERNEL(k_perm, "v_perm_b32 %0, %0, %1, %2", NOCLOB)
PROBE_KERNEL(k_or_sdwa_w1, "v_or_b32_sdwa %0, %0, %1 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:WORD_1 src1_sel:DWORD", NOCLOB)
PROBE_KERNEL(k_cndmask, "v_cndmask_b32_e32 %0, %0, %1, vcc", NOCLOB)
PROBE_KERNEL(k_cmp_lt_f32, "v_cmp_lt_f32_e32 vcc, %0, %1", VCC)
// half-rate candidates
PROBE_KERNEL(k_rndne_f32, "v_rndne_f32_e32 %0, %0", NOCLOB)
PROBE_KERNEL(k_floor_f32, "v_floor_f32_e32 %0, %0", NOCLOB)
PROBE_KERNEL(k_cvt_f32_u32, "v_cvt_f32_u32_e32 %0, %0", NOCLOB)
PROBE_KERNEL(k_cvt_f32_u32_sdwa_w1, "v_cvt_f32_u32_sdwa %0, %0 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:WORD_1", NOCLOB)
PROBE_KERNEL(k_cvt_f32_ubyte0, "v_cvt_f32_ubyte0_e32 %0, %0", NOCLOB)
PROBE_KERNEL(k_cvt_u32_f32, "v_cvt_u32_f32_e32 %0, %0", NOCLOB)
PROBE_KERNEL(k_cvt_i32_f32, "v_cvt_i32_f32_e32 %0, %0", NOCLOB)
PROBE_KERNEL(k_max_f32, "v_max_f32_e32 %0, %0, %1", NOCLOB)
PROBE_KERNEL(k_min_f32, "v_min_f32_e32 %0, %0, %1", NOCLOB)
PROBE_KERNEL(k_med3_f32, "v_med3_f32 %0, %0, %1, %2", NOCLOB)
PROBE_KERNEL(k_max_u32, "v_max_u32_e32 %0, %0, %1", NOCLOB)
PROBE_KERNEL(k_pk_max_u16, "v_pk_max_u16 %0, %0, %1", NOCLOB)
PROBE_KERNEL(k_lshlrev_b32, "v_lshlrev_b32_e32 %0, %1, %0", NOCLOB)
PROBE_KERNEL(k_lshrrev_b32, "v_lshrrev_b32_e32 %0, %1, %0", NOCLOB)
PROBE_KERNEL(k_bfe_u32, "v_bfe_u32 %0, %0, %1, %2", NOCLOB)
PROBE_KERNEL(k_lshl_or, "v_lshl_or_b32 %0, %0, %1, %2", NOCLOB)
PROBE_KERNEL(k_lshl_add, "v_lshl_add_u32 %0, %0, %1, %2", NOCLOB)
PROBE_KERNEL(k_alignbit, "v_alignbit_b32 %0, %0, %1, %2", NOCLOB)
PROBE_KERNEL(k_add3_u32, "v_add3_u32 %0, %0, %1, %2", NOCLOB)
PROBE_KERNEL(k_mul_lo_u32, "v_mul_lo_u32 %0, %0, %1", NOCLOB)
PROBE_KERNEL(k_mul_hi_u32, "v_mul_hi_u32 %0, %0, %1", NOCLOB)
PROBE_KERNEL(k_rcp_f32, "v_rcp_f32_e32 %0, %0", NOCLOB)
// fixed pairs (two instructions per chain and iteration)
PROBE_KERNEL(k_pair_fma_fma, "v_fma_f32 %0, %0, %1, %2\n v_fma_f32 %0, %0, %2, %1", NOCLOB)
PROBE_KERNEL(k_pair_fma_xor, "v_fma_f32 %0, %0, %1, %2\n v_xor_b32_e32 %0, %0, %1", NOCLOB)
PROBE_KERNEL(k_pair_rndne_add, "v_rndne_f32_e32 %0, %0\n v_add_f32_e32 %0, %0, %1", NOCLOB)
PROBE_KERNEL(k_pair_rndne_xor, "v_rndne_f32_e32 %0, %0\n v_xor_b32_e32 %0, %0, %1", NOCLOB)
PROBE_KERNEL(k_pair_cvt_fma, "v_cvt_f32_u32_e32 %0, %0\n v_fma_f32 %0, %0, %1, %2", NOCLOB)
PROBE_KERNEL(k_pair_alignbit_fma, "v_alignbit_b32 %0, %0, %1, %2\n v_fma_f32 %0, %0, %1, %2", NOCLOB)
PROBE_KERNEL(k_pair_alignbit_xor, "v_alignbit_b32 %0, %0, %1, %2\n v_xor_b32_e32 %0, %0, %1", NOCLOB)
PROBE_KERNEL(k_pair_med3_fma, "v_med3_f32 %0, %0, %1, %2\n v_fma_f32 %0, %0, %1, %2", NOCLOB)

// 32x32 -> 64 multiply-add (the Philox round's multiply): a 64-bit chain
__global__ void k_mad_u64_u32(uint32_t* out, Clocks* clk, uint32_t p, uint32_t q)
{
    uint64_t a[kChains];
    for (int c = 0; c < kChains; ++c) a[c] = (threadIdx.x + 1u) * (2u * c + 3u);
    uint32_t vp = p ^ threadIdx.x, vq = q + threadIdx.x;
    const unsigned long long s0 = __builtin_readcyclecounter();
    const unsigned long long r0 = __builtin_amdgcn_s_memrealtime();
    for (int it = 0; it < kIters; ++it) {
#pragma unroll
        for (int c = 0; c < kChains; ++c)
            asm volatile("v_mad_u64_u32 %0, vcc, %1, %2, %0" : "+v"(a[c]) : "v"(vp), "v"(vq) : "vcc");
    }
    const unsigned long long s1 = __builtin_readcyclecounter();
    const unsigned long long r1 = __builtin_amdgcn_s_memrealtime();
    uint64_t sum = 0;
    for (int c = 0; c < kChains; ++c) sum += a[c];
    out[blockIdx.x * blockDim.x + threadIdx.x] = (uint32_t)sum ^ (uint32_t)(sum >> 32);
    if (threadIdx.x == 0 && blockIdx.x == 0) { clk->shader = s1 - s0; clk->realtime = r1 - r0; }
}

// the Philox round as the kernels run it: two multiplies and two three-input xors
__global__ void k_philox_round(uint32_t* out, Clocks* clk, uint32_t p, uint32_t q)
{
    uint32_t c0[2], c1[2], c2[2], c3[2];
    for (int c = 0; c < 2; ++c) { c0[c] = threadIdx.x + c; c1[c] = p; c2[c] = q; c3[c] = threadIdx.x * 3u + c; }
    const unsigned long long s0 = __builtin_readcyclecounter();
    const unsigned long long r0 = __builtin_amdgcn_s_memrealtime();
    for (int it = 0; it < kIters; ++it) {
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            const uint64_t p0 = (uint64_t)0xD2511F53u * c0[c];
            const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2[c];
            const uint32_t n0 = __builtin_amdgcn_bitop3_b32((uint32_t)(p1 >> 32), c1[c], p, 0x96);
            const uint32_t n2 = __builtin_amdgcn_bitop3_b32((uint32_t)(p0 >> 32), c3[c], q, 0x96);
            c1[c] = (uint32_t)p1; c3[c] = (uint32_t)p0; c0[c] = n0; c2[c] = n2;
        }
    }
    const unsigned long long s1 = __builtin_readcyclecounter();
    const unsigned long long r1 = __builtin_amdgcn_s_memrealtime();
    out[blockIdx.x * blockDim.x + threadIdx.x] = c0[0] ^ c1[0] ^ c2[0] ^ c3[0] ^ c0[1] ^ c1[1] ^ c2[1] ^ c3[1];
    if (threadIdx.x == 0 && blockIdx.x == 0) { clk->shader = s1 - s0; clk->realtime = r1 - r0; }
}

// Dependent issue: ONE chain per lane, every instruction needs the result of the
// one before it.  With one wave per SIMD this is the latency from issue to the
// next dependent issue; with eight waves it shows how far other waves fill the gap.
#define CHAIN_KERNEL(NAME, ASM)                                                           \
    __global__ void NAME(uint32_t* out, Clocks* clk, uint32_t p, uint32_t q)              \
    {                                                                                     \
        uint32_t a = threadIdx.x + 1u;                                                    \
        uint32_t vp = p ^ threadIdx.x, vq = q + threadIdx.x;                              \
        const unsigned long long s0 = __builtin_readcyclecounter();                      \
        const unsigned long long r0 = __builtin_amdgcn_s_memrealtime();                  \
        for (int it = 0; it < kIters; ++it) {                                             \
            _Pragma("unroll") for (int c = 0; c < kChains; ++c)                           \
                asm volatile(ASM : "+v"(a) : "v"(vp), "v"(vq));                           \
        }                                                                                 \
        const unsigned long long s1 = __builtin_readcyclecounter();                      \
        const unsigned long long r1 = __builtin_amdgcn_s_memrealtime();                  \
        out[blockIdx.x * blockDim.x + threadIdx.x] = a;                                   \
        if (threadIdx.x == 0 && blockIdx.x == 0) { clk->shader = s1 - s0; clk->realtime = r1 - r0; } \
    }
CHAIN_KERNEL(c_fma_f32, "v_fma_f32 %0, %0, %1, %2")
CHAIN_KERNEL(c_add_f32, "v_add_f32_e32 %0, %0, %1")
CHAIN_KERNEL(c_bitop3, "v_bitop3_b32 %0, %0, %1, %2 bitop3:0x96")
CHAIN_KERNEL(c_alignbit, "v_alignbit_b32 %0, %0, %1, %2")
CHAIN_KERNEL(c_rndne, "v_rndne_f32_e32 %0, %0")
CHAIN_KERNEL(c_mul_hi, "v_mul_hi_u32 %0, %0, %1")
CHAIN_KERNEL(c_fma_then_bitop3, "v_fma_f32 %0, %0, %1, %2\n v_bitop3_b32 %0, %0, %1, %2 bitop3:0x96")

typedef void (*Kernel)(uint32_t*, Clocks*, uint32_t, uint32_t);

// waves_per_simd: 1 (1,024 one-wave workgroups: one per SIMD) or 8
static void run_chain(const char* name, Kernel k, int per_iter, int waves_per_simd, uint32_t* out, Clocks* clk_d)
{
    const int grid = 1024 * waves_per_simd, block = 64;
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    for (int w = 0; w < 3; ++w) hipLaunchKernelGGL(k, dim3(grid), dim3(block), 0, 0, out, clk_d, 3u, 5u);
    CHECK(hipDeviceSynchronize());
    const int launches = 5;
    CHECK(hipEventRecord(e0));
    for (int w = 0; w < launches; ++w) hipLaunchKernelGGL(k, dim3(grid), dim3(block), 0, 0, out, clk_d, 3u, 5u);
    CHECK(hipEventRecord(e1));
    CHECK(hipEventSynchronize(e1));
    float ms = 0.f;
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    Clocks clk;
    CHECK(hipMemcpy(&clk, clk_d, sizeof(clk), hipMemcpyDeviceToHost));
    const double ghz = clk.realtime ? (double)clk.shader / ((double)clk.realtime * 10.0) : 0.0;
    // per wave: kIters * per_iter dependent instructions, measured by the wave's own cycle counter
    const double cycles_per_instr_in_wave = (double)clk.shader / ((double)kIters * per_iter);
    const double ns = (double)ms / launches * 1e6 / ((double)kIters * per_iter * waves_per_simd);
    printf("%-24s %d wave(s)/SIMD: a wave issues one dependent instruction every %6.2f cycles (its own counter, %5.3f GHz); "
           "SIMD: %6.3f ns per instruction\n", name, waves_per_simd, cycles_per_instr_in_wave, ghz, ns);
    CHECK(hipEventDestroy(e0));
    CHECK(hipEventDestroy(e1));
}

static void run(const char* name, Kernel k, int per_iter, uint32_t* out, Clocks* clk_d)
{
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    for (int w = 0; w < 3; ++w) hipLaunchKernelGGL(k, dim3(kGrid), dim3(kBlockThreads), 0, 0, out, clk_d, 3u, 5u);
    CHECK(hipDeviceSynchronize());
    const int launches = 5;
    CHECK(hipEventRecord(e0));
    for (int w = 0; w < launches; ++w) hipLaunchKernelGGL(k, dim3(kGrid), dim3(kBlockThreads), 0, 0, out, clk_d, 3u, 5u);
    CHECK(hipEventRecord(e1));
    CHECK(hipEventSynchronize(e1));
    float ms = 0.f;
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    Clocks clk;
    CHECK(hipMemcpy(&clk, clk_d, sizeof(clk), hipMemcpyDeviceToHost));
    const double ghz = clk.realtime ? (double)clk.shader / ((double)clk.realtime * 10.0) : 0.0;   // 100 MHz counter
    const double wave_instr_per_simd = (double)kGrid * (kBlockThreads / 64) * kIters * per_iter / 1024.0;
    const double ns = (double)ms / launches * 1e6 / wave_instr_per_simd;
    printf("%-24s %7.3f ns per wave64 instruction per SIMD   shader clock %5.3f GHz   %5.2f cycles at that clock   %5.2f at 2.4 GHz\n",
           name, ns, ghz, ns * ghz, ns * 2.4);
    CHECK(hipEventDestroy(e0));
    CHECK(hipEventDestroy(e1));
}

int main()
{
    uint32_t* out;
    Clocks* clk_d;
    CHECK(hipMalloc(&out, (size_t)kGrid * kBlockThreads * sizeof(uint32_t)));
    CHECK(hipMalloc(&clk_d, sizeof(Clocks)));
    // some hundred milliseconds of load first: the clock settles only after that
    for (int w = 0; w < 400; ++w) hipLaunchKernelGGL(k_fma_f32, dim3(kGrid), dim3(kBlockThreads), 0, 0, out, clk_d, 3u, 5u);
    CHECK(hipDeviceSynchronize());
#define RUN1(k) run(#k, k, kChains, out, clk_d)
#define RUN2(k) run(#k, k, 2 * kChains, out, clk_d)
    RUN1(k_mov); RUN1(k_add_f32); RUN1(k_sub_f32); RUN1(k_mul_f32); RUN1(k_fma_f32); RUN1(k_fmac_f32);
    RUN1(k_add_u32); RUN1(k_and_b32); RUN1(k_xor_b32); RUN1(k_bitop3); RUN1(k_and_or); RUN1(k_or3); RUN1(k_bfi);
    RUN1(k_mul_u32_u24); RUN1(k_mad_u32_u24); RUN1(k_perm); RUN1(k_or_sdwa_w1); RUN1(k_cndmask); RUN1(k_cmp_lt_f32);
    RUN1(k_rndne_f32); RUN1(k_floor_f32); RUN1(k_cvt_f32_u32); RUN1(k_cvt_f32_u32_sdwa_w1); RUN1(k_cvt_f32_ubyte0);
    RUN1(k_cvt_u32_f32); RUN1(k_cvt_i32_f32); RUN1(k_max_f32); RUN1(k_min_f32); RUN1(k_med3_f32); RUN1(k_max_u32);
    RUN1(k_pk_max_u16); RUN1(k_lshlrev_b32); RUN1(k_lshrrev_b32); RUN1(k_bfe_u32); RUN1(k_lshl_or); RUN1(k_lshl_add);
    RUN1(k_alignbit); RUN1(k_add3_u32); RUN1(k_mul_lo_u32); RUN1(k_mul_hi_u32); RUN1(k_rcp_f32);
    run("k_mad_u64_u32", k_mad_u64_u32, kChains, out, clk_d);
    run("k_philox_round(2mad+2xor3)", k_philox_round, 2 * 4, out, clk_d);
    RUN2(k_pair_fma_fma); RUN2(k_pair_fma_xor); RUN2(k_pair_rndne_add); RUN2(k_pair_rndne_xor); RUN2(k_pair_cvt_fma);
    RUN2(k_pair_alignbit_fma); RUN2(k_pair_alignbit_xor); RUN2(k_pair_med3_fma);
    for (int waves : {1, 2, 4, 8}) {
        run_chain("c_fma_f32", c_fma_f32, kChains, waves, out, clk_d);
        run_chain("c_add_f32", c_add_f32, kChains, waves, out, clk_d);
        run_chain("c_bitop3", c_bitop3, kChains, waves, out, clk_d);
        run_chain("c_alignbit", c_alignbit, kChains, waves, out, clk_d);
        run_chain("c_rndne", c_rndne, kChains, waves, out, clk_d);
        run_chain("c_mul_hi", c_mul_hi, kChains, waves, out, clk_d);
        run_chain("c_fma_then_bitop3", c_fma_then_bitop3, 2 * kChains, waves, out, clk_d);
    }
    CHECK(hipFree(out));
    CHECK(hipFree(clk_d));
    return 0;
}
