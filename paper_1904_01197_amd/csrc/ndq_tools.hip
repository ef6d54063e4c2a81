// libndq, beyond the headline path (gfx950): entropy of an index stream, dense
// base-L stream, sigma_z^2 estimate and Thm 4's parameter helpers, size rules and
// status text.  See include/ndq.h for the contract.
#include <hip/hip_runtime.h>

#include <math.h>

#include <mutex>

#include "ndq.h"
#include "ndq_device.hpp"
#include "ndq_host.hpp"

namespace ndq {

// ---------------------------------------------------------------------------
// Histogram and entropy of an index stream (Sec. 4: the bit rate after entropy
// coding is reported through the entropy of the transmitted indices).
// Few, large workgroups in both kernels: every workgroup ends with one atomic per
// bin on the same few addresses, and those serialize.
//
// Codes of 3 to 8 bits: a thread reads units of 32 codes (= BITS consecutive
// 32-bit words, the next unit already in flight) and takes the codes out with
// shifts known at compile time.  Counting: 32 copies of the workgroup's histogram
// in LDS, a lane adding to copy (lane mod 32) -- the word index is
// code * 32 + copy, so the 32 lanes that LDS serves together always fall into 32
// different banks, whatever the distribution of the codes (index streams are
// heavily peaked); the two halves of a wave are served one after the other anyway.
// ---------------------------------------------------------------------------
constexpr uint32_t kHistThreads = 1024;
constexpr uint32_t kHistBlocks = 256;
constexpr uint32_t kHistCopies = 32;

// The workgroup that finishes last closes the histogram inside the counting kernel
// (no launch of its own): it fills in a bin that was left to be derived and computes
// the entropy.  `ticket` is a 64-bit word that is zero when the kernel starts.
// Every thread calls this after its last atomic on the histogram.  The barrier makes
// every wave wait until its atomics are done; one thread's fence then orders them
// before the workgroup's ticket (a fence per thread would write back and invalidate
// the L2 sixteen times per workgroup while the others still stream through it).  The
// workgroup that draws the last ticket therefore finds all counts in memory; it reads
// them with atomics of device scope, like the additions that made them.
__device__ __forceinline__ bool last_workgroup(unsigned long long* ticket, uint32_t* flag)
{
    __syncthreads();
    if (threadIdx.x == 0u) {
        __threadfence();
        *flag = atomicAdd(ticket, 1ull) == (unsigned long long)gridDim.x - 1ull ? 1u : 0u;
        __threadfence();
    }
    __syncthreads();
    return *flag != 0u;
}

// -sum p log2 p over at most 256 bins, binary64, fixed reduction order; called by all
// threads of one workgroup of at least 256 threads.  derive_bin0 (at most 4 bins):
// bin 0 was not counted and is what the other bins leave of n.
__device__ __forceinline__ void close_histogram(unsigned long long* hist, uint32_t nbins, uint64_t n,
                                                double* entropy_out, bool derive_bin0, double* term,
                                                unsigned long long* few)
{
    const uint32_t tid = threadIdx.x;
    unsigned long long h = 0ull;
    if (tid < nbins && !(derive_bin0 && tid == 0u))
        h = __hip_atomic_load(hist + tid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (derive_bin0) {
        if (tid >= 1u && tid < nbins) few[tid] = h;
        __syncthreads();
        if (tid == 0u) {
            unsigned long long rest = n;
            for (uint32_t b = 1; b < nbins; ++b) rest -= few[b];
            hist[0] = rest;
            h = rest;
        }
    }
    if (!entropy_out) return;     // (the same for every thread)
    double t = 0.0;
    if (tid < nbins && h) {
        const double p = (double)h / (double)n;
        t = -p * log2(p);
    }
    if (tid < 256u) term[tid] = t;
    __syncthreads();
    for (uint32_t s = 128; s >= 1; s >>= 1) {
        if (tid < s) term[tid] += term[tid + s];
        __syncthreads();
    }
    if (tid == 0u) entropy_out[0] = term[0];
}

template <int BITS>
__device__ __forceinline__ void load_unit(const uint32_t* __restrict__ words, uint64_t u, uint32_t (&w)[BITS])
{
    const uint32_t* p = words + u * BITS;
    if constexpr (BITS % 4 == 0) {      // 16-byte aligned: the stream is, and so is every unit
#pragma unroll
        for (int k = 0; k < BITS / 4; ++k) {
            const uint4 x = reinterpret_cast<const uint4*>(p)[k];
            w[4 * k] = x.x; w[4 * k + 1] = x.y; w[4 * k + 2] = x.z; w[4 * k + 3] = x.w;
        }
    } else {
#pragma unroll
        for (int k = 0; k < BITS; ++k) w[k] = p[k];
    }
}

template <int BITS>
__global__ __launch_bounds__(kHistThreads) void histogram_kernel(const uint32_t* __restrict__ words, uint64_t n,
                                                                 unsigned long long* hist, double* entropy_out)
{
    constexpr uint32_t NB = 1u << BITS;
    constexpr uint32_t MASK = NB - 1u;
    __shared__ uint32_t cnt[NB * kHistCopies];
    __shared__ double term[256];
    __shared__ uint32_t flag;
    const uint32_t tid = threadIdx.x;
    for (uint32_t i = tid; i < NB * kHistCopies; i += kHistThreads) cnt[i] = 0u;
    __syncthreads();

    const uint32_t copy = tid & (kHistCopies - 1u);
    const uint64_t units = n >> 5;                  // whole units; the last n mod 32 codes below
    const uint64_t stride = (uint64_t)gridDim.x * kHistThreads;
    uint64_t u = (uint64_t)blockIdx.x * kHistThreads + tid;
    uint32_t w[BITS], ahead[BITS];
    if (u < units) load_unit<BITS>(words, u, w);
    while (u < units) {
        const uint64_t un = u + stride;
        if (un < units) load_unit<BITS>(words, un, ahead);
#pragma unroll
        for (int j = 0; j < 32; ++j) {
            const int bit = j * BITS, k = bit >> 5, sh = bit & 31;
            uint32_t code = w[k] >> sh;
            if (sh + BITS > 32) code |= w[k + 1] << (32 - sh);
            atomicAdd(&cnt[(code & MASK) * kHistCopies + copy], 1u);     // result unused: a plain LDS add
        }
#pragma unroll
        for (int k = 0; k < BITS; ++k) w[k] = ahead[k];
        u = un;
    }
    const uint32_t rest = (uint32_t)(n & 31u);
    if (blockIdx.x == 0 && tid < rest) {
        // one code per thread; a code that crosses into the next word is a valid code,
        // so that word lies inside the stream
        const uint64_t bit = ((units << 5) + tid) * BITS;
        const uint64_t k = bit >> 5;
        const uint32_t sh = (uint32_t)(bit & 31u);
        uint32_t code = words[k] >> sh;
        if (sh + BITS > 32u) code |= words[k + 1] << (32u - sh);
        atomicAdd(&cnt[(code & MASK) * kHistCopies + copy], 1u);
    }
    __syncthreads();
    for (uint32_t b = tid; b < NB; b += kHistThreads) {
        unsigned long long sum = 0u;
        for (uint32_t c = 0; c < kHistCopies; ++c) sum += cnt[b * kHistCopies + ((c + b) & (kHistCopies - 1u))];
        if (sum) atomicAdd(hist + b, sum);
    }
    // the entropy's eight bytes hold the ticket until the last workgroup writes the entropy there
    if (entropy_out && last_workgroup(reinterpret_cast<unsigned long long*>(entropy_out), &flag))
        close_histogram(hist, NB, n, entropy_out, false, term, nullptr);
}

// 1- and 2-bit codes: a thread takes 16 bytes (128 or 64 codes) at a time, eight
// such loads in flight, and counts with population counts.  Few, large workgroups
// (at most kSmallBlocks of kSmallThreads), because every workgroup ends with one
// atomic per bin on the same few addresses and those serialize.  A thread sees at
// most n / 2^18 + 1024 codes (n < 2^40), a wave 64 times that: 32-bit counts up to
// the wave's sum, 64-bit ones across waves.
constexpr uint32_t kSmallBlocks = 256;
constexpr uint32_t kSmallThreads = 1024;
constexpr int kSmallInFlight = 8;

template <int BITS>
__device__ __forceinline__ void count_small(uint32_t w, uint32_t& c1, uint32_t& c2, uint32_t& c3)
{
    if (BITS == 1) {
        c1 += __builtin_popcount(w);
    } else {
        const uint32_t lo = w & 0x55555555u, hi = (w >> 1) & 0x55555555u;
        c1 += __builtin_popcount(lo & ~hi);
        c2 += __builtin_popcount(hi & ~lo);
        c3 += __builtin_popcount(lo & hi);
    }
}

template <int BITS>
__device__ __forceinline__ void count_small(const uint4& x, uint32_t& c1, uint32_t& c2, uint32_t& c3)
{
    count_small<BITS>(x.x, c1, c2, c3); count_small<BITS>(x.y, c1, c2, c3);
    count_small<BITS>(x.z, c1, c2, c3); count_small<BITS>(x.w, c1, c2, c3);
}

// (the code width is a template parameter: as a run-time value it put a branch around every
// word's counting, and the loop then waited for all its loads before the first count)
template <int BITS>
__global__ __launch_bounds__(kSmallThreads) void histogram_small_kernel(const uint4* __restrict__ vec, uint64_t n,
                                                                        unsigned long long* hist,
                                                                        double* entropy_out)
{
    constexpr uint32_t bits = BITS;
    __shared__ uint32_t part[3][kSmallThreads / 64];
    __shared__ double term[256];
    __shared__ unsigned long long few[4];
    __shared__ uint32_t flag;
    const uint32_t tid = threadIdx.x;
    // whole 16-byte vectors here; the last, partial one (the stream is allocated in
    // multiples of 16 bytes) is masked to its valid bits below.  Bits masked away
    // read as code 0, and bin 0 is n minus the other bins anyway.
    const uint64_t vectors = (n * bits) >> 7;
    const uint64_t stride = (uint64_t)gridDim.x * kSmallThreads;
    uint32_t c[3] = {0u, 0u, 0u};
    uint64_t u = (uint64_t)blockIdx.x * kSmallThreads + tid;
    for (; u + (kSmallInFlight - 1) * stride < vectors; u += kSmallInFlight * stride) {
        uint4 x[kSmallInFlight];
#pragma unroll
        for (int j = 0; j < kSmallInFlight; ++j) x[j] = vec[u + (uint64_t)j * stride];
#pragma unroll
        for (int j = 0; j < kSmallInFlight; ++j) count_small<BITS>(x[j], c[0], c[1], c[2]);
    }
    for (; u < vectors; u += stride) count_small<BITS>(vec[u], c[0], c[1], c[2]);
    const uint32_t tail_bits = (uint32_t)((n * bits) & 127u);
    if (blockIdx.x == 0 && tid == 0 && tail_bits != 0u) {
        const uint4 x = vec[vectors];
        const uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
        for (uint32_t j = 0; j < 4u; ++j) {
            const uint32_t have = tail_bits > 32u * j ? tail_bits - 32u * j : 0u;
            const uint32_t mask = have >= 32u ? 0xffffffffu : ((1u << have) - 1u);
            count_small<BITS>(w[j] & mask, c[0], c[1], c[2]);
        }
    }
#pragma unroll
    for (int b = 0; b < 3; ++b) {
        for (int off = 32; off >= 1; off >>= 1) c[b] += __shfl_down(c[b], off, 64);
        if ((tid & 63u) == 0u) part[b][tid >> 6] = c[b];
    }
    __syncthreads();
    // bins 1..3 (or bin 1) by atomics; bin 0 is not counted: its eight bytes hold the
    // ticket, and the last workgroup writes there what the other bins leave of n
    const uint32_t nbins = 1u << bits;
    if (tid >= 1u && tid < nbins) {
        unsigned long long sum = 0u;
        for (uint32_t w = 0; w < kSmallThreads / 64u; ++w) sum += part[tid - 1u][w];
        if (sum) atomicAdd(hist + tid, sum);
    }
    if (last_workgroup(hist, &flag)) close_histogram(hist, nbins, n, entropy_out, true, term, few);
}

// clears the bins and, when an entropy is wanted, its eight bytes (+0.0: the entropy of
// an empty stream, and the zero the ticket starts from)
__global__ void clear_histogram_kernel(unsigned long long* hist, uint32_t nbins, unsigned long long* entropy_bits)
{
    if (threadIdx.x < nbins) hist[threadIdx.x] = 0ull;
    if (threadIdx.x == 0u && entropy_bits) entropy_bits[0] = 0ull;
}

// ---------------------------------------------------------------------------
// Dense base-L stream (Sec. 4 Table 1 counts log2 L bits per index): k indices
// per 32-bit word as the number sum_j c_j L^j.  Transcoders between the
// fixed-width stream and the dense one.  A thread owns 8 dense words = 8k
// indices = k*bits whole bytes of the fixed-width stream, so no two threads
// share a byte.
// ---------------------------------------------------------------------------
struct DenseArgs {
    unsigned char* fixed;     // fixed-width stream (read by pack, written by unpack)
    uint32_t* dense;          // dense stream (written by pack, read by unpack)
    uint64_t n;               // indices
    uint64_t fixed_total;     // its padded size
    uint64_t dense_valid;     // ceil(n/k) words that hold indices
    uint64_t dense_total;     // padded size in words
    uint32_t levels, k, bits;
    // division of a 32-bit number by `levels` through one high multiply (division by
    // an invariant integer, round-up method): with l = ceil(log2 levels) and
    // magic = floor(2^32 (2^l - levels) / levels) + 1, for every 32-bit x
    // x / levels = (t + ((x - t) >> 1)) >> (l - 1), t = high word of x * magic
    uint32_t magic, shift;
};

__device__ __forceinline__ uint32_t divide_by_levels(uint32_t x, const DenseArgs& a)
{
    const uint32_t t = __umulhi(x, a.magic);
    return (t + ((x - t) >> 1)) >> a.shift;
}

// Both transcoders stage a workgroup's share of the two streams in LDS: a thread's
// bytes lie k*bits (at most kDenseThreadBytes) apart from its neighbour's, so direct
// byte accesses would each be a memory transaction of their own; the workgroup's
// share is contiguous and moves as whole 32-bit words instead.
constexpr uint32_t kDenseThreadBytes = 40;     // max of k * bits over levels 2..256
constexpr uint32_t kDenseBlock = 256;
constexpr uint32_t kDenseWordsPerThread = 8;

struct DenseStage {
    uint32_t dense[kDenseBlock * kDenseWordsPerThread];
    uint32_t fixed[kDenseBlock * kDenseThreadBytes / 4];
};

// bytes of the fixed-width stream that belong to this workgroup (a multiple of 4:
// its first byte is a multiple of 256 and the stream's size one of 16)
__device__ __forceinline__ uint32_t dense_block_bytes(const DenseArgs& a, uint64_t block_byte0)
{
    const uint64_t share = (uint64_t)kDenseBlock * a.k * a.bits;
    if (block_byte0 >= a.fixed_total) return 0u;
    const uint64_t left = a.fixed_total - block_byte0;
    return (uint32_t)(left < share ? left : share);
}

__global__ __launch_bounds__(kDenseBlock) void dense_pack_kernel(DenseArgs a)
{
    __shared__ DenseStage st;
    const uint32_t tid = threadIdx.x;
    const uint32_t thread_bytes = a.k * a.bits;
    const uint64_t block_byte0 = (uint64_t)blockIdx.x * kDenseBlock * thread_bytes;
    const uint64_t block_w0 = (uint64_t)blockIdx.x * kDenseBlock * kDenseWordsPerThread;
    const uint32_t words_in = dense_block_bytes(a, block_byte0) / 4u;
    const uint32_t* fixed32 = reinterpret_cast<const uint32_t*>(a.fixed + block_byte0);
    for (uint32_t i = tid; i < kDenseBlock * thread_bytes / 4u; i += kDenseBlock)
        st.fixed[i] = i < words_in ? fixed32[i] : 0u;
    __syncthreads();
    const unsigned char* mine = reinterpret_cast<const unsigned char*>(st.fixed) + tid * thread_bytes;
    const uint32_t mask = (1u << a.bits) - 1u;
    uint32_t buf = 0u, have = 0u, byte = 0u;
    for (uint32_t j = 0; j < kDenseWordsPerThread; ++j) {
        const uint64_t w = block_w0 + tid * kDenseWordsPerThread + j;
        // sum_j c_j L^j <= L^k - 1 < 2^32; the weight may wrap after the last digit, unused
        uint32_t value = 0u, weight = 1u;
        for (uint32_t d = 0; d < a.k; ++d) {
            if (have < a.bits) {
                buf |= (uint32_t)mine[byte++] << have;
                have += 8u;
            }
            uint32_t c = buf & mask;
            buf >>= a.bits;
            have -= a.bits;
            if (w * a.k + d >= a.n) c = 0u;      // also hides whatever the padding holds
            value += c * weight;
            weight *= a.levels;
        }
        st.dense[tid * kDenseWordsPerThread + j] = value;
    }
    __syncthreads();
    for (uint32_t i = tid; i < kDenseBlock * kDenseWordsPerThread; i += kDenseBlock)
        if (block_w0 + i < a.dense_total) a.dense[block_w0 + i] = st.dense[i];
}

__global__ __launch_bounds__(kDenseBlock) void dense_unpack_kernel(DenseArgs a)
{
    __shared__ DenseStage st;
    const uint32_t tid = threadIdx.x;
    const uint32_t thread_bytes = a.k * a.bits;
    const uint64_t block_byte0 = (uint64_t)blockIdx.x * kDenseBlock * thread_bytes;
    const uint64_t block_w0 = (uint64_t)blockIdx.x * kDenseBlock * kDenseWordsPerThread;
    for (uint32_t i = tid; i < kDenseBlock * kDenseWordsPerThread; i += kDenseBlock)
        st.dense[i] = block_w0 + i < a.dense_valid ? a.dense[block_w0 + i] : 0u;
    __syncthreads();
    unsigned char* mine = reinterpret_cast<unsigned char*>(st.fixed) + tid * thread_bytes;
    uint32_t buf = 0u, have = 0u, byte = 0u;
    for (uint32_t j = 0; j < kDenseWordsPerThread; ++j) {
        const uint64_t w = block_w0 + tid * kDenseWordsPerThread + j;
        uint32_t value = st.dense[tid * kDenseWordsPerThread + j];
        for (uint32_t d = 0; d < a.k; ++d) {
            const uint32_t q = divide_by_levels(value, a);
            uint32_t c = value - q * a.levels;
            value = q;
            if (w * a.k + d >= a.n) c = 0u;
            buf |= c << have;
            have += a.bits;
            if (have >= 8u) {
                mine[byte++] = (unsigned char)buf;
                buf >>= 8;
                have -= 8u;
            }
        }
    }
    // 8 k bits per thread are whole bytes: nothing is left in buf
    __syncthreads();
    const uint32_t words_out = dense_block_bytes(a, block_byte0) / 4u;
    uint32_t* fixed32 = reinterpret_cast<uint32_t*>(a.fixed + block_byte0);
    for (uint32_t i = tid; i < words_out; i += kDenseBlock) fixed32[i] = st.fixed[i];
}

// The level counts of the paper's own experiments (Sec. 4: three levels, M = 1, and five,
// M = 2) with everything known at compile time: the same partition as above (a thread
// owns 8 dense words = 8 K indices = TB = K * BITS bytes of the fixed-width stream), but
// the thread's bytes sit in registers as one bit string, every index at a fixed
// position, the digits come and go with constant multipliers, and both streams move
// between memory and LDS sixteen bytes at a time.
template <uint32_t L, uint32_t K, uint32_t BITS> struct DenseFixed {
    static constexpr uint32_t TB = K * BITS;                       // a thread's bytes of the fixed-width stream
    static constexpr uint32_t NX = (TB + 3u) / 4u;                 // as 32-bit words
    static constexpr uint32_t NR = TB % 4u == 0u ? NX : TB / 4u + 2u;   // aligned words that cover them at any offset
    static constexpr uint32_t FIXED_WORDS = kDenseBlock * TB / 4u;  // per workgroup (256 * TB is a multiple of 16)
    static constexpr uint32_t DENSE_WORDS = kDenseBlock * kDenseWordsPerThread;
    static_assert(TB <= kDenseThreadBytes && FIXED_WORDS % 4u == 0u, "partition");
};

// keeps the first `valid_bits` bits of a bit string held in NX words
template <uint32_t NX>
__device__ __forceinline__ void keep_bits(uint32_t (&x)[NX], uint32_t valid_bits)
{
#pragma unroll
    for (uint32_t i = 0; i < NX; ++i) {
        const uint32_t have = valid_bits > 32u * i ? valid_bits - 32u * i : 0u;
        x[i] &= have >= 32u ? 0xffffffffu : ((1u << have) - 1u);
    }
}

// bits of the thread's share that belong to indices below n
template <uint32_t K, uint32_t BITS>
__device__ __forceinline__ uint32_t dense_valid_bits(const DenseArgs& a, uint64_t first_word)
{
    const uint64_t first = first_word * K;
    if (first >= a.n) return 0u;
    const uint64_t left = a.n - first;
    return left >= 8u * K ? 8u * K * BITS : (uint32_t)left * BITS;
}

template <uint32_t L, uint32_t K, uint32_t BITS>
__global__ __launch_bounds__(kDenseBlock) void dense_pack_fixed_kernel(DenseArgs a)
{
    using D = DenseFixed<L, K, BITS>;
    __shared__ __align__(16) DenseStage st;
    const uint32_t tid = threadIdx.x;
    const uint64_t block_byte0 = (uint64_t)blockIdx.x * kDenseBlock * D::TB;
    const uint64_t block_w0 = (uint64_t)blockIdx.x * D::DENSE_WORDS;
    const uint32_t vectors_in = dense_block_bytes(a, block_byte0) / 16u;
    const uint4* fixed128 = reinterpret_cast<const uint4*>(a.fixed + block_byte0);
    uint4* stage128 = reinterpret_cast<uint4*>(st.fixed);
    for (uint32_t i = tid; i < D::FIXED_WORDS / 4u; i += kDenseBlock)
        stage128[i] = i < vectors_in ? fixed128[i] : make_uint4(0u, 0u, 0u, 0u);
    __syncthreads();

    // the thread's TB bytes, from the aligned words around them
    const uint32_t byte0 = tid * D::TB;
    uint32_t r[D::NR], x[D::NX];
#pragma unroll
    for (uint32_t i = 0; i < D::NR; ++i) {
        const uint32_t w = byte0 / 4u + i;
        r[i] = w < D::FIXED_WORDS ? st.fixed[w] : 0u;
    }
    if constexpr (D::TB % 4u == 0u) {
#pragma unroll
        for (uint32_t i = 0; i < D::NX; ++i) x[i] = r[i];
    } else {
#pragma unroll
        for (uint32_t i = 0; i < D::NX; ++i) x[i] = __builtin_amdgcn_alignbyte(r[i + 1], r[i], byte0 & 3u);
    }
    // indices at or beyond n count as digit 0, whatever the padding holds
    keep_bits<D::NX>(x, dense_valid_bits<K, BITS>(a, block_w0 + (uint64_t)tid * kDenseWordsPerThread));

    uint32_t value[kDenseWordsPerThread];
#pragma unroll
    for (uint32_t j = 0; j < kDenseWordsPerThread; ++j) {
        uint32_t v = 0u;
#pragma unroll
        for (int d = (int)K - 1; d >= 0; --d) {       // sum_d c_d L^d, highest digit first
            constexpr uint32_t MASK = (1u << BITS) - 1u;
            const uint32_t bit = (j * K + (uint32_t)d) * BITS, k = bit >> 5, sh = bit & 31u;
            uint32_t c = x[k] >> sh;
            if (sh + BITS > 32u) c |= x[k + 1] << (32u - sh);
            v = v * L + (c & MASK);
        }
        value[j] = v;
    }
    uint4* mine = reinterpret_cast<uint4*>(st.dense + tid * kDenseWordsPerThread);
    mine[0] = make_uint4(value[0], value[1], value[2], value[3]);
    mine[1] = make_uint4(value[4], value[5], value[6], value[7]);
    __syncthreads();
    const uint4* out128 = reinterpret_cast<const uint4*>(st.dense);
    uint4* dense128 = reinterpret_cast<uint4*>(a.dense + block_w0);
    for (uint32_t i = tid; i < D::DENSE_WORDS / 4u; i += kDenseBlock)
        if (block_w0 + 4u * i < a.dense_total) dense128[i] = out128[i];      // dense_total is a multiple of 4
}

template <uint32_t L, uint32_t K, uint32_t BITS>
__global__ __launch_bounds__(kDenseBlock) void dense_unpack_fixed_kernel(DenseArgs a)
{
    using D = DenseFixed<L, K, BITS>;
    __shared__ __align__(16) DenseStage st;
    const uint32_t tid = threadIdx.x;
    const uint64_t block_byte0 = (uint64_t)blockIdx.x * kDenseBlock * D::TB;
    const uint64_t block_w0 = (uint64_t)blockIdx.x * D::DENSE_WORDS;
    const uint4* dense128 = reinterpret_cast<const uint4*>(a.dense + block_w0);
    uint4* in128 = reinterpret_cast<uint4*>(st.dense);
    for (uint32_t i = tid; i < D::DENSE_WORDS / 4u; i += kDenseBlock)
        in128[i] = block_w0 + 4u * i < a.dense_total ? dense128[i] : make_uint4(0u, 0u, 0u, 0u);
    __syncthreads();

    const uint4* mine = reinterpret_cast<const uint4*>(st.dense + tid * kDenseWordsPerThread);
    const uint4 lo4 = mine[0], hi4 = mine[1];
    const uint32_t value[kDenseWordsPerThread] = {lo4.x, lo4.y, lo4.z, lo4.w, hi4.x, hi4.y, hi4.z, hi4.w};
    uint32_t x[D::NX];
#pragma unroll
    for (uint32_t i = 0; i < D::NX; ++i) x[i] = 0u;
    auto put = [&](uint32_t index, uint32_t c) __attribute__((always_inline)) {
        const uint32_t bit = index * BITS, k = bit >> 5, sh = bit & 31u;
        x[k] |= c << sh;
        if (sh + BITS > 32u) x[k + 1] |= c >> (32u - sh);
    };
#pragma unroll
    for (uint32_t j = 0; j < kDenseWordsPerThread; ++j) {
        if constexpr (L == 3u && K == 20u) {
            // two halves of ten digits, each below 3^10 < 2^16, taken two digits at a time:
            // y / 9 = (y * 58255) >> 19 exactly for y < 2^16, and for the remainder r in 0..8
            // the two codes c0 + 4 c1 = r + r / 3 with r / 3 = (r * 11) >> 5.  All factors lie
            // below 2^24 and the products fit 32 bits, which the compiler sees: it picks
            // the multiplies of the fast 24-bit kind.
            const uint32_t top = value[j] / 59049u;
            uint32_t half[2] = {value[j] - top * 59049u, top};
#pragma unroll
            for (uint32_t h = 0; h < 2u; ++h) {
                uint32_t y = half[h] & 0xffffu;       // (a word that is not a valid number stays in range)
#pragma unroll
                for (uint32_t d = 0; d < 10u; d += 2u) {
                    const uint32_t q = (y * 58255u) >> 19;
                    const uint32_t r = y - q * 9u;
                    put(j * K + 10u * h + d, r + ((r * 11u) >> 5));     // an even index: four bits inside one word
                    y = q;
                }
            }
        } else {
            uint32_t v = value[j];
#pragma unroll
            for (uint32_t d = 0; d < K; ++d) {
                const uint32_t q = v / L;
                put(j * K + d, v - q * L);
                v = q;
            }
        }
    }
    keep_bits<D::NX>(x, dense_valid_bits<K, BITS>(a, block_w0 + (uint64_t)tid * kDenseWordsPerThread));

    const uint32_t byte0 = tid * D::TB;
    if constexpr (D::TB % 4u == 0u) {
#pragma unroll
        for (uint32_t i = 0; i < D::NX; ++i) st.fixed[byte0 / 4u + i] = x[i];
    } else {
        unsigned char* bytes = reinterpret_cast<unsigned char*>(st.fixed) + byte0;
#pragma unroll
        for (uint32_t b = 0; b < D::TB; ++b) bytes[b] = (unsigned char)(x[b / 4u] >> (8u * (b & 3u)));
    }
    __syncthreads();
    const uint32_t vectors_out = dense_block_bytes(a, block_byte0) / 16u;
    const uint4* stage128 = reinterpret_cast<const uint4*>(st.fixed);
    uint4* fixed128 = reinterpret_cast<uint4*>(a.fixed + block_byte0);
    for (uint32_t i = tid; i < vectors_out; i += kDenseBlock) fixed128[i] = stage128[i];
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

// Partial sums of ndq_sqdiff_static: one per workgroup of the first pass, in
// memory the library owns (8 KB on every GPU it runs on, until the process ends).
// In host code this name is only a handle for hipGetSymbolAddress; the kernels get
// the per-device address kept in g_scratch_ptr.
static __device__ __align__(256) double scratch[kSqBlocks];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static double* g_scratch_ptr[kMaxDevices];   // address of `scratch` on each device, looked up once

// Address of `scratch` on the current device (null: the runtime refused).
static double* scratch_on_current_device()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = (double*)p;
    }
    return g_scratch_ptr[dev];
}

// Argument checks and the two launches shared by ndq_sqdiff and ndq_sqdiff_static.
static int sqdiff_common(const float* a, const float* b, size_t n, double* partial, double* out,
                         void* stream)
{
    if (!out) return NDQ_EINVAL;
    if (n != 0 && (!a || !b)) return NDQ_EINVAL;
    if (n >= kMaxN) return NDQ_EUNSUPPORTED;
    if (((uintptr_t)partial & 7u) || ((uintptr_t)out & 7u)) return NDQ_EALIGN;
    if (n != 0 && (!aligned16(a) || !aligned16(b))) return NDQ_EALIGN;
    hipStream_t s = (hipStream_t)stream;
    if (launch(sqdiff_partial_kernel, dim3(kSqBlocks), dim3(256), s, a, b, (uint64_t)n, partial) != NDQ_OK)
        return NDQ_ELAUNCH;
    return launch(sqdiff_final_kernel, dim3(1), dim3(256), s, (const double*)partial, out);
}

}  // namespace ndq

extern "C" {

uint32_t ndq_code_bits(uint32_t levels_or_M) { return ndq::code_bits(levels_or_M); }

size_t ndq_packed_bytes(size_t n, uint32_t bits) { return ndq::packed_bytes(n, bits); }

size_t ndq_num_buckets(size_t n, uint32_t bucket)
{
    return bucket ? (n + bucket - 1u) / bucket : 1u;
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
    if (launch(clear_histogram_kernel, dim3(1), dim3(256), s, (unsigned long long*)hist_out, nbins,
               (unsigned long long*)entropy_out) != NDQ_OK)
        return NDQ_ELAUNCH;
    if (n == 0) return NDQ_OK;
    if (bits <= 2u) {
        const uint64_t vectors = ((uint64_t)n * bits) >> 7;
        uint64_t blocks = (vectors + kSmallInFlight * kSmallThreads - 1) / (kSmallInFlight * kSmallThreads);
        if (blocks > kSmallBlocks) blocks = kSmallBlocks;
        if (blocks == 0u) blocks = 1u;
        if (bits == 1u)
            return launch(histogram_small_kernel<1>, dim3((uint32_t)blocks), dim3(kSmallThreads), s,
                          (const uint4*)codes, (uint64_t)n, (unsigned long long*)hist_out, entropy_out);
        return launch(histogram_small_kernel<2>, dim3((uint32_t)blocks), dim3(kSmallThreads), s,
                      (const uint4*)codes, (uint64_t)n, (unsigned long long*)hist_out, entropy_out);
    }
    const uint64_t units = (uint64_t)n >> 5;
    uint64_t blocks = (units + kHistThreads - 1) / kHistThreads;
    if (blocks > kHistBlocks) blocks = kHistBlocks;
    if (blocks == 0u) blocks = 1u;
    const dim3 grid((uint32_t)blocks), block(kHistThreads);
    const uint32_t* words = (const uint32_t*)codes;
    unsigned long long* h = (unsigned long long*)hist_out;
    switch (bits) {
    case 3: return launch(histogram_kernel<3>, grid, block, s, words, (uint64_t)n, h, entropy_out);
    case 4: return launch(histogram_kernel<4>, grid, block, s, words, (uint64_t)n, h, entropy_out);
    case 5: return launch(histogram_kernel<5>, grid, block, s, words, (uint64_t)n, h, entropy_out);
    case 6: return launch(histogram_kernel<6>, grid, block, s, words, (uint64_t)n, h, entropy_out);
    case 7: return launch(histogram_kernel<7>, grid, block, s, words, (uint64_t)n, h, entropy_out);
    default: return launch(histogram_kernel<8>, grid, block, s, words, (uint64_t)n, h, entropy_out);
    }
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
    a.shift = a.bits - 1u;      // bits = ceil(log2 levels) >= 1
    a.magic = (uint32_t)((((uint64_t)1 << 32) * (((uint64_t)1 << a.bits) - levels)) / levels + 1u);
    a.fixed_total = packed_bytes(n, a.bits);
    a.dense_valid = ((uint64_t)n + a.k - 1u) / a.k;
    a.dense_total = ndq_dense_bytes(n, levels) / 4u;
    const uint64_t per_thread_bytes = (uint64_t)a.k * a.bits;
    const uint64_t threads = pack ? (a.dense_total + 7u) / 8u
                                  : (a.fixed_total + per_thread_bytes - 1u) / per_thread_bytes;
    const uint64_t blocks = (threads + 255u) / 256u;
    if (blocks >= ((uint64_t)1 << 31)) return NDQ_EUNSUPPORTED;
    if (per_thread_bytes > kDenseThreadBytes) return NDQ_EUNSUPPORTED;   // cannot happen for levels <= 256
    const dim3 grid((uint32_t)blocks), block(kDenseBlock);
    hipStream_t s = (hipStream_t)stream;
    if (levels == 3u && a.k == 20u && a.bits == 2u)
        return pack ? launch((dense_pack_fixed_kernel<3, 20, 2>), grid, block, s, a)
                    : launch((dense_unpack_fixed_kernel<3, 20, 2>), grid, block, s, a);
    if (levels == 5u && a.k == 13u && a.bits == 3u)
        return pack ? launch((dense_pack_fixed_kernel<5, 13, 3>), grid, block, s, a)
                    : launch((dense_unpack_fixed_kernel<5, 13, 3>), grid, block, s, a);
    if (pack) return launch(dense_pack_kernel, grid, block, s, a);
    return launch(dense_unpack_kernel, grid, block, s, a);
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

uint32_t ndq_nesting_ratio_for_error(double delta1, double alpha, double sigma_z2, double p_max)
{
    if (!(delta1 > 0.0) || !(alpha >= 0.0 && alpha <= 1.0) || !(sigma_z2 >= 0.0) || !(p_max > 0.0))
        return 0;
    // bound(M) = c / M^2 with c = 1/3 + 4 alpha^2 sigma_z^2 / Delta_1^2: start at
    // the real-valued root and let the bound itself settle the last unit.
    const double c = 1.0 / 3.0 + 4.0 * alpha * alpha * sigma_z2 / (delta1 * delta1);
    const double root = sqrt(c / p_max);
    if (!(root <= 257.0)) return 0;
    uint32_t M = root < 2.0 ? 2u : (uint32_t)root;
    while (M > 2 && ndq_decode_error_bound(delta1, M - 1, alpha, sigma_z2) <= p_max) --M;
    while (M <= 256 && ndq_decode_error_bound(delta1, M, alpha, sigma_z2) > p_max) ++M;
    return M <= 256 ? M : 0;
}

size_t ndq_sqdiff_workspace(void) { return ndq::kSqBlocks * sizeof(double); }

int ndq_sqdiff(const float* a, const float* b, size_t n, double* workspace, double* out,
               void* stream)
{
    if (!workspace) return NDQ_EINVAL;
    return ndq::sqdiff_common(a, b, n, workspace, out, stream);
}

int ndq_sqdiff_static(const float* a, const float* b, size_t n, double* out, void* stream)
{
    if (n >= ndq::kMaxN) return NDQ_EUNSUPPORTED;   // beyond what the fixed grid is sized for
    double* partial = ndq::scratch_on_current_device();
    if (!partial) return NDQ_ELAUNCH;
    return ndq::sqdiff_common(a, b, n, partial, out, stream);
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
