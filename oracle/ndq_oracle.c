/*
 * ndq_oracle.c -- CPU oracle (test infrastructure, see ndq_oracle.h).
 *
 * Plain scalar C, one element at a time, in the order the paper states the
 * steps.  Build with -O2 -ffp-contract=off -fno-fast-math so that every line
 * below is exactly one IEEE-754 binary32 operation where it says so.
 */
#include "ndq_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------- */
/* Dither stream.  The paper (Sec. 2.1 Remark 1; Sec. 3.1, paragraph before    */
/* Algorithm 1) only asks that sender and receiver run the same generator from  */
/* the same seed and that the seed changes every iteration.  Choice made here:  */
/* the counter-based Philox4x32 with 10 rounds of Salmon, Moraes, Dror & Shaw,  */
/* "Parallel random numbers: as easy as 1, 2, 3" (SC'11).  One 128-bit block     */
/* serves eight consecutive elements, 16 bits each: element i uses half (i mod  */
/* 2) of word ((i/2) mod 4) of the block whose counter is (i/8 low, i/8 high,   */
/* step, worker) under key (seed low, seed high); "updating the seed" is the    */
/* step counter.                                                                */
/* ------------------------------------------------------------------------- */

void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    const uint32_t MUL0 = 0xD2511F53u, MUL1 = 0xCD9E8D57u;  /* round multipliers   */
    const uint32_t WEYL0 = 0x9E3779B9u, WEYL1 = 0xBB67AE85u; /* key schedule steps  */
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t prod0 = (uint64_t)MUL0 * c0;
        uint64_t prod1 = (uint64_t)MUL1 * c2;
        uint32_t hi0 = (uint32_t)(prod0 >> 32), lo0 = (uint32_t)prod0;
        uint32_t hi1 = (uint32_t)(prod1 >> 32), lo1 = (uint32_t)prod1;
        c0 = hi1 ^ c1 ^ k0;
        c1 = lo1;
        c2 = hi0 ^ c3 ^ k1;
        c3 = lo0;
        k0 += WEYL0;
        k1 += WEYL1;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

float oracle_unit_dither(uint64_t seed, uint32_t step, uint32_t worker, uint64_t i)
{
    uint64_t block = i >> 3;
    uint32_t ctr[4] = { (uint32_t)block, (uint32_t)(block >> 32), step, worker };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t r[4];
    oracle_philox4x32_10(ctr, key, r);
    uint32_t word = r[(i >> 1) & 3u];
    uint32_t cell = (i & 1u) ? (word >> 16) : (word & 0xFFFFu);
    /* (cell + 1/2) * 2^-16 - 1/2 : the mid-point of cell `cell` of 2^16 equal
     * cells of [-1/2, 1/2).  Every such value is a binary32 number, so the fma
     * is exact; the grid is symmetric, hence has mean exactly 0.  A dither on
     * K equally spaced points meets condition 2 of Thm 1 for every l that is
     * not a multiple of K, so the reconstruction error is uniform and
     * independent of the input down to a resolution of Delta/K = 2^-16 Delta. */
    return fmaf((float)cell, 0x1p-16f, -0.5f + 0x1p-17f);
}

/* ------------------------------------------------------------------------- */
/* Scalar building blocks                                                      */
/* ------------------------------------------------------------------------- */

uint32_t oracle_code_bits(uint32_t x)
{
    if (x < 2u || x > 256u) return 0u;
    uint32_t b = 0u;
    while ((1u << b) < x) ++b;
    return b;
}

/* Sec. 3.1 eq. (2): kappa = max|g_i| maps g into [-1,1] and the normalised step
 * is 1/M for 2M+1 levels, i.e. 2/(L-1).  In absolute units the step is
 * kappa * 2/(L-1); it is what travels with the codes in place of kappa. */
float oracle_step_from_kappa(float kappa, uint32_t levels)
{
    float step = (2.0f * kappa) / (float)(levels - 1u);
    if (!(step >= 0x1p-100f)) step = 0.0f; /* all-zero (or vanishing) bucket */
    return step;
}

float oracle_inv_step(float delta)
{
    return (delta > 0.0f) ? 1.0f / delta : 0.0f;
}

static float round_half_even(float t) { return rintf(t); } /* default rounding mode */

int32_t oracle_fine_index(float g, float inv_delta, float v)
{
    /* Alg. 1: q = round(t/Delta), t = g/kappa + u.  With absolute step and
     * unit dither: q = round(g/Delta + v); one fused multiply-add, one round. */
    float t = fmaf(g, inv_delta, v);
    float r = round_half_even(t);
    if (r > 16777216.0f) r = 16777216.0f;
    if (r < -16777216.0f) r = -16777216.0f;
    return (int32_t)r;
}

uint32_t oracle_dq_code(float g, float inv_delta, float v, uint32_t levels)
{
    int32_t q_min = -(int32_t)(levels / 2u);
    int32_t q_max = q_min + (int32_t)levels - 1;
    int32_t q = oracle_fine_index(g, inv_delta, v);
    if (q < q_min) q = q_min; /* the quantizer has L levels: saturate */
    if (q > q_max) q = q_max;
    return (uint32_t)(q - q_min);
}

float oracle_index_value(int32_t q, float delta, float v)
{
    /* Alg. 1 server: g~ = kappa*(Delta*q - u) = Delta_abs * (q - v). */
    float centred = (float)q - v;
    return delta * centred;
}

float oracle_dq_value(uint32_t code, float delta, float v, uint32_t levels)
{
    int32_t q_min = -(int32_t)(levels / 2u);
    return oracle_index_value((int32_t)code + q_min, delta, v);
}

float oracle_dq_value_half(uint32_t code, float delta, uint32_t levels)
{
    /* x~_h = Q(x+u) = Delta * q */
    int32_t q_min = -(int32_t)(levels / 2u);
    return delta * (float)((int32_t)code + q_min);
}

double oracle_dq_value_f64(uint32_t code, double delta, double v, uint32_t levels)
{
    int32_t q_min = -(int32_t)(levels / 2u);
    return delta * ((double)((int32_t)code + q_min) - v);
}

uint32_t oracle_nested_code(float g, float inv_delta, float v, uint32_t M)
{
    /* eq. (7): s = Q1(t) - Q2(t) with Delta_2 = M*Delta_1.  s/Delta_1 is the
     * fine index minus a multiple of M; the decoder of eq. (8) is unchanged
     * by adding multiples of Delta_2 to s, so the residue mod M carries all
     * the information and fits ceil(log2 M) bits for even M too. */
    int32_t q = oracle_fine_index(g, inv_delta, v);
    int32_t m = q % (int32_t)M;
    if (m < 0) m += (int32_t)M;
    return (uint32_t)m;
}

float oracle_coset_k(uint32_t m, float y, float inv_delta, float v, uint32_t M)
{
    /* eq. (8), alpha = 1, s = m*Delta_1:
     *   x^ = y + r - Q2(r),  r = s - u - y
     *      = (m*Delta_1 - u) - Delta_2 * round((m*Delta_1 - u - y)/Delta_2)
     * i.e. the point (m + M*k)*Delta_1 - u of the coset nearest to y.  In index
     * units: k = round((y/Delta_1 + v - m)/M).  Eq. (8) puts no bound on k. */
    float c = fmaf(y, inv_delta, v);
    return round_half_even((c - (float)m) / (float)M);
}

int32_t oracle_coset_index(uint32_t m, float y, float inv_delta, float v, uint32_t M)
{
    /* q^ = m + M*k as a 32-bit integer, for the callers that count decode errors
     * (saturated where it does not fit: side information 2^31 steps away) */
    float k = oracle_coset_k(m, y, inv_delta, v, M);
    if (!(k > -8388608.0f * 256.0f)) return INT32_MIN;
    if (!(k < 8388608.0f * 256.0f)) return INT32_MAX;
    int64_t q = (int64_t)m + (int64_t)M * (int64_t)k;
    if (q > INT32_MAX) q = INT32_MAX;
    if (q < INT32_MIN) q = INT32_MIN;
    return (int32_t)q;
}

float oracle_coset_value(float k, uint32_t m, uint32_t M, float delta, float v)
{
    /* Alg. 2 server: Delta_1 * (q^ - v) with q^ = m + M*k brought to binary32 by one
     * rounding of its exact value (what fmaf returns), however large k is */
    float q = fmaf(k, (float)M, (float)m);
    float centred = q - v;
    return delta * centred;
}

/* ------------------------------------------------------------------------- */
/* Shrinkage factor alpha (Sec. 3.2 eqs. (7)-(8), Thm 4)                        */
/* ------------------------------------------------------------------------- */

uint32_t oracle_nested_code_alpha(float g, float inv_delta, float alpha, float v, uint32_t M)
{
    /* t = alpha*x + u in units of Delta_1: g * (alpha/Delta_1) + v.  The factor
     * alpha/Delta_1 is formed once (one rounding); with alpha = 1 it is 1/Delta_1. */
    float a = alpha * inv_delta;
    return oracle_nested_code(g, a, v, M);
}

float oracle_nested_value_alpha(uint32_t m, float y, float delta, float alpha, float v, uint32_t M)
{
    /* r - Q2(r) = Delta_1*(q^ - v) - alpha*y with q^ = m + M*k the coset point
     * nearest to alpha*y/Delta_1 + v, hence
     *   x^ = y + alpha*(r - Q2(r)) = (1 - alpha^2)*y + alpha*Delta_1*(q^ - v). */
    float a = alpha * oracle_inv_step(delta);
    float k = oracle_coset_k(m, y, a, v, M);
    float lattice = oracle_coset_value(k, m, M, delta, v);
    float beta = (float)(1.0 - (double)alpha * (double)alpha);
    float scaled = alpha * lattice;
    return fmaf(beta, y, scaled);
}

double oracle_alpha_for_equal_variance(double delta1, double sigma_z2)
{
    double arg = 1.0 - delta1 * delta1 / (12.0 * sigma_z2);
    return arg > 0.0 ? sqrt(arg) : 0.0;
}

double oracle_decode_error_bound(double delta1, uint32_t M, double alpha, double sigma_z2)
{
    double delta2 = (double)M * delta1;
    return delta1 * delta1 / (3.0 * delta2 * delta2) + 4.0 * alpha * alpha * sigma_z2 / (delta2 * delta2);
}

/* Smallest nesting ratio whose Thm 4 bound is at most p_max: the definition,
 * tried in increasing order (fewest bits first); 0 if none up to 256 fits. */
uint32_t oracle_nesting_ratio_for_error(double delta1, double alpha, double sigma_z2, double p_max)
{
    if (!(delta1 > 0.0) || !(alpha >= 0.0 && alpha <= 1.0) || !(sigma_z2 >= 0.0) || !(p_max > 0.0))
        return 0;
    for (uint32_t M = 2; M <= 256; ++M)
        if (oracle_decode_error_bound(delta1, M, alpha, sigma_z2) <= p_max) return M;
    return 0;
}

double oracle_sqdiff_sum(const float* a, const float* b, size_t n)
{
    double acc = 0.0;
    for (size_t i = 0; i < n; ++i) {
        double d = (double)a[i] - (double)b[i];
        acc += d * d;
    }
    return acc;
}

/* ------------------------------------------------------------------------- */
/* Bitstream: fixed-width codes, least-significant bit first.                  */
/* ------------------------------------------------------------------------- */

size_t oracle_packed_bytes(size_t n, uint32_t bits)
{
    size_t bytes = (n * (size_t)bits + 7u) / 8u;
    return (bytes + 15u) / 16u * 16u;
}

size_t oracle_num_buckets(size_t n, uint32_t bucket)
{
    if (bucket == 0u) return 1u;
    return (n + bucket - 1u) / bucket;
}

void oracle_pack(const uint32_t* codes, size_t n, uint32_t bits, uint8_t* out)
{
    memset(out, 0, oracle_packed_bytes(n, bits));
    for (size_t i = 0; i < n; ++i)
        for (uint32_t j = 0; j < bits; ++j) {
            size_t k = i * bits + j; /* position in the stream */
            if ((codes[i] >> j) & 1u) out[k / 8u] |= (uint8_t)(1u << (k % 8u));
        }
}

void oracle_unpack(const uint8_t* in, size_t n, uint32_t bits, uint32_t* codes)
{
    for (size_t i = 0; i < n; ++i) {
        uint32_t c = 0u;
        for (uint32_t j = 0; j < bits; ++j) {
            size_t k = i * bits + j;
            c |= (uint32_t)((in[k / 8u] >> (k % 8u)) & 1u) << j;
        }
        codes[i] = c;
    }
}

/* ------------------------------------------------------------------------- */
/* Dense base-L stream.  Table 1 (Sec. 4) counts log2(L) bits per index; k      */
/* base-L digits in a 32-bit word spend 32/k, e.g. 1.6 bits for L = 3 (k = 20). */
/* ------------------------------------------------------------------------- */

uint32_t oracle_dense_group(uint32_t levels)
{
    if (levels < 2u || levels > 256u) return 0u;
    uint32_t k = 0u;
    uint64_t power = 1u;                        /* levels^k */
    while (power * levels <= ((uint64_t)1 << 32)) { power *= levels; ++k; }
    return k;
}

size_t oracle_dense_bytes(size_t n, uint32_t levels)
{
    uint32_t k = oracle_dense_group(levels);
    size_t words = (n + k - 1u) / k;
    return (words * 4u + 15u) / 16u * 16u;
}

void oracle_dense_pack(const uint32_t* codes, size_t n, uint32_t levels, uint8_t* out)
{
    uint32_t k = oracle_dense_group(levels);
    size_t bytes = oracle_dense_bytes(n, levels);
    memset(out, 0, bytes);
    size_t words = (n + k - 1u) / k;
    for (size_t w = 0; w < words; ++w) {
        uint64_t value = 0u, weight = 1u;
        for (uint32_t j = 0; j < k; ++j) {
            size_t i = w * k + j;
            uint32_t digit = i < n ? codes[i] : 0u;
            value += digit * weight;
            weight *= levels;
        }
        for (uint32_t b = 0; b < 4u; ++b) out[4u * w + b] = (uint8_t)(value >> (8u * b));
    }
}

void oracle_dense_unpack(const uint8_t* in, size_t n, uint32_t levels, uint32_t* codes)
{
    uint32_t k = oracle_dense_group(levels);
    for (size_t i = 0; i < n; ++i) {
        size_t w = i / k;
        uint32_t value = (uint32_t)in[4u * w] | ((uint32_t)in[4u * w + 1u] << 8) |
                         ((uint32_t)in[4u * w + 2u] << 16) | ((uint32_t)in[4u * w + 3u] << 24);
        for (uint32_t j = 0; j < i % k; ++j) value /= levels;
        codes[i] = value % levels;
    }
}

/* ------------------------------------------------------------------------- */
/* Entropy of the index stream (Sec. 4, paragraph before Table 1: adaptive      */
/* arithmetic coding gets within a few percent of the entropy, so the entropy  */
/* of the indices is what is reported).                                         */
/* ------------------------------------------------------------------------- */

void oracle_code_histogram(const uint8_t* codes, size_t n, uint32_t bits, uint64_t* hist)
{
    uint32_t nbins = 1u << bits;
    for (uint32_t c = 0; c < nbins; ++c) hist[c] = 0u;
    uint32_t* q = (uint32_t*)malloc((n ? n : 1u) * sizeof *q);
    oracle_unpack(codes, n, bits, q);
    for (size_t i = 0; i < n; ++i) hist[q[i]] += 1u;
    free(q);
}

double oracle_entropy_bits(const uint64_t* hist, uint32_t nbins)
{
    uint64_t total = 0u;
    for (uint32_t c = 0; c < nbins; ++c) total += hist[c];
    if (total == 0u) return 0.0;
    double h = 0.0;
    for (uint32_t c = 0; c < nbins; ++c)
        if (hist[c]) {
            double p = (double)hist[c] / (double)total;
            h -= p * log2(p);
        }
    return h;
}

/* ------------------------------------------------------------------------- */
/* Vector calls                                                                */
/* ------------------------------------------------------------------------- */

static float load_elem(const void* g, int dtype, size_t i)
{
    if (dtype == 0) return ((const float*)g)[i];
    uint32_t wide = (uint32_t)((const uint16_t*)g)[i] << 16; /* bfloat16 -> binary32, exact */
    float f;
    memcpy(&f, &wide, sizeof f);
    return f;
}

static size_t bucket_of(size_t i, uint32_t bucket) { return bucket ? i / bucket : 0u; }

void oracle_unit_dithers(oracle_dither d, size_t n, float* v_out)
{
    for (size_t i = 0; i < n; ++i)
        v_out[i] = oracle_unit_dither(d.seed, d.step, d.worker, d.offset + i);
}

void oracle_absmax(const void* g, int dtype, size_t n, uint32_t bucket, float* kappa_out)
{
    size_t K = oracle_num_buckets(n, bucket);
    for (size_t b = 0; b < K; ++b) kappa_out[b] = 0.0f;
    for (size_t i = 0; i < n; ++i) {
        float a = fabsf(load_elem(g, dtype, i));
        size_t b = bucket_of(i, bucket);
        if (a > kappa_out[b]) kappa_out[b] = a;
    }
}

/* Partitioned scaling (Sec. 3.1, paragraph after Lemma 2): one scale factor
 * per sub-vector.  bucket==0 with a caller-set delta is the preset step of
 * Algorithm 1's initialisation. */
static void make_steps(const void* g, int dtype, size_t n, float delta, uint32_t levels,
                       uint32_t bucket, float* steps_out)
{
    if (bucket == 0u && delta > 0.0f) { steps_out[0] = delta; return; }
    size_t K = oracle_num_buckets(n, bucket);
    oracle_absmax(g, dtype, n, bucket, steps_out);
    for (size_t b = 0; b < K; ++b) steps_out[b] = oracle_step_from_kappa(steps_out[b], levels);
}

/* The codes are produced one at a time and then packed by oracle_pack; the
 * temporary index array is the "q_p" of Algorithm 1. */
void oracle_dq_encode(const void* g, int dtype, size_t n, float delta, uint32_t levels,
                      uint32_t bucket, oracle_dither d, uint8_t* codes_out, float* steps_out)
{
    uint32_t bits = oracle_code_bits(levels);
    make_steps(g, dtype, n, delta, levels, bucket, steps_out);
    uint32_t* q = (uint32_t*)malloc((n ? n : 1u) * sizeof *q);
    for (size_t i = 0; i < n; ++i) {
        float inv = oracle_inv_step(steps_out[bucket_of(i, bucket)]);
        float v = oracle_unit_dither(d.seed, d.step, d.worker, d.offset + i);
        q[i] = oracle_dq_code(load_elem(g, dtype, i), inv, v, levels);
    }
    oracle_pack(q, n, bits, codes_out);
    free(q);
}

void oracle_dq_decode(const uint8_t* codes, size_t n, uint32_t levels, uint32_t bucket,
                      const float* steps, oracle_dither d, float* out, int accumulate)
{
    uint32_t bits = oracle_code_bits(levels);
    uint32_t* q = (uint32_t*)malloc((n ? n : 1u) * sizeof *q);
    oracle_unpack(codes, n, bits, q);
    for (size_t i = 0; i < n; ++i) {
        float step = steps[bucket_of(i, bucket)];
        float v = oracle_unit_dither(d.seed, d.step, d.worker, d.offset + i);
        float value = oracle_dq_value(q[i], step, v, levels);
        out[i] = accumulate ? out[i] + value : value;
    }
    free(q);
}

void oracle_dq_decode_half(const uint8_t* codes, size_t n, uint32_t levels, uint32_t bucket,
                           const float* steps, float* out, int accumulate)
{
    uint32_t bits = oracle_code_bits(levels);
    uint32_t* q = (uint32_t*)malloc((n ? n : 1u) * sizeof *q);
    oracle_unpack(codes, n, bits, q);
    for (size_t i = 0; i < n; ++i) {
        float value = oracle_dq_value_half(q[i], steps[bucket_of(i, bucket)], levels);
        out[i] = accumulate ? out[i] + value : value;
    }
    free(q);
}

void oracle_nested_encode(const void* g, int dtype, size_t n, float delta, uint32_t levels,
                          uint32_t M, float alpha, uint32_t bucket, oracle_dither d,
                          uint8_t* codes_out, float* steps_out)
{
    uint32_t bits = oracle_code_bits(M);
    make_steps(g, dtype, n, delta, levels, bucket, steps_out);
    uint32_t* m = (uint32_t*)malloc((n ? n : 1u) * sizeof *m);
    for (size_t i = 0; i < n; ++i) {
        float inv = oracle_inv_step(steps_out[bucket_of(i, bucket)]);
        float v = oracle_unit_dither(d.seed, d.step, d.worker, d.offset + i);
        m[i] = oracle_nested_code_alpha(load_elem(g, dtype, i), inv, alpha, v, M);
    }
    oracle_pack(m, n, bits, codes_out);
    free(m);
}

void oracle_nested_decode(const uint8_t* codes, size_t n, uint32_t M, float alpha,
                          uint32_t bucket, const float* steps, oracle_dither d, const float* side,
                          float side_scale, float* out, int accumulate)
{
    uint32_t bits = oracle_code_bits(M);
    uint32_t* m = (uint32_t*)malloc((n ? n : 1u) * sizeof *m);
    oracle_unpack(codes, n, bits, m);
    for (size_t i = 0; i < n; ++i) {
        float step = steps[bucket_of(i, bucket)];
        float v = oracle_unit_dither(d.seed, d.step, d.worker, d.offset + i);
        float y = side[i] * side_scale; /* running sum times 1/count = running mean */
        float value = oracle_nested_value_alpha(m[i], y, step, alpha, v, M);
        out[i] = accumulate ? out[i] + value : value;
    }
    free(m);
}

void oracle_aggregate(const float* const* gs, uint32_t W, size_t n, float scale, float* out)
{
    for (size_t i = 0; i < n; ++i) {
        float acc = 0.0f;
        for (uint32_t w = 0; w < W; ++w) acc = acc + gs[w][i];
        out[i] = scale * acc;
    }
}

void oracle_fine_indices(const void* g, int dtype, size_t n, uint32_t bucket, const float* steps,
                         oracle_dither d, int32_t* q_out)
{
    for (size_t i = 0; i < n; ++i) {
        float inv = oracle_inv_step(steps[bucket_of(i, bucket)]);
        float v = oracle_unit_dither(d.seed, d.step, d.worker, d.offset + i);
        q_out[i] = oracle_fine_index(load_elem(g, dtype, i), inv, v);
    }
}

void oracle_coset_indices(const uint8_t* codes, size_t n, uint32_t M, uint32_t bucket,
                          const float* steps, oracle_dither d, const float* side,
                          float side_scale, int32_t* q_out)
{
    uint32_t bits = oracle_code_bits(M);
    uint32_t* m = (uint32_t*)malloc((n ? n : 1u) * sizeof *m);
    oracle_unpack(codes, n, bits, m);
    for (size_t i = 0; i < n; ++i) {
        float inv = oracle_inv_step(steps[bucket_of(i, bucket)]);
        float v = oracle_unit_dither(d.seed, d.step, d.worker, d.offset + i);
        q_out[i] = oracle_coset_index(m[i], side[i] * side_scale, inv, v, M);
    }
    free(m);
}
