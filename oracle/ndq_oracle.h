/*
 * ndq_oracle.h -- CPU oracle for dithered (DQSG) and nested dithered (NDQSG)
 * quantization of stochastic-gradient vectors.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, scalar
 * restatement of the method (Sec. 2.1 Definition and Remark 1; Sec. 3.1 eq. (2)
 * and Algorithm 1; Sec. 3.2 eqs. (7)-(8) and Algorithm 2) used only to check the
 * GPU library and to be timed beside it.  It shares no code with the GPU path.
 *
 * Precision.  The paper fixes none.  Every step that decides an integer (the
 * quantization index, the coset representative) is taken in IEEE-754 binary32,
 * the precision the GPU kernels use, so that codes can be compared bit for bit.
 * Decoded values are binary32 as well because they feed the next worker's coset
 * decision in Algorithm 2; oracle_dq_value_f64 gives the same quantity in
 * binary64 from the definition, and the tests bound the difference.
 *
 * Free choices the paper leaves open (all pinned here, see each function):
 *   - the random-number generator: Philox4x32-10 (Salmon et al., SC'11), counter
 *     (i>>3 low, i>>3 high, step, worker), key (seed low, seed high); one block
 *     gives the dithers of eight consecutive elements, 16 bits each;
 *   - the dither grid: 2^16 mid-points of equal cells of [-1/2, 1/2);
 *   - "nearest integer" ties: to even;
 *   - number of levels L (odd L is the paper's 2M+1 case; even L uses
 *     indices -L/2 .. L/2-1);
 *   - the bitstream: fixed-width codes, LSB first.
 *
 * Parity unpinned by the paper (our own definitions, pinned only by round-trip
 * and brute-force tests): packed-byte layout, code offset q_min, dither grid.
 */
#ifndef NDQ_ORACLE_H
#define NDQ_ORACLE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ---- dither stream (Remark 1; Algorithm 1 "generate u_p using seed s_p") ---- */

/* One Philox4x32-10 block: out = Philox(ctr, key). */
void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);

/* Unit dither v_i in (-1/2, 1/2) for element i of (seed, step, worker); the
 * dither of the paper is u_i = Delta * v_i. */
float oracle_unit_dither(uint64_t seed, uint32_t step, uint32_t worker, uint64_t i);

/* ---- scalar building blocks (take the unit dither v explicitly) ---- */

/* bits per code: ceil(log2(x)), x in [2,256]; 0 if x out of range */
uint32_t oracle_code_bits(uint32_t x);

/* Step for a bucket with max-norm kappa and L levels: 2*kappa/(L-1); steps
 * below 2^-100 are treated as an all-zero bucket and returned as 0. */
float oracle_step_from_kappa(float kappa, uint32_t levels);

/* 1/Delta, or 0 when Delta == 0 (all-zero bucket). */
float oracle_inv_step(float delta);

/* eq. (2) / Alg. 1 worker: clipped index q = round(g/Delta + v) in
 * [-(L/2), -(L/2)+L-1]; returns the code c = q - q_min in [0, L). */
uint32_t oracle_dq_code(float g, float inv_delta, float v, uint32_t levels);

/* Alg. 1 server: g~ = Delta * (q - v) with q = code + q_min. */
float oracle_dq_value(uint32_t code, float delta, float v, uint32_t levels);
double oracle_dq_value_f64(uint32_t code, double delta, double v, uint32_t levels);

/* Sec. 2.1, half-dithered quantization x~_h = Q(x+u): the receiver does not
 * subtract the dither (the reconstruction rule of the stochastic and ternary
 * quantizers the paper compares with, Lemma 1). */
float oracle_dq_value_half(uint32_t code, float delta, uint32_t levels);

/* unclipped fine index round(g/Delta + v) (saturated at +-2^24) */
int32_t oracle_fine_index(float g, float inv_delta, float v);

/* eq. (7) with alpha = 1, Delta_2 = M*Delta_1: the fine index modulo M in [0, M). */
uint32_t oracle_nested_code(float g, float inv_delta, float v, uint32_t M);

/* eq. (8) with alpha = 1: the integer congruent to m (mod M) nearest to
 * y/Delta + v; the decoded value is Delta * (that integer - v). */
float oracle_coset_k(uint32_t m, float y, float inv_delta, float v, uint32_t M);
int32_t oracle_coset_index(uint32_t m, float y, float inv_delta, float v, uint32_t M);
float oracle_coset_value(float k, uint32_t m, uint32_t M, float delta, float v);
float oracle_index_value(int32_t q, float delta, float v);

/* eqs. (7)-(8) with a shrinkage factor 0 < alpha <= 1 (Sec. 3.2; Thm 4):
 *   encoder  t = alpha*x + u, transmitted residue = round(t/Delta_1) mod M
 *   decoder  r = s - u - alpha*y,  x^ = y + alpha*(r - Q2(r))
 *            = (1 - alpha^2)*y + alpha*Delta_1*(q^ - v),
 *   q^ the integer congruent to the residue nearest to alpha*y/Delta_1 + v.
 * alpha = 1 gives oracle_nested_code / oracle_coset_index / oracle_index_value
 * bit for bit. */
uint32_t oracle_nested_code_alpha(float g, float inv_delta, float alpha, float v, uint32_t M);
float oracle_nested_value_alpha(uint32_t m, float y, float delta, float alpha, float v, uint32_t M);

/* Thm 4 / last paragraph of Sec. 3.2: the shrinkage that gives NDQSG the
 * variance Delta_1^2/12 of DQSG, alpha = sqrt(1 - Delta_1^2/(12 sigma_z^2))
 * (0 if the argument is not positive), and the bound on the probability of a
 * coset decode error, Delta_1^2/(3 Delta_2^2) + 4 alpha^2 sigma_z^2/Delta_2^2. */
double oracle_alpha_for_equal_variance(double delta1, double sigma_z2);
double oracle_decode_error_bound(double delta1, uint32_t M, double alpha, double sigma_z2);
uint32_t oracle_nesting_ratio_for_error(double delta1, double alpha, double sigma_z2, double p_max);
/* sigma_z^2 estimate: sum_i (a_i - b_i)^2 in binary64 (divide by n for the mean) */
double oracle_sqdiff_sum(const float* a, const float* b, size_t n);

/* ---- bitstream ---- */
size_t oracle_packed_bytes(size_t n, uint32_t bits); /* ceil(n*bits/8) rounded up to 16 */
size_t oracle_num_buckets(size_t n, uint32_t bucket); /* bucket==0 -> 1 */
/* code i occupies stream bits [i*b,(i+1)*b), bit k = bit (k%8) of byte k/8; padding zero */
void oracle_pack(const uint32_t* codes, size_t n, uint32_t bits, uint8_t* out);
void oracle_unpack(const uint8_t* in, size_t n, uint32_t bits, uint32_t* codes);

/* ---- dense base-L stream (Sec. 4 Table 1 counts log2(L) bits per index, e.g.
 * 1.585 for three levels; fixed-width codes spend ceil(log2 L)) ----
 * k = oracle_dense_group(L) is the largest k with L^k <= 2^32; codes are taken in
 * groups of k and each group is stored as the 32-bit number sum_j c_j L^j
 * (little-endian words, first code = lowest digit); the last group is filled
 * with zero digits and the stream is padded with zero words to a multiple of 16
 * bytes. */
uint32_t oracle_dense_group(uint32_t levels);
size_t oracle_dense_bytes(size_t n, uint32_t levels);
void oracle_dense_pack(const uint32_t* codes, size_t n, uint32_t levels, uint8_t* out);
void oracle_dense_unpack(const uint8_t* in, size_t n, uint32_t levels, uint32_t* codes);

/* ---- entropy of an index stream (Sec. 4: bits after entropy coding are
 * reported through the entropy of the transmitted indices) ---- */
/* hist[c] = number of codes equal to c, c in [0, 2^bits) */
void oracle_code_histogram(const uint8_t* codes, size_t n, uint32_t bits, uint64_t* hist);
/* -sum_c p_c log2 p_c with p_c = hist[c]/n, in bits per code; 0 for n == 0 */
double oracle_entropy_bits(const uint64_t* hist, uint32_t nbins);

/* ---- vector calls, mirroring the library's entry points ---- */

/* seed s_p, iteration, worker p, and the index within the worker's whole
 * gradient of the first element of this call (0 unless a slice is processed). */
typedef struct { uint64_t seed; uint32_t step; uint32_t worker; uint64_t offset; } oracle_dither;

/* the n unit dithers a call with this descriptor draws */
void oracle_unit_dithers(oracle_dither d, size_t n, float* v_out);

/* dtype: 0 = binary32, 1 = bfloat16 (widened exactly). */
void oracle_absmax(const void* g, int dtype, size_t n, uint32_t bucket, float* kappa_out);

/* Worker side of Alg. 1.  bucket==0: one step for the whole vector: `delta` if
 * delta > 0, else 2*max|g|/(L-1); bucket>0: one step per bucket from its own
 * max-norm.  Writes the packed codes and the steps. */
void oracle_dq_encode(const void* g, int dtype, size_t n, float delta, uint32_t levels,
                      uint32_t bucket, oracle_dither d, uint8_t* codes_out, float* steps_out);

/* Server side of Alg. 1.  accumulate: out += g~ instead of out = g~. */
void oracle_dq_decode(const uint8_t* codes, size_t n, uint32_t levels, uint32_t bucket,
                      const float* steps, oracle_dither d, float* out, int accumulate);

/* Half-dithered server side: out = Delta * q, no dither regenerated. */
void oracle_dq_decode_half(const uint8_t* codes, size_t n, uint32_t levels, uint32_t bucket,
                           const float* steps, float* out, int accumulate);

/* Worker side of Alg. 2 for p in P2.  `levels` only sets the fine step. */
void oracle_nested_encode(const void* g, int dtype, size_t n, float delta, uint32_t levels,
                          uint32_t M, float alpha, uint32_t bucket, oracle_dither d,
                          uint8_t* codes_out, float* steps_out);

/* Server side of Alg. 2 for p in P2; side information y_i = side[i]*side_scale. */
void oracle_nested_decode(const uint8_t* codes, size_t n, uint32_t M, float alpha,
                          uint32_t bucket, const float* steps, oracle_dither d, const float* side,
                          float side_scale, float* out, int accumulate);

/* Alg. 1 server: out_i = scale * sum_w gs[w][i], w ascending. */
void oracle_aggregate(const float* const* gs, uint32_t W, size_t n, float scale, float* out);

/* diagnostics: unclipped fine indices of a vector (for counting coset decode errors) */
void oracle_fine_indices(const void* g, int dtype, size_t n, uint32_t bucket, const float* steps,
                         oracle_dither d, int32_t* q_out);
/* coset-resolved indices the nested decoder used (same inputs as oracle_nested_decode) */
void oracle_coset_indices(const uint8_t* codes, size_t n, uint32_t M, uint32_t bucket,
                          const float* steps, oracle_dither d, const float* side,
                          float side_scale, int32_t* q_out);

#ifdef __cplusplus
}
#endif
#endif
