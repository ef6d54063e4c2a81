/*
 * ndq.h -- C ABI of libndq: dithered (DQSG) and nested dithered (NDQSG)
 * quantization of stochastic-gradient vectors on one AMD MI355X (gfx950).
 *
 * Method: A. Abdi, F. Fekri, "Nested Dithered Quantization for Communication
 * Reduction in Distributed Training" (arXiv 1904.01197).  A worker holds a
 * gradient vector g, a step Delta (or a number of levels and a max-norm scale),
 * a dither seed s_p and the iteration number; it sends quantization indices and
 * scale factors (Algorithm 1, "Workers"; Algorithm 2, "Workers").  The server
 * holds the indices, the scale factors and the same seed, and for nested
 * workers the side information: the mean of what it has decoded so far
 * (Algorithm 1, "Server"; Algorithm 2, "Server").
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers owned by the caller; `d` (the dither
 *     descriptor) and the pointer array of ndq_aggregate are HOST pointers, read
 *     before the call returns.
 *   - The library never allocates, frees, retains or synchronises.  A call only
 *     enqueues kernels on `stream` (a hipStream_t passed as void*; NULL = the
 *     default stream) and returns.
 *   - Return value: 0 on success, a negative ndq_status on error.  Arguments are
 *     checked before anything is launched: with NDQ_EINVAL, NDQ_EALIGN or
 *     NDQ_EUNSUPPORTED nothing has been enqueued.  NDQ_ELAUNCH comes from the
 *     runtime's launch call itself; calls made of several kernels (a max-norm
 *     pass or a step copy before the encoder, ndq_code_entropy, ndq_sqdiff, more than 32 workers
 *     in ndq_decode_chain / ndq_aggregate) may then already have enqueued their
 *     first kernels, and the outputs are unspecified.  n == 0 is a successful no-op.
 *   - g, codes, out and side must be 16-byte aligned; steps 4-byte aligned.
 *     bucket must be 0 or a multiple of 64; d->offset a multiple of 8 (and of
 *     bucket when a slice of a bucketed vector is processed).
 *   - Inputs must be finite; this is not checked.
 *   - No global state: calls are thread-safe.  Calls that write the same buffers
 *     on different streams race.
 *
 * Arithmetic (binary32, round-to-nearest-even, no contraction)
 *   unit dither   v_i = (k + 1/2) 2^-16 - 1/2, k = 16-bit half (I mod 2) of word
 *                 ((I/2) mod 4) of Philox4x32-10(counter = (I/8 low, I/8 high, step,
 *                 worker), key = (seed low, seed high)), I = offset + i: one block
 *                 serves eight consecutive elements.  The dither of the paper is
 *                 u_i = Delta v_i; it is never transmitted (Sec. 2.1, Remark 1).
 *   step          Delta_b = 2 kappa_b / (L-1), kappa_b = max |g_i| over bucket b
 *                 (Sec. 3.1 eq. (2) and the partitioning paragraph after Lemma 2);
 *                 Delta_b < 2^-100 is sent as 0 (all-zero bucket).  1/Delta_b := 0
 *                 when Delta_b == 0.
 *   DQSG index    q_i = clip(rint(fma(g_i, 1/Delta_b, v_i)), -(L/2), -(L/2)+L-1),
 *                 code c_i = q_i + L/2 (integer division).
 *   DQSG value    g~_i = Delta_b * ((float)q_i - v_i)         (Algorithm 1, server)
 *   nested code   m_i = rint(fma(g_i, 1/Delta_b, v_i)) mod M, in [0, M)
 *                 (eq. (7) with Delta_2 = M Delta_1: the position of the fine bin
 *                 relative to the coarse one; shown for alpha = 1)
 *   nested value  y_i = side_i * side_scale; k = rint((fma(y_i, 1/Delta_b, v_i) - m_i)/M);
 *                 q^_i = m_i + M k; g~_i = Delta_b * ((float)q^_i - v_i)
 *                 (eq. (8): the point of the coset nearest to y_i; shown for alpha = 1,
 *                 see ndq_nested_decode for a shrinkage factor alpha < 1)
 *   bitstream     code i occupies stream bits [i b, (i+1) b), b = ndq_code_bits(L or M);
 *                 stream bit k is bit (k mod 8) of byte k/8; the stream is padded
 *                 with zero bits to ndq_packed_bytes(n, b) bytes.
 */
#ifndef NDQ_H
#define NDQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Element types of a gradient vector.  The entry points take the value as a plain
 * int, so that a caller's out-of-range value is an NDQ_EINVAL, not an enum load
 * outside its enumerators. */
typedef enum { NDQ_F32 = 0, NDQ_BF16 = 1 } ndq_dtype;

typedef enum {
    NDQ_OK = 0,
    NDQ_EINVAL = -1,       /* NULL pointer, levels/M outside [2,256], bad bucket, bad W */
    NDQ_EALIGN = -2,       /* pointer, bucket or offset alignment violated             */
    NDQ_EUNSUPPORTED = -3, /* n too large for one call (limits lie between 2^38 and 2^40) */
    NDQ_ELAUNCH = -4       /* the HIP runtime refused a launch                         */
} ndq_status;

/* Identity of a dither stream: the seed s_p shared by worker p and the server
 * (Algorithm 1, initialisation), the training iteration (stands for the "seed
 * update" of Algorithm 1), the worker p, and the index within the worker's
 * whole gradient of the first element handed to this call (0 unless the vector
 * is processed in slices). */
typedef struct {
    uint64_t seed;
    uint32_t step;
    uint32_t worker;
    uint64_t offset;
} ndq_dither;

/* Bits per code: ceil(log2(x)) for x = levels or M in [2,256]; 0 otherwise.
 * (Sec. 3.2, last paragraph: log2(Delta_2/Delta_1) bits per nested value.) */
uint32_t ndq_code_bits(uint32_t levels_or_M);

/* Size in bytes of a packed code stream: ceil(n*bits/8) rounded up to 16 (the
 * message of Algorithm 1's worker step "send q_p": n indices of `bits` bits). */
size_t ndq_packed_bytes(size_t n, uint32_t bits);

/* Number of scale factors: 1 if bucket == 0, else ceil(n/bucket) (Sec. 3.1, the
 * paragraph after Lemma 2: the gradient is partitioned into sub-vectors, each
 * quantized with its own scale factor; `bucket` is the sub-vector length). */
size_t ndq_num_buckets(size_t n, uint32_t bucket);

/* Max-norm scale factors kappa_b = max |g_i| per bucket (Sec. 3.1 eq. (2): the
 * scale factor kappa = ||g||_inf; Algorithm 1 worker step "kappa_p").
 * g: n elements of type dt (an ndq_dtype value).  kappa_out: ndq_num_buckets(n, bucket) floats. */
int ndq_absmax(const void* g, int dt, size_t n, uint32_t bucket, float* kappa_out,
               void* stream);

/* Worker side of Algorithm 1 (generate dither, quantization index, send kappa and
 * q): writes the packed DQSG codes of g and the step of every bucket.
 *   bucket == 0, delta > 0 : one preset step delta (Algorithm 1 initialisation)
 *   bucket == 0, delta <= 0: one step 2 max|g| / (levels-1) for the whole vector
 *   bucket  > 0            : one step per bucket from the bucket's own max-norm
 * codes_out: ndq_packed_bytes(n, ndq_code_bits(levels)) bytes, fully written.
 * (Every bucket size gives the same bytes; speed differs.  One pass over g:
 * buckets of 512, 1024, 2048, 4096 or 8192 elements (bfloat16: also 16384), and
 * a preset step.  Other sizes, and bucket == 0 without a preset step, read g
 * twice.)
 * steps_out: ndq_num_buckets(n, bucket) floats -- the transmitted scale factors
 * (Delta_b = 2 kappa_b/(L-1) travels in place of kappa_b: the same 32 bits). */
int ndq_dq_encode(const void* g, int dt, size_t n, float delta, uint32_t levels,
                  uint32_t bucket, const ndq_dither* d, void* codes_out, float* steps_out,
                  void* stream);

/* Server side of Algorithm 1 (regenerate the dither, reconstruct g~_p).
 * accumulate == 0: out_i = g~_i; accumulate != 0: out_i += g~_i (running sum of
 * the workers decoded so far).  out: n floats. */
int ndq_dq_decode(const void* codes, size_t n, uint32_t levels, uint32_t bucket,
                  const float* steps, const ndq_dither* d, float* out, int accumulate,
                  void* stream);

/* Half-dithered server side (Sec. 2.1, last paragraph; Sec. 2.1.1, Lemma 1): the
 * receiver does not regenerate the dither, out_i = Delta_b * q_i (or += with
 * accumulate).  Applied to the codes of ndq_dq_encode this is the reconstruction
 * rule of stochastic quantization (levels = 2M+1) and of ternary quantization
 * (levels = 3): unbiased, but with an error that depends on the signal. */
int ndq_dq_decode_half(const void* codes, size_t n, uint32_t levels, uint32_t bucket,
                       const float* steps, float* out, int accumulate, void* stream);

/* Worker side of Algorithm 2 for a worker of group P2 (eq. (7)): the fine index of
 * t = alpha*g + u, modulo M.  The step is chosen exactly as in ndq_dq_encode
 * (`levels` only fixes the fine step; it does not clip).  alpha in (0, 1] is the
 * shrinkage factor of Sec. 3.2 (1 = plain nested quantization); the index is
 * rint(fma(g_i, a, v_i)) with a = alpha * (1/Delta_b) formed once per bucket.
 * codes_out: ndq_packed_bytes(n, ndq_code_bits(M)) bytes. */
int ndq_nested_encode(const void* g, int dt, size_t n, float delta, uint32_t levels,
                      uint32_t M, float alpha, uint32_t bucket, const ndq_dither* d,
                      void* codes_out, float* steps_out, void* stream);

/* ndq_dq_encode / ndq_nested_encode with one step for the whole vector that already
 * lies in DEVICE memory: Algorithms 1 and 2 are written for steps Delta (Delta_1,
 * Delta_2) that all workers and the server share (their initialisation), and the
 * natural source of such a step is the steps_out of the worker that chose it.  The
 * call reads *step_in when its kernels run, so no device-to-host copy sits between
 * the two encode calls.  Codes: exactly those of the call above with bucket == 0 and
 * delta == *step_in; for *step_in == 0 every fine index is 0 (1/Delta := 0, as for an
 * all-zero vector).  *step_in must be finite and >= 0; this is not checked.
 * step_in: one float (device, 4-byte aligned).  steps_out: one float, set to
 * *step_in (step_in == steps_out is allowed).  The nested form takes no `levels`:
 * that argument only ever served to derive a step. */
int ndq_dq_encode_with_step(const void* g, int dt, size_t n, const float* step_in, uint32_t levels,
                            const ndq_dither* d, void* codes_out, float* steps_out, void* stream);
int ndq_nested_encode_with_step(const void* g, int dt, size_t n, const float* step_in, uint32_t M,
                                float alpha, const ndq_dither* d, void* codes_out, float* steps_out,
                                void* stream);

/* Server side of Algorithm 2 for a worker of group P2 (eq. (8)).
 * The side information is y_i = side[i] * side_scale, so `side` may be the
 * running SUM of the gradients decoded so far and side_scale = 1/count (the
 * "update the mean" step of Algorithm 2).  With the encoder's alpha:
 *   q^_i = m_i + M rint((fma(y_i, a, v_i) - m_i)/M),  a = alpha * (1/Delta_b)
 *   g~_i = Delta_b ((float)q^_i - v_i)                                 if alpha == 1
 *   g~_i = fma(1 - alpha^2, y_i, alpha * (Delta_b ((float)q^_i - v_i)))  otherwise
 * (eq. (8): y + alpha (r - Q2(r)); 1 - alpha^2 is formed in binary64 and rounded).
 * accumulate as in ndq_dq_decode; out may be the same buffer as side (in-place
 * update of the running sum), but must not overlap it otherwise. */
int ndq_nested_decode(const void* codes, size_t n, uint32_t M, float alpha, uint32_t bucket,
                      const float* steps, const ndq_dither* d, const float* side,
                      float side_scale, float* out, int accumulate, void* stream);

/* Parameter selection for nested workers (Thm 4 and the last paragraph of Sec. 3.2);
 * plain host arithmetic.  ndq_alpha_for_equal_variance: alpha = sqrt(1 -
 * Delta_1^2/(12 sigma_z^2)), the shrinkage that gives NDQSG the variance
 * Delta_1^2/12 of DQSG (0 when the argument is not positive: the side
 * information alone is already better).  ndq_decode_error_bound: Thm 4's bound
 * Delta_1^2/(3 Delta_2^2) + 4 alpha^2 sigma_z^2/Delta_2^2 on the probability of a
 * coset decode error, Delta_2 = M Delta_1.  ndq_nesting_ratio_for_error: the
 * smallest nesting ratio M in [2, 256] (fewest bits per code) for which that
 * bound is at most p_max; 0 when even M = 256 does not reach it or an argument
 * is out of range (delta1 <= 0, alpha outside [0, 1], sigma_z2 < 0, p_max <= 0). */
double ndq_alpha_for_equal_variance(double delta1, double sigma_z2);
double ndq_decode_error_bound(double delta1, uint32_t M, double alpha, double sigma_z2);
uint32_t ndq_nesting_ratio_for_error(double delta1, double alpha, double sigma_z2, double p_max);

/* Estimate of n*sigma_z^2 for that selection (Thm 4's model g = y + z): out[0] =
 * sum_i (a_i - b_i)^2 in binary64, with a fixed reduction order (the same inputs
 * give the same bits).  a, b: n floats each (device, 16-byte aligned); workspace:
 * ndq_sqdiff_workspace() bytes of device memory (8-byte aligned) the call may
 * overwrite; out: one double (device). */
size_t ndq_sqdiff_workspace(void);
int ndq_sqdiff(const float* a, const float* b, size_t n, double* workspace, double* out,
               void* stream);

/* ndq_sqdiff for callers that cannot allocate device memory (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): the same
 * kernels, arguments, result bits and errors, but the partial sums live in
 * ndq_sqdiff_workspace() = 8192 bytes of device memory that the library itself
 * holds in a static array, on every GPU it runs on, until the process ends.  The
 * call allocates and frees nothing.  n >= 2^40 is refused with NDQ_EUNSUPPORTED
 * (the fixed grid and the array are sized for vectors below that).  The first
 * call on a device looks up the array's address on that device (no allocation;
 * make that call outside a graph capture); NDQ_ELAUNCH if the runtime refuses.
 * All calls on one GPU share the array -- every call overwrites all of it before
 * reading it, so nothing needs clearing, but two calls that overlap in time on
 * one GPU (different streams) race; calls on one stream are safe. */
int ndq_sqdiff_static(const float* a, const float* b, size_t n, double* out, void* stream);

/* Server side of Algorithm 1, last step: out_i = scale * sum_w gs[w][i], summed
 * in ascending w.  gs: HOST array of W device pointers (1 <= W <= 1024), each n
 * floats; out may be one of the inputs only if W <= 32. */
int ndq_aggregate(const float* const* gs, uint32_t W, size_t n, float scale, float* out,
                  void* stream);

/* One worker's message as the server holds it (Algorithm 2, "Server"): the packed
 * codes and steps it sent (DEVICE pointers), how they were made, and its dither. */
typedef enum { NDQ_WORKER_DQ = 0, NDQ_WORKER_NESTED = 1 } ndq_worker_kind;
typedef struct {
    const void* codes;      /* ndq_packed_bytes(n, ndq_code_bits(levels_or_M)) bytes   */
    const float* steps;     /* ndq_num_buckets(n, bucket) floats                        */
    uint32_t kind;          /* ndq_worker_kind: group P1 (DQSG) or group P2 (nested)    */
    uint32_t levels_or_M;   /* levels for a DQSG worker, M for a nested worker          */
    float alpha;            /* nested worker: its shrinkage factor in (0,1]; else unused */
    ndq_dither dither;
} ndq_worker;

/* The whole server loop of Algorithm 2 in one pass over the elements.  With S the
 * running sum and c the number of workers folded in so far (S = 0, c = 0 at the
 * start), for p = 0 .. W-1 in the given order:
 *     DQSG worker  : S_i <- g~_p,i if c == 0, else S_i + g~_p,i   (as ndq_dq_decode)
 *     nested worker: y_i = S_i * (1/c);  S_i <- S_i + g~_p,i      (as ndq_nested_decode
 *                    with side = out = S, side_scale = 1/c, its alpha, accumulate)
 *     c <- c + 1
 * and finally out_i = S_i if scale == 1, else scale * S_i.  Element for element
 * this is the result of the corresponding sequence of ndq_dq_decode /
 * ndq_nested_decode calls (and ndq_aggregate for the scale), but S stays in
 * registers: the codes are read once and out is written once.
 * workers: HOST array of W entries (1 <= W <= 1024), the first must be a DQSG
 * worker; all share n and bucket.  out: n floats, written only. */
int ndq_decode_chain(const ndq_worker* workers, uint32_t W, size_t n, uint32_t bucket,
                     float scale, float* out, void* stream);

/* Dense base-L stream.  Table 1 (Sec. 4) counts log2(L) bits per index (1.585 for
 * three levels); the fixed-width stream spends ceil(log2 L).  The dense stream
 * stores k = ndq_dense_group(L) = max{k : L^k <= 2^32} indices per 32-bit word as
 * the number sum_j c_j L^j (first index = lowest digit; the last group is
 * filled with zero digits; zero words pad the stream to ndq_dense_bytes(n, L), a
 * multiple of 16): 1.6 bits per index for L = 3.  `levels` is L of a DQSG worker
 * or M of a nested one; every index must be < levels.
 * ndq_dense_pack:   codes (fixed-width stream, ndq_packed_bytes(n, ndq_code_bits(
 *                   levels)) bytes) -> dense_out (ndq_dense_bytes(n, levels) bytes)
 * ndq_dense_unpack: the inverse; codes_out is fully written, padding zero. */
uint32_t ndq_dense_group(uint32_t levels);
size_t ndq_dense_bytes(size_t n, uint32_t levels);
int ndq_dense_pack(const void* codes, size_t n, uint32_t levels, void* dense_out, void* stream);
int ndq_dense_unpack(const void* dense, size_t n, uint32_t levels, void* codes_out, void* stream);

/* Histogram and empirical entropy of a packed code stream (Sec. 4: the bits left
 * after entropy coding are reported through the entropy of the transmitted
 * indices).  hist_out: 2^bits uint64 (device, 8-byte aligned), hist_out[c] = number
 * of the n codes equal to c.  codes: the ndq_packed_bytes(n, bits) bytes of the
 * stream (device, 16-byte aligned; all of them may be read); what the padding
 * holds is not counted and need not be zero.  entropy_out: one
 * double (device) = -sum_c p_c log2 p_c in bits per code, p_c = hist_out[c]/n
 * (0 when n == 0); may be NULL to get the histogram only.  bits in [1,8].
 * Unlike the other calls this one also runs for n == 0 (it clears its outputs). */
int ndq_code_entropy(const void* codes, size_t n, uint32_t bits, uint64_t* hist_out,
                     double* entropy_out, void* stream);

/* Static, human-readable text for a status code. */
const char* ndq_strerror(int rc);

#ifdef __cplusplus
}
#endif
#endif /* NDQ_H */
