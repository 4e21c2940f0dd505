/*
 * dq.h -- C ABI of the double-quantization hot path on one AMD MI355X (gfx950).
 *
 * Method: Yu, Wu, Huang, "Double Quantization for Communication-Efficient
 * Distributed Optimization" (arXiv 1805.10111): AsyLPG (Alg. 1), Sparse-AsyLPG
 * (Alg. 2), Acc-AsyLPG (Alg. 3) for  min_x P(x) = f(x) + h(x)  (eq. (1)) with
 *   f_i(x) = log(1 + exp(-y_i a_i.x)) + (l2/2)||x||^2,   h(x) = l1 ||x||_1 .
 * The M workers of the parameter-server network are a batch dimension: every
 * entry point that takes M processes M workers (rows) in one launch.
 *
 * Conventions (all entry points)
 *  - Every data pointer is a DEVICE pointer unless the comment says "host".
 *    The dq_problem struct itself lives in host memory and holds device pointers.
 *  - The caller owns every buffer.  The library allocates nothing, frees
 *    nothing, and keeps no state between calls except a thread-local record of
 *    the last HIP error (dq_last_device_error) and the fact that a kernel's
 *    launch attribute (its on-chip memory limit) has been raised, which happens
 *    once per process on first use and is safe from concurrent threads.  No
 *    environment variable is read.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Calls only enqueue work and return; results, including scalars (delta,
 *    norms, counts, status), land in device memory.  The caller synchronises.
 *  - Return value: DQ_OK, or a negative DQ_ERR_* code; on error nothing has
 *    been enqueued unless the code is DQ_ERR_DEVICE.
 *  - Alignment: vectors of floats / words that are read or written with
 *    128-bit accesses must be 16-byte aligned and row strides (`ld`, `lda`,
 *    in elements) multiples of 4; the comments say where this is required.
 *  - b is the number of bits per coordinate.  Packed buffers: any b in [2,16] for
 *    dq_quantize_pack, dq_unpack_dequant_sum and the model message (b_x); gradient
 *    messages of the worker / master calls use b in {2,4,8} (or 32 = float32, not
 *    quantized); unpacked int8 codes support any b in [2,8].
 *  - `status` (nullable) is a device uint32 that is OR-ed into, never cleared:
 *    bit 0 = a scale delta was not finite (NaN/Inf in the input vector).
 *  - Random streams are addressed, not stateful: (seed, iter, worker, tag,
 *    coordinate) names one variate; the same address gives the same variate in
 *    any call, any launch shape.  Generator: Philox4x32-10; key = halves of
 *    seed; counter = (coordinate/4, iter, worker, tag); variate = word
 *    coordinate%4; uniform = (word >> 8) * 2^-24.
 */
#ifndef DQ_H_
#define DQ_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DQ_OK                0
#define DQ_ERR_INVALID_ARG  (-1)  /* null / misaligned pointer, size <= 0, b out of range */
#define DQ_ERR_UNSUPPORTED  (-2)  /* valid request the library has no kernel for */
#define DQ_ERR_WORKSPACE    (-3)  /* workspace smaller than dq_workspace_bytes() */
#define DQ_ERR_DEVICE       (-4)  /* a HIP call failed; see dq_last_device_error() */

/* Stream tags: which random decision a variate is used for. */
#define DQ_TAG_GRAD      0u   /* rounding of a worker's gradient (Alg. 1, worker (ii))     */
#define DQ_TAG_MODEL     1u   /* rounding of the model (Alg. 1, master (i))                */
#define DQ_TAG_SPARSIFY  2u   /* Bernoulli keep decisions of eq. (3)                       */
#define DQ_TAG_SAMPLE    3u   /* mini-batch sampling (Alg. 1, worker (i))                  */
#define DQ_MASTER_ID     0xFFFFFFFFu   /* worker id used for the master's own stream       */

/* Finite-sum problem of eq. (1) with logistic loss (Section 5.1).
 * layout 0: dense row-major features, row i at dense + i*lda, lda % 4 == 0, lda >= d,
 *           dense 16-byte aligned and n*lda floats long (the padding of a row may be read, never used).
 * layout 1: CSR; indptr[n+1], indices sorted and unique within a row; indices and values must
 *           be non-null even when the matrix has no nonzeros (they are then never read).
 * y[n] holds +1/-1.  l2 multiplies ||x||^2/2 inside every f_i (smooth part),
 * l1 multiplies ||x||_1 in h (handled by the prox). */
typedef struct dq_problem {
    int32_t layout;
    int64_t n, d;
    const float *dense;
    int64_t lda;
    const int64_t *indptr;
    const int32_t *indices;
    const float *values;
    const float *y;
    float l2, l1;
} dq_problem;

/* Operations that need a workspace (argument of dq_workspace_bytes). */
#define DQ_OP_FULL_GRAD    1
#define DQ_OP_VR_GRAD      2   /* dq_vr_grad, dq_worker_step and dq_run_rounds (which also keeps data there between the
                                  rounds of a call) */
#define DQ_OP_WORKER_STEP  3   /* one dq_vr_grad or dq_worker_step call alone: never more than DQ_OP_VR_GRAD */

const char *dq_version(void);
/* Last hipError_t (as int) seen by this thread inside the library, 0 if none. */
int32_t dq_last_device_error(void);
/* Bytes of device workspace `op` needs for this problem with M workers of batch B
 * (a multiple of 16, possibly 0; negative = DQ_ERR_*).  Workspaces are 16-byte aligned.
 * Limits that make a problem DQ_ERR_UNSUPPORTED: dense rows wider than 16384 floats; CSR with 2^20
 * columns or more. */
int64_t dq_workspace_bytes(int32_t op, const dq_problem *prob /*host*/, int64_t M, int64_t B);
/* Zero-fills a workspace (optional: no operation needs initialised workspace memory;
 * provided so that a caller can keep its buffers defined).  Two calls that share a
 * workspace must not run concurrently.  ws_bytes must be a multiple of 16. */
int32_t dq_workspace_init(void *ws, int64_t ws_bytes, void *stream);

/* ---- Section 3.1: the (delta, b) representation and the quantizer Q ------------- */

/* absmax_out[m] = ||v_m||_inf for M rows v_m = v + m*ld of length d
 * (numerator of delta in Alg. 1, master (i) and worker (ii)).
 * A NaN anywhere in a row gives a NaN result (max over the magnitude bit patterns). */
int32_t dq_absmax(const float *v, int64_t d, int64_t M, int64_t ld, float *absmax_out, void *stream);

/* Stochastic quantization Q_(delta,b) of Section 3.1, coordinate-wise, with
 * delta_m = ||v_m||_inf / (2^(b-1)-1).  codes_out[m*ld_codes + i] = k with
 * Q(v_mi) = k*delta_m.  Row m uses the stream (seed, iter, worker0+m, tag).
 * Per coordinate (float32): t = v*(L/amax), z = floor(t), k = z + [u < t-z],
 * clamped to [-2^(b-1), 2^(b-1)-1].  A row whose delta is zero or below the
 * smallest normal float gives delta 0 and all-zero codes; a non-finite delta
 * gives zero codes and sets status bit 0.
 * absmax: device float[M]; if absmax_given == 0 it is overwritten with
 * ||v_m||_inf first, else it is read as supplied.  delta_out: device float[M]. */
int32_t dq_quantize(const float *v, int64_t d, int64_t M, int64_t ld, int32_t b,
                    float *absmax, int32_t absmax_given,
                    uint64_t seed, uint32_t iter, uint32_t tag, uint32_t worker0,
                    int8_t *codes_out, int64_t ld_codes, float *delta_out,
                    uint32_t *status, void *stream);

/* v_out[m*ld + i] = delta[m] * codes[m*ld_codes + i]  (the value a code represents). */
int32_t dq_dequantize(const int8_t *codes, int64_t ld_codes, const float *delta, int64_t d, int64_t M,
                      float *v_out, int64_t ld, void *stream);

/* Wire format of Section 3.1 (32 + b*d bits per vector: delta plus b bits per
 * coordinate).  Field i of a row = bits [(i*b)%32, (i*b)%32+b) of word
 * floor(i*b/32), two's complement, low bits first; unused tail bits are 0.
 * For a width that does not divide 32 the row is one little-endian bit string with field i at
 * bits [i*b, i*b+b): a field may continue in the low bits of the next word (the model-precision
 * study of Section 5.2 uses b_x from 2 to 11).
 * Rows of packed words have stride ld_words >= ceil(d*b/32).  b in [2,8] here (int8 codes);
 * dq_quantize_pack, dq_unpack_dequant_sum and the model message of the worker and master
 * calls take any width in [2,16]. */
int32_t dq_pack(const int8_t *codes, int64_t ld_codes, int64_t d, int64_t M, int32_t b,
                uint32_t *packed_out, int64_t ld_words, void *stream);
int32_t dq_unpack(const uint32_t *packed, int64_t ld_words, int64_t d, int64_t M, int32_t b,
                  int8_t *codes_out, int64_t ld_codes, void *stream);

/* Sparse message of Section 4.2 (after sparsification most codes are zero): the scale plus,
 * per NONZERO coordinate in ascending order, an entry of ceil(log2 d) position bits (low) and
 * the b-bit two's-complement code (high), entries back to back, low bits first across 32-bit
 * words: 32 + nnz*(ceil(log2 d) + b) bits in all.  dq_sparse_stream_words(d, b) is the row
 * capacity (every coordinate nonzero).  dq_sparse_encode turns M rows of dense packed codes
 * into M streams (stride ld_stream >= capacity, words past the used ones zero) and writes
 * nnz_out[M]; dq_sparse_decode is the inverse (packed_out rows fully rewritten).  b in {2,4,8};
 * streams of more than 36864 words (144 KB) are DQ_ERR_UNSUPPORTED. */
int64_t dq_sparse_stream_words(int64_t d, int32_t b);
int32_t dq_sparse_encode(const uint32_t *packed, int64_t ld_words, int64_t d, int64_t M, int32_t b,
                         uint32_t *stream_out, int64_t ld_stream, int32_t *nnz_out, void *stream);
int32_t dq_sparse_decode(const uint32_t *stream_in, int64_t ld_stream, const int32_t *nnz, int64_t d, int64_t M,
                         int32_t b, uint32_t *packed_out, int64_t ld_words, void *stream);

/* dq_quantize followed by dq_pack in one pass (same bits as the two calls), for any
 * width b in [2,16] (2, 4 and 8 take the word-aligned fast path).
 * v and packed_out 16-byte aligned; with M > 1, ld % 4 == 0 and ld_words % 4 == 0. */
int32_t dq_quantize_pack(const float *v, int64_t d, int64_t M, int64_t ld, int32_t b,
                         float *absmax, int32_t absmax_given,
                         uint64_t seed, uint32_t iter, uint32_t tag, uint32_t worker0,
                         uint32_t *packed_out, int64_t ld_words, float *delta_out,
                         uint32_t *status, void *stream);

/* Master's receive side (Alg. 1, master (ii), first half): decode M packed
 * gradients and aggregate,  out[i] = scale * sum_{m<M} delta[m]*k_mi,
 * summed in the order m = 0..M-1 with fused multiply-adds, then one multiply
 * by scale (1/M for the mean over a synchronous round of M workers).  b in [2,16]. */
int32_t dq_unpack_dequant_sum(const uint32_t *packed, int64_t ld_words, const float *delta,
                              int64_t d, int64_t M, int32_t b, float scale, float *out, void *stream);

/* ---- sampling, gradients -------------------------------------------------------- */

/* Mini-batch of Alg. 1, worker (i) (Section 5.1 uses mini-batches): for worker
 * m and slot j, idx_out[m*B + j] = floor(word * n / 2^32) with the variate at
 * (seed, iter, worker0+m, DQ_TAG_SAMPLE, j): uniform on {0..n-1}, with replacement. */
int32_t dq_sample_indices(int64_t n, int64_t M, int64_t B, uint64_t seed, uint32_t iter,
                          uint32_t worker0, int32_t *idx_out, void *stream);

/* Epoch prologue (Alg. 1, global gradient computation):
 *   g_out = (1/n) sum_i grad f_i(x) = (1/n) sum_i s_i a_i + l2*x,
 *   s_i = -y_i / (1 + exp(y_i a_i.x)).
 * z_out (nullable, float[n]) receives the margins a_i.x; obj_out (nullable,
 * double[1]) receives P(x) of eq. (1).  Deterministic for a given problem shape (dense features: float32
 * sums in a fixed order; CSR features: the sums over rows are accumulated per column in fixed point -- int32
 * multiples of a power of two chosen so that no sum can overflow, flushed to float32 every 1024 rows -- and do
 * not depend on the order of the additions; a term is rounded to within 2^-31 of the bound of its column's sum). */
int32_t dq_full_grad(const dq_problem *prob /*host*/, const float *x, float *g_out, float *z_out,
                     double *obj_out, void *ws, int64_t ws_bytes, void *stream);

/* Worker step (i) of Alg. 1 for M workers with mini-batches idx[m*B .. m*B+B):
 *   alpha_m = (1/B) sum_{i in I_m} [grad f_i(q) - grad f_i(x_snap)],
 * q = delta_x * (codes unpacked from xq_packed) is the b_x-bit model the worker
 * received (Alg. 1, master (i)), b_x in [2,16]; b_x == 32 means xq_packed holds float32
 * values of the model itself (no quantization; delta_x ignored).
 * model_is_snapshot != 0 is the flag-bit case of Section 4.1 (q = x_snap): alpha = 0.
 * z_snap (nullable) = margins a_i.x_snap cached by dq_full_grad; if NULL they
 * are recomputed.  alpha_out rows have stride ld (ld % 4 == 0, 16-byte aligned).
 * absmax_out[M] = ||alpha_m||_inf; l1norm_out (nullable) [M] = ||alpha_m||_1.
 * CSR features: the sum over the mini-batch is accumulated in fixed point as in dq_full_grad (bit-reproducible;
 * the bound, hence the unit, follows the size of the coefficients, which shrink as q approaches x_snap); a NaN
 * or Inf among the values, labels or cached margins of a mini-batch makes the whole alpha_m NaN. */
int32_t dq_vr_grad(const dq_problem *prob /*host*/, const int32_t *idx, int64_t M, int64_t B,
                   const uint32_t *xq_packed, const float *delta_x, int32_t b_x,
                   int32_t model_is_snapshot, const float *x_snap, const float *z_snap,
                   float *alpha_out, int64_t ld, float *absmax_out, float *l1norm_out,
                   void *ws, int64_t ws_bytes, void *stream);

/* Eq. (3), gradient sparsification (Alg. 2, worker (ii)):
 *   beta_i = Z_i alpha_i / p_i,  Z_i ~ Bernoulli(p_i)  (keep iff u_i < p_i),
 * phi == NULL: the budget of Section 5.1, phi = ||alpha||_1/||alpha||_inf, i.e.
 *   p_i = |alpha_i| / ||alpha||_inf;
 * else p_i = min(1, |alpha_i| * phi[m] / ||alpha_m||_1)  (Lemma 2).
 * Outputs: beta_out (stride ld_out), absmax_out[M] = ||beta_m||_inf,
 * nnz_out[M] = kept coordinates.  Stream tag DQ_TAG_SPARSIFY. */
int32_t dq_sparsify(const float *alpha, int64_t d, int64_t M, int64_t ld, const float *phi,
                    uint64_t seed, uint32_t iter, uint32_t worker0,
                    float *beta_out, int64_t ld_out, float *absmax_out, int32_t *nnz_out, void *stream);

/* The whole worker side of one round, fused (Alg. 1, worker (i)-(ii); with
 * sparsify != 0: Alg. 2, worker (i)-(iii)):  dq_vr_grad -> [dq_sparsify] ->
 * dq_quantize_pack with tag DQ_TAG_GRAD, bit-identical to those calls, without
 * writing alpha to memory (dense features with B > 32: partial sums of alpha pass through
 * `ws`; CSR with a model too wide for the on-chip buffer: alpha is assembled in `ws`; CSR with
 * sparsify != 0 and few workers: the sparsified gradient passes through `ws` between two launches).
 * ws, ws_bytes: at least dq_workspace_bytes(DQ_OP_WORKER_STEP, prob, M, B) bytes (a DQ_OP_VR_GRAD workspace is never
 * smaller).  CSR features whose model fits the on-chip buffer also run without (NULL, 0), in a single launch.  packed_out: M rows of ld_words words; delta_out[M];
 * nnz_out (nullable) [M] = nonzero codes.  alpha_out (nullable): also store alpha.
 * idx == NULL: the mini-batches are sampled inside the kernel, exactly as
 * dq_sample_indices(n, M, B, seed, iter, worker0, .) would produce them.
 * b == 32: no gradient quantization, packed_out rows receive alpha (or beta) as
 * float32 (ld_words >= d) and delta_out = 1.  Gradient widths: b in {2,4,8,32}
 * (others in [2,8]: DQ_ERR_UNSUPPORTED). */
int32_t dq_worker_step(const dq_problem *prob /*host*/, const int32_t *idx, int64_t M, int64_t B,
                       const uint32_t *xq_packed, const float *delta_x, int32_t b_x,
                       int32_t model_is_snapshot, const float *x_snap, const float *z_snap,
                       int32_t sparsify, int32_t b, uint64_t seed, uint32_t iter, uint32_t worker0,
                       uint32_t *packed_out, int64_t ld_words, float *delta_out, int32_t *nnz_out,
                       float *alpha_out, int64_t ld, uint32_t *status,
                       void *ws, int64_t ws_bytes, void *stream);

/* dq_worker_step for callers that cannot allocate device memory or hand over a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): same arguments without ws / ws_bytes, same
 * results bit for bit.  The partial sums and per-worker rows that dq_worker_step passes through `ws` live in a
 * workspace of DQ_STATIC_WS_BYTES bytes built into the library, one copy per GPU, held until the process ends;
 * nothing is allocated or freed by the call.  A problem whose dq_workspace_bytes(DQ_OP_WORKER_STEP, prob, M, B) exceeds
 * DQ_STATIC_WS_BYTES returns DQ_ERR_WORKSPACE and enqueues nothing.  All calls on one GPU share that workspace:
 * calls that may overlap on the GPU (different streams without an ordering between them) race; calls on one
 * stream, or otherwise ordered, are safe, and no call depends on what an earlier one left there. */
#define DQ_STATIC_WS_BYTES  (8ll << 20)
int32_t dq_worker_step_static(const dq_problem *prob /*host*/, const int32_t *idx, int64_t M, int64_t B,
                              const uint32_t *xq_packed, const float *delta_x, int32_t b_x,
                              int32_t model_is_snapshot, const float *x_snap, const float *z_snap,
                              int32_t sparsify, int32_t b, uint64_t seed, uint32_t iter, uint32_t worker0,
                              uint32_t *packed_out, int64_t ld_words, float *delta_out, int32_t *nnz_out,
                              float *alpha_out, int64_t ld, uint32_t *status, void *stream);

/* ---- master --------------------------------------------------------------------- */

/* Master step for one synchronous round of M workers (Alg. 1, master (ii) and (i);
 * Alg. 3 with y != NULL):
 *   u     = scale * sum_m delta[m]*k_m + g_snap                    (as dq_unpack_dequant_sum)
 *   Alg.1: x <- prox_{eta h}(x - eta*u)         prox = soft-threshold at eta*l1
 *   Alg.3: y <- prox_{eta h}(y - eta*u);  x <- x_snap + theta*(y - x_snap);  xsum += x
 * then the new model is quantized to b_x bits with the master's stream
 * (seed, iter, DQ_MASTER_ID, DQ_TAG_MODEL) and packed into xq_packed_out, with
 * delta_x_out[0] its scale and absmax_x_out[0] = ||x||_inf (scratch + output).
 * b == 32: `packed` holds M rows of float32 gradients (stride ld_words, delta
 * ignored).  b_x == 32: no model quantization, xq_packed_out receives x as float32.
 * b in {2,4,8,32}; b_x in [2,16] or 32.  One launch for d <= 8192 with b_x in {2,4,8,32}, else three
 * (update with ||x||_inf, quantize + pack, and a one-word fill before them).
 * All float32, in the order written; x, y, xsum are updated in place. */
int32_t dq_master_step(const uint32_t *packed, int64_t ld_words, const float *delta, int64_t M, int32_t b,
                       float scale, const float *g_snap, float *x, float *y, const float *x_snap,
                       float *xsum, float eta, float theta, float l1, int64_t d,
                       int32_t b_x, uint64_t seed, uint32_t iter,
                       uint32_t *xq_packed_out, float *delta_x_out, float *absmax_x_out,
                       uint32_t *status, void *stream);

/* The master's rule of Alg. 1 (Alg. 3 with y != NULL) taken one received gradient at a time: the M
 * messages are applied in worker order, each as its own update with the full step,
 *   for m:  u = delta[m]*k_m + g_snap;  x <- prox_{eta h}(x - eta*u)
 *           (Alg. 3: y <- prox_{eta h}(y - eta*u);  x <- x_snap + theta*(y - x_snap);  xsum += x, i.e. M terms per call),
 * then the model is quantized and packed once, exactly as in dq_master_step.  Same arguments
 * without `scale`, same limits. */
int32_t dq_master_step_each(const uint32_t *packed, int64_t ld_words, const float *delta, int64_t M, int32_t b,
                            const float *g_snap, float *x, float *y, const float *x_snap,
                            float *xsum, float eta, float theta, float l1, int64_t d,
                            int32_t b_x, uint64_t seed, uint32_t iter,
                            uint32_t *xq_packed_out, float *delta_x_out, float *absmax_x_out,
                            uint32_t *status, void *stream);

/* The two sides of the precision-loss condition on the model quantization (eq. (2); eq. (4) for
 * Alg. 3):  out[0] = E_Q ||Q_(delta_x,b)(x) - x||^2 over the rounding decisions, which is
 * delta_x^2 * sum_i p_i (1 - p_i) (proof of Lemma 5; nothing is sampled), and
 * out[1] = ||x - x_snap||^2.  The condition holds for a given mu iff out[0] <= mu * out[1]
 * (theta_s * mu for Alg. 3).  out: device double[2].  b in [2,16].  Diagnostic, one block. */
int32_t dq_mu_terms(const float *x, const float *x_snap, int64_t d, int32_t b, double *out, void *stream);

/* Parameters of epoch s = 1, 2, ... of Alg. 3 as Section 5.1 sets them: theta_s = 2/(s+2), eta_s = lr/theta_s,
 * both in float32.  theta_out, eta_out: HOST pointers.  s < 1: DQ_ERR_INVALID_ARG. */
int32_t dq_acc_params(float lr, int64_t s, float *theta_out /*host*/, float *eta_out /*host*/);

/* Start of an epoch of Alg. 3:  x_out = x_snap + theta*(y - x_snap)  (= theta*y + (1-theta)*x_snap). */
int32_t dq_acc_mix(const float *y, const float *x_snap, float theta, int64_t d, float *x_out, void *stream);
/* End of an epoch of Alg. 3:  x_snap_out = xsum / m. */
int32_t dq_acc_snapshot(const float *xsum, int64_t m, int64_t d, float *x_snap_out, void *stream);

/* ---- message sizes ---------------------------------------------------------------- */

/* Bits on the wire of one message (host arithmetic, nothing is enqueued); negative = DQ_ERR_INVALID_ARG.
 * DQ_MSG_DENSE : Section 3.1, a vector of d coordinates at b bits each plus its 32-bit scale, 32 + b*d;
 *                b == 32 (not quantized): 32*d.  nnz is ignored.
 * DQ_MSG_FLAG  : Section 4.1, the model equals the snapshot and the master sends one flag bit: 1.
 * DQ_MSG_SPARSE: Section 4.2, the scale plus ceil(log2 d) position bits and b value bits per nonzero code,
 *                32 + nnz*(ceil(log2 d) + b); b == 32: nnz*(ceil(log2 d) + 32) (no scale).  0 <= nnz <= d.
 * b in [2,16] or 32. */
#define DQ_MSG_DENSE   0
#define DQ_MSG_FLAG    1
#define DQ_MSG_SPARSE  2
int64_t dq_message_bits(int32_t kind, int64_t d, int32_t b, int64_t nnz);

/* ---- inner loop ------------------------------------------------------------------ */

#define DQ_ALGO_ASYLPG  0   /* Alg. 1 */
#define DQ_ALGO_SPARSE  1   /* Alg. 2: sparsify before quantizing */
#define DQ_ALGO_ACC     2   /* Alg. 3: momentum */

/* Settings of a run (host struct). */
typedef struct dq_run_config {
    int32_t algo;        /* DQ_ALGO_* */
    int64_t M, B;        /* workers per round, mini-batch per worker */
    int32_t b_x, b;      /* bits of the model message and of the gradient message (32 = not quantized) */
    int64_t m;           /* rounds per epoch */
    uint64_t seed;
    int32_t tau;         /* emulated bounded delay (Assumption 3): 0 = every worker reads the current model;
                            tau > 0: the workers form tau+1 contiguous groups, worker w belongs to group
                            g = floor(w*(tau+1)/M) and reads the model message of round max(0, t-g) */
    int32_t each;        /* 0: one master update per round with the mean of the M gradients (dq_master_step,
                            scale 1/M); 1: one update per received gradient (dq_master_step_each); Alg. 3 then
                            averages m*M iterates for its snapshot */
} dq_run_config;

/* Device buffers of a run (host struct holding device pointers; all caller-owned).
 * x, x_snap, g_snap: float[d].  y, xsum: float[d], Alg. 3 only.  z_snap: float[n] margins at the
 * snapshot from dq_full_grad, nullable.  xq: ring of tau+1 model messages, slot s at
 * xq + s*xq_stride_words (each ceil(d*b_x/32) words, or d floats; 16-byte aligned slots);
 * delta_x: float[tau+1], one scale per slot; absmax_x: float[2] (scratch: the largest magnitude of the model after
 * the last two rounds, in alternating entries).  The message of round t lives in
 * slot t mod (tau+1).  packed: M rows of ld_words words; delta: float[M];
 * nnz: int32[m*M] nonzero codes per round and worker (written by Alg. 2 only), nullable.  ws: DQ_OP_VR_GRAD workspace
 * (scratch of the call: between the rounds of one call it also carries what one round leaves for the next, e.g. the
 * sparsified gradients that the master quantizes and, on CSR features, the decoded model minus the snapshot and the
 * next round's mini-batches -- row numbers drawn, extents, labels and entries read -- laid out by the round before).
 * wire (nullable, Alg. 2 with b in {2,4,8} only): M rows of ld_wire >= dq_sparse_stream_words(d, b) words.  When
 * given, every round really sends the sparse message of Section 4.2: the workers' packed codes are encoded into
 * `wire` (dq_sparse_encode), then the master's input is rebuilt from `wire` alone (dq_sparse_decode); wire_nnz:
 * int32[M], required with wire. */
typedef struct dq_run_state {
    float *x, *x_snap, *y, *xsum, *g_snap;
    const float *z_snap;
    uint32_t *xq;
    float *delta_x, *absmax_x;
    uint32_t *packed;
    int64_t ld_words;
    float *delta;
    int32_t *nnz;
    uint32_t *status;
    void *ws;
    int64_t ws_bytes;
    int64_t xq_stride_words;
    uint32_t *wire;
    int64_t ld_wire;
    int32_t *wire_nnz;
} dq_run_state;

/* Enqueues rounds t0 .. t0+rounds-1 of epoch `epoch` (0-based) of Alg. 1, 2 or 3: per round the
 * worker side (dq_worker_step with in-kernel sampling; the flag-bit case of Section 4.1 at the
 * first round of an epoch whose start equals the snapshot) and the master side (dq_master_step with
 * the mean over the M workers, or dq_master_step_each; model re-quantized for the next round).  Random streams use
 * iter = epoch*m + t.  eta, theta: step size and momentum weight of this epoch (theta unused by
 * Alg. 1/2; for Alg. 3 they are dq_acc_params(lr, epoch + 1, ...)).  The epoch prologue (dq_full_grad,
 * dq_acc_mix / copy) and epilogue stay with the caller.  Everything is validated before the first launch
 * (null or misaligned state pointers, a workspace smaller than dq_workspace_bytes(DQ_OP_VR_GRAD, prob, M, B),
 * which covers every worker group of a delayed run).  worker_events (host array, nullable): 2*rounds hipEvent_t handles created by the caller; for
 * round k the pair [2k], [2k+1] receives the start and the end time of the kernel of the worker step
 * that streams the feature rows (its first kernel; for CSR its only one; with tau > 0 the one of the
 * first worker group): they are the start and stop events of that launch (hipExtLaunchKernel), so
 * hipEventElapsedTime over the pair is the kernel's own duration.  A flag-bit round leaves its pair
 * untouched; a pair of null handles makes that round's launch a plain one.  Pass null while `stream` is being
 * captured into a graph. */
int32_t dq_run_rounds(const dq_problem *prob /*host*/, const dq_run_config *cfg /*host*/, const dq_run_state *st /*host*/,
                      int64_t epoch, int64_t t0, int64_t rounds, float eta, float theta,
                      void **worker_events /*host*/, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* DQ_H_ */
