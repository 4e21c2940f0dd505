/*
 * dq_oracle.c -- TEST INFRASTRUCTURE, not a product path.
 *
 * Plain, slow, single-threaded CPU reference for the double-quantization hot
 * path of "Double Quantization for Communication-Efficient Distributed
 * Optimization" (Yu, Wu, Huang; arXiv 1805.10111).  It is written to be checked
 * against the paper by eye: one function per step, the steps in the paper's
 * order and notation, no blocking, no fusion, no vectorisation.  Floating point
 * that the paper leaves to real arithmetic (margins, sigmoids, gradient sums) is
 * done in double and rounded to float once; the quantizer, sparsifier and master
 * update are elementwise float32 procedures whose operation order is spelled
 * out, because their results are integers / grid points that must be
 * reproducible bit for bit.
 *
 * Only tests, the smoke check and the benchmark's CPU-baseline leg may call
 * this file.  It shares no code, header, table or constant generator with the
 * GPU library.
 *
 * Build: gcc -O2 -std=c11 -ffp-contract=off -fPIC -shared dq_oracle.c -lm
 * (no fast-math, no flush-to-zero).
 *
 * Parity pins (tests/test_oracle_*.py): every exported function below is pinned
 * to something other than itself; none is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <float.h>

/* ------------------------------------------------------------------------- */
/* Counter-based random numbers: Philox4x32-10 (Salmon, Moraes, Dror, Shaw,   */
/* "Parallel random numbers: as easy as 1, 2, 3", SC'11), written from its    */
/* published definition.  The paper only says "with probability"; the stream  */
/* addressing below (what goes in the key and the counter) is a choice made here. */
/* ------------------------------------------------------------------------- */

enum { REF_TAG_GRAD = 0, REF_TAG_MODEL = 1, REF_TAG_SPARSIFY = 2, REF_TAG_SAMPLE = 3 };

void ref_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    const uint32_t MUL0 = 0xD2511F53u, MUL1 = 0xCD9E8D57u; /* round multipliers */
    const uint32_t WEYL0 = 0x9E3779B9u, WEYL1 = 0xBB67AE85u; /* key increments  */
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)MUL0 * c0;
        uint64_t p1 = (uint64_t)MUL1 * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += WEYL0; k1 += WEYL1;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* The 32-bit random word that belongs to one coordinate of one stream.
 * key = (low, high half of seed); counter = (coord/4, iter, worker, tag);
 * the word is output number coord%4 of that block. */
uint32_t ref_random_word(uint64_t seed, uint32_t iter, uint32_t worker, uint32_t tag, uint64_t coord)
{
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t ctr[4] = { (uint32_t)(coord >> 2), iter, worker, tag };
    uint32_t out[4];
    ref_philox4x32_10(ctr, key, out);
    return out[coord & 3u];
}

/* Uniform on {0,1,...,2^24-1}/2^24: the top 24 bits of the word. */
static float uniform24(uint32_t word) { return (float)(word >> 8) * 0x1p-24f; }

float ref_uniform(uint64_t seed, uint32_t iter, uint32_t worker, uint32_t tag, uint64_t coord)
{
    return uniform24(ref_random_word(seed, iter, worker, tag, coord));
}

/* u[i] = uniform of coordinate coord0 + i, i < count. */
void ref_uniform_range(uint64_t seed, uint32_t iter, uint32_t worker, uint32_t tag, uint64_t coord0,
                       int64_t count, float *u)
{
    for (int64_t i = 0; i < count; ++i) u[i] = ref_uniform(seed, iter, worker, tag, coord0 + (uint64_t)i);
}

/* Mini-batch sampling: B indices, uniform on {0..n-1}, with replacement
 * (the worker "stochastically samples a data-point", Alg. 1, worker (i); the
 * experiments use a mini-batch, Section 5.1).  idx = floor(word * n / 2^32). */
void ref_sample_indices(int64_t n, int64_t B, uint64_t seed, uint32_t iter, uint32_t worker,
                        int32_t *idx_out)
{
    for (int64_t j = 0; j < B; ++j) {
        uint32_t w = ref_random_word(seed, iter, worker, REF_TAG_SAMPLE, (uint64_t)j);
        idx_out[j] = (int32_t)(((uint64_t)w * (uint64_t)n) >> 32);
    }
}

/* ------------------------------------------------------------------------- */
/* Section 3.1: low-precision representation (delta, b) and the quantizer Q.  */
/* ------------------------------------------------------------------------- */

/* Largest positive level index 2^(b-1)-1 of dom(delta,b). */
static int level_max(int b) { return (1 << (b - 1)) - 1; }

float ref_absmax(const float *v, int64_t d)
{
    float m = 0.0f;
    for (int64_t i = 0; i < d; ++i) {
        float a = fabsf(v[i]);
        if (a > m || isnan(a)) m = a;
        if (isnan(m)) return m;
    }
    return m;
}

/* Scale of Alg. 1, master (i) and worker (ii): delta = ||v||_inf / (2^(b-1)-1).
 * Returns 0 for a vector whose scale is not a normal float (all-zero vector,
 * or so tiny that delta underflows): such a vector quantizes to all zeros. */
float ref_delta(float amax, int b)
{
    float delta = amax / (float)level_max(b);
    if (!(delta >= FLT_MIN)) return isnan(delta) ? delta : 0.0f;
    return delta;
}

/* Q_(delta,b) applied coordinate-wise (Section 3.1 rules (i) and (ii)), with
 * delta chosen from the max norm.  codes[i] is the integer k with
 * Q(v_i) = k*delta, k in {-2^(b-1), ..., 2^(b-1)-1}.  u[i] in [0,1) is the
 * uniform variate that decides coordinate i.
 *
 * Per coordinate, in float32: t = v_i * (L/amax) locates v_i on the grid in
 * units of delta; z = floor(t) is the grid point below; the point above is
 * taken with probability p = t - z, i.e. when u < p (rule (i)); the result is
 * clamped to the end points (rule (ii), reachable only through rounding of t).
 * Returns 1 if the scale is not finite (NaN/Inf in v), else 0; codes are then 0. */
int ref_quantize_given_uniforms_wide(const float *v, int64_t d, int b, const float *u, int32_t *codes,
                                     float *delta_out)
{
    const int L = level_max(b);
    const int kmin = -(1 << (b - 1)), kmax = L;
    float amax = ref_absmax(v, d);
    float delta = ref_delta(amax, b);
    *delta_out = delta;
    if (!(delta > 0.0f) || isinf(delta)) {          /* zero, NaN or Inf scale */
        for (int64_t i = 0; i < d; ++i) codes[i] = 0;
        return (isnan(delta) || isinf(delta)) ? 1 : 0;
    }
    const float inv_delta = (float)L / amax;
    for (int64_t i = 0; i < d; ++i) {
        float t = v[i] * inv_delta;
        float z = floorf(t);
        float p = t - z;                              /* exact in float32 */
        int k = (int)z + (u[i] < p ? 1 : 0);
        if (k < kmin) k = kmin;
        if (k > kmax) k = kmax;
        codes[i] = k;
    }
    return 0;
}

/* Codes of at most 8 bits in one byte each (2 <= b <= 8). */
int ref_quantize_given_uniforms(const float *v, int64_t d, int b, const float *u, int8_t *codes,
                                float *delta_out)
{
    int32_t *wide = (int32_t *)malloc(sizeof(int32_t) * (size_t)(d > 0 ? d : 1));
    int st = ref_quantize_given_uniforms_wide(v, d, b, u, wide, delta_out);
    for (int64_t i = 0; i < d; ++i) codes[i] = (int8_t)wide[i];
    free(wide);
    return st;
}

/* The same with u[i] drawn from stream (seed, iter, worker, tag) at coordinate i. */
int ref_quantize_wide(const float *v, int64_t d, int b, uint64_t seed, uint32_t iter, uint32_t worker,
                      uint32_t tag, int32_t *codes, float *delta_out)
{
    float *u = (float *)malloc(sizeof(float) * (size_t)(d > 0 ? d : 1));
    for (int64_t i = 0; i < d; ++i) u[i] = ref_uniform(seed, iter, worker, tag, (uint64_t)i);
    int st = ref_quantize_given_uniforms_wide(v, d, b, u, codes, delta_out);
    free(u);
    return st;
}

int ref_quantize(const float *v, int64_t d, int b, uint64_t seed, uint32_t iter, uint32_t worker,
                 uint32_t tag, int8_t *codes, float *delta_out)
{
    float *u = (float *)malloc(sizeof(float) * (size_t)(d > 0 ? d : 1));
    for (int64_t i = 0; i < d; ++i) u[i] = ref_uniform(seed, iter, worker, tag, (uint64_t)i);
    int st = ref_quantize_given_uniforms(v, d, b, u, codes, delta_out);
    free(u);
    return st;
}

/* Value represented by a code: k*delta. */
void ref_dequantize(const int8_t *codes, float delta, int64_t d, float *v_out)
{
    for (int64_t i = 0; i < d; ++i) v_out[i] = delta * (float)codes[i];
}

/* Wire format of the b bits per coordinate (Section 3.1: 32 + b*d bits per
 * vector).  Field i occupies bits [(i*b)%32, (i*b)%32+b) of 32-bit word
 * floor(i*b/32), two's complement, b in {2,4,8}; unused tail bits are zero. */
int64_t ref_packed_words(int64_t d, int b) { return (d * b + 31) / 32; }

void ref_pack(const int8_t *codes, int64_t d, int b, uint32_t *words)
{
    int64_t nw = ref_packed_words(d, b);
    uint32_t mask = (1u << b) - 1u;
    for (int64_t w = 0; w < nw; ++w) words[w] = 0;
    for (int64_t i = 0; i < d; ++i) {
        int64_t bit = i * b;
        words[bit / 32] |= ((uint32_t)(int32_t)codes[i] & mask) << (bit % 32);
    }
}

void ref_unpack(const uint32_t *words, int64_t d, int b, int8_t *codes)
{
    uint32_t mask = (1u << b) - 1u;
    for (int64_t i = 0; i < d; ++i) {
        int64_t bit = i * b;
        uint32_t f = (words[bit / 32] >> (bit % 32)) & mask;
        int k = (int)f;
        if (f >> (b - 1)) k -= (1 << b);              /* sign extension */
        codes[i] = (int8_t)k;
    }
}

/* Any width 2 <= b <= 16 (the model-precision study of Section 5.2 varies b_x from 2 to 11):
 * the same layout, field i at bits [i*b, i*b+b) of the row read as one little-endian bit
 * string; a field that does not fit in the rest of its word continues in the low bits of the
 * next word. */
void ref_pack_wide(const int32_t *codes, int64_t d, int b, uint32_t *words)
{
    int64_t nw = ref_packed_words(d, b);
    uint32_t mask = (1u << b) - 1u;
    for (int64_t w = 0; w < nw; ++w) words[w] = 0;
    for (int64_t i = 0; i < d; ++i) {
        int64_t bit = i * b;
        int sh = (int)(bit % 32);
        uint32_t f = (uint32_t)codes[i] & mask;
        words[bit / 32] |= f << sh;
        if (sh + b > 32) words[bit / 32 + 1] |= f >> (32 - sh);
    }
}

void ref_unpack_wide(const uint32_t *words, int64_t d, int b, int32_t *codes)
{
    uint32_t mask = (1u << b) - 1u;
    for (int64_t i = 0; i < d; ++i) {
        int64_t bit = i * b;
        int sh = (int)(bit % 32);
        uint32_t f = words[bit / 32] >> sh;
        if (sh + b > 32) f |= words[bit / 32 + 1] << (32 - sh);
        f &= mask;
        int k = (int)f;
        if (f >> (b - 1)) k -= (1 << b);              /* sign extension */
        codes[i] = k;
    }
}

void ref_dequantize_wide(const int32_t *codes, float delta, int64_t d, float *v_out)
{
    for (int64_t i = 0; i < d; ++i) v_out[i] = delta * (float)codes[i];
}

/* Section 4.2: a sparsified message lists only the nonzero coordinates, each as its
 * position (ceil(log2 d) bits) followed by its b-bit value.  Entry e occupies bits
 * [e*E, (e+1)*E) of the stream, E = posbits + b, low bits first across 32-bit words;
 * position in the low posbits bits of the entry, two's-complement code above it. */
int ref_position_bits(int64_t d)
{
    int bits = 0;
    while (((int64_t)1 << bits) < d) ++bits;        /* ceil(log2 d); the paper's logarithm is base 2 */
    return bits;
}

int64_t ref_sparse_encode(const int8_t *codes, int64_t d, int b, uint32_t *words, int64_t capacity_words)
{
    const int pb = ref_position_bits(d), E = pb + b;
    int64_t nnz = 0;
    for (int64_t w = 0; w < capacity_words; ++w) words[w] = 0;
    for (int64_t i = 0; i < d; ++i) {
        if (codes[i] == 0) continue;
        uint64_t entry = (uint64_t)i | ((uint64_t)((uint32_t)(int32_t)codes[i] & ((1u << b) - 1u)) << pb);
        int64_t bit = nnz * E;
        for (int k = 0; k < E; ++k, ++bit)
            if ((entry >> k) & 1u) words[bit / 32] |= 1u << (bit % 32);
        ++nnz;
    }
    return nnz;
}

void ref_sparse_decode(const uint32_t *words, int64_t nnz, int64_t d, int b, int8_t *codes)
{
    const int pb = ref_position_bits(d), E = pb + b;
    for (int64_t i = 0; i < d; ++i) codes[i] = 0;
    for (int64_t e = 0; e < nnz; ++e) {
        uint64_t entry = 0;
        int64_t bit = e * E;
        for (int k = 0; k < E; ++k, ++bit)
            entry |= (uint64_t)((words[bit / 32] >> (bit % 32)) & 1u) << k;
        int64_t pos = (int64_t)(entry & (((uint64_t)1 << pb) - 1));
        uint32_t f = (uint32_t)(entry >> pb) & ((1u << b) - 1u);
        int k = (int)f;
        if (f >> (b - 1)) k -= (1 << b);
        codes[pos] = (int8_t)k;
    }
}

/* ------------------------------------------------------------------------- */
/* Problem (1): P(x) = f(x) + h(x), f = (1/n) sum f_i,                        */
/*   f_i(x) = log(1 + exp(-y_i a_i.x)) + (l2/2)||x||^2   (smooth part)        */
/*   h(x)   = l1 ||x||_1                                  (prox part)         */
/* Section 5.1 uses logistic regression with L1 and L2 weights; putting the   */
/* L2 term in f and the L1 term in h is the reading taken here.                */
/* Rows are dense (row-major, leading dimension lda) or CSR.                  */
/* ------------------------------------------------------------------------- */

typedef struct {
    int32_t layout;          /* 0 dense, 1 CSR */
    int64_t n, d;
    const float *dense; int64_t lda;
    const int64_t *indptr; const int32_t *indices; const float *values;
    const float *y;
    float l2, l1;
} ref_problem;

static double row_dot(const ref_problem *P, int64_t i, const float *x)
{
    double s = 0.0;
    if (P->layout == 0) {
        const float *a = P->dense + i * P->lda;
        for (int64_t j = 0; j < P->d; ++j) s += (double)a[j] * (double)x[j];
    } else {
        for (int64_t e = P->indptr[i]; e < P->indptr[i + 1]; ++e)
            s += (double)P->values[e] * (double)x[P->indices[e]];
    }
    return s;
}

static void row_axpy(const ref_problem *P, int64_t i, double coef, double *acc)
{
    if (P->layout == 0) {
        const float *a = P->dense + i * P->lda;
        for (int64_t j = 0; j < P->d; ++j) acc[j] += coef * (double)a[j];
    } else {
        for (int64_t e = P->indptr[i]; e < P->indptr[i + 1]; ++e)
            acc[P->indices[e]] += coef * (double)P->values[e];
    }
}

/* d/dz of log(1+exp(-y z)) = -y / (1 + exp(y z)). */
static double loss_slope(double y, double z) { return -y / (1.0 + exp(y * z)); }

/* log(1+exp(-m)) without overflow. */
static double loss_value(double m) { return m > 0 ? log1p(exp(-m)) : -m + log1p(exp(m)); }

/* P(x). */
double ref_objective(const ref_problem *P, const float *x)
{
    double loss = 0.0, sq = 0.0, ab = 0.0;
    for (int64_t i = 0; i < P->n; ++i) loss += loss_value((double)P->y[i] * row_dot(P, i, x));
    for (int64_t j = 0; j < P->d; ++j) { sq += (double)x[j] * x[j]; ab += fabs((double)x[j]); }
    return loss / (double)P->n + 0.5 * (double)P->l2 * sq + (double)P->l1 * ab;
}

/* Epoch prologue (Alg. 1, global gradient computation): grad f(x) = (1/n) sum_i grad f_i(x).
 * z_out (nullable) receives the margins a_i.x. */
void ref_full_grad(const ref_problem *P, const float *x, float *g_out, float *z_out)
{
    double *acc = (double *)calloc((size_t)P->d, sizeof(double));
    for (int64_t i = 0; i < P->n; ++i) {
        double z = row_dot(P, i, x);
        if (z_out) z_out[i] = (float)z;
        row_axpy(P, i, loss_slope((double)P->y[i], z) / (double)P->n, acc);
    }
    for (int64_t j = 0; j < P->d; ++j) g_out[j] = (float)(acc[j] + (double)P->l2 * (double)x[j]);
    free(acc);
}

/* Worker step (i) of Alg. 1 with a mini-batch I of B sampled points:
 *   alpha = (1/B) sum_{i in I} [grad f_i(q) - grad f_i(xs)]
 * where q is the (dequantized) model the worker received and xs the snapshot. */
void ref_vr_grad(const ref_problem *P, const int32_t *idx, int64_t B, const float *q,
                 const float *xs, float *alpha_out)
{
    double *acc = (double *)calloc((size_t)P->d, sizeof(double));
    for (int64_t r = 0; r < B; ++r) {
        int64_t i = idx[r];
        double y = (double)P->y[i];
        double diff = loss_slope(y, row_dot(P, i, q)) - loss_slope(y, row_dot(P, i, xs));
        row_axpy(P, i, diff / (double)B, acc);
    }
    for (int64_t j = 0; j < P->d; ++j)
        alpha_out[j] = (float)(acc[j] + (double)P->l2 * ((double)q[j] - (double)xs[j]));
    free(acc);
}

/* ------------------------------------------------------------------------- */
/* Eq. (3): gradient sparsification (Alg. 2, worker (ii)).                      */
/*   beta_i = Z_i alpha_i / p_i,  Z_i ~ Bernoulli(p_i),                        */
/*   p_i = |alpha_i| phi / ||alpha||_1  (Lemma 2), capped at 1.                */
/* phi < 0 selects the budget of Section 5.1, phi = ||alpha||_1/||alpha||_inf, */
/* for which p_i = |alpha_i| / ||alpha||_inf (the 1-norm cancels).             */
/* Returns the number of kept coordinates.                                     */
/* ------------------------------------------------------------------------- */
float ref_l1norm(const float *v, int64_t d)
{
    double s = 0.0;
    for (int64_t i = 0; i < d; ++i) s += fabs((double)v[i]);
    return (float)s;
}

int64_t ref_sparsify_given_uniforms(const float *alpha, int64_t d, float phi, const float *u,
                                    float *beta_out)
{
    float amax = ref_absmax(alpha, d);
    int64_t kept = 0;
    float c = 0.0f;
    if (phi >= 0.0f) c = phi / ref_l1norm(alpha, d);
    for (int64_t i = 0; i < d; ++i) {
        float a = fabsf(alpha[i]);
        float p;
        if (a == 0.0f) { beta_out[i] = 0.0f; continue; }   /* p_i = 0: never kept */
        if (phi >= 0.0f) { p = a * c; if (p > 1.0f) p = 1.0f; }
        else p = a / amax;
        if (u[i] < p) { beta_out[i] = alpha[i] / p; ++kept; }   /* Z_i = 1 */
        else beta_out[i] = 0.0f;
    }
    return kept;
}

/* The same with u[i] drawn from the worker's sparsifier stream. */
int64_t ref_sparsify(const float *alpha, int64_t d, float phi, uint64_t seed, uint32_t iter,
                     uint32_t worker, float *beta_out)
{
    float *u = (float *)malloc(sizeof(float) * (size_t)(d > 0 ? d : 1));
    for (int64_t i = 0; i < d; ++i) u[i] = ref_uniform(seed, iter, worker, REF_TAG_SPARSIFY, (uint64_t)i);
    int64_t kept = ref_sparsify_given_uniforms(alpha, d, phi, u, beta_out);
    free(u);
    return kept;
}

/* ------------------------------------------------------------------------- */
/* Master step (ii) of Alg. 1 and of Alg. 3.                                  */
/* codes: M rows of d integer codes; delta[M].  One synchronous round of M     */
/* workers is aggregated as  gbar = scale * sum_w delta_w k_w  (scale = 1/M    */
/* for the mean), then  u = gbar + grad f(xs).                                 */
/*  AsyLPG:  x <- prox_{eta h}(x - eta u)                                       */
/*  Acc   :  y <- prox_{eta h}(y - eta u);  x <- xs + theta (y - xs);           */
/*           xsum += x   (for the epoch-end snapshot of Alg. 3)                  */
/* prox_{eta h} for h = l1||.||_1 is soft-thresholding at eta*l1.               */
/* y == NULL selects AsyLPG.  All arithmetic float32 in the order written.      */
/* ------------------------------------------------------------------------- */
static float soft_threshold(float z, float kappa)
{
    float m = fabsf(z) - kappa;
    return m > 0.0f ? copysignf(m, z) : 0.0f;
}

static void master_apply(int64_t j, float acc, float scale, const float *g_snap, float *x, float *y,
                         const float *x_snap, float *xsum, float eta, float theta, float kappa)
{
    float gbar = scale * acc;
    float u = gbar + g_snap[j];
    if (!y) {
        float step = eta * u;
        x[j] = soft_threshold(x[j] - step, kappa);
    } else {
        float step = eta * u;
        y[j] = soft_threshold(y[j] - step, kappa);
        float dy = y[j] - x_snap[j];
        float mv = theta * dy;
        x[j] = x_snap[j] + mv;
        if (xsum) xsum[j] = xsum[j] + x[j];
    }
}

void ref_master_update(const int8_t *codes, const float *delta, int64_t M, int64_t d, float scale,
                       const float *g_snap, float *x, float *y, const float *x_snap, float *xsum,
                       float eta, float theta, float l1)
{
    const float kappa = eta * l1;
    for (int64_t j = 0; j < d; ++j) {
        float acc = 0.0f;
        for (int64_t w = 0; w < M; ++w) acc = fmaf(delta[w], (float)codes[w * d + j], acc);
        master_apply(j, acc, scale, g_snap, x, y, x_snap, xsum, eta, theta, kappa);
    }
}

/* The same update when the workers send their gradients unquantized (the full-precision
 * comparison algorithms of Section 5.1): grads holds M rows of d floats, summed in worker order. */
void ref_master_update_full(const float *grads, int64_t M, int64_t d, float scale,
                            const float *g_snap, float *x, float *y, const float *x_snap, float *xsum,
                            float eta, float theta, float l1)
{
    const float kappa = eta * l1;
    for (int64_t j = 0; j < d; ++j) {
        float acc = 0.0f;
        for (int64_t w = 0; w < M; ++w) acc = acc + grads[w * d + j];
        master_apply(j, acc, scale, g_snap, x, y, x_snap, xsum, eta, theta, kappa);
    }
}

/* Alg. 1, master (ii) (Alg. 3, master (ii) when y is given) taken one received gradient at a
 * time, as the paper states the master's rule: every message triggers its own update of the
 * model with the full step size.  The M messages of a round are applied in worker order:
 *   for w:  u = delta_w * k_w + grad f(snapshot);   x <- prox(x - eta u)      (Alg. 1)
 *           y <- prox(y - eta u);  x <- snapshot + theta (y - snapshot);  xsum += x   (Alg. 3)
 * (xsum therefore gains M terms per call). */
void ref_master_update_each(const int8_t *codes, const float *delta, int64_t M, int64_t d,
                            const float *g_snap, float *x, float *y, const float *x_snap, float *xsum,
                            float eta, float theta, float l1)
{
    const float kappa = eta * l1;
    for (int64_t w = 0; w < M; ++w)
        for (int64_t j = 0; j < d; ++j) {
            float g = delta[w] * (float)codes[w * d + j];
            master_apply(j, g, 1.0f, g_snap, x, y, x_snap, xsum, eta, theta, kappa);
        }
}

/* The same with unquantized gradients (M rows of d floats). */
void ref_master_update_each_full(const float *grads, int64_t M, int64_t d,
                                 const float *g_snap, float *x, float *y, const float *x_snap, float *xsum,
                                 float eta, float theta, float l1)
{
    const float kappa = eta * l1;
    for (int64_t w = 0; w < M; ++w)
        for (int64_t j = 0; j < d; ++j)
            master_apply(j, grads[w * d + j], 1.0f, g_snap, x, y, x_snap, xsum, eta, theta, kappa);
}

/* Momentum mix used at the start of an epoch of Alg. 3, in the same
 * form as its master update:  x = xs + theta (y - xs)  ( = theta y + (1-theta) xs ). */
void ref_acc_mix(const float *y, const float *x_snap, float theta, int64_t d, float *x_out)
{
    for (int64_t j = 0; j < d; ++j) {
        float dy = y[j] - x_snap[j];
        float mv = theta * dy;
        x_out[j] = x_snap[j] + mv;
    }
}

/* Epoch end of Alg. 3: snapshot = (1/m) sum_t x_{t+1}. */
void ref_acc_snapshot(const float *xsum, int64_t m, int64_t d, float *x_snap_out)
{
    for (int64_t j = 0; j < d; ++j) x_snap_out[j] = xsum[j] / (float)m;
}

/* Left side of condition (2) / (4): E_Q ||Q_(delta,b)(x) - x||^2 over the rounding decisions.
 * Coordinate i moves to z+delta with probability p_i and to z with 1-p_i, so its expected
 * squared error is delta^2 p_i (1 - p_i) (proof of Lemma 5); p_i as the quantizer computes it. */
double ref_expected_sq_error(const float *x, int64_t d, int b)
{
    const int L = level_max(b);
    float amax = ref_absmax(x, d);
    float delta = ref_delta(amax, b);
    if (!(delta > 0.0f) || isinf(delta)) {          /* all codes are zero: the error is ||x||^2 */
        double s = 0.0;
        for (int64_t i = 0; i < d; ++i) s += (double)x[i] * (double)x[i];
        return s;
    }
    const float inv_delta = (float)L / amax;
    double s = 0.0;
    for (int64_t i = 0; i < d; ++i) {
        float t = x[i] * inv_delta;
        float p = t - floorf(t);
        s += (double)p * (1.0 - (double)p);
    }
    return (double)delta * (double)delta * s;
}

/* Right side of condition (2) without mu: ||x - xs||^2. */
double ref_sq_distance(const float *x, const float *xs, int64_t d)
{
    double r = 0.0;
    for (int64_t j = 0; j < d; ++j) r += ((double)x[j] - (double)xs[j]) * ((double)x[j] - (double)xs[j]);
    return r;
}

/* Squared distances of condition (2): ||Q(x)-x||^2 and ||x-xs||^2 (double). */
void ref_mu_terms(const int8_t *codes, float delta, const float *x, const float *x_snap, int64_t d,
                  double out[2])
{
    double e = 0.0, r = 0.0;
    for (int64_t j = 0; j < d; ++j) {
        double q = (double)(delta * (float)codes[j]);
        e += (q - (double)x[j]) * (q - (double)x[j]);
        r += ((double)x[j] - (double)x_snap[j]) * ((double)x[j] - (double)x_snap[j]);
    }
    out[0] = e; out[1] = r;
}
