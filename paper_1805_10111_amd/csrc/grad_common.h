// Pieces shared by the dense and CSR gradient kernels: logistic-loss scalars, access
// to the model message, and the tail of a worker step (sparsify -> scale -> quantize
// -> pack) operating on a gradient held in LDS.
#pragma once

#include "dq_common.h"
#include "elementwise.h"

namespace dq {

// ---- logistic loss of Section 5.1:  l(z; y) = log(1 + exp(-y z)) -------------------
// dl/dz = -y / (1 + exp(y z)).
__device__ __forceinline__ float logistic_slope(float y, float z) { return -y / (1.0f + expf(y * z)); }

// log(1 + exp(-m)) for the signed margin m = y z, without overflow.
__device__ __forceinline__ float logistic_loss(float m)
{
    return m > 0.0f ? log1pf(expf(-m)) : -m + log1pf(expf(m));
}

// exp(x) and 1/x in one hardware instruction each (plus the scaling of the argument): about 2 ulp, and a relative
// error of |x| * 2^-24 from rounding x * log2(e) -- far inside the 1e-5 tolerance of the gradients, which the
// float32 dot products in front of them already use up to about 1e-6.
__device__ __forceinline__ float fast_exp(float x) { return __builtin_amdgcn_exp2f(x * 1.44269504088896341f); }
__device__ __forceinline__ float fast_rcp(float x) { return __builtin_amdgcn_rcpf(x); }

// exp(e) - 1 for |e| < 1 without cancellation: e * sum_{k=0..10} e^k / (k+1)!   (the first omitted term is below
// 2.6e-8 relative).
__device__ __forceinline__ float expm1_small(float e)
{
    float p = 1.0f / 39916800.0f;                     // 1/11!
    p = fmaf(p, e, 1.0f / 3628800.0f);
    p = fmaf(p, e, 1.0f / 362880.0f);
    p = fmaf(p, e, 1.0f / 40320.0f);
    p = fmaf(p, e, 1.0f / 5040.0f);
    p = fmaf(p, e, 1.0f / 720.0f);
    p = fmaf(p, e, 1.0f / 120.0f);
    p = fmaf(p, e, 1.0f / 24.0f);
    p = fmaf(p, e, 1.0f / 6.0f);
    p = fmaf(p, e, 0.5f);
    p = fmaf(p, e, 1.0f);
    return e * p;
}

// The slope and the loss with the hardware exponential, reciprocal and logarithm (the row-streaming kernels evaluate
// them on a few lanes while every other lane of the block waits).  Relative error of the slope about 1e-6 for
// margins up to ~15; absolute error of the loss about 1e-7 -- both far inside the 1e-5 of the gradients and the
// objective.
__device__ __forceinline__ float logistic_slope_fast(float y, float z) { return -y * fast_rcp(1.0f + fast_exp(y * z)); }

__device__ __forceinline__ float logistic_loss_fast(float m)
{
    // log(1 + exp(-|m|)) + max(-m, 0); the logarithm's argument lies in [1, 2]
    const float t = __builtin_amdgcn_logf(1.0f + fast_exp(-fabsf(m))) * 0.693147180559945309f;
    return t + fmaxf(-m, 0.0f);
}

// slope(z_snap + dz) - slope(z_snap): the scalar of the variance-reduced difference
// grad f_i(q) - grad f_i(snapshot) (Alg. 1, worker (i)) along a_i.  When the model is
// close to the snapshot the two slopes agree in most digits, so the difference is
// formed analytically for small dz:
//   with m = y z_snap, e = y dz:   diff = y * expm1(e) * sigma(m) * sigma(-(m+e)).
// The block that streams rows evaluates this once per row on a few lanes while every other lane waits, so it is
// kept to about thirty instructions (hardware exp and reciprocal, a polynomial for expm1).
__device__ __forceinline__ float vr_slope_diff(float y, float z_snap, float dz)
{
    const float m = y * z_snap, e = y * dz;
    if (fabsf(e) < 1.0f) {
        const float sig_m = fast_rcp(1.0f + fast_exp(-m));
        const float sig_n = fast_rcp(1.0f + fast_exp(m + e));
        return y * (expm1_small(e) * sig_m * sig_n);
    }
    return logistic_slope(y, z_snap + dz) - logistic_slope(y, z_snap);
}

// ---- the model message: b_x-bit codes with scale delta_x, or float32 when b_x == 32 ----
struct ModelMsg {
    const uint32_t *words;
    float delta_x;
    int b_x;
};

__device__ __forceinline__ float model_value(const ModelMsg &q, int64_t j)
{
    if (q.b_x == 32) return __uint_as_float(q.words[j]);
    const int64_t bit = j * q.b_x;
    const unsigned sh = static_cast<unsigned>(bit & 31);
    uint32_t f = q.words[bit >> 5] >> sh;
    if (sh + q.b_x > 32) f |= q.words[(bit >> 5) + 1] << (32 - sh);      // widths that do not divide 32: the field
                                                                        // continues in the next word of the row
    return q.delta_x * static_cast<float>(sext_field(f, 0, static_cast<unsigned>(q.b_x)));
}

// The same for the four coordinates col..col+3 (col a multiple of 4), in two steps so that a caller can have the
// words in flight together with its other loads.  The code bits of such a quad start at bit col*b_x of the message
// and lie in at most four consecutive words for every width (b_x = 32: exactly four).  The request has no branch:
// a word index past `last_word` (the last word of the message) repeats that word, which no coordinate below d needs.
struct ModelQuad {
    uint32_t w[4];
};

template <bool MODEL8 = false>
__device__ __forceinline__ ModelQuad model_quad_request(const ModelMsg &q, int64_t col, int64_t last_word)
{
    ModelQuad r;
    if (MODEL8 || q.b_x == 8) {            // (the width is the same for every thread) the quad is one word
        r.w[0] = q.words[min(col >> 2, last_word)];
        r.w[1] = r.w[2] = r.w[3] = 0u;
        return r;
    }
    const int64_t first = (col * q.b_x) >> 5;
#pragma unroll
    for (int k = 0; k < 4; ++k) r.w[k] = q.words[min(first + k, last_word)];
    return r;
}

// Values of coordinates col..col+3 from the requested words; coordinates at or past d read as 0.
template <bool MODEL8 = false>
__device__ __forceinline__ void model_quad_values(const ModelMsg &q, const ModelQuad &r, int64_t col, int64_t d, float (&v)[4])
{
    if (MODEL8 || q.b_x == 8) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            v[e] = col + e < d ? q.delta_x * static_cast<float>(sext_field(r.w[0], 8u * e, 8u)) : 0.0f;
        return;
    }
    const unsigned shift = static_cast<unsigned>((col * q.b_x) & 31);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const unsigned f = shift + static_cast<unsigned>(e * q.b_x);
        const unsigned wi = f >> 5, sh = f & 31u;
        const uint32_t lo = wi == 0 ? r.w[0] : wi == 1 ? r.w[1] : wi == 2 ? r.w[2] : r.w[3];
        const uint32_t hi = wi == 0 ? r.w[1] : wi == 1 ? r.w[2] : wi == 2 ? r.w[3] : 0u;
        const uint32_t bits = __funnelshift_r(lo, hi, sh);                 // bits f.. of the four words
        const float val = q.b_x == 32 ? __uint_as_float(bits)
                                      : q.delta_x * static_cast<float>(sext_field(bits, 0, static_cast<unsigned>(q.b_x)));
        v[e] = col + e < d ? val : 0.0f;
    }
}

// v[col..col+3] of a vector of d floats (v 16-byte aligned, col a multiple of 4), coordinates at or past d reading
// as 0, without a per-lane branch (clamped loads), so that the request can stay in flight next to others.
__device__ __forceinline__ float4 load4_or_zero(const float *__restrict__ v, int64_t col, int64_t d)
{
    if ((d & 3) == 0) {                    // (the same for every thread) whole quads only: one 16-byte load
        const float4 t = *reinterpret_cast<const float4 *>(v + min(col, d - 4));
        return col < d ? t : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    }
    float r[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const float t = v[min(col + e, d - 1)];
        r[e] = col + e < d ? t : 0.0f;
    }
    return make_float4(r[0], r[1], r[2], r[3]);
}

// Alg. 2, worker (ii) on one slice of the quads, for a worker whose identical blocks (one per slice) each hold the whole
// alpha in `alpha`: the block finds ||alpha||_inf over the whole vector like every other, sparsifies the quads of its own
// slice only, writes them to beta_row (memory) and leaves the slice's largest magnitude and its number of kept
// coordinates in part_max[0], part_kept[0]; a later kernel (quantize_pack_kernel with parts) combines the slices.  The
// slice boundaries are those of worker_tail_from_lds.  su, si: one entry per wavefront of the block.
// WHOLE: alpha is padded with zeros to whole quads (read as 16-byte values without a test per lane).
template <bool WHOLE = false>
__device__ __forceinline__ void sparsify_slice_from_lds(const float *alpha, int64_t d, StreamKey key, int slice, int nslices,
                                                        float *__restrict__ beta_row, float *__restrict__ part_max,
                                                        int32_t *__restrict__ part_kept, uint32_t *su, int *si,
                                                        const uint32_t *seen_max = nullptr)
{
    const int64_t quads = (d + 3) / 4;
    const int64_t per = ((quads + nslices - 1) / nslices + kWave - 1) / kWave * kWave;
    const int64_t q_lo = min(quads, per * slice), q_hi = min(quads, q_lo + per);
    const auto quad = [&](int64_t q) { return WHOLE ? reinterpret_cast<const float4 *>(alpha)[q] : load_quad(alpha, q, d); };
    // seen_max: the caller's threads have already seen every coordinate (each its share): their maxima
    uint32_t vmax = seen_max ? *seen_max : 0u;
    if (!seen_max)
        for (int64_t q = threadIdx.x; q < quads; q += blockDim.x) {
            const float4 a = quad(q);
            vmax = max(max(vmax, abs_bits(a.x)), max(max(abs_bits(a.y), abs_bits(a.z)), abs_bits(a.w)));
        }
    vmax = block_max_u32(vmax, su);
    const SparsifyRule rule{__uint_as_float(vmax), 0.0f, false};
    key.tag = DQ_TAG_SPARSIFY;
    uint32_t bmax = 0;
    int kept = 0;
    for (int64_t q = q_lo + threadIdx.x; q < q_hi; q += blockDim.x) {
        float4 a = quad(q);
        const uint4 w = stream_block(key, static_cast<uint32_t>(q));
        a.x = sparsify_one(a.x, rule, w.x);
        a.y = sparsify_one(a.y, rule, w.y);
        a.z = sparsify_one(a.z, rule, w.z);
        a.w = sparsify_one(a.w, rule, w.w);
        bmax = max(max(bmax, abs_bits(a.x)), max(max(abs_bits(a.y), abs_bits(a.z)), abs_bits(a.w)));
        kept += (a.x != 0.0f) + (a.y != 0.0f) + (a.z != 0.0f) + (a.w != 0.0f);
        store_quad(beta_row, q, d, a);
    }
    block_max_u32_sum_i32(bmax, kept, su, si);
    if (threadIdx.x == 0) {
        part_max[0] = __uint_as_float(bmax);
        part_kept[0] = kept;
    }
}

// ---- tail of a worker step on alpha[d] in LDS (one block per worker) -------------------
struct WorkerOut {
    uint32_t *packed;       // row of packed words
    int64_t row_words;
    float *delta_out;       // one float
    int32_t *nnz_out;       // nullable, one int
    uint32_t *status;       // nullable
};

// Scratch: su >= blockDim.x/64 uint32, si >= blockDim.x/64 int.  alpha is 16-byte aligned.
// Alg. 2, worker (ii)-(iii) when `sparsify`, else Alg. 1, worker (ii).
// The unit of work is a quad of four consecutive coordinates (one Philox block, one 16-byte
// LDS access per lane, consecutive lanes on consecutive quads).  A quad yields 4*FIELD code
// bits; for FIELD < 8 the lanes of a pair (FIELD 4) or of a group of four (FIELD 2) combine
// theirs into one word with cross-lane moves, and the first lane of the group stores it.
// Several blocks may hold identical copies of alpha (the CSR worker step launches `nslices` of them per worker when
// compute units would otherwise idle): each repeats the norms and the sparsifier on the whole vector, which gives
// every block the same scale, and quantizes + packs only its own slice of the quads.  The number of nonzero codes
// is then only available after the sparsifier with b >= 4, where it equals the number of kept coordinates: a kept
// coordinate has magnitude ||alpha||_inf up to two roundings, hence |t| > L - 1 >= 2 and a nonzero code whatever the
// rounding decision, and a dropped one is exactly zero.  Otherwise out.nnz_out must be null when nslices > 1.
template <int FIELD, bool WHOLE = false>
__device__ __forceinline__ void worker_tail_from_lds(float *alpha, int64_t d, bool sparsify, int b, StreamKey key,
                                                     const WorkerOut &out, uint32_t *su, int *si, int slice = 0,
                                                     int nslices = 1, const uint32_t *seen_max = nullptr)
{
    const int64_t quads = (d + 3) / 4;
    // slice boundaries are multiples of 64 quads, so no packed word is shared between two slices
    const int64_t per = ((quads + nslices - 1) / nslices + kWave - 1) / kWave * kWave;
    const int64_t q_lo = min(quads, per * slice), q_hi = min(quads, q_lo + per);
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t first = threadIdx.x - lane;           // quad of lane 0 in the first sweep (wave-uniform)
    // WHOLE: alpha is padded with zeros to whole quads
    const auto quad = [&](int64_t q) { return WHOLE ? reinterpret_cast<const float4 *>(alpha)[q] : load_quad(alpha, q, d); };
    // seen_max: the caller's threads have already seen every coordinate (each its share): their maxima
    uint32_t vmax = seen_max ? *seen_max : 0u;
    if (!seen_max)
        for (int64_t q = threadIdx.x; q < quads; q += blockDim.x) {
            const float4 a = quad(q);
            vmax = max(max(vmax, abs_bits(a.x)), max(max(abs_bits(a.y), abs_bits(a.z)), abs_bits(a.w)));
        }
    vmax = block_max_u32(vmax, su);
    if (sparsify) {
        SparsifyRule rule{__uint_as_float(vmax), 0.0f, false};
        StreamKey sk = key;
        sk.tag = DQ_TAG_SPARSIFY;
        uint32_t bmax = 0;
        int kept = 0;
        for (int64_t q = threadIdx.x; q < quads; q += blockDim.x) {
            float4 a = quad(q);
            const uint4 w = stream_block(sk, static_cast<uint32_t>(q));
            a.x = sparsify_one(a.x, rule, w.x);
            a.y = sparsify_one(a.y, rule, w.y);
            a.z = sparsify_one(a.z, rule, w.z);
            a.w = sparsify_one(a.w, rule, w.w);
            bmax = max(max(bmax, abs_bits(a.x)), max(max(abs_bits(a.y), abs_bits(a.z)), abs_bits(a.w)));
            kept += (a.x != 0.0f) + (a.y != 0.0f) + (a.z != 0.0f) + (a.w != 0.0f);
            if (WHOLE) reinterpret_cast<float4 *>(alpha)[q] = a;          // (a zero stays zero)
            else store_quad(alpha, q, d, a);
        }
        vmax = block_max_u32(bmax, su);      // (barriers inside also publish the beta writes)
        if (nslices > 1 && out.nnz_out) {    // see above: equals the number of nonzero codes (b >= 4)
            kept = block_sum_i32(kept, si);
            if (threadIdx.x == 0 && slice == 0) out.nnz_out[0] = kept;
        }
    }
    if constexpr (FIELD == 32) {
        // no gradient quantization (the full-precision comparison runs of Section 5.1):
        // the message is the float32 vector itself and its scale is 1
        if (slice != 0) return;                      // the float32 message is copied by the first block alone
        if (threadIdx.x == 0) out.delta_out[0] = 1.0f;
        int nzf = 0;
        for (int64_t i = threadIdx.x; i < d; i += blockDim.x) {
            const float a = alpha[i];
            out.packed[i] = __float_as_uint(a);
            nzf += a != 0.0f ? 1 : 0;
        }
        if (out.nnz_out) {
            nzf = block_sum_i32(nzf, si);
            if (threadIdx.x == 0) out.nnz_out[0] = nzf;
        }
        return;
    } else {
        const Scale s = make_scale(__uint_as_float(vmax), b);
        if (threadIdx.x == 0 && slice == 0) {
            out.delta_out[0] = s.delta;
            if (s.bad && out.status) atomicOr(out.status, 1u);
        }
        key.tag = DQ_TAG_GRAD;
        int nz = 0;
        // every lane of a wavefront takes the same number of sweeps, so that the cross-lane
        // moves of the store always see all lanes; lanes past the end contribute zero bits
        for (int64_t q0 = q_lo + first; q0 < q_hi; q0 += blockDim.x) {
            const int64_t q = q0 + lane;
            uint32_t bits = 0;
            if (q < q_hi) bits = quantize_quad<FIELD>(quad(q), s, key, q, nz);
            store_quad_bits<FIELD>(bits, q, q_hi, out.packed);
        }
        if (out.nnz_out && nslices == 1) {
            nz = block_sum_i32(nz, si);
            if (threadIdx.x == 0) out.nnz_out[0] = nz;
        }
    }
}

// The same tail (without sparsifier, b in {2, 4, 8}) when the block's threads hold the whole gradient in registers, thread t
// the quad t (coordinates past d are zero): no trip through LDS, one block reduction for the scale.
template <int FIELD>
__device__ __forceinline__ void worker_tail_one_quad(float4 v, int64_t d, int b, StreamKey key, const WorkerOut &out,
                                                     uint32_t *su, int *si, int slice, int nslices)
{
    const int64_t quads = (d + 3) / 4;
    const int64_t per = ((quads + nslices - 1) / nslices + kWave - 1) / kWave * kWave;       // as in worker_tail_from_lds
    const int64_t q_lo = min(quads, per * slice), q_hi = min(quads, q_lo + per);
    const int64_t q = threadIdx.x;
    const uint32_t vmax = block_max_u32(max(max(abs_bits(v.x), abs_bits(v.y)), max(abs_bits(v.z), abs_bits(v.w))), su);
    const Scale s = make_scale(__uint_as_float(vmax), b);
    if (threadIdx.x == 0 && slice == 0) {
        out.delta_out[0] = s.delta;
        if (s.bad && out.status) atomicOr(out.status, 1u);
    }
    key.tag = DQ_TAG_GRAD;
    int nz = 0;
    uint32_t bits = 0;
    if (q >= q_lo && q < q_hi) bits = quantize_quad<FIELD>(v, s, key, q, nz);
    // (slices begin at multiples of 64 quads: the lanes that share a word are all inside or all outside)
    store_quad_bits<FIELD>(bits, q >= q_lo ? q : q_hi, q_hi, out.packed);
    if (out.nnz_out && nslices == 1) {
        nz = block_sum_i32(nz, si);
        if (threadIdx.x == 0) out.nnz_out[0] = nz;
    }
}

}  // namespace dq
