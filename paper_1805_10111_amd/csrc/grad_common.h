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

// slope(z_snap + dz) - slope(z_snap): the scalar of the variance-reduced difference
// grad f_i(q) - grad f_i(snapshot) (Alg. 1, worker (i)) along a_i.  When the model is
// close to the snapshot the two slopes agree in most digits, so the difference is
// formed analytically for small dz:
//   with m = y z_snap, e = y dz:   diff = y * expm1(e) * sigma(m) * sigma(-(m+e)).
__device__ __forceinline__ float vr_slope_diff(float y, float z_snap, float dz)
{
    const float m = y * z_snap, e = y * dz;
    if (fabsf(e) < 1.0f) {
        const float sig_m = 1.0f / (1.0f + expf(-m));
        const float sig_n = 1.0f / (1.0f + expf(m + e));
        return y * (expm1f(e) * sig_m * sig_n);
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
template <int FIELD>
__device__ __forceinline__ void worker_tail_from_lds(float *alpha, int64_t d, bool sparsify, int b, StreamKey key,
                                                     const WorkerOut &out, uint32_t *su, int *si, int slice = 0,
                                                     int nslices = 1)
{
    const int64_t quads = (d + 3) / 4;
    // slice boundaries are multiples of 64 quads, so no packed word is shared between two slices
    const int64_t per = ((quads + nslices - 1) / nslices + kWave - 1) / kWave * kWave;
    const int64_t q_lo = min(quads, per * slice), q_hi = min(quads, q_lo + per);
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t first = threadIdx.x - lane;           // quad of lane 0 in the first sweep (wave-uniform)
    uint32_t vmax = 0;
    for (int64_t q = threadIdx.x; q < quads; q += blockDim.x) {
        const float4 a = load_quad(alpha, q, d);
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
            float4 a = load_quad(alpha, q, d);
            const uint4 w = stream_block(sk, static_cast<uint32_t>(q));
            a.x = sparsify_one(a.x, rule, w.x);
            a.y = sparsify_one(a.y, rule, w.y);
            a.z = sparsify_one(a.z, rule, w.z);
            a.w = sparsify_one(a.w, rule, w.w);
            bmax = max(max(bmax, abs_bits(a.x)), max(max(abs_bits(a.y), abs_bits(a.z)), abs_bits(a.w)));
            kept += (a.x != 0.0f) + (a.y != 0.0f) + (a.z != 0.0f) + (a.w != 0.0f);
            store_quad(alpha, q, d, a);
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
            if (q < q_hi) bits = quantize_quad<FIELD>(load_quad(alpha, q, d), s, key, q, nz);
            store_quad_bits<FIELD>(bits, q, q_hi, out.packed);
        }
        if (out.nnz_out && nslices == 1) {
            nz = block_sum_i32(nz, si);
            if (threadIdx.x == 0) out.nnz_out[0] = nz;
        }
    }
}

}  // namespace dq
