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
    const int k = sext_field(q.words[bit >> 5], static_cast<unsigned>(bit & 31), static_cast<unsigned>(q.b_x));
    return q.delta_x * static_cast<float>(k);
}

// ---- tail of a worker step on alpha[d] in LDS (one block per worker) -------------------
struct WorkerOut {
    uint32_t *packed;       // row of packed words
    int64_t row_words;
    float *delta_out;       // one float
    int32_t *nnz_out;       // nullable, one int
    uint32_t *status;       // nullable
};

// Scratch: su >= blockDim.x/64 uint32, si >= blockDim.x/64 int.
// Alg. 2, worker (ii)-(iii) when `sparsify`, else Alg. 1, worker (ii).
template <int FIELD>
__device__ __forceinline__ void worker_tail_from_lds(float *alpha, int64_t d, bool sparsify, int b, StreamKey key,
                                                     const WorkerOut &out, uint32_t *su, int *si)
{
    const int64_t chunks = (d + 15) / 16;
    uint32_t vmax = 0;
    for (int64_t i = threadIdx.x; i < d; i += blockDim.x) vmax = max(vmax, abs_bits(alpha[i]));
    vmax = block_max_u32(vmax, su);
    if (sparsify) {
        SparsifyRule rule{__uint_as_float(vmax), 0.0f, false};
        StreamKey sk = key;
        sk.tag = DQ_TAG_SPARSIFY;
        uint32_t bmax = 0;
        for (int64_t c = threadIdx.x; c < chunks; c += blockDim.x) {
            float a[16];
#pragma unroll
            for (int j = 0; j < 16; ++j) a[j] = (c * 16 + j < d) ? alpha[c * 16 + j] : 0.0f;
            sparsify16(a, rule, sk, c);
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                bmax = max(bmax, abs_bits(a[j]));
                if (c * 16 + j < d) alpha[c * 16 + j] = a[j];
            }
        }
        vmax = block_max_u32(bmax, su);      // (barriers inside also publish the beta writes)
    }
    if constexpr (FIELD == 32) {
        // no gradient quantization (the full-precision comparison runs of Section 5.1):
        // the message is the float32 vector itself and its scale is 1
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
    if (threadIdx.x == 0) {
        out.delta_out[0] = s.delta;
        if (s.bad && out.status) atomicOr(out.status, 1u);
    }
    key.tag = DQ_TAG_GRAD;
    int nz = 0;
    for (int64_t c = threadIdx.x; c < chunks; c += blockDim.x) {
        float a[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) a[j] = (c * 16 + j < d) ? alpha[c * 16 + j] : 0.0f;
        uint32_t w[Words16<FIELD>::n];
        nz += quantize16<FIELD>(a, s, key, c, w);
        store_words<FIELD>(out.packed, c, out.row_words, w);
    }
    if (out.nnz_out) {
        nz = block_sum_i32(nz, si);
        if (threadIdx.x == 0) out.nnz_out[0] = nz;
    }
    }
}

}  // namespace dq
