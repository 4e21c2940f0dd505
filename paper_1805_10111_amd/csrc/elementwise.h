// Per-thread building blocks shared by the quantizer, master and worker kernels.
// Two granularities: chunks of 16 coordinates (whole words for 2, 4 and 8-bit fields; the
// streaming kernels over long vectors) and quads of 4 coordinates (one Philox block, one
// 16-byte access; the one-block kernels, where consecutive lanes take consecutive quads).
// Also the soft-threshold prox and the per-coordinate sparsifier rule.
#pragma once

#include "dq_common.h"

namespace dq {

// Words of a thread's 16 coordinates: FIELD in {2,4,8} -> 1, 2, 4 words; FIELD == 32 -> 16 floats.
template <int FIELD>
struct Words16 {
    static constexpr int n = 16 * FIELD / 32;
};

// 16-byte accesses marked non-temporal: for data that is touched once by a kernel streaming over a long
// vector (measured on this part: a plain read of 1 GiB goes from 5.6 to 6.1 TB/s with the mark).
typedef float dq_v4f __attribute__((ext_vector_type(4)));
typedef uint32_t dq_v4u __attribute__((ext_vector_type(4)));
typedef uint32_t dq_v2u __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float4 load_f4_stream(const float *p)
{
    const dq_v4f t = __builtin_nontemporal_load(reinterpret_cast<const dq_v4f *>(p));
    return make_float4(t.x, t.y, t.z, t.w);
}

__device__ __forceinline__ void store_f4_stream(float *p, float4 v)
{
    dq_v4f t;
    t.x = v.x; t.y = v.y; t.z = v.z; t.w = v.w;
    __builtin_nontemporal_store(t, reinterpret_cast<dq_v4f *>(p));
}

template <int FIELD, bool STREAM = false>
__device__ __forceinline__ void load_words(const uint32_t *__restrict__ row, int64_t c, int64_t row_words,
                                           uint32_t (&w)[Words16<FIELD>::n])
{
    constexpr int kWords = Words16<FIELD>::n;
    const int64_t w0 = c * kWords;
    if (w0 + kWords <= row_words) {
        if constexpr (kWords >= 4) {
#pragma unroll
            for (int q = 0; q < kWords / 4; ++q) {
                if constexpr (STREAM) {
                    const dq_v4u t = __builtin_nontemporal_load(reinterpret_cast<const dq_v4u *>(row + w0) + q);
                    w[4 * q] = t.x; w[4 * q + 1] = t.y; w[4 * q + 2] = t.z; w[4 * q + 3] = t.w;
                } else {
                    const uint4 t = reinterpret_cast<const uint4 *>(row + w0)[q];
                    w[4 * q] = t.x; w[4 * q + 1] = t.y; w[4 * q + 2] = t.z; w[4 * q + 3] = t.w;
                }
            }
        } else if constexpr (kWords == 2) {
            if constexpr (STREAM) {
                const dq_v2u t = __builtin_nontemporal_load(reinterpret_cast<const dq_v2u *>(row + w0));
                w[0] = t.x; w[1] = t.y;
            } else {
                const uint2 t = reinterpret_cast<const uint2 *>(row + w0)[0];
                w[0] = t.x; w[1] = t.y;
            }
        } else {
            w[0] = STREAM ? __builtin_nontemporal_load(row + w0) : row[w0];
        }
    } else {
#pragma unroll
        for (int i = 0; i < kWords; ++i) w[i] = (w0 + i < row_words) ? row[w0 + i] : 0u;
    }
}

// Code j (0..15) of the thread's words as a float: sign-extended field, or the float itself.
template <int FIELD>
__device__ __forceinline__ int code_of(const uint32_t (&w)[Words16<FIELD>::n], int j)
{
    static_assert(FIELD == 2 || FIELD == 4 || FIELD == 8, "packed field width");
    return sext_field(w[(j * FIELD) / 32], (j * FIELD) % 32, FIELD);
}

template <int FIELD>
__device__ __forceinline__ float value_of(const uint32_t (&w)[Words16<FIELD>::n], int j)
{
    if constexpr (FIELD == 32) return __uint_as_float(w[j]);
    else return static_cast<float>(code_of<FIELD>(w, j));
}

template <bool STREAM = false>
__device__ __forceinline__ void load16(const float *__restrict__ src, int64_t base, int64_t d, float (&a)[16])
{
    if (base + 16 <= d) {
        const float4 *p = reinterpret_cast<const float4 *>(src + base);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float4 t = STREAM ? load_f4_stream(src + base + 4 * q) : p[q];
            a[4 * q] = t.x; a[4 * q + 1] = t.y; a[4 * q + 2] = t.z; a[4 * q + 3] = t.w;
        }
    } else {
#pragma unroll
        for (int j = 0; j < 16; ++j) a[j] = (base + j < d) ? src[base + j] : 0.0f;
    }
}

template <bool STREAM = false>
__device__ __forceinline__ void store16(float *__restrict__ out, int64_t base, int64_t d, const float (&a)[16])
{
    if (base + 16 <= d) {
        if constexpr (STREAM) {
#pragma unroll
            for (int q = 0; q < 4; ++q)
                store_f4_stream(out + base + 4 * q, make_float4(a[4 * q], a[4 * q + 1], a[4 * q + 2], a[4 * q + 3]));
            return;
        }
        float4 *p = reinterpret_cast<float4 *>(out + base);
        p[0] = make_float4(a[0], a[1], a[2], a[3]);
        p[1] = make_float4(a[4], a[5], a[6], a[7]);
        p[2] = make_float4(a[8], a[9], a[10], a[11]);
        p[3] = make_float4(a[12], a[13], a[14], a[15]);
    } else {
#pragma unroll
        for (int j = 0; j < 16; ++j)
            if (base + j < d) out[base + j] = a[j];
    }
}

// acc[j] = fma(dm, code j of the thread's words, acc[j]) for its 16 coordinates.
// SCALED (2- and 4-bit fields): the sign-extending bit-field extract per code is avoided.  One shift and one mask
// per field position move that field of every byte to the top of its byte, where it reads as the signed byte 64*k
// (16*k), which converts to float in one instruction; the product with dm/64 (dm/16) is the same real number as
// dm*k, so the fused multiply-add rounds to the same result bit for bit as long as the division is exact, i.e. dm
// is zero or not within a factor 2^26 of the smallest normal number.  The caller tests that once for all scales
// (a test per call would make the two paths meet after every worker, and the accumulators would be copied there).
// Measured at M = 16 on 2^28 coordinates: 4-bit 5.26 -> 5.73 TB/s, 2-bit 4.76 -> 5.1 TB/s.
// float(signed byte N of r), one instruction (sub-dword source select with sign extension)
template <int N>
__device__ __forceinline__ float signed_byte_to_float(uint32_t r)
{
    float f;
    if constexpr (N == 0) asm("v_cvt_f32_i32_sdwa %0, sext(%1) dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_0" : "=v"(f) : "v"(r));
    else if constexpr (N == 1) asm("v_cvt_f32_i32_sdwa %0, sext(%1) dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_1" : "=v"(f) : "v"(r));
    else if constexpr (N == 2) asm("v_cvt_f32_i32_sdwa %0, sext(%1) dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_2" : "=v"(f) : "v"(r));
    else asm("v_cvt_f32_i32_sdwa %0, sext(%1) dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_3" : "=v"(f) : "v"(r));
    return f;
}

template <int FIELD, bool SCALED>
__device__ __forceinline__ void fold_codes16(float dm, const uint32_t (&w)[Words16<FIELD>::n], float (&acc)[16])
{
    if constexpr (FIELD == 2 && SCALED) {
        {
            const float ds = dm * 0.015625f;
            // field t of every byte moved to the top of its byte: the signed byte 64*k of coordinates t, 4+t, 8+t, 12+t
            const uint32_t r0 = (w[0] << 6) & 0xC0C0C0C0u, r1 = (w[0] << 4) & 0xC0C0C0C0u,
                           r2 = (w[0] << 2) & 0xC0C0C0C0u, r3 = w[0] & 0xC0C0C0C0u;
            acc[0] = fmaf(ds, signed_byte_to_float<0>(r0), acc[0]);
            acc[1] = fmaf(ds, signed_byte_to_float<0>(r1), acc[1]);
            acc[2] = fmaf(ds, signed_byte_to_float<0>(r2), acc[2]);
            acc[3] = fmaf(ds, signed_byte_to_float<0>(r3), acc[3]);
            acc[4] = fmaf(ds, signed_byte_to_float<1>(r0), acc[4]);
            acc[5] = fmaf(ds, signed_byte_to_float<1>(r1), acc[5]);
            acc[6] = fmaf(ds, signed_byte_to_float<1>(r2), acc[6]);
            acc[7] = fmaf(ds, signed_byte_to_float<1>(r3), acc[7]);
            acc[8] = fmaf(ds, signed_byte_to_float<2>(r0), acc[8]);
            acc[9] = fmaf(ds, signed_byte_to_float<2>(r1), acc[9]);
            acc[10] = fmaf(ds, signed_byte_to_float<2>(r2), acc[10]);
            acc[11] = fmaf(ds, signed_byte_to_float<2>(r3), acc[11]);
            acc[12] = fmaf(ds, signed_byte_to_float<3>(r0), acc[12]);
            acc[13] = fmaf(ds, signed_byte_to_float<3>(r1), acc[13]);
            acc[14] = fmaf(ds, signed_byte_to_float<3>(r2), acc[14]);
            acc[15] = fmaf(ds, signed_byte_to_float<3>(r3), acc[15]);
            return;
        }
    }
    if constexpr (FIELD == 4 && SCALED) {
        {
            const float ds = dm * 0.0625f;
#pragma unroll
            for (int i = 0; i < Words16<FIELD>::n; ++i) {
                const uint32_t lo = (w[i] << 4) & 0xF0F0F0F0u, hi = w[i] & 0xF0F0F0F0u;
#pragma unroll
                for (int n = 0; n < 4; ++n) {
                    acc[8 * i + 2 * n] = fmaf(ds, static_cast<float>(sext_field(lo, 8u * n, 8u)), acc[8 * i + 2 * n]);
                    acc[8 * i + 2 * n + 1] = fmaf(ds, static_cast<float>(sext_field(hi, 8u * n, 8u)), acc[8 * i + 2 * n + 1]);
                }
            }
            return;
        }
    }
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[j] = fmaf(dm, value_of<FIELD>(w, j), acc[j]);
}

// Alg. 1, master (ii), receive side: acc[j] = sum_{m<M} delta[m] * k_m[16c + j], m ascending, one fma each.
// For FIELD == 32 the rows hold float32 values and delta is taken as 1.
// True when the byte-scaled decode of 2- and 4-bit fields is exact for this scale: delta/64 (delta/16) must be
// computed without rounding, i.e. delta is zero or far enough above the smallest normal number.
__device__ __forceinline__ bool scale_divides_exactly(float dm) { return dm == 0.0f || fabsf(dm) >= 0x1p-100f; }

template <int FIELD, bool STREAM, bool SCALED>
__device__ __forceinline__ void decode_sum16_impl(const uint32_t *__restrict__ packed, int64_t ld_words, int64_t row_words,
                                                  const float *__restrict__ delta, int M, int64_t c, float (&acc)[16])
{
    // the words of several workers are requested together, then folded in in worker order: 8 workers of 2- or 4-bit
    // fields, 4 of 8-bit fields (16 bytes per lane and worker: 955 -> 940 us for 16 workers of 2^28 coordinates)
    constexpr int kGroup = FIELD == 32 ? 2 : FIELD == 8 ? 4 : 8;
    int m = 0;
    for (; m + kGroup <= M; m += kGroup) {
        uint32_t w[kGroup][Words16<FIELD>::n];
        float dm[kGroup];
#pragma unroll
        for (int u = 0; u < kGroup; ++u) {
            load_words<FIELD, STREAM>(packed + static_cast<int64_t>(m + u) * ld_words, c, row_words, w[u]);
            dm[u] = FIELD == 32 ? 1.0f : delta[m + u];
        }
#pragma unroll
        for (int u = 0; u < kGroup; ++u) fold_codes16<FIELD, SCALED>(dm[u], w[u], acc);
    }
    for (; m < M; ++m) {
        uint32_t w[Words16<FIELD>::n];
        load_words<FIELD, STREAM>(packed + static_cast<int64_t>(m) * ld_words, c, row_words, w);
        const float dm = FIELD == 32 ? 1.0f : delta[m];
        fold_codes16<FIELD, SCALED>(dm, w, acc);
    }
}

// Alg. 1, master (ii), receive side: acc[j] = sum_{m<M} delta[m] * k_m[16c + j], m ascending, one fma each.
// For FIELD == 32 the rows hold float32 values and delta is taken as 1.
// `scaled`: every delta[m] passes scale_divides_exactly (the same for all threads; ignored unless FIELD is 2 or 4).
template <int FIELD, bool STREAM = false>
__device__ __forceinline__ void decode_sum16(const uint32_t *__restrict__ packed, int64_t ld_words, int64_t row_words,
                                             const float *__restrict__ delta, int M, int64_t c, int64_t d, bool scaled,
                                             float (&acc)[16])
{
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[j] = 0.0f;
    if constexpr (FIELD == 2 || FIELD == 4) {
        if (scaled) {
            decode_sum16_impl<FIELD, STREAM, true>(packed, ld_words, row_words, delta, M, c, acc);
            return;
        }
    }
    decode_sum16_impl<FIELD, STREAM, false>(packed, ld_words, row_words, delta, M, c, acc);
}

// The test for `scaled` above, over all M scales (every thread gets the same answer).
__device__ __forceinline__ bool scales_divide_exactly(const float *__restrict__ delta, int M)
{
    bool ok = true;
    for (int m = 0; m < M; ++m) ok = ok && scale_divides_exactly(delta[m]);
    return ok;
}

// ---- quads: four consecutive coordinates 4q .. 4q+3 (one Philox block, one 16-byte access) -------
// v is 16-byte aligned; coordinates past the end of the vector read as zero and are not written.
__device__ __forceinline__ float4 load_quad(const float *v, int64_t q, int64_t d)
{
    // d a multiple of 4 (the same for every thread, so this branch is not a divergent one): every quad is whole.
    // Only the per-lane test below makes the compiler wait for earlier loads before the next one is issued.
    if ((d & 3) == 0) return reinterpret_cast<const float4 *>(v)[q];
    if (4 * q + 3 < d) return reinterpret_cast<const float4 *>(v)[q];
    float4 r = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    if (4 * q + 0 < d) r.x = v[4 * q + 0];
    if (4 * q + 1 < d) r.y = v[4 * q + 1];
    if (4 * q + 2 < d) r.z = v[4 * q + 2];
    return r;
}

__device__ __forceinline__ void store_quad(float *v, int64_t q, int64_t d, float4 r)
{
    if (4 * q + 3 < d) {
        reinterpret_cast<float4 *>(v)[q] = r;
        return;
    }
    if (4 * q + 0 < d) v[4 * q + 0] = r.x;
    if (4 * q + 1 < d) v[4 * q + 1] = r.y;
    if (4 * q + 2 < d) v[4 * q + 2] = r.z;
}

// The four values of quad q of one message row: codes as floats (FIELD 2, 4, 8: the quad is a
// byte, a half word or a word of the packed row) or the floats themselves (FIELD 32).
// In two steps, so that the loads of many rows can be in flight together: what is fetched (the word that holds
// the quad, or the four floats), then its four values.
template <int FIELD>
struct QuadRaw {
    uint32_t w;
};
template <>
struct QuadRaw<32> {
    float4 v;
};

template <int FIELD>
__device__ __forceinline__ QuadRaw<FIELD> quad_request(const uint32_t *__restrict__ row, int64_t q, int64_t d)
{
    QuadRaw<FIELD> r;
    if constexpr (FIELD == 32) r.v = load_quad(reinterpret_cast<const float *>(row), q, d);
    else r.w = row[static_cast<uint32_t>(q / (8 / FIELD))];     // 32-bit index: the row pointer stays a scalar base
    return r;
}

template <int FIELD>
__device__ __forceinline__ float4 quad_decode(const QuadRaw<FIELD> &r, int64_t q)
{
    if constexpr (FIELD == 32) {
        return r.v;
    } else {
        constexpr int kQuadsPerWord = 8 / FIELD;
        const unsigned sh = static_cast<unsigned>(q % kQuadsPerWord) * (4 * FIELD);
        return make_float4(static_cast<float>(sext_field(r.w, sh, FIELD)), static_cast<float>(sext_field(r.w, sh + FIELD, FIELD)),
                           static_cast<float>(sext_field(r.w, sh + 2 * FIELD, FIELD)),
                           static_cast<float>(sext_field(r.w, sh + 3 * FIELD, FIELD)));
    }
}

template <int FIELD>
__device__ __forceinline__ float4 quad_values(const uint32_t *__restrict__ row, int64_t q, int64_t d)
{
    return quad_decode<FIELD>(quad_request<FIELD>(row, q, d), q);
}

// Four codes, each within the two's-complement range of a FIELD-bit field, as 4*FIELD bits (first code lowest).
// Bytes: two byte permutes and an or.  Narrower fields: the codes plus 2^(FIELD-1) are non-negative, so they are
// shifted into place without masking off sign bits; flipping the top bit of every field afterwards (kFieldTops, which
// the caller may apply once per word instead: FLIP = false) turns k + 2^(FIELD-1) into the two's-complement field.
template <int FIELD>
struct FieldTops {
    static constexpr uint32_t quad = (1u << (FIELD - 1)) * (1u | (1u << FIELD) | (1u << (2 * FIELD)) | (1u << (3 * FIELD)));
    static constexpr uint32_t word = FIELD == 8 ? quad : FIELD == 4 ? quad * 0x10001u : quad * 0x01010101u;
};

// BIASED: the four values are codes + 2^(FIELD-1) already (see quantize_one<BIAS>); FIELD < 8 only.
template <int FIELD, bool FLIP = true, bool BIASED = false>
__device__ __forceinline__ uint32_t pack4(int k0, int k1, int k2, int k3)
{
    if constexpr (FIELD == 8) {
        static_assert(!BIASED, "bytes are packed from the codes themselves");
        return __builtin_amdgcn_perm(static_cast<uint32_t>(k1), static_cast<uint32_t>(k0), 0x0c0c0400u) |
               __builtin_amdgcn_perm(static_cast<uint32_t>(k3), static_cast<uint32_t>(k2), 0x04000c0cu);
    } else {
        constexpr int kBias = BIASED ? 0 : 1 << (FIELD - 1);
        const uint32_t u = static_cast<uint32_t>(k0 + kBias) | (static_cast<uint32_t>(k1 + kBias) << FIELD) |
                           (static_cast<uint32_t>(k2 + kBias) << (2 * FIELD)) | (static_cast<uint32_t>(k3 + kBias) << (3 * FIELD));
        return FLIP ? u ^ FieldTops<FIELD>::quad : u;
    }
}

// Bias that quantize_one adds for pack4<FIELD, ., true>.
template <int FIELD>
struct CodeBias {
    static constexpr int value = FIELD == 8 ? 0 : 1 << (FIELD - 1);
};

// Q_(delta,b) on quad q: the 4*FIELD code bits (coordinate 4q in the low field) and the number of
// nonzero codes added to nz.  Coordinates past the end must be passed as 0.
template <int FIELD>
__device__ __forceinline__ uint32_t quantize_quad(float4 a, const Scale &s, const StreamKey &key, int64_t q, int &nz)
{
    if (s.inv_delta == 0.0f) return 0u;              // degenerate scale: all codes are zero
    const uint4 r = stream_block(key, static_cast<uint32_t>(q));
    constexpr int kB = CodeBias<FIELD>::value;
    const int k0 = quantize_one<kB>(a.x, s, r.x), k1 = quantize_one<kB>(a.y, s, r.y);
    const int k2 = quantize_one<kB>(a.z, s, r.z), k3 = quantize_one<kB>(a.w, s, r.w);
    nz += (k0 != kB) + (k1 != kB) + (k2 != kB) + (k3 != kB);
    return pack4<FIELD, true, FIELD != 8>(k0, k1, k2, k3);
}

// Stores the code bits of quad q = q0 + lane, where q0 is a multiple of 64 common to the wavefront.
// For FIELD < 8 the lanes of a pair (FIELD 4) or of a group of four (FIELD 2) first combine their
// bits into one word with cross-lane moves, and the first lane of the group stores it.  Every lane
// of the wavefront must make the call; lanes with q >= quads pass bits == 0.
template <int FIELD>
__device__ __forceinline__ void store_quad_bits(uint32_t bits, int64_t q, int64_t quads, uint32_t *__restrict__ out)
{
    constexpr int kQuadsPerWord = 8 / FIELD;             // 1, 2 or 4 lanes share a word
    const int sub = static_cast<int>(q) & (kQuadsPerWord - 1);
    if constexpr (kQuadsPerWord > 1) {
        bits <<= (4 * FIELD) * sub;
        bits |= dq_i2u(dpp_move_or_zero<0xb1, 0xf>(dq_u2i(bits)));                                   // lane ^ 1
        if constexpr (kQuadsPerWord == 4) bits |= dq_i2u(dpp_move_or_zero<0x4e, 0xf>(dq_u2i(bits)));   // lane ^ 2
    }
    if (q < quads && sub == 0) out[q / kQuadsPerWord] = bits;
}

// prox of eta*l1*|.| : soft-threshold at kappa = eta*l1.
__device__ __forceinline__ float soft_threshold(float z, float kappa)
{
    const float m = fabsf(z) - kappa;
    return m > 0.0f ? copysignf(m, z) : 0.0f;
}

// Eq. (3): keep coordinate with probability p, rescale by 1/p.
struct SparsifyRule {
    float amax;        // ||alpha||_inf
    float c;           // phi / ||alpha||_1 (caller's budget)
    bool use_budget;   // false: the budget ||alpha||_1/||alpha||_inf, p = |alpha|/amax
};

__device__ __forceinline__ float sparsify_one(float alpha, const SparsifyRule &r, uint32_t word)
{
    const float a = fabsf(alpha);
    if (a == 0.0f) return 0.0f;
    float p;
    if (r.use_budget) p = fminf(a * r.c, 1.0f);
    else p = a / r.amax;
    return bernoulli(word, p) ? alpha / p : 0.0f;
}

// Q_(delta,b) on a thread's 16 coordinates (chunk c) packed into FIELD-bit fields.
// Coordinates past the end of the vector must be passed as 0 (they encode as 0).
// Returns the number of nonzero codes.
template <int FIELD>
__device__ __forceinline__ int quantize16(const float (&v)[16], const Scale &s, const StreamKey &key, int64_t c,
                                          uint32_t (&w)[Words16<FIELD>::n])
{
    int nz = 0;
#pragma unroll
    for (int i = 0; i < Words16<FIELD>::n; ++i) w[i] = 0u;
    if (s.inv_delta == 0.0f) return 0;               // degenerate scale: all codes are zero
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const uint4 r = stream_block(key, static_cast<uint32_t>(c * 4 + g));
        constexpr int kB = CodeBias<FIELD>::value;
        const int k0 = quantize_one<kB>(v[4 * g], s, r.x), k1 = quantize_one<kB>(v[4 * g + 1], s, r.y);
        const int k2 = quantize_one<kB>(v[4 * g + 2], s, r.z), k3 = quantize_one<kB>(v[4 * g + 3], s, r.w);
        nz += (k0 != kB) + (k1 != kB) + (k2 != kB) + (k3 != kB);
        w[(4 * g * FIELD) / 32] |= pack4<FIELD, false, FIELD != 8>(k0, k1, k2, k3) << ((4 * g * FIELD) % 32);
    }
    if constexpr (FIELD != 8) {
#pragma unroll
        for (int i = 0; i < Words16<FIELD>::n; ++i) w[i] ^= FieldTops<FIELD>::word;
    }
    return nz;
}

template <int FIELD>
__device__ __forceinline__ void store_words(uint32_t *__restrict__ out, int64_t c, int64_t row_words,
                                            const uint32_t (&w)[Words16<FIELD>::n])
{
    constexpr int kWords = Words16<FIELD>::n;
    const int64_t w0 = c * kWords;
    if (w0 + kWords <= row_words) {
        if constexpr (kWords == 4) reinterpret_cast<uint4 *>(out + w0)[0] = make_uint4(w[0], w[1], w[2], w[3]);
        else if constexpr (kWords == 2) reinterpret_cast<uint2 *>(out + w0)[0] = make_uint2(w[0], w[1]);
        else out[w0] = w[0];
    } else {
#pragma unroll
        for (int i = 0; i < kWords; ++i)
            if (w0 + i < row_words) out[w0 + i] = w[i];
    }
}

}  // namespace dq
