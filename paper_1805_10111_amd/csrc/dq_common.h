// Internal helpers shared by the HIP translation units of libdq (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <float.h>

#include "../../include/dq.h"

namespace dq {

constexpr int kWave = 64;

// ---- host-side error plumbing ------------------------------------------------
void set_last_error(hipError_t e);

#define DQ_HIP_TRY(expr)                                   \
    do {                                                   \
        hipError_t e_ = (expr);                            \
        if (e_ != hipSuccess) {                            \
            ::dq::set_last_error(e_);                      \
            return DQ_ERR_DEVICE;                          \
        }                                                  \
    } while (0)

#define DQ_LAUNCH_CHECK() DQ_HIP_TRY(hipGetLastError())

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline int64_t packed_words(int64_t d, int b) { return (d * b + 31) / 32; }

// ---- Philox4x32-10 (Salmon et al., SC'11), from its published definition -------
// Stream addressing: key = (seed_lo, seed_hi); counter = (coord/4, iter, worker, tag).
struct StreamKey {
    uint32_t k0, k1;      // seed halves
    uint32_t iter, worker, tag;
};

__device__ __forceinline__ uint4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                               uint32_t k0, uint32_t k1)
{
    constexpr uint32_t kMul0 = 0xD2511F53u, kMul1 = 0xCD9E8D57u;
    constexpr uint32_t kWeyl0 = 0x9E3779B9u, kWeyl1 = 0xBB67AE85u;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = static_cast<uint64_t>(kMul0) * c0;
        const uint64_t p1 = static_cast<uint64_t>(kMul1) * c2;
        // a ^ b ^ c as one three-input bit operation (truth table 0x96) instead of two exclusive-ors
        const uint32_t n0 = __builtin_amdgcn_bitop3_b32(static_cast<uint32_t>(p1 >> 32), c1, k0, 0x96);
        const uint32_t n2 = __builtin_amdgcn_bitop3_b32(static_cast<uint32_t>(p0 >> 32), c3, k1, 0x96);
        c1 = static_cast<uint32_t>(p1);
        c3 = static_cast<uint32_t>(p0);
        c0 = n0;
        c2 = n2;
        k0 += kWeyl0;
        k1 += kWeyl1;
    }
    return make_uint4(c0, c1, c2, c3);
}

// The four 32-bit variates of coordinates 4*block .. 4*block+3 of a stream.
__device__ __forceinline__ uint4 stream_block(const StreamKey &s, uint32_t block)
{
    return philox4x32_10(block, s.iter, s.worker, s.tag, s.k0, s.k1);
}

// Single variate of one coordinate (slow path: tails, samplers).
__device__ __forceinline__ uint32_t stream_word(const StreamKey &s, uint64_t coord)
{
    const uint4 w = stream_block(s, static_cast<uint32_t>(coord >> 2));
    const uint32_t lane = static_cast<uint32_t>(coord & 3u);
    return lane == 0 ? w.x : lane == 1 ? w.y : lane == 2 ? w.z : w.w;
}

// "u < p" with u = (word >> 8) * 2^-24: both sides scaled by 2^24 are exact floats.
__device__ __forceinline__ bool bernoulli(uint32_t word, float p)
{
    return static_cast<float>(word >> 8) < p * 16777216.0f;
}

// ---- quantizer scalars -------------------------------------------------------
// Everything the per-coordinate rule needs, derived from ||v||_inf and b.
struct Scale {
    float delta;      // amax / L, or 0 (degenerate), or non-finite
    float inv_delta;  // L / amax (0 when codes must be all zero)
    float tmin, tmax; // code range -2^(b-1) .. L as floats
    bool bad;         // non-finite delta
};

__device__ __forceinline__ Scale make_scale(float amax, int b)
{
    Scale s;
    const int L = (1 << (b - 1)) - 1;
    s.tmin = -static_cast<float>(1 << (b - 1));
    s.tmax = static_cast<float>(L);
    float delta = amax / static_cast<float>(L);
    s.bad = !(delta == delta) || delta > FLT_MAX;           // NaN or Inf
    if (s.bad) {
        s.delta = delta;
        s.inv_delta = 0.0f;
    } else if (!(delta >= FLT_MIN)) {                        // zero or subnormal scale
        s.delta = 0.0f;
        s.inv_delta = 0.0f;
    } else {
        s.delta = delta;
        s.inv_delta = static_cast<float>(L) / amax;
    }
    return s;
}

// One coordinate of Q_(delta,b): returns the integer code plus BIAS (a bias rides for free on the add-with-carry
// that applies the rounding decision; the packers of 2- and 4-bit fields want codes made non-negative that way).
template <int BIAS = 0>
__device__ __forceinline__ int quantize_one(float v, const Scale &s, uint32_t word)
{
    // The code is clamped to [-2^(b-1), L].  Clamping v/delta to that range first (one three-operand median) gives
    // the same code as clamping the rounded integer: inside the range nothing changes (floor(t) + 1 <= L for
    // t < L, and t = L has p = 0), and outside it t becomes a bound, whose code is that bound.
    const float t = __builtin_amdgcn_fmed3f(v * s.inv_delta, s.tmin, s.tmax);
    const float z = floorf(t);
    const float p = t - z;
    return static_cast<int>(z) + BIAS + (bernoulli(word, p) ? 1 : 0);
}

// ---- kernel arguments ------------------------------------------------------------
// The arguments of a kernel lie in memory and are read with scalar loads where the compiler first needs them; a
// kernel whose arguments span several 64-byte lines so pays one trip to memory per line, one after the other, spread
// over its prologue (measured: 0.5-0.7 us each).  Reading one word of every line at the very start puts those trips
// side by side: what follows finds its arguments in the scalar cache.  BYTES: size of the kernel's arguments.
template <int BYTES>
__device__ __forceinline__ void touch_kernel_arguments()
{
    typedef const uint32_t __attribute__((address_space(4))) *const_words;
    const_words ka = (const_words)__builtin_amdgcn_kernarg_segment_ptr();
    uint32_t t = ka[(BYTES - 1) / 4];
#pragma unroll
    for (int w = 0; w < BYTES / 4; w += 16) t ^= ka[w];
    asm volatile("" ::"s"(t));            // (the loads must be made, their result is of no interest)
}

// ---- magnitude bit pattern: monotone in |v| for non-NaN, NaN sorts above Inf ----
__device__ __forceinline__ uint32_t abs_bits(float v) { return __float_as_uint(v) & 0x7FFFFFFFu; }

// ---- wave / block reductions (fixed order, hence deterministic) ---------------------
// Cross-lane moves on the VALU data path (DPP) instead of LDS permutes: two quad
// permutes, two row shifts and two row broadcasts leave the wave's total in lane 63,
// from where it is read back as a wave-uniform value.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int dpp_move_or_zero(int v)
{
    return __builtin_amdgcn_update_dpp(0, v, CTRL, ROW_MASK, 0xf, true);
}

#define DQ_WAVE_REDUCE(v, OP, TO_INT, FROM_INT)                                               \
    do {                                                                                      \
        v = OP(v, FROM_INT(dpp_move_or_zero<0xb1, 0xf>(TO_INT(v))));  /* quad_perm [1,0,3,2] */ \
        v = OP(v, FROM_INT(dpp_move_or_zero<0x4e, 0xf>(TO_INT(v))));  /* quad_perm [2,3,0,1] */ \
        v = OP(v, FROM_INT(dpp_move_or_zero<0x114, 0xf>(TO_INT(v)))); /* row_shr:4           */ \
        v = OP(v, FROM_INT(dpp_move_or_zero<0x118, 0xf>(TO_INT(v)))); /* row_shr:8           */ \
        v = OP(v, FROM_INT(dpp_move_or_zero<0x142, 0xa>(TO_INT(v)))); /* row_bcast:15        */ \
        v = OP(v, FROM_INT(dpp_move_or_zero<0x143, 0xc>(TO_INT(v)))); /* row_bcast:31        */ \
        v = FROM_INT(__builtin_amdgcn_readlane(TO_INT(v), 63));                                \
    } while (0)

__device__ __forceinline__ float dq_addf(float a, float b) { return a + b; }
__device__ __forceinline__ int dq_addi(int a, int b) { return a + b; }
__device__ __forceinline__ uint32_t dq_maxu(uint32_t a, uint32_t b) { return max(a, b); }
__device__ __forceinline__ int dq_u2i(uint32_t a) { return static_cast<int>(a); }
__device__ __forceinline__ uint32_t dq_i2u(int a) { return static_cast<uint32_t>(a); }
__device__ __forceinline__ int dq_id(int a) { return a; }

__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v)
{
    DQ_WAVE_REDUCE(v, dq_maxu, dq_u2i, dq_i2u);     // lanes without a source contribute 0, the identity of max
    return v;
}

__device__ __forceinline__ float wave_sum_f32(float v)
{
    DQ_WAVE_REDUCE(v, dq_addf, __float_as_int, __int_as_float);
    return v;
}

__device__ __forceinline__ int wave_sum_i32(int v)
{
    DQ_WAVE_REDUCE(v, dq_addi, dq_id, dq_id);
    return v;
}

__device__ __forceinline__ double wave_sum_f64(double v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

// Block-wide reductions; `scratch` has >= blockDim.x/64 entries (at most 64 wavefronts).  Result in all threads.
// Every wavefront leaves its value in scratch, then every wavefront reduces those (one LDS read per lane and a second
// cross-lane reduction) -- a loop over scratch would wait for one LDS read after the other.
__device__ __forceinline__ uint32_t block_max_u32(uint32_t v, uint32_t *scratch)
{
    v = wave_max_u32(v);
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave, nw = (blockDim.x + kWave - 1) / kWave;
    __syncthreads();
    if (lane == 0) scratch[wave] = v;
    __syncthreads();
    return wave_max_u32(lane < nw ? scratch[lane] : 0u);
}

__device__ __forceinline__ double block_sum_f64(double v, double *scratch)
{
    v = wave_sum_f64(v);
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave, nw = (blockDim.x + kWave - 1) / kWave;
    __syncthreads();
    if (lane == 0) scratch[wave] = v;
    __syncthreads();
    return wave_sum_f64(lane < nw ? scratch[lane] : 0.0);
}

__device__ __forceinline__ int block_sum_i32(int v, int *scratch)
{
    v = wave_sum_i32(v);
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave, nw = (blockDim.x + kWave - 1) / kWave;
    __syncthreads();
    if (lane == 0) scratch[wave] = v;
    __syncthreads();
    return wave_sum_i32(lane < nw ? scratch[lane] : 0);
}

// Both at once (one pair of barriers): m becomes the block-wide max, s the block-wide sum.
__device__ __forceinline__ void block_max_u32_sum_i32(uint32_t &m, int &s, uint32_t *scratch_m, int *scratch_s)
{
    m = wave_max_u32(m);
    s = wave_sum_i32(s);
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave, nw = (blockDim.x + kWave - 1) / kWave;
    __syncthreads();
    if (lane == 0) {
        scratch_m[wave] = m;
        scratch_s[wave] = s;
    }
    __syncthreads();
    m = wave_max_u32(lane < nw ? scratch_m[lane] : 0u);
    s = wave_sum_i32(lane < nw ? scratch_s[lane] : 0);
}

// ---- values left per slice by several producers of one row -----------------------
// A row's largest magnitude / count arrives as up to kMaxParts values.  All of them are requested at once (an index
// past the last one re-reads the last one): a loop that stops at `parts` would wait for every load before the next.
constexpr int kMaxParts = 8;

// (in two steps for callers that have other work to place between the requests and the first use of their result)
struct PartsRaw {
    float t[kMaxParts];
};

__device__ __forceinline__ PartsRaw parts_request(const float *__restrict__ v, int parts)
{
    PartsRaw r;
#pragma unroll
    for (int s = 0; s < kMaxParts; ++s) r.t[s] = v[min(s, parts - 1)];
    return r;
}

__device__ __forceinline__ float parts_absmax_of(const PartsRaw &r)
{
    float amax = r.t[0];               // (magnitudes compare like their bit patterns, and so does a NaN)
#pragma unroll
    for (int s = 1; s < kMaxParts; ++s) amax = __float_as_uint(r.t[s]) > __float_as_uint(amax) ? r.t[s] : amax;
    return amax;
}

__device__ __forceinline__ float parts_absmax(const float *__restrict__ v, int parts)
{
    return parts_absmax_of(parts_request(v, parts));
}

__device__ __forceinline__ int parts_sum(const int32_t *__restrict__ v, int parts)
{
    int t[kMaxParts];
#pragma unroll
    for (int s = 0; s < kMaxParts; ++s) t[s] = v[min(s, parts - 1)];
    int sum = 0;
#pragma unroll
    for (int s = 0; s < kMaxParts; ++s) sum += s < parts ? t[s] : 0;
    return sum;
}

// Sign-extended bit field [offset, offset+width) of a word.  (The builtin returns its
// result as an unsigned value; the conversion to int here keeps later int->float
// conversions signed.)
__device__ __forceinline__ int sext_field(uint32_t word, unsigned offset, unsigned width)
{
    return static_cast<int>(__builtin_amdgcn_sbfe(word, offset, width));
}

}  // namespace dq
