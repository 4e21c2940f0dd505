// Sparse message format of Section 4.2 of the paper: a sparsified, quantized gradient is sent as
// its scale plus, per nonzero coordinate, ceil(log2 d) bits of position and b bits of value.
// Encoder: packed dense codes -> entry stream (order-preserving compaction); decoder: the inverse.
// One block of 1024 threads per worker; the stream (encoder) or the dense row (decoder) is
// assembled in LDS with bitwise-OR atomics on disjoint bits (order-free, hence deterministic).
#include <mutex>

#include "dq_common.h"
#include "elementwise.h"

namespace dq {

constexpr int kWireThreads = 1024;
constexpr int64_t kWireLdsWords = 36 * 1024;          // 144 KB of the 160 KB per compute unit

static inline int position_bits(int64_t d)
{
    int bits = 0;
    while ((int64_t{1} << bits) < d) ++bits;
    return bits;
}

// Inclusive prefix sum over the block's threads; `scratch` holds one int per thread.  Returns the
// inclusive sum of this thread; *total receives the block total.
__device__ __forceinline__ int block_scan_inclusive(int v, int *scratch, int *total)
{
    scratch[threadIdx.x] = v;
    __syncthreads();
    for (int off = 1; off < kWireThreads; off <<= 1) {
        const int add = threadIdx.x >= static_cast<unsigned>(off) ? scratch[threadIdx.x - off] : 0;
        __syncthreads();
        scratch[threadIdx.x] += add;
        __syncthreads();
    }
    const int r = scratch[threadIdx.x];
    *total = scratch[kWireThreads - 1];
    __syncthreads();
    return r;
}

__device__ __forceinline__ void or_bits(uint32_t *words, int64_t bit, uint64_t value, int width)
{
    const int64_t w = bit >> 5;
    const int sh = static_cast<int>(bit & 31);
    const uint64_t shifted = value << sh;                        // width + sh <= 63
    atomicOr(words + w, static_cast<uint32_t>(shifted));
    if (sh + width > 32) atomicOr(words + w + 1, static_cast<uint32_t>(shifted >> 32));
}

template <int FIELD>
__global__ __launch_bounds__(kWireThreads) void sparse_encode_kernel(
    const uint32_t *__restrict__ packed, int64_t ld_words, int64_t row_words, int64_t d, int pos_bits,
    uint32_t *__restrict__ stream, int64_t ld_stream, int64_t cap_words, int32_t *__restrict__ nnz_out)
{
    extern __shared__ uint32_t sh_stream[];
    __shared__ int sh_scan[kWireThreads];
    const int m = blockIdx.x;
    const uint32_t *row = packed + static_cast<int64_t>(m) * ld_words;
    for (int64_t w = threadIdx.x; w < cap_words; w += kWireThreads) sh_stream[w] = 0u;
    __syncthreads();
    const int E = pos_bits + FIELD;
    const int64_t chunks = (d + 15) / 16;
    int base = 0;                                                 // entries emitted by earlier chunk rounds
    for (int64_t c0 = 0; c0 < chunks; c0 += kWireThreads) {
        const int64_t c = c0 + threadIdx.x;
        uint32_t w[Words16<FIELD>::n];
        int count = 0;
        if (c < chunks) {
            load_words<FIELD>(row, c, row_words, w);
#pragma unroll
            for (int j = 0; j < 16; ++j) count += (c * 16 + j < d && code_of<FIELD>(w, j) != 0) ? 1 : 0;
        }
        int total;
        int e = base + block_scan_inclusive(count, sh_scan, &total) - count;     // first entry of this chunk
        if (c < chunks) {
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const int64_t i = c * 16 + j;
                const int k = code_of<FIELD>(w, j);
                if (i < d && k != 0) {
                    const uint64_t entry = static_cast<uint64_t>(i) |
                                           (static_cast<uint64_t>(static_cast<uint32_t>(k) & ((1u << FIELD) - 1u)) << pos_bits);
                    or_bits(sh_stream, static_cast<int64_t>(e) * E, entry, E);
                    ++e;
                }
            }
        }
        base += total;
    }
    __syncthreads();
    uint32_t *out = stream + static_cast<int64_t>(m) * ld_stream;
    for (int64_t w = threadIdx.x; w < cap_words; w += kWireThreads) out[w] = sh_stream[w];
    if (threadIdx.x == 0) nnz_out[m] = base;
}

template <int FIELD>
__global__ __launch_bounds__(kWireThreads) void sparse_decode_kernel(
    const uint32_t *__restrict__ stream, int64_t ld_stream, const int32_t *__restrict__ nnz, int64_t d, int pos_bits,
    uint32_t *__restrict__ packed, int64_t ld_words, int64_t row_words)
{
    extern __shared__ uint32_t sh_row[];
    const int m = blockIdx.x;
    const uint32_t *in = stream + static_cast<int64_t>(m) * ld_stream;
    for (int64_t w = threadIdx.x; w < row_words; w += kWireThreads) sh_row[w] = 0u;
    __syncthreads();
    const int E = pos_bits + FIELD;
    const int count = nnz[m];
    for (int e = threadIdx.x; e < count; e += kWireThreads) {
        const int64_t bit = static_cast<int64_t>(e) * E;
        const int64_t w = bit >> 5;
        const int sh = static_cast<int>(bit & 31);
        uint64_t v = in[w];
        if (sh + E > 32) v |= static_cast<uint64_t>(in[w + 1]) << 32;
        const uint64_t entry = (v >> sh) & ((uint64_t{1} << E) - 1);
        const int64_t pos = static_cast<int64_t>(entry & ((uint64_t{1} << pos_bits) - 1));
        const uint32_t field = static_cast<uint32_t>(entry >> pos_bits);
        if (pos < d) atomicOr(sh_row + ((pos * FIELD) >> 5), field << ((pos * FIELD) & 31));
    }
    __syncthreads();
    uint32_t *out = packed + static_cast<int64_t>(m) * ld_words;
    for (int64_t w = threadIdx.x; w < row_words; w += kWireThreads) out[w] = sh_row[w];
}

template <auto kernel>
static int allow_lds()
{
    // one flag and one result per kernel (every instantiation has its own): set once per process, safely from any thread
    static std::once_flag once;
    static hipError_t once_rc = hipSuccess;
    std::call_once(once, [&] {
        once_rc = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                      static_cast<int>(kWireLdsWords * 4));
    });
    DQ_HIP_TRY(once_rc);
    return DQ_OK;
}

}  // namespace dq

using namespace dq;
static inline hipStream_t as_stream(void *s) { return reinterpret_cast<hipStream_t>(s); }

extern "C" int64_t dq_sparse_stream_words(int64_t d, int32_t b)
{
    if (d <= 0 || b < 2 || b > 8) return DQ_ERR_INVALID_ARG;
    return (d * (position_bits(d) + b) + 31) / 32;
}

extern "C" int32_t dq_sparse_encode(const uint32_t *packed, int64_t ld_words, int64_t d, int64_t M, int32_t b,
                                    uint32_t *stream_out, int64_t ld_stream, int32_t *nnz_out, void *stream)
{
    if (d <= 0 || M <= 0 || !packed || !stream_out || !nnz_out) return DQ_ERR_INVALID_ARG;
    if (b != 2 && b != 4 && b != 8) return (b >= 2 && b <= 8) ? DQ_ERR_UNSUPPORTED : DQ_ERR_INVALID_ARG;
    const int64_t row_words = packed_words(d, b), cap = dq_sparse_stream_words(d, b);
    if (ld_words < row_words || ld_stream < cap || !aligned16(packed) || (M > 1 && ld_words % 4 != 0)) return DQ_ERR_INVALID_ARG;
    if (cap > kWireLdsWords) return DQ_ERR_UNSUPPORTED;
    const int pb = position_bits(d);
    const size_t lds = static_cast<size_t>(cap) * 4;
    const dim3 grid(static_cast<unsigned>(M)), block(kWireThreads);
    hipStream_t st = as_stream(stream);
    int rc;
    if (b == 8) { if ((rc = allow_lds<sparse_encode_kernel<8>>()) != DQ_OK) return rc; sparse_encode_kernel<8><<<grid, block, lds, st>>>(packed, ld_words, row_words, d, pb, stream_out, ld_stream, cap, nnz_out); }
    else if (b == 4) { if ((rc = allow_lds<sparse_encode_kernel<4>>()) != DQ_OK) return rc; sparse_encode_kernel<4><<<grid, block, lds, st>>>(packed, ld_words, row_words, d, pb, stream_out, ld_stream, cap, nnz_out); }
    else { if ((rc = allow_lds<sparse_encode_kernel<2>>()) != DQ_OK) return rc; sparse_encode_kernel<2><<<grid, block, lds, st>>>(packed, ld_words, row_words, d, pb, stream_out, ld_stream, cap, nnz_out); }
    DQ_LAUNCH_CHECK();
    return DQ_OK;
}

extern "C" int32_t dq_sparse_decode(const uint32_t *stream_in, int64_t ld_stream, const int32_t *nnz, int64_t d, int64_t M,
                                    int32_t b, uint32_t *packed_out, int64_t ld_words, void *stream)
{
    if (d <= 0 || M <= 0 || !stream_in || !nnz || !packed_out) return DQ_ERR_INVALID_ARG;
    if (b != 2 && b != 4 && b != 8) return (b >= 2 && b <= 8) ? DQ_ERR_UNSUPPORTED : DQ_ERR_INVALID_ARG;
    const int64_t row_words = packed_words(d, b), cap = dq_sparse_stream_words(d, b);
    if (ld_words < row_words || ld_stream < cap) return DQ_ERR_INVALID_ARG;
    if (row_words > kWireLdsWords) return DQ_ERR_UNSUPPORTED;
    const int pb = position_bits(d);
    const size_t lds = static_cast<size_t>(row_words) * 4;
    const dim3 grid(static_cast<unsigned>(M)), block(kWireThreads);
    hipStream_t st = as_stream(stream);
    int rc;
    if (b == 8) { if ((rc = allow_lds<sparse_decode_kernel<8>>()) != DQ_OK) return rc; sparse_decode_kernel<8><<<grid, block, lds, st>>>(stream_in, ld_stream, nnz, d, pb, packed_out, ld_words, row_words); }
    else if (b == 4) { if ((rc = allow_lds<sparse_decode_kernel<4>>()) != DQ_OK) return rc; sparse_decode_kernel<4><<<grid, block, lds, st>>>(stream_in, ld_stream, nnz, d, pb, packed_out, ld_words, row_words); }
    else { if ((rc = allow_lds<sparse_decode_kernel<2>>()) != DQ_OK) return rc; sparse_decode_kernel<2><<<grid, block, lds, st>>>(stream_in, ld_stream, nnz, d, pb, packed_out, ld_words, row_words); }
    DQ_LAUNCH_CHECK();
    return DQ_OK;
}
