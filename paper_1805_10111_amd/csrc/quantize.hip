// Quantizer family: ||v||_inf reduction, stochastic quantization, bit packing,
// unpacking and the master's decode-and-sum (Section 3.1 of the paper; Alg. 1,
// master (i)/(ii) and worker (ii)).  All kernels stream their operands once with
// 128-bit accesses; each thread owns 16 consecutive coordinates so that it emits
// whole 32-bit words for every supported field width.
#include "dq_common.h"
#include "elementwise.h"

namespace dq {

constexpr int kThreads = 256;
constexpr int kCoordsPerThread = 16;
constexpr int64_t kMaxBlocksX = 1 << 24;   // one 16-coordinate chunk per thread up to 2^36 coordinates, grid-stride beyond

static inline dim3 grid_for(int64_t d, int64_t M)
{
    const int64_t chunks = ceil_div(d, kCoordsPerThread);
    int64_t bx = ceil_div(chunks, kThreads);
    if (bx > kMaxBlocksX) bx = kMaxBlocksX;
    if (bx < 1) bx = 1;
    return dim3(static_cast<unsigned>(bx), static_cast<unsigned>(M), 1);
}

// ---------------------------------------------------------------- fill
__global__ void fill_u32_kernel(uint32_t *p, int64_t n, uint32_t value)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < n) p[i] = value;
}

int fill_u32(uint32_t *p, int64_t n, uint32_t value, hipStream_t st)
{
    if (n <= 0) return DQ_OK;
    fill_u32_kernel<<<dim3(static_cast<unsigned>(ceil_div(n, 256))), dim3(256), 0, st>>>(p, n, value);
    DQ_LAUNCH_CHECK();
    return DQ_OK;
}

// ---------------------------------------------------------------- absmax
// Max over the magnitude bit patterns: exact, order-free, NaN-propagating.
__global__ __launch_bounds__(kThreads) void absmax_kernel(const float *__restrict__ v, int64_t d, int64_t ld,
                                                          uint32_t *__restrict__ absmax_bits)
{
    __shared__ uint32_t scratch[kThreads / kWave];
    const float *row = v + static_cast<int64_t>(blockIdx.y) * ld;
    // a block sweeps tiles of 4 x 256 quads; within a tile consecutive lanes read consecutive quads
    const int64_t quads = (d + 3) / 4;
    const int64_t tiles = (quads + 4 * kThreads - 1) / (4 * kThreads);
    uint32_t m = 0;
    for (int64_t t = blockIdx.x; t < tiles; t += gridDim.x) {
        const int64_t q0 = t * 4 * kThreads + threadIdx.x;
        float4 a[4];
        if ((t + 1) * 16 * kThreads <= d) {                  // a whole tile (the same for every thread): no condition
#pragma unroll                                               // on any load, so all four are in flight together
            for (int k = 0; k < 4; ++k) a[k] = load_f4_stream(row + 4 * (q0 + k * kThreads));
        } else {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int64_t q = q0 + k * kThreads;
                a[k] = q < quads ? load_quad(row, q, d) : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            }
        }
#pragma unroll
        for (int k = 0; k < 4; ++k)
            m = max(m, max(max(abs_bits(a[k].x), abs_bits(a[k].y)), max(abs_bits(a[k].z), abs_bits(a[k].w))));
    }
    m = block_max_u32(m, scratch);
    if (threadIdx.x == 0 && m != 0) atomicMax(absmax_bits + blockIdx.y, m);
}

int launch_absmax(const float *v, int64_t d, int64_t M, int64_t ld, float *absmax_out, hipStream_t st)
{
    int rc = fill_u32(reinterpret_cast<uint32_t *>(absmax_out), M, 0u, st);
    if (rc != DQ_OK) return rc;
    if (d > 0) {
        // every block ends in one atomic on the row's slot: keep the grid small (grid-stride loop)
        dim3 grid = grid_for(d, M);
        const unsigned cap = static_cast<unsigned>(ceil_div(1024, M));   // (measured on 2^28 coordinates: 1024 blocks 152 us,
                                                                         // 4096 blocks 169 us, 16384 blocks 239 us)
        if (grid.x > cap) grid.x = cap;
        absmax_kernel<<<grid, dim3(kThreads), 0, st>>>(v, d, ld, reinterpret_cast<uint32_t *>(absmax_out));
        DQ_LAUNCH_CHECK();
    }
    return DQ_OK;
}

// ---------------------------------------------------------------- any width 2 <= b <= 16
// The model-precision study of Section 5.2 varies b_x from 2 to 11, so fields may straddle the
// 32-bit words of a packed row.  A group of 32 consecutive coordinates always occupies exactly b
// whole words (words g*b .. g*b+b-1 of the row), so one thread takes one group and streams its
// fields through a 64-bit shift register: no two threads ever touch the same word.
constexpr int kGroupCoords = 32;

static inline dim3 grid_for_groups(int64_t d, int64_t M)
{
    const int64_t groups = ceil_div(d > 0 ? d : 1, kGroupCoords);
    return dim3(static_cast<unsigned>(ceil_div(groups, kThreads)), static_cast<unsigned>(M));
}

__global__ __launch_bounds__(kThreads) void quantize_pack_any_kernel(
    const float *__restrict__ v, int64_t d, int64_t ld, const float *__restrict__ absmax, int b, StreamKey key,
    uint32_t worker0, uint32_t *__restrict__ packed, int64_t ld_words, int64_t row_words,
    float *__restrict__ delta_out, uint32_t *__restrict__ status)
{
    const int m = blockIdx.y;
    const float *row = v + static_cast<int64_t>(m) * ld;
    uint32_t *out = packed + static_cast<int64_t>(m) * ld_words;
    const Scale s = make_scale(absmax[m], b);
    key.worker = worker0 + static_cast<uint32_t>(m);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        delta_out[m] = s.delta;
        if (s.bad && status) atomicOr(status, 1u);
    }
    const int64_t g = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
    const int64_t base = g * kGroupCoords;
    if (base >= d) return;
    const uint64_t mask = (1ull << b) - 1ull;
    uint64_t window = 0;                     // bits not yet written, low bits first
    int fill = 0;
    int64_t wo = g * b;
    for (int j = 0; j < kGroupCoords; j += 4) {
        const float4 a = load_quad(row, (base + j) >> 2, d);          // zeros past the end -> code 0
        const float av[4] = {a.x, a.y, a.z, a.w};
        uint32_t rw[4] = {0u, 0u, 0u, 0u};
        if (s.inv_delta != 0.0f && base + j < d) {
            const uint4 r = stream_block(key, static_cast<uint32_t>((base + j) >> 2));
            rw[0] = r.x; rw[1] = r.y; rw[2] = r.z; rw[3] = r.w;
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int k = (s.inv_delta != 0.0f && base + j + e < d) ? quantize_one(av[e], s, rw[e]) : 0;
            window |= (static_cast<uint64_t>(static_cast<uint32_t>(k)) & mask) << fill;
            fill += b;
            if (fill >= 32) {
                if (wo < row_words) out[wo] = static_cast<uint32_t>(window);
                ++wo;
                window >>= 32;
                fill -= 32;
            }
        }
    }
}

__global__ __launch_bounds__(kThreads) void unpack_dequant_sum_any_kernel(
    const uint32_t *__restrict__ packed, int64_t ld_words, int64_t row_words, const float *__restrict__ delta,
    int64_t d, int M, int b, float scale, float *__restrict__ out)
{
    const int64_t g = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
    const int64_t base = g * kGroupCoords;
    if (base >= d) return;
    float acc[kGroupCoords];
#pragma unroll
    for (int j = 0; j < kGroupCoords; ++j) acc[j] = 0.0f;
    for (int m = 0; m < M; ++m) {
        const uint32_t *row = packed + static_cast<int64_t>(m) * ld_words;
        const float dm = delta[m];
        uint64_t window = 0;
        int fill = 0;
        int64_t wi = g * b;
#pragma unroll
        for (int j = 0; j < kGroupCoords; ++j) {
            if (fill < b) {
                const uint32_t w = wi < row_words ? row[wi] : 0u;
                ++wi;
                window |= static_cast<uint64_t>(w) << fill;
                fill += 32;
            }
            const int k = sext_field(static_cast<uint32_t>(window), 0, static_cast<unsigned>(b));
            window >>= b;
            fill -= b;
            acc[j] = fmaf(dm, static_cast<float>(k), acc[j]);
        }
    }
#pragma unroll
    for (int j = 0; j < kGroupCoords; j += 4)
        store_quad(out, (base + j) >> 2, d, make_float4(scale * acc[j], scale * acc[j + 1], scale * acc[j + 2], scale * acc[j + 3]));
}

// int8 codes <-> fields of any width 2 <= b <= 8
__global__ __launch_bounds__(kThreads) void pack_any_kernel(const int8_t *__restrict__ codes, int64_t ld_codes, int64_t d,
                                                            int b, uint32_t *__restrict__ packed, int64_t ld_words,
                                                            int64_t row_words)
{
    const int m = blockIdx.y;
    const int8_t *in = codes + static_cast<int64_t>(m) * ld_codes;
    uint32_t *out = packed + static_cast<int64_t>(m) * ld_words;
    const int64_t g = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
    const int64_t base = g * kGroupCoords;
    if (base >= d) return;
    const uint64_t mask = (1ull << b) - 1ull;
    uint64_t window = 0;
    int fill = 0;
    int64_t wo = g * b;
    for (int j = 0; j < kGroupCoords; ++j) {
        const int k = base + j < d ? in[base + j] : 0;
        window |= (static_cast<uint64_t>(static_cast<uint32_t>(k)) & mask) << fill;
        fill += b;
        if (fill >= 32) {
            if (wo < row_words) out[wo] = static_cast<uint32_t>(window);
            ++wo;
            window >>= 32;
            fill -= 32;
        }
    }
}

__global__ __launch_bounds__(kThreads) void unpack_any_kernel(const uint32_t *__restrict__ packed, int64_t ld_words,
                                                              int64_t row_words, int64_t d, int b,
                                                              int8_t *__restrict__ codes, int64_t ld_codes)
{
    const int m = blockIdx.y;
    const uint32_t *row = packed + static_cast<int64_t>(m) * ld_words;
    int8_t *out = codes + static_cast<int64_t>(m) * ld_codes;
    const int64_t g = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
    const int64_t base = g * kGroupCoords;
    if (base >= d) return;
    uint64_t window = 0;
    int fill = 0;
    int64_t wi = g * b;
    for (int j = 0; j < kGroupCoords; ++j) {
        if (fill < b) {
            const uint32_t w = wi < row_words ? row[wi] : 0u;
            ++wi;
            window |= static_cast<uint64_t>(w) << fill;
            fill += 32;
        }
        const int k = sext_field(static_cast<uint32_t>(window), 0, static_cast<unsigned>(b));
        window >>= b;
        fill -= b;
        if (base + j < d) out[base + j] = static_cast<int8_t>(k);
    }
}

// ---------------------------------------------------------------- lane-contiguous access for 16 coordinates per thread
// A thread of the streaming kernels owns 16 consecutive coordinates (64 bytes), so that it emits whole words for
// every field width.  Read or written directly, that is four 16-byte accesses per lane at a lane stride of 64
// bytes: every instruction touches 64 different cache lines, a sixth of a line each.  Measured on 1 GiB with plain
// kernels: stores of that shape reach 3.6 TB/s against 6.1 TB/s for stores in which consecutive lanes write
// consecutive 16 bytes (a wavefront writes 1 KB of whole lines per instruction), loads 4.1 against 7.1 TB/s
// (non-temporal).  So memory is always accessed lane-contiguously -- quad 64 u + lane of the wavefront's tile of
// 256 quads by access u -- and the 4 KB tile is transposed through LDS (no barrier: a wavefront only exchanges
// data with itself).  Slot of quad q in the tile, skewed so that neither direction has bank conflicts: q + q / 8.
constexpr int kTileSlots = 256 + 256 / 8;                 // float4 slots per wavefront

__device__ __forceinline__ int tile_slot(int q) { return q + (q >> 3); }

// The thread's 16 coordinates (quads 4 lane .. 4 lane + 3 of the tile that starts at `tile`, whole and inside the
// vector) from lane-contiguous non-temporal loads.
__device__ __forceinline__ void load16_tile(const float *__restrict__ tile, float4 *__restrict__ lds, int lane, float (&a)[16])
{
    float4 t[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) t[u] = load_f4_stream(tile + 4 * (64 * u + lane));
#pragma unroll
    for (int u = 0; u < 4; ++u) lds[tile_slot(64 * u + lane)] = t[u];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const float4 v = lds[tile_slot(4 * lane + u)];
        a[4 * u] = v.x; a[4 * u + 1] = v.y; a[4 * u + 2] = v.z; a[4 * u + 3] = v.w;
    }
    __builtin_amdgcn_wave_barrier();                      // the tile is free again only when every lane has read
}

// The inverse: the thread's 16 values leave as lane-contiguous 16-byte stores.
__device__ __forceinline__ void store16_tile(float *__restrict__ tile, float4 *__restrict__ lds, int lane, const float (&a)[16])
{
#pragma unroll
    for (int u = 0; u < 4; ++u) lds[tile_slot(4 * lane + u)] = make_float4(a[4 * u], a[4 * u + 1], a[4 * u + 2], a[4 * u + 3]);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    float4 t[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) t[u] = lds[tile_slot(64 * u + lane)];
#pragma unroll
    for (int u = 0; u < 4; ++u) *reinterpret_cast<float4 *>(tile + 4 * (64 * u + lane)) = t[u];
    __builtin_amdgcn_wave_barrier();
}

// ---------------------------------------------------------------- quantize (+pack)
// FIELD = width of the stored field (2, 4, 8 bits); `b` = bits of the code range.
// With FIELD == 8 and any b in [2,8] the output words are four int8 codes each.
// TILE: the input is read lane-contiguously and transposed through LDS (see load16_tile).  Measured on 2^28
// coordinates it pays for 8-bit fields only (228 -> 220 us); with narrower fields, whose packing costs more
// arithmetic, the kernel is bound by instruction issue and the exchange costs more than the better access pattern
// brings (4 bits 214 -> 217 us, 2 bits 197 -> 212 us).
template <int FIELD, bool TILE = FIELD == 8>
__global__ __launch_bounds__(kThreads) void quantize_pack_kernel(
    const float *__restrict__ v, int64_t d, int64_t ld, const float *__restrict__ absmax, int b, StreamKey key,
    uint32_t worker0, uint32_t *__restrict__ packed, int64_t ld_words, int64_t row_words,
    float *__restrict__ delta_out, uint32_t *__restrict__ status, int parts, const int32_t *__restrict__ count_parts,
    int32_t *__restrict__ count_out)
{
    const int m = blockIdx.y;
    const float *row = v + static_cast<int64_t>(m) * ld;
    uint32_t *out = packed + static_cast<int64_t>(m) * ld_words;
    // the largest magnitude of row m, or the largest of the `parts` values that the producers of its slices left
    // (magnitudes compare like their bit patterns, and so does a NaN that has to reach the status word)
    const float amax = parts_absmax(absmax + static_cast<int64_t>(m) * parts, parts);
    const Scale s = make_scale(amax, b);
    key.worker = worker0 + static_cast<uint32_t>(m);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        delta_out[m] = s.delta;
        if (s.bad && status) atomicOr(status, 1u);
        // a per-slice count summed on the way (see csr_worker)
        if (count_out) count_out[m] = parts_sum(count_parts + static_cast<int64_t>(m) * parts, parts);
    }
    __shared__ float4 tiles[kThreads / kWave][kTileSlots];
    const int lane = threadIdx.x & (kWave - 1);
    float4 *lds = tiles[threadIdx.x / kWave];
    const int64_t chunks = (d + kCoordsPerThread - 1) / kCoordsPerThread;
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kThreads;
    // (the loop bound is the same for the whole wavefront: its lanes go through the tile exchange together)
    for (int64_t c0 = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x - lane; c0 < chunks; c0 += stride) {
        const int64_t c = c0 + lane;
        float a[16];
        if (TILE && (c0 + kWave) * kCoordsPerThread <= d) {          // the wavefront's 1024 coordinates are all there
            load16_tile(row + c0 * kCoordsPerThread, lds, lane, a);
        } else {
            if (c >= chunks) continue;
            load16(row, c * kCoordsPerThread, d, a);         // coordinates past d read as 0 -> code 0
        }
        uint32_t w[Words16<FIELD>::n];
        quantize16<FIELD>(a, s, key, c, w);
        store_words<FIELD>(out, c, row_words, w);
    }
}

// The model message of Alg. 1, master (i), for vectors of up to a million coordinates or so: such a launch is all
// latency, so a thread takes one quad (one Philox block) and everything it reads -- the scale's input, the model, the
// snapshot -- is requested before the Philox rounds, which depend on none of it, and waited for after them.
// DIFF: together with diff_out[i] = delta * code_i - x_snap[i], the model a worker decodes minus the snapshot, which
// every worker of the next round would otherwise form again, per column it touches, from the message (dq_run_rounds
// on CSR features).  Same bits as quantize_pack_kernel on one row with the master's stream.
template <int FIELD, bool DIFF>
__global__ __launch_bounds__(kThreads) void model_message_kernel(
    const float *__restrict__ x, int64_t d, const float *__restrict__ absmax, int b, StreamKey key,
    uint32_t *__restrict__ packed, float *__restrict__ delta_out, uint32_t *__restrict__ status,
    const float *__restrict__ x_snap, float *__restrict__ diff_out)
{
    touch_kernel_arguments<88>();                        // (five pointers, d, b, the key, three more pointers)
    const int64_t quads = (d + 3) / 4;
    const int64_t q = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
    const int64_t qc = min(q, quads - 1);                // (threads past the end repeat the last quad and store nothing)
    // (single elements at clamped positions: the same requests whether or not the vector ends inside a quad; and the
    // scale's input through a vector load like the rest -- as a scalar load it would share its counter with the
    // arguments that the Philox rounds need, and those would wait for it)
    int lane_zero;
    asm volatile("v_mov_b32 %0, 0" : "=v"(lane_zero));
    const float amax = absmax[lane_zero];
    float xv[4], sv[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        xv[e] = x[min(4 * qc + e, d - 1)];
        if constexpr (DIFF) sv[e] = x_snap[min(4 * qc + e, d - 1)];
    }
    key.worker = DQ_MASTER_ID;
    const uint4 r = stream_block(key, static_cast<uint32_t>(qc));
    asm volatile("" ::"v"(r.x), "v"(r.y), "v"(r.z), "v"(r.w));      // (the rounds stay ahead of the first wait)
    const Scale s = make_scale(amax, b);
    if (q == 0) {
        delta_out[0] = s.delta;
        if (s.bad && status) atomicOr(status, 1u);
    }
    constexpr int kB = CodeBias<FIELD>::value;
    int k[4] = {kB, kB, kB, kB};
    uint32_t bits = 0;
    if (s.inv_delta != 0.0f) {                           // (a degenerate scale: every code is zero)
#pragma unroll
        for (int e = 0; e < 4; ++e) xv[e] = 4 * qc + e < d ? xv[e] : 0.0f;      // past the end: code 0
        k[0] = quantize_one<kB>(xv[0], s, r.x); k[1] = quantize_one<kB>(xv[1], s, r.y);
        k[2] = quantize_one<kB>(xv[2], s, r.z); k[3] = quantize_one<kB>(xv[3], s, r.w);
        bits = pack4<FIELD, true, FIELD != 8>(k[0], k[1], k[2], k[3]);
    }
    // (every lane makes the call: lanes that share a word combine their bits; lanes past the end bring none)
    store_quad_bits<FIELD>(q < quads ? bits : 0u, q < quads ? q : quads, quads, packed);
    if (DIFF && q < quads) {
        float o[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = s.delta * static_cast<float>(k[e] - kB) - sv[e];
        if (4 * q + 3 < d) {
            reinterpret_cast<float4 *>(diff_out)[q] = make_float4(o[0], o[1], o[2], o[3]);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (4 * q + e < d) diff_out[4 * q + e] = o[e];
        }
    }
}

int launch_quantize_pack_parts(const float *v, int64_t d, int64_t M, int64_t ld, int b, int field, const float *absmax,
                               int parts, const int32_t *count_parts, int32_t *count_out, const StreamKey &key,
                               uint32_t worker0, uint32_t *packed, int64_t ld_words, float *delta_out, uint32_t *status,
                               hipStream_t st);

int launch_quantize_pack(const float *v, int64_t d, int64_t M, int64_t ld, int b, int field,
                         const float *absmax, const StreamKey &key, uint32_t worker0,
                         uint32_t *packed, int64_t ld_words, float *delta_out, uint32_t *status, hipStream_t st)
{
    return launch_quantize_pack_parts(v, d, M, ld, b, field, absmax, 1, nullptr, nullptr, key, worker0, packed, ld_words,
                                      delta_out, status, st);
}

// The model message (one row; widths 2, 4, 8) by model_message_kernel; x_snap and diff_out both given or both null.
int launch_model_message(const float *x, int64_t d, int b_x, const float *absmax, const StreamKey &key, uint32_t *packed,
                         float *delta_out, uint32_t *status, const float *x_snap, float *diff_out, hipStream_t st)
{
    if (d < 1 || (x_snap == nullptr) != (diff_out == nullptr)) return DQ_ERR_INVALID_ARG;
    const dim3 grid(static_cast<unsigned>(ceil_div(ceil_div(d, 4), kThreads))), block(kThreads);
#define DQ_MESSAGE(F)                                                                                                       \
    if (diff_out) model_message_kernel<F, true><<<grid, block, 0, st>>>(x, d, absmax, b_x, key, packed, delta_out, status, x_snap, diff_out); \
    else model_message_kernel<F, false><<<grid, block, 0, st>>>(x, d, absmax, b_x, key, packed, delta_out, status, nullptr, nullptr)
    switch (b_x) {
    case 8: DQ_MESSAGE(8); break;
    case 4: DQ_MESSAGE(4); break;
    case 2: DQ_MESSAGE(2); break;
    default: return DQ_ERR_UNSUPPORTED;
    }
#undef DQ_MESSAGE
    DQ_LAUNCH_CHECK();
    return DQ_OK;
}

// absmax holds `parts` values per row (the row's scale comes from their maximum); count_parts / count_out: optional
// per-slice counts and where their sum per row goes (widths 2, 4, 8 only).
int launch_quantize_pack_parts(const float *v, int64_t d, int64_t M, int64_t ld, int b, int field, const float *absmax,
                               int parts, const int32_t *count_parts, int32_t *count_out, const StreamKey &key,
                               uint32_t worker0, uint32_t *packed, int64_t ld_words, float *delta_out, uint32_t *status,
                               hipStream_t st)
{
    if (parts < 1 || parts > kMaxParts) return DQ_ERR_INVALID_ARG;
    const int64_t row_words = packed_words(d, field);
    const dim3 grid = grid_for(d, M), block(kThreads);
    switch (field) {
    case 8: quantize_pack_kernel<8><<<grid, block, 0, st>>>(v, d, ld, absmax, b, key, worker0, packed, ld_words, row_words, delta_out, status, parts, count_parts, count_out); break;
    case 4: quantize_pack_kernel<4><<<grid, block, 0, st>>>(v, d, ld, absmax, b, key, worker0, packed, ld_words, row_words, delta_out, status, parts, count_parts, count_out); break;
    case 2: quantize_pack_kernel<2><<<grid, block, 0, st>>>(v, d, ld, absmax, b, key, worker0, packed, ld_words, row_words, delta_out, status, parts, count_parts, count_out); break;
    default:
        if (field != b || b < 2 || b > 16 || parts != 1 || count_out) return DQ_ERR_UNSUPPORTED;
        quantize_pack_any_kernel<<<grid_for_groups(d, M), block, 0, st>>>(v, d, ld, absmax, b, key, worker0, packed, ld_words, row_words, delta_out, status);
        break;
    }
    DQ_LAUNCH_CHECK();
    return DQ_OK;
}

// ---------------------------------------------------------------- unpack + dequantize + sum over M
template <int FIELD>
__global__ __launch_bounds__(kThreads) void unpack_dequant_sum_kernel(
    const uint32_t *__restrict__ packed, int64_t ld_words, int64_t row_words, const float *__restrict__ delta,
    int64_t d, int M, float scale, float *__restrict__ out)
{
    __shared__ float4 tiles[kThreads / kWave][kTileSlots];
    const int lane = threadIdx.x & (kWave - 1);
    float4 *lds = tiles[threadIdx.x / kWave];
    const int64_t chunks = (d + kCoordsPerThread - 1) / kCoordsPerThread;
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kThreads;
    const bool scaled = (FIELD == 2 || FIELD == 4) && scales_divide_exactly(delta, M);
    for (int64_t c0 = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x - lane; c0 < chunks; c0 += stride) {
        const int64_t c = c0 + lane;
        const bool whole = (c0 + kWave) * kCoordsPerThread <= d;     // the wavefront's 1024 coordinates are all there
        if (!whole && c >= chunks) continue;
        float acc[16];
        decode_sum16<FIELD, true>(packed, ld_words, row_words, delta, M, c, d, scaled, acc);
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[j] = scale * acc[j];
        if (whole) store16_tile(out + c0 * kCoordsPerThread, lds, lane, acc);
        else store16<false>(out, c * kCoordsPerThread, d, acc);
    }
}

int launch_unpack_dequant_sum(const uint32_t *packed, int64_t ld_words, const float *delta, int64_t d, int64_t M,
                              int b, float scale, float *out, hipStream_t st)
{
    const int64_t row_words = packed_words(d, b);
    const dim3 grid = grid_for(d, 1), block(kThreads);
    switch (b) {
    case 8: unpack_dequant_sum_kernel<8><<<grid, block, 0, st>>>(packed, ld_words, row_words, delta, d, static_cast<int>(M), scale, out); break;
    case 4: unpack_dequant_sum_kernel<4><<<grid, block, 0, st>>>(packed, ld_words, row_words, delta, d, static_cast<int>(M), scale, out); break;
    case 2: unpack_dequant_sum_kernel<2><<<grid, block, 0, st>>>(packed, ld_words, row_words, delta, d, static_cast<int>(M), scale, out); break;
    default:
        if (b < 2 || b > 16) return DQ_ERR_UNSUPPORTED;
        unpack_dequant_sum_any_kernel<<<grid_for_groups(d, 1), block, 0, st>>>(packed, ld_words, row_words, delta, d, static_cast<int>(M), b, scale, out);
        break;
    }
    DQ_LAUNCH_CHECK();
    return DQ_OK;
}

// ---------------------------------------------------------------- dequantize (int8 codes)
__global__ __launch_bounds__(kThreads) void dequantize_kernel(const uint32_t *__restrict__ codes_words, int64_t ld_code_words,
                                                              int64_t row_words, const float *__restrict__ delta,
                                                              int64_t d, float *__restrict__ out, int64_t ld)
{
    const int m = blockIdx.y;
    const float dm = delta[m];
    const int64_t chunks = (d + kCoordsPerThread - 1) / kCoordsPerThread;
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kThreads;
    for (int64_t c = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x; c < chunks; c += stride) {
        uint32_t w[4];
        load_words<8>(codes_words + static_cast<int64_t>(m) * ld_code_words, c, row_words, w);
        float a[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) a[j] = dm * static_cast<float>(code_of<8>(w, j));
        store16(out + static_cast<int64_t>(m) * ld, c * kCoordsPerThread, d, a);
    }
}

// ---------------------------------------------------------------- pack / unpack (int8 <-> FIELD bits)
template <int FIELD>
__global__ __launch_bounds__(kThreads) void pack_kernel(const uint32_t *__restrict__ codes_words, int64_t ld_code_words,
                                                        int64_t code_row_words, int64_t d,
                                                        uint32_t *__restrict__ packed, int64_t ld_words, int64_t row_words)
{
    constexpr int kWords = kCoordsPerThread * FIELD / 32;
    constexpr uint32_t kMask = (1u << FIELD) - 1u;
    const int m = blockIdx.y;
    uint32_t *out = packed + static_cast<int64_t>(m) * ld_words;
    const int64_t chunks = (d + kCoordsPerThread - 1) / kCoordsPerThread;
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kThreads;
    for (int64_t c = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x; c < chunks; c += stride) {
        uint32_t in[4];
        load_words<8>(codes_words + static_cast<int64_t>(m) * ld_code_words, c, code_row_words, in);
        uint32_t w[kWords];
#pragma unroll
        for (int i = 0; i < kWords; ++i) w[i] = 0u;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            int k = code_of<8>(in, j);
            if (c * kCoordsPerThread + j >= d) k = 0;
            w[(j * FIELD) / 32] |= (static_cast<uint32_t>(k) & kMask) << ((j * FIELD) % 32);
        }
        const int64_t w0 = c * kWords;
#pragma unroll
        for (int i = 0; i < kWords; ++i)
            if (w0 + i < row_words) out[w0 + i] = w[i];
    }
}

template <int FIELD>
__global__ __launch_bounds__(kThreads) void unpack_kernel(const uint32_t *__restrict__ packed, int64_t ld_words, int64_t row_words,
                                                          int64_t d, int8_t *__restrict__ codes, int64_t ld_codes)
{
    constexpr int kWords = kCoordsPerThread * FIELD / 32;
    const int m = blockIdx.y;
    int8_t *out = codes + static_cast<int64_t>(m) * ld_codes;
    const int64_t chunks = (d + kCoordsPerThread - 1) / kCoordsPerThread;
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kThreads;
    for (int64_t c = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x; c < chunks; c += stride) {
        uint32_t w[kWords];
        load_words<FIELD>(packed + static_cast<int64_t>(m) * ld_words, c, row_words, w);
        const int64_t base = c * kCoordsPerThread;
        if (base + 16 <= d) {
            uint32_t o[4] = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int j = 0; j < 16; ++j) o[j / 4] |= (static_cast<uint32_t>(code_of<FIELD>(w, j)) & 0xFFu) << ((j % 4) * 8);
            reinterpret_cast<uint4 *>(out + base)[0] = make_uint4(o[0], o[1], o[2], o[3]);
        } else {
#pragma unroll
            for (int j = 0; j < 16; ++j)
                if (base + j < d) out[base + j] = static_cast<int8_t>(code_of<FIELD>(w, j));
        }
    }
}

}  // namespace dq

// =============================================================================== C ABI
using namespace dq;

static inline hipStream_t as_stream(void *s) { return reinterpret_cast<hipStream_t>(s); }

static inline bool rows_ok(const void *p, int64_t M, int64_t ld, int64_t d, int64_t elems_per_16B)
{
    if (!p || !aligned16(p)) return false;
    if (ld < d) return false;
    if (M > 1 && (ld % elems_per_16B) != 0) return false;
    return true;
}

extern "C" int32_t dq_absmax(const float *v, int64_t d, int64_t M, int64_t ld, float *absmax_out, void *stream)
{
    if (d < 0 || M <= 0 || !absmax_out) return DQ_ERR_INVALID_ARG;
    if (d > 0 && !rows_ok(v, M, ld, d, 4)) return DQ_ERR_INVALID_ARG;
    return launch_absmax(v, d, M, ld, absmax_out, as_stream(stream));
}

static int32_t quantize_common(const float *v, int64_t d, int64_t M, int64_t ld, int32_t b, int field,
                               float *absmax, int32_t absmax_given, uint64_t seed, uint32_t iter, uint32_t tag,
                               uint32_t worker0, uint32_t *out_words, int64_t ld_words, float *delta_out,
                               uint32_t *status, void *stream)
{
    if (d < 0 || M <= 0 || !absmax || !delta_out) return DQ_ERR_INVALID_ARG;
    if (b < 2 || b > 16 || b > field) return DQ_ERR_INVALID_ARG;
    const int64_t row_words = packed_words(d, field);
    if (d > 0) {
        if (!rows_ok(v, M, ld, d, 4)) return DQ_ERR_INVALID_ARG;
        if (!rows_ok(out_words, M, ld_words, row_words, 4)) return DQ_ERR_INVALID_ARG;
    }
    hipStream_t st = as_stream(stream);
    if (!absmax_given) {
        int rc = launch_absmax(v, d, M, ld, absmax, st);
        if (rc != DQ_OK) return rc;
    }
    StreamKey key{static_cast<uint32_t>(seed), static_cast<uint32_t>(seed >> 32), iter, 0u, tag};
    // d == 0 still writes delta (= scale of an empty vector, 0): one block per row does that.
    return launch_quantize_pack(v, d, M, ld, b, field, absmax, key, worker0, out_words, ld_words, delta_out,
                                status, st);
}

extern "C" int32_t dq_quantize(const float *v, int64_t d, int64_t M, int64_t ld, int32_t b, float *absmax,
                               int32_t absmax_given, uint64_t seed, uint32_t iter, uint32_t tag, uint32_t worker0,
                               int8_t *codes_out, int64_t ld_codes, float *delta_out, uint32_t *status, void *stream)
{
    if ((ld_codes % 4) != 0 || ld_codes < d) return DQ_ERR_INVALID_ARG;
    // int8 codes are 8-bit fields: the packed layout with FIELD = 8 is exactly an int8 array.
    return quantize_common(v, d, M, ld, b, 8, absmax, absmax_given, seed, iter, tag, worker0,
                           reinterpret_cast<uint32_t *>(codes_out), ld_codes / 4, delta_out, status, stream);
}

extern "C" int32_t dq_quantize_pack(const float *v, int64_t d, int64_t M, int64_t ld, int32_t b, float *absmax,
                                    int32_t absmax_given, uint64_t seed, uint32_t iter, uint32_t tag,
                                    uint32_t worker0, uint32_t *packed_out, int64_t ld_words, float *delta_out,
                                    uint32_t *status, void *stream)
{
    if (b < 2 || b > 16) return DQ_ERR_INVALID_ARG;
    return quantize_common(v, d, M, ld, b, b, absmax, absmax_given, seed, iter, tag, worker0, packed_out, ld_words,
                           delta_out, status, stream);
}

extern "C" int32_t dq_dequantize(const int8_t *codes, int64_t ld_codes, const float *delta, int64_t d, int64_t M,
                                 float *v_out, int64_t ld, void *stream)
{
    if (d < 0 || M <= 0 || !delta) return DQ_ERR_INVALID_ARG;
    if (d == 0) return DQ_OK;
    if ((ld_codes % 4) != 0) return DQ_ERR_INVALID_ARG;
    if (!rows_ok(codes, M, ld_codes, d, 16) || !rows_ok(v_out, M, ld, d, 4)) return DQ_ERR_INVALID_ARG;
    dequantize_kernel<<<grid_for(d, M), dim3(kThreads), 0, as_stream(stream)>>>(
        reinterpret_cast<const uint32_t *>(codes), ld_codes / 4, packed_words(d, 8), delta, d, v_out, ld);
    DQ_LAUNCH_CHECK();
    return DQ_OK;
}

extern "C" int32_t dq_pack(const int8_t *codes, int64_t ld_codes, int64_t d, int64_t M, int32_t b,
                           uint32_t *packed_out, int64_t ld_words, void *stream)
{
    if (d < 0 || M <= 0) return DQ_ERR_INVALID_ARG;
    if (b < 2 || b > 8) return DQ_ERR_INVALID_ARG;
    if (d == 0) return DQ_OK;
    const int64_t row_words = packed_words(d, b);
    if ((ld_codes % 4) != 0) return DQ_ERR_INVALID_ARG;
    if (!rows_ok(codes, M, ld_codes, d, 16) || !rows_ok(packed_out, M, ld_words, row_words, 4)) return DQ_ERR_INVALID_ARG;
    const dim3 grid = grid_for(d, M), block(kThreads);
    const uint32_t *cw = reinterpret_cast<const uint32_t *>(codes);
    const int64_t cld = ld_codes / 4, crw = packed_words(d, 8);
    hipStream_t st = as_stream(stream);
    if (b == 8) pack_kernel<8><<<grid, block, 0, st>>>(cw, cld, crw, d, packed_out, ld_words, row_words);
    else if (b == 4) pack_kernel<4><<<grid, block, 0, st>>>(cw, cld, crw, d, packed_out, ld_words, row_words);
    else if (b == 2) pack_kernel<2><<<grid, block, 0, st>>>(cw, cld, crw, d, packed_out, ld_words, row_words);
    else pack_any_kernel<<<grid_for_groups(d, M), block, 0, st>>>(codes, ld_codes, d, b, packed_out, ld_words, row_words);
    DQ_LAUNCH_CHECK();
    return DQ_OK;
}

extern "C" int32_t dq_unpack(const uint32_t *packed, int64_t ld_words, int64_t d, int64_t M, int32_t b,
                             int8_t *codes_out, int64_t ld_codes, void *stream)
{
    if (d < 0 || M <= 0) return DQ_ERR_INVALID_ARG;
    if (b < 2 || b > 8) return DQ_ERR_INVALID_ARG;
    if (d == 0) return DQ_OK;
    const int64_t row_words = packed_words(d, b);
    if (!rows_ok(packed, M, ld_words, row_words, 4) || !rows_ok(codes_out, M, ld_codes, d, 16)) return DQ_ERR_INVALID_ARG;
    const dim3 grid = grid_for(d, M), block(kThreads);
    hipStream_t st = as_stream(stream);
    if (b == 8) unpack_kernel<8><<<grid, block, 0, st>>>(packed, ld_words, row_words, d, codes_out, ld_codes);
    else if (b == 4) unpack_kernel<4><<<grid, block, 0, st>>>(packed, ld_words, row_words, d, codes_out, ld_codes);
    else if (b == 2) unpack_kernel<2><<<grid, block, 0, st>>>(packed, ld_words, row_words, d, codes_out, ld_codes);
    else unpack_any_kernel<<<grid_for_groups(d, M), block, 0, st>>>(packed, ld_words, row_words, d, b, codes_out, ld_codes);
    DQ_LAUNCH_CHECK();
    return DQ_OK;
}

extern "C" int32_t dq_unpack_dequant_sum(const uint32_t *packed, int64_t ld_words, const float *delta, int64_t d,
                                         int64_t M, int32_t b, float scale, float *out, void *stream)
{
    if (d < 0 || M <= 0 || !delta) return DQ_ERR_INVALID_ARG;
    if (b < 2 || b > 16) return DQ_ERR_INVALID_ARG;
    if (d == 0) return DQ_OK;
    if (!rows_ok(packed, M, ld_words, packed_words(d, b), 4) || !out || !aligned16(out)) return DQ_ERR_INVALID_ARG;
    return launch_unpack_dequant_sum(packed, ld_words, delta, d, M, b, scale, out, as_stream(stream));
}
