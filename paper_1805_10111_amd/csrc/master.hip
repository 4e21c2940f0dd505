// Master side of a round (Alg. 1, master (ii) then (i); Alg. 3 momentum update),
// the epoch-boundary vector operations of Alg. 3, mini-batch index sampling and the
// stand-alone gradient sparsifier of eq. (3).
#include <type_traits>

#include "dq_common.h"
#include "elementwise.h"
#include "grad_launch.h"

namespace dq {

int fill_u32(uint32_t *p, int64_t n, uint32_t value, hipStream_t st);
int launch_quantize_pack(const float *v, int64_t d, int64_t M, int64_t ld, int b, int field, const float *absmax,
                         const StreamKey &key, uint32_t worker0, uint32_t *packed, int64_t ld_words, float *delta_out,
                         uint32_t *status, hipStream_t st);
int launch_model_message(const float *x, int64_t d, int b_x, const float *absmax, const StreamKey &key, uint32_t *packed,
                         float *delta_out, uint32_t *status, const float *x_snap, float *diff_out, hipStream_t st);

constexpr int kThreads = 256;

// ------------------------------------------------------------------ master update
// FIELD in {2,4,8}: packed codes; FIELD == 32: rows of float32 gradients (delta ignored).
struct MasterArgs {
    const uint32_t *packed; int64_t ld_words, row_words;
    const float *delta; int M;
    float scale;              // mean mode: multiplies the sum of the M decoded gradients
    int each;                 // != 0: one update per received gradient, in worker order, scale unused (selects EACH)
    const float *g_snap;
    float *x, *y; const float *x_snap; float *xsum;
    float eta, theta, kappa;
    int64_t d;
};

// Alg. 1, master (ii) (Alg. 3 when ACC) for one direction u on a quad; the state is updated in registers.
template <bool ACC>
__device__ __forceinline__ void master_apply_quad(const float (&u)[4], float (&xn)[4], float (&yn)[4], const float (&xs)[4],
                                                  float (&sm)[4], bool have_sum, float eta, float theta, float kappa)
{
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        if (ACC) {
            yn[e] = soft_threshold(yn[e] - eta * u[e], kappa);      // y <- prox(y - eta u)
            xn[e] = xs[e] + theta * (yn[e] - xs[e]);                // x <- snapshot + theta (y - snapshot)
            if (have_sum) sm[e] = sm[e] + xn[e];
        } else {
            xn[e] = soft_threshold(xn[e] - eta * u[e], kappa);      // x <- prox(x - eta u)
        }
    }
}

// The master update on quad q (coordinates 4q..4q+3): decodes the M messages, updates x (and y, xsum) in
// memory and returns the new x (zeros past the end of the vector).
template <int FIELD, bool ACC, bool EACH>
__device__ __forceinline__ float4 master_quad(const MasterArgs &a, int64_t q)
{
    const int64_t d = a.d;
    float xn[4] = {0.0f, 0.0f, 0.0f, 0.0f}, yn[4] = {0.0f, 0.0f, 0.0f, 0.0f}, xs[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    float sm[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    const bool have_sum = ACC && a.xsum != nullptr;
    // The state vectors of the quad.  With whole quads (d a multiple of 4, the same for every thread) the requests
    // stand side by side in one piece of straight-line code; load_quad's per-lane tests for a ragged end make the
    // compiler wait for each vector before it asks for the next.
    float4 gs4, y4 = make_float4(0.0f, 0.0f, 0.0f, 0.0f), s4 = y4, t4 = y4, x4 = y4;
    if ((d & 3) == 0) {
        gs4 = reinterpret_cast<const float4 *>(a.g_snap)[q];
        if (ACC) {
            y4 = reinterpret_cast<const float4 *>(a.y)[q];
            s4 = reinterpret_cast<const float4 *>(a.x_snap)[q];
            if (have_sum) t4 = reinterpret_cast<const float4 *>(a.xsum)[q];
        } else {
            x4 = reinterpret_cast<const float4 *>(a.x)[q];
        }
    } else {
        gs4 = load_quad(a.g_snap, q, d);
        if (ACC) {
            y4 = load_quad(a.y, q, d);
            s4 = load_quad(a.x_snap, q, d);
            if (have_sum) t4 = load_quad(a.xsum, q, d);
        } else {
            x4 = load_quad(a.x, q, d);
        }
    }
    const float gs[4] = {gs4.x, gs4.y, gs4.z, gs4.w};
    if (ACC) {
        yn[0] = y4.x; yn[1] = y4.y; yn[2] = y4.z; yn[3] = y4.w;
        xs[0] = s4.x; xs[1] = s4.y; xs[2] = s4.z; xs[3] = s4.w;
        sm[0] = t4.x; sm[1] = t4.y; sm[2] = t4.z; sm[3] = t4.w;
    } else {
        xn[0] = x4.x; xn[1] = x4.y; xn[2] = x4.z; xn[3] = x4.w;
    }
    float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};             // mean mode: sum_m delta_m * code_m, messages in order
    // The words of a group of messages are requested together, then decoded and applied in message order; groups
    // of 32, then of 8, then single messages.  The one block of the fused step is bound by the number of
    // instructions it issues, so a group has no per-message test and the message rows are addressed from a
    // uniform base.
    const auto group = [&](int m, auto width) {
        constexpr int G = decltype(width)::value;
        QuadRaw<FIELD> raw[G];
        float dm[G];
#pragma unroll
        for (int u = 0; u < G; ++u) {
            raw[u] = quad_request<FIELD>(a.packed + static_cast<int64_t>(m + u) * a.ld_words, q, d);
            dm[u] = FIELD == 32 ? 1.0f : a.delta[m + u];
        }
#pragma unroll
        for (int u = 0; u < G; ++u) {
            const float4 v = quad_decode<FIELD>(raw[u], q);
            const float vv[4] = {v.x, v.y, v.z, v.w};
            if (EACH) {
                const float dir[4] = {dm[u] * vv[0] + gs[0], dm[u] * vv[1] + gs[1], dm[u] * vv[2] + gs[2],
                                      dm[u] * vv[3] + gs[3]};
                master_apply_quad<ACC>(dir, xn, yn, xs, sm, have_sum, a.eta, a.theta, a.kappa);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[e] = fmaf(dm[u], vv[e], acc[e]);
            }
        }
    };
    int m = 0;
    if constexpr (FIELD != 32 && !EACH)                   // (the per-message update needs the registers itself)
        for (; m + 32 <= a.M; m += 32) group(m, std::integral_constant<int, 32>{});
    for (; m + 8 <= a.M; m += 8) group(m, std::integral_constant<int, 8>{});
    for (; m < a.M; ++m) group(m, std::integral_constant<int, 1>{});
    if (!EACH) {
        const float dir[4] = {a.scale * acc[0] + gs[0], a.scale * acc[1] + gs[1], a.scale * acc[2] + gs[2],
                              a.scale * acc[3] + gs[3]};     // u = mean of the decoded gradients + grad f(snapshot)
        master_apply_quad<ACC>(dir, xn, yn, xs, sm, have_sum, a.eta, a.theta, a.kappa);
    }
#pragma unroll
    for (int e = 0; e < 4; ++e)
        if (4 * q + e >= d) xn[e] = 0.0f;
    const float4 xq4 = make_float4(xn[0], xn[1], xn[2], xn[3]);
    store_quad(a.x, q, d, xq4);
    if (ACC) {
        store_quad(a.y, q, d, make_float4(yn[0], yn[1], yn[2], yn[3]));
        if (have_sum) store_quad(a.xsum, q, d, make_float4(sm[0], sm[1], sm[2], sm[3]));
    }
    return xq4;
}

__device__ __forceinline__ uint32_t quad_abs_bits(float4 v)
{
    return max(max(abs_bits(v.x), abs_bits(v.y)), max(abs_bits(v.z), abs_bits(v.w)));
}

// Any model size: grid-stride over quads; ||x||_inf through one atomic max per block on the
// magnitude bit pattern (absmax_bits must be zero on entry).
template <int FIELD, bool ACC, bool EACH, int TB = kThreads>
__global__ __launch_bounds__(TB) void master_update_kernel(const MasterArgs a, uint32_t *__restrict__ absmax_bits)
{
    touch_kernel_arguments<sizeof(MasterArgs) + sizeof(uint32_t *)>();
    __shared__ uint32_t scratch[TB / kWave];
    const int64_t quads = (a.d + 3) / 4;
    const int64_t stride = static_cast<int64_t>(gridDim.x) * TB;
    uint32_t amax = 0;
    for (int64_t q = static_cast<int64_t>(blockIdx.x) * TB + threadIdx.x; q < quads; q += stride)
        amax = max(amax, quad_abs_bits(master_quad<FIELD, ACC, EACH>(a, q)));
    amax = block_max_u32(amax, scratch);
    if (threadIdx.x == 0 && amax != 0) atomicMax(absmax_bits, amax);
}

template <int FIELD, int TB = kThreads>
static int launch_master_update(bool acc, dim3 grid, hipStream_t st, const MasterArgs &a, uint32_t *absmax_bits)
{
    const dim3 block(TB);
    if (acc && a.each) master_update_kernel<FIELD, true, true, TB><<<grid, block, 0, st>>>(a, absmax_bits);
    else if (acc) master_update_kernel<FIELD, true, false, TB><<<grid, block, 0, st>>>(a, absmax_bits);
    else if (a.each) master_update_kernel<FIELD, false, true, TB><<<grid, block, 0, st>>>(a, absmax_bits);
    else master_update_kernel<FIELD, false, false, TB><<<grid, block, 0, st>>>(a, absmax_bits);
    DQ_LAUNCH_CHECK();
    return DQ_OK;
}

// ------------------------------------------------------------------ Alg. 2: quantization inside the master update
// The workers of a round left their sparsified gradients beta_m unquantized (SparsifiedParts).  A block of 16 x 64
// threads takes 64 quads of the model: thread (worker lane, quad lane) quantizes its worker's quad -- scale
// ||beta_m||_inf from the slice maxima, the worker's own Philox stream -- stores the message bits and leaves the four
// codes in LDS; after the barrier the threads of worker lane 0 (one wavefront) aggregate delta_m * code_m in worker
// order and update the model exactly as master_quad does.  More than 16 workers take several passes over two LDS
// buffers.  (64 quads per block: a block then writes whole 128-byte lines of every message row, and 82 blocks cover
// 20958 coordinates.  With 16 quads per block -- 328 blocks, a quarter line per row and block -- two or three blocks
// of every launch waited 1 to 4 us for the acknowledgement of such a store before they could end: 6.9 us per launch
// under the profiler against 4.6.)
constexpr int kPartsWorkers = 16, kPartsQuads = 64;

struct PartsArgs {
    SparsifiedParts in;
    int b; StreamKey key; uint32_t worker0;
    uint32_t *packed;                                    // rows of MasterArgs::ld_words words
    float *delta_out; int32_t *nnz_out; uint32_t *status;
};

template <int FIELD, bool EACH>
__global__ __launch_bounds__(kPartsWorkers * kPartsQuads) void master_from_parts_kernel(const MasterArgs a, const PartsArgs p,
                                                                                       uint32_t *__restrict__ absmax_bits)
{
    touch_kernel_arguments<sizeof(MasterArgs) + sizeof(PartsArgs) + sizeof(uint32_t *)>();
    __shared__ float4 codes[2][kPartsWorkers][kPartsQuads];
    __shared__ float deltas[2][kPartsWorkers];
    const int ql = threadIdx.x % kPartsQuads, wl = threadIdx.x / kPartsQuads;
    const int64_t d = a.d, quads = (d + 3) / 4;
    if (blockIdx.x == gridDim.x - 1) {
        // one block more than the quads need: what a worker step reports per message (scale, status, nonzeros =
        // coordinates its sparsifier kept), off the path of the blocks that do the arithmetic
        for (int m = threadIdx.x; m < a.M; m += kPartsWorkers * kPartsQuads) {
            const Scale s = make_scale(parts_absmax(p.in.part_max + static_cast<int64_t>(m) * p.in.parts, p.in.parts), p.b);
            p.delta_out[m] = s.delta;
            if (s.bad && p.status) atomicOr(p.status, 1u);
            if (p.nnz_out) p.nnz_out[m] = parts_sum(p.in.part_kept + static_cast<int64_t>(m) * p.in.parts, p.in.parts);
        }
        return;
    }
    const int64_t q = static_cast<int64_t>(blockIdx.x) * kPartsQuads + ql;
    const bool inside = q < quads;
    constexpr int kB = CodeBias<FIELD>::value;
    float gs[4] = {0.0f, 0.0f, 0.0f, 0.0f}, xn[4] = {0.0f, 0.0f, 0.0f, 0.0f}, acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    float unused_y[4] = {0.0f, 0.0f, 0.0f, 0.0f}, unused_s[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    const float unused_xs[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    if (wl == 0 && inside) {
        // requested here, looked at only after the first barrier: whole quads, or single elements at clamped
        // positions where the vector ends inside the quad (what was read past d is discarded there)
        const int64_t i = 4 * q, last = d - 1;
        if ((d & 3) == 0) {
            const float4 g4 = reinterpret_cast<const float4 *>(a.g_snap)[q], x4 = reinterpret_cast<const float4 *>(a.x)[q];
            gs[0] = g4.x; gs[1] = g4.y; gs[2] = g4.z; gs[3] = g4.w;
            xn[0] = x4.x; xn[1] = x4.y; xn[2] = x4.z; xn[3] = x4.w;
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                gs[e] = a.g_snap[min(i + e, last)];
                xn[e] = a.x[min(i + e, last)];
            }
        }
    }
    for (int m0 = 0; m0 < a.M; m0 += kPartsWorkers) {
        const int buf = (m0 / kPartsWorkers) & 1;
        const int m = m0 + wl;
        const bool live = m < a.M;
        float4 c = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        uint32_t bits = 0;
        if (live) {
            // everything is requested before anything is waited for: slice maxima and the quad; the random bits do
            // not depend on either
            const PartsRaw maxima = parts_request(p.in.part_max + static_cast<int64_t>(m) * p.in.parts, p.in.parts);
            // (rows are padded to whole quads; what lies past d is not part of the vector)
            float4 v = reinterpret_cast<const float4 *>(p.in.beta + static_cast<int64_t>(m) * p.in.ld)[inside ? q : 0];
            __builtin_amdgcn_sched_barrier(0);           // (the requests go out, then the Philox rounds, then the waits)
            StreamKey key = p.key;
            key.worker = p.worker0 + static_cast<uint32_t>(m);
            const uint4 r = stream_block(key, static_cast<uint32_t>(q));
            asm volatile("" ::"v"(r.x), "v"(r.y), "v"(r.z), "v"(r.w));      // (... here, not where r is first used)
            __builtin_amdgcn_sched_barrier(0);
            const float amax = parts_absmax_of(maxima);
            v.y = 4 * q + 1 < d ? v.y : 0.0f;
            v.z = 4 * q + 2 < d ? v.z : 0.0f;
            v.w = 4 * q + 3 < d ? v.w : 0.0f;
            const Scale s = make_scale(amax, p.b);
            if (ql == 0) deltas[buf][wl] = s.delta;
            if (inside && s.inv_delta != 0.0f) {         // (a degenerate scale: every code is zero)
                const int k0 = quantize_one<kB>(v.x, s, r.x), k1 = quantize_one<kB>(v.y, s, r.y);
                const int k2 = quantize_one<kB>(v.z, s, r.z), k3 = quantize_one<kB>(v.w, s, r.w);
                bits = pack4<FIELD, true, FIELD != 8>(k0, k1, k2, k3);
                c = make_float4(static_cast<float>(k0 - kB), static_cast<float>(k1 - kB), static_cast<float>(k2 - kB),
                                static_cast<float>(k3 - kB));
            }
        }
        // (every lane makes the call; the lanes that share a word belong to one worker and to neighbouring quads)
        store_quad_bits<FIELD>(bits, live ? q : quads, quads, p.packed + static_cast<int64_t>(live ? m : 0) * a.ld_words);
        codes[buf][wl][ql] = c;
        __syncthreads();
        if (wl == 0 && inside) {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (4 * q + e >= d) gs[e] = xn[e] = 0.0f;
            const auto apply = [&](int u) {
                const float4 v = codes[buf][u][ql];
                const float dm = deltas[buf][u];
                const float vv[4] = {v.x, v.y, v.z, v.w};
                if (EACH) {
                    const float dir[4] = {dm * vv[0] + gs[0], dm * vv[1] + gs[1], dm * vv[2] + gs[2], dm * vv[3] + gs[3]};
                    master_apply_quad<false>(dir, xn, unused_y, unused_xs, unused_s, false, a.eta, a.theta, a.kappa);
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[e] = fmaf(dm, vv[e], acc[e]);
                }
            };
            const int count = min(kPartsWorkers, a.M - m0);
            if (count == kPartsWorkers) {                // a full pass: all LDS reads go out together
#pragma unroll
                for (int u = 0; u < kPartsWorkers; ++u) apply(u);
            } else {
                for (int u = 0; u < count; ++u) apply(u);
            }
        }
    }
    uint32_t amax = 0;
    if (wl == 0 && inside) {
        if (!EACH) {
            const float dir[4] = {a.scale * acc[0] + gs[0], a.scale * acc[1] + gs[1], a.scale * acc[2] + gs[2],
                                  a.scale * acc[3] + gs[3]};
            master_apply_quad<false>(dir, xn, unused_y, unused_xs, unused_s, false, a.eta, a.theta, a.kappa);
        }
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (4 * q + e >= d) xn[e] = 0.0f;
        const float4 x4 = make_float4(xn[0], xn[1], xn[2], xn[3]);
        store_quad(a.x, q, d, x4);
        amax = quad_abs_bits(x4);
    }
    if (threadIdx.x < kWave) {                           // (worker lane 0 lies in the first wavefront)
        amax = wave_max_u32(amax);
        if (threadIdx.x == 0 && amax != 0) atomicMax(absmax_bits, amax);
    }
}

// ------------------------------------------------------------------ fused master step, one block
// For d <= kFusedMaxD the whole master step is one block of 1024 threads: thread t owns the quads
// (four consecutive coordinates) t and t+1024 of the model, keeps their updated values in
// registers across the block-wide ||x||_inf reduction and quantizes + packs them right away
// (Alg. 1, master (ii) then (i)).  Consecutive lanes work on consecutive quads, so message words
// and model vectors are read in whole cache lines and all threads are busy from d = 4096 up.
// Beyond that size one compute unit doing all the Philox blocks is slower than three small
// launches spread over the chip (measured at d = 20958: 12.8 us against about 8 us).
constexpr int kFusedThreads = 1024;
constexpr int64_t kFusedMaxD = 8192;

template <int FIELD, bool ACC, bool EACH, int NQ>
__global__ __launch_bounds__(kFusedThreads) void master_fused_kernel(
    const MasterArgs a, int b_x, StreamKey key, uint32_t *__restrict__ xq_out, float *__restrict__ delta_x_out,
    float *__restrict__ absmax_x_out, uint32_t *__restrict__ status)
{
    touch_kernel_arguments<sizeof(MasterArgs) + 64>();
    __shared__ uint32_t scratch[kFusedThreads / kWave];
    const int64_t d = a.d, quads = (d + 3) / 4;
    float4 xv[NQ];                                       // the thread's quads threadIdx.x + 1024*k of the new model
    uint32_t amax = 0;
#pragma unroll
    for (int k = 0; k < NQ; ++k) {
        const int64_t q = threadIdx.x + static_cast<int64_t>(kFusedThreads) * k;
        xv[k] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        if (q >= quads) continue;
        xv[k] = master_quad<FIELD, ACC, EACH>(a, q);
        amax = max(amax, quad_abs_bits(xv[k]));
    }
    amax = block_max_u32(amax, scratch);
    if (threadIdx.x == 0) absmax_x_out[0] = __uint_as_float(amax);
    if (b_x == 32) {
        if (threadIdx.x == 0) delta_x_out[0] = 1.0f;
#pragma unroll
        for (int k = 0; k < NQ; ++k) {
            const int64_t q = threadIdx.x + static_cast<int64_t>(kFusedThreads) * k;
            if (q < quads) store_quad(reinterpret_cast<float *>(xq_out), q, d, xv[k]);
        }
        return;
    }
    // Alg. 1, master (i) for the next round: quantize the new model
    const Scale s = make_scale(__uint_as_float(amax), b_x);
    if (threadIdx.x == 0) {
        delta_x_out[0] = s.delta;
        if (s.bad && status) atomicOr(status, 1u);
    }
    key.worker = DQ_MASTER_ID;
    int nz = 0;
#pragma unroll
    for (int k = 0; k < NQ; ++k) {                       // all lanes make every store call (cross-lane moves inside)
        const int64_t q = threadIdx.x + static_cast<int64_t>(kFusedThreads) * k;
        const bool in = q < quads;
        if (b_x == 8) store_quad_bits<8>(in ? quantize_quad<8>(xv[k], s, key, q, nz) : 0u, q, quads, xq_out);
        else if (b_x == 4) store_quad_bits<4>(in ? quantize_quad<4>(xv[k], s, key, q, nz) : 0u, q, quads, xq_out);
        else store_quad_bits<2>(in ? quantize_quad<2>(xv[k], s, key, q, nz) : 0u, q, quads, xq_out);
    }
}

template <int FIELD, bool ACC, bool EACH>
static void launch_master_fused2(int ch, hipStream_t st, const MasterArgs &a, int b_x, const StreamKey &key,
                                 uint32_t *xq_out, float *delta_x_out, float *absmax_x_out, uint32_t *status)
{
    const dim3 grid(1), block(kFusedThreads);
#define DQ_FUSED(NQ) master_fused_kernel<FIELD, ACC, EACH, NQ><<<grid, block, 0, st>>>(a, b_x, key, xq_out, delta_x_out, absmax_x_out, status)
    if (ch == 1) DQ_FUSED(1);                           // quads per thread that cover d
    else DQ_FUSED(2);
#undef DQ_FUSED
}

template <int FIELD>
static int launch_master_fused(bool acc, int ch, hipStream_t st, const MasterArgs &a, int b_x, const StreamKey &key,
                               uint32_t *xq_out, float *delta_x_out, float *absmax_x_out, uint32_t *status)
{
    if (acc && a.each) launch_master_fused2<FIELD, true, true>(ch, st, a, b_x, key, xq_out, delta_x_out, absmax_x_out, status);
    else if (acc) launch_master_fused2<FIELD, true, false>(ch, st, a, b_x, key, xq_out, delta_x_out, absmax_x_out, status);
    else if (a.each) launch_master_fused2<FIELD, false, true>(ch, st, a, b_x, key, xq_out, delta_x_out, absmax_x_out, status);
    else launch_master_fused2<FIELD, false, false>(ch, st, a, b_x, key, xq_out, delta_x_out, absmax_x_out, status);
    DQ_LAUNCH_CHECK();
    return DQ_OK;
}

__global__ __launch_bounds__(kThreads) void copy_f32_kernel(const float *__restrict__ a, float *__restrict__ b, int64_t n)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
    if (i < n) b[i] = a[i];
}

// ------------------------------------------------------------------ Alg. 3 epoch boundary
__global__ __launch_bounds__(kThreads) void acc_mix_kernel(const float *__restrict__ y, const float *__restrict__ xs, float theta,
                                                           int64_t d, float *__restrict__ x)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
    if (i < d) x[i] = xs[i] + theta * (y[i] - xs[i]);
}

__global__ __launch_bounds__(kThreads) void acc_snapshot_kernel(const float *__restrict__ xsum, float m, int64_t d,
                                                                float *__restrict__ xs)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
    if (i < d) xs[i] = xsum[i] / m;
}

// ------------------------------------------------------------------ sampling
__global__ __launch_bounds__(kThreads) void sample_indices_kernel(uint32_t n, int64_t B, StreamKey key, uint32_t worker0,
                                                                  int32_t *__restrict__ idx)
{
    const int64_t j = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
    if (j >= B) return;
    key.worker = worker0 + blockIdx.y;
    const uint32_t w = stream_word(key, static_cast<uint64_t>(j));
    idx[static_cast<int64_t>(blockIdx.y) * B + j] = static_cast<int32_t>(__umulhi(w, n));
}

// ------------------------------------------------------------------ sparsifier, one block per row
constexpr int kSparsifyThreads = 1024;

__global__ __launch_bounds__(kSparsifyThreads) void sparsify_kernel(
    const float *__restrict__ alpha, int64_t d, int64_t ld, const float *__restrict__ phi, StreamKey key, uint32_t worker0,
    float *__restrict__ beta, int64_t ld_out, float *__restrict__ absmax_out, int32_t *__restrict__ nnz_out)
{
    __shared__ uint32_t su[kSparsifyThreads / kWave];
    __shared__ double sd[kSparsifyThreads / kWave];
    __shared__ int si[kSparsifyThreads / kWave];
    const int m = blockIdx.x;
    const float *row = alpha + static_cast<int64_t>(m) * ld;
    float *out = beta + static_cast<int64_t>(m) * ld_out;
    key.worker = worker0 + static_cast<uint32_t>(m);
    key.tag = DQ_TAG_SPARSIFY;
    // pass 1: ||alpha||_inf and, for a caller-supplied budget, ||alpha||_1 (double, fixed order)
    uint32_t mb = 0;
    double s1 = 0.0;
    for (int64_t i = threadIdx.x; i < d; i += kSparsifyThreads) {
        const float a = row[i];
        mb = max(mb, abs_bits(a));
        s1 += static_cast<double>(fabsf(a));
    }
    mb = block_max_u32(mb, su);
    SparsifyRule rule;
    rule.amax = __uint_as_float(mb);
    rule.use_budget = phi != nullptr;
    rule.c = 0.0f;
    if (rule.use_budget) {
        const double total = block_sum_f64(s1, sd);
        rule.c = phi[m] / static_cast<float>(total);
    }
    // pass 2: Bernoulli keep, rescale
    uint32_t bmax = 0;
    int kept = 0;
    for (int64_t i = threadIdx.x; i < d; i += kSparsifyThreads) {
        const float b = sparsify_one(row[i], rule, stream_word(key, static_cast<uint64_t>(i)));
        out[i] = b;
        bmax = max(bmax, abs_bits(b));
        kept += b != 0.0f ? 1 : 0;
    }
    bmax = block_max_u32(bmax, su);
    kept = block_sum_i32(kept, si);
    if (threadIdx.x == 0) {
        absmax_out[m] = __uint_as_float(bmax);
        nnz_out[m] = kept;
    }
}

// ------------------------------------------------------------------ condition (2) / (4) of the paper
// out[0] = E_Q ||Q_(delta,b)(x) - x||^2 = delta^2 sum_i p_i (1 - p_i)   (p_i as the quantizer forms it)
// out[1] = ||x - x_snap||^2.   One block; double accumulation in a fixed order.
__global__ __launch_bounds__(kSparsifyThreads) void mu_terms_kernel(const float *__restrict__ x, const float *__restrict__ xs,
                                                                    int64_t d, int b, double *__restrict__ out)
{
    __shared__ uint32_t su[kSparsifyThreads / kWave];
    __shared__ double sd[kSparsifyThreads / kWave];
    uint32_t mb = 0;
    for (int64_t i = threadIdx.x; i < d; i += kSparsifyThreads) mb = max(mb, abs_bits(x[i]));
    mb = block_max_u32(mb, su);
    const Scale s = make_scale(__uint_as_float(mb), b);
    double e = 0.0, r = 0.0;
    for (int64_t i = threadIdx.x; i < d; i += kSparsifyThreads) {
        const float xi = x[i];
        if (s.inv_delta == 0.0f) {
            e += static_cast<double>(xi) * static_cast<double>(xi);          // every code is zero
        } else {
            const float t = xi * s.inv_delta;
            const float p = t - floorf(t);
            e += static_cast<double>(p) * (1.0 - static_cast<double>(p));
        }
        const double dxs = static_cast<double>(xi) - static_cast<double>(xs[i]);
        r += dxs * dxs;
    }
    e = block_sum_f64(e, sd);
    r = block_sum_f64(r, sd);
    if (threadIdx.x == 0) {
        out[0] = s.inv_delta == 0.0f ? e : static_cast<double>(s.delta) * static_cast<double>(s.delta) * e;
        out[1] = r;
    }
}

}  // namespace dq

using namespace dq;
static inline hipStream_t as_stream(void *s) { return reinterpret_cast<hipStream_t>(s); }

extern "C" int32_t dq_mu_terms(const float *x, const float *x_snap, int64_t d, int32_t b, double *out, void *stream)
{
    if (d <= 0 || !x || !x_snap || !out) return DQ_ERR_INVALID_ARG;
    if (b < 2 || b > 16) return DQ_ERR_INVALID_ARG;
    mu_terms_kernel<<<dim3(1), dim3(kSparsifyThreads), 0, as_stream(stream)>>>(x, x_snap, d, b, out);
    DQ_LAUNCH_CHECK();
    return DQ_OK;
}

static int32_t check_master_args(const uint32_t *packed, int64_t ld_words, const float *delta, int64_t M, int32_t b,
                                 const float *g_snap, const float *x, const float *y, const float *x_snap,
                                 const float *xsum, int64_t d)
{
    if (d <= 0 || M <= 0 || M > 0x7FFFFFFFll || !packed || !g_snap || !x) return DQ_ERR_INVALID_ARG;
    if (b != 32 && !delta) return DQ_ERR_INVALID_ARG;
    if (y && !x_snap) return DQ_ERR_INVALID_ARG;
    if (b != 2 && b != 4 && b != 8 && b != 32) return (b >= 2 && b <= 8) ? DQ_ERR_UNSUPPORTED : DQ_ERR_INVALID_ARG;
    const int64_t row_words = b == 32 ? d : packed_words(d, b);
    if (ld_words < row_words || (M > 1 && ld_words % 4 != 0)) return DQ_ERR_INVALID_ARG;
    const void *ptrs[] = {packed, g_snap, x, y, x_snap, xsum};
    for (const void *p : ptrs)
        if (p && !aligned16(p)) return DQ_ERR_INVALID_ARG;
    return DQ_OK;
}

// Alg. 1, master (i) once ||x||_inf is known: the message (and its scale) of the updated model.
// diff_out (nullable, with x_snap; message widths 2, 4, 8): also receives Q(x) - x_snap, see master_leaves_model_diff.
static int model_message(const float *x, int64_t d, int32_t b_x, const StreamKey &key, uint32_t *xq_packed_out,
                         float *delta_x_out, const float *absmax_x, uint32_t *status, hipStream_t st,
                         const float *x_snap = nullptr, float *diff_out = nullptr)
{
    // (below a million coordinates the launch is latency, not throughput: see model_message_kernel)
    constexpr int64_t kSmallModel = 1 << 20;
    const bool leave_diff = diff_out && x_snap;
    if ((b_x == 2 || b_x == 4 || b_x == 8) && (leave_diff || d <= kSmallModel))
        return launch_model_message(x, d, b_x, absmax_x, key, xq_packed_out, delta_x_out, status,
                                    leave_diff ? x_snap : nullptr, leave_diff ? diff_out : nullptr, st);
    if (b_x == 32) {
        // full-precision model: "packed" output is x itself, delta is 1
        copy_f32_kernel<<<dim3(static_cast<unsigned>(ceil_div(d, kThreads))), dim3(kThreads), 0, st>>>(
            x, reinterpret_cast<float *>(xq_packed_out), d);
        DQ_LAUNCH_CHECK();
        return fill_u32(reinterpret_cast<uint32_t *>(delta_x_out), 1, 0x3F800000u, st);
    }
    return launch_quantize_pack(x, d, 1, d, b_x, b_x, absmax_x, key, DQ_MASTER_ID, xq_packed_out,
                                packed_words(d, b_x), delta_x_out, status, st);
}

// One wavefront per block: at d = 4096 the 1024 quads of the model are 16 blocks on 16 compute units.
constexpr int kRoundThreads = 64;

int32_t dq::master_update_impl(const uint32_t *packed, int64_t ld_words, const float *delta, int64_t M, int32_t b,
                               float scale, int each, const float *g_snap, float *x, float *y, const float *x_snap,
                               float *xsum, float eta, float theta, float l1, int64_t d, uint32_t *absmax_bits,
                               void *stream)
{
    const int32_t rc = check_master_args(packed, ld_words, delta, M, b, g_snap, x, y, x_snap, xsum, d);
    if (rc != DQ_OK) return rc;
    if (!absmax_bits) return DQ_ERR_INVALID_ARG;
    const int64_t row_words = b == 32 ? d : packed_words(d, b);
    const MasterArgs a{packed, ld_words, row_words, delta, static_cast<int>(M), scale, each, g_snap,
                       x, y, x_snap, xsum, eta, theta, eta * l1, d};
    const bool acc = y != nullptr;
    int64_t blocks = ceil_div(ceil_div(d, 4), kRoundThreads);
    if (blocks > 4096) blocks = 4096;                                  // grid-stride beyond
    const dim3 grid(static_cast<unsigned>(blocks));
    hipStream_t st = as_stream(stream);
    switch (b) {
    case 8: return launch_master_update<8, kRoundThreads>(acc, grid, st, a, absmax_bits);
    case 4: return launch_master_update<4, kRoundThreads>(acc, grid, st, a, absmax_bits);
    case 2: return launch_master_update<2, kRoundThreads>(acc, grid, st, a, absmax_bits);
    default: return launch_master_update<32, kRoundThreads>(acc, grid, st, a, absmax_bits);
    }
}

int32_t dq::master_step_impl(const uint32_t *packed, int64_t ld_words, const float *delta, int64_t M, int32_t b,
                             float scale, int each, const float *g_snap, float *x, float *y, const float *x_snap,
                             float *xsum, float eta, float theta, float l1, int64_t d, int32_t b_x, uint64_t seed,
                             uint32_t iter, uint32_t *xq_packed_out, float *delta_x_out, float *absmax_x_out,
                             uint32_t *status, bool absmax_zeroed, void *stream, float *model_diff_out)
{
    int32_t rc0 = check_master_args(packed, ld_words, delta, M, b, g_snap, x, y, x_snap, xsum, d);
    if (rc0 != DQ_OK) return rc0;
    if (!xq_packed_out || !delta_x_out || !absmax_x_out || !aligned16(xq_packed_out)) return DQ_ERR_INVALID_ARG;
    if (b_x < 2 || (b_x > 16 && b_x != 32)) return DQ_ERR_INVALID_ARG;
    const int64_t row_words = b == 32 ? d : packed_words(d, b);
    hipStream_t st = as_stream(stream);
    const MasterArgs a{packed, ld_words, row_words, delta, static_cast<int>(M), scale, each, g_snap,
                       x, y, x_snap, xsum, eta, theta, eta * l1, d};
    const StreamKey key{static_cast<uint32_t>(seed), static_cast<uint32_t>(seed >> 32), iter, 0u, DQ_TAG_MODEL};
    const bool acc = y != nullptr;
    const bool word_aligned_bx = b_x == 2 || b_x == 4 || b_x == 8 || b_x == 32;
    if (d <= kFusedMaxD && word_aligned_bx) {
        // small model: the whole step in one block, one launch
        const int ch = static_cast<int>(ceil_div(ceil_div(d, 4), kFusedThreads));     // 1 or 2
        switch (b) {
        case 8: return launch_master_fused<8>(acc, ch, st, a, b_x, key, xq_packed_out, delta_x_out, absmax_x_out, status);
        case 4: return launch_master_fused<4>(acc, ch, st, a, b_x, key, xq_packed_out, delta_x_out, absmax_x_out, status);
        case 2: return launch_master_fused<2>(acc, ch, st, a, b_x, key, xq_packed_out, delta_x_out, absmax_x_out, status);
        default: return launch_master_fused<32>(acc, ch, st, a, b_x, key, xq_packed_out, delta_x_out, absmax_x_out, status);
        }
    }
    uint32_t *absmax_bits = reinterpret_cast<uint32_t *>(absmax_x_out);
    int rc = absmax_zeroed ? DQ_OK : fill_u32(absmax_bits, 1, 0u, st);
    if (rc != DQ_OK) return rc;
    const dim3 grid(static_cast<unsigned>(ceil_div(ceil_div(d, 4), kThreads)));
    switch (b) {
    case 8: rc = launch_master_update<8>(acc, grid, st, a, absmax_bits); break;
    case 4: rc = launch_master_update<4>(acc, grid, st, a, absmax_bits); break;
    case 2: rc = launch_master_update<2>(acc, grid, st, a, absmax_bits); break;
    default: rc = launch_master_update<32>(acc, grid, st, a, absmax_bits); break;
    }
    if (rc != DQ_OK) return rc;
    return model_message(x, d, b_x, key, xq_packed_out, delta_x_out, absmax_x_out, status, st, x_snap, model_diff_out);
}

bool dq::master_leaves_model_diff(int64_t d, int32_t b_x, bool from_parts)
{
    return (b_x == 2 || b_x == 4 || b_x == 8) && (from_parts || d > kFusedMaxD);
}

int32_t dq::master_step_from_parts_impl(const SparsifiedParts &parts, uint32_t worker0, uint32_t worker_iter, uint32_t *packed, int64_t ld_words,
                                        float *delta_out, int32_t *nnz_out, int64_t M, int32_t b, float scale, int each,
                                        const float *g_snap, float *x, float eta, float l1, int64_t d, int32_t b_x,
                                        uint64_t seed, uint32_t iter, uint32_t *xq_packed_out, float *delta_x_out,
                                        float *absmax_x_out, uint32_t *status, bool absmax_zeroed, void *stream,
                                        const float *x_snap, float *model_diff_out)
{
    int32_t rc0 = check_master_args(packed, ld_words, delta_out, M, b, g_snap, x, nullptr, nullptr, nullptr, d);
    if (rc0 != DQ_OK) return rc0;
    if (b == 32 || !parts.beta || !parts.part_max || !parts.part_kept || parts.parts <= 0 || parts.parts > kMaxParts || parts.ld < (d + 3) / 4 * 4 ||
        parts.ld % 4 != 0 || !aligned16(parts.beta))
        return DQ_ERR_INVALID_ARG;
    if (!xq_packed_out || !delta_x_out || !absmax_x_out || !aligned16(xq_packed_out)) return DQ_ERR_INVALID_ARG;
    if (b_x < 2 || (b_x > 16 && b_x != 32)) return DQ_ERR_INVALID_ARG;
    hipStream_t st = as_stream(stream);
    const MasterArgs a{packed, ld_words, packed_words(d, b), delta_out, static_cast<int>(M), scale, each, g_snap,
                       x, nullptr, nullptr, nullptr, eta, 0.0f, eta * l1, d};
    const StreamKey wkey{static_cast<uint32_t>(seed), static_cast<uint32_t>(seed >> 32), worker_iter, 0u, DQ_TAG_GRAD};
    const PartsArgs p{parts, b, wkey, worker0, packed, delta_out, nnz_out, status};
    uint32_t *absmax_bits = reinterpret_cast<uint32_t *>(absmax_x_out);
    int rc = absmax_zeroed ? DQ_OK : fill_u32(absmax_bits, 1, 0u, st);
    if (rc != DQ_OK) return rc;
    const dim3 grid(static_cast<unsigned>(ceil_div(ceil_div(d, 4), kPartsQuads)) + 1u), block(kPartsWorkers * kPartsQuads);
#define DQ_PARTS(FIELD)                                                                        \
    if (each) master_from_parts_kernel<FIELD, true><<<grid, block, 0, st>>>(a, p, absmax_bits); \
    else master_from_parts_kernel<FIELD, false><<<grid, block, 0, st>>>(a, p, absmax_bits)
    switch (b) {
    case 8: DQ_PARTS(8); break;
    case 4: DQ_PARTS(4); break;
    default: DQ_PARTS(2); break;
    }
#undef DQ_PARTS
    DQ_LAUNCH_CHECK();
    const StreamKey key{static_cast<uint32_t>(seed), static_cast<uint32_t>(seed >> 32), iter, 0u, DQ_TAG_MODEL};
    return model_message(x, d, b_x, key, xq_packed_out, delta_x_out, absmax_x_out, status, st, x_snap, model_diff_out);
}

extern "C" int32_t dq_master_step(const uint32_t *packed, int64_t ld_words, const float *delta, int64_t M, int32_t b,
                                  float scale, const float *g_snap, float *x, float *y, const float *x_snap, float *xsum,
                                  float eta, float theta, float l1, int64_t d, int32_t b_x, uint64_t seed, uint32_t iter,
                                  uint32_t *xq_packed_out, float *delta_x_out, float *absmax_x_out, uint32_t *status,
                                  void *stream)
{
    return master_step_impl(packed, ld_words, delta, M, b, scale, 0, g_snap, x, y, x_snap, xsum, eta, theta, l1, d, b_x,
                            seed, iter, xq_packed_out, delta_x_out, absmax_x_out, status, false, stream, nullptr);
}

extern "C" int32_t dq_master_step_each(const uint32_t *packed, int64_t ld_words, const float *delta, int64_t M, int32_t b,
                                       const float *g_snap, float *x, float *y, const float *x_snap, float *xsum,
                                       float eta, float theta, float l1, int64_t d, int32_t b_x, uint64_t seed,
                                       uint32_t iter, uint32_t *xq_packed_out, float *delta_x_out, float *absmax_x_out,
                                       uint32_t *status, void *stream)
{
    return master_step_impl(packed, ld_words, delta, M, b, 1.0f, 1, g_snap, x, y, x_snap, xsum, eta, theta, l1, d, b_x,
                            seed, iter, xq_packed_out, delta_x_out, absmax_x_out, status, false, stream, nullptr);
}

extern "C" int32_t dq_acc_mix(const float *y, const float *x_snap, float theta, int64_t d, float *x_out, void *stream)
{
    if (d <= 0 || !y || !x_snap || !x_out) return DQ_ERR_INVALID_ARG;
    acc_mix_kernel<<<dim3(static_cast<unsigned>(ceil_div(d, kThreads))), dim3(kThreads), 0, as_stream(stream)>>>(y, x_snap, theta, d, x_out);
    DQ_LAUNCH_CHECK();
    return DQ_OK;
}

extern "C" int32_t dq_acc_snapshot(const float *xsum, int64_t m, int64_t d, float *x_snap_out, void *stream)
{
    if (d <= 0 || m <= 0 || !xsum || !x_snap_out) return DQ_ERR_INVALID_ARG;
    acc_snapshot_kernel<<<dim3(static_cast<unsigned>(ceil_div(d, kThreads))), dim3(kThreads), 0, as_stream(stream)>>>(
        xsum, static_cast<float>(m), d, x_snap_out);
    DQ_LAUNCH_CHECK();
    return DQ_OK;
}

extern "C" int32_t dq_sample_indices(int64_t n, int64_t M, int64_t B, uint64_t seed, uint32_t iter, uint32_t worker0,
                                     int32_t *idx_out, void *stream)
{
    if (n <= 0 || n > 0x7FFFFFFFll || M <= 0 || B <= 0 || !idx_out) return DQ_ERR_INVALID_ARG;
    StreamKey key{static_cast<uint32_t>(seed), static_cast<uint32_t>(seed >> 32), iter, 0u, DQ_TAG_SAMPLE};
    const dim3 grid(static_cast<unsigned>(ceil_div(B, kThreads)), static_cast<unsigned>(M));
    sample_indices_kernel<<<grid, dim3(kThreads), 0, as_stream(stream)>>>(static_cast<uint32_t>(n), B, key, worker0, idx_out);
    DQ_LAUNCH_CHECK();
    return DQ_OK;
}

extern "C" int32_t dq_sparsify(const float *alpha, int64_t d, int64_t M, int64_t ld, const float *phi, uint64_t seed,
                               uint32_t iter, uint32_t worker0, float *beta_out, int64_t ld_out, float *absmax_out,
                               int32_t *nnz_out, void *stream)
{
    if (d <= 0 || M <= 0 || !alpha || !beta_out || !absmax_out || !nnz_out || ld < d || ld_out < d)
        return DQ_ERR_INVALID_ARG;
    StreamKey key{static_cast<uint32_t>(seed), static_cast<uint32_t>(seed >> 32), iter, 0u, DQ_TAG_SPARSIFY};
    sparsify_kernel<<<dim3(static_cast<unsigned>(M)), dim3(kSparsifyThreads), 0, as_stream(stream)>>>(
        alpha, d, ld, phi, key, worker0, beta_out, ld_out, absmax_out, nnz_out);
    DQ_LAUNCH_CHECK();
    return DQ_OK;
}
