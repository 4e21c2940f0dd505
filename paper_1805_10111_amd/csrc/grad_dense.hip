// Dense-feature gradient kernels: the epoch prologue (full gradient, Alg. 1) and the
// worker's variance-reduced mini-batch gradient (Alg. 1, worker (i)) fused with the rest
// of the worker step (Alg. 1 worker (ii) / Alg. 2 worker (ii)-(iii)).
//
// Work shape: GEMV-like -- every matrix element feeds one or two dot products and one
// rank-1 update, about 1.5 flop per byte -- so the bound is HBM and the kernels are
// built around reading each feature row exactly once.  A block of 256 threads owns a
// group of rows of one worker; thread t holds float4 columns t, t+256, ... of R rows at
// a time in registers (R*NC float4), so R full rows (R*16 KB at d = 4096) are in flight
// per block -- twice that where the worker kernel keeps two such batches, one being
// reduced while the other is in flight.  The R margins are reduced through LDS with one
// barrier per batch, the coefficients are formed by R lanes and read back wave-uniformly,
// and coef*row is accumulated into NC float4 registers per thread.  When one block owns a worker's whole mini-batch it
// goes straight on to the tail of the worker step; otherwise each block writes its
// partial sum and a second small kernel adds the partial sums in a fixed order and runs
// the tail (the kernel boundary is what makes the partial sums visible across the
// chip's L2 slices; a per-block device-scope fence was measured to cost far more).
// Either way the summation order is fixed, so results are run-to-run deterministic.
#include <algorithm>
#include <mutex>

#include <hip/hip_ext.h>

#include "dq_common.h"
#include "elementwise.h"
#include "grad_common.h"
#include "grad_launch.h"

namespace dq {

constexpr int kRowThreads = 256;
constexpr int kRowWaves = kRowThreads / kWave;
constexpr int kMaxRowsPerBlock = 64;             // mini-batch rows a block may own: lane j of a wavefront keeps row j

// Thread's share of a row: float4 columns tid + T*c, c < NC (T threads per block); zero past d.
// STREAM: the row is read once and not again soon (the gathered rows of a mini-batch), so the load is
// marked non-temporal; the contiguous sweep of the full gradient is faster without the mark (measured).
// FULL: d equals 4 * T * NC, every column of every thread is a whole float4 inside the row and the loads
// carry no condition at all.
// The thread's columns of a vector of exactly d floats (zeros past its end).
template <int NC, bool FULL = false, int T = kRowThreads>
__device__ __forceinline__ void load_vec_cols(const float *__restrict__ v, int64_t d, float4 (&a)[NC])
{
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        const int64_t col = 4ll * (threadIdx.x + T * c);
        if (FULL || col + 3 < d) {
            a[c] = *reinterpret_cast<const float4 *>(v + col);
        } else {
            a[c].x = col + 0 < d ? v[col + 0] : 0.0f;
            a[c].y = col + 1 < d ? v[col + 1] : 0.0f;
            a[c].z = col + 2 < d ? v[col + 2] : 0.0f;
            a[c].w = 0.0f;
        }
    }
}

// The thread's columns of a feature row (row stride lda >= d rounded up to 4, so the quad that holds the row's last
// coordinate lies inside the row's own stride).  Without FULL the loads still carry no condition -- a test per lane
// in front of a load, or a select behind it, is a wait for every load in flight, once per row --: a column past the
// end reads the row's last quad instead, and mask_cols() clears what is not part of the row when the row is used.
template <int NC, bool STREAM = false, bool FULL = false, int T = kRowThreads>
__device__ __forceinline__ void load_cols(const float *__restrict__ row, int64_t d, float4 (&a)[NC])
{
    const int64_t last = (d + 3) / 4 * 4 - 4;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        const int64_t col = FULL ? 4ll * (threadIdx.x + T * c) : min<int64_t>(4ll * (threadIdx.x + T * c), last);
        if constexpr (STREAM) {
            typedef float v4f __attribute__((ext_vector_type(4)));
            const v4f t = __builtin_nontemporal_load(reinterpret_cast<const v4f *>(row + col));
            a[c] = make_float4(t.x, t.y, t.z, t.w);
        } else {
            a[c] = *reinterpret_cast<const float4 *>(row + col);
        }
    }
}

template <int NC, bool FULL = false, int T = kRowThreads>
__device__ __forceinline__ void mask_cols(float4 (&a)[NC], int64_t d)
{
    if constexpr (!FULL) {
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            const int64_t col = 4ll * (threadIdx.x + T * c);
            a[c].x = col + 0 < d ? a[c].x : 0.0f;
            a[c].y = col + 1 < d ? a[c].y : 0.0f;
            a[c].z = col + 2 < d ? a[c].z : 0.0f;
            a[c].w = col + 3 < d ? a[c].w : 0.0f;
        }
    }
}

template <int NC>
__device__ __forceinline__ void zero_cols(float4 (&a)[NC])
{
#pragma unroll
    for (int c = 0; c < NC; ++c) a[c] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
}

template <int NC>
__device__ __forceinline__ float dot_cols(const float4 (&a)[NC], const float4 (&v)[NC])
{
    float s = 0.0f;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        s = fmaf(a[c].x, v[c].x, s);
        s = fmaf(a[c].y, v[c].y, s);
        s = fmaf(a[c].z, v[c].z, s);
        s = fmaf(a[c].w, v[c].w, s);
    }
    return s;
}

template <int NC>
__device__ __forceinline__ void axpy_cols(float coef, const float4 (&a)[NC], float4 (&acc)[NC])
{
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        acc[c].x = fmaf(coef, a[c].x, acc[c].x);
        acc[c].y = fmaf(coef, a[c].y, acc[c].y);
        acc[c].z = fmaf(coef, a[c].z, acc[c].z);
        acc[c].w = fmaf(coef, a[c].w, acc[c].w);
    }
}

template <int NC, int T = kRowThreads>
__device__ __forceinline__ void store_cols(float *__restrict__ dst, int64_t ldp, const float4 (&a)[NC])
{
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        const int64_t col = 4ll * (threadIdx.x + T * c);
        if (col < ldp) *reinterpret_cast<float4 *>(dst + col) = a[c];       // ldp is a multiple of 4
    }
}

// Block-wide sums of R per-thread values: wave butterflies, then the wave sums are
// added in wave order by every thread.  `sh` holds 2 buffers of [T / 64][R] floats and
// is used alternately, so one barrier per call is enough.
template <int R, int T = kRowThreads>
__device__ __forceinline__ void block_sum_R(float (&v)[R], float *sh, int &buf)
{
    constexpr int kWaves = T / kWave;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    float *mine = sh + buf * (kWaves * R);
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const float s = wave_sum_f32(v[r]);
        if (lane == 0) mine[wave * R + r] = s;
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < R; ++r) {
        float s = mine[r];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) s += mine[w * R + r];
        v[r] = s;
    }
    buf ^= 1;
}

// ------------------------------------------------------------------ worker step
struct VrDenseArgs {
    const float *X; int64_t lda, n, d;
    const float *y;
    const int32_t *idx;              // nullable: sampled in the kernel
    int B, P;
    const uint32_t *xq; const float *delta_x; int b_x;
    int64_t model_last_word;         // index of the last word of the model message
    const float *x_snap, *z_snap;
    float l2;
    float *partial; int64_t ldp;
    // outputs (written by the block that runs the tail)
    float *alpha_out; int64_t ld;
    float *absmax_out, *l1norm_out;
    int sparsify, b;
    StreamKey key; uint32_t worker0;
    uint32_t *packed; int64_t ld_words, row_words;
    float *delta_out; int32_t *nnz_out; uint32_t *status;
    uint32_t *zero_word;             // nullable: set to 0 by one thread of the grid
    int die_major;                   // grid is (8, P, M / 8) instead of (P, M): see vr_dense_kernel
    // MODEL == 2 (Alg. 1, master (i) done here): the model itself, its largest magnitude, the master's stream, and
    // where one block leaves the message (xq_out words, delta_x_out[0])
    const float *x_model, *absmax_model;
    StreamKey model_key;
    uint32_t *xq_out; float *delta_x_out;
};

// The thread's columns of the model message (or, MODEL == 2, of the model itself) and of the snapshot, requested
// without waiting for anything (the requests have no dependence on the rows and stay in flight next to them).
// MODEL: 0 message of any width or float32; 1 message with 8-bit fields (one word per quad of coordinates);
// 2 the float32 model, which the kernel quantizes to b_x bits itself.
template <int NC>
struct ModelCols {
    ModelQuad mq[NC];
    float4 xv[NC];
    float4 xs[NC];
    float amax;
};

template <int NC, bool FULL, int T, int MODEL>
__device__ __forceinline__ void request_model_cols(const VrDenseArgs &a, const ModelMsg &msg, int zero, ModelCols<NC> &mc)
{
    const int64_t d = a.d;
    if constexpr (MODEL == 2) mc.amax = a.absmax_model[zero];
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        const int64_t col = 4ll * (threadIdx.x + T * c);
        if constexpr (MODEL == 2) {
            if constexpr (FULL) mc.xv[c] = *reinterpret_cast<const float4 *>(a.x_model + col);
            else mc.xv[c] = load4_or_zero(a.x_model, col, d);
        } else {
            mc.mq[c] = model_quad_request<MODEL == 1>(msg, col, a.model_last_word);
        }
        if constexpr (FULL) mc.xs[c] = *reinterpret_cast<const float4 *>(a.x_snap + col);
        else mc.xs[c] = load4_or_zero(a.x_snap, col, d);
    }
}

// dx = q - snapshot for the thread's columns (q: the dequantized model message); xs = the
// snapshot itself when HAVE_Z is false (margins at the snapshot must then be recomputed).
// MODEL == 2: q = Q_(delta_x, b_x)(x) is formed here, exactly as the master would have (Section 3.1; Alg. 1,
// master (i): scale from ||x||_inf, the master's random stream, quad by quad), and the block that `store` names
// also leaves the packed message and its scale in memory for the kernels and calls that come after.
template <int NC, bool HAVE_Z, int T, int MODEL>
__device__ __forceinline__ void model_minus_snapshot(const VrDenseArgs &a, const ModelMsg &msg, const ModelCols<NC> &mc,
                                                     bool store, float4 (&dx)[NC], float4 (&xs)[HAVE_Z ? 1 : NC])
{
    if constexpr (MODEL == 2) {
        const Scale s = make_scale(mc.amax, a.b_x);
        const int64_t quads = (a.d + 3) / 4;
        if (store && threadIdx.x == 0) {
            a.delta_x_out[0] = s.delta;
            if (s.bad && a.status) atomicOr(a.status, 1u);
        }
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            const int64_t qd = threadIdx.x + T * c;                  // quad of coordinates 4 qd .. 4 qd + 3
            int k[4] = {0, 0, 0, 0};
            if (s.inv_delta != 0.0f) {
                const uint4 r = stream_block(a.model_key, static_cast<uint32_t>(qd));
                k[0] = quantize_one(mc.xv[c].x, s, r.x); k[1] = quantize_one(mc.xv[c].y, s, r.y);
                k[2] = quantize_one(mc.xv[c].z, s, r.z); k[3] = quantize_one(mc.xv[c].w, s, r.w);
            }
            // (coordinates past the end were loaded as 0, have code 0 and a zero snapshot entry: dx = 0 there)
            dx[c] = make_float4(s.delta * static_cast<float>(k[0]) - mc.xs[c].x, s.delta * static_cast<float>(k[1]) - mc.xs[c].y,
                                s.delta * static_cast<float>(k[2]) - mc.xs[c].z, s.delta * static_cast<float>(k[3]) - mc.xs[c].w);
            if constexpr (!HAVE_Z) xs[c] = mc.xs[c];
            if (store) {                                             // (the same for every thread of the block)
                const bool in = qd < quads;
                if (a.b_x == 8) store_quad_bits<8>(in ? pack4<8>(k[0], k[1], k[2], k[3]) : 0u, qd, quads, a.xq_out);
                else if (a.b_x == 4) store_quad_bits<4>(in ? pack4<4>(k[0], k[1], k[2], k[3]) : 0u, qd, quads, a.xq_out);
                else store_quad_bits<2>(in ? pack4<2>(k[0], k[1], k[2], k[3]) : 0u, qd, quads, a.xq_out);
            }
        }
        return;
    }
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        const int64_t col = 4ll * (threadIdx.x + T * c);
        float q[4];
        model_quad_values<MODEL == 1>(msg, mc.mq[c], col, a.d, q);
        dx[c] = make_float4(q[0] - mc.xs[c].x, q[1] - mc.xs[c].y, q[2] - mc.xs[c].z, q[3] - mc.xs[c].w);
        if constexpr (!HAVE_Z) xs[c] = mc.xs[c];
    }
}

// With alpha of worker m in LDS: its norms (dq_vr_grad) or the tail of the worker step
// (dq_worker_step).  Scratch arrays hold one entry per wavefront of the block.
__device__ __forceinline__ void worker_outputs(const VrDenseArgs &a, int m, float *sh_alpha, uint32_t *su, int *si, double *sd,
                                               int slice = 0, int nslices = 1)
{
    const int64_t d = a.d;
    if (!a.packed) {
        uint32_t vmax = 0;
        double s1 = 0.0;
        for (int64_t i = threadIdx.x; i < d; i += blockDim.x) {
            vmax = max(vmax, abs_bits(sh_alpha[i]));
            s1 += static_cast<double>(fabsf(sh_alpha[i]));
        }
        vmax = block_max_u32(vmax, su);
        if (threadIdx.x == 0) a.absmax_out[m] = __uint_as_float(vmax);
        if (a.l1norm_out) {
            s1 = block_sum_f64(s1, sd);
            if (threadIdx.x == 0) a.l1norm_out[m] = static_cast<float>(s1);
        }
        return;
    }
    StreamKey key = a.key;
    key.worker = a.worker0 + static_cast<uint32_t>(m);
    const WorkerOut out{a.packed + static_cast<int64_t>(m) * a.ld_words, a.row_words, a.delta_out + m,
                        a.nnz_out ? a.nnz_out + m : nullptr, a.status};
    switch (a.b) {
    case 2: worker_tail_from_lds<2>(sh_alpha, d, a.sparsify != 0, a.b, key, out, su, si, slice, nslices); break;
    case 4: worker_tail_from_lds<4>(sh_alpha, d, a.sparsify != 0, a.b, key, out, su, si, slice, nslices); break;
    case 32: worker_tail_from_lds<32>(sh_alpha, d, a.sparsify != 0, a.b, key, out, su, si, slice, nslices); break;
    default: worker_tail_from_lds<8>(sh_alpha, d, a.sparsify != 0, a.b, key, out, su, si, slice, nslices); break;
    }
}

// One block owned the whole mini-batch of worker m: alpha = acc + l2*(q - snapshot), then the outputs.
template <int NC, int T>
__device__ __forceinline__ void worker_finish(const VrDenseArgs &a, int m, const float4 (&acc)[NC], const float4 (&dx)[NC],
                                              float *sh_alpha, uint32_t *su, int *si, double *sd)
{
    const int64_t d = a.d;
    if constexpr (NC == 1) {
        // thread t holds quad t of the whole gradient (zeros past d): the plain quantization runs from the registers
        if (a.packed && !a.sparsify && a.b != 32) {            // (the same for every thread)
            const float4 v = make_float4(acc[0].x + a.l2 * dx[0].x, acc[0].y + a.l2 * dx[0].y, acc[0].z + a.l2 * dx[0].z,
                                         acc[0].w + a.l2 * dx[0].w);
            if (a.alpha_out) store_quad(a.alpha_out + static_cast<int64_t>(m) * a.ld, threadIdx.x, d, v);
            StreamKey key = a.key;
            key.worker = a.worker0 + static_cast<uint32_t>(m);
            const WorkerOut out{a.packed + static_cast<int64_t>(m) * a.ld_words, a.row_words, a.delta_out + m,
                                a.nnz_out ? a.nnz_out + m : nullptr, a.status};
            switch (a.b) {
            case 2: worker_tail_one_quad<2>(v, d, a.b, key, out, su, si, 0, 1); break;
            case 4: worker_tail_one_quad<4>(v, d, a.b, key, out, su, si, 0, 1); break;
            default: worker_tail_one_quad<8>(v, d, a.b, key, out, su, si, 0, 1); break;
            }
            return;
        }
    }
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        const int64_t col = 4ll * (threadIdx.x + T * c);
        const float v[4] = {acc[c].x + a.l2 * dx[c].x, acc[c].y + a.l2 * dx[c].y, acc[c].z + a.l2 * dx[c].z,
                            acc[c].w + a.l2 * dx[c].w};
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (col + e < d) {
                sh_alpha[col + e] = v[e];
                if (a.alpha_out) a.alpha_out[static_cast<int64_t>(m) * a.ld + col + e] = v[e];
            }
    }
    __syncthreads();
    worker_outputs(a, m, sh_alpha, su, si, sd);
}

// A zero the compiler cannot see through: an address formed with it is a per-lane address, so the load is a vector
// load (counted with the other vector loads of the prologue) and not a scalar one, whose wait would also hold up
// the scalar loads of the kernel arguments behind it.
__device__ __forceinline__ int opaque_zero()
{
    int z;
    asm volatile("v_mov_b32 %0, 0" : "=v"(z));
    return z;
}

// MODEL: where the model comes from (see ModelCols).
// DB: 0 one row buffer; 1 two row buffers where a block's rows allow it (decided in the kernel: all rows valid, a
// whole number of batch pairs); 2 two row buffers, the host vouching for that (mini-batches drawn in the kernel,
// the same even number of batches in every block): the kernel then holds no branch at all between its first
// instruction and the loop, and the compiler keeps the requests in the order written.
template <int NC, int R, bool HAVE_Z, bool FULL, int DB, int T, int MODEL>
__global__ __launch_bounds__(T) void vr_dense_kernel(const VrDenseArgs a)
{
    touch_kernel_arguments<sizeof(VrDenseArgs)>();
    constexpr int kWaves = T / kWave;
    __shared__ float sh_red[2 * kWaves * R * 2];
    // the in-kernel tail (one block owns the worker's whole mini-batch) exists for rows of up to 4096 floats;
    // wider rows always go through the partial sums and the second kernel
    constexpr bool kOwnTail = NC * T <= 1024;
    __shared__ __align__(16) float sh_alpha[kOwnTail ? 4 * T * NC : 4];
    __shared__ uint32_t su[kWaves];
    __shared__ int si[kWaves];
    __shared__ double sd[kWaves];

    // Workgroups go to the eight dies of the part in turn (linear workgroup number mod 8), and each die has its own
    // L2.  With a multiple of 8 workers the blocks of worker m all run on die m mod 8 -- the die that block m of
    // the second kernel runs on, which then finds most of their partial sums in its L2 (measured at M = 32,
    // d = 4096: second kernel 6.1 -> 5.75 us).
    // Such a launch has the grid (8, P, M / 8): the linear workgroup number is x + 8 (y + P z), so x is the die.
    int m = blockIdx.y, part = blockIdx.x;                 // grid (P, M)
    if (a.die_major) {
        m = static_cast<int>(blockIdx.x + 8u * blockIdx.z);
        part = static_cast<int>(blockIdx.y);
    }
    const int64_t d = a.d;
    const int lane = threadIdx.x & (kWave - 1);
    if (a.zero_word && blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0 && threadIdx.x == 0) *a.zero_word = 0u;

    // ---- The order of the prologue is the order in which memory is asked for.  Nothing of a round is on the chip
    //      when the kernel starts, and every dependent request costs a trip to memory, so the feature rows -- the
    //      134 MB that the kernel exists to stream -- are requested before anything else: the row numbers need no
    //      memory (they are drawn here, lane j of every wavefront draws and keeps row j of the block, at most 64
    //      rows per block; no shared memory and no barrier), the first batch of rows is requested, and only then
    //      labels and cached margins, all without a condition and none of them waited for before the second batch
    //      of rows is in flight too.
    //      The few small requests that depend on nothing at all -- the thread's columns of the model (message or
    //      vector), of the snapshot, and the scale -- go out while the row numbers are being drawn: they are the
    //      oldest requests, so the wait for them does not wait for rows, and the model is decoded (or quantized)
    //      while the first rows are still on their way.
    const int zero = opaque_zero();
    // (b_x = 32: delta_x is a valid dummy address and the value unused; MODEL == 2: the scale is formed here)
    const ModelMsg msg{a.xq, MODEL == 2 ? 0.0f : a.delta_x[zero], a.b_x};
    ModelCols<NC> mc;
    request_model_cols<NC, FULL, T, MODEL>(a, msg, zero, mc);
    const bool store_model = MODEL == 2 && blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0;
    const int per = (a.B + a.P - 1) / a.P;
    const int r0 = part * per;
    const int nrows = max(0, min(a.B, r0 + per) - r0);        // at most kMaxRowsPerBlock = 64 (the host sees to it)
    int my_row = -1;
    if (lane < nrows) {
        const int r = r0 + lane;
        int64_t i;
        if (DB != 2 && a.idx) {
            i = a.idx[static_cast<int64_t>(m) * a.B + r];
        } else {
            StreamKey sk = a.key;
            sk.worker = a.worker0 + static_cast<uint32_t>(m);
            sk.tag = DQ_TAG_SAMPLE;
            i = __umulhi(stream_word(sk, static_cast<uint64_t>(r)), static_cast<uint32_t>(a.n));
        }
        my_row = static_cast<uint64_t>(i) < static_cast<uint64_t>(a.n) ? static_cast<int>(i) : -1;   // out of range: ignored
    }
    // whole batches of valid rows only (the usual case): the row loads then carry no condition, so a wait for one
    // batch can leave the loads of the next one in flight.  (Every wavefront holds the same row numbers and takes
    // the same decision.)
    const bool plain = DB == 2 || (nrows > 0 && nrows % R == 0 && __all(lane >= nrows || my_row >= 0));
    const auto row_number = [&](int j) { return __builtin_amdgcn_readlane(my_row, j); };      // j < 64, wave-uniform

    float4 dx[NC], xs[HAVE_Z ? 1 : NC], acc[NC];
    const float inv_B = 1.0f / static_cast<float>(a.B);      // the mean over the mini-batch, as one multiplication per row
    float yv, zv;                                            // label and cached margin of row `lane`
    int buf = 0;
    auto load_batch = [&](int rb, float4 (&row)[R][NC]) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int i = rb + r < nrows ? row_number(rb + r) : -1;
            if (i >= 0) load_cols<NC, true, FULL, T>(a.X + static_cast<int64_t>(i) * a.lda, d, row[r]);
            else zero_cols<NC>(row[r]);
        }
    };
    auto load_rows = [&](int rb, float4 (&row)[R][NC]) {          // `plain` blocks only
#pragma unroll
        for (int r = 0; r < R; ++r)
            load_cols<NC, true, FULL, T>(a.X + static_cast<int64_t>(row_number(rb + r)) * a.lda, d, row[r]);
    };
    auto compute_batch = [&](int rb, float4 (&row)[R][NC]) {
        float dots[HAVE_Z ? R : 2 * R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            mask_cols<NC, FULL, T>(row[r], d);
            dots[r] = dot_cols<NC>(row[r], dx);
            if constexpr (!HAVE_Z) dots[R + r] = dot_cols<NC>(row[r], xs);
        }
        block_sum_R<HAVE_Z ? R : 2 * R, T>(dots, sh_red, buf);
        // lane r of every wave evaluates the coefficient of row rb + r once (the exponentials and reciprocals are
        // the expensive part of a batch); the R results are then read back wave-uniformly.  Row number, label and
        // margin of row rb + r sit in lane rb + r and are brought over as wave-uniform values.
        float dz = dots[0], zs = HAVE_Z ? 0.0f : dots[HAVE_Z ? 0 : R];
        float yl = 1.0f;
        int il = -1;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int src = min(rb + r, kWave - 1);
            const int ir = rb + r < nrows ? __builtin_amdgcn_readlane(my_row, src) : -1;
            const float yr = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(yv), src));
            il = lane == r ? ir : il;
            yl = lane == r ? yr : yl;
            dz = lane == r ? dots[r] : dz;
            if constexpr (HAVE_Z) {
                const float zr = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(zv), src));
                zs = lane == r ? zr : zs;
            } else {
                zs = lane == r ? dots[R + r] : zs;
            }
        }
        float coef_l = 0.0f;
        if (lane < R && (DB == 2 || il >= 0)) coef_l = vr_slope_diff(yl, zs, dz) * inv_B;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const float coef = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(coef_l), r));
            axpy_cols<NC>(coef, row[r], acc);          // dead rows: coef = 0 and the row registers are 0
        }
    };

    float4 row[R][NC];
    if (DB == 2 || plain) load_rows(0, row);
    else load_batch(0, row);
    {
        const int i = max(my_row, 0);                          // lanes without a row ask for sample 0; nothing reads
        yv = a.y[i];                                           // their values (a select here would be the first use
        zv = HAVE_Z ? a.z_snap[i] : 0.0f;                      // of the loads and put a wait in front of the next rows)
    }
    zero_cols<NC>(acc);

    // ---- stream the rows, R at a time
    if (DB == 2 || (DB == 1 && plain && nrows % (2 * R) == 0)) {
        // two row buffers: while one batch is reduced the other one is in flight; no load sits behind a condition
        float4 row2[R][NC];
        load_rows(R, row2);
        model_minus_snapshot<NC, HAVE_Z, T, MODEL>(a, msg, mc, store_model, dx, xs);
        int rb = 0;
        for (; rb + 2 * R < nrows; rb += 2 * R) {
            compute_batch(rb, row);
            load_rows(rb + 2 * R, row);
            compute_batch(rb + R, row2);
            load_rows(rb + 3 * R, row2);
        }
        compute_batch(rb, row);
        compute_batch(rb + R, row2);
    } else if (plain) {
        model_minus_snapshot<NC, HAVE_Z, T, MODEL>(a, msg, mc, store_model, dx, xs);
        compute_batch(0, row);
        for (int rb = R; rb < nrows; rb += R) {
            load_rows(rb, row);
            compute_batch(rb, row);
        }
    } else {
        model_minus_snapshot<NC, HAVE_Z, T, MODEL>(a, msg, mc, store_model, dx, xs);
        for (int rb = 0; rb < nrows; rb += R) {
            if (rb > 0) load_batch(rb, row);
            compute_batch(rb, row);
        }
    }

    if (a.P > 1 || !kOwnTail) {          // leave the partial sum for vr_dense_finish_kernel
        store_cols<NC, T>(a.partial + (static_cast<int64_t>(m) * a.P + part) * a.ldp, a.ldp, acc);
        return;
    }
    if constexpr (kOwnTail) worker_finish<NC, T>(a, m, acc, dx, sh_alpha, su, si, sd);
}

// Second stage when a worker's mini-batch was split over P > 1 blocks.  grid (M), 1024
// threads: thread t adds the P partial sums of float4 columns t, t+1024, ... in the order
// p = 0..P-1 (loads issued eight at a time), adds l2*(q - snapshot), leaves alpha in LDS
// and the block runs the tail of the worker step.
constexpr int kFinishThreads = 1024;
// MODEL8: the model message has 8-bit fields; WANT_ALPHA: the gradient itself is also stored (dq_vr_grad, tests).
// The kernel is a chain of latencies (launch, one trip to memory, two block reductions, the Philox rounds), so all
// of its memory requests are made up front and none of them sits behind a branch that would have to wait first.
template <bool MODEL8, bool WANT_ALPHA>
__global__ __launch_bounds__(kFinishThreads) void vr_dense_finish_kernel(const VrDenseArgs a)
{
    touch_kernel_arguments<sizeof(VrDenseArgs)>();
    extern __shared__ __align__(16) float sh_alpha_dyn[];
    __shared__ uint32_t su[kFinishThreads / kWave];
    __shared__ int si[kFinishThreads / kWave];
    __shared__ double sd[kFinishThreads / kWave];
    const int m = blockIdx.x;
    const int64_t d = a.d;
    const ModelMsg msg{a.xq, a.delta_x[opaque_zero()], a.b_x};     // (b_x = 32: a valid dummy address, value unused)
    const float *base = a.partial + static_cast<int64_t>(m) * a.P * a.ldp;
    // one sweep covers the vector and the tail is the plain quantization: then thread t keeps quad t in registers and the
    // tail runs from there (no trip through LDS)
    const bool in_registers = a.ldp <= 4ll * kFinishThreads && a.packed && !a.sparsify && a.b != 32;
    float4 mine = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    for (int64_t col = 4ll * threadIdx.x; col < a.ldp; col += 4ll * kFinishThreads) {
        float4 s = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        int p = 0;
        float4 first[8];
        const bool eight = a.P >= 8;                                // (the same for every thread)
        if (eight) {
#pragma unroll
            for (int u = 0; u < 8; ++u) first[u] = *reinterpret_cast<const float4 *>(base + u * a.ldp + col);
        }
        const ModelQuad mq = model_quad_request<MODEL8>(msg, col, a.model_last_word);
        const float4 xs4 = load4_or_zero(a.x_snap, col, d);
        const float xs[4] = {xs4.x, xs4.y, xs4.z, xs4.w};
        if (eight) {
#pragma unroll
            for (int u = 0; u < 8; ++u) { s.x += first[u].x; s.y += first[u].y; s.z += first[u].z; s.w += first[u].w; }
            p = 8;
        }
        for (; p + 8 <= a.P; p += 8) {
            float4 t[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) t[u] = *reinterpret_cast<const float4 *>(base + (p + u) * a.ldp + col);
#pragma unroll
            for (int u = 0; u < 8; ++u) { s.x += t[u].x; s.y += t[u].y; s.z += t[u].z; s.w += t[u].w; }
        }
        for (; p + 4 <= a.P; p += 4) {
            float4 t[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) t[u] = *reinterpret_cast<const float4 *>(base + (p + u) * a.ldp + col);
#pragma unroll
            for (int u = 0; u < 4; ++u) { s.x += t[u].x; s.y += t[u].y; s.z += t[u].z; s.w += t[u].w; }
        }
        for (; p < a.P; ++p) {
            const float4 t = *reinterpret_cast<const float4 *>(base + p * a.ldp + col);
            s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
        }
        float q[4];
        model_quad_values<MODEL8>(msg, mq, col, d, q);
        const float4 v = make_float4(s.x + a.l2 * (q[0] - xs[0]), s.y + a.l2 * (q[1] - xs[1]), s.z + a.l2 * (q[2] - xs[2]),
                                     s.w + a.l2 * (q[3] - xs[3]));
        if constexpr (WANT_ALPHA) {
            if (blockIdx.y == 0) store_quad(a.alpha_out + static_cast<int64_t>(m) * a.ld, col >> 2, d, v);
        }
        if (in_registers) mine = v;
        else store_quad(sh_alpha_dyn, col >> 2, d, v);
    }
    if (in_registers) {                  // (the same for every thread of the block)
        StreamKey key = a.key;
        key.worker = a.worker0 + static_cast<uint32_t>(m);
        const WorkerOut out{a.packed + static_cast<int64_t>(m) * a.ld_words, a.row_words, a.delta_out + m,
                            a.nnz_out ? a.nnz_out + m : nullptr, a.status};
        switch (a.b) {
        case 2: worker_tail_one_quad<2>(mine, d, a.b, key, out, su, si, blockIdx.y, gridDim.y); break;
        case 4: worker_tail_one_quad<4>(mine, d, a.b, key, out, su, si, blockIdx.y, gridDim.y); break;
        default: worker_tail_one_quad<8>(mine, d, a.b, key, out, su, si, blockIdx.y, gridDim.y); break;
        }
        return;
    }
    __syncthreads();
    // gridDim.y identical blocks per worker: each has the whole alpha and quantizes its own slice of it
    worker_outputs(a, m, sh_alpha_dyn, su, si, sd, blockIdx.y, gridDim.y);
}

// Flag-bit round (Section 4.1: the model equals the snapshot): alpha = 0 for every worker.
__global__ __launch_bounds__(kRowThreads) void worker_zero_kernel(
    int64_t d, float *__restrict__ alpha_out, int64_t ld, float *__restrict__ absmax_out, float *__restrict__ l1norm_out,
    uint32_t *__restrict__ packed, int64_t ld_words, int64_t row_words, float *__restrict__ delta_out, float delta_value,
    int32_t *__restrict__ nnz_out, uint32_t *__restrict__ zero_word)
{
    const int m = blockIdx.y;
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kRowThreads + threadIdx.x;
    if (zero_word && i == 0 && m == 0) *zero_word = 0u;
    if (alpha_out && i < d) alpha_out[static_cast<int64_t>(m) * ld + i] = 0.0f;
    if (packed && i < row_words) packed[static_cast<int64_t>(m) * ld_words + i] = 0u;
    if (i == 0) {
        if (absmax_out) absmax_out[m] = 0.0f;
        if (l1norm_out) l1norm_out[m] = 0.0f;
        if (delta_out) delta_out[m] = delta_value;
        if (nnz_out) nnz_out[m] = 0;
    }
}

int launch_worker_zero(const WorkerArgs &a, int64_t d, int64_t row_words, hipStream_t st)
{
    const int64_t span = row_words > d ? row_words : d;
    worker_zero_kernel<<<dim3(static_cast<unsigned>(ceil_div(span, kRowThreads)), static_cast<unsigned>(a.M)), dim3(kRowThreads), 0, st>>>(
        d, a.alpha_out, a.ld, a.absmax_out, a.l1norm_out, a.packed, a.ld_words, row_words, a.delta_out,
        a.b == 32 ? 1.0f : 0.0f, a.nnz_out, a.zero_word);
    DQ_LAUNCH_CHECK();
    return DQ_OK;
}

// ------------------------------------------------------------------ epoch prologue: partial sums
// grid (P).  Block p owns rows [p*per, (p+1)*per) and takes them in chunks of kFullChunk rows: the labels of a
// chunk are brought into LDS first and its margins leave through LDS afterwards, so that the loop over the
// chunk's rows contains no memory access but the row loads themselves, none of them behind a condition -- only
// then can a wait for one batch leave the loads of the next batch in flight (two row buffers).
constexpr int kFullChunk = 1024;

template <int NC, int R, bool FULL, int T = kRowThreads, bool STREAM = false>
__global__ __launch_bounds__(T) void full_dense_partial_kernel(
    const float *__restrict__ X, int64_t lda, int64_t n, int64_t d, const float *__restrict__ yv,
    const float *__restrict__ x, float *__restrict__ z_out, float *__restrict__ partial, int64_t ldp,
    double *__restrict__ loss_partial)
{
    __shared__ float sh_red[2 * (T / kWave) * R];
    __shared__ float sh_y[kFullChunk], sh_z[kFullChunk];
    const int64_t per = (n + gridDim.x - 1) / gridDim.x;
    const int64_t i0 = blockIdx.x * per, i1 = min(n, i0 + per);
    float4 xv[NC], acc[NC];
    zero_cols<NC>(acc);
    load_vec_cols<NC, FULL, T>(x, d, xv);
    const float inv_n = 1.0f / static_cast<float>(n);
    double loss = 0.0;
    int buf = 0;
    auto load_rows = [&](int64_t ib, float4 (&row)[R][NC]) {          // rows ib .. ib+R-1 all exist
#pragma unroll
        for (int r = 0; r < R; ++r) load_cols<NC, STREAM, FULL, T>(X + (ib + r) * lda, d, row[r]);
    };
    auto load_batch = [&](int64_t ib, float4 (&row)[R][NC]) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (ib + r < i1) load_cols<NC, STREAM, FULL, T>(X + (ib + r) * lda, d, row[r]);
            else zero_cols<NC>(row[r]);
        }
    };
    // rows c0 + rel .. of the current chunk (cn rows); labels in sh_y, margins to sh_z
    auto compute_batch = [&](int rel, int cn, float4 (&row)[R][NC]) {
        float z[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            mask_cols<NC, FULL, T>(row[r], d);
            z[r] = dot_cols<NC>(row[r], xv);
        }
        block_sum_R<R, T>(z, sh_red, buf);
        // lane r evaluates row rel + r (slope, loss) once; wave 0 also records margin and loss
        const int lane = threadIdx.x & (kWave - 1);
        float zl = z[0];
#pragma unroll
        for (int r = 1; r < R; ++r) zl = lane == r ? z[r] : zl;
        float coef_l = 0.0f;
        if (lane < R && rel + lane < cn) {
            const float y = sh_y[rel + lane];
            coef_l = logistic_slope_fast(y, zl) * inv_n;
            if (threadIdx.x < R) {
                loss += static_cast<double>(logistic_loss_fast(y * zl));
                sh_z[rel + lane] = zl;
            }
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const float coef = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(coef_l), r));
            axpy_cols<NC>(coef, row[r], acc);
        }
    };
    for (int64_t c0 = i0; c0 < i1; c0 += kFullChunk) {
        const int cn = static_cast<int>(min<int64_t>(kFullChunk, i1 - c0));
        for (int t = threadIdx.x; t < cn; t += T) sh_y[t] = yv[c0 + t];
        __syncthreads();
        float4 rowA[R][NC], rowB[R][NC];
        const int fast = cn / (2 * R) * (2 * R);             // whole pairs of batches
        int rel = 0;
        if (fast > 0) {
            load_rows(c0, rowA);
            for (; rel + 2 * R < fast; rel += 2 * R) {
                load_rows(c0 + rel + R, rowB);
                compute_batch(rel, cn, rowA);
                load_rows(c0 + rel + 2 * R, rowA);
                compute_batch(rel + R, cn, rowB);
            }
            load_rows(c0 + rel + R, rowB);
            compute_batch(rel, cn, rowA);
            compute_batch(rel + R, cn, rowB);
            rel += 2 * R;
        }
        for (; rel < cn; rel += R) {                          // the last rows of the block
            load_batch(c0 + rel, rowA);
            compute_batch(rel, cn, rowA);
        }
        __syncthreads();
        if (z_out)
            for (int t = threadIdx.x; t < cn; t += T) z_out[c0 + t] = sh_z[t];
        __syncthreads();
    }
    store_cols<NC, T>(partial + static_cast<int64_t>(blockIdx.x) * ldp, ldp, acc);
    if (threadIdx.x < kWave) {                       // lanes 0..R-1 of wave 0 hold the block's loss terms
        loss = wave_sum_f64(loss);
        if (threadIdx.x == 0) loss_partial[blockIdx.x] = loss;
    }
}

// g = sum_p partial_p + l2*x.  Block (16 x 64): thread (tx, ty) adds partials ty, ty+64, ... of
// float4 column blockIdx.x*16 + tx; the 64 sub-sums are then added in two fixed steps (8 threads add
// 8 each, one adds those 8).  Narrow column tiles keep many compute units busy (d = 4096: 64 blocks).
// Block 0 also writes P(x) = loss/n + (l2/2)||x||^2 + l1||x||_1.
constexpr int kFinishX = 16, kFinishY = 64;
__global__ __launch_bounds__(kFinishX *kFinishY) void full_finish_kernel(
    const float *__restrict__ partial, int P, int64_t ldp, int64_t n, int64_t d, const float *__restrict__ x, float l2,
    float l1, const double *__restrict__ loss_partial, float *__restrict__ g_out, double *__restrict__ obj_out)
{
    __shared__ float4 sh[kFinishY][kFinishX];
    __shared__ float4 sh2[8][kFinishX];
    __shared__ double sdl[(kFinishX * kFinishY / kWave) * 3];
    const int tx = threadIdx.x, ty = threadIdx.y;
    const int64_t k = static_cast<int64_t>(blockIdx.x) * kFinishX + tx;      // float4 index
    const int64_t col = 4 * k;
    float4 s = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    if (col < ldp) {
        for (int p = ty; p < P; p += kFinishY) {
            const float4 t = reinterpret_cast<const float4 *>(partial + static_cast<int64_t>(p) * ldp)[k];
            s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
        }
    }
    sh[ty][tx] = s;
    __syncthreads();
    if (ty < 8) {
        float4 t = sh[ty][tx];
        for (int j = 1; j < kFinishY / 8; ++j) {
            const float4 u = sh[ty + 8 * j][tx];
            t.x += u.x; t.y += u.y; t.z += u.z; t.w += u.w;
        }
        sh2[ty][tx] = t;
    }
    __syncthreads();
    if (ty == 0 && col < d) {
        float4 t = sh2[0][tx];
        for (int j = 1; j < 8; ++j) {
            t.x += sh2[j][tx].x; t.y += sh2[j][tx].y; t.z += sh2[j][tx].z; t.w += sh2[j][tx].w;
        }
        const float v[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (col + e < d) g_out[col + e] = v[e] + l2 * x[col + e];
    }
    if (blockIdx.x == 0 && obj_out) {
        const int tid = ty * kFinishX + tx, nt = kFinishX * kFinishY;
        double loss = 0.0, sq = 0.0, ab = 0.0;
        for (int p = tid; p < P; p += nt) loss += loss_partial[p];
        for (int64_t j = tid; j < d; j += nt) {
            const double xj = static_cast<double>(x[j]);
            sq += xj * xj;
            ab += fabs(xj);
        }
        loss = wave_sum_f64(loss);
        sq = wave_sum_f64(sq);
        ab = wave_sum_f64(ab);
        if ((tid & (kWave - 1)) == 0) { const int w = tid / kWave; sdl[w * 3] = loss; sdl[w * 3 + 1] = sq; sdl[w * 3 + 2] = ab; }
        __syncthreads();
        if (tid == 0) {
            double L = 0.0, S = 0.0, A = 0.0;
            for (int j = 0; j < nt / kWave; ++j) { L += sdl[j * 3]; S += sdl[j * 3 + 1]; A += sdl[j * 3 + 2]; }
            obj_out[0] = L / static_cast<double>(n) + 0.5 * static_cast<double>(l2) * S + static_cast<double>(l1) * A;
        }
    }
}

int launch_full_finish(const float *partial, int P, int64_t ldp, int64_t n, int64_t d, const float *x, float l2, float l1,
                       const double *loss_partial, float *g_out, double *obj_out, hipStream_t st)
{
    full_finish_kernel<<<dim3(static_cast<unsigned>(ceil_div(ceil_div(d, 4), kFinishX))), dim3(kFinishX, kFinishY), 0, st>>>(
        partial, P, ldp, n, d, x, l2, l1, loss_partial, g_out, obj_out);
    DQ_LAUNCH_CHECK();
    return DQ_OK;
}

// ------------------------------------------------------------------ host side
// float4 columns per thread that cover a row: rows of up to 16384 floats are supported
static int dense_nc(int64_t d) { return d <= 1024 ? 1 : d <= 2048 ? 2 : d <= 4096 ? 4 : d <= 8192 ? 8 : d <= 16384 ? 16 : 0; }

int64_t dense_vr_splits(int64_t M, int64_t B, int64_t d)
{
    // blocks per worker.  A mini-batch of at most 32 rows stays in one block, which then runs the
    // whole worker step in a single launch; larger ones are split so that about 512 blocks
    // (two per compute unit) stream rows, each owning at least 4 of them.  Rows wider than 1024 floats
    // are streamed with two row buffers per block (see dense_worker): one block per compute unit
    // then, and a whole number of batch pairs per block.
    const bool two_buffers = dense_nc(d) >= 2;
    const int64_t target = two_buffers ? 256 : 512;
    if (B <= 32) return 1;
    int64_t P = ceil_div(target, M);
    const int64_t by_rows = ceil_div(B, 4);
    if (P > by_rows) P = by_rows;
    const int64_t need = ceil_div(B, kMaxRowsPerBlock);        // a block owns at most kMaxRowsPerBlock rows
    if (P < need) P = need;
    if (P < 1) P = 1;
    if (two_buffers) P = ceil_div(B, ceil_div(ceil_div(B, P), 4) * 4);   // rows per block: a multiple of 4
    return P;
}

// rows whose every float4 column is whole for 512 threads: the widths with a 512-thread full-gradient kernel
static bool dense_full_wide(int64_t d) { return d == 2048 || d == 4096 || d == 8192 || d == 16384; }

int64_t dense_full_splits(int64_t n, int64_t d)
{
    int64_t P = ceil_div(n, 16);
    if (dense_full_wide(d)) {
        if (P > 256) P = 256;       // one block of 512 threads per compute unit
        return P < 1 ? 1 : P;
    }
    if (P > 512) P = 512;           // two blocks per compute unit; 256 ... 2048 measured within 6 % of each other
    if (P < 1) P = 1;
    return P;
}

static int64_t pad4(int64_t d) { return (d + 3) / 4 * 4; }

// Workspace of a worker step: partial sums, M*P*ldp floats (unused when P == 1).
int64_t dense_workspace_bytes(int32_t op, const dq_problem *prob, int64_t M, int64_t B)
{
    const int64_t ldp = pad4(prob->d);
    if (op == DQ_OP_FULL_GRAD) {
        const int64_t P = dense_full_splits(prob->n, prob->d);
        return P * ldp * 4 + P * 8;
    }
    // dq_run_rounds with a bounded delay runs the worker step on contiguous groups of the M workers with this same
    // workspace, and a smaller group may be split over more blocks per worker: the size covers every group size
    int64_t rows = 0;
    for (int64_t g = 1; g <= M; ++g) rows = std::max(rows, g * dense_vr_splits(g, B, prob->d));
    return rows * ldp * 4;
}

int dense_full_grad(const dq_problem *prob, const float *x, float *g_out, float *z_out, double *obj_out, void *ws,
                    int64_t ws_bytes, hipStream_t st)
{
    const int64_t d = prob->d, n = prob->n;
    const int nc = dense_nc(d);
    if (nc == 0) return DQ_ERR_UNSUPPORTED;
    if (ws_bytes < dense_workspace_bytes(DQ_OP_FULL_GRAD, prob, 0, 0) || !ws) return DQ_ERR_WORKSPACE;
    const int64_t ldp = pad4(d);
    const int P = static_cast<int>(dense_full_splits(n, d));
    float *partial = static_cast<float *>(ws);
    double *loss_partial = reinterpret_cast<double *>(partial + static_cast<int64_t>(P) * ldp);
    const dim3 grid(P), block(kRowThreads);
    const bool full = d == 4ll * kRowThreads * nc;          // every thread's columns are whole float4s of the row
#define DQ_FULL(NC, R)                                                                                              \
    do {                                                                                                            \
        if (full) full_dense_partial_kernel<NC, R, true><<<grid, block, 0, st>>>(prob->dense, prob->lda, n, d, prob->y, x, z_out, partial, ldp, loss_partial); \
        else full_dense_partial_kernel<NC, R, false><<<grid, block, 0, st>>>(prob->dense, prob->lda, n, d, prob->y, x, z_out, partial, ldp, loss_partial); \
    } while (0)
    // Rows of 2048, 4096, 8192 or 16384 floats (every thread's columns whole): 512 threads per block, one block per
    // compute unit, non-temporal loads.  Measured on 1.6-3.3 GB of rows against 256 threads, two blocks per unit and
    // plain loads: 280 -> 240 us, 540 -> 479 us (6.84 TB/s), 282 -> 243 us, 294 -> 253 us.  (For other widths the
    // same change is a loss -- 299 -> 439 us at 3000 floats -- and they keep the kernels below.)
    if (dense_full_wide(d)) {
        const dim3 b512(512);
#define DQ_F512(NC, R) full_dense_partial_kernel<NC, R, true, 512, true><<<grid, b512, 0, st>>>(prob->dense, prob->lda, n, d, prob->y, x, z_out, partial, ldp, loss_partial)
        if (nc == 2) DQ_F512(1, 8);
        else if (nc == 4) DQ_F512(2, 4);
        else if (nc == 8) DQ_F512(4, 2);
        else DQ_F512(8, 1);
#undef DQ_F512
        DQ_LAUNCH_CHECK();
        return launch_full_finish(partial, P, ldp, n, d, x, prob->l2, prob->l1, loss_partial, g_out, obj_out, st);
    }
    switch (nc) {
    case 1: DQ_FULL(1, 8); break;
    case 2: DQ_FULL(2, 4); break;
    case 4: DQ_FULL(4, 4); break;
    case 8: DQ_FULL(8, 2); break;
    default: DQ_FULL(16, 1); break;
    }
#undef DQ_FULL
    DQ_LAUNCH_CHECK();
    return launch_full_finish(partial, P, ldp, n, d, x, prob->l2, prob->l1, loss_partial, g_out, obj_out, st);
}

// A launch whose start and end times go to the two events (when given): the kernel's own time stamps, without the
// stream time a pair of recorded events adds around it.
template <typename K>
static void launch_timed(K kernel, dim3 grid, dim3 block, size_t lds, hipStream_t st, hipEvent_t ev_start, hipEvent_t ev_stop,
                         const VrDenseArgs &k)
{
    if (ev_start && ev_stop) hipExtLaunchKernelGGL(kernel, grid, block, static_cast<uint32_t>(lds), st, ev_start, ev_stop, 0u, k);
    else kernel<<<grid, block, lds, st>>>(k);
}

template <int NC, int R, int DB, int T, bool HAVE_Z, int MODEL>
static void launch_vr2(dim3 grid, hipStream_t st, const VrDenseArgs &k, hipEvent_t e0, hipEvent_t e1)
{
    const bool full = k.d == 4ll * T * NC;       // every thread's columns are whole float4s of the row
    const dim3 block(T);
    if (full) launch_timed(vr_dense_kernel<NC, R, HAVE_Z, true, DB, T, MODEL>, grid, block, 0, st, e0, e1, k);
    else launch_timed(vr_dense_kernel<NC, R, HAVE_Z, false, DB, T, MODEL>, grid, block, 0, st, e0, e1, k);
}

template <int NC, int R, int DB, int T>
static void launch_vr1(bool have_z, dim3 grid, hipStream_t st, const VrDenseArgs &k, hipEvent_t e0, hipEvent_t e1)
{
    const bool model8 = k.b_x == 8;
    if constexpr (DB == 2) {
        if (k.x_model) {                          // (dense_model_fusable: cached margins, static two-buffer form)
            launch_vr2<NC, R, DB, T, true, 2>(grid, st, k, e0, e1);
            return;
        }
    }
    if (have_z) {
        if (model8) launch_vr2<NC, R, DB, T, true, 1>(grid, st, k, e0, e1);
        else launch_vr2<NC, R, DB, T, true, 0>(grid, st, k, e0, e1);
    } else {
        if (model8) launch_vr2<NC, R, DB, T, false, 1>(grid, st, k, e0, e1);
        else launch_vr2<NC, R, DB, T, false, 0>(grid, st, k, e0, e1);
    }
}

// two_buffers: the row width has a two-buffer kernel at all; then the static form (DB = 2) is taken when the
// mini-batches are drawn in the kernel (every row number valid) and every block owns the same whole number of
// batch pairs, else the form that decides per block.
static bool static_two_buffers(int64_t B, int64_t P, int R) { return B % P == 0 && (B / P) % (2 * R) == 0; }

template <int NC, int R, bool TWO = false, int T = kRowThreads>
static void launch_vr(bool have_z, dim3 grid, hipStream_t st, const VrDenseArgs &k, hipEvent_t e0, hipEvent_t e1)
{
    if constexpr (TWO) {
        if (!k.idx && static_two_buffers(k.B, k.P, R)) launch_vr1<NC, R, 2, T>(have_z, grid, st, k, e0, e1);
        else launch_vr1<NC, R, 1, T>(have_z, grid, st, k, e0, e1);
    } else {
        launch_vr1<NC, R, 0, T>(have_z, grid, st, k, e0, e1);
    }
}

// Rows per batch of the two-buffer kernels, by float4 columns per 256 threads (0: no two-buffer kernel).
static int two_buffer_rows(int nc) { return nc == 2 ? 4 : nc == 4 ? 2 : nc >= 8 ? 1 : 0; }

bool dense_model_fusable(const dq_problem *prob, int64_t M, int64_t B, int b_x, bool have_z)
{
    if (prob->layout != 0 || !have_z || (b_x != 2 && b_x != 4 && b_x != 8)) return false;
    const int R = two_buffer_rows(dense_nc(prob->d));
    return R > 0 && static_two_buffers(B, dense_vr_splits(M, B, prob->d), R);
}

int dense_worker(const dq_problem *prob, const WorkerArgs &a, hipStream_t st)
{
    const int64_t d = prob->d;
    const int nc = dense_nc(d);
    if (nc == 0) return DQ_ERR_UNSUPPORTED;
    const int64_t row_words = a.packed ? (a.b == 32 ? d : packed_words(d, a.b)) : 0;
    if (a.model_is_snapshot) return launch_worker_zero(a, d, row_words, st);
    if (a.ws_bytes < dense_workspace_bytes(DQ_OP_VR_GRAD, prob, a.M, a.B) || !a.ws) return DQ_ERR_WORKSPACE;
    VrDenseArgs k{};
    k.X = prob->dense; k.lda = prob->lda; k.n = prob->n; k.d = d; k.y = prob->y;
    k.idx = a.idx; k.B = static_cast<int>(a.B); k.P = static_cast<int>(dense_vr_splits(a.M, a.B, d));
    k.xq = a.xq; k.b_x = a.b_x; k.x_snap = a.x_snap; k.z_snap = a.z_snap; k.l2 = prob->l2;
    k.delta_x = a.b_x == 32 ? a.x_snap : a.delta_x;      // float32 model: no scale; the kernels read a valid dummy
    k.model_last_word = (a.b_x == 32 ? d : packed_words(d, a.b_x)) - 1;
    k.partial = static_cast<float *>(a.ws);
    k.ldp = pad4(d);
    k.alpha_out = a.alpha_out; k.ld = a.ld; k.absmax_out = a.absmax_out; k.l1norm_out = a.l1norm_out;
    k.sparsify = a.sparsify; k.b = a.b;
    k.key = StreamKey{static_cast<uint32_t>(a.seed), static_cast<uint32_t>(a.seed >> 32), a.iter, 0u, DQ_TAG_GRAD};
    k.worker0 = a.worker0;
    k.packed = a.packed; k.ld_words = a.ld_words; k.row_words = row_words;
    k.delta_out = a.delta_out; k.nnz_out = a.nnz_out; k.status = a.status; k.zero_word = a.zero_word;
    if (a.x_model) {
        if (!a.absmax_model || a.idx || !a.packed || !dense_model_fusable(prob, a.M, a.B, a.b_x, a.z_snap != nullptr))
            return DQ_ERR_INVALID_ARG;
        k.x_model = a.x_model; k.absmax_model = a.absmax_model;
        k.model_key = StreamKey{static_cast<uint32_t>(a.seed), static_cast<uint32_t>(a.seed >> 32), a.iter, DQ_MASTER_ID, DQ_TAG_MODEL};
        k.xq_out = const_cast<uint32_t *>(a.xq); k.delta_x_out = const_cast<float *>(a.delta_x);
    }
    k.die_major = a.M % 8 == 0 && a.M / 8 <= 65535;
    const dim3 grid = k.die_major ? dim3(8, k.P, static_cast<unsigned>(a.M / 8)) : dim3(k.P, static_cast<unsigned>(a.M));
    const bool have_z = a.z_snap != nullptr;
    // Rows wider than 1024 floats are streamed with two row buffers, one block per compute unit: a batch is reduced
    // while the next one is in flight, and half as many partial sums are written and added again.  Measured for the
    // two kernels of the worker step at M = 32 and 134 MB of rows, against one buffer and two blocks per unit:
    // d = 2048 31.6 against 32.4 us, d = 4096 32.1 against 34.5 us, d = 8192 36.3 against 40.8 us, d = 16384 44.7
    // against 61.7 us; at d = 1024 one buffer of 16 rows is faster (34.9 against 42.4 us).
    switch (nc) {
    case 1: launch_vr<1, 16>(have_z, grid, st, k, a.ev_start, a.ev_stop); break;
    case 2: launch_vr<1, 4, true, 512>(have_z, grid, st, k, a.ev_start, a.ev_stop); break;   // 512 threads from here on
    case 4: launch_vr<2, 2, true, 512>(have_z, grid, st, k, a.ev_start, a.ev_stop); break;
    case 8: launch_vr<4, 1, true, 512>(have_z, grid, st, k, a.ev_start, a.ev_stop); break;
    default: launch_vr<8, 1, true, 512>(have_z, grid, st, k, a.ev_start, a.ev_stop); break;
    }
    DQ_LAUNCH_CHECK();
    if (k.P > 1 || nc > 4) {
        const size_t lds = static_cast<size_t>(d) * sizeof(float);
        if (lds > 48 * 1024) {                            // more than 64 KB of dynamic LDS has to be requested once
            static std::once_flag once;
            static hipError_t once_rc = hipSuccess;
            std::call_once(once, [] {
                for (const void *f : {reinterpret_cast<const void *>(vr_dense_finish_kernel<false, false>),
                                      reinterpret_cast<const void *>(vr_dense_finish_kernel<false, true>),
                                      reinterpret_cast<const void *>(vr_dense_finish_kernel<true, false>),
                                      reinterpret_cast<const void *>(vr_dense_finish_kernel<true, true>)}) {
                    const hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, 16384 * 4);
                    if (e != hipSuccess) once_rc = e;
                }
            });
            DQ_HIP_TRY(once_rc);
        }
        // with few workers, identical blocks share the final quantization of a worker (see worker_tail_from_lds)
        // (measured at d = 4096, M = 32: two blocks per worker 0.65 us faster than one, four or eight no better)
        const bool count_ok = !a.nnz_out || (a.sparsify && a.b >= 4);
        const unsigned slices = (a.packed && count_ok && a.b != 32 && d >= 2048 && a.M <= 128) ? 2u : 1u;
        const dim3 fgrid(static_cast<unsigned>(a.M), slices), fblock(kFinishThreads);
        if (a.b_x == 8) {
            if (a.alpha_out) vr_dense_finish_kernel<true, true><<<fgrid, fblock, lds, st>>>(k);
            else vr_dense_finish_kernel<true, false><<<fgrid, fblock, lds, st>>>(k);
        } else {
            if (a.alpha_out) vr_dense_finish_kernel<false, true><<<fgrid, fblock, lds, st>>>(k);
            else vr_dense_finish_kernel<false, false><<<fgrid, fblock, lds, st>>>(k);
        }
        DQ_LAUNCH_CHECK();
    }
    return DQ_OK;
}

}  // namespace dq
