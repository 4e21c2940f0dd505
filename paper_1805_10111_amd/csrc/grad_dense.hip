// Dense-feature gradient kernels: the epoch prologue (full gradient, Alg. 1) and the
// worker's variance-reduced mini-batch gradient (Alg. 1, worker (i)), optionally fused
// with the rest of the worker step (Alg. 1 worker (ii) / Alg. 2 worker (ii)-(iii)).
//
// Work shape: GEMV-like (every matrix element is used for two dot products and one
// rank-1 update, ~1.5 flop per byte), so the bound is HBM and the kernels are built
// around reading each feature row exactly once: one wavefront owns a row, holds it in
// registers (NCH float4 per lane, covering d <= 256*NCH), reduces the margin with a
// butterfly, and accumulates coef * row into a per-wave register accumulator.  Partial
// sums leave the block through LDS in a fixed order and are combined by a second
// small kernel, so results are run-to-run deterministic.
#include "dq_common.h"
#include "elementwise.h"
#include "grad_common.h"
#include "grad_launch.h"

namespace dq {

constexpr int kRowThreads = 256;                 // 4 wavefronts per block
constexpr int kRowWaves = kRowThreads / kWave;

// Loads the lane's share of a row: float4 number lane + 64*c for c < NCH; zero past d.
template <int NCH>
__device__ __forceinline__ void load_row(const float *__restrict__ row, int64_t d, int lane, float4 (&a)[NCH])
{
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int64_t col = 4ll * (lane + kWave * c);
        if (col + 3 < d) {
            a[c] = *reinterpret_cast<const float4 *>(row + col);
        } else {
            a[c].x = col + 0 < d ? row[col + 0] : 0.0f;
            a[c].y = col + 1 < d ? row[col + 1] : 0.0f;
            a[c].z = col + 2 < d ? row[col + 2] : 0.0f;
            a[c].w = 0.0f;
        }
    }
}

template <int NCH>
__device__ __forceinline__ float dot_row(const float4 (&a)[NCH], const float4 (&v)[NCH])
{
    float s = 0.0f;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        s = fmaf(a[c].x, v[c].x, s);
        s = fmaf(a[c].y, v[c].y, s);
        s = fmaf(a[c].z, v[c].z, s);
        s = fmaf(a[c].w, v[c].w, s);
    }
    return s;
}

template <int NCH>
__device__ __forceinline__ void axpy_row(float coef, const float4 (&a)[NCH], float4 (&acc)[NCH])
{
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        acc[c].x = fmaf(coef, a[c].x, acc[c].x);
        acc[c].y = fmaf(coef, a[c].y, acc[c].y);
        acc[c].z = fmaf(coef, a[c].z, acc[c].z);
        acc[c].w = fmaf(coef, a[c].w, acc[c].w);
    }
}

// Sum of the block's per-wave accumulators in wave order, through LDS, then to `dst`.
template <int NCH>
__device__ __forceinline__ void block_reduce_store(const float4 (&acc)[NCH], float4 *sh, int lane, int wave,
                                                   float *__restrict__ dst, int64_t d)
{
    for (int w = 0; w < kRowWaves; ++w) {
        if (wave == w) {
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                const int k = lane + kWave * c;
                if (w == 0) {
                    sh[k] = acc[c];
                } else {
                    float4 t = sh[k];
                    t.x += acc[c].x; t.y += acc[c].y; t.z += acc[c].z; t.w += acc[c].w;
                    sh[k] = t;
                }
            }
        }
        __syncthreads();
    }
    const int64_t d4 = (d + 3) / 4;                       // dst rows are padded to a multiple of 4
    for (int64_t k = threadIdx.x; k < d4; k += kRowThreads) reinterpret_cast<float4 *>(dst)[k] = sh[k];
}

// ------------------------------------------------------------------ worker: partial sums
// grid (P, M).  Wave (blockIdx.x*4 + wave) of worker m takes mini-batch slots r, r+4P, ...
// partial[(m*P + blockIdx.x) * ldp + j] = sum over the block's rows of coef_i * a_ij.
template <int NCH, bool HAVE_Z>
__global__ __launch_bounds__(kRowThreads) void vr_dense_partial_kernel(
    const float *__restrict__ X, int64_t lda, int64_t n, int64_t d, const float *__restrict__ yv,
    const int32_t *__restrict__ idx, int B, const uint32_t *__restrict__ xq, const float *__restrict__ delta_x, int b_x,
    const float *__restrict__ x_snap, const float *__restrict__ z_snap, float *__restrict__ partial, int64_t ldp)
{
    __shared__ float4 sh[kWave * NCH];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int m = blockIdx.y, P = gridDim.x;
    const ModelMsg msg{xq, b_x == 32 ? 1.0f : delta_x[0], b_x};
    float4 dx[NCH], xs[HAVE_Z ? 1 : NCH], acc[NCH];
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int64_t col = 4ll * (lane + kWave * c);
        float q[4], s[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const bool in = col + e < d;
            s[e] = in ? x_snap[col + e] : 0.0f;
            q[e] = in ? model_value(msg, col + e) : 0.0f;
        }
        dx[c] = make_float4(q[0] - s[0], q[1] - s[1], q[2] - s[2], q[3] - s[3]);
        if constexpr (!HAVE_Z) xs[c] = make_float4(s[0], s[1], s[2], s[3]);
        acc[c] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    }
    const int32_t *my_idx = idx + static_cast<int64_t>(m) * B;
    const float fB = static_cast<float>(B);
    for (int r = blockIdx.x * kRowWaves + wave; r < B; r += P * kRowWaves) {
        const int64_t i = my_idx[r];
        if (static_cast<uint64_t>(i) >= static_cast<uint64_t>(n)) continue;      // out-of-range index: ignored
        float4 a[NCH];
        load_row<NCH>(X + i * lda, d, lane, a);
        const float dz = wave_sum_f32(dot_row<NCH>(a, dx));
        float zs;
        if constexpr (HAVE_Z) zs = z_snap[i];
        else zs = wave_sum_f32(dot_row<NCH>(a, xs));
        const float coef = vr_slope_diff(yv[i], zs, dz) / fB;
        axpy_row<NCH>(coef, a, acc);
    }
    block_reduce_store<NCH>(acc, sh, lane, wave, partial + (static_cast<int64_t>(m) * P + blockIdx.x) * ldp, d);
}

// ------------------------------------------------------------------ worker: combine + tail
// grid (M), dynamic LDS: d floats.  alpha = sum_p partial_p + l2*(q - snapshot), then either
// store alpha and its norms (packed == nullptr) or run the worker tail.
template <int FIELD>
__global__ __launch_bounds__(kRowThreads) void vr_dense_finish_kernel(
    const float *__restrict__ partial, int P, int64_t ldp, int64_t d, const uint32_t *__restrict__ xq,
    const float *__restrict__ delta_x, int b_x, const float *__restrict__ x_snap, float l2,
    float *__restrict__ alpha_out, int64_t ld, float *__restrict__ absmax_out, float *__restrict__ l1norm_out,
    int sparsify, int b, StreamKey key, uint32_t worker0, uint32_t *__restrict__ packed, int64_t ld_words,
    int64_t row_words, float *__restrict__ delta_out, int32_t *__restrict__ nnz_out, uint32_t *__restrict__ status)
{
    extern __shared__ float sh_alpha[];
    __shared__ uint32_t su[kRowWaves];
    __shared__ int si[kRowWaves];
    __shared__ double sd[kRowWaves];
    const int m = blockIdx.x;
    const ModelMsg msg{xq, b_x == 32 ? 1.0f : delta_x[0], b_x};
    const int64_t chunks = (d + 15) / 16;
    for (int64_t c = threadIdx.x; c < chunks; c += kRowThreads) {
        const int64_t base = c * 16;
        float a[16], t[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) a[j] = 0.0f;
        for (int p = 0; p < P; ++p) {
            load16(partial + (static_cast<int64_t>(m) * P + p) * ldp, base, ldp, t);
#pragma unroll
            for (int j = 0; j < 16; ++j) a[j] += t[j];
        }
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            if (base + j < d) {
                const float dxj = model_value(msg, base + j) - x_snap[base + j];
                a[j] = a[j] + l2 * dxj;
                sh_alpha[base + j] = a[j];
            }
        }
        if (alpha_out) store16(alpha_out + static_cast<int64_t>(m) * ld, base, d, a);
    }
    __syncthreads();
    if (!packed) {
        uint32_t vmax = 0;
        double s1 = 0.0;
        for (int64_t i = threadIdx.x; i < d; i += kRowThreads) {
            vmax = max(vmax, abs_bits(sh_alpha[i]));
            s1 += static_cast<double>(fabsf(sh_alpha[i]));
        }
        vmax = block_max_u32(vmax, su);
        if (threadIdx.x == 0) absmax_out[m] = __uint_as_float(vmax);
        if (l1norm_out) {
            s1 = block_sum_f64(s1, sd);
            if (threadIdx.x == 0) l1norm_out[m] = static_cast<float>(s1);
        }
        return;
    }
    key.worker = worker0 + static_cast<uint32_t>(m);
    const WorkerOut out{packed + static_cast<int64_t>(m) * ld_words, row_words, delta_out + m,
                        nnz_out ? nnz_out + m : nullptr, status};
    worker_tail_from_lds<FIELD>(sh_alpha, d, sparsify != 0, b, key, out, su, si);
}

// Flag-bit round (Section 4.1: the model equals the snapshot): alpha = 0 for every worker.
__global__ __launch_bounds__(kRowThreads) void worker_zero_kernel(
    int64_t d, float *__restrict__ alpha_out, int64_t ld, float *__restrict__ absmax_out, float *__restrict__ l1norm_out,
    uint32_t *__restrict__ packed, int64_t ld_words, int64_t row_words, float *__restrict__ delta_out, float delta_value,
    int32_t *__restrict__ nnz_out)
{
    const int m = blockIdx.y;
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kRowThreads + threadIdx.x;
    if (alpha_out && i < d) alpha_out[static_cast<int64_t>(m) * ld + i] = 0.0f;
    if (packed && i < row_words) packed[static_cast<int64_t>(m) * ld_words + i] = 0u;
    if (i == 0) {
        if (absmax_out) absmax_out[m] = 0.0f;
        if (l1norm_out) l1norm_out[m] = 0.0f;
        if (delta_out) delta_out[m] = delta_value;
        if (nnz_out) nnz_out[m] = 0;
    }
}

// ------------------------------------------------------------------ epoch prologue: partial sums
// grid (P).  Wave g = blockIdx.x*4 + wave takes rows g, g + 4P, ...
template <int NCH>
__global__ __launch_bounds__(kRowThreads) void full_dense_partial_kernel(
    const float *__restrict__ X, int64_t lda, int64_t n, int64_t d, const float *__restrict__ yv,
    const float *__restrict__ x, float *__restrict__ z_out, float *__restrict__ partial, int64_t ldp,
    double *__restrict__ loss_partial)
{
    __shared__ float4 sh[kWave * NCH];
    __shared__ double sh_loss[kRowWaves];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int P = gridDim.x;
    float4 xv[NCH], acc[NCH];
#pragma unroll
    for (int c = 0; c < NCH; ++c) acc[c] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    load_row<NCH>(x, d, lane, xv);
    const float fn = static_cast<float>(n);
    double loss = 0.0;
    for (int64_t i = blockIdx.x * kRowWaves + wave; i < n; i += static_cast<int64_t>(P) * kRowWaves) {
        float4 a[NCH];
        load_row<NCH>(X + i * lda, d, lane, a);
        const float z = wave_sum_f32(dot_row<NCH>(a, xv));
        const float y = yv[i];
        if (z_out && lane == 0) z_out[i] = z;
        loss += static_cast<double>(logistic_loss(y * z));
        axpy_row<NCH>(logistic_slope(y, z) / fn, a, acc);
    }
    if (lane == 0) sh_loss[wave] = loss;
    block_reduce_store<NCH>(acc, sh, lane, wave, partial + static_cast<int64_t>(blockIdx.x) * ldp, d);
    if (threadIdx.x == 0) {
        double t = sh_loss[0];
        for (int w = 1; w < kRowWaves; ++w) t += sh_loss[w];
        loss_partial[blockIdx.x] = t;
    }
}

// g = sum_p partial_p + l2*x; block 0 also writes P(x) = loss/n + (l2/2)||x||^2 + l1||x||_1.
__global__ __launch_bounds__(kWave) void full_finish_kernel(
    const float *__restrict__ partial, int P, int64_t ldp, int64_t n, int64_t d, const float *__restrict__ x, float l2,
    float l1, const double *__restrict__ loss_partial, float *__restrict__ g_out, double *__restrict__ obj_out)
{
    const int64_t k = static_cast<int64_t>(blockIdx.x) * kWave + threadIdx.x;      // float4 index
    const int64_t col = 4 * k;
    if (col < d) {
        float4 s = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        for (int p = 0; p < P; ++p) {
            const float4 t = reinterpret_cast<const float4 *>(partial + static_cast<int64_t>(p) * ldp)[k];
            s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
        }
        const float v[4] = {s.x, s.y, s.z, s.w};
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (col + e < d) g_out[col + e] = v[e] + l2 * x[col + e];
    }
    if (blockIdx.x == 0 && obj_out) {
        double loss = 0.0, sq = 0.0, ab = 0.0;
        for (int p = threadIdx.x; p < P; p += kWave) loss += loss_partial[p];
        for (int64_t j = threadIdx.x; j < d; j += kWave) {
            const double xj = static_cast<double>(x[j]);
            sq += xj * xj;
            ab += fabs(xj);
        }
        loss = wave_sum_f64(loss);
        sq = wave_sum_f64(sq);
        ab = wave_sum_f64(ab);
        if (threadIdx.x == 0)
            obj_out[0] = loss / static_cast<double>(n) + 0.5 * static_cast<double>(l2) * sq + static_cast<double>(l1) * ab;
    }
}

// ------------------------------------------------------------------ host side
static int dense_nch(int64_t d) { return d <= 1024 ? 4 : d <= 2048 ? 8 : d <= 4096 ? 16 : 0; }

int64_t dense_vr_splits(int64_t M, int64_t B)
{
    // blocks per worker: aim at ~768 blocks in flight, at least one mini-batch row per wavefront
    int64_t P = ceil_div(768, M);
    const int64_t by_rows = ceil_div(B, kRowWaves);
    if (P > by_rows) P = by_rows;
    if (P < 1) P = 1;
    return P;
}

int64_t dense_full_splits(int64_t n)
{
    int64_t P = ceil_div(n, kRowWaves * 8);
    if (P > 1024) P = 1024;
    if (P < 1) P = 1;
    return P;
}

static int64_t pad4(int64_t d) { return (d + 3) / 4 * 4; }

int64_t dense_workspace_bytes(int32_t op, const dq_problem *prob, int64_t M, int64_t B)
{
    const int64_t ldp = pad4(prob->d);
    if (op == DQ_OP_FULL_GRAD) {
        const int64_t P = dense_full_splits(prob->n);
        return P * ldp * 4 + P * 8;
    }
    return M * dense_vr_splits(M, B) * ldp * 4;
}

int dense_full_grad(const dq_problem *prob, const float *x, float *g_out, float *z_out, double *obj_out, void *ws,
                    int64_t ws_bytes, hipStream_t st)
{
    const int64_t d = prob->d, n = prob->n;
    const int nch = dense_nch(d);
    if (nch == 0) return DQ_ERR_UNSUPPORTED;
    if (ws_bytes < dense_workspace_bytes(DQ_OP_FULL_GRAD, prob, 0, 0) || !ws) return DQ_ERR_WORKSPACE;
    const int64_t ldp = pad4(d);
    const int P = static_cast<int>(dense_full_splits(n));
    float *partial = static_cast<float *>(ws);
    double *loss_partial = reinterpret_cast<double *>(partial + static_cast<int64_t>(P) * ldp);
    const dim3 grid(P), block(kRowThreads);
    switch (nch) {
    case 4: full_dense_partial_kernel<4><<<grid, block, 0, st>>>(prob->dense, prob->lda, n, d, prob->y, x, z_out, partial, ldp, loss_partial); break;
    case 8: full_dense_partial_kernel<8><<<grid, block, 0, st>>>(prob->dense, prob->lda, n, d, prob->y, x, z_out, partial, ldp, loss_partial); break;
    default: full_dense_partial_kernel<16><<<grid, block, 0, st>>>(prob->dense, prob->lda, n, d, prob->y, x, z_out, partial, ldp, loss_partial); break;
    }
    DQ_LAUNCH_CHECK();
    full_finish_kernel<<<dim3(static_cast<unsigned>(ceil_div(ceil_div(d, 4), kWave))), dim3(kWave), 0, st>>>(
        partial, P, ldp, n, d, x, prob->l2, prob->l1, loss_partial, g_out, obj_out);
    DQ_LAUNCH_CHECK();
    return DQ_OK;
}

template <int NCH>
static void launch_vr_partial(bool have_z, dim3 grid, hipStream_t st, const dq_problem *prob, const int32_t *idx, int B,
                              const uint32_t *xq, const float *delta_x, int b_x, const float *x_snap, const float *z_snap,
                              float *partial, int64_t ldp)
{
    if (have_z)
        vr_dense_partial_kernel<NCH, true><<<grid, dim3(kRowThreads), 0, st>>>(prob->dense, prob->lda, prob->n, prob->d, prob->y, idx, B, xq, delta_x, b_x, x_snap, z_snap, partial, ldp);
    else
        vr_dense_partial_kernel<NCH, false><<<grid, dim3(kRowThreads), 0, st>>>(prob->dense, prob->lda, prob->n, prob->d, prob->y, idx, B, xq, delta_x, b_x, x_snap, z_snap, partial, ldp);
}

int dense_worker(const dq_problem *prob, const WorkerArgs &a, hipStream_t st)
{
    const int64_t d = prob->d;
    const int nch = dense_nch(d);
    if (nch == 0) return DQ_ERR_UNSUPPORTED;
    const int64_t row_words = a.packed ? (a.b == 32 ? d : packed_words(d, a.b)) : 0;
    if (a.model_is_snapshot) {
        const int64_t span = row_words > d ? row_words : d;
        worker_zero_kernel<<<dim3(static_cast<unsigned>(ceil_div(span, kRowThreads)), static_cast<unsigned>(a.M)), dim3(kRowThreads), 0, st>>>(
            d, a.alpha_out, a.ld, a.absmax_out, a.l1norm_out, a.packed, a.ld_words, row_words, a.delta_out,
            a.b == 32 ? 1.0f : 0.0f, a.nnz_out);
        DQ_LAUNCH_CHECK();
        return DQ_OK;
    }
    if (a.ws_bytes < dense_workspace_bytes(DQ_OP_VR_GRAD, prob, a.M, a.B) || !a.ws) return DQ_ERR_WORKSPACE;
    const int64_t ldp = pad4(d);
    const int P = static_cast<int>(dense_vr_splits(a.M, a.B));
    float *partial = static_cast<float *>(a.ws);
    const dim3 grid(P, static_cast<unsigned>(a.M));
    const bool have_z = a.z_snap != nullptr;
    const int B = static_cast<int>(a.B);
    switch (nch) {
    case 4: launch_vr_partial<4>(have_z, grid, st, prob, a.idx, B, a.xq, a.delta_x, a.b_x, a.x_snap, a.z_snap, partial, ldp); break;
    case 8: launch_vr_partial<8>(have_z, grid, st, prob, a.idx, B, a.xq, a.delta_x, a.b_x, a.x_snap, a.z_snap, partial, ldp); break;
    default: launch_vr_partial<16>(have_z, grid, st, prob, a.idx, B, a.xq, a.delta_x, a.b_x, a.x_snap, a.z_snap, partial, ldp); break;
    }
    DQ_LAUNCH_CHECK();
    const size_t lds = static_cast<size_t>(d) * sizeof(float);
    const dim3 fgrid(static_cast<unsigned>(a.M)), fblock(kRowThreads);
    const StreamKey key{static_cast<uint32_t>(a.seed), static_cast<uint32_t>(a.seed >> 32), a.iter, 0u, DQ_TAG_GRAD};
#define DQ_FINISH(F)                                                                                                   \
    vr_dense_finish_kernel<F><<<fgrid, fblock, lds, st>>>(partial, P, ldp, d, a.xq, a.delta_x, a.b_x, a.x_snap, prob->l2, \
        a.alpha_out, a.ld, a.absmax_out, a.l1norm_out, a.sparsify, a.b, key, a.worker0, a.packed, a.ld_words, row_words,  \
        a.delta_out, a.nnz_out, a.status)
    switch (a.packed ? a.b : 8) {
    case 2: DQ_FINISH(2); break;
    case 4: DQ_FINISH(4); break;
    case 32: DQ_FINISH(32); break;
    default: DQ_FINISH(8); break;
    }
#undef DQ_FINISH
    DQ_LAUNCH_CHECK();
    return DQ_OK;
}

}  // namespace dq
