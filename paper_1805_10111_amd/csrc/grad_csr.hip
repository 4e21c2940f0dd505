// CSR-feature gradient kernels: epoch prologue (full gradient, Alg. 1) and the worker step
// (Alg. 1 worker (i)-(ii), Alg. 2 worker (i)-(iii)) for bag-of-words shaped data.
//
// A mini-batch of such rows touches a few thousand entries, far too few to be bandwidth
// bound; what matters is that one launch does the whole worker step and that the result
// is reproducible.  One block of 1024 threads owns a worker: the gradient alpha (d floats)
// lives in LDS for the whole step and never goes to memory.
//   1. margins: one wavefront per row gathers q and the snapshot at the row's columns and
//      reduces the two dot products; lane 0 forms the row's coefficient;
//   2. the rows' entries, pre-multiplied by their coefficient, are staged in LDS;
//   3. scatter: each wavefront owns a contiguous range of columns and walks the staged rows
//      in order, adding the entries that fall in its range -- no two lanes ever add to the
//      same address at once and every column sees its rows in index order, so no atomics
//      are needed and the sum is deterministic;
//   4. the tail of the worker step (sparsify, scale, quantize, pack) runs from LDS.
// The full gradient uses the same block procedure over many blocks, each leaving a partial
// d-vector that a second kernel adds up in a fixed order.
#include "dq_common.h"
#include "elementwise.h"
#include "grad_common.h"
#include "grad_launch.h"

namespace dq {

constexpr int kCsrThreads = 1024;
constexpr int kCsrWaves = kCsrThreads / kWave;
constexpr int kCsrMaxRows = 256;                 // rows a block handles per pass (LDS metadata)
constexpr int64_t kLdsBudget = 152 * 1024;       // of the 160 KB per compute unit
constexpr int64_t kCsrFixedLds = 12 * 1024;      // static arrays below, rounded up

struct CsrView {
    const int64_t *indptr;
    const int32_t *indices;
    const float *values;
    const float *y;
    int64_t n, d;
};

// Per-block LDS metadata of the rows in flight.
struct RowMeta {
    int row[kCsrMaxRows];        // sample index, -1 = ignored
    int64_t start[kCsrMaxRows];  // first entry
    int len[kCsrMaxRows];
    int off[kCsrMaxRows];        // offset in the staging buffer (rows of the current group)
    float coef[kCsrMaxRows];
};

// Steps 2 and 3 for rows [0, nrows) described by `meta`, accumulating into alpha (LDS).
// stage_col / stage_val hold `cap` entries.  Rows longer than `cap` are read from memory.
__device__ __forceinline__ void csr_scatter_rows(const CsrView &A, RowMeta &meta, int nrows, float *alpha,
                                                 int *stage_col, float *stage_val, int cap, int *sh_ctl)
{
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int64_t span = (A.d + kCsrWaves - 1) / kCsrWaves;
    const int64_t lo = wave * span, hi = min(A.d, lo + span);
    int g0 = 0;
    while (g0 < nrows) {
        // group of consecutive rows that fits the staging buffer (thread 0 decides, all follow)
        if (threadIdx.x == 0) {
            int g = g0, off = 0, direct = 0;
            if (meta.len[g0] > cap) {
                g = g0 + 1;
                direct = 1;
            } else {
                while (g < nrows && meta.len[g] <= cap && off + meta.len[g] <= cap) {
                    meta.off[g] = off;
                    off += meta.len[g];
                    ++g;
                }
            }
            sh_ctl[0] = g;
            sh_ctl[1] = direct;
        }
        __syncthreads();
        const int g1 = sh_ctl[0];
        const bool direct = sh_ctl[1] != 0;
        if (!direct) {
            for (int r = g0 + wave; r < g1; r += kCsrWaves) {          // stage: one wave per row
                const float cf = meta.coef[r];
                const int64_t s = meta.start[r];
                for (int k = lane; k < meta.len[r]; k += kWave) {
                    stage_col[meta.off[r] + k] = A.indices[s + k];
                    stage_val[meta.off[r] + k] = cf * A.values[s + k];
                }
            }
            __syncthreads();
            for (int r = g0; r < g1; ++r) {                              // scatter: rows in order
                const int base = meta.off[r];
                for (int k = lane; k < meta.len[r]; k += kWave) {
                    const int c = stage_col[base + k];
                    if (c >= lo && c < hi) alpha[c] += stage_val[base + k];
                }
            }
        } else {
            const float cf = meta.coef[g0];
            const int64_t s = meta.start[g0];
            for (int k = lane; k < meta.len[g0]; k += kWave) {
                const int c = A.indices[s + k];
                if (c >= lo && c < hi) alpha[c] += cf * A.values[s + k];
            }
        }
        __syncthreads();
        g0 = g1;
    }
}

// ------------------------------------------------------------------ worker step
struct CsrWorkerArgs {
    CsrView A;
    const int32_t *idx;
    int B;
    const uint32_t *xq; const float *delta_x; int b_x;
    const float *x_snap, *z_snap;
    float l2;
    float *alpha_out; int64_t ld;
    float *absmax_out, *l1norm_out;
    int sparsify, b;
    StreamKey key; uint32_t worker0;
    uint32_t *packed; int64_t ld_words, row_words;
    float *delta_out; int32_t *nnz_out; uint32_t *status;
    int cap;                       // staging capacity in entries
};

__global__ __launch_bounds__(kCsrThreads) void csr_worker_kernel(const CsrWorkerArgs a)
{
    extern __shared__ float lds[];
    __shared__ RowMeta meta;
    __shared__ float sh_y[kCsrMaxRows];
    __shared__ uint32_t su[kCsrWaves];
    __shared__ int si[kCsrWaves];
    __shared__ double sd[kCsrWaves];
    __shared__ int sh_ctl[2];
    const int64_t d = a.A.d;
    float *alpha = lds;
    int *stage_col = reinterpret_cast<int *>(lds + ((d + 3) / 4) * 4);
    float *stage_val = reinterpret_cast<float *>(stage_col + a.cap);

    const int m = blockIdx.x;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const ModelMsg msg{a.xq, a.b_x == 32 ? 1.0f : a.delta_x[0], a.b_x};

    // alpha starts as the dense part  l2*(q - snapshot)
    for (int64_t j = threadIdx.x; j < d; j += kCsrThreads) alpha[j] = a.l2 * (model_value(msg, j) - a.x_snap[j]);

    const float fB = static_cast<float>(a.B);
    for (int r0 = 0; r0 < a.B; r0 += kCsrMaxRows) {                     // passes of at most kCsrMaxRows rows
        const int nrows = min(kCsrMaxRows, a.B - r0);
        if (static_cast<int>(threadIdx.x) < nrows) {
            const int r = r0 + threadIdx.x;
            int64_t i;
            if (a.idx) {
                i = a.idx[static_cast<int64_t>(m) * a.B + r];
            } else {
                StreamKey sk = a.key;
                sk.worker = a.worker0 + static_cast<uint32_t>(m);
                sk.tag = DQ_TAG_SAMPLE;
                i = __umulhi(stream_word(sk, static_cast<uint64_t>(r)), static_cast<uint32_t>(a.A.n));
            }
            const bool ok = static_cast<uint64_t>(i) < static_cast<uint64_t>(a.A.n);
            meta.row[threadIdx.x] = ok ? static_cast<int>(i) : -1;
            const int64_t s = ok ? a.A.indptr[i] : 0;
            meta.start[threadIdx.x] = s;
            meta.len[threadIdx.x] = ok ? static_cast<int>(a.A.indptr[i + 1] - s) : 0;
            sh_y[threadIdx.x] = ok ? a.A.y[i] : 1.0f;
        }
        __syncthreads();
        // 1. margins and coefficients: one wave per row
        for (int r = wave; r < nrows; r += kCsrWaves) {
            const int64_t s = meta.start[r];
            float dz = 0.0f, zs = 0.0f;
            for (int k = lane; k < meta.len[r]; k += kWave) {
                const int c = a.A.indices[s + k];
                const float v = a.A.values[s + k];
                const float xc = a.x_snap[c];
                dz = fmaf(v, model_value(msg, c) - xc, dz);
                if (!a.z_snap) zs = fmaf(v, xc, zs);
            }
            dz = wave_sum_f32(dz);
            if (!a.z_snap) zs = wave_sum_f32(zs);
            if (lane == 0) {
                float cf = 0.0f;
                if (meta.row[r] >= 0) {
                    if (a.z_snap) zs = a.z_snap[meta.row[r]];
                    cf = vr_slope_diff(sh_y[r], zs, dz) / fB;
                }
                meta.coef[r] = cf;
            }
        }
        __syncthreads();
        // 2.-3. staged, ordered scatter into alpha
        csr_scatter_rows(a.A, meta, nrows, alpha, stage_col, stage_val, a.cap, sh_ctl);
    }

    // 4. outputs
    if (a.alpha_out)
        for (int64_t j = threadIdx.x; j < d; j += kCsrThreads) a.alpha_out[static_cast<int64_t>(m) * a.ld + j] = alpha[j];
    if (!a.packed) {
        uint32_t vmax = 0;
        double s1 = 0.0;
        for (int64_t j = threadIdx.x; j < d; j += kCsrThreads) {
            vmax = max(vmax, abs_bits(alpha[j]));
            s1 += static_cast<double>(fabsf(alpha[j]));
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
    case 2: worker_tail_from_lds<2>(alpha, d, a.sparsify != 0, a.b, key, out, su, si); break;
    case 4: worker_tail_from_lds<4>(alpha, d, a.sparsify != 0, a.b, key, out, su, si); break;
    case 32: worker_tail_from_lds<32>(alpha, d, a.sparsify != 0, a.b, key, out, su, si); break;
    default: worker_tail_from_lds<8>(alpha, d, a.sparsify != 0, a.b, key, out, su, si); break;
    }
}

// ------------------------------------------------------------------ epoch prologue
// grid (P): block p owns rows [p*per, (p+1)*per), processed kCsrMaxRows at a time.
__global__ __launch_bounds__(kCsrThreads) void csr_full_partial_kernel(
    const CsrView A, const float *__restrict__ x, float *__restrict__ z_out, float *__restrict__ partial, int64_t ldp,
    double *__restrict__ loss_partial, int cap)
{
    extern __shared__ float lds[];
    __shared__ RowMeta meta;
    __shared__ double sh_loss[kCsrWaves];
    __shared__ int sh_ctl[2];
    const int64_t d = A.d;
    float *acc = lds;
    int *stage_col = reinterpret_cast<int *>(lds + ((d + 3) / 4) * 4);
    float *stage_val = reinterpret_cast<float *>(stage_col + cap);
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    for (int64_t j = threadIdx.x; j < ldp; j += kCsrThreads) acc[j] = 0.0f;
    const int64_t per = (A.n + gridDim.x - 1) / gridDim.x;
    const int64_t i0 = blockIdx.x * per, i1 = min(A.n, i0 + per);
    const float fn = static_cast<float>(A.n);
    double loss = 0.0;                                   // lane 0 of each wave
    for (int64_t ib = i0; ib < i1; ib += kCsrMaxRows) {
        const int nrows = static_cast<int>(min<int64_t>(kCsrMaxRows, i1 - ib));
        if (static_cast<int>(threadIdx.x) < nrows) {
            const int64_t i = ib + threadIdx.x;
            const int64_t s = A.indptr[i];
            meta.row[threadIdx.x] = static_cast<int>(i);
            meta.start[threadIdx.x] = s;
            meta.len[threadIdx.x] = static_cast<int>(A.indptr[i + 1] - s);
        }
        __syncthreads();
        for (int r = wave; r < nrows; r += kCsrWaves) {
            const int64_t s = meta.start[r];
            float z = 0.0f;
            for (int k = lane; k < meta.len[r]; k += kWave) z = fmaf(A.values[s + k], x[A.indices[s + k]], z);
            z = wave_sum_f32(z);
            if (lane == 0) {
                const int64_t i = ib + r;
                const float y = A.y[i];
                if (z_out) z_out[i] = z;
                loss += static_cast<double>(logistic_loss(y * z));
                meta.coef[r] = logistic_slope(y, z) / fn;
            }
        }
        __syncthreads();
        csr_scatter_rows(A, meta, nrows, acc, stage_col, stage_val, cap, sh_ctl);
    }
    for (int64_t j = threadIdx.x; j < ldp; j += kCsrThreads) partial[static_cast<int64_t>(blockIdx.x) * ldp + j] = acc[j];
    if (lane == 0) sh_loss[wave] = loss;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = sh_loss[0];
        for (int w = 1; w < kCsrWaves; ++w) t += sh_loss[w];
        loss_partial[blockIdx.x] = t;
    }
}

// defined in grad_dense.hip
int launch_full_finish(const float *partial, int P, int64_t ldp, int64_t n, int64_t d, const float *x, float l2, float l1,
                       const double *loss_partial, float *g_out, double *obj_out, hipStream_t st);
int launch_worker_zero(const WorkerArgs &a, int64_t d, int64_t row_words, hipStream_t st);

// ------------------------------------------------------------------ host side
static int64_t pad4(int64_t d) { return (d + 3) / 4 * 4; }

// Staging capacity (entries) that fits next to the d-vector; 0 if the vector itself does not fit.
static int csr_stage_cap(int64_t d)
{
    const int64_t left = kLdsBudget - kCsrFixedLds - pad4(d) * 4;
    if (left < 8 * 512) return 0;
    const int64_t cap = left / 8;
    return static_cast<int>(cap > 8192 ? 8192 : cap);
}

static int64_t csr_full_splits(int64_t n)
{
    int64_t P = ceil_div(n, 64);
    if (P > 256) P = 256;
    if (P < 1) P = 1;
    return P;
}

int64_t csr_workspace_bytes(int32_t op, const dq_problem *prob, int64_t, int64_t)
{
    if (op == DQ_OP_FULL_GRAD) {
        const int64_t P = csr_full_splits(prob->n);
        return P * pad4(prob->d) * 4 + P * 8;
    }
    return 0;                                    // the worker step keeps everything in LDS
}

// Kernels that use more than 64 KB of dynamic LDS must be told so once (the limit is raised to the budget).
template <typename K>
static int allow_big_lds(K kernel, bool &done)
{
    if (!done) {
        DQ_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       static_cast<int>(kLdsBudget - kCsrFixedLds)));
        done = true;
    }
    return DQ_OK;
}

int csr_full_grad(const dq_problem *prob, const float *x, float *g_out, float *z_out, double *obj_out, void *ws,
                  int64_t ws_bytes, hipStream_t st)
{
    const int64_t d = prob->d, n = prob->n;
    const int cap = csr_stage_cap(d);
    if (cap == 0) return DQ_ERR_UNSUPPORTED;
    if (ws_bytes < csr_workspace_bytes(DQ_OP_FULL_GRAD, prob, 0, 0) || !ws) return DQ_ERR_WORKSPACE;
    const int64_t ldp = pad4(d);
    const int P = static_cast<int>(csr_full_splits(n));
    float *partial = static_cast<float *>(ws);
    double *loss_partial = reinterpret_cast<double *>(partial + static_cast<int64_t>(P) * ldp);
    const size_t lds = static_cast<size_t>(ldp) * 4 + static_cast<size_t>(cap) * 8;
    static bool attr_done = false;
    int rc = allow_big_lds(csr_full_partial_kernel, attr_done);
    if (rc != DQ_OK) return rc;
    const CsrView A{prob->indptr, prob->indices, prob->values, prob->y, n, d};
    csr_full_partial_kernel<<<dim3(P), dim3(kCsrThreads), lds, st>>>(A, x, z_out, partial, ldp, loss_partial, cap);
    DQ_LAUNCH_CHECK();
    return launch_full_finish(partial, P, ldp, n, d, x, prob->l2, prob->l1, loss_partial, g_out, obj_out, st);
}

int csr_worker(const dq_problem *prob, const WorkerArgs &a, hipStream_t st)
{
    const int64_t d = prob->d;
    const int cap = csr_stage_cap(d);
    if (cap == 0) return DQ_ERR_UNSUPPORTED;
    const int64_t row_words = a.packed ? (a.b == 32 ? d : packed_words(d, a.b)) : 0;
    if (a.model_is_snapshot) return launch_worker_zero(a, d, row_words, st);
    CsrWorkerArgs k{};
    k.A = CsrView{prob->indptr, prob->indices, prob->values, prob->y, prob->n, d};
    k.idx = a.idx; k.B = static_cast<int>(a.B);
    k.xq = a.xq; k.delta_x = a.delta_x; k.b_x = a.b_x; k.x_snap = a.x_snap; k.z_snap = a.z_snap; k.l2 = prob->l2;
    k.alpha_out = a.alpha_out; k.ld = a.ld; k.absmax_out = a.absmax_out; k.l1norm_out = a.l1norm_out;
    k.sparsify = a.sparsify; k.b = a.b;
    k.key = StreamKey{static_cast<uint32_t>(a.seed), static_cast<uint32_t>(a.seed >> 32), a.iter, 0u, DQ_TAG_GRAD};
    k.worker0 = a.worker0;
    k.packed = a.packed; k.ld_words = a.ld_words; k.row_words = row_words;
    k.delta_out = a.delta_out; k.nnz_out = a.nnz_out; k.status = a.status;
    k.cap = cap;
    const size_t lds = static_cast<size_t>(pad4(d)) * 4 + static_cast<size_t>(cap) * 8;
    static bool attr_done = false;
    int rc = allow_big_lds(csr_worker_kernel, attr_done);
    if (rc != DQ_OK) return rc;
    csr_worker_kernel<<<dim3(static_cast<unsigned>(a.M)), dim3(kCsrThreads), lds, st>>>(k);
    DQ_LAUNCH_CHECK();
    if (a.ev_after_stream) DQ_HIP_TRY(hipEventRecord(a.ev_after_stream, st));
    return DQ_OK;
}

}  // namespace dq
