// CSR-feature gradient kernels: epoch prologue (full gradient, Alg. 1) and the worker step
// (Alg. 1 worker (i)-(ii), Alg. 2 worker (i)-(iii)) for bag-of-words shaped data.
//
// A mini-batch of such rows touches a few thousand entries, far too few to be bandwidth
// bound; what matters is that one launch does the whole worker step and that the result
// is reproducible.  One block of 1024 threads owns a worker: the gradient alpha (d floats)
// lives in LDS for the whole step and never goes to memory.
//   1. stage: the (column, value) pairs of the mini-batch rows are copied into LDS as one flat run
//      (the row of an entry is found by bisection on the prefix sums of the row lengths and is
//      kept in the bits above the column);
//   2. margins: one wavefront per row, four rows in flight, gathers q and the snapshot at the
//      row's columns and reduces the dot products; one lane per row forms its coefficient;
//   3. scatter: a few wavefronts each own a contiguous range of columns and stream over the
//      staged entries (which are in row order), adding coefficient*value for the entries in
//      their range with LDS float adds that return nothing.  All adds to a column come from one
//      wavefront, whose LDS operations execute in issue order, so every column receives its
//      terms in row order: the sum is reproducible and nothing waits on a read-modify-write;
//   4. the tail of the worker step (sparsify, scale, quantize, pack) runs from LDS.
// The full gradient uses the same block procedure over many blocks, each leaving a partial
// d-vector that a second kernel adds up in a fixed order.
#include <mutex>

#include <hip/hip_ext.h>

#include "dq_common.h"
#include "elementwise.h"
#include "grad_common.h"
#include "grad_launch.h"

namespace dq {

constexpr int kCsrThreads = 1024;
constexpr int kCsrWaves = kCsrThreads / kWave;
constexpr int kScatterWaves = 4;                 // wavefronts that add rows into the LDS vector (one per SIMD)
constexpr int kColBits = 20;                     // staged entries carry column | row << kColBits
constexpr int kColMask = (1 << kColBits) - 1;
constexpr int kFlight = 4;                       // rows a wavefront reduces at the same time
constexpr int kCsrMaxRows = 256;                 // rows a block handles per pass (LDS metadata)
constexpr int64_t kLdsBudget = 152 * 1024;       // of the 160 KB per compute unit
constexpr int64_t kCsrFixedLds = 10 * 1024;      // static arrays below, rounded up

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
    int pre[kCsrMaxRows + 1];    // exclusive prefix sum of len
    float coef[kCsrMaxRows];
    float z[kCsrMaxRows];        // cached margin at the snapshot (worker step only)
};

// Fills meta.pre with the exclusive prefix sums of meta.len[0..nrows) (pre[nrows] = total).
// The first wavefront scans the lengths, kCsrMaxRows/64 consecutive rows per lane; all threads of
// the block must call it (barriers before and after).
__device__ __forceinline__ void csr_prefix_lengths(RowMeta &meta, int nrows)
{
    constexpr int kPer = kCsrMaxRows / kWave;
    __syncthreads();
    if (threadIdx.x < kWave) {
        const int lane = threadIdx.x;
        int v[kPer], sum = 0;
#pragma unroll
        for (int u = 0; u < kPer; ++u) {
            const int r = lane * kPer + u;
            v[u] = r < nrows ? meta.len[r] : 0;
            sum += v[u];
        }
        int incl = sum;                                  // inclusive scan of the lane sums
#pragma unroll
        for (int off = 1; off < kWave; off <<= 1) {
            const int up = __shfl_up(incl, off, kWave);
            if (lane >= off) incl += up;
        }
        int run = incl - sum;
#pragma unroll
        for (int u = 0; u < kPer; ++u) {
            meta.pre[lane * kPer + u] = run;
            run += v[u];
        }
        if (lane == kWave - 1) meta.pre[kCsrMaxRows] = run;
    }
    __syncthreads();
}

// Stage, margins and scatter (the first three phases of the file header) for rows [0, nrows) described by `meta`,
// accumulating into alpha (LDS).
// The rows are taken in groups that fit the staging buffer (`stage`, `cap` (column, value) entries):
//   stage  : the group's (column, value) pairs are copied to LDS as one flat run, four entries per thread
//            in flight, the row number packed above the column;
//   margins: one wavefront per row (kFlight rows in flight) reduces sum_k value_k * vec(column_k), where
//            vec_val(vec_req(c), c) returns {first, second} operands gathered from memory -- vec_req only requests
//            (no branch, no use of what it loads), so the gathers of all rows in flight wait for memory once;
//            lane u hands the sums of its
//            u-th row to coef_of(row, first_sum, second_sum), which returns the row's coefficient;
//   scatter: kScatterWaves wavefronts own a contiguous range of columns each and stream over the staged
//            entries, adding coefficient*value for the entries that fall in their range.
// A row longer than `cap` is handled alone, straight from memory.
// Only the columns of the window [c0, c1) are accumulated, into alpha[column - c0]: a vector too long for
// LDS is built one window at a time (the caller repeats the call per window; margins are recomputed).
template <bool SECOND, typename VecReq, typename VecVal, typename CoefFn>
__device__ __forceinline__ void csr_process_rows(const CsrView &A, RowMeta &meta, int nrows, float *alpha, int c0, int c1,
                                                 int2 *stage, int cap, int *sh_ctl, VecReq vec_req, VecVal vec_val,
                                                 CoefFn coef_of)
{
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int span = (c1 - c0 + kScatterWaves - 1) / kScatterWaves;
    const int lo = c0 + wave * span, hi = wave < kScatterWaves ? min(c1, lo + span) : lo;
    int g0 = 0;
    while (g0 < nrows) {
        // group of consecutive rows that fits the staging buffer: rows g0..g1-1 with
        // pre[g1] - pre[g0] <= cap; a first row longer than cap is taken alone, unstaged
        const int base = meta.pre[g0];
        int g1 = nrows;
        bool direct = false;
        if (meta.pre[nrows] - base > cap) {            // (the same for every thread) not all remaining rows fit
            if (threadIdx.x == 0) {
                sh_ctl[0] = nrows;
                sh_ctl[1] = meta.len[g0] > cap;
            }
            __syncthreads();
            if (static_cast<int>(threadIdx.x) >= g0 && static_cast<int>(threadIdx.x) < nrows &&
                meta.pre[threadIdx.x + 1] - base > cap)
                atomicMin(&sh_ctl[0], max(static_cast<int>(threadIdx.x), g0 + 1));
            __syncthreads();
            g1 = sh_ctl[0];
            direct = sh_ctl[1] != 0;
        }
        if (!direct) {
            // ---- stage: flat copy of the group's entries; the row of an entry by bisection on pre[]
            const int total = meta.pre[g1] - base;
            for (int p0 = threadIdx.x; p0 < total; p0 += 4 * kCsrThreads) {     // four entries per thread in flight
                int64_t src[4];
                int tag[4];                                         // row number, shifted above the column bits
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int p = p0 + u * kCsrThreads;
                    int lo_r = g0, hi_r = g1;                       // pre[lo_r] - base <= p < pre[hi_r] - base
                    while (hi_r - lo_r > 1) {
                        const int mid = (lo_r + hi_r) >> 1;
                        if (meta.pre[mid] - base <= p) lo_r = mid; else hi_r = mid;
                    }
                    src[u] = p < total ? meta.start[lo_r] + (p - (meta.pre[lo_r] - base)) : -1;
                    tag[u] = lo_r << kColBits;
                }
                int2 e[4];
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if (src[u] >= 0) e[u] = make_int2(A.indices[src[u]] | tag[u], __float_as_int(A.values[src[u]]));
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if (src[u] >= 0) stage[p0 + u * kCsrThreads] = e[u];
            }
            __syncthreads();
            // ---- margins and coefficients: four rows per wavefront in flight; lane u evaluates row u's scalar
            for (int r = g0 + wave; r < g1; r += kFlight * kCsrWaves) {
                int len[kFlight], off[kFlight], maxlen = 0;
                float sa[kFlight], sb[kFlight];
#pragma unroll
                for (int u = 0; u < kFlight; ++u) {
                    const int ru = r + u * kCsrWaves;
                    len[u] = ru < g1 ? meta.len[ru] : 0;
                    off[u] = ru < g1 ? meta.pre[ru] - base : 0;
                    maxlen = max(maxlen, len[u]);
                    sa[u] = sb[u] = 0.0f;
                }
                for (int k = lane; k < maxlen; k += kWave) {
                    int2 e[kFlight];
                    float2 f[kFlight];
                    decltype(vec_req(0)) raw[kFlight];
#pragma unroll
                    for (int u = 0; u < kFlight; ++u) e[u] = k < len[u] ? stage[off[u] + k] : make_int2(0, 0);
#pragma unroll
                    for (int u = 0; u < kFlight; ++u) raw[u] = vec_req(e[u].x & kColMask);
#pragma unroll
                    for (int u = 0; u < kFlight; ++u) f[u] = vec_val(raw[u], e[u].x & kColMask);
#pragma unroll
                    for (int u = 0; u < kFlight; ++u) {
                        sa[u] = fmaf(__int_as_float(e[u].y), f[u].x, sa[u]);
                        if (SECOND) sb[u] = fmaf(__int_as_float(e[u].y), f[u].y, sb[u]);
                    }
                }
                float mine_a = 0.0f, mine_b = 0.0f;
#pragma unroll
                for (int u = 0; u < kFlight; ++u) {
                    const float ta = wave_sum_f32(sa[u]);
                    const float tb = SECOND ? wave_sum_f32(sb[u]) : 0.0f;
                    if (lane == u) {
                        mine_a = ta;
                        mine_b = tb;
                    }
                }
                const int rl = r + lane * kCsrWaves;
                if (lane < kFlight && rl < g1) meta.coef[rl] = coef_of(rl, mine_a, mine_b);
            }
            __syncthreads();
            // ---- scatter: kScatterWaves wavefronts each own a contiguous range of columns and stream over the
            //      staged entries (which are in row order), adding coefficient*value for the entries in their
            //      range with LDS float adds that return nothing.  All adds to one column come from one
            //      wavefront, whose LDS operations execute in issue order, so every column receives its
            //      terms in row order and nothing waits on a read-modify-write round trip.
            if (wave < kScatterWaves) {
                for (int p0 = lane; p0 < total; p0 += 4 * kWave) {       // four entries per lane in flight
                    int2 e[4];
                    float term[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int p = p0 + u * kWave;
                        e[u] = stage[min(p, total - 1)];
                        if (p >= total) e[u].x = kColMask;              // a column nobody owns: models have fewer than 2^20
                    }
#pragma unroll
                    for (int u = 0; u < 4; ++u) term[u] = meta.coef[(e[u].x >> kColBits) & (kCsrMaxRows - 1)];
                    asm volatile("" : "+v"(term[0]), "+v"(term[1]), "+v"(term[2]), "+v"(term[3]));   // all four loads issued here,
                                                                                                     // not inside the branches below
#pragma unroll
                    for (int u = 0; u < 4; ++u) term[u] *= __int_as_float(e[u].y);
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int c = e[u].x & kColMask;
                        if (c >= lo && c < hi) atomicAdd(&alpha[c - c0], term[u]);
                    }
                }
            }
        } else {
            // ---- one very long row, straight from memory (every wavefront computes the same sums)
            const int64_t s = meta.start[g0];
            float a1 = 0.0f, b1 = 0.0f;
            for (int k = lane; k < meta.len[g0]; k += kWave) {
                const int ck = A.indices[s + k];
                const float2 f = vec_val(vec_req(ck), ck);
                const float v = A.values[s + k];
                a1 = fmaf(v, f.x, a1);
                if (SECOND) b1 = fmaf(v, f.y, b1);
            }
            a1 = wave_sum_f32(a1);
            if (SECOND) b1 = wave_sum_f32(b1);
            __syncthreads();
            if (threadIdx.x == 0) meta.coef[g0] = coef_of(g0, a1, b1);
            __syncthreads();
            const float cf = meta.coef[g0];
            for (int k = lane; k < meta.len[g0]; k += kWave) {
                const int c = A.indices[s + k];
                if (c >= lo && c < hi) alpha[c - c0] += cf * A.values[s + k];
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
    int64_t model_last_word;       // index of the last word of the model message
    const float *x_snap, *z_snap;
    float l2;
    float *alpha_out; int64_t ld;
    float *absmax_out, *l1norm_out;
    int sparsify, b;
    StreamKey key; uint32_t worker0;
    uint32_t *packed; int64_t ld_words, row_words;
    float *delta_out; int32_t *nnz_out; uint32_t *status;
    int cap;                       // staging capacity in entries
    uint32_t *zero_word;           // nullable: set to 0 by one thread of the grid
    int win;                       // columns of the gradient held in LDS at a time (multiple of 4; >= d: all of it)
    float *alpha_ws; int64_t ld_ws; // with several windows: M rows of workspace for the whole gradient, else null
    // sparsifier split over the identical blocks of a worker (beta_ws != null): each block sparsifies its slice into
    // row m of beta_ws and leaves the slice's largest magnitude and kept count; the quantization is a second launch
    float *beta_ws; float *part_max; int32_t *part_kept;
};

__global__ __launch_bounds__(kCsrThreads) void csr_worker_kernel(const CsrWorkerArgs a)
{
    extern __shared__ __align__(16) float lds[];
    __shared__ RowMeta meta;
    __shared__ float sh_y[kCsrMaxRows];
    __shared__ uint32_t su[kCsrWaves];
    __shared__ int si[kCsrWaves];
    __shared__ double sd[kCsrWaves];
    __shared__ int sh_ctl[2];
    const int64_t d = a.A.d;
    const int win = a.win;                                     // columns per window, a multiple of 4
    float *alpha = lds;                                        // the window of the gradient being built
    int2 *stage = reinterpret_cast<int2 *>(lds + win);

    const int m = blockIdx.x;
    const ModelMsg msg{a.xq, a.b_x == 32 ? 1.0f : a.delta_x[0], a.b_x};
    const int slice = blockIdx.y, nslices = gridDim.y;       // identical copies of the worker; they share only the tail
    if (a.zero_word && blockIdx.x == 0 && slice == 0 && threadIdx.x == 0) *a.zero_word = 0u;
    float *alpha_row = a.alpha_ws ? a.alpha_ws + static_cast<int64_t>(m) * a.ld_ws : nullptr;   // only with several windows

    const float inv_B = 1.0f / static_cast<float>(a.B);      // the mean over the mini-batch, as one multiplication per row
    const bool have_z = a.z_snap != nullptr;
    // the model value and the snapshot at column c: the field of column c starts at bit c*b_x of the message and
    // may continue in the next word; both words and the snapshot value are requested without any condition
    struct Gather { uint32_t w0, w1; float xs; };
    auto vec_req = [&](int c) {
        const int w = (c * a.b_x) >> 5, last = static_cast<int>(a.model_last_word);   // (fewer than 2^20 words)
        return Gather{a.xq[w], a.xq[w + 1 < last ? w + 1 : last], a.x_snap[c]};
    };
    auto vec_val = [&](const Gather &g, int c) {
        const uint32_t bits = __funnelshift_r(g.w0, g.w1, static_cast<unsigned>(c * a.b_x) & 31u);
        const float q = a.b_x == 32 ? __uint_as_float(bits)
                                    : msg.delta_x * static_cast<float>(sext_field(bits, 0, static_cast<unsigned>(a.b_x)));
        return make_float2(q - g.xs, g.xs);
    };
    auto coef_of = [&](int r, float dz, float zs) {
        if (meta.row[r] < 0) return 0.0f;
        if (have_z) zs = meta.z[r];
        return vr_slope_diff(sh_y[r], zs, dz) * inv_B;
    };
    // the rows of one pass: which sample, where its entries start, how many, its label and cached margin
    struct RowInfo { int row; int64_t start; int len; float y, z; };
    auto row_info = [&](int r0) {
        RowInfo ri{-1, 0, 0, 1.0f, 0.0f};
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
            if (static_cast<uint64_t>(i) < static_cast<uint64_t>(a.A.n)) {
                ri.row = static_cast<int>(i);
                ri.start = a.A.indptr[i];
                ri.len = static_cast<int>(a.A.indptr[i + 1] - ri.start);
                ri.y = a.A.y[i];
                ri.z = have_z ? a.z_snap[i] : 0.0f;
            }
        }
        return ri;
    };
    // the first pass's rows are requested before the window is initialised: both sets of loads are in flight together
    const RowInfo first_rows = row_info(0);
    for (int64_t c0 = 0; c0 < d; c0 += win) {
        const int64_t c1 = min(d, c0 + win);
        // the window starts as the dense part  l2*(q - snapshot); four coordinates per thread and step
        for (int64_t j = c0 + 4ll * threadIdx.x; j < c1; j += 4ll * kCsrThreads) {
            float *dst = alpha + (j - c0);
            if (j + 3 < d && a.b_x == 8) {
                const float4 xs = *reinterpret_cast<const float4 *>(a.x_snap + j);
                const uint32_t w = a.xq[j >> 2];
                dst[0] = a.l2 * (msg.delta_x * static_cast<float>(sext_field(w, 0, 8)) - xs.x);
                dst[1] = a.l2 * (msg.delta_x * static_cast<float>(sext_field(w, 8, 8)) - xs.y);
                dst[2] = a.l2 * (msg.delta_x * static_cast<float>(sext_field(w, 16, 8)) - xs.z);
                dst[3] = a.l2 * (msg.delta_x * static_cast<float>(sext_field(w, 24, 8)) - xs.w);
            } else {
                for (int64_t e = j; e < min(d, j + 4); ++e) dst[e - j] = a.l2 * (model_value(msg, e) - a.x_snap[e]);
            }
        }
        for (int r0 = 0; r0 < a.B; r0 += kCsrMaxRows) {                     // passes of at most kCsrMaxRows rows
            const int nrows = min(kCsrMaxRows, a.B - r0);
            const RowInfo ri = r0 == 0 ? first_rows : row_info(r0);
            if (static_cast<int>(threadIdx.x) < nrows) {
                meta.row[threadIdx.x] = ri.row;
                meta.start[threadIdx.x] = ri.start;
                meta.len[threadIdx.x] = ri.len;
                sh_y[threadIdx.x] = ri.y;
                meta.z[threadIdx.x] = ri.z;
            }
            csr_prefix_lengths(meta, nrows);
            if (have_z)
                csr_process_rows<false>(a.A, meta, nrows, alpha, static_cast<int>(c0), static_cast<int>(c1), stage, a.cap,
                                        sh_ctl, vec_req, vec_val, coef_of);
            else
                csr_process_rows<true>(a.A, meta, nrows, alpha, static_cast<int>(c0), static_cast<int>(c1), stage, a.cap,
                                       sh_ctl, vec_req, vec_val, coef_of);
        }
        if (alpha_row) {                                       // several windows: the finished one goes to memory
            for (int64_t j = c0 + threadIdx.x; j < c1; j += kCsrThreads) alpha_row[j] = alpha[j - c0];
            __syncthreads();
        }
    }
    // the whole gradient: in LDS when it fits in one window, else in this worker's workspace row (the block's own
    // writes, visible to all its threads after the barrier above)
    float *av = alpha_row ? alpha_row : alpha;

    // 4. outputs
    if (a.alpha_out && slice == 0)
        for (int64_t j = threadIdx.x; j < d; j += kCsrThreads) a.alpha_out[static_cast<int64_t>(m) * a.ld + j] = av[j];
    if (!a.packed) {
        uint32_t vmax = 0;
        double s1 = 0.0;
        for (int64_t j = threadIdx.x; j < d; j += kCsrThreads) {
            vmax = max(vmax, abs_bits(av[j]));
            s1 += static_cast<double>(fabsf(av[j]));
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
    if (a.beta_ws) {
        sparsify_slice_from_lds(av, d, key, slice, nslices, a.beta_ws + static_cast<int64_t>(m) * a.ld_ws,
                                a.part_max + static_cast<int64_t>(m) * nslices + slice,
                                a.part_kept + static_cast<int64_t>(m) * nslices + slice, su, si);
        return;
    }
    const WorkerOut out{a.packed + static_cast<int64_t>(m) * a.ld_words, a.row_words, a.delta_out + m,
                        a.nnz_out ? a.nnz_out + m : nullptr, a.status};
    switch (a.b) {
    case 2: worker_tail_from_lds<2>(av, d, a.sparsify != 0, a.b, key, out, su, si, slice, nslices); break;
    case 4: worker_tail_from_lds<4>(av, d, a.sparsify != 0, a.b, key, out, su, si, slice, nslices); break;
    case 32: worker_tail_from_lds<32>(av, d, a.sparsify != 0, a.b, key, out, su, si, slice, nslices); break;
    default: worker_tail_from_lds<8>(av, d, a.sparsify != 0, a.b, key, out, su, si, slice, nslices); break;
    }
}

// ------------------------------------------------------------------ epoch prologue
// grid (P): block p owns rows [p*per, (p+1)*per), processed kCsrMaxRows at a time.
__global__ __launch_bounds__(kCsrThreads) void csr_full_partial_kernel(
    const CsrView A, const float *__restrict__ x, float *__restrict__ z_out, float *__restrict__ partial, int64_t ldp,
    double *__restrict__ loss_partial, int cap, int win)
{
    extern __shared__ __align__(16) float lds[];
    __shared__ RowMeta meta;
    __shared__ double sh_loss[kCsrWaves];
    __shared__ int sh_ctl[2];
    float *acc = lds;                                    // the window [c0, c1) of this block's partial sum
    int2 *stage = reinterpret_cast<int2 *>(lds + win);
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int64_t per = (A.n + gridDim.x - 1) / gridDim.x;
    const int64_t i0 = blockIdx.x * per, i1 = min(A.n, i0 + per);
    const float fn = static_cast<float>(A.n);
    double loss = 0.0;                                   // the lanes that evaluate row scalars add to theirs
    float *mine = partial + static_cast<int64_t>(blockIdx.x) * ldp;
    for (int64_t c0 = 0; c0 < ldp; c0 += win) {          // one window when the vector fits in LDS
        const int64_t c1 = min(ldp, c0 + win);
        for (int64_t j = threadIdx.x; j < c1 - c0; j += kCsrThreads) acc[j] = 0.0f;
        const bool first = c0 == 0;                      // margins and losses are recorded once
        for (int64_t ib = i0; ib < i1; ib += kCsrMaxRows) {
            const int nrows = static_cast<int>(min<int64_t>(kCsrMaxRows, i1 - ib));
            if (static_cast<int>(threadIdx.x) < nrows) {
                const int64_t i = ib + threadIdx.x;
                const int64_t s = A.indptr[i];
                meta.row[threadIdx.x] = static_cast<int>(i);
                meta.start[threadIdx.x] = s;
                meta.len[threadIdx.x] = static_cast<int>(A.indptr[i + 1] - s);
            }
            csr_prefix_lengths(meta, nrows);
            const int64_t ib_now = ib;
            auto vec_req = [&](int c) { return x[c]; };
            auto vec_val = [&](float xc, int) { return make_float2(xc, 0.0f); };
            auto coef_of = [&](int r, float z, float) {
                const int64_t i = ib_now + r;
                const float y = A.y[i];
                if (first) {
                    if (z_out) z_out[i] = z;
                    loss += static_cast<double>(logistic_loss(y * z));
                }
                return logistic_slope(y, z) / fn;
            };
            csr_process_rows<false>(A, meta, nrows, acc, static_cast<int>(c0), static_cast<int>(min(A.d, c1)), stage, cap,
                                    sh_ctl, vec_req, vec_val, coef_of);
        }
        __syncthreads();
        for (int64_t j = c0 + threadIdx.x; j < c1; j += kCsrThreads) mine[j] = acc[j - c0];
        __syncthreads();
    }
    loss = wave_sum_f64(loss);
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
int launch_quantize_pack_parts(const float *v, int64_t d, int64_t M, int64_t ld, int b, int field, const float *absmax,
                               int parts, const int32_t *count_parts, int32_t *count_out, const StreamKey &key,
                               uint32_t worker0, uint32_t *packed, int64_t ld_words, float *delta_out, uint32_t *status,
                               hipStream_t st);

// ------------------------------------------------------------------ host side
static int64_t pad4(int64_t d) { return (d + 3) / 4 * 4; }

// LDS plan for a d-vector plus the staging buffer.  When both fit, the vector is one window; otherwise it is built
// in several equal windows (multiples of 4 columns) that leave room for at least kMinStage staged entries.
// Columns carry the row number in the bits above kColBits while staged, hence the limit on d.
constexpr int64_t kMinStage = 4096;
struct CsrPlan {
    int win;        // columns per window
    int cap;        // staged (column, value) entries
    int nwin;
};

static bool csr_plan(int64_t d, CsrPlan &p)
{
    if (d >= (1ll << kColBits)) return false;      // column 2^20 - 1 marks the end of the staged entries in the scatter
    const int64_t budget = kLdsBudget - kCsrFixedLds;                     // bytes for window + staging
    int64_t nwin = 1;
    if (pad4(d) * 4 + 8 * 512 > budget) nwin = ceil_div(pad4(d) * 4, budget - 8 * kMinStage);
    const int64_t win = pad4(ceil_div(pad4(d), nwin));
    int64_t cap = (budget - win * 4) / 8;
    if (cap > 8192) cap = 8192;
    p.win = static_cast<int>(win);
    p.cap = static_cast<int>(cap);
    p.nwin = static_cast<int>(ceil_div(pad4(d), win));
    return true;
}

static int64_t csr_full_splits(int64_t n)
{
    int64_t P = ceil_div(n, 64);
    if (P > 256) P = 256;
    if (P < 1) P = 1;
    return P;
}

constexpr int kMaxSlices = kMaxParts;       // identical blocks per worker that share the tail of a worker step

int64_t csr_workspace_bytes(int32_t op, const dq_problem *prob, int64_t M, int64_t)
{
    CsrPlan plan;
    if (!csr_plan(prob->d, plan)) return DQ_ERR_UNSUPPORTED;
    if (op == DQ_OP_FULL_GRAD) {
        const int64_t P = csr_full_splits(prob->n);
        return P * pad4(prob->d) * 4 + P * 8;
    }
    // a row per worker: the whole gradient when it does not fit in LDS, else the sparsified gradient when the
    // sparsifier is split over several blocks per worker (see csr_worker); then 8 values + 8 counts per worker
    return M * pad4(prob->d) * 4 + M * kMaxSlices * 8;
}

// Kernels that use more than 64 KB of dynamic LDS must be told so once (the limit is raised to the budget).
template <typename K>
static int allow_big_lds(K kernel, std::once_flag &once, hipError_t &once_rc)
{
    std::call_once(once, [&] {
        once_rc = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                      static_cast<int>(kLdsBudget - kCsrFixedLds));
    });
    DQ_HIP_TRY(once_rc);
    return DQ_OK;
}

int csr_full_grad(const dq_problem *prob, const float *x, float *g_out, float *z_out, double *obj_out, void *ws,
                  int64_t ws_bytes, hipStream_t st)
{
    const int64_t d = prob->d, n = prob->n;
    CsrPlan plan;
    if (!csr_plan(d, plan)) return DQ_ERR_UNSUPPORTED;
    if (ws_bytes < csr_workspace_bytes(DQ_OP_FULL_GRAD, prob, 0, 0) || !ws) return DQ_ERR_WORKSPACE;
    const int64_t ldp = pad4(d);
    const int P = static_cast<int>(csr_full_splits(n));
    float *partial = static_cast<float *>(ws);
    double *loss_partial = reinterpret_cast<double *>(partial + static_cast<int64_t>(P) * ldp);
    const size_t lds = static_cast<size_t>(plan.win) * 4 + static_cast<size_t>(plan.cap) * 8;
    static std::once_flag attr_once;
    static hipError_t attr_rc = hipSuccess;
    int rc = allow_big_lds(csr_full_partial_kernel, attr_once, attr_rc);
    if (rc != DQ_OK) return rc;
    const CsrView A{prob->indptr, prob->indices, prob->values, prob->y, n, d};
    csr_full_partial_kernel<<<dim3(P), dim3(kCsrThreads), lds, st>>>(A, x, z_out, partial, ldp, loss_partial, plan.cap, plan.win);
    DQ_LAUNCH_CHECK();
    return launch_full_finish(partial, P, ldp, n, d, x, prob->l2, prob->l1, loss_partial, g_out, obj_out, st);
}

int csr_worker(const dq_problem *prob, const WorkerArgs &a, hipStream_t st)
{
    const int64_t d = prob->d;
    CsrPlan plan;
    if (!csr_plan(d, plan)) return DQ_ERR_UNSUPPORTED;
    const int64_t row_words = a.packed ? (a.b == 32 ? d : packed_words(d, a.b)) : 0;
    if (a.model_is_snapshot) return launch_worker_zero(a, d, row_words, st);
    if (plan.nwin > 1 && (!a.ws || a.ws_bytes < a.M * pad4(d) * 4)) return DQ_ERR_WORKSPACE;
    CsrWorkerArgs k{};
    k.A = CsrView{prob->indptr, prob->indices, prob->values, prob->y, prob->n, d};
    k.idx = a.idx; k.B = static_cast<int>(a.B);
    k.xq = a.xq; k.delta_x = a.delta_x; k.b_x = a.b_x; k.x_snap = a.x_snap; k.z_snap = a.z_snap; k.l2 = prob->l2;
    k.model_last_word = (a.b_x == 32 ? prob->d : packed_words(prob->d, a.b_x)) - 1;
    k.alpha_out = a.alpha_out; k.ld = a.ld; k.absmax_out = a.absmax_out; k.l1norm_out = a.l1norm_out;
    k.sparsify = a.sparsify; k.b = a.b;
    k.key = StreamKey{static_cast<uint32_t>(a.seed), static_cast<uint32_t>(a.seed >> 32), a.iter, 0u, DQ_TAG_GRAD};
    k.worker0 = a.worker0;
    k.packed = a.packed; k.ld_words = a.ld_words; k.row_words = row_words;
    k.delta_out = a.delta_out; k.nnz_out = a.nnz_out; k.status = a.status; k.zero_word = a.zero_word;
    k.cap = plan.cap; k.win = plan.win;
    k.alpha_ws = plan.nwin > 1 ? static_cast<float *>(a.ws) : nullptr; k.ld_ws = pad4(d);
    const size_t lds = static_cast<size_t>(plan.win) * 4 + static_cast<size_t>(plan.cap) * 8;
    static std::once_flag attr_once;
    static hipError_t attr_rc = hipSuccess;
    int rc = allow_big_lds(csr_worker_kernel, attr_once, attr_rc);
    if (rc != DQ_OK) return rc;
    // Few workers leave most compute units idle while each block spends a third of its time on the Philox rounds of
    // the final quantization: then several identical blocks per worker share that part (not when the nonzero count is
    // wanted and would need a sum across blocks, nor when the gradient lives in the per-worker workspace row).
    const bool count_ok = !a.nnz_out || (a.sparsify && a.b >= 4);      // after the sparsifier: count = kept coordinates
    unsigned slices = 1;
    if (a.packed && count_ok && plan.nwin == 1 && a.b != 32 && d >= 4096 && a.M * 4 <= 128) slices = a.M * 8 <= 128 ? 8 : 4;
    // After the sparsifier the scale is ||beta||_inf, which needs every coordinate's random decision: sharing only the
    // quantization would leave each identical block a whole Philox-and-two-divisions pass over the vector (9 of the
    // 33 us of the step at d = 20958).  With workspace for a row per worker each block sparsifies its own slice into
    // memory instead and the quantization becomes a second launch that takes the scale from the slices' maxima.
    const bool split_sparsifier = slices > 1 && a.sparsify && a.ws &&
                                  a.ws_bytes >= csr_workspace_bytes(DQ_OP_VR_GRAD, prob, a.M, a.B);
    if (split_sparsifier) {
        k.beta_ws = static_cast<float *>(a.ws);
        k.part_max = k.beta_ws + a.M * k.ld_ws;
        k.part_kept = reinterpret_cast<int32_t *>(k.part_max + a.M * kMaxSlices);
    }
    if (a.ev_start && a.ev_stop)      // the kernel's own start and end times go to the two events
        hipExtLaunchKernelGGL(csr_worker_kernel, dim3(static_cast<unsigned>(a.M), slices), dim3(kCsrThreads),
                              static_cast<uint32_t>(lds), st, a.ev_start, a.ev_stop, 0u, k);
    else
        csr_worker_kernel<<<dim3(static_cast<unsigned>(a.M), slices), dim3(kCsrThreads), lds, st>>>(k);
    DQ_LAUNCH_CHECK();
    if (a.deferred) *a.deferred = SparsifiedParts{nullptr, 0, nullptr, nullptr, 0};
    if (split_sparsifier && a.deferred) {             // the master quantizes while it aggregates
        *a.deferred = SparsifiedParts{k.beta_ws, k.ld_ws, k.part_max, k.part_kept, static_cast<int>(slices)};
        return DQ_OK;
    }
    if (split_sparsifier)
        return launch_quantize_pack_parts(k.beta_ws, d, a.M, k.ld_ws, a.b, a.b, k.part_max, static_cast<int>(slices),
                                          a.nnz_out ? k.part_kept : nullptr, a.nnz_out, k.key, a.worker0, a.packed,
                                          a.ld_words, a.delta_out, a.status, st);
    return DQ_OK;
}

}  // namespace dq
