// CSR-feature gradient kernels: epoch prologue (full gradient, Alg. 1) and the worker step
// (Alg. 1 worker (i)-(ii), Alg. 2 worker (i)-(iii)) for bag-of-words shaped data.
//
// A mini-batch of such rows touches a few thousand entries, far too few to be bandwidth
// bound; what matters is that one launch does the whole worker step and that the result
// is reproducible.  One block of 1024 threads owns a worker: the gradient alpha (d floats)
// lives in LDS for the whole step and never goes to memory.
//   1. stage: the (column, value) pairs of the mini-batch rows are copied into LDS as one flat run, spread evenly
//      over the threads whatever the row lengths (the row of an entry comes from a table of the rows at every 64th
//      entry plus the starts of the next few rows, and is kept in the bits above the column); the thread that copies an
//      entry also gathers the model and the snapshot at its column and leaves value * operand next to it -- two
//      trips to memory for the whole mini-batch, however long its longest row;
//   2. margins: one wavefront per row, four rows in flight, adds up the products of its row from LDS; one lane per
//      row forms its coefficient;
//   3. scatter: every thread adds coefficient*value of the entries it staged to the columns' accumulators in LDS --
//      integer atomic adds of fixed-point terms (see FixedAcc), whose sum does not depend on the order of the adds:
//      the result is reproducible whichever wavefront gets there first;
//   4. the accumulators become float32 in place, the dense part l2*(q - snapshot) added, and the tail of the worker
//      step (sparsify, scale, quantize, pack) runs from LDS.
// Between the rounds of one dq_run_rounds call, everything of step 1 that does not depend on the model (which rows,
// their extents and labels, the flat run itself) is laid out one round ahead by an extra block per worker of the
// previous round's launch (see kPrepInts).
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
constexpr int kColBits = 20;                     // staged entries carry column | row << kColBits
constexpr int kColMask = (1 << kColBits) - 1;
constexpr int kFlight = 4;                       // rows a wavefront reduces at the same time
constexpr int kStageFlight = 4;                  // entries a thread stages at the same time (worker step)
constexpr int kFullFlight = 8;                   // ... in the full gradient, whose groups of rows fill the staging buffer
constexpr int kFlushRows = 1024;                 // rows between two flushes of the fixed-point sums (full gradient)
constexpr int kCsrMaxRows = 256;                 // rows a block handles per pass (LDS metadata)
constexpr int kMaxStage = 8192;                  // most entries the staging buffer is given
constexpr int kChunkSlots = kMaxStage / kWave;   // see RowMeta::chunk_row
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
    float z[kCsrMaxRows];        // cached margin at the snapshot (worker step); the label (full gradient)
    int chunk_row[kChunkSlots];  // the row that holds entry 64 c of the rows' concatenation, for the entries below 64 * kChunkSlots
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
    // every row leaves its number at the multiples of 64 that it holds (an empty row holds none)
    if (static_cast<int>(threadIdx.x) < nrows) {
        const int lo = meta.pre[threadIdx.x], hi = meta.pre[threadIdx.x + 1];
        for (int c = (lo + kWave - 1) / kWave; c * kWave < hi && c < kChunkSlots; ++c) meta.chunk_row[c] = threadIdx.x;
    }
    __syncthreads();
}

// The staging buffer in LDS: `cap` entries of (column | row << kColBits, value), and per entry value * first operand
// (prod_a) and, for callers that need a second sum, value * second operand (prod_b, else null).
struct CsrStage {
    int2 *entry;
    float *prod_a, *prod_b;
    int cap;
};

__device__ __forceinline__ CsrStage csr_stage_in(float *after_window, int cap, bool second)
{
    CsrStage sg;
    sg.entry = reinterpret_cast<int2 *>(after_window);
    sg.prod_a = after_window + 2 * static_cast<int64_t>(cap);
    sg.prod_b = second ? sg.prod_a + cap : nullptr;
    sg.cap = cap;
    return sg;
}

// ---- fixed-point accumulation of the scattered terms
// LDS float atomic adds take about three cycles per lane on this part (measured: the 3328 adds of a 64-row
// mini-batch take 4.3-4.9 us however they are spread over wavefronts), integer ones a fifteenth of that, and an
// integer sum does not depend on the order of its terms.  So coefficient * value is accumulated in int32 as a multiple
// of the unit 2^-k, with k from a bound on the magnitude any column's sum can have reached: the sum over the groups
// of rows added so far of (sum of the group's |coefficient|) * (the group's largest |value|), times 2^k, stays
// <= 2^30, so a sum cannot overflow.  The coefficients of the variance-reduced gradient shrink with the distance
// between model and snapshot, and the unit shrinks with them.  A term is rounded to the nearest unit, i.e. within
// 2^-31 of that bound -- float32 addition loses up to 2^-25 of the partial sum per term, which is coarser for sums of
// the bound's order and finer for much smaller ones; either way far inside the tolerance of the gradient.  When a
// further group of rows raises the bound past a power of two, the window is first rescaled to the coarser unit.
// A value or coefficient that is not finite poisons the block: its result is NaN.
struct FixedAcc {
    float bound;            // see above; 0 while nothing but zeros has been added
    int k;                  // the unit is 2^-k
};

// k with bound * 2^k <= 2^30 (clamped so that 2^k and 2^-k are normal numbers)
__device__ __forceinline__ int fixed_exponent(float bound)
{
    int e = 0;
    (void)frexpf(bound, &e);                 // bound = m * 2^e with 0.5 <= m < 1; e = 0 for bound = 0
    return max(-100, min(100, 30 - e));
}

// A group of rows whose terms are bounded by group_bound (in sum, per column) is about to be added to acc[0..ncols):
// coarsen the unit if need be.  Every thread calls it with the same arguments, after a barrier that follows all
// earlier adds; a rescaled window is published by the barrier inside.
__device__ __forceinline__ void fixed_admit(FixedAcc &fx, float group_bound, int *acc, int ncols, int *poison)
{
    if (!(group_bound <= FLT_MAX)) {         // Inf or NaN among the values or coefficients
        if (threadIdx.x == 0) *poison = 1;
        return;
    }
    const float bound = fx.bound + group_bound;
    const int k_new = fixed_exponent(bound);
    if (fx.bound > 0.0f && k_new < fx.k) {
        const int sh = fx.k - k_new;
        for (int j = threadIdx.x; j < ncols; j += kCsrThreads)
            acc[j] = sh >= 31 ? 0 : (acc[j] + (1 << (sh - 1))) >> sh;       // nearest multiple of the new unit
        __syncthreads();
    }
    if (!(fx.bound > 0.0f) || k_new < fx.k) fx.k = k_new;
    fx.bound = bound;
}

// sum of |coef[r0..r1)| (at most kCsrMaxRows of them), the same value in every thread of the block
__device__ __forceinline__ float coef_abs_sum(const float *coef, int r0, int r1)
{
    const int lane = threadIdx.x & (kWave - 1);
    float t = 0.0f;
#pragma unroll
    for (int u = 0; u < kCsrMaxRows / kWave; ++u) {
        const int r = r0 + lane + kWave * u;
        const float c = coef[min(r, kCsrMaxRows - 1)];
        t += r < r1 ? fabsf(c) : 0.0f;
    }
    return wave_sum_f32(t);
}

__device__ __forceinline__ int fixed_term(float coef, float value, float two_k)
{
    return __float2int_rn(coef * value * two_k);          // (the scaling by a power of two is exact)
}

// The row of staged position p: the last r in [g0, g1) with pre[r] - base <= p, by halving steps of fixed number.
__device__ __forceinline__ int csr_row_of(const RowMeta &meta, int g0, int g1, int base, int p)
{
    int r = g0;
#pragma unroll
    for (int step = kCsrMaxRows / 2; step >= 1; step >>= 1) {
        const int cand = r + step;
        const int first = meta.pre[min(cand, g1)] - base;
        r = (cand < g1 && first <= p) ? cand : r;
    }
    return r;
}

// The same for the 64 consecutive positions P + lane of a wavefront when the group starts at row 0 (base = 0) and P is a
// multiple of 64, from the table of the rows at the multiples of 64 (RowMeta::chunk_row): the row of P is read there,
// and a lane's row lies as many rows further as start at or before its position among the next kNextRows (their
// starts are the same few LDS words for the whole wavefront).  More rows than that starting inside the chunk (short
// rows) is left to csr_row_of.  `p` = min(P + lane, total - 1).
constexpr int kNextRows = 4;
__device__ __forceinline__ int csr_row_in_chunk(const RowMeta &meta, int g1, int P, int p)
{
    const int r0 = meta.chunk_row[P >> 6];
    const int beyond = r0 + kNextRows + 1;
    if (beyond < g1 && meta.pre[min(beyond, kCsrMaxRows)] <= P + kWave - 1)       // (the same for all lanes)
        return csr_row_of(meta, 0, g1, 0, p);
    int r = r0;
#pragma unroll
    for (int j = 1; j <= kNextRows; ++j) {
        const int rj = r0 + j;
        const int first = meta.pre[min(rj, kCsrMaxRows)];
        r += (rj < g1 && first <= p) ? 1 : 0;
    }
    return r;
}

// Where the entry of staged position P + lane lies in the matrix, and its row number shifted above the column bits.
// A wavefront whose 64 positions all lie past the end (P >= total) gets `inside`, the source of a position that
// does exist, so that no load sits behind a test.
__device__ __forceinline__ int64_t csr_stage_source(const RowMeta &meta, int g0, int g1, int base, int total, int P,
                                                    int lane, int64_t inside, int &tag)
{
    const int p = min(P + lane, total - 1);
    const int r = P >= total ? g1 - 1
                  : g0 == 0  ? csr_row_in_chunk(meta, g1, P, p)
                             : csr_row_of(meta, g0, g1, base, p);
    tag = r << kColBits;
    return P < total ? meta.start[r] + (p - (meta.pre[r] - base)) : inside;
}

// Margins and scatter for the staged group of rows [g0, g1) (`total` entries; base = pre[g0]); vmax = the largest
// |value| among the entries this thread staged, as bits.
template <bool SECOND, typename CoefFn>
__device__ __forceinline__ void csr_reduce_group(RowMeta &meta, int g0, int g1, int base, int total, uint32_t vmax,
                                                 int *acc, int c0, int c1, const CsrStage &sg, FixedAcc &fx, uint32_t *su,
                                                 int *poison, CoefFn coef_of)
{
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int2 *stage = sg.entry;
    vmax = block_max_u32(vmax, su);            // (its barriers also publish the staged entries)
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
        for (int k = lane; k < maxlen; k += kWave) {           // (maxlen > 0 implies total > 0)
            float pa[kFlight], pb[kFlight];
#pragma unroll
            for (int u = 0; u < kFlight; ++u) {
                const int at = min(off[u] + k, total - 1);
                pa[u] = sg.prod_a[at];
                pb[u] = SECOND ? sg.prod_b[at] : 0.0f;
            }
#pragma unroll
            for (int u = 0; u < kFlight; ++u) {
                sa[u] += k < len[u] ? pa[u] : 0.0f;
                if (SECOND) sb[u] += k < len[u] ? pb[u] : 0.0f;
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
        if (lane < kFlight && rl < g1) {
            const float cf = coef_of(rl, mine_a, mine_b);
            meta.coef[rl] = cf;
        }
    }
    __syncthreads();
    // ---- scatter: fixed-point terms, integer atomic adds
    fixed_admit(fx, coef_abs_sum(meta.coef, g0, g1) * __uint_as_float(vmax), acc, c1 - c0, poison);
    const float two_k = ldexpf(1.0f, fx.k);
    for (int p0 = threadIdx.x; p0 < total; p0 += kStageFlight * kCsrThreads) {
        int2 e[kStageFlight];
        float cf[kStageFlight];
#pragma unroll
        for (int u = 0; u < kStageFlight; ++u) e[u] = stage[min(p0 + u * kCsrThreads, total - 1)];
#pragma unroll
        for (int u = 0; u < kStageFlight; ++u) cf[u] = meta.coef[(e[u].x >> kColBits) & (kCsrMaxRows - 1)];
#pragma unroll
        for (int u = 0; u < kStageFlight; ++u) {
            const int c = e[u].x & kColMask;
            if (p0 + u * kCsrThreads < total && c >= c0 && c < c1)
                atomicAdd(&acc[c - c0], fixed_term(cf[u], __int_as_float(e[u].y), two_k));
        }
    }
}

// Stage, margins and scatter (the first three phases of the file header) for rows [0, nrows) described by `meta`,
// accumulating into acc (LDS, fixed point, see FixedAcc).
// The rows are taken in groups that fit the staging buffer:
//   stage  : the group's (column, value) pairs are copied to LDS as one flat run, kStageFlight entries per thread in
//            flight, the row number packed above the column; vec_val(vec_req(c), c) returns the {first, second}
//            operands of column c gathered from memory -- vec_req only requests (no branch, no use of what it
//            loads), so a thread's gathers wait for memory once -- and value * operand is staged with the entry;
//   margins: one wavefront per row (kFlight rows in flight) adds up its row's products; lane u hands the sums of its
//            u-th row to coef_of(row, first_sum, second_sum), which returns the row's coefficient;
//   scatter: every thread adds coefficient*value of its share of the staged entries to acc[column - c0].
// A row longer than `cap` is handled alone, straight from memory.
// Only the columns of the window [c0, c1) are accumulated: a vector too long for LDS is built one window at a
// time (the caller repeats the call per window; margins are recomputed).
// FLIGHT: entries a thread stages at the same time.
template <bool SECOND, int FLIGHT, typename VecReq, typename VecVal, typename CoefFn>
__device__ __forceinline__ void csr_process_rows(const CsrView &A, RowMeta &meta, int nrows, int *acc, int c0, int c1,
                                                 const CsrStage &sg, FixedAcc &fx, uint32_t *su, int *poison,
                                                 VecReq vec_req, VecVal vec_val, CoefFn coef_of)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int cap = sg.cap;
    int2 *stage = sg.entry;
    int g0 = 0;
    while (g0 < nrows) {
        // group of consecutive rows that fits the staging buffer: rows g0..g1-1 with
        // pre[g1] - pre[g0] <= cap; a first row longer than cap is taken alone, unstaged
        const int base = meta.pre[g0];
        int g1 = nrows;
        bool direct = false;
        if (meta.pre[nrows] - base > cap) {            // (the same for every thread) not all remaining rows fit
            // the first row whose end lies past the buffer, by halving (every thread finds the same one)
            int lo = g0, hi = nrows - 1;
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                if (meta.pre[mid + 1] - base > cap) hi = mid;
                else lo = mid + 1;
            }
            g1 = max(lo, g0 + 1);
            direct = meta.len[g0] > cap;
        }
        if (!direct) {
            // ---- stage: flat copy of the group's entries with their products
            const int total = meta.pre[g1] - base;
            uint32_t vmax = 0;
            // (the loop bound is the same for a whole wavefront: its lanes find their rows together)
            for (int p0 = threadIdx.x; p0 - lane < total; p0 += FLIGHT * kCsrThreads) {
                int64_t src[FLIGHT];
                int tag[FLIGHT], col[FLIGHT];
                float val[FLIGHT];
#pragma unroll
                for (int u = 0; u < FLIGHT; ++u)     // (a position past the end repeats an entry and is not stored)
                    src[u] = csr_stage_source(meta, g0, g1, base, total, p0 - lane + u * kCsrThreads, lane, u ? src[0] : 0, tag[u]);
#pragma unroll
                for (int u = 0; u < FLIGHT; ++u) {
                    col[u] = A.indices[src[u]];
                    val[u] = A.values[src[u]];
                }
                decltype(vec_req(0)) raw[FLIGHT];
#pragma unroll
                for (int u = 0; u < FLIGHT; ++u) raw[u] = vec_req(col[u]);
#pragma unroll
                for (int u = 0; u < FLIGHT; ++u) {
                    const int p = p0 + u * kCsrThreads;
                    const float2 f = vec_val(raw[u], col[u]);
                    vmax = max(vmax, abs_bits(val[u]));
                    if (p < total) {
                        stage[p] = make_int2(col[u] | tag[u], __float_as_int(val[u]));
                        sg.prod_a[p] = val[u] * f.x;
                        if (SECOND) sg.prod_b[p] = val[u] * f.y;
                    }
                }
            }
            csr_reduce_group<SECOND>(meta, g0, g1, base, total, vmax, acc, c0, c1, sg, fx, su, poison, coef_of);
        } else {
            // ---- one very long row, straight from memory (every wavefront computes the same sums)
            const int64_t s = meta.start[g0];
            float a1 = 0.0f, b1 = 0.0f;
            uint32_t vmax = 0;
            for (int k = lane; k < meta.len[g0]; k += kWave) {
                const int ck = A.indices[s + k];
                const float2 f = vec_val(vec_req(ck), ck);
                const float v = A.values[s + k];
                vmax = max(vmax, abs_bits(v));
                a1 += v * f.x;
                if (SECOND) b1 += v * f.y;
            }
            a1 = wave_sum_f32(a1);
            if (SECOND) b1 = wave_sum_f32(b1);
            vmax = wave_max_u32(vmax);                 // (the same in every wavefront)
            __syncthreads();
            if (threadIdx.x == 0) meta.coef[g0] = coef_of(g0, a1, b1);
            __syncthreads();
            const float cf = meta.coef[g0];
            fixed_admit(fx, fabsf(cf) * __uint_as_float(vmax), acc, c1 - c0, poison);
            const float two_k = ldexpf(1.0f, fx.k);
            for (int k = threadIdx.x; k < meta.len[g0]; k += kCsrThreads) {
                const int c = A.indices[s + k];
                if (c >= c0 && c < c1) atomicAdd(&acc[c - c0], fixed_term(cf, A.values[s + k], two_k));
            }
        }
        __syncthreads();
        g0 = g1;
    }
}

// ---- a mini-batch prepared ahead of its round
// What a worker step does before it first needs the model -- drawing its rows (Alg. 1, worker step 2: the sample stream),
// reading their extents, labels and cached margins, the prefix sums, and the copy of the rows' entries into one flat run
// -- does not depend on the model.  Between two rounds of one dq_run_rounds call an extra block per worker of the
// worker launch does all of that for the NEXT round, on compute units the launch leaves idle, and leaves it in
// memory as kPrepInts(cap) 32-bit words per worker:
//   [0] 1 when the flat run is there (the batch fits the staging buffer), else 0   [1] number of entries
//   row[kCsrMaxRows] len[kCsrMaxRows] pre[kCsrMaxRows + 4] y[kCsrMaxRows] z[kCsrMaxRows]      (RowMeta's fields)
//   cap pairs (column | row << kColBits, value bits), the first [1] of them written
// The next round's blocks then start from one round trip to memory instead of a chain of five.
constexpr int kPrepRow = 4, kPrepLen = kPrepRow + kCsrMaxRows, kPrepPre = kPrepLen + kCsrMaxRows,
              kPrepY = kPrepPre + kCsrMaxRows + 4, kPrepZ = kPrepY + kCsrMaxRows, kPrepEntries = kPrepZ + kCsrMaxRows;
__host__ __device__ constexpr int64_t kPrepInts(int64_t cap) { return kPrepEntries + (2 * cap + 3) / 4 * 4; }

// Stage, margins and scatter for a prepared mini-batch: `entry` is its flat run of `total` <= cap entries, `first`
// what the caller has already loaded of it (positions threadIdx.x + u * kCsrThreads, clamped to the buffer), meta
// holds the rows.  The rest as csr_process_rows.
template <bool SECOND, typename VecReq, typename VecVal, typename CoefFn>
__device__ __forceinline__ void csr_process_prepared(const int2 *entry, const int2 (&first)[kStageFlight], int total,
                                                     RowMeta &meta, int nrows, int *acc, int c0, int c1, const CsrStage &sg,
                                                     FixedAcc &fx, uint32_t *su, int *poison, VecReq vec_req,
                                                     VecVal vec_val, CoefFn coef_of)
{
    uint32_t vmax = 0;
    const auto stage_batch = [&](int p0, const int2 (&e)[kStageFlight]) {
        int col[kStageFlight];
        decltype(vec_req(0)) raw[kStageFlight];
#pragma unroll
        for (int u = 0; u < kStageFlight; ++u) {
            // (past the end `first` holds whatever the buffer held: column 0 is gathered instead)
            col[u] = p0 + u * kCsrThreads < total ? e[u].x & kColMask : 0;
            raw[u] = vec_req(col[u]);
        }
#pragma unroll
        for (int u = 0; u < kStageFlight; ++u) {
            const int p = p0 + u * kCsrThreads;
            const float2 f = vec_val(raw[u], col[u]);
            const float val = __int_as_float(e[u].y);
            if (p < total) {
                vmax = max(vmax, abs_bits(val));
                sg.entry[p] = e[u];
                sg.prod_a[p] = val * f.x;
                if (SECOND) sg.prod_b[p] = val * f.y;
            }
        }
    };
    stage_batch(threadIdx.x, first);
    for (int p0 = threadIdx.x + kStageFlight * kCsrThreads; p0 < total; p0 += kStageFlight * kCsrThreads) {
        int2 e[kStageFlight];
#pragma unroll
        for (int u = 0; u < kStageFlight; ++u) e[u] = entry[min(p0 + u * kCsrThreads, total - 1)];
        stage_batch(p0, e);
    }
    csr_reduce_group<SECOND>(meta, 0, nrows, 0, total, vmax, acc, c0, c1, sg, fx, su, poison, coef_of);
    __syncthreads();
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
    const float *model_diff;       // nullable: (decoded model) - snapshot for every column, see WorkerArgs::model_diff
    // a mini-batch prepared ahead (see kPrepInts): prep_in (nullable) holds this round's, one block of prep_stride words
    // per worker; with prep_out the grid has one more block per worker (the last blockIdx.y), which prepares the round
    // whose streams carry next_iter into prep_out.  Both need B <= kCsrMaxRows, drawn rows (idx == null) and win >= d.
    const int32_t *prep_in;
    int32_t *prep_out;
    int64_t prep_stride;
    uint32_t next_iter;
};

// DIFF: the model comes as a.model_diff (one float per column) instead of the message and the snapshot.
// COMMON: the gradient fits in LDS as one window, the mini-batch in one pass of rows (B <= kCsrMaxRows), and the
// margins at the snapshot are cached (z_snap given) -- the kernel is then straight-line code with one set of the
// row-processing routines, which leaves the compiler far fewer values to keep alive across its phases.
template <bool DIFF, bool COMMON>
__global__ __launch_bounds__(kCsrThreads) void csr_worker_kernel(const CsrWorkerArgs a)
{
    touch_kernel_arguments<sizeof(CsrWorkerArgs)>();
    extern __shared__ __align__(16) float lds[];
    __shared__ RowMeta meta;
    __shared__ float sh_y[kCsrMaxRows];
    __shared__ uint32_t su[kCsrWaves];
    __shared__ int si[kCsrWaves];
    __shared__ double sd[kCsrWaves];
    __shared__ int sh_poison;
    const int64_t d = a.A.d;
    const int win = a.win;                                     // columns per window, a multiple of 4
    float *alpha = lds;                                        // the window of the gradient being built: fixed-point sums
    int *acc = reinterpret_cast<int *>(lds);                   // while the rows are added, float32 afterwards
    if (threadIdx.x == 0) sh_poison = 0;                       // (published by the barriers of the first row pass)
    const CsrStage sg = csr_stage_in(lds + win, a.cap, !COMMON && a.z_snap == nullptr);

    const int m = blockIdx.x;
    const ModelMsg msg{a.xq, a.b_x == 32 ? 1.0f : a.delta_x[0], a.b_x};
    // identical copies of the worker; they share only the tail (a last one more prepares the next round instead)
    const int slice = blockIdx.y, nslices = static_cast<int>(gridDim.y) - (a.prep_out ? 1 : 0);
    if (a.zero_word && blockIdx.x == 0 && slice == 0 && threadIdx.x == 0) *a.zero_word = 0u;
    float *alpha_row = (!COMMON && a.alpha_ws) ? a.alpha_ws + static_cast<int64_t>(m) * a.ld_ws : nullptr;   // only with several windows

    const float inv_B = 1.0f / static_cast<float>(a.B);      // the mean over the mini-batch, as one multiplication per row
    const bool have_z = COMMON || a.z_snap != nullptr;
    uint32_t seen_max = 0;                                     // largest magnitude among the coordinates this thread finishes
    // the model value and the snapshot at column c: the field of column c starts at bit c*b_x of the message and
    // may continue in the next word; both words and the snapshot value are requested without any condition
    struct Gather { uint32_t w0, w1; float xs, diff; };
    const bool straddles = (32 % a.b_x) != 0;                 // (the same for every thread) else a field lies in one word
    auto vec_req = [&](int c) {
        if constexpr (DIFF) {
            return Gather{0u, 0u, a.x_snap[c], a.model_diff[c]};     // (the snapshot value is only used without cached margins)
        } else {
            const int w = (c * a.b_x) >> 5, last = static_cast<int>(a.model_last_word);   // (fewer than 2^20 words)
            return Gather{a.xq[w], straddles ? a.xq[w + 1 < last ? w + 1 : last] : 0u, a.x_snap[c], 0.0f};
        }
    };
    auto vec_val = [&](const Gather &g, int c) {
        if constexpr (DIFF) return make_float2(g.diff, g.xs);
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
    auto row_info = [&](int r0, const StreamKey &round_key) {
        RowInfo ri{-1, 0, 0, 1.0f, 0.0f};
        const int nrows = min(kCsrMaxRows, a.B - r0);
        if (static_cast<int>(threadIdx.x) < nrows) {
            const int r = r0 + threadIdx.x;
            int64_t i;
            if (a.idx) {
                i = a.idx[static_cast<int64_t>(m) * a.B + r];
            } else {
                StreamKey sk = round_key;
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
    if (a.prep_out && slice == nslices) {
        // ---- the extra block: worker m's mini-batch of the next round, left in memory (see kPrepInts)
        StreamKey next_key = a.key;
        next_key.iter = a.next_iter;
        const int nrows = a.B;
        const RowInfo ri = row_info(0, next_key);
        if (static_cast<int>(threadIdx.x) < nrows) {
            meta.row[threadIdx.x] = ri.row;
            meta.start[threadIdx.x] = ri.start;
            meta.len[threadIdx.x] = ri.len;
        }
        csr_prefix_lengths(meta, nrows);
        int32_t *out = a.prep_out + static_cast<int64_t>(m) * a.prep_stride;
        const int total = meta.pre[nrows];
        const bool fits = total <= a.cap;
        if (static_cast<int>(threadIdx.x) < nrows) {
            out[kPrepRow + threadIdx.x] = ri.row;
            out[kPrepLen + threadIdx.x] = ri.len;
            out[kPrepPre + threadIdx.x] = meta.pre[threadIdx.x];
            out[kPrepY + threadIdx.x] = __float_as_int(ri.y);
            out[kPrepZ + threadIdx.x] = __float_as_int(ri.z);
        }
        if (threadIdx.x == 0) {
            out[0] = fits ? 1 : 0;
            out[1] = total;
            out[kPrepPre + nrows] = total;
        }
        if (!fits) return;
        int2 *entry = reinterpret_cast<int2 *>(out + kPrepEntries);
        const int lane = threadIdx.x & (kWave - 1);
        for (int p0 = threadIdx.x; p0 - lane < total; p0 += kStageFlight * kCsrThreads) {
            int64_t src[kStageFlight];
            int tag[kStageFlight], col[kStageFlight];
            float val[kStageFlight];
#pragma unroll
            for (int u = 0; u < kStageFlight; ++u)
                src[u] = csr_stage_source(meta, 0, nrows, 0, total, p0 - lane + u * kCsrThreads, lane, u ? src[0] : 0, tag[u]);
#pragma unroll
            for (int u = 0; u < kStageFlight; ++u) {
                col[u] = a.A.indices[src[u]];
                val[u] = a.A.values[src[u]];
            }
#pragma unroll
            for (int u = 0; u < kStageFlight; ++u)
                if (p0 + u * kCsrThreads < total) entry[p0 + u * kCsrThreads] = make_int2(col[u] | tag[u], __float_as_int(val[u]));
        }
        return;
    }
    for (int64_t c0 = 0; c0 < d; c0 += win) {
        const int64_t c1 = min(d, c0 + win);
        const int64_t c1p = min((d + 3) / 4 * 4, c0 + win);     // the window, up to a whole quad past the end of the vector
        FixedAcc fx{0.0f, 0};
        bool rows_done = false;
        if (a.prep_in) {
            // ---- this round's mini-batch was prepared: descriptors and the first entries are requested together
            // (a.B <= kCsrMaxRows, one window)
            const int32_t *in = a.prep_in + static_cast<int64_t>(m) * a.prep_stride;
            const int2 *entry = reinterpret_cast<const int2 *>(in + kPrepEntries);
            const int nrows = a.B;
            const int tr = min(static_cast<int>(threadIdx.x), kCsrMaxRows - 1);
            const int ready = in[0], total = in[1];
            const int p_row = in[kPrepRow + tr], p_len = in[kPrepLen + tr], p_pre = in[kPrepPre + tr];
            const int p_last = in[kPrepPre + nrows];
            const float p_y = __int_as_float(in[kPrepY + tr]), p_z = __int_as_float(in[kPrepZ + tr]);
            int2 first[kStageFlight];
#pragma unroll
            for (int u = 0; u < kStageFlight; ++u) first[u] = entry[min(static_cast<int>(threadIdx.x) + u * kCsrThreads, a.cap - 1)];
            for (int64_t j = 4ll * threadIdx.x; j < c1p - c0; j += 4ll * kCsrThreads)
                *reinterpret_cast<int4 *>(acc + j) = make_int4(0, 0, 0, 0);
            if (ready) {                                          // (the same for every thread)
                if (static_cast<int>(threadIdx.x) < nrows) {
                    meta.row[threadIdx.x] = p_row;
                    meta.len[threadIdx.x] = p_len;
                    meta.pre[threadIdx.x] = p_pre;
                    sh_y[threadIdx.x] = p_y;
                    meta.z[threadIdx.x] = p_z;
                }
                if (threadIdx.x == 0) meta.pre[nrows] = p_last;
                __syncthreads();
                if (have_z)
                    csr_process_prepared<false>(entry, first, total, meta, nrows, acc, static_cast<int>(c0), static_cast<int>(c1),
                                                sg, fx, su, &sh_poison, vec_req, vec_val, coef_of);
                else
                    csr_process_prepared<true>(entry, first, total, meta, nrows, acc, static_cast<int>(c0), static_cast<int>(c1),
                                               sg, fx, su, &sh_poison, vec_req, vec_val, coef_of);
                rows_done = true;
            }
        }
        for (int r0 = 0; r0 < a.B && !rows_done; r0 += kCsrMaxRows) {     // passes of at most kCsrMaxRows rows
            const int nrows = min(kCsrMaxRows, a.B - r0);
            const RowInfo ri = row_info(r0, a.key);
            if (r0 == 0)                                       // (the window is cleared while the row loads are on their way)
                for (int64_t j = 4ll * threadIdx.x; j < c1p - c0; j += 4ll * kCsrThreads)
                    *reinterpret_cast<int4 *>(acc + j) = make_int4(0, 0, 0, 0);
            if (static_cast<int>(threadIdx.x) < nrows) {
                meta.row[threadIdx.x] = ri.row;
                meta.start[threadIdx.x] = ri.start;
                meta.len[threadIdx.x] = ri.len;
                sh_y[threadIdx.x] = ri.y;
                meta.z[threadIdx.x] = ri.z;
            }
            csr_prefix_lengths(meta, nrows);
            if (have_z)
                csr_process_rows<false, kStageFlight>(a.A, meta, nrows, acc, static_cast<int>(c0), static_cast<int>(c1), sg, fx, su,
                                        &sh_poison, vec_req, vec_val, coef_of);
            else
                csr_process_rows<true, kStageFlight>(a.A, meta, nrows, acc, static_cast<int>(c0), static_cast<int>(c1), sg, fx, su,
                                       &sh_poison, vec_req, vec_val, coef_of);
            if constexpr (COMMON) break;                       // (one pass)
        }
        // the window becomes float32: the dense part  l2*(q - snapshot)  plus the accumulated sums, zero past the end
        // of the vector; four coordinates per thread and step
        {
            const float unit = sh_poison ? __uint_as_float(0x7FC00000u) : ldexpf(1.0f, -fx.k);
            // (nothing was added past the end of the vector: the sums there are zero)
            const auto finish_quad = [&](int64_t j, float4 v) {
                const int4 sum = *reinterpret_cast<const int4 *>(acc + (j - c0));
                v.x += static_cast<float>(sum.x) * unit; v.y += static_cast<float>(sum.y) * unit;
                v.z += static_cast<float>(sum.z) * unit; v.w += static_cast<float>(sum.w) * unit;
                *reinterpret_cast<float4 *>(alpha + (j - c0)) = v;
                seen_max = max(max(seen_max, abs_bits(v.x)), max(max(abs_bits(v.y), abs_bits(v.z)), abs_bits(v.w)));
            };
            const auto slow_quad = [&](int64_t j) {
                float t[4];
                for (int e = 0; e < 4; ++e) {
                    if constexpr (DIFF) t[e] = j + e < d ? a.l2 * a.model_diff[j + e] : 0.0f;
                    else t[e] = j + e < d ? a.l2 * (model_value(msg, j + e) - a.x_snap[j + e]) : 0.0f;
                }
                finish_quad(j, make_float4(t[0], t[1], t[2], t[3]));
            };
            const int64_t whole = min(c1p, d / 4 * 4);            // whole quads of the vector end here
            if constexpr (DIFF) {
                constexpr int kInitFlight = 6;                   // (as below: requested together, at clamped positions)
                for (int64_t j0 = c0 + 4ll * threadIdx.x; j0 < whole; j0 += 4ll * kCsrThreads * kInitFlight) {
                    float4 df[kInitFlight];
#pragma unroll
                    for (int u = 0; u < kInitFlight; ++u)
                        df[u] = *reinterpret_cast<const float4 *>(
                            a.model_diff + min<int64_t>(j0 + 4ll * kCsrThreads * u, whole - 4));
#pragma unroll
                    for (int u = 0; u < kInitFlight; ++u) {
                        const int64_t j = j0 + 4ll * kCsrThreads * u;
                        if (j < whole) finish_quad(j, make_float4(a.l2 * df[u].x, a.l2 * df[u].y, a.l2 * df[u].z, a.l2 * df[u].w));
                    }
                }
                if (threadIdx.x == 0 && whole >= c0 && whole < c1p) slow_quad(whole);      // the vector ends inside a quad
            } else if (a.b_x == 8) {
                // the loads of kInitFlight steps are requested together (at clamped positions: a load behind a
                // per-lane test would be waited for before the next one is issued)
                constexpr int kInitFlight = 6;
                for (int64_t j0 = c0 + 4ll * threadIdx.x; j0 < whole; j0 += 4ll * kCsrThreads * kInitFlight) {
                    float4 xs[kInitFlight];
                    uint32_t w[kInitFlight];
#pragma unroll
                    for (int u = 0; u < kInitFlight; ++u) {
                        const int64_t jc = min(j0 + 4ll * kCsrThreads * u, whole - 4);
                        xs[u] = *reinterpret_cast<const float4 *>(a.x_snap + jc);
                        w[u] = a.xq[jc >> 2];
                    }
#pragma unroll
                    for (int u = 0; u < kInitFlight; ++u) {
                        const int64_t j = j0 + 4ll * kCsrThreads * u;
                        if (j < whole)
                            finish_quad(j, make_float4(a.l2 * (msg.delta_x * static_cast<float>(sext_field(w[u], 0, 8)) - xs[u].x),
                                                       a.l2 * (msg.delta_x * static_cast<float>(sext_field(w[u], 8, 8)) - xs[u].y),
                                                       a.l2 * (msg.delta_x * static_cast<float>(sext_field(w[u], 16, 8)) - xs[u].z),
                                                       a.l2 * (msg.delta_x * static_cast<float>(sext_field(w[u], 24, 8)) - xs[u].w)));
                    }
                }
                if (threadIdx.x == 0 && whole >= c0 && whole < c1p) slow_quad(whole);      // the vector ends inside a quad
            } else {
                for (int64_t j = c0 + 4ll * threadIdx.x; j < c1p; j += 4ll * kCsrThreads) slow_quad(j);
            }
            __syncthreads();
        }
        if (alpha_row) {                                       // several windows: the finished one goes to memory
            for (int64_t j = c0 + threadIdx.x; j < c1p; j += kCsrThreads) alpha_row[j] = alpha[j - c0];
            __syncthreads();
        }
        if constexpr (COMMON) break;                           // (one window)
    }
    // the whole gradient, padded with zeros to a whole quad: in LDS when it fits in one window, else in this worker's
    // workspace row (the block's own writes, visible to all its threads after the barrier above)
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
        sparsify_slice_from_lds<true>(av, d, key, slice, nslices, a.beta_ws + static_cast<int64_t>(m) * a.ld_ws,
                                      a.part_max + static_cast<int64_t>(m) * nslices + slice,
                                      a.part_kept + static_cast<int64_t>(m) * nslices + slice, su, si, &seen_max);
        return;
    }
    const WorkerOut out{a.packed + static_cast<int64_t>(m) * a.ld_words, a.row_words, a.delta_out + m,
                        a.nnz_out ? a.nnz_out + m : nullptr, a.status};
    switch (a.b) {
    case 2: worker_tail_from_lds<2, true>(av, d, a.sparsify != 0, a.b, key, out, su, si, slice, nslices, &seen_max); break;
    case 4: worker_tail_from_lds<4, true>(av, d, a.sparsify != 0, a.b, key, out, su, si, slice, nslices, &seen_max); break;
    case 32: worker_tail_from_lds<32, true>(av, d, a.sparsify != 0, a.b, key, out, su, si, slice, nslices, &seen_max); break;
    default: worker_tail_from_lds<8, true>(av, d, a.sparsify != 0, a.b, key, out, su, si, slice, nslices, &seen_max); break;
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
    __shared__ uint32_t su[kCsrWaves];
    __shared__ int sh_poison;
    int *acc = reinterpret_cast<int *>(lds);             // the window [c0, c1) of this block's partial sum, fixed point
    const CsrStage sg = csr_stage_in(lds + win, cap, false);
    if (threadIdx.x == 0) sh_poison = 0;                 // (published by the barriers of the first row pass)
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int64_t per = (A.n + gridDim.x - 1) / gridDim.x;
    const int64_t i0 = blockIdx.x * per, i1 = min(A.n, i0 + per);
    const float inv_n = 1.0f / static_cast<float>(A.n);
    double loss = 0.0;                                   // the lanes that evaluate row scalars add to theirs
    float *mine = partial + static_cast<int64_t>(blockIdx.x) * ldp;
    for (int64_t c0 = 0; c0 < ldp; c0 += win) {          // one window when the vector fits in LDS
        const int64_t c1 = min(ldp, c0 + win);
        for (int64_t j = threadIdx.x; j < c1 - c0; j += kCsrThreads) acc[j] = 0;
        FixedAcc fx{0.0f, 0};
        const bool first = c0 == 0;                      // margins and losses are recorded once
        // The fixed-point sums go to this block's float32 partial vector at the end, and in between whenever
        // kFlushRows rows have been added: a term is rounded relative to the bound of everything in the accumulator,
        // which grows with the number of rows, so that number is kept small.
        int since_flush = 0;
        bool wrote = false;
        for (int64_t ib = i0; ib < i1; ib += kCsrMaxRows) {
            const int nrows = static_cast<int>(min<int64_t>(kCsrMaxRows, i1 - ib));
            if (static_cast<int>(threadIdx.x) < nrows) {
                const int64_t i = ib + threadIdx.x;
                const int64_t s = A.indptr[i];
                meta.row[threadIdx.x] = static_cast<int>(i);
                meta.start[threadIdx.x] = s;
                meta.len[threadIdx.x] = static_cast<int>(A.indptr[i + 1] - s);
                meta.z[threadIdx.x] = A.y[i];            // (here: the row's label, so that no lane fetches it later)
            }
            csr_prefix_lengths(meta, nrows);
            const int64_t ib_now = ib;
            auto vec_req = [&](int c) { return x[c]; };
            auto vec_val = [&](float xc, int) { return make_float2(xc, 0.0f); };
            auto coef_of = [&](int r, float z, float) {
                const int64_t i = ib_now + r;
                const float y = meta.z[r];
                if (first) {
                    if (z_out) z_out[i] = z;
                    loss += static_cast<double>(logistic_loss_fast(y * z));
                }
                // (a few lanes evaluate this while every other lane of the block waits: hardware exp, log and
                // reciprocal, as in the dense kernel)
                return logistic_slope_fast(y, z) * inv_n;
            };
            csr_process_rows<false, kFullFlight>(A, meta, nrows, acc, static_cast<int>(c0), static_cast<int>(min(A.d, c1)), sg, fx, su,
                                    &sh_poison, vec_req, vec_val, coef_of);
            since_flush += nrows;
            if (since_flush >= kFlushRows || ib + kCsrMaxRows >= i1) {         // (ends with a barrier: all adds are in)
                const float unit = sh_poison ? __uint_as_float(0x7FC00000u) : ldexpf(1.0f, -fx.k);
                for (int64_t j = c0 + threadIdx.x; j < c1; j += kCsrThreads) {
                    const float v = static_cast<float>(acc[j - c0]) * unit;
                    mine[j] = wrote ? mine[j] + v : v;
                    acc[j - c0] = 0;
                }
                __syncthreads();
                fx = FixedAcc{0.0f, 0};
                since_flush = 0;
                wrote = true;
            }
        }
        if (!wrote)                                      // a block without rows
            for (int64_t j = c0 + threadIdx.x; j < c1; j += kCsrThreads) mine[j] = 0.0f;
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
    size_t lds;     // bytes of dynamic LDS: window + staging
};

// A staged entry takes 12 bytes of LDS, 16 when the caller needs two sums per row (see CsrStage).
static bool csr_plan(int64_t d, bool second, CsrPlan &p)
{
    if (d >= (1ll << kColBits)) return false;      // a staged entry keeps its row number above kColBits column bits
    const int64_t budget = kLdsBudget - kCsrFixedLds;                     // bytes for window + staging
    const int64_t each = second ? 16 : 12;
    int64_t nwin = 1;
    if (pad4(d) * 4 + each * 512 > budget) nwin = ceil_div(pad4(d) * 4, budget - each * kMinStage);
    const int64_t win = pad4(ceil_div(pad4(d), nwin));
    int64_t cap = (budget - win * 4) / each;
    if (cap > kMaxStage) cap = kMaxStage;
    p.lds = static_cast<size_t>(win * 4 + cap * each);
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
    if (!csr_plan(prob->d, true, plan)) return DQ_ERR_UNSUPPORTED;
    if (op == DQ_OP_FULL_GRAD) {
        const int64_t P = csr_full_splits(prob->n);
        return P * pad4(prob->d) * 4 + P * 8;
    }
    // a row per worker: the whole gradient when it does not fit in LDS, else the sparsified gradient when the
    // sparsifier is split over several blocks per worker (see csr_worker); then 8 values + 8 counts per worker: all
    // that a single step uses
    if (op == DQ_OP_WORKER_STEP) return csr_model_diff_offset(prob, M);
    // then one more row, in which dq_run_rounds keeps (decoded model) - snapshot between two rounds of a call; then two
    // sets of prepared mini-batches (see kPrepInts), the one a round reads and the one it leaves for the next
    return csr_prep_offset(prob, M) + 2 * M * csr_prep_stride(prob) * 4;
}

int64_t csr_prep_offset(const dq_problem *prob, int64_t M)
{
    return csr_model_diff_offset(prob, M) + pad4(prob->d) * 4;
}

// 32-bit words per worker of a prepared mini-batch, for the larger of the two staging capacities
int64_t csr_prep_stride(const dq_problem *prob)
{
    CsrPlan plan;
    if (!csr_plan(prob->d, false, plan)) return 0;
    return kPrepInts(plan.cap);
}

int64_t csr_model_diff_offset(const dq_problem *prob, int64_t M)
{
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
    if (!csr_plan(d, false, plan)) return DQ_ERR_UNSUPPORTED;
    if (ws_bytes < csr_workspace_bytes(DQ_OP_FULL_GRAD, prob, 0, 0) || !ws) return DQ_ERR_WORKSPACE;
    const int64_t ldp = pad4(d);
    const int P = static_cast<int>(csr_full_splits(n));
    float *partial = static_cast<float *>(ws);
    double *loss_partial = reinterpret_cast<double *>(partial + static_cast<int64_t>(P) * ldp);
    const size_t lds = plan.lds;
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
    if (!csr_plan(d, a.z_snap == nullptr, plan)) return DQ_ERR_UNSUPPORTED;
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
    const size_t lds = plan.lds;
    k.model_diff = a.b_x == 32 ? nullptr : a.model_diff;
    // (see csr_worker_kernel for the two switches)
    const bool diff = k.model_diff != nullptr;
    const bool common = plan.nwin == 1 && a.B <= kCsrMaxRows && a.z_snap != nullptr;
    static std::once_flag attr_once[4];
    static hipError_t attr_rc[4] = {hipSuccess, hipSuccess, hipSuccess, hipSuccess};
    void (*const kernels[4])(const CsrWorkerArgs) = {csr_worker_kernel<false, false>, csr_worker_kernel<false, true>,
                                                     csr_worker_kernel<true, false>, csr_worker_kernel<true, true>};
    const int which = (diff ? 2 : 0) + (common ? 1 : 0);
    const auto kernel = kernels[which];
    int rc = allow_big_lds(kernel, attr_once[which], attr_rc[which]);
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
                                  a.ws_bytes >= csr_workspace_bytes(DQ_OP_WORKER_STEP, prob, a.M, a.B);
    if (split_sparsifier) {
        k.beta_ws = static_cast<float *>(a.ws);
        k.part_max = k.beta_ws + a.M * k.ld_ws;
        k.part_kept = reinterpret_cast<int32_t *>(k.part_max + a.M * kMaxSlices);
    }
    // a round of dq_run_rounds that has a successor in its call prepares that round's mini-batches in one more block
    // per worker (on compute units the launch leaves idle), and reads its own if the round before left them
    const bool can_prepare = !a.idx && a.B <= kCsrMaxRows && plan.nwin == 1 && a.M * (slices + 1) <= 256;
    if (can_prepare) {
        k.prep_in = a.prep_in;
        k.prep_out = a.prep_out;
        k.prep_stride = csr_prep_stride(prob);
        k.next_iter = a.iter + 1u;
    }
    if (a.prepared_next) *a.prepared_next = k.prep_out != nullptr;
    const dim3 grid(static_cast<unsigned>(a.M), slices + (k.prep_out ? 1u : 0u)), block(kCsrThreads);
    if (a.ev_start && a.ev_stop)      // the kernel's own start and end times go to the two events
        hipExtLaunchKernelGGL(kernel, grid, block, static_cast<uint32_t>(lds), st, a.ev_start, a.ev_stop, 0u, k);
    else
        kernel<<<grid, block, lds, st>>>(k);
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
