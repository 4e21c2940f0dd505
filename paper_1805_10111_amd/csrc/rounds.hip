// Host-side sequencing of the inner loop of Alg. 1-3: enqueues the kernels of several
// consecutive synchronous rounds with one call, so that the launch rate is not limited
// by the caller's language runtime.  No numerical work happens here.
#include "dq_common.h"
#include "grad_launch.h"

static inline hipStream_t as_stream(void *s) { return reinterpret_cast<hipStream_t>(s); }

extern "C" int32_t dq_run_rounds(const dq_problem *prob, const dq_run_config *cfg, const dq_run_state *st,
                                 int64_t epoch, int64_t t0, int64_t rounds, float eta, float theta,
                                 void **worker_events, void *stream)
{
    if (!prob || !cfg || !st || epoch < 0 || t0 < 0 || rounds < 0 || cfg->m <= 0 || t0 + rounds > cfg->m)
        return DQ_ERR_INVALID_ARG;
    if (cfg->algo < DQ_ALGO_ASYLPG || cfg->algo > DQ_ALGO_ACC) return DQ_ERR_INVALID_ARG;
    if (!st->packed || !st->delta || !st->xq || !st->delta_x || !st->x || !st->x_snap || !st->g_snap || !st->absmax_x ||
        !dq::aligned16(st->packed) || !dq::aligned16(st->xq))
        return DQ_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(st->status) & 3u) || (reinterpret_cast<uintptr_t>(st->nnz) & 3u) ||
        (reinterpret_cast<uintptr_t>(st->delta) & 3u) || (reinterpret_cast<uintptr_t>(st->delta_x) & 3u))
        return DQ_ERR_INVALID_ARG;
    if (cfg->M <= 0 || cfg->B <= 0) return DQ_ERR_INVALID_ARG;
    if (cfg->b != 2 && cfg->b != 4 && cfg->b != 8 && cfg->b != 32) return DQ_ERR_UNSUPPORTED;
    {
        const int64_t row_words = cfg->b == 32 ? prob->d : dq::packed_words(prob->d, cfg->b);
        if (st->ld_words < row_words || (cfg->M > 1 && st->ld_words % 4 != 0)) return DQ_ERR_INVALID_ARG;
    }
    const bool acc = cfg->algo == DQ_ALGO_ACC;
    if (acc && (!st->y || !st->xsum)) return DQ_ERR_INVALID_ARG;
    if (st->wire && !st->wire_nnz) return DQ_ERR_INVALID_ARG;
    if (cfg->tau < 0 || cfg->tau >= cfg->M || (cfg->each != 0 && cfg->each != 1)) return DQ_ERR_INVALID_ARG;
    const int64_t slots = cfg->tau + 1;
    const int64_t xq_words = cfg->b_x == 32 ? prob->d : dq::packed_words(prob->d, cfg->b_x);
    if (slots > 1 && (st->xq_stride_words < xq_words || st->xq_stride_words % 4 != 0)) return DQ_ERR_INVALID_ARG;
    {
        // the workspace is checked once, for every worker group of the call, before anything is enqueued
        const int64_t need = dq_workspace_bytes(DQ_OP_VR_GRAD, prob, cfg->M, cfg->B);
        if (need < 0) return static_cast<int32_t>(need);
        if (need > 0 && (!st->ws || st->ws_bytes < need)) return DQ_ERR_WORKSPACE;
    }
    const float scale = 1.0f / static_cast<float>(cfg->M);
    // the model equals the snapshot bit for bit at the first round of an epoch of Alg. 1/2 and of the
    // first epoch of Alg. 3: flag-bit case of Section 4.1
    const bool start_is_snapshot = !acc || epoch == 0;
    // Alg. 1, master (i) without a launch of its own: between two rounds of one call the master kernel stops at the
    // update and ||x||_inf (spread over the chip), and the next round's row-streaming kernel quantizes the model in
    // its prologue, while its first rows are on their way -- every block for itself, one of them storing the message.
    // The two slots of absmax_x alternate: the kernel that reads one clears the other for the master of its round.
    const bool fusable = cfg->tau == 0 && cfg->b_x != 32 &&
                         dq::dense_model_fusable(prob, cfg->M, cfg->B, cfg->b_x, st->z_snap != nullptr);
    // Alg. 2, one group of workers, messages not crossing as (position, value) streams: a worker step whose sparsifier
    // is split over several blocks leaves the quantization of its messages to the master kernel (one launch less)
    const bool defer_ok = cfg->algo == DQ_ALGO_SPARSE && cfg->b != 32 && cfg->tau == 0 && !st->wire;
    // CSR features, one group of workers: the master that quantizes the model in a launch of its own also leaves
    // (decoded model) - snapshot in the workspace for the workers of the next round of this call
    const bool csr = prob->layout == 1;
    float *model_diff = nullptr;
    if (csr && cfg->tau == 0 && st->ws) {
        const int64_t off = dq::csr_model_diff_offset(prob, cfg->M);
        if (st->ws_bytes >= off + (prob->d + 3) / 4 * 4 * 4) model_diff = reinterpret_cast<float *>(static_cast<char *>(st->ws) + off);
    }
    bool diff_ready = false;             // model_diff holds the difference for the model message of this round
    // ... and each worker launch prepares the mini-batches of the next round (two sets, alternating)
    int32_t *prep_sets = nullptr;
    int64_t prep_set_words = 0;
    if (csr && cfg->tau == 0 && st->ws) {
        const int64_t off = dq::csr_prep_offset(prob, cfg->M);
        prep_set_words = cfg->M * dq::csr_prep_stride(prob);
        if (prep_set_words > 0 && st->ws_bytes >= off + 2 * prep_set_words * 4)
            prep_sets = reinterpret_cast<int32_t *>(static_cast<char *>(st->ws) + off);
    }
    bool prep_ready = false;             // the set of this round's parity holds this round's mini-batches
    bool model_pending = false;          // the model of this round is still x itself (not yet a message)
    for (int64_t t = t0; t < t0 + rounds; ++t) {
        const uint32_t it = static_cast<uint32_t>(epoch * cfg->m + t);
        uint32_t *xq_now = st->xq + (t % slots) * st->xq_stride_words;
        float *dx_now = st->delta_x + (t % slots);
        int32_t rc;
        if (t == 0 && !start_is_snapshot) {
            // Alg. 3, later epochs: x_0 = snapshot + theta (y - snapshot) is quantized by the master
            if (cfg->b_x == 32) {
                DQ_HIP_TRY(hipMemcpyAsync(xq_now, st->x, static_cast<size_t>(prob->d) * sizeof(float),
                                          hipMemcpyDeviceToDevice, as_stream(stream)));
            } else {
                rc = dq_quantize_pack(st->x, prob->d, 1, prob->d, cfg->b_x, st->absmax_x, 0, cfg->seed, it, DQ_TAG_MODEL,
                                      DQ_MASTER_ID, xq_now, xq_words, dx_now, st->status, stream);
                if (rc != DQ_OK) return rc;
            }
        }
        // worker side: group g of the workers is g rounds behind (g = 0 only when tau = 0)
        dq::SparsifiedParts parts{nullptr, 0, nullptr, nullptr, 0};
        for (int64_t g = 0; g < slots; ++g) {
            const int64_t w_lo = dq::ceil_div(g * cfg->M, slots), w_hi = dq::ceil_div((g + 1) * cfg->M, slots);
            if (w_hi <= w_lo) continue;
            const int64_t tm = t - g > 0 ? t - g : 0;                  // round whose model message the group holds
            dq::WorkerArgs w{};
            w.M = w_hi - w_lo; w.B = cfg->B;
            w.xq = st->xq + (tm % slots) * st->xq_stride_words; w.delta_x = st->delta_x + (tm % slots); w.b_x = cfg->b_x;
            w.model_is_snapshot = tm == 0 && start_is_snapshot;
            w.x_snap = st->x_snap; w.z_snap = st->z_snap;
            w.sparsify = cfg->algo == DQ_ALGO_SPARSE; w.b = cfg->b; w.seed = cfg->seed; w.iter = it;
            w.worker0 = static_cast<uint32_t>(w_lo);
            w.packed = st->packed + w_lo * st->ld_words; w.ld_words = st->ld_words; w.delta_out = st->delta + w_lo;
            // nonzero counts are what the sparse message size is computed from; the other algorithms do not need them
            w.nnz_out = (st->nnz && cfg->algo == DQ_ALGO_SPARSE) ? st->nnz + t * cfg->M + w_lo : nullptr;
            w.status = st->status;
            w.ws = st->ws; w.ws_bytes = st->ws_bytes;
            if (g == 0) w.zero_word = reinterpret_cast<uint32_t *>(st->absmax_x + (t & 1));   // for the master's max below
            if (model_pending) {                  // (fusable: a single group)
                w.x_model = st->x;
                w.absmax_model = st->absmax_x + ((t - 1) & 1);
            }
            if (defer_ok) w.deferred = &parts;
            if (diff_ready) w.model_diff = model_diff;
            bool prepared_next = false;
            if (prep_sets) {
                if (prep_ready) w.prep_in = prep_sets + (t & 1) * prep_set_words;
                if (t + 1 < t0 + rounds) w.prep_out = prep_sets + ((t + 1) & 1) * prep_set_words;
                w.prepared_next = &prepared_next;
            }
            if (worker_events && g == 0) {                       // (a null pair: this round's launch is a plain one)
                w.ev_start = static_cast<hipEvent_t>(worker_events[2 * (t - t0)]);
                w.ev_stop = static_cast<hipEvent_t>(worker_events[2 * (t - t0) + 1]);
            }
            rc = dq::worker_step_impl(prob, w, stream);
            if (rc != DQ_OK) return rc;
            prep_ready = prepared_next;
        }
        // Section 4.2 on request: the sparsified messages cross to the master as (position, value) streams
        if (st->wire && cfg->algo == DQ_ALGO_SPARSE && cfg->b != 32) {
            rc = dq_sparse_encode(st->packed, st->ld_words, prob->d, cfg->M, cfg->b, st->wire, st->ld_wire, st->wire_nnz, stream);
            if (rc != DQ_OK) return rc;
            rc = dq_sparse_decode(st->wire, st->ld_wire, st->wire_nnz, prob->d, cfg->M, cfg->b, st->packed, st->ld_words, stream);
            if (rc != DQ_OK) return rc;
        }
        // master side; the new model is the message of round t+1
        uint32_t *xq_next = st->xq + ((t + 1) % slots) * st->xq_stride_words;
        float *dx_next = st->delta_x + ((t + 1) % slots);
        model_pending = fusable && t + 1 < t0 + rounds;
        // (the difference is of use only to a next round of this call)
        float *diff_out = (model_diff && t + 1 < t0 + rounds &&
                           dq::master_leaves_model_diff(prob->d, cfg->b_x, parts.parts > 0)) ? model_diff : nullptr;
        diff_ready = diff_out != nullptr;
        if (parts.parts > 0)
            rc = dq::master_step_from_parts_impl(parts, 0u, it, st->packed, st->ld_words, st->delta,
                                                 st->nnz ? st->nnz + t * cfg->M : nullptr, cfg->M, cfg->b, scale, cfg->each,
                                                 st->g_snap, st->x, eta, prob->l1, prob->d, cfg->b_x, cfg->seed, it + 1u,
                                                 xq_next, dx_next, st->absmax_x + (t & 1), st->status,
                                                 /*absmax_zeroed=*/true, stream, st->x_snap, diff_out);
        else if (model_pending)
            rc = dq::master_update_impl(st->packed, st->ld_words, st->delta, cfg->M, cfg->b, scale, cfg->each, st->g_snap,
                                        st->x, acc ? st->y : nullptr, st->x_snap, acc ? st->xsum : nullptr, eta, theta,
                                        prob->l1, prob->d, reinterpret_cast<uint32_t *>(st->absmax_x + (t & 1)), stream);
        else
            rc = dq::master_step_impl(st->packed, st->ld_words, st->delta, cfg->M, cfg->b, scale, cfg->each, st->g_snap,
                                      st->x, acc ? st->y : nullptr, st->x_snap, acc ? st->xsum : nullptr, eta, theta,
                                      prob->l1, prob->d, cfg->b_x, cfg->seed, it + 1u, xq_next, dx_next,
                                      st->absmax_x + (t & 1), st->status, /*absmax_zeroed=*/true, stream, diff_out);
        if (rc != DQ_OK) return rc;
    }
    return DQ_OK;
}

// Section 5.1 (parameters of Alg. 3 as used in the experiments): theta_s = 2/(s+2), eta_s = lr/theta_s, in float32.
extern "C" int32_t dq_acc_params(float lr, int64_t s, float *theta_out, float *eta_out)
{
    if (s < 1 || !theta_out || !eta_out) return DQ_ERR_INVALID_ARG;
    const float theta = static_cast<float>(2.0 / static_cast<double>(s + 2));
    *theta_out = theta;
    *eta_out = lr / theta;
    return DQ_OK;
}

// Message sizes: Section 3.1 (32 + b*d bits for a quantized vector, 32*d unquantized), Section 4.1 (one flag bit
// when the model equals the snapshot), Section 4.2 (scale + position and value per nonzero of a sparsified vector).
extern "C" int64_t dq_message_bits(int32_t kind, int64_t d, int32_t b, int64_t nnz)
{
    if (d <= 0 || b < 2 || (b > 16 && b != 32)) return DQ_ERR_INVALID_ARG;
    switch (kind) {
    case DQ_MSG_DENSE: return b == 32 ? 32 * d : 32 + static_cast<int64_t>(b) * d;
    case DQ_MSG_FLAG: return 1;
    case DQ_MSG_SPARSE: {
        if (nnz < 0 || nnz > d) return DQ_ERR_INVALID_ARG;
        int pos = 0;
        while ((1ll << pos) < d) ++pos;                       // ceil(log2 d) position bits
        return (b == 32 ? 0 : 32) + nnz * (pos + b);
    }
    default: return DQ_ERR_INVALID_ARG;
    }
}
