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
    if (!st->packed || !st->delta || !st->xq || !st->x || !st->x_snap || !st->g_snap || !dq::aligned16(st->packed))
        return DQ_ERR_INVALID_ARG;
    if (cfg->b != 2 && cfg->b != 4 && cfg->b != 8 && cfg->b != 32) return DQ_ERR_UNSUPPORTED;
    {
        const int64_t row_words = cfg->b == 32 ? prob->d : dq::packed_words(prob->d, cfg->b);
        if (st->ld_words < row_words || (cfg->M > 1 && st->ld_words % 4 != 0)) return DQ_ERR_INVALID_ARG;
    }
    const bool acc = cfg->algo == DQ_ALGO_ACC;
    if (acc && (!st->y || !st->xsum)) return DQ_ERR_INVALID_ARG;
    const float scale = 1.0f / static_cast<float>(cfg->M);
    for (int64_t t = t0; t < t0 + rounds; ++t) {
        const uint32_t it = static_cast<uint32_t>(epoch * cfg->m + t);
        // the model equals the snapshot bit for bit at the first round of an epoch of Alg. 1/2 and
        // of the first epoch of Alg. 3: flag-bit case of Section 4.1
        const int flag = t == 0 && (!acc || epoch == 0);
        int32_t rc;
        if (t == 0 && !flag) {
            // Alg. 3, later epochs: x_0 = snapshot + theta (y - snapshot) is quantized by the master
            if (cfg->b_x == 32) {
                DQ_HIP_TRY(hipMemcpyAsync(st->xq, st->x, static_cast<size_t>(prob->d) * sizeof(float),
                                          hipMemcpyDeviceToDevice, as_stream(stream)));
            } else {
                rc = dq_quantize_pack(st->x, prob->d, 1, prob->d, cfg->b_x, st->absmax_x, 0, cfg->seed, it, DQ_TAG_MODEL,
                                      DQ_MASTER_ID, st->xq, dq::packed_words(prob->d, cfg->b_x), st->delta_x, st->status,
                                      stream);
                if (rc != DQ_OK) return rc;
            }
        }
        dq::WorkerArgs w{};
        w.M = cfg->M; w.B = cfg->B; w.xq = st->xq; w.delta_x = st->delta_x; w.b_x = cfg->b_x;
        w.model_is_snapshot = flag; w.x_snap = st->x_snap; w.z_snap = st->z_snap;
        w.sparsify = cfg->algo == DQ_ALGO_SPARSE; w.b = cfg->b; w.seed = cfg->seed; w.iter = it; w.worker0 = 0u;
        w.packed = st->packed; w.ld_words = st->ld_words; w.delta_out = st->delta;
        w.nnz_out = st->nnz ? st->nnz + t * cfg->M : nullptr; w.status = st->status;
        w.ws = st->ws; w.ws_bytes = st->ws_bytes;
        if (worker_events) {
            DQ_HIP_TRY(hipEventRecord(static_cast<hipEvent_t>(worker_events[2 * (t - t0)]), as_stream(stream)));
            w.ev_after_stream = static_cast<hipEvent_t>(worker_events[2 * (t - t0) + 1]);
        }
        rc = dq::worker_step_impl(prob, w, stream);
        if (rc != DQ_OK) return rc;
        rc = dq_master_step(st->packed, st->ld_words, st->delta, cfg->M, cfg->b, scale, st->g_snap, st->x,
                            acc ? st->y : nullptr, st->x_snap, acc ? st->xsum : nullptr, eta, theta, prob->l1, prob->d,
                            cfg->b_x, cfg->seed, it + 1u, st->xq, st->delta_x, st->absmax_x, st->status, stream);
        if (rc != DQ_OK) return rc;
    }
    return DQ_OK;
}
