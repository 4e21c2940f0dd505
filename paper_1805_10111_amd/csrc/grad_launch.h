// Host-side argument bundle of a worker step and the per-layout launchers.
#pragma once

#include "dq_common.h"

namespace dq {

// M sparsified gradients as the split sparsifier leaves them in the workspace: rows of ld floats, and per worker
// `parts` slice maxima (the scale is ||beta||_inf, their largest) and kept counts.
struct SparsifiedParts {
    const float *beta; int64_t ld;
    const float *part_max; const int32_t *part_kept; int parts;
};

struct WorkerArgs {
    const int32_t *idx;
    int64_t M, B;
    const uint32_t *xq;
    const float *delta_x;
    int b_x;
    int model_is_snapshot;
    const float *x_snap, *z_snap;
    // dq_vr_grad outputs (alpha_out also optional in dq_worker_step)
    float *alpha_out;
    int64_t ld;
    float *absmax_out, *l1norm_out;
    // dq_worker_step outputs; packed == nullptr selects the dq_vr_grad behaviour
    int sparsify, b;
    uint64_t seed;
    uint32_t iter, worker0;
    uint32_t *packed;
    int64_t ld_words;
    float *delta_out;
    int32_t *nnz_out;
    uint32_t *status;
    void *ws;
    int64_t ws_bytes;
    hipEvent_t ev_start, ev_stop; // nullable (both or none): receive the start and the end time of the kernel that
                                  // streams the feature rows (start/stop events of an extended launch)
    uint32_t *zero_word;          // nullable: one device word the worker kernel sets to 0 (dq_run_rounds uses it to
                                  // prepare the master's ||x||_inf accumulator without a launch of its own)
    // Alg. 1, master (i) done by the worker kernel itself (dq_run_rounds, dense features): when x_model is given the
    // kernel that streams the rows quantizes the model x_model[d] with scale ||x||_inf = *absmax_model and the master's
    // stream (seed, iter, DQ_MASTER_ID, DQ_TAG_MODEL) -- every block for its own use, one block also storing the
    // message to `xq` and its scale to `delta_x`, which are then outputs of the call.  Needs dense_model_fusable().
    // (The same for CSR features was built and measured on the real-sim-shaped configurations: every block
    // quantizing the 20958-coordinate model for itself, and again per gathered entry, made the worker kernel 4.5 us
    // longer, more than the 4.2 us launch it saves -- not kept.)
    const float *x_model, *absmax_model;
    // Alg. 2 with the sparsifier split over several blocks per worker (CSR features): when `deferred` is given and the
    // step takes that route, it stops after the sparsifier -- no message is quantized, `packed`, `delta_out` and
    // `nnz_out` stay untouched -- and describes what it left in *deferred for master_step_from_parts_impl, which
    // quantizes while it aggregates.  deferred->parts == 0 on return: the step was a complete one.
    SparsifiedParts *deferred;
    // CSR features (nullable): model_diff[c] = (model as decoded from `xq`) - x_snap[c] for every column, formed by
    // the master of the previous round (master_leaves_model_diff) in exactly the worker's arithmetic; the worker then
    // reads one float per column instead of decoding the message and subtracting the snapshot.
    const float *model_diff;
    // CSR features, between the rounds of one dq_run_rounds call (all nullable): what a worker step does before it
    // first needs the model (Alg. 1, worker step 2: drawing the rows; reading their extents and entries) is done one
    // round ahead.  prep_out: this launch also prepares the mini-batches of round iter + 1 there (2 * M *
    // csr_prep_stride words from csr_prep_offset in the workspace hold two such sets); *prepared_next tells whether it
    // did.  prep_in: the set a previous launch prepared for this round, same M, B, worker0 and problem.
    const int32_t *prep_in;
    int32_t *prep_out;
    bool *prepared_next;
};

// Whether the dense worker step can take the model from x_model (see WorkerArgs) for this shape.
bool dense_model_fusable(const dq_problem *prob, int64_t M, int64_t B, int b_x, bool have_z);

// Alg. 1, master (ii) alone (Alg. 3 with y): decode + aggregate + prox / momentum update, spread over the chip, with
// ||x||_inf accumulated into *absmax_bits (bit pattern, must hold 0 on entry).  No model quantization.
int32_t master_update_impl(const uint32_t *packed, int64_t ld_words, const float *delta, int64_t M, int32_t b, float scale,
                           int each, const float *g_snap, float *x, float *y, const float *x_snap, float *xsum, float eta,
                           float theta, float l1, int64_t d, uint32_t *absmax_bits, void *stream);

// Validation + dispatch shared by dq_vr_grad, dq_worker_step and dq_run_rounds.
int32_t worker_step_impl(const dq_problem *prob, const WorkerArgs &a, void *stream);

// dq_master_step / dq_master_step_each (each != 0).  absmax_zeroed: *absmax_x_out already holds 0 (see zero_word).
int32_t master_step_impl(const uint32_t *packed, int64_t ld_words, const float *delta, int64_t M, int32_t b, float scale,
                         int each, const float *g_snap, float *x, float *y, const float *x_snap, float *xsum, float eta,
                         float theta, float l1, int64_t d, int32_t b_x, uint64_t seed, uint32_t iter,
                         uint32_t *xq_packed_out, float *delta_x_out, float *absmax_x_out, uint32_t *status,
                         bool absmax_zeroed, void *stream, float *model_diff_out = nullptr);

// model_diff_out (nullable, d floats; master_step_impl and master_step_from_parts_impl): the master also leaves
// Q(x) - x_snap, the difference every worker of the next round needs (WorkerArgs::model_diff) -- when it quantizes the
// model in a launch of its own with a message width of 2, 4 or 8 bits, which this function tells beforehand.
bool master_leaves_model_diff(int64_t d, int32_t b_x, bool from_parts);

// The master step of a round of Alg. 2 whose workers deferred their quantization (WorkerArgs::deferred): one kernel
// quantizes the M sparsified gradients with the workers' streams (seed, worker_iter, worker0 + m, DQ_TAG_GRAD), stores the
// messages, scales and nonzero counts exactly as the worker step would have, and applies the master update; the model
// quantization follows as in master_step_impl.  nnz_out nullable.
int32_t master_step_from_parts_impl(const SparsifiedParts &parts, uint32_t worker0, uint32_t worker_iter, uint32_t *packed, int64_t ld_words,
                                    float *delta_out, int32_t *nnz_out, int64_t M, int32_t b, float scale, int each,
                                    const float *g_snap, float *x, float eta, float l1, int64_t d, int32_t b_x,
                                    uint64_t seed, uint32_t iter, uint32_t *xq_packed_out, float *delta_x_out,
                                    float *absmax_x_out, uint32_t *status, bool absmax_zeroed, void *stream,
                                    const float *x_snap = nullptr, float *model_diff_out = nullptr);

int64_t dense_workspace_bytes(int32_t op, const dq_problem *prob, int64_t M, int64_t B);
int dense_full_grad(const dq_problem *prob, const float *x, float *g_out, float *z_out, double *obj_out, void *ws,
                    int64_t ws_bytes, hipStream_t st);
int dense_worker(const dq_problem *prob, const WorkerArgs &a, hipStream_t st);

int64_t csr_workspace_bytes(int32_t op, const dq_problem *prob, int64_t M, int64_t B);
// where in a DQ_OP_VR_GRAD workspace of a CSR problem dq_run_rounds keeps the d floats of WorkerArgs::model_diff
int64_t csr_model_diff_offset(const dq_problem *prob, int64_t M);
// where the two sets of prepared mini-batches lie there (WorkerArgs::prep_in / prep_out), and the words of one worker's
int64_t csr_prep_offset(const dq_problem *prob, int64_t M);
int64_t csr_prep_stride(const dq_problem *prob);
int csr_full_grad(const dq_problem *prob, const float *x, float *g_out, float *z_out, double *obj_out, void *ws,
                  int64_t ws_bytes, hipStream_t st);
int csr_worker(const dq_problem *prob, const WorkerArgs &a, hipStream_t st);

}  // namespace dq
