// CSR-feature gradient kernels (placeholder until written).
#include "dq_common.h"
#include "grad_launch.h"
namespace dq {
int64_t csr_workspace_bytes(int32_t, const dq_problem *, int64_t, int64_t) { return 0; }
int csr_full_grad(const dq_problem *, const float *, float *, float *, double *, void *, int64_t, hipStream_t) { return DQ_ERR_UNSUPPORTED; }
int csr_worker(const dq_problem *, const WorkerArgs &, hipStream_t) { return DQ_ERR_UNSUPPORTED; }
}
