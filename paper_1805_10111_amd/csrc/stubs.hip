// Entry points whose kernels are not written yet: they report DQ_ERR_UNSUPPORTED.
#include "dq_common.h"

extern "C" int64_t dq_workspace_bytes(int32_t, const dq_problem *, int64_t, int64_t) { return 0; }

extern "C" int32_t dq_full_grad(const dq_problem *, const float *, float *, float *, double *, void *, int64_t, void *) { return DQ_ERR_UNSUPPORTED; }
extern "C" int32_t dq_vr_grad(const dq_problem *, const int32_t *, int64_t, int64_t, const uint32_t *, const float *, int32_t,
                              int32_t, const float *, const float *, float *, int64_t, float *, float *, void *, int64_t, void *) { return DQ_ERR_UNSUPPORTED; }

extern "C" int32_t dq_worker_step(const dq_problem *, const int32_t *, int64_t, int64_t, const uint32_t *, const float *, int32_t,
                                  int32_t, const float *, const float *, int32_t, int32_t, uint64_t, uint32_t, uint32_t,
                                  uint32_t *, int64_t, float *, int32_t *, float *, int64_t, uint32_t *, void *, int64_t, void *) { return DQ_ERR_UNSUPPORTED; }



