// C ABI of the gradient entry points: argument validation and dispatch on the feature layout.
#include <mutex>

#include "dq_common.h"
#include "grad_launch.h"

using namespace dq;

// Workspace of dq_worker_step_static: one array per GPU inside the library's code object, alive until the process
// ends.  In host code the array's name only stands for the symbol; its device address is asked for once per device
// (hipGetSymbolAddress with that device current) and that pointer is what kernels receive.
constexpr int64_t kStaticWsBytes = DQ_STATIC_WS_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticWsBytes];
constexpr int kMaxDevices = 64;
static void *g_scratch_ptr[kMaxDevices];
static std::mutex g_scratch_mutex;

// Device address of `scratch` on the current device (looked up on the first call per device).
static int32_t static_workspace(void **out)
{
    int dev = 0;
    DQ_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return DQ_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        DQ_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return DQ_ERR_DEVICE;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return DQ_OK;
}

static inline hipStream_t as_stream(void *s) { return reinterpret_cast<hipStream_t>(s); }

static int32_t check_problem(const dq_problem *p)
{
    if (!p || p->n <= 0 || p->d <= 0 || !p->y || p->n > 0x7FFFFFFFll) return DQ_ERR_INVALID_ARG;
    if (p->layout == 0) {
        if (!p->dense || !aligned16(p->dense) || p->lda < p->d || (p->lda % 4) != 0) return DQ_ERR_INVALID_ARG;
    } else if (p->layout == 1) {
        if (!p->indptr || !p->indices || !p->values) return DQ_ERR_INVALID_ARG;
    } else {
        return DQ_ERR_INVALID_ARG;
    }
    return DQ_OK;
}

static bool gradient_bits_ok(int b) { return b == 2 || b == 4 || b == 8 || b == 32; }

extern "C" int64_t dq_workspace_bytes(int32_t op, const dq_problem *prob, int64_t M, int64_t B)
{
    if (check_problem(prob) != DQ_OK) return DQ_ERR_INVALID_ARG;
    if (op != DQ_OP_FULL_GRAD && op != DQ_OP_VR_GRAD && op != DQ_OP_WORKER_STEP) return DQ_ERR_INVALID_ARG;
    if (op != DQ_OP_FULL_GRAD && (M <= 0 || B <= 0)) return DQ_ERR_INVALID_ARG;
    // (only CSR problems keep data between the rounds of a dq_run_rounds call)
    const int64_t bytes = prob->layout == 0 ? dense_workspace_bytes(op == DQ_OP_FULL_GRAD ? op : DQ_OP_VR_GRAD, prob, M, B)
                                            : csr_workspace_bytes(op, prob, M, B);
    return bytes < 0 ? bytes : (bytes + 15) / 16 * 16;
}

__global__ void ws_zero_kernel(uint4 *p, int64_t n16)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < n16) p[i] = make_uint4(0u, 0u, 0u, 0u);
}

extern "C" int32_t dq_workspace_init(void *ws, int64_t ws_bytes, void *stream)
{
    if (!ws || ws_bytes < 0 || !aligned16(ws) || (ws_bytes % 16) != 0) return DQ_ERR_INVALID_ARG;
    const int64_t n16 = ws_bytes / 16;
    if (n16 == 0) return DQ_OK;
    ws_zero_kernel<<<dim3(static_cast<unsigned>(ceil_div(n16, 256))), dim3(256), 0, as_stream(stream)>>>(
        static_cast<uint4 *>(ws), n16);
    DQ_LAUNCH_CHECK();
    return DQ_OK;
}

extern "C" int32_t dq_full_grad(const dq_problem *prob, const float *x, float *g_out, float *z_out, double *obj_out,
                                void *ws, int64_t ws_bytes, void *stream)
{
    int32_t rc = check_problem(prob);
    if (rc != DQ_OK) return rc;
    if (!x || !g_out || !aligned16(x) || !aligned16(g_out) || (ws && !aligned16(ws))) return DQ_ERR_INVALID_ARG;
    return prob->layout == 0 ? dense_full_grad(prob, x, g_out, z_out, obj_out, ws, ws_bytes, as_stream(stream))
                             : csr_full_grad(prob, x, g_out, z_out, obj_out, ws, ws_bytes, as_stream(stream));
}

int32_t dq::worker_step_impl(const dq_problem *prob, const WorkerArgs &a, void *stream)
{
    int32_t rc = check_problem(prob);
    if (rc != DQ_OK) return rc;
    if (a.M <= 0 || a.B <= 0 || a.B > 0x7FFFFFFFll || !a.x_snap || !aligned16(a.x_snap)) return DQ_ERR_INVALID_ARG;
    if (!a.idx && !a.packed) return DQ_ERR_INVALID_ARG;          // only dq_worker_step can sample in the kernel
    if (!a.model_is_snapshot) {
        if (!a.xq || !aligned16(a.xq)) return DQ_ERR_INVALID_ARG;
        if (a.b_x < 2 || (a.b_x > 16 && a.b_x != 32)) return DQ_ERR_INVALID_ARG;
        if (a.b_x != 32 && !a.delta_x) return DQ_ERR_INVALID_ARG;
    }
    if (a.alpha_out && (!aligned16(a.alpha_out) || a.ld < prob->d || (a.M > 1 && a.ld % 4 != 0))) return DQ_ERR_INVALID_ARG;
    if (a.ws && !aligned16(a.ws)) return DQ_ERR_INVALID_ARG;
    return prob->layout == 0 ? dense_worker(prob, a, as_stream(stream)) : csr_worker(prob, a, as_stream(stream));
}

extern "C" int32_t dq_vr_grad(const dq_problem *prob, const int32_t *idx, int64_t M, int64_t B, const uint32_t *xq_packed,
                              const float *delta_x, int32_t b_x, int32_t model_is_snapshot, const float *x_snap,
                              const float *z_snap, float *alpha_out, int64_t ld, float *absmax_out, float *l1norm_out,
                              void *ws, int64_t ws_bytes, void *stream)
{
    if (!alpha_out || !absmax_out) return DQ_ERR_INVALID_ARG;
    WorkerArgs a{};
    a.idx = idx; a.M = M; a.B = B; a.xq = xq_packed; a.delta_x = delta_x; a.b_x = b_x;
    a.model_is_snapshot = model_is_snapshot; a.x_snap = x_snap; a.z_snap = z_snap;
    a.alpha_out = alpha_out; a.ld = ld; a.absmax_out = absmax_out; a.l1norm_out = l1norm_out;
    a.b = 8; a.ws = ws; a.ws_bytes = ws_bytes;
    return worker_step_impl(prob, a, stream);
}

extern "C" int32_t dq_worker_step(const dq_problem *prob, const int32_t *idx, int64_t M, int64_t B,
                                  const uint32_t *xq_packed, const float *delta_x, int32_t b_x, int32_t model_is_snapshot,
                                  const float *x_snap, const float *z_snap, int32_t sparsify, int32_t b, uint64_t seed,
                                  uint32_t iter, uint32_t worker0, uint32_t *packed_out, int64_t ld_words, float *delta_out,
                                  int32_t *nnz_out, float *alpha_out, int64_t ld, uint32_t *status, void *ws,
                                  int64_t ws_bytes, void *stream)
{
    if (!packed_out || !delta_out || !aligned16(packed_out) || !prob) return DQ_ERR_INVALID_ARG;
    if (b < 2 || (b > 8 && b != 32)) return DQ_ERR_INVALID_ARG;
    if (!gradient_bits_ok(b)) return DQ_ERR_UNSUPPORTED;
    const int64_t row_words = b == 32 ? prob->d : packed_words(prob->d, b);
    if (ld_words < row_words || (M > 1 && ld_words % 4 != 0)) return DQ_ERR_INVALID_ARG;
    WorkerArgs a{};
    a.idx = idx; a.M = M; a.B = B; a.xq = xq_packed; a.delta_x = delta_x; a.b_x = b_x;
    a.model_is_snapshot = model_is_snapshot; a.x_snap = x_snap; a.z_snap = z_snap;
    a.alpha_out = alpha_out; a.ld = ld;
    a.sparsify = sparsify; a.b = b; a.seed = seed; a.iter = iter; a.worker0 = worker0;
    a.packed = packed_out; a.ld_words = ld_words; a.delta_out = delta_out; a.nnz_out = nnz_out; a.status = status;
    a.ws = ws; a.ws_bytes = ws_bytes;
    return worker_step_impl(prob, a, stream);
}

extern "C" int32_t dq_worker_step_static(const dq_problem *prob, const int32_t *idx, int64_t M, int64_t B,
                                         const uint32_t *xq_packed, const float *delta_x, int32_t b_x,
                                         int32_t model_is_snapshot, const float *x_snap, const float *z_snap,
                                         int32_t sparsify, int32_t b, uint64_t seed, uint32_t iter, uint32_t worker0,
                                         uint32_t *packed_out, int64_t ld_words, float *delta_out, int32_t *nnz_out,
                                         float *alpha_out, int64_t ld, uint32_t *status, void *stream)
{
    const int64_t need = dq_workspace_bytes(DQ_OP_WORKER_STEP, prob, M, B);
    if (need < 0) return static_cast<int32_t>(need);
    if (need > kStaticWsBytes) return DQ_ERR_WORKSPACE;          // beyond the built-in workspace: use dq_worker_step
    void *ws = nullptr;
    const int32_t rc = static_workspace(&ws);
    if (rc != DQ_OK) return rc;
    return dq_worker_step(prob, idx, M, B, xq_packed, delta_x, b_x, model_is_snapshot, x_snap, z_snap, sparsify, b, seed,
                          iter, worker0, packed_out, ld_words, delta_out, nnz_out, alpha_out, ld, status, ws,
                          kStaticWsBytes, stream);
}
