// Library-wide plumbing: version string and the thread-local record of the last HIP error.
#include "dq_common.h"

namespace dq {
static thread_local int32_t g_last_error = 0;
void set_last_error(hipError_t e) { g_last_error = static_cast<int32_t>(e); }
}  // namespace dq

extern "C" const char *dq_version(void) { return "dq 0.1 (gfx950)"; }
extern "C" int32_t dq_last_device_error(void) { return dq::g_last_error; }
