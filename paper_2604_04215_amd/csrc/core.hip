// Error reporting and version of libdlm.
#include "common.hpp"

namespace dlm {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
}

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

int check_hip(hipError_t e, const char* what) {
    if (e == hipSuccess) return DLM_OK;
    return fail(DLM_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

}  // namespace dlm

extern "C" const char* dlm_last_error(void) { return dlm::g_err; }
extern "C" int dlm_version(void) { return 100; }
