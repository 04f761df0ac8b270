// Error state, version and small host utilities of libhyb.
#include "common.h"

#include <string.h>

static thread_local char g_err[512] = "no error";

int hyb_set_error(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

int hyb_check_launch(const char* what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hyb_set_error(HYB_ERR_LAUNCH, "%s: kernel launch failed: %s", what, hipGetErrorString(e));
    return HYB_OK;
}

extern "C" int hyb_version(void) { return 100; }

extern "C" const char* hyb_last_error_string(void) { return g_err; }
