// Error reporting shared by the C-ABI entry points.
#include "s3_common.h"

#include <stdarg.h>
#include <stdio.h>

static thread_local char g_err[512] = "";

int s3_fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

extern "C" const char* s3_last_error(void) { return g_err; }

int s3_allow_lds(S3LdsOnce& once, const void* kernel, int bytes) {
    int dev = 0;
    S3_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kS3MaxDevices) {      // beyond the table: set it on every call
        S3_HIP(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes));
        return S3_OK;
    }
    std::call_once(once.flag[dev], [&] {
        once.err[dev] = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    });
    if (once.err[dev] != hipSuccess)
        return s3_fail(S3_EHIP, "hipFuncSetAttribute failed: %s", hipGetErrorString(once.err[dev]));
    return S3_OK;
}
