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
