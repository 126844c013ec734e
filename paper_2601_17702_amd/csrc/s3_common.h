// Internal declarations shared by the library's translation units (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/s3attn.h"

int s3_fail(int code, const char* fmt, ...);   // records the thread-local message, returns code

#define S3_HIP(call)                                                                     \
    do {                                                                                 \
        hipError_t e_ = (call);                                                          \
        if (e_ != hipSuccess)                                                            \
            return s3_fail(S3_EHIP, "%s failed: %s", #call, hipGetErrorString(e_));      \
    } while (0)

static inline size_t s3_align(size_t n, size_t a = 256) { return (n + a - 1) / a * a; }
static inline int s3_ceil_log2(unsigned v) {
    int b = 0;
    while ((1u << b) < v) ++b;
    return b;
}

// Read-only view of an index for the scoring translation unit (defined in index.hip).
void s3_index_view(const s3_index* idx, int* n_heads, int* n_feat, int* k, int64_t* tokens,
                   const int32_t** offsets, int64_t* off_stride, const int32_t** positions,
                   int64_t* pos_stride, bool* finalized);
