#include "s3_common.h"
struct s3_index { int dummy; };
extern "C" {
int s3_index_create(int, int, int, int64_t, s3_index**) { return s3_fail(S3_ESTATE, "not implemented"); }
void s3_index_destroy(s3_index*) {}
int s3_index_append(s3_index*, const int32_t*, int, const int32_t*, int32_t, void*) { return s3_fail(S3_ESTATE, "not implemented"); }
int s3_index_finalize(s3_index*, void*) { return s3_fail(S3_ESTATE, "not implemented"); }
int s3_index_csr(const s3_index*, int, const int32_t**, const int32_t**, int64_t*) { return s3_fail(S3_ESTATE, "not implemented"); }
int s3_index_export(const s3_index*, int, int32_t*, int32_t*, void*) { return s3_fail(S3_ESTATE, "not implemented"); }
int64_t s3_index_tokens(const s3_index*) { return 0; }
size_t s3_index_build_workspace(int, int, int) { return 0; }
int s3_index_build(const int32_t*, const int32_t*, int, int, int, int32_t*, int32_t*, void*, size_t, void*) { return s3_fail(S3_ESTATE, "not implemented"); }
size_t s3_coactivate_score_workspace(const s3_index*, int64_t) { return 0; }
int s3_coactivate_score(const s3_index*, const int32_t*, const float*, int, int64_t, int, int, int32_t, int, float*, int32_t*, float*, int32_t*, void*, size_t, void*) { return s3_fail(S3_ESTATE, "not implemented"); }
}
