// C ABI, part 2 (placeholder while the decomposition kernels are being brought up).
#include "lq_internal.h"
extern "C" {
size_t lq_factorize_workspace_bytes(int64_t, int64_t, int, const lq_svd_params*) { return 0; }
int lq_factorize(const float*, int64_t, int64_t, int, const float*, const float*, uint64_t, const lq_svd_params*,
                 float*, float*, double*, void*, size_t, void*) { return LQ_ERR_ARG; }
size_t lq_decompose_workspace_bytes(int64_t, int64_t, int, const lq_svd_params*) { return 0; }
int lq_decompose(const float*, int64_t, int64_t, int, lq_config, int, int, const float*, const float*, uint64_t,
                 const lq_svd_params*, float*, float*, uint8_t*, uint8_t*, float*, float*, double*, double*, int32_t*,
                 double*, void*, size_t, void*) { return LQ_ERR_ARG; }
size_t lq_error_table_workspace_bytes(int64_t, int64_t, int, int, const lq_svd_params*) { return 0; }
int lq_error_table(const float*, int64_t, int64_t, int, const lq_config*, int, int, int, const float*, const float*,
                   uint64_t, const lq_svd_params*, double*, double*, double*, void*, size_t, void*) { return LQ_ERR_ARG; }
}
