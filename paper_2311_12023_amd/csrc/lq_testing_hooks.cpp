// Test hooks (include/lq_testing.h): single kernels of the randomized SVD, the host evaluation of the code search and
// the capture of one configuration's iterate inside the sweep.  This file is compiled only into the testing build of
// the library (liblq_hip_testing.so, everything compiled with -DLQ_TESTING_HOOKS); the product library exports none of it.
#include <cmath>

#include "../../include/lq_testing.h"
#include "kernels.h"
#include "nf_device.h"
#include "testing_capture.h"

namespace lq {
size_t lds_limit_for_tests();
namespace testing {
Capture& capture() {
  static thread_local Capture c;
  return c;
}
}  // namespace testing
}  // namespace lq

using namespace lq;

extern "C" {

int lq_test_capture_iterate(int cfg_index, int iter, float* Q_dense, double* sigma_next) {
  testing::Capture& c = testing::capture();
  c = testing::Capture();
  if (cfg_index < 0) return LQ_OK;                      // disarm
  if (iter < 1 || !Q_dense) return LQ_ERR_ARG;
  c.armed = true; c.cfg = cfg_index; c.iter = iter; c.Q = Q_dense; c.sigma = sigma_next;
  return LQ_OK;
}

int lq_test_wide_gemm(int mode, int l, int64_t big, int64_t K, const float* X, int64_t ldx, const float* A,
                      int64_t lda, float* C, int64_t ldc, int batch, int workgroups, float* part, size_t part_floats,
                      int precision, void* stream) {
  if (!X || !A || !C) return LQ_ERR_NULL;
  if ((precision != 0 && precision != 1) || workgroups < -32768 || workgroups > 32768 || batch < 1) return LQ_ERR_ARG;
  const size_t sA = (size_t)(mode == MODE_NT ? big : K) * lda;
  return launch_wide_gemm(mode, l, big, K, X, ldx, (size_t)l * ldx, A, lda, sA, C, ldc, (size_t)l * ldc, batch, part,
                          part_floats, (hipStream_t)stream, precision, workgroups);
}

int lq_test_wide_gemm_f16(int mode, int l, int64_t big, int64_t K, const float* X, int64_t ldx, const uint16_t* A,
                          const uint8_t* A_lo, int64_t lda, float* C, int64_t ldc, int batch, int workgroups, float* part, size_t part_floats,
                          float x_scale, const double* lam0, float out_scale, void* stream) {
  if (!X || !A || !C) return LQ_ERR_NULL;
  if (workgroups < -32768 || workgroups > 32768 || batch < 1) return LQ_ERR_ARG;
  const size_t sA = (size_t)(mode == MODE_NT ? big : K) * lda;
  return launch_wide_gemm_f16(mode, l, big, K, X, ldx, (size_t)l * ldx, A, A_lo, lda, sA, C, ldc, (size_t)l * ldc, batch, part,
                              part_floats, x_scale, lam0, 1, out_scale, (hipStream_t)stream, workgroups);
}

size_t lq_test_wide_gemm_part_floats(int l, int workgroups) {
  if (l % 32 != 0 || l < 32 || l > 256) return 0;
  return gemm_part_floats(l, workgroups);
}

int lq_test_orthonormalize(float* X, int l, int64_t m, int64_t ldx, double* scratch, float* alt, void* stream) {
  if (!X || !scratch) return LQ_ERR_NULL;
  if (l % 32 || l < 32 || l > 256) return LQ_ERR_ARG;
  double* G = scratch;
  double* part = scratch + (size_t)l * l;
  LQ_TRY(launch_gram(X, l, m, ldx, 0, part, G, 1, (hipStream_t)stream));
  if (cholinv_supported(l) && alt) {
    float* Cinv = reinterpret_cast<float*>(part);       // the Gram partials are dead by now
    LQ_TRY(launch_cholinv(G, l, Cinv, 1, (hipStream_t)stream));
    LQ_TRY(launch_wide_gemm(MODE_NN, l, ldx, l, Cinv, l, 0, X, ldx, 0, alt, ldx, 0, 1, nullptr, 0, (hipStream_t)stream));
    LQ_HIP_TRY(hipMemcpyAsync(X, alt, (size_t)l * ldx * sizeof(float), hipMemcpyDeviceToDevice, (hipStream_t)stream));
    return LQ_OK;
  }
  LQ_TRY(launch_cholesky(G, l, 1, (hipStream_t)stream));
  return launch_trsm(G, l, X, m, ldx, 0, 1, (hipStream_t)stream);
}

int lq_test_sym_eig(double* G, int l, float* Ut, double* lambda, double* scratch, void* stream) {
  if (!G || !Ut || !lambda || !scratch) return LQ_ERR_NULL;
  if (l % 2 || l < 2 || l > 256) return LQ_ERR_ARG;
  return launch_jacobi_eig(G, l, scratch, Ut, lambda, 1, (hipStream_t)stream);
}

int lq_test_sym_eig_fast(const double* G, int l, float* Ut, double* lambda, void* stream) {
  if (!G || !Ut || !lambda) return LQ_ERR_NULL;
  if (!jacobi_fast_supported(l)) return LQ_ERR_ARG;
  return launch_jacobi_fast(G, l, Ut, lambda, 1, (hipStream_t)stream);
}

int lq_test_lincomb3(float* X, float a, const float* Y, float b, const float* Z, float c, int l, int64_t ldx, void* stream) {
  if (!X || !Y) return LQ_ERR_NULL;
  if (l < 1 || ldx < 4 || ldx % 4) return LQ_ERR_ARG;
  return launch_lincomb3(X, a, Y, b, Z, c, (int64_t)l * ldx, (hipStream_t)stream);
}

int lq_test_deflate_rows(float* X, const float* L, int l, int locked, int64_t m, int64_t ldx, void* stream) {
  if (!X || !L) return LQ_ERR_NULL;
  if (l < 1 || m < 1 || m > ldx || locked > l) return LQ_ERR_ARG;
  return launch_deflate_rows(X, L, l, locked, m, ldx, (hipStream_t)stream);
}

int lq_test_ritz_residual(const float* G, const float* Y, const double* lam, int rows, int64_t m, int64_t ldx, double* res,
                          void* stream) {
  if (!G || !Y || !lam || !res) return LQ_ERR_NULL;
  if (rows < 1 || m < 1 || m > ldx) return LQ_ERR_ARG;
  return launch_ritz_residual(G, Y, lam, rows, m, ldx, res, (hipStream_t)stream);
}

int lq_test_bucket_code(int bits, float x) {
  const int slot = bits_slot(bits);
  if (slot < 0) return -1;
  const HostTables& t = host_tables();
  // the search of the decomposition's quantize pass (search_code in fused_kernels.hip): bucket table, then one
  // comparison (two for 8 bits); the stand-alone quantizer counts thresholds for 2 and 3 bits, which is the definition
  int j = (int)std::fmaf(x, 256.0f, 256.0f);
  if (!(std::fmaf(x, 256.0f, 256.0f) >= 0.0f)) j = 0;   // NaN and negatives as the device's conversion treats them
  j = j < 0 ? 0 : (j > 513 ? 513 : j);
  const int c0 = t.lut[slot][j < 511 ? j : 511];
  if (bits <= 4) return c0 + (x >= t.thr[slot][c0]);          // one threshold per bucket at most
  return c0 + (x >= t.thr[slot][c0]) + (x >= t.thr[slot][c0 + 1]);
}

size_t lq_test_lds_limit(void) { return lds_limit_for_tests(); }

}  // extern "C"
