// Optional per-kernel timing with HIP events on the launch stream (off by default; see lq_profile_enable).
#pragma once

#include <hip/hip_runtime.h>

namespace lq {
namespace prof {

enum Cls {
  GEMM_BASE = 0,            // + mode * 8 + (l/32 - 1): 16 classes of wide_gemm_kernel
  GEMM_FIXUP = 16,
  GRAM = 17,
  CHOLESKY = 18,
  TRSM = 19,
  JACOBI = 20,
  LOWRANK_BLOCKQUANT = 21,
  SCALEQUANT_ERROR = 22,
  RESIDUAL = 23,
  QUANTIZE = 24,
  DEQUANTIZE = 25,
  MISC = 26,
  GEMM_SPLIT_BASE = 27,     // + mode * 8 + (l/32 - 1): the bf16 hi/lo split variants of wide_gemm_kernel
  QMATMUL = 43,             // qmatmul_kernel (work = flops of the product)
  QMATVEC = 44,             // qmatvec_kernel (work = bytes)
  SPLIT_PROJECT = 45,       // split_project_kernel (work = bytes)
  GEMM_F16_BASE = 46,       // + planes * 8 + mode * 4 + (l/32 - 1): wide_gemm_f16_kernel (work = flops of the product)
  ABSMAX = 62,
  NUM_CLASSES = 63
};

bool enabled();
// Brackets the launches issued while it is alive.  `work`: algorithmic flops (GEMM classes) or bytes.
class Scope {
 public:
  Scope(int cls, hipStream_t st, double work);
  ~Scope();
 private:
  int slot_;
  hipStream_t st_;
};

}  // namespace prof
}  // namespace lq
