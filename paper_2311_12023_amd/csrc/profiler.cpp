#include "profiler.h"

#include <mutex>
#include <vector>

#include "lq_internal.h"

namespace lq {
namespace prof {

struct Rec { int cls; hipEvent_t a, b; double work; };
static bool g_on = false;
static std::vector<Rec> g_recs;        // every bracket since the last reset
static std::vector<hipEvent_t> g_pool; // events free for reuse
static std::mutex g_mu;

bool enabled() { return g_on; }

static hipEvent_t take_event() {
  if (!g_pool.empty()) { hipEvent_t e = g_pool.back(); g_pool.pop_back(); return e; }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}

Scope::Scope(int cls, hipStream_t st, double work) : slot_(-1), st_(st) {
  if (!g_on) return;
  std::lock_guard<std::mutex> lock(g_mu);
  Rec r; r.cls = cls; r.work = work; r.a = take_event(); r.b = take_event();
  if (!r.a || !r.b) return;
  (void)hipEventRecord(r.a, st);
  g_recs.push_back(r);
  slot_ = (int)g_recs.size() - 1;
}

Scope::~Scope() {
  if (slot_ < 0) return;
  std::lock_guard<std::mutex> lock(g_mu);
  (void)hipEventRecord(g_recs[slot_].b, st_);
}

static const char* const kNames[NUM_CLASSES] = {
    "wide_gemm_kernel<1,0,2,0>", "wide_gemm_kernel<2,0,2,0>", "wide_gemm_kernel<3,0,2,0>", "wide_gemm_kernel<4,0,2,0>",
    "wide_gemm_kernel<5,0,1,0>", "wide_gemm_kernel<6,0,1,0>", "wide_gemm_kernel<7,0,1,0>", "wide_gemm_kernel<8,0,1,0>",
    "wide_gemm_kernel<1,1,2,0>", "wide_gemm_kernel<2,1,2,0>", "wide_gemm_kernel<3,1,2,0>", "wide_gemm_kernel<4,1,2,0>",
    "wide_gemm_kernel<5,1,1,0>", "wide_gemm_kernel<6,1,1,0>", "wide_gemm_kernel<7,1,1,0>", "wide_gemm_kernel<8,1,1,0>",
    "gemm_fixup_kernel", "gram_partial_kernel+gram_reduce_kernel", "cholesky_kernel", "trsm_kernel",
    "jacobi_eig_kernel", "lowrank_blockquant_kernel", "scalequant_error_kernel+error_finalize_kernel",
    "residual_kernel", "quantize_fused_kernel", "dequant_kernel", "misc",
    "wide_gemm_kernel<1,0,2,1>", "wide_gemm_kernel<2,0,2,1>", "wide_gemm_kernel<3,0,2,1>", "wide_gemm_kernel<4,0,2,1>",
    "wide_gemm_kernel<5,0,1,1>", "wide_gemm_kernel<6,0,1,1>", "wide_gemm_kernel<7,0,1,1>", "wide_gemm_kernel<8,0,1,1>",
    "wide_gemm_kernel<1,1,2,1>", "wide_gemm_kernel<2,1,2,1>", "wide_gemm_kernel<3,1,2,1>", "wide_gemm_kernel<4,1,2,1>",
    "wide_gemm_kernel<5,1,1,1>", "wide_gemm_kernel<6,1,1,1>", "wide_gemm_kernel<7,1,1,1>", "wide_gemm_kernel<8,1,1,1>",
    "qmatmul_kernel", "qmatvec_kernel", "split_project_kernel",
    "wide_gemm_f16_kernel<1,0,1>", "wide_gemm_f16_kernel<2,0,1>", "wide_gemm_f16_kernel<3,0,1>", "wide_gemm_f16_kernel<4,0,1>",
    "wide_gemm_f16_kernel<1,1,1>", "wide_gemm_f16_kernel<2,1,1>", "wide_gemm_f16_kernel<3,1,1>", "wide_gemm_f16_kernel<4,1,1>",
    "wide_gemm_f16_kernel<1,0,2>", "wide_gemm_f16_kernel<2,0,2>", "wide_gemm_f16_kernel<3,0,2>", "wide_gemm_f16_kernel<4,0,2>",
    "wide_gemm_f16_kernel<1,1,2>", "wide_gemm_f16_kernel<2,1,2>", "wide_gemm_f16_kernel<3,1,2>", "wide_gemm_f16_kernel<4,1,2>",
    "absmax_kernel"};

}  // namespace prof
}  // namespace lq

using namespace lq::prof;

extern "C" {

int lq_profile_enable(int on) {
  std::lock_guard<std::mutex> lock(g_mu);
  g_on = on != 0;
  return LQ_OK;
}

int lq_profile_reset(void) {
  if (hipDeviceSynchronize() != hipSuccess) return LQ_ERR_HIP;
  std::lock_guard<std::mutex> lock(g_mu);
  for (auto& r : g_recs) { g_pool.push_back(r.a); g_pool.push_back(r.b); }
  g_recs.clear();
  return LQ_OK;
}

int lq_profile_num_classes(void) { return NUM_CLASSES; }

const char* lq_profile_class_name(int cls) { return (cls >= 0 && cls < NUM_CLASSES) ? kNames[cls] : ""; }

int lq_profile_read(int cls, double* total_ms, int64_t* launches, double* work) {
  if (cls < 0 || cls >= NUM_CLASSES) return LQ_ERR_ARG;
  if (hipDeviceSynchronize() != hipSuccess) return LQ_ERR_HIP;
  std::lock_guard<std::mutex> lock(g_mu);
  double ms = 0, wk = 0; int64_t n = 0;
  for (auto& r : g_recs) {
    if (r.cls != cls) continue;
    float t = 0;
    if (hipEventElapsedTime(&t, r.a, r.b) != hipSuccess) continue;
    ms += t; wk += r.work; ++n;
  }
  if (total_ms) *total_ms = ms;
  if (launches) *launches = n;
  if (work) *work = wk;
  return LQ_OK;
}

}  // extern "C"
