// C ABI of the forward product with a decomposed weight (Section 3.2 "Implementation", Appendix A).
#include <algorithm>
#include <mutex>

#include "kernels.h"

namespace lq {
int check_quant_args(int64_t n, lq_config& c);

static size_t up256(size_t b) { return (b + 255) & ~(size_t)255; }
static int64_t up32(int64_t x) { return (x + 31) & ~(int64_t)31; }

// Few rows of X: the product is bound by reading the weights and runs on the vector ALU (measured faster than the
// MFMA path up to 8 rows).
constexpr int64_t SMALL_M = QMATVEC_MAX_ROWS;
constexpr int SMALL_RANK = 512;
// Up to this many rows (and when the main kernel's reduction is cut into ranges anyway) the kernel that adds the
// ranges also adds the ranges of T = X L1 and the product T L2: one launch and the main kernel's dense steps less.
constexpr int64_t LEAN_M = 128;

struct MatmulPlan {
  bool small;
  bool fused;      // T = X L1 comes out of the pass that splits X (rank up to SPLIT_PROJECT_MAX_RANK)
  bool lean;       // fused, and T L2 is added by the kernel that adds the main kernel's reduction ranges
  int64_t r32, rows_pad;
  size_t x_plane, t_floats, t_plane, part_floats, scale_floats;   // elements
};
static MatmulPlan plan_matmul(int64_t m, int64_t d, int64_t k, int rank) {
  MatmulPlan p{};
  p.small = m <= SMALL_M && rank <= SMALL_RANK;
  if (p.small) {
    const int mc = (int)std::min<int64_t>(m, QMATVEC_MAX_ROWS);
    p.part_floats = qmatvec_part_floats(mc, d, k, rank);
    return p;
  }
  p.r32 = up32(rank);
  p.rows_pad = (m + 255) / 256 * 256;
  p.x_plane = (size_t)p.rows_pad * (size_t)d;
  p.fused = rank > 0 && rank <= SPLIT_PROJECT_MAX_RANK;
  p.lean = p.fused && m <= LEAN_M && qmatmul_splits(m, k, (int)(d / 32)) > 1;
  if (p.lean) {    // the ranges of T stay alive until the last kernel: a region of their own
    p.t_floats = split_project_part_floats(p.rows_pad, d);
    p.part_floats = qmatmul_part_floats(m, k, (int)(d / 32));
    p.scale_floats = (size_t)(d * k / 16);
    return p;
  }
  p.t_floats = rank > 0 && !p.fused ? (size_t)m * (size_t)p.r32 : 0;
  p.t_plane = rank > 0 ? (size_t)p.rows_pad * (size_t)p.r32 : 0;
  const size_t p1 = p.fused ? split_project_part_floats(p.rows_pad, d)
                            : rank > 0 ? qmatmul_part_floats(m, p.r32, (int)(d / 32)) : 0;
  const size_t p2 = qmatmul_part_floats(m, k, (int)(d / 32 + p.r32 / 32));
  p.part_floats = p1 > p2 ? p1 : p2;
  p.scale_floats = (size_t)(d * k / 16);            // one scale per block, block size at least 16
  return p;
}
static size_t plan_bytes(const MatmulPlan& p) {
  return 2 * up256(p.x_plane * 2) + up256(p.t_floats * 4) + 2 * up256(p.t_plane * 2) + up256(p.part_floats * 4) +
         up256(p.scale_floats * 4);
}

// Scratch of lq_matmul_few_rows_static: a fixed array in device memory (every GPU the library runs on holds its own copy
// until the process ends).  Host code never uses the array's name as an address: the device address is looked up once per
// device and kept.
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)4 << 20;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[64] = {nullptr};

static int static_scratch(void** out) {
  int dev = 0;
  LQ_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= 64) return LQ_ERR_HIP;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    LQ_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return LQ_ERR_HIP;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return LQ_OK;
}
}  // namespace lq

using namespace lq;

extern "C" {

size_t lq_matmul_workspace_bytes(int64_t m, int64_t d, int64_t k, int rank) {
  if (m <= 0 || d <= 0 || k <= 0 || rank < 0 || (d % 32) != 0) return 0;
  return plan_bytes(plan_matmul(m, d, k, rank)) + 256;
}

int lq_matmul(const float* X, int64_t m, int64_t d, int64_t k, const uint8_t* codes_packed, const uint8_t* scale_idx,
              const float* v, lq_config c, const float* L1, const float* L2, int rank, int precision, float* Y,
              void* workspace, size_t workspace_bytes, void* stream) {
  if (!X || !codes_packed || !scale_idx || !v || !Y) return LQ_ERR_NULL;
  if (rank < 0 || rank > 1024) return LQ_ERR_RANK;
  if (rank > 0 && (!L1 || !L2)) return LQ_ERR_NULL;
  if (m <= 0 || d <= 0 || k <= 0 || m >= ((int64_t)1 << 31) || d >= ((int64_t)1 << 31) || k >= ((int64_t)1 << 31))
    return LQ_ERR_SHAPE;
  if ((d % 32) != 0) return LQ_ERR_SHAPE;
  LQ_TRY(check_quant_args(d * k, c));
  if ((k % c.block) != 0) return LQ_ERR_SHAPE;
  if (precision != 0 && precision != 1) return LQ_ERR_ARG;
  if (((uintptr_t)X & 15) != 0 || ((uintptr_t)Y & 15) != 0 || (rank > 0 && ((uintptr_t)L2 & 15) != 0)) return LQ_ERR_ARG;
  const MatmulPlan p = plan_matmul(m, d, k, rank);
  if (p.rows_pad * d >= ((int64_t)1 << 31)) return LQ_ERR_SHAPE;   // planes are addressed with 32-bit byte offsets
  if (!p.small && d * k >= ((int64_t)1 << 31)) return LQ_ERR_SHAPE;   // and so are the codes
  const size_t need = plan_bytes(p) + 256;
  if (!workspace || ((uintptr_t)workspace & 255) != 0 || workspace_bytes < need) return LQ_ERR_WORKSPACE;
  char* w = reinterpret_cast<char*>(workspace);
  hipStream_t st = (hipStream_t)stream;
  if (p.small) {
    // plan_bytes lays the regions out in the same order with empty planes
    float* part = reinterpret_cast<float*>(w);           // the only region of the plan that is not empty
    const MvWeights q{codes_packed, scale_idx, v, c.bits, c.block, c.scale_block, scale_levels(c)};
    for (int64_t r0 = 0; r0 < m; r0 += QMATVEC_MAX_ROWS) {
      const int mc = (int)std::min<int64_t>(QMATVEC_MAX_ROWS, m - r0);
      LQ_TRY(launch_qmatvec(q, X + r0 * d, d, d, L1, L2, k, rank, mc, k, Y + r0 * k, k, part, p.part_floats, st));
    }
    return LQ_OK;
  }
  uint16_t* xh = reinterpret_cast<uint16_t*>(w); w += up256(p.x_plane * 2);
  uint16_t* xl = reinterpret_cast<uint16_t*>(w); w += up256(p.x_plane * 2);
  float* T = reinterpret_cast<float*>(w); w += up256(p.t_floats * 4);
  uint16_t* th = reinterpret_cast<uint16_t*>(w); w += up256(p.t_plane * 2);
  uint16_t* tl = reinterpret_cast<uint16_t*>(w); w += up256(p.t_plane * 2);
  float* part = reinterpret_cast<float*>(w); w += up256(p.part_floats * 4);
  float* bscale = reinterpret_cast<float*>(w);

  QmmPart none{};
  if (p.lean) {
    const BlockScales bs{scale_idx, v, d * k / c.block, c.scale_block, scale_levels(c), bscale};
    LQ_TRY(launch_split_project(X, m, d, d, p.rows_pad, L1, rank, precision, xh, xl, T, p.t_floats, nullptr, nullptr,
                                (int)p.r32, bs, st));
    const QmmPart q{xh, xl, d, codes_packed, bscale, c.bits, c.block};
    const DensePart nodense{};
    int splits = 1;
    LQ_TRY(launch_qmatmul(q, nodense, m, p.rows_pad, k, Y, k, part, p.part_floats, precision, st, &splits));
    // without ranges the main kernel has written X Q into Y: each thread then reads and rewrites its own outputs
    return launch_range_sum_lowrank(splits > 1 ? part : Y, (size_t)m * (size_t)k, splits, T,
                                    (size_t)p.rows_pad * SPLIT_PROJECT_MAX_RANK, SPLIT_PROJECT_MAX_RANK,
                                    split_project_splits(p.rows_pad, d), m, k, rank, L2, k, Y, k, st);
  }
  if (p.fused) {    // planes of X and of T = X L1 from one pass over X, the block scales of Q in the same launch
    const BlockScales bs{scale_idx, v, d * k / c.block, c.scale_block, scale_levels(c), bscale};
    LQ_TRY(launch_split_project(X, m, d, d, p.rows_pad, L1, rank, precision, xh, xl, part, p.part_floats, th, tl,
                                (int)p.r32, bs, st));
  } else {
    LQ_TRY(launch_block_scales(scale_idx, v, d * k / c.block, c.scale_block, scale_levels(c), bscale, st));
    LQ_TRY(launch_split_planes(X, m, d, d, p.rows_pad, xh, xl, st));
  }
  if (rank > 0 && !p.fused) {   // T = X L1, m x r32 with zero columns beyond r, then its planes
    DensePart xl1{xh, xl, d, L1, rank, d, rank};
    LQ_TRY(launch_qmatmul(none, xl1, m, p.rows_pad, p.r32, T, p.r32, part, p.part_floats, precision, st));
    LQ_TRY(launch_split_planes(T, m, p.r32, p.r32, p.rows_pad, th, tl, st));
  }
  QmmPart q{xh, xl, d, codes_packed, bscale, c.bits, c.block};
  DensePart tl2{th, tl, rank > 0 ? p.r32 : 0, L2, k, rank, k};
  return launch_qmatmul(q, tl2, m, p.rows_pad, k, Y, k, part, p.part_floats, precision, st);
}

size_t lq_matmul_few_rows_static_scratch_bytes(void) { return STATIC_SCRATCH_BYTES; }

int lq_matmul_few_rows_static(const float* X, int64_t m, int64_t d, int64_t k, const uint8_t* codes_packed,
                              const uint8_t* scale_idx, const float* v, lq_config c, const float* L1, const float* L2,
                              int rank, float* Y, void* stream) {
  if (!X || !codes_packed || !scale_idx || !v || !Y) return LQ_ERR_NULL;
  if (rank < 0 || rank > SMALL_RANK) return LQ_ERR_RANK;
  if (rank > 0 && (!L1 || !L2)) return LQ_ERR_NULL;
  if (m <= 0 || m > SMALL_M || d <= 0 || k <= 0 || d >= ((int64_t)1 << 31) || k >= ((int64_t)1 << 31)) return LQ_ERR_SHAPE;
  if ((d % 32) != 0) return LQ_ERR_SHAPE;
  LQ_TRY(check_quant_args(d * k, c));
  if ((k % c.block) != 0) return LQ_ERR_SHAPE;
  if (((uintptr_t)X & 15) != 0 || ((uintptr_t)Y & 15) != 0 || (rank > 0 && ((uintptr_t)L2 & 15) != 0)) return LQ_ERR_ARG;
  const size_t part_floats = qmatvec_part_floats((int)m, d, k, rank);
  if (part_floats * sizeof(float) > STATIC_SCRATCH_BYTES) return LQ_ERR_WORKSPACE;   // beyond the fixed scratch: use lq_matmul
  void* sp = nullptr;
  LQ_TRY(static_scratch(&sp));
  const MvWeights q{codes_packed, scale_idx, v, c.bits, c.block, c.scale_block, scale_levels(c)};
  // every partial sum the second kernel reads is written by the first in the same call: nothing has to start at zero
  return launch_qmatvec(q, X, d, d, L1, L2, k, rank, (int)m, k, Y, k, reinterpret_cast<float*>(sp),
                        STATIC_SCRATCH_BYTES / sizeof(float), (hipStream_t)stream);
}

}  // extern "C"
