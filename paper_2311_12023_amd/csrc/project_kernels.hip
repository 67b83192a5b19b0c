// First stage of the forward product Y = X (Q + L1 L2) (Section 3.2 "Implementation"): one pass over X that
//   - writes the bf16 hi / lo planes of X which the main kernel's operand transfers read, and
//   - computes T = X L1 (m x r, r <= 64) from the same registers,
// so that X is read from HBM once, as fp32, and the narrow product costs no pass of its own.
//
// Mapping: a workgroup of 256 threads owns 64 rows of X and a contiguous range of the reduction, walked in 64-deep
// steps.  Per step every thread loads four float4 of X (16 lanes cover 256 contiguous bytes of a row) and four float4
// of L1, one step ahead of their use; it splits them into bf16 halves, stores the X halves to the planes (128
// contiguous bytes per 16 lanes) and both operands to LDS (rows = output rows or output columns, 64 reduction indices
// contiguous, pitch 72 so that the 128-bit operand reads are conflict-free).  Each of the four wavefronts owns one
// 32 x 32 tile of the 64 x 64 result and issues v_mfma_f32_32x32x16_bf16 for hi*lo + lo*hi + hi*hi (fp32
// accumulation; the bf16-only variant keeps hi*hi and leaves the lo plane unwritten).  The kernel is bound by the
// HBM traffic of X and its planes; four workgroups fit a CU and cover each other's barriers.
// The partial tiles of the reduction ranges go to scratch; a second kernel sums them in range order and writes T
// directly as bf16 planes, the form in which the main kernel consumes it.  Extra rows of the grid reconstruct the
// block scales of Q (they depend on the weights alone), which saves the forward product a launch.
#include <algorithm>

#include "kernels.h"
#include "nf_device.h"
#include "profiler.h"

namespace lq {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));

constexpr int XP_ROWS = 64, XP_COLS = 64, XP_BK = 64, XP_THREADS = 256, XP_PITCH = 72;

struct XpArgs {
  const float* X; int64_t m, K, ldx;         // rows beyond m read as zero
  const float* L1; int rank;                 // K x rank, leading dimension rank
  int l1_vec;                                // rank % 4 == 0 and L1 16-byte aligned: whole float4 loads
  uint16_t* xh; uint16_t* xl;                // planes, rows_pad x K
  float* part; int64_t rows_pad;             // splits x rows_pad x 64
  int nsteps, splits;
  // the reconstructed block scales of Q ride along in extra grid rows (nblocks == 0: none)
  const uint8_t* sidx; const float* v; float* bscale; int64_t nblocks; int group_shift, levels;
};

// hi = bf16(v), lo = bf16(v - hi): v = hi + lo + O(2^-17 v).
__device__ __forceinline__ void xp_split(floatx4 v, bf16x4& hi, bf16x4& lo) {
  hi = __builtin_convertvector(v, bf16x4);
  lo = __builtin_convertvector(v - __builtin_convertvector(hi, floatx4), bf16x4);
}

// Registers of one step: the thread's four pieces of the X tile (rows tid / 16 + 16 i, reduction indices
// 4 (tid % 16) ..) and its 4 x 4 patch of L1 (reduction indices 4 (tid / 16) + j, columns 4 (tid % 16) ..).
struct XpRegs { floatx4 x[4], w[4]; };

__device__ __forceinline__ void xp_load(const XpArgs& a, int64_t row0, int step, int tid, XpRegs& r) {
  const int64_t k0 = (int64_t)step * XP_BK;
  const int64_t kx = k0 + 4 * (tid & 15);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int64_t row = row0 + (tid >> 4) + 16 * i;
    r.x[i] = (row < a.m && kx < a.K) ? *reinterpret_cast<const floatx4*>(a.X + row * a.ldx + kx) : floatx4{0.f, 0.f, 0.f, 0.f};
  }
  const int col = 4 * (tid & 15);
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int64_t kr = k0 + 4 * (tid >> 4) + j;
    floatx4 w = {0.f, 0.f, 0.f, 0.f};
    if (kr < a.K) {
      const float* p = a.L1 + kr * a.rank + col;
      if (a.l1_vec) {
        if (col < a.rank) w = *reinterpret_cast<const floatx4*>(p);
      } else {
        if (col + 0 < a.rank) w.x = p[0];
        if (col + 1 < a.rank) w.y = p[1];
        if (col + 2 < a.rank) w.z = p[2];
        if (col + 3 < a.rank) w.w = p[3];
      }
    }
    r.w[j] = w;
  }
}

template <bool SPLIT>
__global__ __launch_bounds__(XP_THREADS, 4) void split_project_kernel(XpArgs a) {
  __shared__ __attribute__((aligned(16))) __bf16 s_a[2][XP_ROWS * XP_PITCH];    // [hi, lo][row][k]
  __shared__ __attribute__((aligned(16))) __bf16 s_b[2][XP_COLS * XP_PITCH];    // [hi, lo][column][k]
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, ln = lane & 31, lh = lane >> 5;
  const int tr = wave >> 1, tc = wave & 1;
  const int64_t row0 = (int64_t)blockIdx.x * XP_ROWS;
  const int split = blockIdx.y;
  if (split >= a.splits) {                   // s^ of every block: fl32(index * fl32(v / levels)), as in Dequantize
    const int64_t wg = (int64_t)(split - a.splits) * gridDim.x + blockIdx.x, nwg = (int64_t)(gridDim.y - a.splits) * gridDim.x;
    for (int64_t b = wg * XP_THREADS + tid; b < a.nblocks; b += nwg * XP_THREADS)
      a.bscale[b] = block_scale(a.sidx[b], a.v[b >> a.group_shift], a.levels);
    return;
  }
  const int s0 = (int)((int64_t)a.nsteps * split / a.splits), s1 = (int)((int64_t)a.nsteps * (split + 1) / a.splits);

  floatx16 acc;
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[e] = 0.0f;

  XpRegs r;
  if (s0 < s1) xp_load(a, row0, s0, tid, r);
  for (int s = s0; s < s1; ++s) {
    // registers -> planes and LDS
    const int64_t kx = (int64_t)s * XP_BK + 4 * (tid & 15);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = (tid >> 4) + 16 * i;
      bf16x4 hi, lo;
      xp_split(r.x[i], hi, lo);
      *reinterpret_cast<bf16x4*>(&s_a[0][row * XP_PITCH + 4 * (tid & 15)]) = hi;
      if constexpr (SPLIT) *reinterpret_cast<bf16x4*>(&s_a[1][row * XP_PITCH + 4 * (tid & 15)]) = lo;
      if (kx < a.K) {                        // rows up to rows_pad are written: zero beyond m
        *reinterpret_cast<bf16x4*>(a.xh + (row0 + row) * a.K + kx) = hi;
        if constexpr (SPLIT) *reinterpret_cast<bf16x4*>(a.xl + (row0 + row) * a.K + kx) = lo;
      }
    }
#pragma unroll
    for (int c = 0; c < 4; ++c) {            // column 4 (tid % 16) + c of L1, reduction indices 4 (tid / 16) .. + 3
      const floatx4 f = {r.w[0][c], r.w[1][c], r.w[2][c], r.w[3][c]};
      bf16x4 hi, lo;
      xp_split(f, hi, lo);
      const int at = (4 * (tid & 15) + c) * XP_PITCH + 4 * (tid >> 4);
      *reinterpret_cast<bf16x4*>(&s_b[0][at]) = hi;
      if constexpr (SPLIT) *reinterpret_cast<bf16x4*>(&s_b[1][at]) = lo;
    }
    __syncthreads();
    if (s + 1 < s1) xp_load(a, row0, s + 1, tid, r);
#pragma unroll
    for (int kk = 0; kk < XP_BK / 16; ++kk) {
      const int ao = (32 * tr + ln) * XP_PITCH + 16 * kk + 8 * lh, bo = (32 * tc + ln) * XP_PITCH + 16 * kk + 8 * lh;
      const bf16x8 ah = *reinterpret_cast<const bf16x8*>(&s_a[0][ao]);
      const bf16x8 bh = *reinterpret_cast<const bf16x8*>(&s_b[0][bo]);
      if constexpr (SPLIT) {
        const bf16x8 al = *reinterpret_cast<const bf16x8*>(&s_a[1][ao]);
        const bf16x8 bl = *reinterpret_cast<const bf16x8*>(&s_b[1][bo]);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, bh, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bl, acc, 0, 0, 0);
      }
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bh, acc, 0, 0, 0);
    }
    __syncthreads();                         // the tiles are overwritten by the next step
  }

  // accumulator element e of a lane is row 8 * (e / 4) + 4 * lh + e % 4, column ln of the wavefront's tile
  float* __restrict__ out = a.part + ((size_t)split * (size_t)a.rows_pad + (size_t)row0 + 32 * tr) * XP_COLS + 32 * tc + ln;
#pragma unroll
  for (int e = 0; e < 16; ++e) out[(size_t)(8 * (e >> 2) + 4 * lh + (e & 3)) * XP_COLS] = acc[e];
}

// T = sum of the partial tiles in range order, written as bf16 planes of rows_pad x Kd (the first Kd of the 64 columns).
__global__ __launch_bounds__(256) void project_finish_kernel(const float* __restrict__ part, int splits, int64_t rows_pad,
                                                             int Kd, uint16_t* __restrict__ th, uint16_t* __restrict__ tl) {
  const int64_t q = Kd >> 2, total = rows_pad * q, stride = rows_pad * XP_COLS;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int64_t row = i / q, c4 = (i % q) << 2;
    const float* p = part + row * XP_COLS + c4;
    floatx4 sum = {0.f, 0.f, 0.f, 0.f};
    for (int s0 = 0; s0 < splits; s0 += 8) {       // the loads issued eight at a time
      floatx4 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u)
        v[u] = s0 + u < splits ? *reinterpret_cast<const floatx4*>(p + (int64_t)(s0 + u) * stride) : floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int u = 0; u < 8; ++u) sum += v[u];
    }
    bf16x4 hi, lo;
    xp_split(sum, hi, lo);
    *reinterpret_cast<bf16x4*>(th + row * Kd + c4) = hi;
    *reinterpret_cast<bf16x4*>(tl + row * Kd + c4) = lo;
  }
}

int split_project_splits(int64_t rows_pad, int64_t K) {
  const int64_t tiles = rows_pad / XP_ROWS, nsteps = (K + XP_BK - 1) / XP_BK;
  const int64_t want = (1024 + tiles - 1) / tiles;
  return (int)std::max<int64_t>(1, std::min<int64_t>(std::min<int64_t>(want, nsteps / 2), 16));
}

size_t split_project_part_floats(int64_t rows_pad, int64_t K) {
  return (size_t)split_project_splits(rows_pad, K) * (size_t)rows_pad * XP_COLS;
}

int launch_split_project(const float* X, int64_t m, int64_t K, int64_t ldx, int64_t rows_pad, const float* L1, int rank,
                         int precision, uint16_t* xh, uint16_t* xl, float* part, size_t part_floats, uint16_t* th,
                         uint16_t* tl, int Kd, const BlockScales& bs, hipStream_t st) {
  if (m <= 0 || K <= 0 || (K & 3) != 0 || (ldx & 3) != 0 || rows_pad < m || (rows_pad % XP_ROWS) != 0) return LQ_ERR_SHAPE;
  if (rank < 1 || rank > SPLIT_PROJECT_MAX_RANK || (Kd != 32 && Kd != 64) || Kd < rank) return LQ_ERR_RANK;
  if (((uintptr_t)X & 15) != 0) return LQ_ERR_ARG;
  XpArgs a{};
  a.X = X; a.m = m; a.K = K; a.ldx = ldx;
  a.L1 = L1; a.rank = rank;
  a.l1_vec = ((rank & 3) == 0 && ((uintptr_t)L1 & 15) == 0) ? 1 : 0;
  a.xh = xh; a.xl = xl; a.part = part; a.rows_pad = rows_pad;
  a.nsteps = (int)((K + XP_BK - 1) / XP_BK);
  a.splits = split_project_splits(rows_pad, K);
  if (part_floats < (size_t)a.splits * (size_t)rows_pad * XP_COLS) return LQ_ERR_WORKSPACE;
  if (bs.nblocks > 0) {
    if (bs.scale_block < 1 || (bs.scale_block & (bs.scale_block - 1)) != 0) return LQ_ERR_SHAPE;
    a.sidx = bs.sidx; a.v = bs.v; a.bscale = bs.out; a.nblocks = bs.nblocks;
    a.group_shift = __builtin_ctz((unsigned)bs.scale_block); a.levels = bs.levels;
  }
  // about four blocks per thread for the scales, at most 1024 workgroups
  const int64_t tiles = rows_pad / XP_ROWS;
  const int64_t scale_wgs = std::min<int64_t>((bs.nblocks + 4 * XP_THREADS - 1) / (4 * XP_THREADS), 1024);
  const int64_t scale_rows = (scale_wgs + tiles - 1) / tiles;
  const dim3 grid((unsigned)tiles, (unsigned)(a.splits + scale_rows));
  {
    // X read once, the planes written; the MFMA work rides along
    prof::Scope ps(prof::SPLIT_PROJECT, st, (double)rows_pad * (double)K * (precision == 0 ? 8.0 : 6.0));
    if (precision == 0) hipLaunchKernelGGL(split_project_kernel<true>, grid, dim3(XP_THREADS), 0, st, a);
    else hipLaunchKernelGGL(split_project_kernel<false>, grid, dim3(XP_THREADS), 0, st, a);
    LQ_HIP_TRY(hipGetLastError());
  }
  if (!th) return LQ_OK;                     // the caller adds the ranges of T itself
  prof::Scope ps(prof::MISC, st, (double)(a.splits + 1) * (double)rows_pad * XP_COLS * 4.0);
  const int64_t total = rows_pad * (Kd >> 2);
  hipLaunchKernelGGL(project_finish_kernel, dim3((unsigned)std::min<int64_t>((total + 255) / 256, 4096)), dim3(256), 0, st,
                     part, a.splits, rows_pad, Kd, th, tl);
  LQ_HIP_TRY(hipGetLastError());
  return LQ_OK;
}

}  // namespace lq
