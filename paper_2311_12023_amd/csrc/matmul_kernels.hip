// Forward product with an LQ-decomposed weight, Y = X (Q + L1 L2), with Q dequantized just in time inside the GEMM
// (Section 3.2 "Implementation" and Appendix A: matrix products between fp32 inputs and quantized matrices).
//
// One kernel computes  Y[m x N] = Xq[m x Kq] * dequant(codes)[Kq x N]  +  Xd[m x Kd] * D[Kd x N]  where either part
// may be empty.  The forward product is two launches of it:
//   T = X L1          (dense part only, N = r rounded up to 32, the extra columns are zero)
//   Y = X Q + T L2    (quantized part followed by r/32 dense steps)
//
// Mapping: a workgroup of 256 threads (2 x 2 wavefronts) owns a 128 x 128 output tile and walks the reduction in
// 32-deep steps.  Per step the X tile (128 x 32 fp32) and the weight tile (32 x 128) are fetched into registers one
// step ahead, then written to LDS as bf16 hi and lo halves in MFMA operand layout (rows = output rows or columns,
// 32 reduction indices contiguous): the X tile is split, the weight tile is decoded from its packed codes, scaled
// by the block's reconstructed scale (the same fl32(code * s^) that the stand-alone dequantizer produces) and split.
// Each wavefront multiplies its 64 x 64 quarter with three v_mfma_f32_32x32x16_bf16 per tile pair (hi*hi + hi*lo +
// lo*hi, fp32 accumulation; the bf16-only variant keeps the hi halves alone).  A thread decodes a 4 (reduction) x 4
// (columns) patch: four code words from four consecutive rows of Q, so that its LDS writes are 8-byte runs.
// When the tile grid is too small to fill the machine the reduction is cut into `splits` contiguous ranges whose
// partial tiles go to scratch and are summed in a fixed order by a second kernel.
#include <algorithm>

#include "kernels.h"
#include "nf_device.h"
#include "profiler.h"

namespace lq {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));

constexpr int QM_BN = 128, QM_BK = 32;    // the tile has 64 * AT rows, AT = 2 or 4 (row tiles of 32 per wavefront)
constexpr int QM_PITCH = 40;     // LDS row pitch in bf16 (80 B): 16-byte aligned rows, conflict-free b128 reads

struct QmmArgs {
  const float* Xq; int64_t ldxq;   // m x Kq
  const float* Xd; int64_t ldxd;   // m x Kd
  const float* D; int64_t ldd;     // Kd x dcols fp32; columns >= dcols count as zero
  const uint8_t* codes; const uint8_t* sidx; const float* v;   // Kq x N, row-major flattening
  float* Y; int64_t ldy;           // m x N (splits == 1), else partials: split s at Y + s * m * ldy
  int64_t m, N, Kq, Kd, drows, dcols;
  int block_shift, group_shift, levels;   // log2 of the block size B0 and of the scale group size B1
  int nq, nsteps, splits;          // quantized steps, all steps, reduction ranges
  int tiles_m, tiles_n;
  const DevTables* tables;
};

// v = hi + lo + O(2^-17 v), both halves bf16.
__device__ __forceinline__ void split4(const float (&x)[4], bf16x4& hi, bf16x4& lo) {
  const floatx4 f = {x[0], x[1], x[2], x[3]};
  hi = __builtin_convertvector(f, bf16x4);
  lo = __builtin_convertvector(f - __builtin_convertvector(hi, floatx4), bf16x4);
}

// Registers of one prefetched reduction step: the X tile (128 rows x 8 float4, four per thread) and the thread's
// 4 x 4 patch of the weight tile, either as stored (code words of its quad in 4 consecutive rows of Q, the scale index
// of each row's block and that block's group scale) or dense.
template <int AT, bool QUANT>
struct QmmStep;
template <int AT>
struct QmmStep<AT, true> {
  floatx4 x[2 * AT];
  uint32_t cw[4], si[4];
  float vv[4];
};
template <int AT>
struct QmmStep<AT, false> {
  floatx4 x[2 * AT];
  floatx4 dn[4];
};

template <int BITS>
__device__ __forceinline__ uint32_t quad_word(const uint8_t* __restrict__ codes, int64_t quad) {
  if constexpr (BITS == 8) return *reinterpret_cast<const uint32_t*>(codes + quad * 4);
  else if constexpr (BITS == 4) return *reinterpret_cast<const uint16_t*>(codes + quad * 2);
  else if constexpr (BITS == 2) return codes[quad];
  else {   // 3 bits: 12 bits starting at bit 12*quad
    const int64_t byte = (quad * 3) >> 1;
    return ((uint32_t)codes[byte] | ((uint32_t)codes[byte + 1] << 8)) >> ((quad & 1) * 4);
  }
}

// Per-thread addressing that does not change from step to step.
template <int AT>
struct QmmLane {
  const float* xq[2 * AT];   // the thread's float4s of the X tile at reduction index 0 (quantized part's X)
  const float* xd[2 * AT];   // same for the dense part's X
  int64_t col;          // first column of the patch
  int64_t colc;         // the same, clamped into the matrix (loaded, never stored)
  int kg, quad;
};

template <int BITS, int AT, bool QUANT>
__device__ __forceinline__ void qmm_fetch(const QmmArgs& a, const QmmLane<AT>& t, int step, QmmStep<AT, QUANT>& r) {
  const int64_t k0 = (int64_t)step * QM_BK;          // within its own part
#pragma unroll
  for (int i = 0; i < 2 * AT; ++i) r.x[i] = *reinterpret_cast<const floatx4*>((QUANT ? t.xq[i] : t.xd[i]) + k0);
  if constexpr (QUANT) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int64_t e = (k0 + 4 * t.kg + j) * a.N + t.colc;
      r.cw[j] = quad_word<BITS>(a.codes, e >> 2);
      const int64_t blk = e >> a.block_shift;
      r.si[j] = a.sidx[blk];
      r.vv[j] = a.v[blk >> a.group_shift];
    }
  } else {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int64_t p = k0 + 4 * t.kg + j;
      float w[4];
#pragma unroll
      for (int c = 0; c < 4; ++c) w[c] = (p < a.drows && t.col + c < a.dcols) ? a.D[p * a.ldd + t.col + c] : 0.0f;
      r.dn[j] = floatx4{w[0], w[1], w[2], w[3]};
    }
  }
}

template <int BITS, int AT, bool SPLIT, bool QUANT>
__device__ __forceinline__ void qmm_stash(const QmmArgs& a, const QmmLane<AT>& t, int tid, const QmmStep<AT, QUANT>& r,
                                          const float* s_code, __bf16* xh, __bf16* xl, __bf16* bh, __bf16* bl) {
#pragma unroll
  for (int i = 0; i < 2 * AT; ++i) {
    const int idx = tid + 256 * i;
    const float f[4] = {r.x[i].x, r.x[i].y, r.x[i].z, r.x[i].w};
    bf16x4 hi, lo;
    split4(f, hi, lo);
    const int at = (idx >> 3) * QM_PITCH + (idx & 7) * 4;
    *reinterpret_cast<bf16x4*>(xh + at) = hi;
    if constexpr (SPLIT) *reinterpret_cast<bf16x4*>(xl + at) = lo;
  }
  float w[4][4];                                     // [reduction index][column]
  if constexpr (QUANT) {
    constexpr uint32_t mask = (1u << BITS) - 1u;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float sh = block_scale(r.si[j], r.vv[j], a.levels);
#pragma unroll
      for (int c = 0; c < 4; ++c) w[j][c] = s_code[(r.cw[j] >> (c * BITS)) & mask] * sh;
    }
  } else {
#pragma unroll
    for (int j = 0; j < 4; ++j) { w[j][0] = r.dn[j].x; w[j][1] = r.dn[j].y; w[j][2] = r.dn[j].z; w[j][3] = r.dn[j].w; }
  }
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    const float f[4] = {w[0][c], w[1][c], w[2][c], w[3][c]};
    bf16x4 hi, lo;
    split4(f, hi, lo);
    const int at = (4 * t.quad + c) * QM_PITCH + 4 * t.kg;
    *reinterpret_cast<bf16x4*>(bh + at) = hi;
    if constexpr (SPLIT) *reinterpret_cast<bf16x4*>(bl + at) = lo;
  }
}

// One 32-deep step of the wavefront's (32 AT) x 64 quarter from the operand tiles in LDS.
template <int AT, bool SPLIT>
__device__ __forceinline__ void qmm_multiply(const __bf16* xh, const __bf16* xl, const __bf16* bhp, const __bf16* blp,
                                             int arow, int brow, int lh, floatx16 (&acc)[AT][2]) {
#pragma unroll
  for (int g = 0; g < 2; ++g) {
    bf16x8 ah[AT], al[AT], bh[2], bl[2];
#pragma unroll
    for (int i = 0; i < AT; ++i) {
      const int at = (arow + 32 * i) * QM_PITCH + 16 * g + 8 * lh;
      ah[i] = *reinterpret_cast<const bf16x8*>(xh + at);
      if constexpr (SPLIT) al[i] = *reinterpret_cast<const bf16x8*>(xl + at);
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int at = (brow + 32 * j) * QM_PITCH + 16 * g + 8 * lh;
      bh[j] = *reinterpret_cast<const bf16x8*>(bhp + at);
      if constexpr (SPLIT) bl[j] = *reinterpret_cast<const bf16x8*>(blp + at);
    }
#pragma unroll
    for (int i = 0; i < AT; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        if constexpr (SPLIT) {
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al[i], bh[j], acc[i][j], 0, 0, 0);
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[i], bl[j], acc[i][j], 0, 0, 0);
        }
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[i], bh[j], acc[i][j], 0, 0, 0);
      }
  }
}

// Steps [sa, sb) of one part (numbered within the part).  Operands are fetched DEPTH steps ahead into a ring of
// register sets; the prefetch index is clamped instead of guarded (the last step is fetched again and dropped), so
// the loop body is branch-free and the loads stay in flight across the barriers.
template <int BITS, int AT, bool SPLIT, bool QUANT, int DEPTH>
__device__ __forceinline__ void qmm_run(const QmmArgs& a, const QmmLane<AT>& t, int sa, int sb, int tid, int arow,
                                        int brow, int lh, const float* s_code, __bf16 (*s_x)[64 * AT * QM_PITCH],
                                        __bf16 (*s_b)[QM_BN * QM_PITCH], floatx16 (&acc)[AT][2]) {
  if (sa >= sb) return;
  const int last = sb - 1;
  QmmStep<AT, QUANT> ring[DEPTH];
  qmm_fetch<BITS, AT, QUANT>(a, t, sa, ring[0]);
  if constexpr (DEPTH > 1) qmm_fetch<BITS, AT, QUANT>(a, t, sa + 1 < last ? sa + 1 : last, ring[1]);
#define LQ_QMM_STEP(U, S)                                                                                  \
  {                                                                                                        \
    __syncthreads(); /* the previous step's operands have been read */                                     \
    qmm_stash<BITS, AT, SPLIT, QUANT>(a, t, tid, ring[(U)], s_code, s_x[0], s_x[1], s_b[0], s_b[1]);       \
    __syncthreads();                                                                                       \
    qmm_fetch<BITS, AT, QUANT>(a, t, (S) + DEPTH < last ? (S) + DEPTH : last, ring[(U)]);                  \
    qmm_multiply<AT, SPLIT>(s_x[0], s_x[1], s_b[0], s_b[1], arow, brow, lh, acc);                          \
  }
  int s = sa;
  if constexpr (DEPTH > 1) {
    for (; s + 2 <= sb; s += 2) {
      LQ_QMM_STEP(0, s)
      LQ_QMM_STEP(1, s + 1)
    }
    if (s < sb) LQ_QMM_STEP(0, s)
  } else {
    for (; s < sb; ++s) LQ_QMM_STEP(0, s)
  }
#undef LQ_QMM_STEP
}

template <int BITS, int AT, bool SPLIT>
__global__ __launch_bounds__(256, 2) void qmatmul_kernel(QmmArgs a) {
  constexpr int BM = 64 * AT;
  constexpr int DEPTH = AT > 2 ? 1 : 2;
  __shared__ __attribute__((aligned(16))) __bf16 s_x[2][BM * QM_PITCH];
  __shared__ __attribute__((aligned(16))) __bf16 s_b[2][QM_BN * QM_PITCH];
  __shared__ float s_code[1 << BITS];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, ln = lane & 31, lh = lane >> 5;
  const int wm = wave >> 1, wn = wave & 1;
  for (int i = tid; i < (1 << BITS); i += 256) s_code[i] = a.tables->code[Slot<BITS>::value][i];

  // Workgroups go to the 8 XCDs round-robin by linear index.  With at least 8 row tiles every XCD keeps to its own
  // row tiles (its X rows stay in its L2) and sweeps the column tiles; smaller grids are taken in plain order.
  const int split = blockIdx.y;
  int bm, bn;
  if (a.tiles_m >= 8) {
    const int xcd = blockIdx.x & 7, s = blockIdx.x >> 3;
    bm = (s / a.tiles_n) * 8 + xcd;
    bn = s % a.tiles_n;
    if (bm >= a.tiles_m) return;
  } else {
    bm = blockIdx.x / a.tiles_n;
    bn = blockIdx.x % a.tiles_n;
  }
  const int64_t row0 = (int64_t)bm * BM, col0 = (int64_t)bn * QM_BN;
  const int s0 = (int)((int64_t)a.nsteps * split / a.splits), s1 = (int)((int64_t)a.nsteps * (split + 1) / a.splits);

  QmmLane<AT> t;
  t.kg = lane & 7;                     // the thread's 4 x 4 patch of the weight tile: reduction rows 4kg.., columns 4quad..
  t.quad = 8 * wave + (lane >> 3);
  t.col = col0 + 4 * t.quad;
  t.colc = t.col < a.N ? t.col : a.N - 4;          // in the quantized part N is a multiple of the block size, hence of 4
#pragma unroll
  for (int i = 0; i < 2 * AT; ++i) {
    const int idx = tid + 256 * i;
    int64_t row = row0 + (idx >> 3);
    row = row < a.m ? row : a.m - 1;               // clamped: loaded, never stored
    t.xq[i] = a.Xq + row * a.ldxq + (idx & 7) * 4;
    t.xd[i] = a.Xd + row * a.ldxd + (idx & 7) * 4;
  }

  floatx16 acc[AT][2];
#pragma unroll
  for (int i = 0; i < AT; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

  // quantized steps first, then the dense ones (the first barrier of either also covers the code book)
  const int arow = 32 * AT * wm + ln, brow = 64 * wn + ln;
  qmm_run<BITS, AT, SPLIT, true, DEPTH>(a, t, s0 < a.nq ? s0 : a.nq, s1 < a.nq ? s1 : a.nq, tid, arow, brow, lh, s_code,
                                        s_x, s_b, acc);
  qmm_run<BITS, AT, SPLIT, false, DEPTH>(a, t, (s0 > a.nq ? s0 : a.nq) - a.nq, (s1 > a.nq ? s1 : a.nq) - a.nq, tid, arow,
                                         brow, lh, s_code, s_x, s_b, acc);

  // accumulator element e of a lane is row 8*(e/4) + 4*lh + e%4, column ln of its 32 x 32 tile
  float* __restrict__ Y = a.Y + (size_t)split * (size_t)a.m * a.ldy;
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int64_t col = col0 + 64 * wn + 32 * j + ln;
    if (col >= a.N) continue;
#pragma unroll
    for (int i = 0; i < AT; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int64_t row = row0 + 32 * AT * wm + 32 * i + 8 * (e >> 2) + 4 * lh + (e & 3);
        if (row < a.m) Y[row * a.ldy + col] = acc[i][j][e];
      }
  }
}

// Y = sum over the reduction ranges of their partial results, in range order.
__global__ __launch_bounds__(256) void qmatmul_reduce_kernel(const float* __restrict__ part, int splits, int64_t m,
                                                             int64_t N, int64_t ldp, float* __restrict__ Y,
                                                             int64_t ldy) {
  const int64_t total = m * N;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int64_t row = i / N, col = i % N;
    float s = 0.0f;
    for (int z = 0; z < splits; ++z) s += part[((size_t)z * m + row) * ldp + col];
    Y[row * ldy + col] = s;
  }
}

// Rows of an output tile: 256 when that still gives every compute unit a tile, else 128.
int qmatmul_tile_rows(int64_t m, int64_t N) {
  return ((m + 255) / 256) * ((N + QM_BN - 1) / QM_BN) >= 256 ? 256 : 128;
}

// Reduction ranges for an m x N product with `nsteps` 32-deep steps: enough workgroups to occupy every compute unit
// twice over, at least four steps per range, at most 16 ranges.
int qmatmul_splits(int64_t m, int64_t N, int nsteps) {
  const int bm = qmatmul_tile_rows(m, N);
  const int64_t tiles = ((m + bm - 1) / bm) * ((N + QM_BN - 1) / QM_BN);
  if (tiles >= 256) return 1;
  const int64_t want = (512 + tiles - 1) / tiles;
  const int64_t cap = std::max<int64_t>(1, nsteps / 4);
  return (int)std::max<int64_t>(1, std::min<int64_t>(std::min(want, cap), 16));
}

size_t qmatmul_part_floats(int64_t m, int64_t N, int nsteps) {
  const int s = qmatmul_splits(m, N, nsteps);
  return s > 1 ? (size_t)s * (size_t)m * (size_t)N : 0;
}

template <int BITS>
static void launch_bits(const QmmArgs& a, dim3 grid, int tile_rows, bool split_precision, hipStream_t st) {
  if (tile_rows == 256) {
    if (split_precision) hipLaunchKernelGGL((qmatmul_kernel<BITS, 4, true>), grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((qmatmul_kernel<BITS, 4, false>), grid, dim3(256), 0, st, a);
  } else {
    if (split_precision) hipLaunchKernelGGL((qmatmul_kernel<BITS, 2, true>), grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((qmatmul_kernel<BITS, 2, false>), grid, dim3(256), 0, st, a);
  }
}

int launch_qmatmul(const QmmPart& q, const DensePart& dn, int64_t m, int64_t N, float* Y, int64_t ldy, float* part,
                   size_t part_floats, int precision, hipStream_t st) {
  if (m <= 0 || N <= 0) return LQ_ERR_SHAPE;
  if ((q.K % QM_BK) != 0 || (dn.K % QM_BK) != 0 || q.K + dn.K <= 0) return LQ_ERR_SHAPE;
  if (q.K > 0 && (q.block < 4 || (q.block & (q.block - 1)) != 0 || q.scale_block < 1 ||
                  (q.scale_block & (q.scale_block - 1)) != 0))
    return LQ_ERR_CONFIG;                                  // block sizes are powers of two
  if (q.K > 0 && ((N % q.block) != 0 || (q.ldx & 3) != 0)) return LQ_ERR_SHAPE;
  if (dn.K > 0 && (dn.ldx & 3) != 0) return LQ_ERR_SHAPE;
  QmmArgs a{};
  a.Xq = q.X; a.ldxq = q.ldx; a.Kq = q.K;
  a.codes = q.codes; a.sidx = q.sidx; a.v = q.v;
  a.block_shift = q.K > 0 ? __builtin_ctz((unsigned)q.block) : 0;
  a.group_shift = q.K > 0 ? __builtin_ctz((unsigned)q.scale_block) : 0;
  a.levels = q.levels;
  a.Xd = dn.X; a.ldxd = dn.ldx; a.Kd = dn.K; a.D = dn.D; a.ldd = dn.ldd; a.drows = dn.rows; a.dcols = dn.cols;
  a.m = m; a.N = N;
  a.nq = (int)(q.K / QM_BK);
  a.nsteps = a.nq + (int)(dn.K / QM_BK);
  const int bm = qmatmul_tile_rows(m, N);
  a.tiles_m = (int)((m + bm - 1) / bm);
  a.tiles_n = (int)((N + QM_BN - 1) / QM_BN);
  a.splits = qmatmul_splits(m, N, a.nsteps);
  if (a.splits > 1 && part_floats < (size_t)a.splits * (size_t)m * (size_t)N) return LQ_ERR_WORKSPACE;
  a.Y = a.splits > 1 ? part : Y;
  a.ldy = a.splits > 1 ? N : ldy;
  const DevTables* tab = nullptr;
  LQ_TRY(device_tables(&tab));
  a.tables = tab;
  const int64_t gx = a.tiles_m >= 8 ? (int64_t)8 * ((a.tiles_m + 7) / 8) * a.tiles_n : (int64_t)a.tiles_m * a.tiles_n;
  if (gx >= (1ll << 31)) return LQ_ERR_SHAPE;
  const dim3 grid((unsigned)gx, (unsigned)a.splits);
  const int bits = q.K > 0 ? q.bits : 4;
  {
    prof::Scope ps(prof::QMATMUL, st, 2.0 * (double)m * (double)N * (double)(q.K + dn.K));
    switch (bits) {
      case 2: launch_bits<2>(a, grid, bm, precision == 0, st); break;
      case 3: launch_bits<3>(a, grid, bm, precision == 0, st); break;
      case 4: launch_bits<4>(a, grid, bm, precision == 0, st); break;
      case 8: launch_bits<8>(a, grid, bm, precision == 0, st); break;
      default: return LQ_ERR_CONFIG;
    }
    LQ_HIP_TRY(hipGetLastError());
  }
  if (a.splits > 1) {
    prof::Scope ps(prof::MISC, st, 4.0 * (double)m * (double)N * (a.splits + 1));
    const int64_t nwg = std::min<int64_t>((m * N + 255) / 256, 4096);
    hipLaunchKernelGGL(qmatmul_reduce_kernel, dim3((unsigned)nwg), dim3(256), 0, st, part, a.splits, m, N, N, Y, ldy);
    LQ_HIP_TRY(hipGetLastError());
  }
  return LQ_OK;
}

}  // namespace lq
