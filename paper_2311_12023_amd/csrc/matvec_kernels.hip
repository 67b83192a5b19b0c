// Forward product with a decomposed weight for a handful of input rows (single tokens, small decode batches):
//     Y[m x N] = X[m x K] * dequant(codes)[K x N] + T[m x Kd] * D[Kd x N],      m <= 8,
// (Section 3.2 "Implementation", Appendix A: the matrix-vector case of the run-time comparison).  With so few rows the
// product is bound by reading the weights once from HBM (b0/8 bytes each), not by arithmetic, so the weights are decoded
// and multiplied on the vector ALU in fp32: exact products of the same fl32(code * s^) values that Dequantize returns,
// fp32 accumulation.  The forward product is T = X L1 (a narrow dense product), then Y = X Q + T L2.
//
// Mapping: a thread owns one 16-weight run (one block scale per run, codes fetched as one 2..16-byte word) in every
// 32nd row of its workgroup's range of reduction rows; a workgroup is 8 runs (128 columns) x 32 row groups, so that
// 256 workgroups of up to 512 rows cover a 4096 x 4096 matrix with every load of a thread issued before the first is
// used (the whole matrix is in flight at once, which is what an HBM-bound kernel needs).  The X values of the range sit in
// LDS.  Row groups are summed by a fixed butterfly inside each wavefront and in wavefront order through LDS; the ranges
// (`splits` of them: enough to fill the machine while the partial sums stay small next to the weights) are added in a
// fixed order by a second kernel, so results are deterministic.
#include <algorithm>

#include "kernels.h"
#include "nf_device.h"
#include "profiler.h"

namespace lq {

constexpr int MV_RUNS = 8;          // 16-weight runs per workgroup: 128 columns
constexpr int MV_COLS = 16 * MV_RUNS;
constexpr int MV_GROUPS = 32;       // row groups per workgroup (256 threads)
constexpr int MV_ROWS_MAX = 512;    // reduction rows per workgroup (its X slice lives in LDS)
constexpr int MV_DEPTH = MV_ROWS_MAX / MV_GROUPS;   // rows per thread at most

struct MvArgs {
  const float* X; int64_t ldx;      // m x K
  const float* Xd; int64_t ldxd;    // m x Kd, given as xd_splits partial sums xd_stride floats apart (added in order)
  int xd_splits; int64_t xd_stride;
  const uint8_t* codes; const uint8_t* sidx; const float* v;   // K x N, row-major flattening
  const float* D; int64_t ldd;      // Kd x N dense
  float* Y; int64_t ldy;            // splits == 1: m x N; else partial sums, range s at Y + s * m * ldy
  int64_t K, Kd, N;
  int m, splits, rows_per_split;
  int block_shift, group_shift, levels;
  const DevTables* tables;
};

template <int BITS, int M>
__global__ __launch_bounds__(256) void qmatvec_kernel(MvArgs a) {
  __shared__ float s_x[M][MV_ROWS_MAX];
  __shared__ float s_code[1 << BITS];
  __shared__ __attribute__((aligned(16))) float s_sum[3][M][MV_COLS];
  const int tid = threadIdx.x, wave = tid >> 6, run = tid & (MV_RUNS - 1), grp = tid >> 3;
  const int64_t col = (int64_t)blockIdx.x * MV_COLS + 16 * run;         // first column of the thread's run
  const int split = blockIdx.y;
  const int64_t ktot = a.K + a.Kd;
  const int64_t ra = (int64_t)split * a.rows_per_split;
  const int64_t rb = ra + a.rows_per_split < ktot ? ra + a.rows_per_split : ktot;
  const int nrows = (int)(rb - ra);
  const int64_t qend = a.K < rb ? a.K : rb;
  const int nq = qend > ra ? (int)(qend - ra) : 0;                      // quantized rows of the range (they come first)
  for (int i = tid; i < (1 << BITS); i += 256) s_code[i] = a.tables->code[Slot<BITS>::value][i];
  for (int i = 0; i < M; ++i)
    for (int r = tid; r < nrows; r += 256) {
      float x = 0.0f;
      if (i < a.m) {
        const int64_t g = ra + r;
        if (g < a.K) {
          x = a.X[(int64_t)i * a.ldx + g];
        } else {
          const float* p = a.Xd + (int64_t)i * a.ldxd + (g - a.K);
#pragma unroll 8
          for (int z = 0; z < a.xd_splits; ++z) x += p[(int64_t)z * a.xd_stride];
        }
      }
      s_x[i][r] = x;
    }
  __syncthreads();

  float acc[M][16];
#pragma unroll
  for (int i = 0; i < M; ++i)
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[i][j] = 0.0f;
  const bool live = col < a.N;                    // N is a multiple of 16
  const int64_t colc = live ? col : 0;

  // quantized rows of the thread: local rows grp, grp + 32, ... below nq; every load is issued before the first use
  // (a row past the end is loaded clamped and skipped)
  if (nq > 0) {
    uint2 cw[MV_DEPTH];                           // at most 64 bits of codes per run for b0 <= 4; 8-bit codes take two passes
    uint32_t si[MV_DEPTH];
    float vv[MV_DEPTH];
    constexpr int PASSES = BITS == 8 ? 2 : 1;
#pragma unroll
    for (int pass = 0; pass < PASSES; ++pass) {
#pragma unroll
      for (int j = 0; j < MV_DEPTH; ++j) {
        int r = grp + MV_GROUPS * j;
        r = r < nq ? r : nq - 1;
        const int64_t e = (ra + r) * a.N + colc;
        const uint8_t* p = a.codes + (e >> 4) * (2 * BITS) + 8 * pass;
        if constexpr (BITS == 2) cw[j] = make_uint2(*reinterpret_cast<const uint32_t*>(p), 0u);
        else if constexpr (BITS == 3) {
          const uint16_t* q = reinterpret_cast<const uint16_t*>(p);
          cw[j] = make_uint2((uint32_t)q[0] | ((uint32_t)q[1] << 16), (uint32_t)q[2]);
        } else cw[j] = *reinterpret_cast<const uint2*>(p);
        if (pass == 0) {
          const int64_t blk = e >> a.block_shift;
          si[j] = a.sidx[blk];
          vv[j] = a.v[blk >> a.group_shift];
        }
      }
      constexpr int PER = 16 / PASSES;            // codes decoded per pass
      constexpr int CB = BITS == 8 ? 8 : BITS;
#pragma unroll
      for (int j = 0; j < MV_DEPTH; ++j) {
        const int r = grp + MV_GROUPS * j;
        if (r < nq) {
          const float sh = block_scale(si[j], vv[j], a.levels);
          const uint64_t word = (uint64_t)cw[j].x | ((uint64_t)cw[j].y << 32);
          float xr[M];
#pragma unroll
          for (int i = 0; i < M; ++i) xr[i] = s_x[i][r];
#pragma unroll
          for (int e = 0; e < PER; ++e) {
            const float w = s_code[(uint32_t)(word >> (e * CB)) & ((1u << CB) - 1u)] * sh;
#pragma unroll
            for (int i = 0; i < M; ++i) acc[i][PER * pass + e] = fmaf(xr[i], w, acc[i][PER * pass + e]);
          }
        }
      }
    }
  }
  // dense rows of the thread: local rows >= nq
  for (int r = grp; r < nrows; r += MV_GROUPS) {
    if (r < nq) continue;
    const float* drow = a.D + (ra + r - a.K) * a.ldd + colc;
    float w[16];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const float4 f = *reinterpret_cast<const float4*>(drow + 4 * q);
      w[4 * q] = f.x; w[4 * q + 1] = f.y; w[4 * q + 2] = f.z; w[4 * q + 3] = f.w;
    }
#pragma unroll
    for (int i = 0; i < M; ++i) {
      const float x = s_x[i][r];
#pragma unroll
      for (int j = 0; j < 16; ++j) acc[i][j] = fmaf(x, w[j], acc[i][j]);
    }
  }

  // the 8 row groups of a wavefront (lanes 8 apart), by a fixed butterfly; then the wavefronts in order through LDS
#pragma unroll
  for (int i = 0; i < M; ++i)
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      float x = acc[i][j];
      x += __shfl_xor(x, 8);
      x += __shfl_xor(x, 16);
      x += __shfl_xor(x, 32);
      acc[i][j] = x;
    }
  const int lane = tid & 63;
  if (wave > 0 && lane < MV_RUNS) {
#pragma unroll
    for (int i = 0; i < M; ++i)
#pragma unroll
      for (int q = 0; q < 4; ++q)
        *reinterpret_cast<float4*>(&s_sum[wave - 1][i][16 * run + 4 * q]) =
            make_float4(acc[i][4 * q], acc[i][4 * q + 1], acc[i][4 * q + 2], acc[i][4 * q + 3]);
  }
  __syncthreads();
  if (wave == 0 && lane < MV_RUNS && live) {
    float* __restrict__ Y = a.Y + (size_t)split * (size_t)a.m * a.ldy;
#pragma unroll
    for (int i = 0; i < M; ++i) {
      if (i >= a.m) break;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        float o[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          float s = acc[i][4 * q + e];
          s += s_sum[0][i][16 * run + 4 * q + e];
          s += s_sum[1][i][16 * run + 4 * q + e];
          s += s_sum[2][i][16 * run + 4 * q + e];
          o[e] = s;
        }
        *reinterpret_cast<float4*>(Y + (int64_t)i * a.ldy + col + 4 * q) = make_float4(o[0], o[1], o[2], o[3]);
      }
    }
  }
}

// T[m x N] = X[m x K] * D[K x N] for a narrow dense D (the d x rank factor): thread (p, g) of a workgroup takes column
// p and every (256 / N')-th row of the workgroup's range (N' = N rounded up to a power of two, at most 256); the row
// groups are added in a fixed order through LDS; the ranges' partial sums (range s at Y + s * m * ldy) are left to the
// consumer, which adds them in range order.
constexpr int XDENSE_ROWS = 128;    // reduction rows per workgroup
template <int M>
__global__ __launch_bounds__(256) void xdense_narrow_kernel(const float* __restrict__ X, int64_t ldx,
                                                            const float* __restrict__ D, int64_t ldd, int64_t K, int N,
                                                            int npow, int m, int rows_per_split, float* __restrict__ Y,
                                                            int64_t ldy) {
  __shared__ float s_x[M][XDENSE_ROWS];
  __shared__ float s_red[M][256];
  const int tid = threadIdx.x;
  const int p0 = tid & (npow - 1), g = tid / npow, groups = 256 / npow;
  const int64_t ra = (int64_t)blockIdx.x * rows_per_split;
  const int64_t rb = ra + rows_per_split < K ? ra + rows_per_split : K;
  const int nrows = (int)(rb - ra);
  for (int i = 0; i < M; ++i)
    for (int r = tid; r < nrows; r += 256) s_x[i][r] = i < m ? X[(int64_t)i * ldx + ra + r] : 0.0f;
  float* __restrict__ out = Y + (size_t)blockIdx.x * (size_t)m * ldy;
  for (int pc = 0; pc < N; pc += npow) {             // column chunks (one, unless N > 256)
    const int p = pc + p0;
    float acc[M];
#pragma unroll
    for (int i = 0; i < M; ++i) acc[i] = 0.0f;
    __syncthreads();                                 // X slice ready; s_red free again
    if (p < N)
      for (int r = g; r < nrows; r += groups) {
        const float w = D[(ra + r) * ldd + p];
#pragma unroll
        for (int i = 0; i < M; ++i) acc[i] = fmaf(s_x[i][r], w, acc[i]);
      }
#pragma unroll
    for (int i = 0; i < M; ++i) s_red[i][tid] = acc[i];
    __syncthreads();
    if (g == 0 && p < N) {
#pragma unroll
      for (int i = 0; i < M; ++i) {
        if (i >= m) break;
        float s = 0.0f;
        for (int gg = 0; gg < groups; ++gg) s += s_red[i][gg * npow + p0];
        out[(int64_t)i * ldy + p] = s;
      }
    }
  }
}

// Reduction ranges for m rows against (K + Kd) x N weights: about 512 workgroups, at most 512 rows each (a multiple
// of 32), and partial sums (splits * m * N floats) that stay below about a quarter of a 4-bit matrix's bytes.
int qmatvec_splits(int m, int64_t ktot, int64_t N) {
  const int64_t tiles = (N + MV_COLS - 1) / MV_COLS;
  int64_t s = (512 + tiles - 1) / tiles;
  s = std::min<int64_t>(s, std::max<int64_t>(1, ktot / (32 * (int64_t)std::max(m, 1))));
  s = std::max<int64_t>(s, (ktot + MV_ROWS_MAX - 1) / MV_ROWS_MAX);     // the X slice must fit in LDS
  int64_t rows = (ktot + s - 1) / s;
  rows = (rows + 31) / 32 * 32;
  return (int)std::max<int64_t>(1, (ktot + rows - 1) / rows);
}

size_t qmatvec_part_floats(int m, int64_t ktot, int64_t N) {
  const int s = qmatvec_splits(m, ktot, N);
  return s > 1 ? (size_t)s * (size_t)m * (size_t)N : 0;
}

// Ranges of XDENSE_ROWS rows each.
int xdense_splits(int64_t K) { return (int)((K + XDENSE_ROWS - 1) / XDENSE_ROWS); }
size_t xdense_part_floats(int m, int64_t K, int64_t N) { return (size_t)xdense_splits(K) * (size_t)m * (size_t)N; }

template <int BITS>
static void launch_m(const MvArgs& a, dim3 grid, hipStream_t st) {
  if (a.m <= 1) hipLaunchKernelGGL((qmatvec_kernel<BITS, 1>), grid, dim3(256), 0, st, a);
  else if (a.m <= 2) hipLaunchKernelGGL((qmatvec_kernel<BITS, 2>), grid, dim3(256), 0, st, a);
  else if (a.m <= 4) hipLaunchKernelGGL((qmatvec_kernel<BITS, 4>), grid, dim3(256), 0, st, a);
  else hipLaunchKernelGGL((qmatvec_kernel<BITS, 8>), grid, dim3(256), 0, st, a);
}

int launch_qmatvec(const MvWeights& q, const float* X, int64_t ldx, int64_t K, const float* Xd, int64_t ldxd,
                   int xd_splits, int64_t xd_stride, const float* D, int64_t ldd, int64_t Kd, int m, int64_t N, float* Y,
                   int64_t ldy, float* part, size_t part_floats, hipStream_t st) {
  if (m < 1 || m > QMATVEC_MAX_ROWS || K <= 0 || Kd < 0 || N <= 0 || (N % 16) != 0) return LQ_ERR_SHAPE;
  if (Kd > 0 && xd_splits < 1) return LQ_ERR_ARG;
  if (q.block < 16 || (q.block & (q.block - 1)) != 0 || q.scale_block < 1 || (q.scale_block & (q.scale_block - 1)) != 0)
    return LQ_ERR_CONFIG;
  if ((N % q.block) != 0 || (ldy & 3) != 0 || (Kd > 0 && (ldd & 3) != 0)) return LQ_ERR_SHAPE;
  MvArgs a{};
  a.X = X; a.ldx = ldx; a.K = K; a.Xd = Xd; a.ldxd = ldxd; a.xd_splits = xd_splits; a.xd_stride = xd_stride; a.D = D; a.ldd = ldd; a.Kd = Kd; a.N = N; a.m = m;
  a.codes = q.codes; a.sidx = q.sidx; a.v = q.v;
  a.block_shift = __builtin_ctz((unsigned)q.block);
  a.group_shift = __builtin_ctz((unsigned)q.scale_block);
  a.levels = q.levels;
  const int64_t ktot = K + Kd;
  a.splits = qmatvec_splits(m, ktot, N);
  int64_t rows = (ktot + a.splits - 1) / a.splits;
  rows = (rows + 31) / 32 * 32;
  if (rows > MV_ROWS_MAX) return LQ_ERR_SHAPE;
  a.rows_per_split = (int)rows;
  a.splits = (int)((ktot + rows - 1) / rows);                           // no empty range
  if (a.splits > 1 && part_floats < (size_t)a.splits * (size_t)m * (size_t)N) return LQ_ERR_WORKSPACE;
  a.Y = a.splits > 1 ? part : Y;
  a.ldy = a.splits > 1 ? N : ldy;
  const DevTables* tab = nullptr;
  LQ_TRY(device_tables(&tab));
  a.tables = tab;
  const int64_t tiles = (N + MV_COLS - 1) / MV_COLS;
  if (tiles >= (1ll << 31)) return LQ_ERR_SHAPE;
  const dim3 grid((unsigned)tiles, (unsigned)a.splits);
  {
    // algorithmic bytes: the weights once (codes, one scale index per block, the dense rows), X, Y
    const double wbytes = (double)K * (double)N * (q.bits / 8.0 + 1.0 / q.block) + 4.0 * (double)Kd * (double)N;
    prof::Scope ps(prof::QMATVEC, st, wbytes + 4.0 * m * (double)(ktot + N));
    switch (q.bits) {
      case 2: launch_m<2>(a, grid, st); break;
      case 3: launch_m<3>(a, grid, st); break;
      case 4: launch_m<4>(a, grid, st); break;
      case 8: launch_m<8>(a, grid, st); break;
      default: return LQ_ERR_CONFIG;
    }
    LQ_HIP_TRY(hipGetLastError());
  }
  if (a.splits > 1) LQ_TRY(launch_qmatmul_reduce(part, a.splits, m, N, Y, ldy, st));
  return LQ_OK;
}

int launch_xdense_narrow(const float* X, int64_t ldx, const float* D, int64_t ldd, int64_t K, int N, int m, float* part,
                         size_t part_floats, hipStream_t st) {
  if (m < 1 || m > QMATVEC_MAX_ROWS || K <= 0 || N <= 0) return LQ_ERR_SHAPE;
  int npow = 1;
  while (npow < N && npow < 256) npow <<= 1;
  const int rows = XDENSE_ROWS;
  if ((K + rows - 1) / rows >= (1 << 16)) return LQ_ERR_SHAPE;
  const int splits = xdense_splits(K);
  if (part_floats < (size_t)splits * (size_t)m * (size_t)N) return LQ_ERR_WORKSPACE;
  prof::Scope ps(prof::MISC, st, 4.0 * (double)K * N);
  const dim3 grid((unsigned)splits), block(256);
  if (m <= 1) hipLaunchKernelGGL((xdense_narrow_kernel<1>), grid, block, 0, st, X, ldx, D, ldd, K, N, npow, m, rows, part, (int64_t)N);
  else if (m <= 2) hipLaunchKernelGGL((xdense_narrow_kernel<2>), grid, block, 0, st, X, ldx, D, ldd, K, N, npow, m, rows, part, (int64_t)N);
  else if (m <= 4) hipLaunchKernelGGL((xdense_narrow_kernel<4>), grid, block, 0, st, X, ldx, D, ldd, K, N, npow, m, rows, part, (int64_t)N);
  else hipLaunchKernelGGL((xdense_narrow_kernel<8>), grid, block, 0, st, X, ldx, D, ldd, K, N, npow, m, rows, part, (int64_t)N);
  LQ_HIP_TRY(hipGetLastError());
  return LQ_OK;
}

}  // namespace lq
