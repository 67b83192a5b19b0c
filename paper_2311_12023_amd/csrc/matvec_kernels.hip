// Forward product with a decomposed weight for a handful of input rows (single tokens, small decode batches):
//     Y[m x N] = X[m x K] * dequant(codes)[K x N] + (X * L1)[m x r] * L2[r x N],      m <= 8,
// (Section 3.2 "Implementation", Appendix A: the matrix-vector case of the run-time comparison).  With so few rows the
// product is bound by reading the weights once from HBM (b0/8 bytes each), not by arithmetic, so the weights are decoded
// and multiplied on the vector ALU in fp32: exact products of the same fl32(code * s^) values that Dequantize returns,
// fp32 accumulation.  Two launches: the first multiplies X with [Q | L1] (the columns of L1 are extra column tiles of
// the same grid), the second adds the reduction ranges of both results and the small product (X L1) L2.
//
// Mapping of the first kernel: a thread owns one 16-weight run (one block scale per run, codes fetched as one
// 2..16-byte word) in every 32nd row of its workgroup's range of reduction rows; a workgroup is 8 runs (128 columns) x
// 32 row groups, so that 256 workgroups of up to 512 rows cover a 4096 x 4096 matrix with every load of a thread issued
// before the first is used (the whole matrix is in flight at once, which is what an HBM-bound kernel needs).  The X
// values of the range sit in LDS.  Row groups are summed by a fixed butterfly inside each wavefront and in wavefront
// order through LDS; the ranges (`splits` of them: enough to fill the machine while the partial sums stay small next to
// the weights) are added in a fixed order by the second kernel, so results are deterministic.
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
  const uint8_t* codes; const uint8_t* sidx; const float* v;   // K x N, row-major flattening
  const float* D; int64_t ldd;      // K x Nd dense (the factor L1), columns tiles_q * 128 onward of the grid
  int d_vec;                        // Nd % 4 == 0 and D 16-byte aligned: float4 loads
  float* Y; int64_t ldy;            // partial sums of X Q: range s at Y + s * m * ldy (splits == 1 and Nd == 0: Y itself)
  float* Yd;                        // partial sums of X D: range s at Yd + s * m * Nd
  int64_t K, N, Nd;
  int m, splits, rows_per_split, tiles_q;
  int block_shift, group_shift, levels;
  const DevTables* tables;
};

template <int BITS, int M>
__global__ __launch_bounds__(256) void qmatvec_kernel(MvArgs a) {
  __shared__ float s_x[M][MV_ROWS_MAX];
  __shared__ float s_code[1 << BITS];
  __shared__ __attribute__((aligned(16))) float s_sum[3][M][MV_COLS];
  const int tid = threadIdx.x, wave = tid >> 6, run = tid & (MV_RUNS - 1), grp = tid >> 3;
  const bool dense = (int)blockIdx.x >= a.tiles_q;                      // a column tile of D instead of the quantized matrix
  const int64_t col = (int64_t)(dense ? blockIdx.x - a.tiles_q : blockIdx.x) * MV_COLS + 16 * run;   // first column of the run
  const int split = blockIdx.y;
  const int64_t ra = (int64_t)split * a.rows_per_split;
  const int64_t rb = ra + a.rows_per_split < a.K ? ra + a.rows_per_split : a.K;
  const int nrows = (int)(rb - ra);
  for (int i = tid; i < (1 << BITS); i += 256) s_code[i] = a.tables->code[Slot<BITS>::value][i];
  for (int i = 0; i < M; ++i)
    for (int r = tid; r < nrows; r += 256) s_x[i][r] = i < a.m ? a.X[(int64_t)i * a.ldx + ra + r] : 0.0f;
  __syncthreads();

  float acc[M][16];
#pragma unroll
  for (int i = 0; i < M; ++i)
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[i][j] = 0.0f;
  const bool live = col < (dense ? a.Nd : a.N);   // N is a multiple of 16
  const int64_t colc = live ? col : 0;

  if (!dense) {
    // rows of the thread: local rows grp, grp + 32, ...; every load is issued before the first use (a row past the
    // end is loaded clamped and skipped)
    uint2 cw[MV_DEPTH];                           // at most 64 bits of codes per run for b0 <= 4; 8-bit codes take two passes
    uint32_t si[MV_DEPTH];
    float vv[MV_DEPTH];
    constexpr int PASSES = BITS == 8 ? 2 : 1;
#pragma unroll
    for (int pass = 0; pass < PASSES; ++pass) {
#pragma unroll
      for (int j = 0; j < MV_DEPTH; ++j) {
        int r = grp + MV_GROUPS * j;
        r = r < nrows ? r : nrows - 1;
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
        if (r < nrows) {
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
  } else if (live) {
    // 16 columns of D in the thread's rows, four rows' loads issued together; columns past Nd count as zero
    constexpr int DCH = 4;
    for (int r0 = grp; r0 < nrows; r0 += DCH * MV_GROUPS) {
      float w[DCH][16];
#pragma unroll
      for (int u = 0; u < DCH; ++u) {
        int r = r0 + u * MV_GROUPS;
        r = r < nrows ? r : nrows - 1;            // loaded clamped, skipped below
        const float* drow = a.D + (ra + r) * a.ldd + col;
        if (a.d_vec) {
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            float4 f = make_float4(0.f, 0.f, 0.f, 0.f);
            if (col + 4 * q < a.Nd) f = *reinterpret_cast<const float4*>(drow + 4 * q);
            w[u][4 * q] = f.x; w[u][4 * q + 1] = f.y; w[u][4 * q + 2] = f.z; w[u][4 * q + 3] = f.w;
          }
        } else {
#pragma unroll
          for (int j = 0; j < 16; ++j) w[u][j] = col + j < a.Nd ? drow[j] : 0.0f;
        }
      }
#pragma unroll
      for (int u = 0; u < DCH; ++u) {
        const int r = r0 + u * MV_GROUPS;
        if (r < nrows) {
#pragma unroll
          for (int i = 0; i < M; ++i) {
            const float x = s_x[i][r];
#pragma unroll
            for (int j = 0; j < 16; ++j) acc[i][j] = fmaf(x, w[u][j], acc[i][j]);
          }
        }
      }
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
    float* __restrict__ Yq = a.Y + (size_t)split * (size_t)a.m * a.ldy;
    float* __restrict__ Yd = a.Yd + (size_t)split * (size_t)a.m * a.Nd;
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
        if (!dense) {
          *reinterpret_cast<float4*>(Yq + (int64_t)i * a.ldy + col + 4 * q) = make_float4(o[0], o[1], o[2], o[3]);
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (col + 4 * q + e < a.Nd) Yd[(int64_t)i * a.Nd + col + 4 * q + e] = o[e];
        }
      }
    }
  }
}

// Second kernel: Y = sum of the ranges of X Q (in range order) + T L2 with T = sum of the ranges of X L1.  A workgroup
// owns 64 columns and M rows (blockIdx.y picks the rows); thread (column, slot) takes rows slot, slot + 4 of them
// (SLOTS = min(M, 4) slots, one wavefront each).  The workgroup first sums the rank values of T per row into LDS; the
// loads of a column of L2 are issued 32 at a time.  Both sets of partial sums are described by the distance between
// ranges and (for T) the row pitch, so the kernel also finishes the MFMA path's products of a few dozen rows.
constexpr int MVF_COLS = 64;
constexpr int MVF_RANK_MAX = 512;
// p[0] + p[stride] + ... (n terms, in this order), the loads issued eight at a time.
__device__ __forceinline__ float mvf_range_sum(const float* __restrict__ p, size_t stride, int n) {
  float s = 0.0f;
  for (int z0 = 0; z0 < n; z0 += 8) {
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = z0 + u < n ? p[(size_t)(z0 + u) * stride] : 0.0f;
#pragma unroll
    for (int u = 0; u < 8; ++u) s += v[u];
  }
  return s;
}
struct MvfArgs {
  const float* part; size_t pstride; int splits;               // ranges of X Q: range z, row i at part + z * pstride + i * N
  const float* tpart; size_t tstride; int64_t tld; int tsplits;  // ranges of T: row i at tpart + z * tstride + i * tld
  int m; int64_t N; int rank;
  const float* L2; int64_t ldl2;
  float* Y; int64_t ldy;
};
template <int M>
__global__ __launch_bounds__(MVF_COLS * (M < 4 ? M : 4)) void qmatvec_finish_kernel(MvfArgs a) {
  constexpr int SLOTS = M < 4 ? M : 4, THREADS = MVF_COLS * SLOTS, RT = (M + SLOTS - 1) / SLOTS;
  __shared__ float s_t[M][MVF_RANK_MAX];
  const int tid = threadIdx.x, slot = tid / MVF_COLS;
  const int64_t col = (int64_t)blockIdx.x * MVF_COLS + (tid % MVF_COLS);
  const int row0 = (int)blockIdx.y * M;
  const int m = a.m - row0 < M ? a.m - row0 : M;     // rows of this workgroup
  const bool live = col < a.N;
  const int64_t colc = live ? col : 0;
  // the thread's rows of X Q
  float acc[RT];
#pragma unroll
  for (int j = 0; j < RT; ++j) {
    const int i = slot + SLOTS * j;
    float s = 0.0f;
    if (i < m) s = mvf_range_sum(a.part + (size_t)(row0 + i) * a.N + colc, a.pstride, a.splits);
    acc[j] = s;
  }
  // T, with the tail up to a multiple of 32 zero
  const int rank32 = (a.rank + 31) & ~31;
  for (int idx = tid; idx < m * rank32; idx += THREADS) {
    const int i = idx / rank32, p = idx % rank32;
    float t = 0.0f;
    if (p < a.rank) t = mvf_range_sum(a.tpart + (size_t)(row0 + i) * a.tld + p, a.tstride, a.tsplits);
    s_t[i][p] = t;
  }
  __syncthreads();
  for (int p0 = 0; p0 < a.rank; p0 += 32) {
    float w[32];
#pragma unroll
    for (int u = 0; u < 32; ++u) w[u] = p0 + u < a.rank ? a.L2[(int64_t)(p0 + u) * a.ldl2 + colc] : 0.0f;
#pragma unroll
    for (int j = 0; j < RT; ++j) {
      const int i = slot + SLOTS * j;
      if (i < M) {
#pragma unroll
        for (int u = 0; u < 32; ++u) acc[j] = fmaf(s_t[i][p0 + u], w[u], acc[j]);
      }
    }
  }
#pragma unroll
  for (int j = 0; j < RT; ++j) {
    const int i = slot + SLOTS * j;
    if (live && i < m) a.Y[(int64_t)(row0 + i) * a.ldy + col] = acc[j];
  }
}

int launch_range_sum_lowrank(const float* part, size_t pstride, int splits, const float* tpart, size_t tstride,
                             int64_t tld, int tsplits, int64_t m, int64_t N, int rank, const float* L2, int64_t ldl2,
                             float* Y, int64_t ldy, hipStream_t st) {
  if (m < 1 || N < 1 || splits < 1 || rank < 0 || rank > MVF_RANK_MAX || (rank > 0 && tsplits < 1)) return LQ_ERR_SHAPE;
  const MvfArgs a{part, pstride, splits, tpart, tstride, tld, tsplits, (int)m, N, rank, L2, ldl2, Y, ldy};
  prof::Scope ps(prof::MISC, st, 4.0 * ((double)splits * m * (double)N + (double)tsplits * m * rank + (double)rank * (double)N + m * (double)N));
  const unsigned gx = (unsigned)((N + MVF_COLS - 1) / MVF_COLS);
  if (m <= 1) hipLaunchKernelGGL((qmatvec_finish_kernel<1>), dim3(gx), dim3(MVF_COLS), 0, st, a);
  else if (m <= 2) hipLaunchKernelGGL((qmatvec_finish_kernel<2>), dim3(gx), dim3(2 * MVF_COLS), 0, st, a);
  else if (m <= 4) hipLaunchKernelGGL((qmatvec_finish_kernel<4>), dim3(gx), dim3(4 * MVF_COLS), 0, st, a);
  else hipLaunchKernelGGL((qmatvec_finish_kernel<8>), dim3(gx, (unsigned)((m + 7) / 8)), dim3(4 * MVF_COLS), 0, st, a);
  LQ_HIP_TRY(hipGetLastError());
  return LQ_OK;
}

// Reduction ranges for m rows against K x (N + rank) weights: at most 512 workgroups (with 8 rows two fit a CU, and a
// few more than the machine holds would cost a second round), at most 512 rows each (a multiple of 32), and partial
// sums (splits * m * (N + rank) floats) that stay below about a quarter of a 4-bit matrix's bytes.
int qmatvec_splits(int m, int64_t K, int64_t N, int rank) {
  const int64_t tiles = (N + MV_COLS - 1) / MV_COLS + (rank + MV_COLS - 1) / MV_COLS;
  int64_t s = std::max<int64_t>(1, 512 / tiles);
  s = std::min<int64_t>(s, std::max<int64_t>(1, K / (32 * (int64_t)std::max(m, 1))));
  s = std::max<int64_t>(s, (K + MV_ROWS_MAX - 1) / MV_ROWS_MAX);        // the X slice must fit in LDS
  int64_t rows = (K + s - 1) / s;
  rows = (rows + 31) / 32 * 32;
  return (int)std::max<int64_t>(1, (K + rows - 1) / rows);
}

size_t qmatvec_part_floats(int m, int64_t K, int64_t N, int rank) {
  const int s = qmatvec_splits(m, K, N, rank);
  return (s > 1 || rank > 0) ? (size_t)s * (size_t)m * (size_t)(N + rank) : 0;
}

template <int BITS>
static void launch_m(const MvArgs& a, dim3 grid, hipStream_t st) {
  if (a.m <= 1) hipLaunchKernelGGL((qmatvec_kernel<BITS, 1>), grid, dim3(256), 0, st, a);
  else if (a.m <= 2) hipLaunchKernelGGL((qmatvec_kernel<BITS, 2>), grid, dim3(256), 0, st, a);
  else if (a.m <= 4) hipLaunchKernelGGL((qmatvec_kernel<BITS, 4>), grid, dim3(256), 0, st, a);
  else hipLaunchKernelGGL((qmatvec_kernel<BITS, 8>), grid, dim3(256), 0, st, a);
}

int launch_qmatvec(const MvWeights& q, const float* X, int64_t ldx, int64_t K, const float* L1, const float* L2,
                   int64_t ldl2, int rank, int m, int64_t N, float* Y, int64_t ldy, float* part, size_t part_floats,
                   hipStream_t st) {
  if (m < 1 || m > QMATVEC_MAX_ROWS || K <= 0 || N <= 0 || (N % 16) != 0) return LQ_ERR_SHAPE;
  if (rank < 0 || rank > MVF_RANK_MAX) return LQ_ERR_RANK;
  if (q.block < 16 || (q.block & (q.block - 1)) != 0 || q.scale_block < 1 || (q.scale_block & (q.scale_block - 1)) != 0)
    return LQ_ERR_CONFIG;
  if ((N % q.block) != 0 || (ldy & 3) != 0) return LQ_ERR_SHAPE;
  MvArgs a{};
  a.X = X; a.ldx = ldx; a.K = K; a.N = N; a.m = m;
  a.D = L1; a.ldd = rank; a.Nd = rank;
  a.d_vec = (rank > 0 && (rank & 3) == 0 && ((uintptr_t)L1 & 15) == 0) ? 1 : 0;
  a.codes = q.codes; a.sidx = q.sidx; a.v = q.v;
  a.block_shift = __builtin_ctz((unsigned)q.block);
  a.group_shift = __builtin_ctz((unsigned)q.scale_block);
  a.levels = q.levels;
  a.splits = qmatvec_splits(m, K, N, rank);
  int64_t rows = (K + a.splits - 1) / a.splits;
  rows = (rows + 31) / 32 * 32;
  if (rows > MV_ROWS_MAX) return LQ_ERR_SHAPE;
  a.rows_per_split = (int)rows;
  a.splits = (int)((K + rows - 1) / rows);                              // no empty range
  const bool direct = a.splits == 1 && rank == 0;                       // nothing to add afterwards
  if (!direct && part_floats < (size_t)a.splits * (size_t)m * (size_t)(N + rank)) return LQ_ERR_WORKSPACE;
  a.Y = direct ? Y : part;
  a.ldy = direct ? ldy : N;
  a.Yd = direct ? nullptr : part + (size_t)a.splits * (size_t)m * (size_t)N;   // after the partial sums of X Q
  const DevTables* tab = nullptr;
  LQ_TRY(device_tables(&tab));
  a.tables = tab;
  const int64_t tiles_q = (N + MV_COLS - 1) / MV_COLS, tiles_d = (rank + MV_COLS - 1) / MV_COLS;
  if (tiles_q + tiles_d >= (1ll << 31)) return LQ_ERR_SHAPE;
  a.tiles_q = (int)tiles_q;
  const dim3 grid((unsigned)(tiles_q + tiles_d), (unsigned)a.splits);
  {
    // algorithmic bytes: the weights once (codes, one scale index per block, both factors), X, Y
    const double wbytes = (double)K * (double)N * (q.bits / 8.0 + 1.0 / q.block) + 4.0 * (double)rank * (double)(K + N);
    prof::Scope ps(prof::QMATVEC, st, wbytes + 4.0 * m * (double)(K + N));
    switch (q.bits) {
      case 2: launch_m<2>(a, grid, st); break;
      case 3: launch_m<3>(a, grid, st); break;
      case 4: launch_m<4>(a, grid, st); break;
      case 8: launch_m<8>(a, grid, st); break;
      default: return LQ_ERR_CONFIG;
    }
    LQ_HIP_TRY(hipGetLastError());
  }
  if (direct) return LQ_OK;
  return launch_range_sum_lowrank(part, (size_t)m * N, a.splits, a.Yd, (size_t)m * rank, rank, a.splits, m, N, rank, L2,
                                  ldl2, Y, ldy, st);
}

}  // namespace lq
