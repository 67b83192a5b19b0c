// fp32 MFMA GEMMs of the randomized SVD (the sketch, power-iteration and projection products of
// Algorithm 4's "SVD(A, r)"), written for gfx950's v_mfma_f32_32x32x2_f32.
//
// Every product has one skinny operand X (l x K, l = 32*LT <= 256 rows, row-major, K contiguous) and
// one large operand A that is streamed from HBM exactly once:
//   MODE_NT:  C[l x M] = X[l x K] * A[M x K]^T      (A row-major, reduction along A's rows)
//   MODE_NN:  C[l x N] = X[l x K] * A[K x N]        (A row-major, reduction down A's columns)
// The result is "wide" again (l rows), so the output of one product is the X of the next.
//
// Mapping: a workgroup has 4 wavefronts.  X's K-chunk (l x 32) is staged in LDS and shared; each
// wavefront fetches its own slice of A straight from global memory in MFMA operand layout (every
// element of A is needed by one wavefront only, so LDS staging would buy nothing) and owns
// LT x NT accumulator tiles of 32x32.  The reduction index inside a 32-chunk is permuted
// (lane half h, register e, sub-chunk c  <->  k = 8c + 4h + e) so that both operands are fetched with
// 128-bit loads; any permutation is valid as long as A and X agree on it.
// gridDim = (tiles along the large dimension, K splits, batch).  With K splits > 1 each split writes
// its own partial result and splitk_reduce_kernel adds them in a fixed order (deterministic).
#include "kernels.h"
#include "profiler.h"

namespace lq {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));   // native vector: arrays of it stay in registers
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

constexpr int PREC_FP32 = 0;     // v_mfma_f32_32x32x2_f32
constexpr int PREC_BF16X3 = 1;   // operands split into bf16 hi + lo, three v_mfma_f32_32x32x16_bf16 per product
constexpr int HPITCH = 40;       // LDS row pitch of the split X tile in bf16 elements (80 B: conflict-free b128 reads)

// a = hi + lo + O(2^-17 a) with hi, lo in bf16.
__device__ __forceinline__ void split_bf16(floatx2 v, bf16x2& hi, bf16x2& lo) {
  hi = __builtin_convertvector(v, bf16x2);
  const floatx2 back = __builtin_convertvector(hi, floatx2);
  lo = __builtin_convertvector(v - back, bf16x2);
}

constexpr int BK = 32;           // K chunk staged per step
constexpr int XPITCH = BK + 4;   // LDS row pitch in floats: 16-byte aligned rows, conflict-free b128 reads

// X tile fetch: L x 32 floats = L*8 float4, LT per thread.  X has a padded, zero-filled leading dimension that
// is a multiple of 32, so no K guard is needed on it.
template <int LT>
__device__ __forceinline__ void fetch_x(const float* __restrict__ X, int64_t ldx, int64_t k0, int tid,
                                        floatx4 (&xreg)[LT]) {
#pragma unroll
  for (int i = 0; i < LT; ++i) {
    const int idx = tid + i * 256;            // float4 index in the tile
    const int row = idx >> 3, c4 = idx & 7;
    xreg[i] = *reinterpret_cast<const floatx4*>(X + (size_t)row * ldx + k0 + c4 * 4);
  }
}

template <int LT>
__device__ __forceinline__ void stash_x(float* xs, int tid, const floatx4 (&xreg)[LT]) {
#pragma unroll
  for (int i = 0; i < LT; ++i) {
    const int idx = tid + i * 256;
    const int row = idx >> 3, c4 = idx & 7;
    *reinterpret_cast<floatx4*>(xs + row * XPITCH + c4 * 4) = xreg[i];
  }
}

// Split-precision X tile: hi and lo halves, columns permuted so that the 8 reduction indices a lane feeds to one
// 16-deep MFMA (k = 16g + 8cc + 4h + e, cc < 2, e < 4) are contiguous: position 16g + 8h + 4cc + e.
template <int LT>
__device__ __forceinline__ void stash_x_split(__bf16* xh, __bf16* xl, int tid, const floatx4 (&xreg)[LT]) {
#pragma unroll
  for (int i = 0; i < LT; ++i) {
    const int idx = tid + i * 256;
    const int row = idx >> 3, c4 = idx & 7;
    const int pos = 16 * (c4 >> 2) + 8 * (c4 & 1) + 4 * ((c4 >> 1) & 1);
    bf16x2 h0, l0, h1, l1;
    split_bf16(floatx2{xreg[i][0], xreg[i][1]}, h0, l0);
    split_bf16(floatx2{xreg[i][2], xreg[i][3]}, h1, l1);
    const bf16x4 hv = {h0[0], h0[1], h1[0], h1[1]}, lv = {l0[0], l0[1], l1[0], l1[1]};
    *reinterpret_cast<bf16x4*>(xh + row * HPITCH + pos) = hv;
    *reinterpret_cast<bf16x4*>(xl + row * HPITCH + pos) = lv;
  }
}

// A operand of one 32-chunk in MFMA layout: breg[c][e][j], k = k0 + 8c + 4h + e.
template <int MODE, int NT>
__device__ __forceinline__ void fetch_a(const float* __restrict__ A, int64_t lda, int64_t big, int64_t big0, int ln,
                                        int lh, int64_t k0, int64_t kend, float (&breg)[4][4][NT]) {
  if constexpr (MODE == MODE_NT) {
    int64_t row = big0 + ln;
    if (row >= big) row = big - 1;            // clamped rows are computed and never stored
    const float* p = A + (size_t)row * lda;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int64_t kk = k0 + 8 * c + 4 * lh;
      floatx4 f = {0.f, 0.f, 0.f, 0.f};
      if (kk < kend) f = *reinterpret_cast<const floatx4*>(p + kk);   // K and kend are multiples of 4
      breg[c][0][0] = f.x; breg[c][1][0] = f.y; breg[c][2][0] = f.z; breg[c][3][0] = f.w;
    }
  } else {
    int64_t col = big0 + (int64_t)ln * NT;
    if (col + NT > big) col = big - NT;       // big is a multiple of NT; clamped columns never stored
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int64_t kk = k0 + 8 * c + 4 * lh + e;
        if constexpr (NT == 2) {
          float2 f = make_float2(0.f, 0.f);
          if (kk < kend) f = *reinterpret_cast<const float2*>(A + (size_t)kk * lda + col);
          breg[c][e][0] = f.x; breg[c][e][1] = f.y;
        } else {
          float f = 0.f;
          if (kk < kend) f = A[(size_t)kk * lda + col];
          breg[c][e][0] = f;
        }
      }
  }
}

template <int LT, int MODE, int NT, int PREC>
__global__ __launch_bounds__(256) void wide_gemm_kernel(GemmArgs g) {
  extern __shared__ __attribute__((aligned(16))) float xs[];   // fp32: [32*LT][XPITCH]; split: hi then lo, [32*LT][HPITCH] bf16
  __bf16* xh = reinterpret_cast<__bf16*>(xs);
  __bf16* xl = xh + 32 * LT * HPITCH;
  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int ln = lane & 31, lh = lane >> 5;
  const int split = blockIdx.y, z = blockIdx.z;

  const float* __restrict__ X = g.X + (size_t)z * g.strideX;
  const float* __restrict__ A = g.A + (size_t)z * g.strideA;
  float* __restrict__ C = g.C + ((size_t)z * g.splits + split) * g.strideC;

  const int64_t kbeg = (int64_t)split * g.kchunk;
  const int64_t kend = (kbeg + g.kchunk < g.K) ? kbeg + g.kchunk : g.K;
  const int nsteps = (int)((kend - kbeg + BK - 1) / BK);

  // this wavefront's slice of the large dimension
  int64_t big0;   // first row (NT mode) or column (NN mode) of the slice
  if constexpr (MODE == MODE_NT) big0 = (int64_t)blockIdx.x * 128 + wave * 32;
  else big0 = (int64_t)blockIdx.x * (128 * NT) + wave * (32 * NT);

  floatx16 acc[LT][NT];
#pragma unroll
  for (int i = 0; i < LT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

  floatx4 xreg[LT];
  float breg[4][4][NT];
  if (nsteps > 0) {
    fetch_x<LT>(X, g.ldx, kbeg, tid, xreg);
    fetch_a<MODE, NT>(A, g.lda, g.big, big0, ln, lh, kbeg, kend, breg);
  }
  for (int step = 0; step < nsteps; ++step) {
    __syncthreads();          // everyone is done reading the previous X tile
    if constexpr (PREC == PREC_FP32) stash_x<LT>(xs, tid, xreg);
    else stash_x_split<LT>(xh, xl, tid, xreg);
    float bcur[4][4][NT];
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
      for (int e = 0; e < 4; ++e)
#pragma unroll
        for (int j = 0; j < NT; ++j) bcur[c][e][j] = breg[c][e][j];
    __syncthreads();
    if (step + 1 < nsteps) {   // next chunk's loads fly while this chunk multiplies
      const int64_t k1 = kbeg + (int64_t)(step + 1) * BK;
      fetch_x<LT>(X, g.ldx, k1, tid, xreg);
      fetch_a<MODE, NT>(A, g.lda, g.big, big0, ln, lh, k1, kend, breg);
    }
    if constexpr (PREC == PREC_BF16X3) {
#pragma unroll
      for (int gk = 0; gk < 2; ++gk) {
        // A operand of this 16-group, split into hi and lo (slot 4cc + e  <->  bcur[2gk + cc][e])
        bf16x8 ah[NT], al[NT];
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
          for (int cc = 0; cc < 2; ++cc)
#pragma unroll
            for (int e2 = 0; e2 < 2; ++e2) {
              bf16x2 h, l;
              split_bf16(floatx2{bcur[2 * gk + cc][2 * e2][j], bcur[2 * gk + cc][2 * e2 + 1][j]}, h, l);
              ah[j][4 * cc + 2 * e2] = h[0]; ah[j][4 * cc + 2 * e2 + 1] = h[1];
              al[j][4 * cc + 2 * e2] = l[0]; al[j][4 * cc + 2 * e2 + 1] = l[1];
            }
#pragma unroll
        for (int i = 0; i < LT; ++i) {
          const bf16x8 xhv = *reinterpret_cast<const bf16x8*>(xh + (32 * i + ln) * HPITCH + 16 * gk + 8 * lh);
          const bf16x8 xlv = *reinterpret_cast<const bf16x8*>(xl + (32 * i + ln) * HPITCH + 16 * gk + 8 * lh);
#pragma unroll
          for (int j = 0; j < NT; ++j) {
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xlv, ah[j], acc[i][j], 0, 0, 0);
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xhv, al[j], acc[i][j], 0, 0, 0);
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xhv, ah[j], acc[i][j], 0, 0, 0);
          }
        }
      }
    } else {
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      float av[LT][4];
#pragma unroll
      for (int i = 0; i < LT; ++i) {
        const floatx4 a4 = *reinterpret_cast<const floatx4*>(xs + (32 * i + ln) * XPITCH + 8 * c + 4 * lh);
        av[i][0] = a4.x; av[i][1] = a4.y; av[i][2] = a4.z; av[i][3] = a4.w;
      }
      // consecutive MFMAs go to different accumulators
#pragma unroll
      for (int e = 0; e < 4; ++e)
#pragma unroll
        for (int i = 0; i < LT; ++i)
#pragma unroll
          for (int j = 0; j < NT; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[i][e], bcur[c][e][j], acc[i][j], 0, 0, 0);
    }
    }
  }

  // ---- store: accumulator element e of a lane is row 8*(e/4) + 4*h + e%4, column n of its tile ----
  if constexpr (MODE == MODE_NT) {
    const int64_t col = big0 + ln;
    if (col < g.big) {
#pragma unroll
      for (int i = 0; i < LT; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int row = 32 * i + 8 * (e >> 2) + 4 * lh + (e & 3);
          C[(size_t)row * g.ldc + col] = acc[i][0][e];
        }
    }
  } else {
    const int64_t col = big0 + (int64_t)ln * NT;
    if (col + NT <= g.big) {
#pragma unroll
      for (int i = 0; i < LT; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int row = 32 * i + 8 * (e >> 2) + 4 * lh + (e & 3);
          if constexpr (NT == 2)
            *reinterpret_cast<float2*>(C + (size_t)row * g.ldc + col) = make_float2(acc[i][0][e], acc[i][1][e]);
          else
            C[(size_t)row * g.ldc + col] = acc[i][0][e];
        }
    }
  }
}

// out[z][i] = sum_s part[z][s][i], i < count (count = rows * ldc), fixed summation order.
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ part, float* __restrict__ out,
                                                            int splits, int64_t count4, size_t part_stride,
                                                            size_t out_stride) {
  const int z = blockIdx.y;
  const float4* p = reinterpret_cast<const float4*>(part + (size_t)z * splits * part_stride);
  float4* o = reinterpret_cast<float4*>(out + (size_t)z * out_stride);
  const size_t ps4 = part_stride / 4;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < count4; i += (int64_t)gridDim.x * 256) {
    float4 s = p[i];
    for (int q = 1; q < splits; ++q) {
      const float4 t = p[(size_t)q * ps4 + i];
      s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
    }
    o[i] = s;
  }
}

template <int LT, int MODE, int NT, int PREC>
static void launch_one(const GemmArgs& g, dim3 grid, hipStream_t st) {
  const size_t lds = PREC == PREC_FP32 ? (size_t)32 * LT * XPITCH * sizeof(float)
                                       : (size_t)2 * 32 * LT * HPITCH * sizeof(__bf16);
  hipLaunchKernelGGL((wide_gemm_kernel<LT, MODE, NT, PREC>), grid, dim3(256), lds, st, g);
}

template <int MODE, int PREC>
static int launch_mode(const GemmArgs& g, int lt, dim3 grid, hipStream_t st) {
  switch (lt) {
    case 1: launch_one<1, MODE, (MODE == MODE_NT ? 1 : 2), PREC>(g, grid, st); break;
    case 2: launch_one<2, MODE, (MODE == MODE_NT ? 1 : 2), PREC>(g, grid, st); break;
    case 3: launch_one<3, MODE, (MODE == MODE_NT ? 1 : 2), PREC>(g, grid, st); break;
    case 4: launch_one<4, MODE, (MODE == MODE_NT ? 1 : 2), PREC>(g, grid, st); break;
    case 5: launch_one<5, MODE, 1, PREC>(g, grid, st); break;
    case 6: launch_one<6, MODE, 1, PREC>(g, grid, st); break;
    case 7: launch_one<7, MODE, 1, PREC>(g, grid, st); break;
    case 8: launch_one<8, MODE, 1, PREC>(g, grid, st); break;
    default: return LQ_ERR_ARG;
  }
  return LQ_OK;
}

int gemm_tile_span(int mode, int lt) { return mode == MODE_NT ? 128 : (lt <= 4 ? 256 : 128); }

// Number of K splits for a product: enough workgroups to fill 256 CUs a few times over, chunks that are
// multiples of 32 and at least 256 long.
int gemm_choose_splits(int mode, int lt, int64_t big, int64_t K, int batch) {
  const int64_t tiles = (big + gemm_tile_span(mode, lt) - 1) / gemm_tile_span(mode, lt);
  const int64_t have = tiles * batch;
  int64_t s = (1024 + have - 1) / have;
  const int64_t smax = (K + 255) / 256;
  if (s > smax) s = smax;
  if (s > 32) s = 32;
  if (s < 1) s = 1;
  return (int)s;
}

// C = X * op(A) for `batch` problems.  `part` is scratch for splits > 1 (batch * splits * l * ldc floats).
int launch_wide_gemm(int mode, int l, int64_t big, int64_t K, const float* X, int64_t ldx, size_t strideX,
                     const float* A, int64_t lda, size_t strideA, float* C, int64_t ldc, size_t strideC, int batch,
                     int splits, float* part, hipStream_t st, int precision) {
  if (l % 32 != 0 || l < 32 || l > 256 || big < 1 || K < 1 || batch < 1) return LQ_ERR_ARG;
  if (mode == MODE_NN && (big % 2) != 0) return LQ_ERR_ARG;
  const int lt = l / 32;
  GemmArgs g;
  g.X = X; g.A = A; g.ldx = ldx; g.lda = lda; g.ldc = ldc; g.strideX = strideX; g.strideA = strideA;
  g.big = big; g.K = K; g.splits = splits;
  int64_t kchunk = (K + splits - 1) / splits;
  kchunk = (kchunk + BK - 1) / BK * BK;
  g.kchunk = kchunk;
  const size_t out_elems = (size_t)l * ldc;
  if (splits > 1) { g.C = part; g.strideC = out_elems; }
  else { g.C = C; g.strideC = strideC; }
  const int span = gemm_tile_span(mode, lt);
  const dim3 grid((unsigned)((big + span - 1) / span), (unsigned)splits, (unsigned)batch);
  {
    prof::Scope ps((precision == PREC_BF16X3 ? prof::GEMM_SPLIT_BASE : prof::GEMM_BASE) + mode * 8 + (lt - 1), st,
                   2.0 * l * (double)big * (double)K * batch);
    int rc;
    if (precision == PREC_BF16X3)
      rc = (mode == MODE_NT) ? launch_mode<MODE_NT, PREC_BF16X3>(g, lt, grid, st)
                             : launch_mode<MODE_NN, PREC_BF16X3>(g, lt, grid, st);
    else
      rc = (mode == MODE_NT) ? launch_mode<MODE_NT, PREC_FP32>(g, lt, grid, st)
                             : launch_mode<MODE_NN, PREC_FP32>(g, lt, grid, st);
    if (rc != LQ_OK) return rc;
  }
  LQ_HIP_TRY(hipGetLastError());
  if (splits > 1) {
    prof::Scope ps(prof::SPLITK_REDUCE, st, (double)(splits + 1) * out_elems * 4.0 * batch);
    const int64_t count4 = (int64_t)(out_elems / 4);
    const dim3 rgrid((unsigned)((count4 + 255) / 256 < 2048 ? (count4 + 255) / 256 : 2048), (unsigned)batch);
    hipLaunchKernelGGL(splitk_reduce_kernel, rgrid, dim3(256), 0, st, (const float*)part, C, splits, count4,
                       out_elems, strideC);
    LQ_HIP_TRY(hipGetLastError());
  }
  return LQ_OK;
}

}  // namespace lq
