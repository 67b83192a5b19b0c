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
// wavefront fetches its own slice of A (32*NT rows or columns) straight from global memory in MFMA operand
// layout (every element of A is needed by one wavefront only, so LDS staging would buy nothing) and owns
// LT x NT accumulator tiles of 32x32.  The reduction index inside a 32-chunk is permuted
// (lane half h, register e, sub-chunk c  <->  k = 8c + 4h + e) so that both operands are fetched with
// 128-bit loads; any permutation is valid as long as A and X agree on it.
// The launch is one-dimensional: see the work decomposition at wide_gemm_kernel.
#include <algorithm>
#include <cstdlib>

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

// Lane-dependent part of the A addresses in bytes.  It does not change along the reduction, so every load is
// "uniform base + 32-bit lane offset" and needs no per-load address registers.
template <int MODE, int NT>
__device__ __forceinline__ void lane_offsets(int64_t lda, int64_t big, int64_t big0, int ln, int lh,
                                             uint32_t (&off)[NT]) {
  if constexpr (MODE == MODE_NT) {
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      int64_t row = big0 + 32 * j + ln;
      if (row >= big) row = big - 1;            // clamped rows are computed and never stored
      off[j] = (uint32_t)((row * lda + 4 * lh) * 4);
    }
  } else {
    int64_t col = big0 + (int64_t)ln * NT;
    if (col + NT > big) col = big - NT;         // big is a multiple of NT; clamped columns never stored
    off[0] = (uint32_t)((4 * lh * lda + col) * 4);
  }
}

// A operand of one 32-chunk in MFMA layout: breg[c][j][e], k = k0 + 8c + 4h + e.  GUARD: the chunk may reach
// past kend (only the last chunk of a split can).
template <int MODE, int NT, bool GUARD>
__device__ __forceinline__ void fetch_a(const float* __restrict__ A, int64_t lda, const uint32_t (&off)[NT], int lh,
                                        int64_t k0, int64_t kend, floatx4 (&breg)[4][NT]) {
  if constexpr (MODE == MODE_NT) {
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const char* base = reinterpret_cast<const char*>(A + k0 + 8 * c);
        floatx4 f = {0.f, 0.f, 0.f, 0.f};
        if (!GUARD || k0 + 8 * c + 4 * lh < kend)                       // K and kend are multiples of 4
          f = *reinterpret_cast<const floatx4*>(base + off[j]);
        breg[c][j] = f;
      }
  } else {
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const char* base = reinterpret_cast<const char*>(A + (size_t)(k0 + 8 * c + e) * lda);
        const bool ok = !GUARD || k0 + 8 * c + 4 * lh + e < kend;
        if constexpr (NT == 2) {
          floatx2 f = {0.f, 0.f};
          if (ok) f = *reinterpret_cast<const floatx2*>(base + off[0]);
          breg[c][0][e] = f.x; breg[c][1][e] = f.y;
        } else {
          float f = 0.f;
          if (ok) f = *reinterpret_cast<const float*>(base + off[0]);
          breg[c][0][e] = f;
        }
      }
  }
}

// One 32-chunk of the reduction: acc += X-chunk (in LDS) * A-chunk (in registers).
template <int LT, int NT, int PREC>
__device__ __forceinline__ void multiply_chunk(const float* xs, const __bf16* xh, const __bf16* xl, int ln, int lh,
                                               const floatx4 (&bcur)[4][NT], floatx16 (&acc)[LT][NT]) {
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
            split_bf16(floatx2{bcur[2 * gk + cc][j][2 * e2], bcur[2 * gk + cc][j][2 * e2 + 1]}, h, l);
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
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[i][e], bcur[c][j][e], acc[i][j], 0, 0, 0);
    }
  }
}

// Stores the accumulators of one wavefront.  `col0`: column of the destination that this wavefront's slice starts
// at; columns >= `limit` are not written.
template <int LT, int MODE, int NT>
__device__ __forceinline__ void store_acc(float* __restrict__ dst, int64_t ld, int64_t col0, int64_t limit, int ln,
                                          int lh, const floatx16 (&acc)[LT][NT]) {
  // accumulator element e of a lane is row 8*(e/4) + 4*h + e%4, column n of its tile
  if constexpr (MODE == MODE_NT) {
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      const int64_t col = col0 + 32 * j + ln;
      if (col < limit) {
#pragma unroll
        for (int i = 0; i < LT; ++i)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int row = 32 * i + 8 * (e >> 2) + 4 * lh + (e & 3);
            dst[(size_t)row * ld + col] = acc[i][j][e];
          }
      }
    }
  } else {
    const int64_t col = col0 + (int64_t)ln * NT;
    if (col + NT <= limit) {
#pragma unroll
      for (int i = 0; i < LT; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int row = 32 * i + 8 * (e >> 2) + 4 * lh + (e & 3);
          if constexpr (NT == 2)
            *reinterpret_cast<float2*>(dst + (size_t)row * ld + col) = make_float2(acc[i][0][e], acc[i][1][e]);
          else
            dst[(size_t)row * ld + col] = acc[i][0][e];
        }
    }
  }
}

// Work decomposition.  Output tiles are l rows x SPAN columns; the reduction of a tile is cut into 32-deep steps.
// The sequence of all steps of all problems, in order (problem, step), is dealt out in equal contiguous shares
// ("stream-K"), so every workgroup streams the same number of bytes whatever the batch size; the workgroups of one
// share, one per tile position along the large dimension, walk through A side by side (in NN mode they read whole
// rows of A between them) and all fetch the same chunks of X.  Workgroups are dispatched to the 8 XCDs round-robin by
// linear index, so the index is decoded as (share mod 8, tile, share div 8): the workgroups of a share land on one XCD
// and the X chunks they have in common are fetched into that XCD's L2 once.  A share that covers a tile's whole reduction stores the tile
// directly; a share that ends or starts inside one stores a partial tile (at most two per workgroup: slot 0 for the
// problem its first step falls in, slot 1 for the problem of its last step) and gemm_fixup_kernel adds the partial
// tiles of each cut tile in step order, which makes the result independent of timing.
//
// STAGES: depth of the register ring that holds A chunks.  While chunk s multiplies, chunks s+1 .. s+STAGES-1 are
// in flight: the kernel streams A once from HBM and what bounds it is the number of bytes each CU keeps in flight.
template <int LT, int MODE, int NT, int PREC, int STAGES>
__global__ __launch_bounds__(256, 2) void wide_gemm_kernel(GemmArgs g) {
  extern __shared__ __attribute__((aligned(16))) float xs[];   // fp32: [32*LT][XPITCH]; split: hi then lo, [32*LT][HPITCH] bf16
  __bf16* xh = reinterpret_cast<__bf16*>(xs);
  __bf16* xl = xh + 32 * LT * HPITCH;
  constexpr int SPAN = 128 * NT;
  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int ln = lane & 31, lh = lane >> 5;

  const int tile = (blockIdx.x >> 3) % g.tiles;
  const int share = (int)(blockIdx.x & 7) + 8 * (int)((blockIdx.x >> 3) / g.tiles);
  const int share0 = share * g.per_wg;
  if (share0 >= g.total) return;                 // padding of the share count to a multiple of 8
  const int share1 = share0 + g.per_wg < g.total ? share0 + g.per_wg : g.total;

  // this wavefront's slice of the large dimension: first row (NT mode) or column (NN mode)
  const int64_t big0 = (int64_t)tile * SPAN + wave * (32 * NT);
  uint32_t off[NT];
  lane_offsets<MODE, NT>(g.lda, g.big, big0, ln, lh, off);

  for (int gs = share0; gs < share1;) {
    const int z = gs / g.ns;
    const int s0 = gs - z * g.ns;
    const int s1 = g.ns - s0 < share1 - gs ? g.ns : s0 + (share1 - gs);
    const float* __restrict__ X = g.X + (size_t)z * g.strideX;
    const float* __restrict__ A = g.A + (size_t)z * g.strideA;
    const int64_t kbeg = (int64_t)s0 * BK;
    const int64_t kend = (int64_t)s1 * BK < g.K ? (int64_t)s1 * BK : g.K;
    const int nsteps = s1 - s0;

    floatx16 acc[LT][NT];
#pragma unroll
    for (int i = 0; i < LT; ++i)
#pragma unroll
      for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    // The last chunk of a reduction whose length is not a multiple of 32 is handled after the pipelined loop, so that
    // the loop itself has no guarded loads and no conditional prefetch: every load in it is issued STAGES-1 steps
    // before its first use and nothing forces an early wait.  Prefetches past the end re-read the last full chunk.
    const bool tail = s1 == g.ns && (g.K & (BK - 1)) != 0;
    const int nfull = tail ? nsteps - 1 : nsteps;
    const int64_t klast = kbeg + (int64_t)(nfull > 0 ? nfull - 1 : 0) * BK;      // last full chunk of this share
    const int64_t kxlast = kbeg + (int64_t)(nsteps - 1) * BK;

    floatx4 xreg[LT];
    floatx4 ring[STAGES][4][NT];
    fetch_x<LT>(X, g.ldx, kbeg, tid, xreg);
    if (nfull > 0) {
#pragma unroll
      for (int u = 0; u < STAGES - 1; ++u) {
        const int64_t k1 = kbeg + (int64_t)u * BK;
        fetch_a<MODE, NT, false>(A, g.lda, off, lh, k1 < klast ? k1 : klast, kend, ring[u]);
      }
    }

    // one step of the ring, U = position of the consumed chunk (compile-time so that the ring stays in registers)
#define LQ_GEMM_RING_STEP(U, STEP, PREFETCH)                                                                      \
  {                                                                                                               \
    __syncthreads(); /* everyone is done reading the previous X tile */                                           \
    if constexpr (PREC == PREC_FP32) stash_x<LT>(xs, tid, xreg);                                                  \
    else stash_x_split<LT>(xh, xl, tid, xreg);                                                                    \
    __syncthreads();                                                                                              \
    {                                                                                                             \
      const int64_t kx = kbeg + (int64_t)((STEP) + 1) * BK;                                                       \
      fetch_x<LT>(X, g.ldx, kx < kxlast ? kx : kxlast, tid, xreg);                                                \
    }                                                                                                             \
    if constexpr (PREFETCH) {                                                                                     \
      const int64_t k1 = kbeg + (int64_t)((STEP) + STAGES - 1) * BK;                                              \
      fetch_a<MODE, NT, false>(A, g.lda, off, lh, k1 < klast ? k1 : klast, kend,                                  \
                               ring[((U) + STAGES - 1) % STAGES]);                                                \
    }                                                                                                             \
    multiply_chunk<LT, NT, PREC>(xs, xh, xl, ln, lh, ring[(U)], acc);                                             \
  }
    int step0 = 0;
    for (; step0 + STAGES <= nfull; step0 += STAGES) {
      LQ_GEMM_RING_STEP(0, step0, true)
      if constexpr (STAGES > 1) LQ_GEMM_RING_STEP(1, step0 + 1, true)
      if constexpr (STAGES > 2) LQ_GEMM_RING_STEP(2, step0 + 2, true)
    }
    // the remaining full chunks are already in the ring
    if (step0 < nfull) LQ_GEMM_RING_STEP(0, step0, false)
    if constexpr (STAGES > 2) {
      if (step0 + 1 < nfull) LQ_GEMM_RING_STEP(1, step0 + 1, false)
    }
    if (tail) {
      fetch_a<MODE, NT, true>(A, g.lda, off, lh, kbeg + (int64_t)nfull * BK, kend, ring[0]);
      LQ_GEMM_RING_STEP(0, nfull, false)
    }
#undef LQ_GEMM_RING_STEP

    // whole reduction: straight into C; otherwise into this workgroup's partial tile (all SPAN columns)
    const bool whole = s0 == 0 && s1 == g.ns;
    const size_t slot = ((size_t)share * g.tiles + tile) * 2 + (gs == share0 ? 0 : 1);
    float* dst = whole ? g.C + (size_t)z * g.strideC : g.part + slot * (size_t)(32 * LT * SPAN);
    store_acc<LT, MODE, NT>(dst, whole ? g.ldc : SPAN, whole ? big0 : wave * (32 * NT), whole ? g.big : SPAN, ln, lh,
                            acc);
    gs += nsteps;
  }
}

// C tile = sum of its partial tiles in step order, for every tile whose reduction was cut between workgroups.
// gridDim = (tiles, problems, l / 8): one workgroup per 8 rows of a tile, at most two float4 per thread.
__global__ __launch_bounds__(256) void gemm_fixup_kernel(GemmArgs g, int l, int span) {
  const int t = blockIdx.x, z = blockIdx.y;
  const int start = z * g.ns, end = start + g.ns;
  const int w0 = start / g.per_wg, w1 = (end - 1) / g.per_wg;
  if (w0 == w1) return;                          // stored directly by its only workgroup
  float* __restrict__ C = g.C + (size_t)z * g.strideC;
  const int64_t col0 = (int64_t)t * span;
  const size_t tile_floats = (size_t)l * span;
  const int quads = span / 4;
  for (int idx = threadIdx.x; idx < 8 * quads; idx += 256) {
    const int row = 8 * blockIdx.z + idx / quads, c4 = (idx % quads) * 4;
    if (col0 + c4 >= g.big) continue;
    const float* p0 = g.part + (size_t)row * span + c4;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll 4
    for (int w = w0; w <= w1; ++w) {
      const size_t slot = ((size_t)w * g.tiles + t) * 2 + (start <= w * g.per_wg ? 0 : 1);
      const float4 p = *reinterpret_cast<const float4*>(p0 + slot * tile_floats);
      s.x += p.x; s.y += p.y; s.z += p.z; s.w += p.w;
    }
    float* o = C + (size_t)row * g.ldc + col0 + c4;
    if (col0 + c4 + 4 <= g.big) *reinterpret_cast<float4*>(o) = s;
    else {
      const float v[4] = {s.x, s.y, s.z, s.w};
      for (int e = 0; e < 4 && col0 + c4 + e < g.big; ++e) o[e] = v[e];
    }
  }
}

// ------------------------------------------------------------------------------------------------
// Products whose large operand is stored in fp16 (the residual W - Q of the warm LQ iterations, scaled by a power of
// two so that it sits in the middle of the fp16 range): half the bytes of the fp32 form stream from HBM, which is
// what bounds these products.  PLANES == 1: A is one fp16 plane and X is rounded to fp16 as well (after scaling by a
// power of two xs that keeps its entries normal numbers): one v_mfma_f32_32x32x16_f16 per product, about 2^-12 relative
// per operand; for the products that only steer a subspace.  PLANES == 2 (NN mode): A comes as the fp16 plane hi plus a byte
// plane, each byte the upper byte of the fp16 number 2^11 (a - hi) (14 significant bits together), X is split into fp16
// hi + lo, and a product is three MFMAs (xl * ah + (2^-11 xh) * al + xh * ah); used where the rounding of an operand to
// fp16 would show in the result to first order.  The result is multiplied by out_scale (a power of two) when stored.
// Same work decomposition, tile shapes and fix-up as wide_gemm_kernel; the reduction is cut into steps of 64 (one
// plane) or 32 (two planes), and both operands keep the natural order of the reduction index.
typedef _Float16 halfx8 __attribute__((ext_vector_type(8)));
typedef _Float16 halfx4 __attribute__((ext_vector_type(4)));
typedef uint32_t uintx4 __attribute__((ext_vector_type(4)));

constexpr int HP16 = 64 + 8;     // LDS row pitch of the X halves in fp16 elements (144 B: conflict-free b128 reads)

// X tile: L x (16 G) floats, LT * G / 2 float4 per thread.  The leading dimension of X is a multiple of 64.
template <int LT, int G>
__device__ __forceinline__ void fetch_x16(const float* __restrict__ X, int64_t ldx, int64_t k0, int tid,
                                          floatx4 (&xreg)[LT * G / 2]) {
#pragma unroll
  for (int i = 0; i < LT * G / 2; ++i) {
    const int idx = tid + i * 256;
    const int row = idx / (4 * G), c4 = idx % (4 * G);
    xreg[i] = *reinterpret_cast<const floatx4*>(X + (size_t)row * ldx + k0 + c4 * 4);
  }
}

template <int LT, int G, bool LO>
__device__ __forceinline__ void stash_x16(_Float16* xh, _Float16* xl, int tid, float xs,
                                          const floatx4 (&xreg)[LT * G / 2]) {
#pragma unroll
  for (int i = 0; i < LT * G / 2; ++i) {
    const int idx = tid + i * 256;
    const int row = idx / (4 * G), c4 = idx % (4 * G);
    const floatx4 v = xreg[i] * xs;
    const halfx4 h = __builtin_convertvector(v, halfx4);
    *reinterpret_cast<halfx4*>(xh + row * HP16 + 4 * c4) = h;
    if constexpr (LO) {
      const halfx4 l = __builtin_convertvector(v - __builtin_convertvector(h, floatx4), halfx4);
      *reinterpret_cast<halfx4*>(xl + row * HP16 + 4 * c4) = l;
    }
  }
}

template <int MODE>
__device__ __forceinline__ void lane_offsets16(int64_t lda, int64_t big, int64_t big0, int ln, int lh,
                                               uint32_t (&off)[2]) {
  if constexpr (MODE == MODE_NT) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      int64_t row = big0 + 32 * j + ln;
      if (row >= big) row = big - 1;            // clamped rows are computed and never stored
      off[j] = (uint32_t)((row * lda + 8 * lh) * 2);
    }
  } else {
    int64_t col = big0 + (int64_t)ln * 2;
    if (col + 2 > big) col = big - 2;           // big is even; clamped columns never stored
    off[0] = (uint32_t)((8 * lh * lda + col) * 2);
    off[1] = 0;
  }
}

// One plane of the A operand of a step as it comes from memory (plain loads: in NT mode a 128-byte line of a row is
// consumed by four loads of the same wavefront, which rely on the caches; streaming loads made that mode 40 % slower).
// NT mode: ring[g][j] = the 8 halves
// k0 + 16 g + 8 h + (0..7) of row j's lane row.  NN mode: ring[g][e / 4][e % 4] = the word holding columns col, col + 1
// of reduction row k0 + 16 g + 8 h + e.
template <int MODE, int G, bool GUARD>
__device__ __forceinline__ void fetch_a16(const _Float16* __restrict__ A, int64_t lda, const uint32_t (&off)[2], int lh,
                                          int64_t k0, int64_t kend, uintx4 (&ring)[G][2]) {
  const uintx4 zero = {0u, 0u, 0u, 0u};
  if constexpr (MODE == MODE_NT) {
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const char* base = reinterpret_cast<const char*>(A + k0 + 16 * g);
        uintx4 f = zero;
        if (!GUARD || k0 + 16 * g + 8 * lh < kend)                      // K and kend are multiples of 8
          f = *reinterpret_cast<const uintx4*>(base + off[j]);
        ring[g][j] = f;
      }
  } else {
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const char* base = reinterpret_cast<const char*>(A + (size_t)(k0 + 16 * g + e) * lda);
        uint32_t f = 0u;
        if (!GUARD || k0 + 16 * g + 8 * lh + e < kend) f = *reinterpret_cast<const uint32_t*>(base + off[0]);
        ring[g][e >> 2][e & 3] = f;
      }
  }
}

// The two MFMA operands (columns j = 0, 1 of the lane's pair) of 16-group g from a fetched plane.
template <int MODE, int G>
__device__ __forceinline__ void operands16(const uintx4 (&cur)[G][2], int g, halfx8 (&av)[2]) {
  if constexpr (MODE == MODE_NT) {
    av[0] = __builtin_bit_cast(halfx8, cur[g][0]);
    av[1] = __builtin_bit_cast(halfx8, cur[g][1]);
  } else {
    // words (col, col + 1) of 8 reduction rows -> the 8 halves of column col and of column col + 1
    uintx4 c0, c1;
#pragma unroll
    for (int m = 0; m < 4; ++m) {
      const uint32_t w0 = cur[g][m >> 1][2 * (m & 1)], w1 = cur[g][m >> 1][2 * (m & 1) + 1];
      c0[m] = __builtin_amdgcn_perm(w1, w0, 0x05040100u);
      c1[m] = __builtin_amdgcn_perm(w1, w0, 0x07060302u);
    }
    av[0] = __builtin_bit_cast(halfx8, c0);
    av[1] = __builtin_bit_cast(halfx8, c1);
  }
}

// The lo plane of the residual: one byte per element, the upper byte of the fp16 number 2^11 (a - hi) (sign, five exponent
// bits, two fraction bits).  NN mode only: ring[g][e / 4][e % 4] = the 16 bits holding columns col, col + 1 of reduction
// row k0 + 16 g + 8 h + e; off is the lane's byte offset in the fp16 plane, i.e. twice the one here.
constexpr float LO8_SCALE = 2048.0f;

template <int G, bool GUARD>
__device__ __forceinline__ void fetch_a8(const uint8_t* __restrict__ A, int64_t lda, uint32_t off, int lh, int64_t k0,
                                         int64_t kend, uintx4 (&ring)[G][2]) {
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const uint8_t* base = A + (size_t)(k0 + 16 * g + e) * lda;
      uint32_t f = 0u;
      if (!GUARD || k0 + 16 * g + 8 * lh + e < kend) f = *reinterpret_cast<const uint16_t*>(base + (off >> 1));
      ring[g][e >> 2][e & 3] = f;
    }
}

// bytes (col, col + 1) of 8 reduction rows -> the 8 halves (byte << 8) of column col and of column col + 1
template <int G>
__device__ __forceinline__ void operands8(const uintx4 (&cur)[G][2], int g, halfx8 (&av)[2]) {
  uintx4 c0, c1;
#pragma unroll
  for (int m = 0; m < 4; ++m) {
    const uint32_t w0 = cur[g][m >> 1][2 * (m & 1)], w1 = cur[g][m >> 1][2 * (m & 1) + 1];
    c0[m] = __builtin_amdgcn_perm(w1, w0, 0x040c000cu);
    c1[m] = __builtin_amdgcn_perm(w1, w0, 0x050c010cu);
  }
  av[0] = __builtin_bit_cast(halfx8, c0);
  av[1] = __builtin_bit_cast(halfx8, c1);
}

// NT mode with one plane, staged through LDS.  Loading a row's 8 halves per lane and MFMA (above) touches every 128-byte
// line of a row with four load instructions of 32 bytes each.  Here a wavefront loads its 64 rows of a 64-deep step with
// full lines (instruction i: lane l takes the 16-byte piece l % 8 of row 8 i + l / 8), writes them to its own LDS
// stage (row pitch 144 bytes) and reads them back in operand layout; only the wavefront itself touches the stage, so no
// barrier is involved (LDS operations of a wavefront complete in order).
constexpr int STAGE_PITCH = 72;                  // fp16 elements per staged row: 64 + 8 (conflict-free 128-bit reads)
constexpr int STAGE_HALVES = 64 * STAGE_PITCH;   // per wavefront

__device__ __forceinline__ void lane_offsets_staged(int64_t lda, int64_t big, int64_t big0, int lane, uint32_t (&off)[8]) {
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    int64_t row = big0 + 8 * i + (lane >> 3);
    if (row >= big) row = big - 1;              // clamped rows are computed and never stored
    off[i] = (uint32_t)((row * lda + 8 * (lane & 7)) * 2);
  }
}

template <bool GUARD>
__device__ __forceinline__ void fetch_a_staged(const _Float16* __restrict__ A, const uint32_t (&off)[8], int lane,
                                               int64_t k0, int64_t kend, uintx4 (&ring)[4][2]) {
  const uintx4 zero = {0u, 0u, 0u, 0u};
  const char* base = reinterpret_cast<const char*>(A + k0);
  const bool ok = !GUARD || k0 + 8 * (lane & 7) < kend;             // K and kend are multiples of 8
#pragma unroll
  for (int i = 0; i < 8; ++i) ring[i >> 1][i & 1] = ok ? *reinterpret_cast<const uintx4*>(base + off[i]) : zero;
}

template <int LT>
__device__ __forceinline__ void multiply_chunk_staged(const _Float16* xh, const _Float16* xl, _Float16* stage, int lane,
                                                      const uintx4 (&cur)[1][4][2], floatx16 (&acc)[LT][2]) {
  const int ln = lane & 31, lh = lane >> 5;
#pragma unroll
  for (int i = 0; i < 8; ++i)
    *reinterpret_cast<uintx4*>(stage + (8 * i + (lane >> 3)) * STAGE_PITCH + 8 * (lane & 7)) = cur[0][i >> 1][i & 1];
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    halfx8 av[2];
#pragma unroll
    for (int j = 0; j < 2; ++j)
      av[j] = *reinterpret_cast<const halfx8*>(stage + (32 * j + ln) * STAGE_PITCH + 16 * g + 8 * lh);
#pragma unroll
    for (int i = 0; i < LT; ++i) {
      const halfx8 xhv = *reinterpret_cast<const halfx8*>(xh + (32 * i + ln) * HP16 + 16 * g + 8 * lh);
#pragma unroll
      for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(xhv, av[j], acc[i][j], 0, 0, 0);
    }
  }
}

template <int LT, int MODE, int PLANES, int G>
__device__ __forceinline__ void multiply_chunk16(const _Float16* xh, const _Float16* xl, int ln, int lh,
                                                 const uintx4 (&cur)[PLANES][G][2], floatx16 (&acc)[LT][2]) {
#pragma unroll
  for (int g = 0; g < G; ++g) {
    halfx8 ah[2], al[2];
    operands16<MODE, G>(cur[0], g, ah);
    if constexpr (PLANES == 2) operands8<G>(cur[1], g, al);
#pragma unroll
    for (int i = 0; i < LT; ++i) {
      const halfx8 xhv = *reinterpret_cast<const halfx8*>(xh + (32 * i + ln) * HP16 + 16 * g + 8 * lh);
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        if constexpr (PLANES == 2) {
          const halfx8 xlv = *reinterpret_cast<const halfx8*>(xl + (32 * i + ln) * HP16 + 16 * g + 8 * lh);
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(xlv, ah[j], acc[i][j], 0, 0, 0);
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(xhv * (_Float16)(1.0f / LO8_SCALE), al[j], acc[i][j], 0, 0, 0);
        }
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(xhv, ah[j], acc[i][j], 0, 0, 0);
      }
    }
  }
}

// Power of two xs with |x| xs <= 2^13 for the rows of a wide matrix whose largest squared row norm is lam0.
__device__ __forceinline__ float x_scale_from(double lam0) {
  const float s = (float)lam0;
  if (!(s > 0.0f) || !(s < 3.0e38f)) return 1.0f;
  return exp2f(13.0f - ceilf(0.5f * log2f(s)));
}

template <int LT, int MODE, int PLANES, int STAGES>
__global__ __launch_bounds__(256, STAGES > 2 ? 1 : 2) void wide_gemm_f16_kernel(GemmArgs g) {
  constexpr int NT = 2;
  constexpr int SPAN = 128 * NT;
  constexpr int G = PLANES == 1 ? 4 : 2;       // 16-groups per step
  constexpr int BKH = 16 * G;
  extern __shared__ __attribute__((aligned(16))) float xs[];   // hi then lo halves of X, [32*LT][HP16] fp16 each
  constexpr bool STAGED = MODE == MODE_NT && PLANES == 1;
  _Float16* xh = reinterpret_cast<_Float16*>(xs);
  _Float16* xl = xh + 32 * LT * HP16;
  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int ln = lane & 31, lh = lane >> 5;
  _Float16* stage = xl + 32 * LT * HP16 + wave * STAGE_HALVES;        // STAGED only

  const int tile = (blockIdx.x >> 3) % g.tiles;
  const int share = (int)(blockIdx.x & 7) + 8 * (int)((blockIdx.x >> 3) / g.tiles);
  const int share0 = share * g.per_wg;
  if (share0 >= g.total) return;                 // padding of the share count to a multiple of 8
  const int share1 = share0 + g.per_wg < g.total ? share0 + g.per_wg : g.total;

  const int64_t big0 = (int64_t)tile * SPAN + wave * (32 * NT);
  uint32_t off[2];
  uint32_t off8[STAGED ? 8 : 1];
  lane_offsets16<MODE>(g.lda, g.big, big0, ln, lh, off);
  if constexpr (STAGED) lane_offsets_staged(g.lda, g.big, big0, lane, off8);

  for (int gs = share0; gs < share1;) {
    const int z = gs / g.ns;
    const int s0 = gs - z * g.ns;
    const int s1 = g.ns - s0 < share1 - gs ? g.ns : s0 + (share1 - gs);
    const float* __restrict__ X = g.X + (size_t)z * g.strideX;
    const _Float16* __restrict__ A = reinterpret_cast<const _Float16*>(g.A) + (size_t)z * g.strideA;
    const uint8_t* __restrict__ A2 = reinterpret_cast<const uint8_t*>(g.A2) + (size_t)z * g.strideA;   // PLANES == 2: NN mode only
    const float xscale = g.lam0 ? x_scale_from(g.lam0[(size_t)z * g.strideLam]) : g.x_scale;
    const int64_t kbeg = (int64_t)s0 * BKH;
    const int64_t kend = (int64_t)s1 * BKH < g.K ? (int64_t)s1 * BKH : g.K;
    const int nsteps = s1 - s0;

    floatx16 acc[LT][NT];
#pragma unroll
    for (int i = 0; i < LT; ++i)
#pragma unroll
      for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    // as in wide_gemm_kernel: the pipelined loop has no guarded load; a partial last step is handled after it
    const bool tail = s1 == g.ns && (g.K & (BKH - 1)) != 0;
    const int nfull = tail ? nsteps - 1 : nsteps;
    const int64_t klast = kbeg + (int64_t)(nfull > 0 ? nfull - 1 : 0) * BKH;
    const int64_t kxlast = kbeg + (int64_t)(nsteps - 1) * BKH;

    floatx4 xreg[LT * G / 2];
    uintx4 ring[STAGES][PLANES][G][2];
    fetch_x16<LT, G>(X, g.ldx, kbeg, tid, xreg);
    if (nfull > 0) {
#pragma unroll
      for (int u = 0; u < STAGES - 1; ++u) {
        const int64_t k1 = kbeg + (int64_t)u * BKH;
        const int64_t k1c = k1 < klast ? k1 : klast;
        if constexpr (STAGED) fetch_a_staged<false>(A, off8, lane, k1c, kend, ring[u][0]);
        else fetch_a16<MODE, G, false>(A, g.lda, off, lh, k1c, kend, ring[u][0]);
        if constexpr (PLANES == 2) fetch_a8<G, false>(A2, g.lda, off[0], lh, k1c, kend, ring[u][1]);
      }
    }

    // one step of the ring, U = position of the consumed chunk (compile-time so that the ring stays in registers)
#define LQ_GEMM16_STEP(U, STEP, PREFETCH)                                                                         \
  {                                                                                                               \
    __syncthreads(); /* everyone is done reading the previous X tile */                                           \
    stash_x16<LT, G, PLANES == 2>(xh, xl, tid, xscale, xreg);                                                                  \
    __syncthreads();                                                                                              \
    {                                                                                                             \
      const int64_t kx = kbeg + (int64_t)((STEP) + 1) * BKH;                                                      \
      fetch_x16<LT, G>(X, g.ldx, kx < kxlast ? kx : kxlast, tid, xreg);                                           \
    }                                                                                                             \
    if constexpr (PREFETCH) {                                                                                     \
      const int64_t k1 = kbeg + (int64_t)((STEP) + STAGES - 1) * BKH;                                             \
      const int64_t k1c = k1 < klast ? k1 : klast;                                                                \
      if constexpr (STAGED) fetch_a_staged<false>(A, off8, lane, k1c, kend, ring[((U) + STAGES - 1) % STAGES][0]); \
      else fetch_a16<MODE, G, false>(A, g.lda, off, lh, k1c, kend, ring[((U) + STAGES - 1) % STAGES][0]);         \
      if constexpr (PLANES == 2)                                                                                  \
        fetch_a8<G, false>(A2, g.lda, off[0], lh, k1c, kend, ring[((U) + STAGES - 1) % STAGES][1]);              \
    }                                                                                                             \
    if constexpr (STAGED) multiply_chunk_staged<LT>(xh, xl, stage, lane, ring[(U)], acc);                         \
    else multiply_chunk16<LT, MODE, PLANES, G>(xh, xl, ln, lh, ring[(U)], acc);                                   \
  }
    int step0 = 0;
    for (; step0 + STAGES <= nfull; step0 += STAGES) {
#pragma unroll
      for (int u = 0; u < STAGES; ++u) LQ_GEMM16_STEP(u, step0 + u, true)
    }
    // the remaining full chunks are already in the ring
#pragma unroll
    for (int u = 0; u < STAGES - 1; ++u)
      if (step0 + u < nfull) LQ_GEMM16_STEP(u, step0 + u, false)
    if (tail) {
      const int64_t kt = kbeg + (int64_t)nfull * BKH;
      if constexpr (STAGED) fetch_a_staged<true>(A, off8, lane, kt, kend, ring[0][0]);
      else fetch_a16<MODE, G, true>(A, g.lda, off, lh, kt, kend, ring[0][0]);
      if constexpr (PLANES == 2) fetch_a8<G, true>(A2, g.lda, off[0], lh, kt, kend, ring[0][1]);
      LQ_GEMM16_STEP(0, nfull, false)
    }
#undef LQ_GEMM16_STEP

    const float os = g.out_scale / (g.lam0 ? xscale : 1.0f);
#pragma unroll
    for (int i = 0; i < LT; ++i)
#pragma unroll
      for (int j = 0; j < NT; ++j) acc[i][j] *= os;
    const bool whole = s0 == 0 && s1 == g.ns;
    const size_t slot = ((size_t)share * g.tiles + tile) * 2 + (gs == share0 ? 0 : 1);
    float* dst = whole ? g.C + (size_t)z * g.strideC : g.part + slot * (size_t)(32 * LT * SPAN);
    store_acc<LT, MODE, NT>(dst, whole ? g.ldc : SPAN, whole ? big0 : wave * (32 * NT), whole ? g.big : SPAN, ln, lh,
                            acc);
    gs += nsteps;
  }
}

template <int LT, int MODE, int NT, int PREC>
static void launch_one(const GemmArgs& g, dim3 grid, hipStream_t st) {
  const size_t lds = PREC == PREC_FP32 ? (size_t)32 * LT * XPITCH * sizeof(float)
                                       : (size_t)2 * 32 * LT * HPITCH * sizeof(__bf16);
  constexpr int STAGES = (LT * NT <= 6) ? 3 : 2;    // accumulators + ring must leave two wavefronts per SIMD
  hipLaunchKernelGGL((wide_gemm_kernel<LT, MODE, NT, PREC, STAGES>), grid, dim3(256), lds, st, g);
}

template <int MODE, int PREC>
static int launch_mode(const GemmArgs& g, int lt, dim3 grid, hipStream_t st) {
  switch (lt) {
    case 1: launch_one<1, MODE, 2, PREC>(g, grid, st); break;
    case 2: launch_one<2, MODE, 2, PREC>(g, grid, st); break;
    case 3: launch_one<3, MODE, 2, PREC>(g, grid, st); break;
    case 4: launch_one<4, MODE, 2, PREC>(g, grid, st); break;
    case 5: launch_one<5, MODE, 1, PREC>(g, grid, st); break;
    case 6: launch_one<6, MODE, 1, PREC>(g, grid, st); break;
    case 7: launch_one<7, MODE, 1, PREC>(g, grid, st); break;
    case 8: launch_one<8, MODE, 1, PREC>(g, grid, st); break;
    default: return LQ_ERR_ARG;
  }
  return LQ_OK;
}

int gemm_tile_span(int lt) { return lt <= 4 ? 256 : 128; }

// Workgroups that are resident at once: two per CU (the kernel is compiled for two wavefronts per SIMD).
static int resident_workgroups() {
  static thread_local int cached[16] = {0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 16) return 512;
  if (cached[dev] == 0) {
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) cus = 256;
    cached[dev] = 2 * cus;
  }
  return cached[dev];
}

// Upper bound of the partial-tile scratch: two tiles per workgroup, at most twice the requested workgroups (plus the
// rounding of the share count to a multiple of 8) run.
size_t gemm_part_floats(int l, int workgroups) {
  if (workgroups <= 0) workgroups = resident_workgroups();
  return (size_t)4 * workgroups * l * gemm_tile_span(l / 32);
}

// Number of shares along the (problem, step) sequence for `tiles` tile columns.  Shares are dealt to the 8 XCDs in
// turn, so their number is a multiple of 8; the smallest such number that fills every resident workgroup slot at
// least once is taken (more shares only add partial tiles), shares of at least 8 steps.  With at least three
// rounds of whole problems nothing is cut: the tail of the last round is short then and there are no partial tiles.
static int choose_groups(int64_t tiles, int total, int batch, int workgroups) {
  if (tiles * batch >= 3 * (int64_t)workgroups) return batch;
  int64_t g = (workgroups + tiles - 1) / tiles;
  g = (g + 7) / 8 * 8;
  while (g > 8 && (total + g - 1) / g < 8) g -= 8;
  if (g > total) g = total;
  return (int)std::max<int64_t>(g, 1);
}

// C = X * op(A) for `batch` problems.  `part` (part_floats floats) is scratch for the partial tiles;
// gemm_part_floats(l, workgroups) is enough for every shape with at most workgroups / 4 tile columns, and when
// it is too small for the chosen shares no reduction is cut (every workgroup gets whole tiles).  workgroups = 0: as
// many as are resident at once; negative: exactly -workgroups shares (for tests).
int launch_wide_gemm(int mode, int l, int64_t big, int64_t K, const float* X, int64_t ldx, size_t strideX,
                     const float* A, int64_t lda, size_t strideA, float* C, int64_t ldc, size_t strideC, int batch,
                     float* part, size_t part_floats, hipStream_t st, int precision, int workgroups) {
  if (l % 32 != 0 || l < 32 || l > 256 || big < 1 || K < 1 || batch < 1) return LQ_ERR_ARG;
  if (mode == MODE_NN && (big % 2) != 0) return LQ_ERR_ARG;
  // lane offsets into A are 32-bit byte offsets
  if ((mode == MODE_NT ? (uint64_t)big * (uint64_t)lda : (uint64_t)8 * lda + (uint64_t)big) * 4 >= (1ull << 32))
    return LQ_ERR_SHAPE;
  const int lt = l / 32;
  const int span = gemm_tile_span(lt);
  GemmArgs g;
  g.X = X; g.A = A; g.C = C; g.part = part; g.ldx = ldx; g.lda = lda; g.ldc = ldc;
  g.strideX = strideX; g.strideA = strideA; g.strideC = strideC;
  g.big = big; g.K = K;
  const int64_t tiles = (big + span - 1) / span;
  const int64_t ns = (K + BK - 1) / BK;
  if (tiles > (1 << 20) || ns * batch >= (1ll << 31)) return LQ_ERR_SHAPE;
  g.ns = (int)ns;
  g.tiles = (int)tiles;
  g.total = (int)(ns * batch);
  const int64_t forced = workgroups < 0 ? -(int64_t)workgroups : 0;     // negative: that many shares exactly
  if (workgroups <= 0) workgroups = resident_workgroups();
  int64_t groups = forced ? std::min<int64_t>(forced, g.total) : choose_groups(tiles, g.total, batch, workgroups);
  int64_t per = (g.total + groups - 1) / groups;
  if (per < 8 && !forced) per = std::min<int64_t>(8, g.total);
  // every workgroup may leave two partial tiles; without room for them only whole reductions are dealt out
  const size_t need = (size_t)2 * tiles * ((g.total + per - 1) / per) * l * span;
  const bool cut = part != nullptr && part_floats >= need && groups > 1 && batch < (1 << 16);
  g.per_wg = cut ? (int)per : (int)ns;
  const int64_t ngroups = (g.total + g.per_wg - 1) / g.per_wg;
  const dim3 grid((unsigned)(tiles * ((ngroups + 7) / 8 * 8)));
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
  if (cut && g.per_wg % g.ns != 0) {
    prof::Scope ps(prof::GEMM_FIXUP, st, (double)tiles * batch * l * span * 4.0);
    hipLaunchKernelGGL(gemm_fixup_kernel, dim3((unsigned)tiles, (unsigned)batch, (unsigned)(l / 8)), dim3(256), 0, st, g,
                       l, span);
    LQ_HIP_TRY(hipGetLastError());
  }
  return LQ_OK;
}

template <int MODE, int PLANES, int STAGES>
static int launch_f16_stages(const GemmArgs& g, int lt, dim3 grid, hipStream_t st) {
  const size_t lds = (size_t)2 * 32 * lt * HP16 * sizeof(_Float16) +
                     (MODE == MODE_NT && PLANES == 1 ? (size_t)4 * STAGE_HALVES * sizeof(_Float16) : 0);
  switch (lt) {
    case 1: hipLaunchKernelGGL((wide_gemm_f16_kernel<1, MODE, PLANES, STAGES>), grid, dim3(256), lds, st, g); break;
    case 2: hipLaunchKernelGGL((wide_gemm_f16_kernel<2, MODE, PLANES, STAGES>), grid, dim3(256), lds, st, g); break;
    case 3: hipLaunchKernelGGL((wide_gemm_f16_kernel<3, MODE, PLANES, STAGES>), grid, dim3(256), lds, st, g); break;
    default: return LQ_ERR_ARG;
  }
  return LQ_OK;
}

template <int MODE, int PLANES>
static int launch_f16_mode(const GemmArgs& g, int lt, dim3 grid, hipStream_t st) {
  // two-deep ring, two workgroups per compute unit: rings of 4 and 6 chunks with one workgroup per compute unit (the
  // registers of a whole SIMD per wavefront) were 8 % slower
  return launch_f16_stages<MODE, PLANES, 2>(g, lt, grid, st);
}

bool wide_gemm_f16_supported(int l) { return l % 32 == 0 && l >= 32 && l <= 96; }   // four row tiles spill registers

// C = out_scale * X * op(A) for `batch` problems with A stored in fp16 (strideA, lda in elements), as one plane
// (A_lo == NULL) or, NN mode only, as a hi plane plus a lo plane of one byte per element in the same layout: the upper
// byte of the fp16 number 2^11 (a - hi), which brings A to 14 significant bits.  X is scaled by x_scale before it is split into fp16 halves,
// or, when lam0 is given, by a power of two derived from lam0[z * strideLam], the largest squared row norm of X[z]
// (that scale is divided out again).  ldx must be a multiple of 64; NT mode needs K and lda to be multiples of 8,
// NN mode an even lda.
int launch_wide_gemm_f16(int mode, int l, int64_t big, int64_t K, const float* X, int64_t ldx, size_t strideX,
                         const uint16_t* A, const uint8_t* A_lo, int64_t lda, size_t strideA, float* C, int64_t ldc,
                         size_t strideC, int batch, float* part, size_t part_floats, float x_scale, const double* lam0,
                         size_t strideLam, float out_scale, hipStream_t st, int workgroups) {
  if (A_lo && mode != MODE_NN) return LQ_ERR_ARG;      // the byte plane is read in NN layout only
  if (!wide_gemm_f16_supported(l) || big < 1 || K < 1 || batch < 1 || ldx % 64 != 0) return LQ_ERR_ARG;
  if (mode == MODE_NN && ((big % 2) != 0 || (lda % 2) != 0)) return LQ_ERR_ARG;
  if (mode == MODE_NT && ((K % 8) != 0 || (lda % 8) != 0)) return LQ_ERR_ARG;
  // lane offsets into A are 32-bit byte offsets
  if ((mode == MODE_NT ? (uint64_t)big * (uint64_t)lda : (uint64_t)16 * lda + (uint64_t)big) * 2 >= (1ull << 32))
    return LQ_ERR_SHAPE;
  const int lt = l / 32;
  const int span = 256;
  const int bk = A_lo ? 32 : 64;
  GemmArgs g;
  g.X = X; g.A = reinterpret_cast<const float*>(A); g.A2 = A_lo ? reinterpret_cast<const float*>(A_lo) : reinterpret_cast<const float*>(A);
  g.C = C; g.part = part; g.ldx = ldx; g.lda = lda; g.ldc = ldc;
  g.strideX = strideX; g.strideA = strideA; g.strideC = strideC;
  g.big = big; g.K = K;
  g.x_scale = x_scale; g.out_scale = out_scale; g.lam0 = lam0; g.strideLam = strideLam;
  const int64_t tiles = (big + span - 1) / span;
  const int64_t ns = (K + bk - 1) / bk;
  if (tiles > (1 << 20) || ns * batch >= (1ll << 31)) return LQ_ERR_SHAPE;
  g.ns = (int)ns;
  g.tiles = (int)tiles;
  g.total = (int)(ns * batch);
  const int64_t forced = workgroups < 0 ? -(int64_t)workgroups : 0;
  if (workgroups <= 0) workgroups = resident_workgroups();
  int64_t groups = forced ? std::min<int64_t>(forced, g.total) : choose_groups(tiles, g.total, batch, workgroups);
  int64_t per = (g.total + groups - 1) / groups;
  if (per < 4 && !forced) per = std::min<int64_t>(4, g.total);
  const size_t need = (size_t)2 * tiles * ((g.total + per - 1) / per) * l * span;
  const bool cut = part != nullptr && part_floats >= need && groups > 1 && batch < (1 << 16);
  g.per_wg = cut ? (int)per : (int)ns;
  const int64_t ngroups = (g.total + g.per_wg - 1) / g.per_wg;
  const dim3 grid((unsigned)(tiles * ((ngroups + 7) / 8 * 8)));
  {
    prof::Scope ps(prof::GEMM_F16_BASE + (A_lo ? 8 : 0) + mode * 4 + (lt - 1), st, 2.0 * l * (double)big * (double)K * batch);
    int rc;
    if (A_lo) rc = launch_f16_mode<MODE_NN, 2>(g, lt, grid, st);
    else rc = mode == MODE_NT ? launch_f16_mode<MODE_NT, 1>(g, lt, grid, st) : launch_f16_mode<MODE_NN, 1>(g, lt, grid, st);
    if (rc != LQ_OK) return rc;
  }
  LQ_HIP_TRY(hipGetLastError());
  if (cut && g.per_wg % g.ns != 0) {
    prof::Scope ps(prof::GEMM_FIXUP, st, (double)tiles * batch * l * span * 4.0);
    hipLaunchKernelGGL(gemm_fixup_kernel, dim3((unsigned)tiles, (unsigned)batch, (unsigned)(l / 8)), dim3(256), 0, st, g,
                       l, span);
    LQ_HIP_TRY(hipGetLastError());
  }
  return LQ_OK;
}

}  // namespace lq
