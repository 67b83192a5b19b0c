// Forward product with an LQ-decomposed weight, Y = X (Q + L1 L2), with Q dequantized just in time inside the GEMM
// (Section 3.2 "Implementation" and Appendix A: matrix products between fp32 inputs and quantized matrices).
//
// One kernel computes  Y[m x N] = Xq[m x Kq] * dequant(codes)[Kq x N]  +  Xd[m x Kd] * D[Kd x N]  where either part
// may be empty.  The forward product is the launch
//   Y = X Q + T L2    (quantized part followed by r/32 dense steps)
// with X and T = X L1 as bf16 planes, which a first stage produces in one pass over X (project_kernels.hip) for ranks
// up to 64.  Higher ranks split X with the small kernel below and form T with a launch of this kernel,
//   T = X L1          (dense part only, N = r rounded up to 32, the extra columns are zero).
//
// Mapping: a workgroup of 512 threads (2 x 4 wavefronts, two per SIMD) owns a 256 x 256 output tile and walks the
// reduction in 32-deep steps.  Both MFMA operands sit in LDS as bf16 hi and lo halves, rows = output rows (X) or
// output columns (weights), the 32 reduction indices of a step contiguous, each double-buffered.
//  - X is split into its two bf16 planes once per call (every column tile needs the same halves); the tiles then
//    travel from global memory straight into LDS (global_load_lds_dwordx4: each lane moves 16 bytes, a wavefront
//    fills 1 KB = 16 rows), one step ahead.  No register or vector-ALU instruction touches X.  Rows are
//    64 bytes without padding; the four 16-byte units of a row are stored in the order unit ^ ((row / 2) % 4), which
//    makes the 128-bit operand reads conflict-free.
//  - The weight tile is decoded in registers: every thread fetches a 4 (reduction) x 4 (columns) patch a step or two
//    ahead (four code words from four consecutive rows of Q and the reconstructed scales of their blocks, which are
//    computed once per call), multiplies code-book value by scale (the same fl32(code * s^) that the
//    stand-alone dequantizer produces), splits it and writes 8-byte runs into the weight buffer of the next step.
//  - Each wavefront multiplies its 128 x 64 part with three v_mfma_f32_32x32x16_bf16 per tile pair (hi*hi + hi*lo +
//    lo*hi, fp32 accumulation; the bf16-only variant keeps the hi halves alone).
// Within a step the decode of the next weight tile and the MFMAs of the current one are independent; the decode is cut
// into small operations that are dealt out, by instruction count, over the individual MFMAs of the same wavefront
// (QM_OPS, qmm_step).  One barrier per step.
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
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

constexpr int QM_BM = 256, QM_BN = 256, QM_BK = 32, QM_THREADS = 512;
constexpr int QM_AT = 4;                  // 32-row tiles per wavefront (its part of the output is 128 x 64)
constexpr int QM_PITCH = 40;              // LDS row pitch of the weight tile in bf16 (80 B): conflict-free b128 reads

struct QmmArgs {
  const uint16_t* Xqh; const uint16_t* Xql;   // bf16 planes of the quantized part's X: rows_pad x Kq
  const uint16_t* Xdh; const uint16_t* Xdl;   // bf16 planes of the dense part's X: rows_pad x Kd
  const float* D; int64_t ldd;     // drows x dcols fp32; rows and columns beyond count as zero
  const uint8_t* codes;            // Kq x N, row-major flattening
  const float* bscale;             // reconstructed scale of every block of Q (Kq * N / B0 floats)
  uint32_t cw_step, blk_step;      // code bytes and blocks per 32 rows of Q
  float* Y; int64_t ldy;           // m x N (splits == 1), else partials: split s at Y + s * m * ldy
  int64_t m, N, Kq, Kd, drows, dcols;
  int block_shift;                 // log2 of the block size B0
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

// X (rows x K fp32, leading dimension ldx) -> bf16 planes hi, lo (rows_pad x K each); rows beyond `rows` are zero.
__global__ __launch_bounds__(256) void split_planes_kernel(const float* __restrict__ X, int64_t rows, int64_t K,
                                                           int64_t ldx, int64_t rows_pad, uint16_t* __restrict__ hi,
                                                           uint16_t* __restrict__ lo) {
  const int64_t kq = K >> 2, total = rows_pad * kq;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int64_t row = i / kq, c4 = (i % kq) << 2;
    float f[4] = {0.f, 0.f, 0.f, 0.f};
    if (row < rows) {
      const floatx4 x = *reinterpret_cast<const floatx4*>(X + row * ldx + c4);
      f[0] = x.x; f[1] = x.y; f[2] = x.z; f[3] = x.w;
    }
    bf16x4 h, l;
    split4(f, h, l);
    *reinterpret_cast<bf16x4*>(hi + row * K + c4) = h;
    *reinterpret_cast<bf16x4*>(lo + row * K + c4) = l;
  }
}

int launch_split_planes(const float* X, int64_t rows, int64_t K, int64_t ldx, int64_t rows_pad, uint16_t* hi,
                        uint16_t* lo, hipStream_t st) {
  if (rows <= 0 || K <= 0 || (K & 3) != 0 || (ldx & 3) != 0 || rows_pad < rows) return LQ_ERR_SHAPE;
  const int64_t total = rows_pad * (K >> 2);
  const int64_t nwg = std::min<int64_t>((total + 255) / 256, 1 << 16);
  prof::Scope ps(prof::MISC, st, 4.0 * (double)rows * (double)K + 4.0 * (double)rows_pad * (double)K);
  hipLaunchKernelGGL(split_planes_kernel, dim3((unsigned)nwg), dim3(256), 0, st, X, rows, K, ldx, rows_pad, hi, lo);
  LQ_HIP_TRY(hipGetLastError());
  return LQ_OK;
}

// Registers of the thread's prefetched 4 x 4 patch of the weight tile, either as stored (code words of its quad in 4
// consecutive rows of Q and the reconstructed scale of each row's block) or dense.
template <bool QUANT>
struct QmmPatch;
template <>
struct QmmPatch<true> {
  uint32_t cw[4];
  float sc[4];
};
template <>
struct QmmPatch<false> {
  floatx4 dn[4];
};

// Per-thread addressing that does not change from step to step.
struct QmmLane {
  int64_t col;          // first column of the weight patch
  int64_t colc;         // the same, clamped into the matrix (loaded, never stored)
  int kg, quad;         // the patch: reduction rows 4kg.., columns 4quad.. of the tile
  uint32_t xvoff;       // byte offset of the lane's 16 bytes inside an X plane for step 0, first row block of the wavefront
  uint32_t xlds;        // LDS byte offset (inside a stage's plane) of the wavefront's first row block
  uint32_t aoff[2];     // LDS byte offsets of the lane's A operand for the two 16-deep halves of a step (row tile 0)
  uint32_t boff;        // LDS element offset of the lane's B operand (column tile 0, first half)
  uint32_t cwoff[4];    // byte offset of the patch's code word in rows 4kg .. 4kg + 3 of the first step
  uint32_t blk0[4];     // index of those rows' blocks
  uint32_t cwshift;     // 3-bit codes: 4 when the quad starts in the upper half of its first byte
};

// The code words and block scales of a step sit at a wavefront-uniform distance (step * cw_step bytes, step * blk_step
// blocks) from those of the first step, so a fetch is a scalar base plus the lane's fixed 32-bit offsets.
template <int BITS, bool QUANT>
__device__ __forceinline__ void qmm_fetch_row(const QmmArgs& a, const QmmLane& t, int step, int j, QmmPatch<QUANT>& r) {
  if constexpr (QUANT) {
    const uint8_t* p = a.codes + (size_t)step * a.cw_step + t.cwoff[j];
    if constexpr (BITS == 8) r.cw[j] = *reinterpret_cast<const uint32_t*>(p);
    else if constexpr (BITS == 4) r.cw[j] = *reinterpret_cast<const uint16_t*>(p);
    else if constexpr (BITS == 2) r.cw[j] = *p;
    else r.cw[j] = ((uint32_t)p[0] | ((uint32_t)p[1] << 8)) >> t.cwshift;   // 12 bits starting at bit 12 * quad
    r.sc[j] = (a.bscale + (size_t)step * a.blk_step)[t.blk0[j]];
  } else {
    const int64_t p = (int64_t)step * QM_BK + 4 * t.kg + j;                  // within its own part
    float w[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) w[c] = (p < a.drows && t.col + c < a.dcols) ? a.D[p * a.ldd + t.col + c] : 0.0f;
    r.dn[j] = floatx4{w[0], w[1], w[2], w[3]};
  }
}

template <int BITS, bool QUANT>
__device__ __forceinline__ void qmm_fetch(const QmmArgs& a, const QmmLane& t, int step, QmmPatch<QUANT>& r) {
#pragma unroll
  for (int j = 0; j < 4; ++j) qmm_fetch_row<BITS, QUANT>(a, t, step, j, r);
}

template <int BITS, bool SPLIT, bool QUANT>
__device__ __forceinline__ void qmm_stash(const QmmArgs& a, const QmmLane& t, const QmmPatch<QUANT>& r,
                                          const float* s_code, __bf16* bh, __bf16* bl) {
  float w[4][4];                                     // [reduction index][column]
  if constexpr (QUANT) {
    constexpr uint32_t mask = (1u << BITS) - 1u;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float sh = r.sc[j];
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

// LDS of one workgroup: two X stages (hi plane, lo plane; 256 rows of 64 bytes), two weight buffers (hi, lo; 256 rows
// of QM_PITCH bf16) and the code book.
struct QmmLds {
  static constexpr uint32_t X_PLANE = QM_BM * 64, X_STAGE = 2 * X_PLANE;             // bytes
  static constexpr uint32_t B_PLANE = QM_BN * QM_PITCH * 2, B_BUF = 2 * B_PLANE;     // bytes
  static constexpr uint32_t B_BASE = 2 * X_STAGE, CODE_BASE = B_BASE + 2 * B_BUF;
  static constexpr size_t BYTES = CODE_BASE + 256 * sizeof(float);
};

// One wavefront's share of the X tile of one step: 2 row blocks of 16 rows per plane, global memory -> LDS.
// hi / lo: the planes; k_elems: the step's first reduction index; M0 carries the LDS address of each 1 KB block.
template <bool SPLIT>
__device__ __forceinline__ void qmm_dma(const uint16_t* hi, const uint16_t* lo, int64_t k_elems, int64_t row_elems,
                                        uint32_t voff, uint32_t lds) {
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const uint16_t* ph = hi + k_elems + (int64_t)j * 128 * row_elems;    // wavefront-uniform
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds + (uint32_t)j * 8192u), "v"(voff), "s"(ph)
                 : "memory", "m0");
    if constexpr (SPLIT) {
      const uint16_t* pl = lo + k_elems + (int64_t)j * 128 * row_elems;
      asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds + QmmLds::X_PLANE + (uint32_t)j * 8192u),
                   "v"(voff), "s"(pl)
                   : "memory", "m0");
    }
  }
}

// The patch fetch that a step weaves into its MFMAs: the registers it fills and the step they belong to.
template <bool QUANT>
struct QmmAhead {
  QmmPatch<QUANT>& patch;
  int fetch_step;
};

// Decode of the thread's 4 x 4 weight patch cut into small operations, so that a few can follow every MFMA of a step
// (see qmm_step).  Per output column: four code-book lookups, four products with the block scales, the bf16 hi halves
// of the column's four reduction indices and their LDS write, the remainders (two operations of two values), the lo
// halves and their write.  The operations of the columns are staggered so that a lookup's LDS latency is covered by
// another column's arithmetic, and each carries a rough instruction count by which they are dealt out evenly.
enum QmmOpKind { QM_FETCH, QM_LOOKUP, QM_SCALE, QM_HI, QM_BACK, QM_REST, QM_LO };
struct QmmOp { int kind, c, j, cost; };
#define LQ_QMM_LOOKUPS(C) {QM_LOOKUP, C, 0, 2}, {QM_LOOKUP, C, 1, 2}, {QM_LOOKUP, C, 2, 2}, {QM_LOOKUP, C, 3, 2}
#define LQ_QMM_SCALES(C) {QM_SCALE, C, 0, 1}, {QM_SCALE, C, 1, 1}, {QM_SCALE, C, 2, 1}, {QM_SCALE, C, 3, 1}
#define LQ_QMM_LOWS(C) {QM_BACK, C, 0, 3}, {QM_REST, C, 0, 2}, {QM_BACK, C, 2, 3}, {QM_REST, C, 2, 2}, {QM_LO, C, 0, 3}
constexpr QmmOp QM_OPS[] = {
    {QM_FETCH, 0, 0, 2}, {QM_FETCH, 0, 1, 2}, {QM_FETCH, 0, 2, 2}, {QM_FETCH, 0, 3, 2},
    LQ_QMM_LOOKUPS(0), LQ_QMM_LOOKUPS(1), LQ_QMM_LOOKUPS(2), LQ_QMM_LOOKUPS(3), LQ_QMM_SCALES(0), {QM_HI, 0, 0, 3},
    LQ_QMM_SCALES(1), LQ_QMM_LOWS(0), {QM_HI, 1, 0, 3}, LQ_QMM_SCALES(2), LQ_QMM_LOWS(1), {QM_HI, 2, 0, 3},
    LQ_QMM_SCALES(3), LQ_QMM_LOWS(2), {QM_HI, 3, 0, 3}, LQ_QMM_LOWS(3)};
#undef LQ_QMM_LOOKUPS
#undef LQ_QMM_SCALES
#undef LQ_QMM_LOWS
constexpr int QM_NOPS = sizeof(QM_OPS) / sizeof(QM_OPS[0]);

// 3-bit code words are assembled from two loads, which would stall a woven fetch: that variant fetches up front.
constexpr bool qmm_woven_fetch(int bits, bool quant, bool split) { return split && (!quant || bits != 3); }
constexpr bool qmm_op_used(int k, bool split, bool woven_fetch) {
  return (split || QM_OPS[k].kind < QM_BACK) && (woven_fetch || QM_OPS[k].kind != QM_FETCH);
}
// The MFMA (0 .. mfmas - 1) of the step that operation k follows: operations are spread by cumulative cost.
constexpr int qmm_op_slot(int k, int mfmas, bool split, bool woven_fetch) {
  int total = 0, before = 0;
  for (int i = 0; i < QM_NOPS; ++i) {
    if (!qmm_op_used(i, split, woven_fetch)) continue;
    if (i < k) before += QM_OPS[i].cost;
    total += QM_OPS[i].cost;
  }
  return before * mfmas / total;
}

template <int BITS, bool SPLIT, bool QUANT, int K>
__device__ __forceinline__ void qmm_stash_op(const QmmArgs& a, const QmmLane& t, const QmmAhead<QUANT>& ahead,
                                             const QmmPatch<QUANT>& r, const float* s_code, float (&w)[4][4],
                                             floatx2& back, __bf16* bh, __bf16* bl) {
  constexpr QmmOp op = QM_OPS[K];
  constexpr int c = op.c, j = op.j;
  if constexpr (op.kind == QM_FETCH) {
    qmm_fetch_row<BITS, QUANT>(a, t, ahead.fetch_step, j, ahead.patch);
  } else if constexpr (op.kind == QM_LOOKUP) {
    if constexpr (QUANT) w[j][c] = s_code[(r.cw[j] >> (c * BITS)) & ((1u << BITS) - 1u)];
    else w[j][c] = c == 0 ? r.dn[j].x : c == 1 ? r.dn[j].y : c == 2 ? r.dn[j].z : r.dn[j].w;
  } else if constexpr (op.kind == QM_SCALE) {      // the same fl32(code * s^) that Dequantize returns
    if constexpr (QUANT) w[j][c] = w[j][c] * r.sc[j];
  } else if constexpr (op.kind == QM_HI) {
    const floatx4 f = {w[0][c], w[1][c], w[2][c], w[3][c]};
    *reinterpret_cast<bf16x4*>(bh + (4 * t.quad + c) * QM_PITCH + 4 * t.kg) = __builtin_convertvector(f, bf16x4);
  } else if constexpr (op.kind == QM_BACK) {       // what the hi halves of values j, j + 1 of the column hold
    const floatx2 f = {w[j][c], w[j + 1][c]};
    back = __builtin_convertvector(__builtin_convertvector(f, bf16x2), floatx2);
  } else if constexpr (op.kind == QM_REST) {       // values j, j + 1 of the column give way to what their hi halves miss
    w[j][c] -= back.x; w[j + 1][c] -= back.y;
  } else {
    const floatx4 f = {w[0][c], w[1][c], w[2][c], w[3][c]};
    *reinterpret_cast<bf16x4*>(bl + (4 * t.quad + c) * QM_PITCH + 4 * t.kg) = __builtin_convertvector(f, bf16x4);
  }
}

// The operations that follow MFMA number M of a step with MFMAS of them.
template <int BITS, bool SPLIT, bool QUANT, int MFMAS, int M, int K = 0>
__device__ __forceinline__ void qmm_stash_after(const QmmArgs& a, const QmmLane& t, const QmmAhead<QUANT>& ahead,
                                                const QmmPatch<QUANT>& r, const float* s_code, float (&w)[4][4],
                                                floatx2& back, __bf16* bh, __bf16* bl) {
  if constexpr (K < QM_NOPS) {
    constexpr bool WF = qmm_woven_fetch(BITS, QUANT, SPLIT);
    if constexpr (qmm_op_used(K, SPLIT, WF) && qmm_op_slot(K, MFMAS, SPLIT, WF) == M)
      qmm_stash_op<BITS, SPLIT, QUANT, K>(a, t, ahead, r, s_code, w, back, bh, bl);
    qmm_stash_after<BITS, SPLIT, QUANT, MFMAS, M, K + 1>(a, t, ahead, r, s_code, w, back, bh, bl);
  }
}

// One 32-deep step of the wavefront's 128 x 64 part from the operand tiles in LDS, with the decode of the next step's
// weight patch (registers r -> LDS buffer nbh / nbl) and, in the three-term variant, the fetch of the patch after
// that (`ahead`) woven in: every MFMA is followed by the operations dealt to it and a scheduling fence, so that the vector ALU works in the shadow of the matrix pipe of the same wavefront (a
// wavefront that has an MFMA waiting for the pipe holds the SIMD's vector issue slot, so the two cannot be overlapped
// across wavefronts).  The weight operands of both 16-deep halves are read first (they are shared by the four row
// tiles); the X operands are read one row tile ahead of the MFMAs that use them.
template <int BITS, bool SPLIT, bool QUANT>
__device__ __forceinline__ void qmm_step(const QmmArgs& a, const QmmLane& t, const unsigned char* xstage,
                                         const __bf16* bhp, const __bf16* blp, const QmmPatch<QUANT>& r,
                                         const QmmAhead<QUANT>& ahead, const float* s_code, __bf16* nbh, __bf16* nbl,
                                         floatx16 (&acc)[QM_AT][2]) {
  constexpr int MFMAS = 2 * QM_AT * 2 * (SPLIT ? 3 : 1), PER = SPLIT ? 6 : 2, LAST = PER - 2;   // MFMAs per row tile
  float w[4][4];
  floatx2 back;
  bf16x8 bh[2][2], bl[2][2];
#pragma unroll
  for (int g = 0; g < 2; ++g)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int at = t.boff + 32 * j * QM_PITCH + 16 * g;
      bh[g][j] = *reinterpret_cast<const bf16x8*>(bhp + at);
      if constexpr (SPLIT) bl[g][j] = *reinterpret_cast<const bf16x8*>(blp + at);
    }
  bf16x8 ah[2], al[2];                   // current and next row tile
  ah[0] = *reinterpret_cast<const bf16x8*>(xstage + t.aoff[0]);
  if constexpr (SPLIT) al[0] = *reinterpret_cast<const bf16x8*>(xstage + QmmLds::X_PLANE + t.aoff[0]);
#define LQ_QMM_MFMA(A, B, I, J, M)                                                                         \
  {                                                                                                        \
    acc[I][J] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A, B, acc[I][J], 0, 0, 0);                         \
    qmm_stash_after<BITS, SPLIT, QUANT, MFMAS, M>(a, t, ahead, r, s_code, w, back, nbh, nbl);                             \
    __builtin_amdgcn_sched_barrier(0);                                                                     \
  }
  // one row tile (IDX = 0 .. 2 * QM_AT - 1: 16-deep half IDX / QM_AT, row tile IDX % QM_AT): the two accumulators of
  // the row tile alternate, three terms each
#define LQ_QMM_TILE(IDX)                                                                                   \
  {                                                                                                        \
    constexpr int g = (IDX) / QM_AT, i = (IDX) % QM_AT, cur = (IDX) & 1, nxt = cur ^ 1, m0 = (IDX) * PER;   \
    if constexpr ((IDX) + 1 < 2 * QM_AT) {                                                                 \
      constexpr int gn = ((IDX) + 1) / QM_AT, in = ((IDX) + 1) % QM_AT;                                    \
      ah[nxt] = *reinterpret_cast<const bf16x8*>(xstage + t.aoff[gn] + in * 2048);                         \
      if constexpr (SPLIT)                                                                                 \
        al[nxt] = *reinterpret_cast<const bf16x8*>(xstage + QmmLds::X_PLANE + t.aoff[gn] + in * 2048);     \
    }                                                                                                      \
    if constexpr (SPLIT) {                                                                                 \
      LQ_QMM_MFMA(al[cur], bh[g][0], i, 0, m0)                                                             \
      LQ_QMM_MFMA(al[cur], bh[g][1], i, 1, m0 + 1)                                                         \
      LQ_QMM_MFMA(ah[cur], bl[g][0], i, 0, m0 + 2)                                                         \
      LQ_QMM_MFMA(ah[cur], bl[g][1], i, 1, m0 + 3)                                                         \
    }                                                                                                      \
    LQ_QMM_MFMA(ah[cur], bh[g][0], i, 0, m0 + LAST)                                                         \
    LQ_QMM_MFMA(ah[cur], bh[g][1], i, 1, m0 + LAST + 1)                                                    \
  }
  static_assert(QM_AT == 4, "eight row-tile steps are written out");
  LQ_QMM_TILE(0) LQ_QMM_TILE(1) LQ_QMM_TILE(2) LQ_QMM_TILE(3)
  LQ_QMM_TILE(4) LQ_QMM_TILE(5) LQ_QMM_TILE(6) LQ_QMM_TILE(7)
#undef LQ_QMM_TILE
#undef LQ_QMM_MFMA
}

// Steps [sa, sb) of one part (numbered within the part).  At the top of step s (iteration `it` of this run) X stage
// it % 2 and weight buffer it % 2 hold step s, and one patch register set holds step s + 1.  The step starts the X
// transfer of s + 1 into the other stage (free since the barrier that ended step s - 1), then multiplies step s while
// fetching the patch of s + 2 and decoding the patch of s + 1 into the other weight buffer, waits for everything it
// has started and meets the barrier.  Prefetch indices are clamped, not guarded (the last step is fetched again and
// dropped): the body is branch-free.
template <int BITS, bool SPLIT, bool QUANT>
__device__ __forceinline__ void qmm_run(const QmmArgs& a, const QmmLane& t, int sa, int sb, const float* s_code,
                                        unsigned char* lds, uint32_t lds_addr, floatx16 (&acc)[QM_AT][2]) {
  if (sa >= sb) return;
  typedef QmmLds L;
  const int last = sb - 1;
  const uint16_t* xh = QUANT ? a.Xqh : a.Xdh;
  const uint16_t* xl = QUANT ? a.Xql : a.Xdl;
  const int64_t row_elems = QUANT ? a.Kq : a.Kd;
  QmmPatch<QUANT> ring[2];
#define LQ_QMM_XSTAGE(U) (lds + (uint32_t)(U) * L::X_STAGE)
#define LQ_QMM_BH(U) reinterpret_cast<__bf16*>(lds + L::B_BASE + (uint32_t)(U) * L::B_BUF)
#define LQ_QMM_BL(U) reinterpret_cast<__bf16*>(lds + L::B_BASE + (uint32_t)(U) * L::B_BUF + L::B_PLANE)
#define LQ_QMM_DMA(S, U)                                                                                     \
  qmm_dma<SPLIT>(xh, xl, (int64_t)((S) < last ? (S) : last) * QM_BK, row_elems, t.xvoff,                    \
                 lds_addr + (uint32_t)(U) * L::X_STAGE + t.xlds)
  LQ_QMM_DMA(sa, 0);
  qmm_fetch<BITS, QUANT>(a, t, sa, ring[0]);
  qmm_fetch<BITS, QUANT>(a, t, sa + 1 < last ? sa + 1 : last, ring[1]);
  qmm_stash<BITS, SPLIT, QUANT>(a, t, ring[0], s_code, LQ_QMM_BH(0), LQ_QMM_BL(0));
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  // U: parity of the step inside this run = its X stage, its weight buffer, and the patch registers that are free
#define LQ_QMM_STEP(U, S)                                                                                    \
  {                                                                                                          \
    const QmmAhead<QUANT> ahead = {ring[(U)], (S) + 2 < last ? (S) + 2 : last};                              \
    if constexpr (!qmm_woven_fetch(BITS, QUANT, SPLIT)) qmm_fetch<BITS, QUANT>(a, t, ahead.fetch_step, ring[(U)]); \
    LQ_QMM_DMA((S) + 1, 1 - (U));                                                                            \
    qmm_step<BITS, SPLIT, QUANT>(a, t, LQ_QMM_XSTAGE(U), LQ_QMM_BH(U), LQ_QMM_BL(U), ring[1 - (U)], ahead,   \
                                 s_code, LQ_QMM_BH(1 - (U)), LQ_QMM_BL(1 - (U)), acc);                       \
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); /* the X tile of S + 1 has landed */                    \
    __syncthreads();                                                                                         \
  }
  int s = sa;
  for (; s + 2 <= sb; s += 2) {
    LQ_QMM_STEP(0, s)
    LQ_QMM_STEP(1, s + 1)
  }
  if (s < sb) LQ_QMM_STEP(0, s)
#undef LQ_QMM_STEP
#undef LQ_QMM_DMA
#undef LQ_QMM_BH
#undef LQ_QMM_BL
#undef LQ_QMM_XSTAGE
}

template <int BITS, bool SPLIT>
__global__ __launch_bounds__(QM_THREADS, 2) void qmatmul_kernel(QmmArgs a) {
  typedef QmmLds L;
  extern __shared__ __attribute__((aligned(16))) unsigned char s_raw[];
  float* s_code = reinterpret_cast<float*>(s_raw + L::CODE_BASE);
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, ln = lane & 31, lh = lane >> 5;
  const int wm = wave >> 2, wn = wave & 3;
  for (int i = tid; i < (1 << BITS); i += QM_THREADS) s_code[i] = a.tables->code[Slot<BITS>::value][i];

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
  const int64_t row0 = (int64_t)bm * QM_BM, col0 = (int64_t)bn * QM_BN;
  const int s0 = (int)((int64_t)a.nsteps * split / a.splits), s1 = (int)((int64_t)a.nsteps * (split + 1) / a.splits);

  QmmLane t;
  t.kg = lane & 7;
  t.quad = 8 * wave + (lane >> 3);
  t.col = col0 + 4 * t.quad;
  t.colc = t.col < a.N ? t.col : a.N - 4;          // in the quantized part N is a multiple of the block size, hence of 4
  // X transfer: the wavefront's row blocks are 16 * (8j + wave), j < 2; lane -> row lane / 4 of the block and the
  // stored unit lane % 4, which holds the row's unit (lane % 4) ^ ((row / 2) % 4)
  const int xr = lane >> 2, xu = (lane & 3) ^ ((xr >> 1) & 3);
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);   // wavefront-uniform, kept in a scalar register
  t.xlds = (uint32_t)wave_s * 1024u;
  // operands: row tile 0 of the wavefront's part, unit (2g + lh) ^ ((row / 2) % 4)
  const int arow = 128 * wm + ln;
  t.aoff[0] = (uint32_t)arow * 64u + (uint32_t)(((0 + lh) ^ ((arow >> 1) & 3)) << 4);
  t.aoff[1] = (uint32_t)arow * 64u + (uint32_t)(((2 + lh) ^ ((arow >> 1) & 3)) << 4);
  t.boff = (uint32_t)((64 * wn + ln) * QM_PITCH + 8 * lh);
  const uint32_t lds_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)s_raw;
  t.cwshift = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j) {                    // the host has checked that Kq * N fits in 31 bits
    const uint32_t e = (uint32_t)(4 * t.kg + j) * (uint32_t)a.N + (uint32_t)t.colc;
    const uint32_t q = e >> 2;
    t.cwoff[j] = BITS == 8 ? 4 * q : BITS == 4 ? 2 * q : BITS == 2 ? q : (3 * q) >> 1;
    t.blk0[j] = e >> a.block_shift;
    if (BITS == 3) t.cwshift = (q & 1) * 4;        // N is a multiple of 16: the parity of q is the same in every row and step
  }

  floatx16 acc[QM_AT][2];
#pragma unroll
  for (int i = 0; i < QM_AT; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;
  __syncthreads();                     // code book in LDS

  // quantized steps first, then the dense ones; the byte offset of the lane's 16 bytes depends on the part's row length
  const int qa = s0 < a.nq ? s0 : a.nq, qb = s1 < a.nq ? s1 : a.nq;
  const int da = (s0 > a.nq ? s0 : a.nq) - a.nq, db = (s1 > a.nq ? s1 : a.nq) - a.nq;
  t.xvoff = (uint32_t)(((row0 + 16 * wave + xr) * a.Kq + 8 * xu) * 2);
  qmm_run<BITS, SPLIT, true>(a, t, qa, qb, s_code, s_raw, lds_addr, acc);
  t.xvoff = (uint32_t)(((row0 + 16 * wave + xr) * a.Kd + 8 * xu) * 2);
  qmm_run<BITS, SPLIT, false>(a, t, da, db, s_code, s_raw, lds_addr, acc);

  // accumulator element e of a lane is row 8*(e/4) + 4*lh + e%4, column ln of its 32 x 32 tile
  float* __restrict__ Y = a.Y + (size_t)split * (size_t)a.m * a.ldy;
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int64_t col = col0 + 64 * wn + 32 * j + ln;
    if (col >= a.N) continue;
#pragma unroll
    for (int i = 0; i < QM_AT; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int64_t row = row0 + 128 * wm + 32 * i + 8 * (e >> 2) + 4 * lh + (e & 3);
        if (row < a.m) Y[row * a.ldy + col] = acc[i][j][e];
      }
  }
}

// s^ of every block: fl32(index * fl32(v / levels)), as in Dequantize (Section 3.2).
__global__ __launch_bounds__(256) void block_scales_kernel(const uint8_t* __restrict__ sidx, const float* __restrict__ v,
                                                           int64_t nblocks, int group_shift, int levels,
                                                           float* __restrict__ out) {
  for (int64_t b = (int64_t)blockIdx.x * 256 + threadIdx.x; b < nblocks; b += (int64_t)gridDim.x * 256)
    out[b] = block_scale(sidx[b], v[b >> group_shift], levels);
}

int launch_block_scales(const uint8_t* sidx, const float* v, int64_t nblocks, int scale_block, int levels, float* out,
                        hipStream_t st) {
  if (nblocks <= 0 || scale_block < 1 || (scale_block & (scale_block - 1)) != 0) return LQ_ERR_SHAPE;
  prof::Scope ps(prof::MISC, st, 5.0 * (double)nblocks);
  const int64_t nwg = std::min<int64_t>((nblocks + 255) / 256, 4096);
  hipLaunchKernelGGL(block_scales_kernel, dim3((unsigned)nwg), dim3(256), 0, st, sidx, v, nblocks,
                     __builtin_ctz((unsigned)scale_block), levels, out);
  LQ_HIP_TRY(hipGetLastError());
  return LQ_OK;
}

// Y = sum over the reduction ranges of their partial results, in range order.
__global__ __launch_bounds__(256) void qmatmul_reduce_kernel(const float* __restrict__ part, int splits, int64_t m,
                                                             int64_t N, int64_t ldp, float* __restrict__ Y,
                                                             int64_t ldy) {
  const int64_t total = m * N;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int64_t row = i / N, col = i % N;
    const float* p = part + (size_t)row * ldp + col;
    float s = 0.0f;
    for (int z0 = 0; z0 < splits; z0 += 8) {       // added in range order, the loads issued eight at a time
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = z0 + u < splits ? p[(size_t)(z0 + u) * m * ldp] : 0.0f;
#pragma unroll
      for (int u = 0; u < 8; ++u) s += v[u];
    }
    Y[row * ldy + col] = s;
  }
}

// Reduction ranges for an m x N product with `nsteps` 32-deep steps: as many as keep the grid within one workgroup per
// compute unit (a second round would cost more than it saves), at least four steps per range, at most 16 ranges.
int qmatmul_splits(int64_t m, int64_t N, int nsteps) {
  const int64_t tiles = ((m + QM_BM - 1) / QM_BM) * ((N + QM_BN - 1) / QM_BN);
  const int64_t want = std::max<int64_t>(1, 256 / tiles);
  const int64_t cap = std::max<int64_t>(1, nsteps / 4);
  return (int)std::max<int64_t>(1, std::min<int64_t>(std::min(want, cap), 16));
}

size_t qmatmul_part_floats(int64_t m, int64_t N, int nsteps) {
  const int s = qmatmul_splits(m, N, nsteps);
  return s > 1 ? (size_t)s * (size_t)m * (size_t)N : 0;
}

template <int BITS, bool SPLIT>
static int launch_variant(const QmmArgs& a, dim3 grid, hipStream_t st) {
  static bool raised[64] = {};          // per device: the kernel uses more than the default 64 KB of LDS
  int dev = 0;
  LQ_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= 64) return LQ_ERR_HIP;
  if (!raised[dev]) {
    LQ_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&qmatmul_kernel<BITS, SPLIT>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)QmmLds::BYTES));
    raised[dev] = true;
  }
  hipLaunchKernelGGL((qmatmul_kernel<BITS, SPLIT>), grid, dim3(QM_THREADS), QmmLds::BYTES, st, a);
  LQ_HIP_TRY(hipGetLastError());
  return LQ_OK;
}

template <int BITS>
static int launch_bits(const QmmArgs& a, dim3 grid, bool split_precision, hipStream_t st) {
  return split_precision ? launch_variant<BITS, true>(a, grid, st) : launch_variant<BITS, false>(a, grid, st);
}

int launch_qmatmul(const QmmPart& q, const DensePart& dn, int64_t m, int64_t rows_pad, int64_t N, float* Y, int64_t ldy,
                   float* part, size_t part_floats, int precision, hipStream_t st, int* splits_out) {
  if (m <= 0 || N <= 0 || rows_pad < m || (rows_pad % 256) != 0) return LQ_ERR_SHAPE;
  if ((q.K % QM_BK) != 0 || (dn.K % QM_BK) != 0 || q.K + dn.K <= 0) return LQ_ERR_SHAPE;
  if (q.K > 0 && (q.block < 16 || (q.block & (q.block - 1)) != 0)) return LQ_ERR_CONFIG;   // a power of two
  if (q.K > 0 && ((N % q.block) != 0 || q.K * N >= ((int64_t)1 << 31))) return LQ_ERR_SHAPE;  // 32-bit code offsets
  // the X transfers address a plane with 32-bit byte offsets
  if (rows_pad * std::max(q.K, dn.K) >= ((int64_t)1 << 31)) return LQ_ERR_SHAPE;
  QmmArgs a{};
  a.Xqh = q.Xh; a.Xql = q.Xl; a.Kq = q.K;
  a.codes = q.codes; a.bscale = q.bscale;
  a.block_shift = q.K > 0 ? __builtin_ctz((unsigned)q.block) : 0;
  a.cw_step = q.K > 0 ? (uint32_t)(QM_BK * N * q.bits / 8) : 0;
  a.blk_step = q.K > 0 ? (uint32_t)(QM_BK * N / q.block) : 0;
  a.Xdh = dn.Xh; a.Xdl = dn.Xl; a.Kd = dn.K; a.D = dn.D; a.ldd = dn.ldd; a.drows = dn.rows; a.dcols = dn.cols;
  a.m = m; a.N = N;
  a.nq = (int)(q.K / QM_BK);
  a.nsteps = a.nq + (int)(dn.K / QM_BK);
  a.tiles_m = (int)((m + QM_BM - 1) / QM_BM);
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
      case 2: LQ_TRY(launch_bits<2>(a, grid, precision == 0, st)); break;
      case 3: LQ_TRY(launch_bits<3>(a, grid, precision == 0, st)); break;
      case 4: LQ_TRY(launch_bits<4>(a, grid, precision == 0, st)); break;
      case 8: LQ_TRY(launch_bits<8>(a, grid, precision == 0, st)); break;
      default: return LQ_ERR_CONFIG;
    }
  }
  if (splits_out) *splits_out = a.splits;
  else if (a.splits > 1) LQ_TRY(launch_qmatmul_reduce(part, a.splits, m, N, Y, ldy, st));
  return LQ_OK;
}

int launch_qmatmul_reduce(const float* part, int splits, int64_t m, int64_t N, float* Y, int64_t ldy, hipStream_t st) {
  prof::Scope ps(prof::MISC, st, 4.0 * (double)m * (double)N * (splits + 1));
  const int64_t nwg = std::min<int64_t>((m * N + 255) / 256, 4096);
  hipLaunchKernelGGL(qmatmul_reduce_kernel, dim3((unsigned)nwg), dim3(256), 0, st, part, splits, m, N, N, Y, ldy);
  LQ_HIP_TRY(hipGetLastError());
  return LQ_OK;
}

}  // namespace lq
