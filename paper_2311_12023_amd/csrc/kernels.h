// Launchers of the randomized-SVD and fused decomposition kernels (host-callable, all asynchronous on
// the given stream).  "Wide" matrices are l x m row-major with l = 32..256 rows (a multiple of 32) and
// a zero-padded leading dimension that is a multiple of 32.
#pragma once

#include "lq_internal.h"

namespace lq {

typedef NfTables DevTables;

constexpr int MODE_NT = 0;   // C[l x M] = X[l x K] * A[M x K]^T
constexpr int MODE_NN = 1;   // C[l x N] = X[l x K] * A[K x N]

struct GemmArgs {
  const float* X;
  const float* A;
  float* C;
  float* part;                        // partial tiles: 2 per workgroup, l x span floats each
  int64_t ldx, lda, ldc;
  size_t strideX, strideA, strideC;   // per-problem strides in floats (0 = shared operand)
  int64_t big;                        // extent of the large output dimension (M or N)
  int64_t K;                          // reduction length
  int tiles, ns;                      // tile positions along the large dimension, 32-deep reduction steps per problem
  int total, per_wg;                  // steps of the whole batch, steps per workgroup (share)
  // fp16-operand products only (launch_wide_gemm_f16)
  const float* A2;                    // lo plane of A: one byte per element, same layout (NN mode)
  float x_scale, out_scale;
  const double* lam0;                 // per problem: largest squared row norm of X, or NULL (x_scale applies)
  size_t strideLam;
};

int gemm_tile_span(int lt);
// Scratch (floats) that lets launch_wide_gemm cut tiles between `workgroups` workgroups (<= 0: the default count).
size_t gemm_part_floats(int l, int workgroups);
// precision 0: fp32 MFMA.  precision 1: both operands split into bf16 hi + lo on the fly and multiplied with
// three bf16 MFMAs (hi*hi + hi*lo + lo*hi, fp32 accumulation): products good to about 2^-16 relative.
int launch_wide_gemm(int mode, int l, int64_t big, int64_t K, const float* X, int64_t ldx, size_t strideX,
                     const float* A, int64_t lda, size_t strideA, float* C, int64_t ldc, size_t strideC, int batch,
                     float* part, size_t part_floats, hipStream_t st, int precision = 0, int workgroups = 0);

// The same products with A stored in fp16 (see gemm_kernels.hip); l <= 96.
bool wide_gemm_f16_supported(int l);
int launch_wide_gemm_f16(int mode, int l, int64_t big, int64_t K, const float* X, int64_t ldx, size_t strideX,
                         const uint16_t* A, const uint8_t* A_lo, int64_t lda, size_t strideA, float* C, int64_t ldc,
                         size_t strideC, int batch, float* part, size_t part_floats, float x_scale, const double* lam0,
                         size_t strideLam, float out_scale, hipStream_t st, int workgroups = 0);

// Row and column Fisher weights from a full Fisher matrix (Section 3.3): row_w = a^2, col_w = (b / mean(sqrt F))^2
// with a, b the row / column means of sqrt(F), accumulated in fp64.  scratch: fisher_scratch_doubles(d, k) doubles.
size_t fisher_scratch_doubles(int64_t d, int64_t k);
int launch_fisher_row_col(const float* F, int64_t d, int64_t k, double* scratch, float* row_w, float* col_w,
                          hipStream_t st);

// ---- forward product with a decomposed weight (matmul_kernels.hip) ------------------------------
// X (rows x K fp32, leading dimension ldx, K and ldx multiples of 4) -> its bf16 halves: hi = bf16(x),
// lo = bf16(x - hi), planes of rows_pad x K with zero rows beyond `rows`.
int launch_split_planes(const float* X, int64_t rows, int64_t K, int64_t ldx, int64_t rows_pad, uint16_t* hi,
                        uint16_t* lo, hipStream_t st);
// The same planes of X and, from the same pass over X, T = X L1 (L1: K x rank fp32, contiguous, rank at most
// SPLIT_PROJECT_MAX_RANK) as bf16 planes th / tl of rows_pad x Kd (Kd = 32 or 64, at least rank; columns beyond rank
// and rows beyond `rows` are zero).  rows_pad is a multiple of 64.  precision 1 computes T from the hi halves alone
// and leaves the lo plane of X unwritten.  `part`: split_project_part_floats(rows_pad, K) floats of scratch.
// th == NULL: the planes of T are not formed; T stays as split_project_splits(rows_pad, K) partial results in `part`
// (range z, row i at part + (z * rows_pad + i) * 64).
// `bs`: block scales to reconstruct in the same launch (see launch_block_scales; nblocks == 0: none).
constexpr int SPLIT_PROJECT_MAX_RANK = 64;
struct BlockScales {
  const uint8_t* sidx; const float* v; int64_t nblocks; int scale_block, levels;
  float* out;
};
int split_project_splits(int64_t rows_pad, int64_t K);
size_t split_project_part_floats(int64_t rows_pad, int64_t K);
int launch_split_project(const float* X, int64_t rows, int64_t K, int64_t ldx, int64_t rows_pad, const float* L1,
                         int rank, int precision, uint16_t* xh, uint16_t* xl, float* part, size_t part_floats,
                         uint16_t* th, uint16_t* tl, int Kd, const BlockScales& bs, hipStream_t st);
// Quantized part of a product: X (planes of rows_pad x K) times the K x N matrix stored as NF codes (row-major
// flattening, N a multiple of `block`, K * N below 2^31).  K is a multiple of 32; K == 0 leaves the part out.
struct QmmPart {
  const uint16_t* Xh; const uint16_t* Xl; int64_t K;
  const uint8_t* codes;
  const float* bscale;      // reconstructed scale of every block (launch_block_scales)
  int bits, block;
};
// out[b] = s^ of block b = fl32(scale_idx[b] * fl32(v[b / scale_block] / levels)), nblocks floats.
int launch_block_scales(const uint8_t* sidx, const float* v, int64_t nblocks, int scale_block, int levels, float* out,
                        hipStream_t st);
// Dense part: X (planes of rows_pad x K, K a multiple of 32, zero-filled padding) times D (rows x cols fp32, leading
// dimension ldd); rows of D beyond `rows` and columns beyond `cols` count as zero.
struct DensePart {
  const uint16_t* Xh; const uint16_t* Xl; int64_t K;
  const float* D; int64_t ldd; int64_t rows, cols;
};
// Y[m x N] (leading dimension ldy) = quantized part + dense part.  rows_pad: rows of the X planes, a multiple of 256.
// precision 0: hi and lo halves, three MFMAs per product (about 2^-16 relative per product); 1: hi halves only.
// `part`: qmatmul_part_floats(m, N, steps) floats of scratch, steps = (Kq + Kd) / 32 (0 when the tile grid fills
// the machine without cutting the reduction).
int qmatmul_splits(int64_t m, int64_t N, int nsteps);
size_t qmatmul_part_floats(int64_t m, int64_t N, int nsteps);
// splits_out: when given and the reduction was cut, the partial results stay in `part` (range z at part + z * m * N,
// nothing is written to Y) and *splits_out is their number; otherwise *splits_out = 1 and Y holds the result.
int launch_qmatmul(const QmmPart& q, const DensePart& dn, int64_t m, int64_t rows_pad, int64_t N, float* Y, int64_t ldy,
                   float* part, size_t part_floats, int precision, hipStream_t st, int* splits_out = nullptr);

// Y = sum of `splits` partial results (each m x N, contiguous, one after the other in `part`), in order.
int launch_qmatmul_reduce(const float* part, int splits, int64_t m, int64_t N, float* Y, int64_t ldy, hipStream_t st);

// ---- forward product for a few rows of X (matvec_kernels.hip) ------------------------------------
constexpr int QMATVEC_MAX_ROWS = 8;
// The K x N quantized right-hand side (row-major flattening, N a multiple of `block` and of 16).
struct MvWeights {
  const uint8_t* codes; const uint8_t* sidx; const float* v;
  int bits, block, scale_block, levels;
};
// Y[m x N] = X[m x K] * dequant(q) + (X L1) L2 with L1 (K x rank, contiguous) and L2 (rank x N, leading dimension
// ldl2), rank at most 512 (0: no low-rank part), m <= QMATVEC_MAX_ROWS, in fp32 on the vector ALU.  ldy is a multiple
// of 4.  part: qmatvec_part_floats(m, K, N, rank) floats of scratch.
int qmatvec_splits(int m, int64_t K, int64_t N, int rank);
size_t qmatvec_part_floats(int m, int64_t K, int64_t N, int rank);
int launch_qmatvec(const MvWeights& q, const float* X, int64_t ldx, int64_t K, const float* L1, const float* L2,
                   int64_t ldl2, int rank, int m, int64_t N, float* Y, int64_t ldy, float* part, size_t part_floats,
                   hipStream_t st);
// Y[m x N] = sum of `splits` partial results (range z, row i at part + z * pstride + i * N, added in order) + T L2,
// T[m x rank] = sum of `tsplits` partial results (range z, row i at tpart + z * tstride + i * tld); rank at most 512.
int launch_range_sum_lowrank(const float* part, size_t pstride, int splits, const float* tpart, size_t tstride,
                             int64_t tld, int tsplits, int64_t m, int64_t N, int rank, const float* L2, int64_t ldl2,
                             float* Y, int64_t ldy, hipStream_t st);

// ---- small dense kernels (small_kernels.hip) --------------------------------------------------
constexpr int GRAM_CHUNKS = 16;
// G[z] (l x l, fp64, row-major) = X[z] X[z]^T for wide X (l x m, fp32).  `part` holds
// batch * GRAM_CHUNKS * l * l doubles of scratch.
int launch_gram(const float* X, int l, int64_t m, int64_t ldx, size_t strideX, double* part, double* G, int batch,
                hipStream_t st);
// In-place Cholesky G = C C^T (lower C, fp64; the strict upper triangle is left untouched).  A pivot that
// is not positive relative to the largest diagonal entry marks a dependent direction: its diagonal entry
// is stored as 0 and the triangular solve zeroes that row.
int launch_cholesky(double* G, int l, int batch, hipStream_t st);
// Cholesky factor of G[z] (l x l fp64, l <= 128) and its inverse in one kernel: Cinv[z] = C^-1 as dense fp32
// l x l (zeros above the diagonal; a dependent direction gives a zero row).  cholinv_supported tells whether
// the factor fits in LDS on this device.
bool cholinv_supported(int l);
int launch_cholinv(const double* G, int l, float* Cinv, int batch, hipStream_t st);
// X[z] <- C[z]^-1 X[z] by forward substitution (C lower triangular, fp64, from launch_cholesky).
int launch_trsm(const double* Cfac, int l, float* X, int64_t m, int64_t ldx, size_t strideX, int batch,
                hipStream_t st);
// Symmetric eigen-decomposition by parallel two-sided Jacobi, fp64.  G (l x l) is destroyed.  Outputs,
// sorted by descending eigenvalue: lambda[z][l] and Ut[z] (l x l fp32, row j = j-th eigenvector).
// `vt` holds batch * l * l doubles of scratch.
int launch_jacobi_eig(double* G, int l, double* vt, float* Ut, double* lambda, int batch, hipStream_t st);
// Approximate eigenvectors (fp32 one-sided Jacobi in LDS, l <= 128) of the symmetric G[z]: rows of Ut[z] ordered by
// descending eigenvalue estimate (lambda[z], accurate to fp32 only).  G is not modified.
bool jacobi_fast_supported(int l);
int launch_jacobi_fast(const double* G, int l, float* Ut, double* lambda, int batch, hipStream_t st);
// lam[z][i] = squared norm of row i of the wide matrix X[z] (l x m), fp64.
int launch_ritz_residual(const float* G, const float* Y, const double* lam, int rows, int64_t m, int64_t ldx, double* res,
                         hipStream_t st);
int launch_row_sumsq(const float* X, int l, int64_t m, int64_t ldx, size_t strideX, double* lam, int batch,
                     hipStream_t st);
// out[1024] = max |x[i]| over n floats (out[0..1023]: per-workgroup maxima); non-finite values are skipped.
int launch_absmax(const float* x, int64_t n, float* out, hipStream_t st);
// X <- X - alpha * Y, both `count` floats (multiple of 4).
constexpr int DEFLATE_ROWS_MAX = 16;
int launch_deflate_rows(float* X, const float* L, int l, int locked, int64_t m, int64_t ldx, hipStream_t st);
int launch_lincomb3(float* X, float a, const float* Y, float b, const float* Z, float c, int64_t count, hipStream_t st);
// Fills a wide matrix (l x m, padded ld) with N(0,1) draws from a counter-based generator; pads are zeroed.
int launch_gaussian_fill(float* X, int l, int64_t m, int64_t ldx, uint64_t seed, hipStream_t st);
// out[i][j] = sr[i] * A[i][j] * sc[j]  (sr = sqrt(row_w), sc = sqrt(col_w): D_row A D_col of Eq. 5).
int launch_scale_matrix(const float* A, int64_t d, int64_t k, const float* sr, const float* sc, float* out,
                        hipStream_t st);
// s[i] = sqrt(w[i]), rs[i] = 1/sqrt(w[i]).
int launch_sqrt_vecs(const float* w, int64_t n, float* s, float* rs, hipStream_t st);
// Balanced factors from Ritz-ordered wide bases (Algorithm 4): L1[i][p] = Y[p][i] sqrt(sigma_p) rsr[i],
// L2[p][j] = B[p][j] / sqrt(sigma_p) * rsc[j], sigma_p = sqrt(lambda_p).  rsr / rsc may be NULL (= 1).
int launch_assemble_factors(const float* Y, int64_t ldy, const float* B, int64_t ldb, const double* lambda, int rank,
                            int64_t d, int64_t k, const float* rsr, const float* rsc, float* L1, float* L2,
                            hipStream_t st);

// ---- fused kernels of the LQ loop (fused_kernels.hip) -------------------------------------------
struct LoopProblem {       // one (matrix, configuration) cell of a lock-step batch; lives in device memory
  lq_config cfg;
  int32_t levels;          // 2^(b1-1) - 1
  int32_t pad[2];
};

struct PhaseArgs {
  const float* W;          // d x k, shared by the batch
  int64_t d, k;
  int rank;
  const float* Y;          // wide Ritz basis (>= rank rows used), ld = ldy, per-problem stride strideY
  const float* B;          // wide projected matrix, ld = ldb, stride strideB
  int64_t ldy, ldb;
  size_t strideY, strideB;
  uint16_t* packed;        // bf16 hi/lo planes of the factors (launch_pack_factors) or NULL: fp32 product
  size_t stridePacked;     // elements
  const float* rsr;        // 1/sqrt(row_w) (d) or NULL
  const float* rsc;        // 1/sqrt(col_w) (k) or NULL
  const float* sr;         // sqrt(row_w) or NULL
  const float* sc;         // sqrt(col_w) or NULL
  const float* row_w;      // Fisher-scale weights or NULL
  const float* col_w;
  const LoopProblem* prob; // batch entries
  const DevTables* tables; // code-books and thresholds on this device
  uint8_t* codes;   size_t strideCodes;     // bytes
  BlockRec* blk;    size_t strideBlk;       // records
  uint8_t* sidx;    size_t strideSidx;
  float* v;         size_t strideV;
  float* R;         size_t strideR;         // scaled residual sqrt(rw_i) (W - Q) sqrt(cw_j), or NULL
  uint16_t* R16;    float r_scale;          // the same residual times r_scale (a power of two) as fp16, clamped to the
                                            // fp16 range (stride strideR, in fp16 elements), or NULL
  uint8_t* R16lo;                           // with R16: what the rounding of R16 dropped, one byte per element (upper byte
                                            // of the fp16 number 2^11 (a - hi)), same layout
  float* Qd;        size_t strideQd;        // dense Q or NULL
  double* err_part; size_t strideErrPart;   // per-workgroup partial sums of the squared error
  double* err_out;  size_t strideErrOut;    // eps (norm) of this iteration, one double per problem
  int batch;
  const uint8_t* bits_host;                 // host copy of the problems' code widths (batch entries), or NULL
  double quant_bytes_per_weight;            // host bookkeeping for the profiler: sum over the batch of the bytes one
                                            // weight occupies in quantized form, b0/8 + 1/B0 + bytes(b2)/(B0 B1)
};

// Splits the first `rank` rows of Y and B into the bf16 hi/lo planes that phase 1 multiplies when a.packed is set
// (a.packed must hold packed_factor_elems(d, k, rank) elements per problem).
size_t packed_factor_elems(int64_t d, int64_t k, int rank);
int launch_pack_factors(const PhaseArgs& a, hipStream_t st);
// Phase 1: T = W - L1 L2 tile by tile (MFMA), block absmax, codes and, with_err, the per-block error sums
// (without them phase 2 still produces scale indices and v, but its error output is meaningless).
int launch_lowrank_blockquant(const PhaseArgs& a, bool with_err, hipStream_t st);
// Phase 2: Quantize-INT of the block absmax values, cast of v, and eps of the iteration (err_out; needs with_err,
// the same value phase 1 was launched with: it decides the layout of the block records).
// min_block: smallest B0 in the batch (sizes the grid).
int launch_scalequant_error(const PhaseArgs& a, int min_block, bool with_err, hipStream_t st);
// Phase 3: R = sqrt(rw_i) (W - Q) sqrt(cw_j) (fp32, or scaled fp16: R16) and / or dense Q.
int launch_residual(const PhaseArgs& a, hipStream_t st);
// Number of error partials phase 2 writes per problem for block size B0.
int64_t err_partials_per_problem(int64_t n, int block);

}  // namespace lq
