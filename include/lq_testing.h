/*
 * lq_testing.h  --  entry points that expose single kernels of the randomized SVD, and one iterate of the sweep, to
 * the test-suite, so that each building block can be checked against a plain reference on the GPU machine.  They exist
 * only in the testing build of the library (liblq_hip_testing.so: the same sources compiled with
 * -DLQ_TESTING_HOOKS plus csrc/lq_testing_hooks.cpp, which also exports everything lq.h declares); the product
 * library liblq_hip.so exports none of them and applications use lq.h only.  All pointers are device pointers, matrices
 * row-major.  "Wide" matrices have l rows (multiple of 32, at most 256) and a leading dimension that
 * is a multiple of 32 with zero padding.  Each call enqueues on `stream` and returns an lq_status.
 */
#ifndef LQ_TESTING_H_
#define LQ_TESTING_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* mode 0: C[l x big] = X[l x K] * A[big x K]^T;  mode 1: C[l x big] = X[l x K] * A[K x big], for `batch` problems
 * stored back to back (X: l x ldx each, A: its rows x lda, C: l x ldc).
 * The reduction steps of the batch are dealt out in equal shares to about `workgroups` workgroups (0 = as many
 * as the device holds at once); part: device scratch of part_floats floats for the tiles whose reduction ends up
 * cut between workgroups, at least lq_test_wide_gemm_part_floats(l, workgroups); with less (or NULL) none is cut.
 * Columns big .. ldc-1 of C are never written.
 * precision 0: fp32 MFMA; 1: bf16 hi/lo split, three bf16 MFMAs per product. */
int lq_test_wide_gemm(int mode, int l, int64_t big, int64_t K, const float* X, int64_t ldx, const float* A,
                      int64_t lda, float* C, int64_t ldc, int batch, int workgroups, float* part, size_t part_floats,
                      int precision, void* stream);
/* The same products with A stored in fp16 (l <= 96, ldx a multiple of 64): C = out_scale * X * op(A), X multiplied by
 * x_scale before it is split into fp16 halves, or, with lam0 (device, one double per problem: the largest squared row
 * norm of that X), by a power of two derived from it that is divided out again.  A_lo: NULL, or (NN mode only) a byte
 * matrix of the same layout, each byte the upper byte of an fp16 number v; the product is then taken with
 * A + v / 2048 and X split into fp16 hi + lo (about 2^-21); with one plane X is rounded to fp16 (2^-12). */
int lq_test_wide_gemm_f16(int mode, int l, int64_t big, int64_t K, const float* X, int64_t ldx, const uint16_t* A,
                          const uint8_t* A_lo, int64_t lda, float* C, int64_t ldc, int batch, int workgroups, float* part, size_t part_floats,
                          float x_scale, const double* lam0, float out_scale, void* stream);
size_t lq_test_wide_gemm_part_floats(int l, int workgroups);
/* Rows of X (l x m) are orthonormalised in place by Cholesky-QR (Gram in fp64).
 * scratch: at least 17 * l * l doubles.  alt: l * ldx floats of scratch, or NULL to force the
 * in-place triangular solve. */
int lq_test_orthonormalize(float* X, int l, int64_t m, int64_t ldx, double* scratch, float* alt, void* stream);
/* Eigen-decomposition of the symmetric l x l fp64 matrix G (destroyed): eigenvalues descending in
 * lambda (l doubles), eigenvectors as rows of Ut (l x l fp32).  scratch: l * l doubles. */
int lq_test_sym_eig(double* G, int l, float* Ut, double* lambda, double* scratch, void* stream);
/* fp32 one-sided Jacobi variant used inside the decomposition for l <= 128 (multiple of 32): rows of Ut are
 * approximate eigenvectors of the symmetric fp64 G (left untouched), ordered by descending eigenvalue
 * estimate lambda (fp32 accuracy). */
int lq_test_sym_eig_fast(const double* G, int l, float* Ut, double* lambda, void* stream);
/* The small kernels of the cold-start filter, one launch each on device arrays of l rows with leading dimension ldx
 * (a multiple of 4, m <= ldx):
 *   lincomb3:       X <- a X + b Y + c Z over all l * ldx entries (Z may be NULL: no third term).
 *   deflate_rows:   rows i >= locked of X lose their components along the first `locked` (<= 16) rows of L, which are
 *                   orthonormal; rows i < locked of X become copies of those rows of L.
 *   ritz_residual:  res[i] = |G_i - lam[i] Y_i|^2 for the first `rows` rows (lam, res: device doubles). */
int lq_test_lincomb3(float* X, float a, const float* Y, float b, const float* Z, float c, int l, int64_t ldx, void* stream);
int lq_test_deflate_rows(float* X, const float* L, int l, int locked, int64_t m, int64_t ldx, void* stream);
int lq_test_ritz_residual(const float* G, const float* Y, const double* lam, int rows, int64_t m, int64_t ldx, double* res,
                          void* stream);
/* Host-side evaluation of the code search the kernels use (threshold count for 2 and 3 bits, bucket table
 * plus two comparisons for 4 and 8 bits) on one normalised weight x; -1 for an unsupported bit width.
 * Needs no GPU. */
int lq_test_bucket_code(int bits, float x);
/* Largest LDS allocation per workgroup the device reports, in bytes. */
size_t lq_test_lds_limit(void);
/* Arms a capture for the next lq_error_table call of this host thread (of the testing library): after iteration `iter`
 * of configuration cfg_index (index into that call's cfgs) the dequantized component Q of that iterate is written to
 * Q_dense (device, d x k fp32), and, if iter < iters and sigma_next != NULL, the singular values that the Factorize of
 * iteration iter + 1 finds for W - Q are written to sigma_next (host, rank doubles).  A test can then redo exactly that
 * step of Algorithm 2 on the CPU from the same Q.  The request serves one call; cfg_index < 0 disarms it. */
int lq_test_capture_iterate(int cfg_index, int iter, float* Q_dense, double* sigma_next);

#ifdef __cplusplus
}
#endif
#endif /* LQ_TESTING_H_ */
