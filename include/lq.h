/*
 * lq.h  --  C ABI of the MI355X (gfx950) LQ decomposition library.
 *
 * The library computes the low-rank plus quantized decomposition  W ~= Q + L1 L2  of LQ-LoRA
 * (arxiv 2311.12023, Section 3) and the per-matrix error table that feeds the paper's integer
 * linear program (Algorithm 3), with every step running in hand-written HIP kernels.
 *
 * Conventions for every entry point
 *  - Matrix and vector arguments are DEVICE pointers unless the comment says "host".  Matrices are
 *    row-major, contiguous, fp32.  `stream` is a hipStream_t passed as void* (NULL = default stream).
 *  - The caller owns every buffer.  The library allocates no device memory: scratch space comes in
 *    through `workspace` (device, 256-byte aligned), sized by the matching *_workspace_bytes call.
 *    State the library keeps, per process: the immutable code-book tables (uploaded once per device on first
 *    use); a pool of idle HIP streams that lq_error_table leases for its interleaved sub-batches (created on demand, at
 *    most concurrent calls x (streams - 1) of them, returned to the pool when the call ends; lq_release_streams
 *    destroys the idle ones); and, while lq_profile_enable is on, the per-launch event records.
 *  - Return value: LQ_OK (0) or a negative lq_status.  Arguments are validated on the host before
 *    anything is launched, so a call that fails validation has no effect on any buffer.
 *    Device data is not inspected: non-finite weights, or non-positive Fisher weights, give
 *    unspecified numbers (never an out-of-bounds access).
 *  - lq_nf_quantize / lq_nf_dequantize / lq_matmul only enqueue work on `stream`.  lq_factorize, lq_decompose
 *    and lq_error_table write host outputs and therefore synchronize `stream` before returning.
 *  - Calls that share a workspace, or that overlap on outputs, must not run concurrently.
 */
#ifndef LQ_H_
#define LQ_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  LQ_OK = 0,
  LQ_ERR_NULL = -1,       /* a required pointer is NULL                                              */
  LQ_ERR_SHAPE = -2,      /* d, k, n <= 0; n not a multiple of the block size; sizes beyond int32 rows; a matrix of
                             2^30 weights or more in lq_factorize / lq_decompose / lq_error_table */
  LQ_ERR_CONFIG = -3,     /* bits / block sizes / scale bits / v dtype outside the supported set      */
  LQ_ERR_RANK = -4,       /* rank < 1, rank >= min(d,k) (Section 2.1 requires r < min(d,k)), rank > 128 */
  LQ_ERR_WEIGHT = -5,     /* exactly one of row_w / col_w is NULL                                     */
  LQ_ERR_WORKSPACE = -6,  /* workspace NULL, misaligned or smaller than *_workspace_bytes             */
  LQ_ERR_HIP = -7,        /* a HIP runtime call failed; lq_last_hip_error() gives its code            */
  LQ_ERR_ARG = -8         /* iters < 1, n_cfgs < 1, bad parameter block                               */
} lq_status;

/* v dtype codes (b2 of the configuration tuple). */
enum { LQ_V_FP32 = 0, LQ_V_BF16 = 1, LQ_V_FP16 = 2 };

/*
 * Quantization configuration c = (b0, b1, b2, B0, B1) of Section 3.2 (Table 1 lists the paper's
 * search grid; b0 = 8 is the "NF-8" variant of Section 4.2).
 *   bits        b0  NF code bits, one of 2, 3, 4, 8
 *   block       B0  weights per absmax block: a power of two in [16, 1024]
 *   scale_block B1  absmax values per second-level group: a power of two in [16, 256]
 *   scale_bits  b1  bits of the integer-quantized absmax values, 2..8; 0 selects 8
 *   v_dtype     b2  LQ_V_FP32 / LQ_V_BF16 / LQ_V_FP16 storage of the group scales v
 */
typedef struct {
  int32_t bits;
  int32_t block;
  int32_t scale_block;
  int32_t scale_bits;
  int32_t v_dtype;
} lq_config;

/*
 * Parameters of the randomized SVD that stands in for "SVD(A, r)" in Algorithm 4 (the paper uses a
 * randomized SVD, Section 3.1 footnote 1, and gives no parameters).  Pass NULL for the defaults.
 * A zero field selects its default.
 *   first_width   sketch width l1 of the cold start (first LQ iteration, Q = 0); multiple of 32,
 *                 rank < l1 <= 256.  Default: round_up32(max(2*rank, rank + 56)).
 *   first_tol     the cold start runs subspace iterations until the top-`rank` Ritz values change
 *                 by less than this relative amount (estimated from the observed geometric decay).  Default 2e-6.
 *   first_check   smallest number of subspace iterations between two Rayleigh-Ritz checks.  Default 8.
 *   first_max     cap on cold-start subspace iterations.  Default 600.
 *   warm_width    subspace width l of later LQ iterations, warm-started from the previous one;
 *                 multiple of 32, rank < l <= first_width.  Default round_up32(rank + max(rank/2, 24)).
 *   warm_power    subspace iterations per later LQ iteration (configurations not covered by warm_power_coarse or
 *                 warm_power_fine).  Default 2.
 *   warm_power_2  subspace iterations of the second LQ iteration (the one whose input differs most
 *                 from its warm start).  Default 3.
 *   warm_power_coarse  subspace iterations per later LQ iteration (the second included) for configurations whose scale
 *                 quantizer has a single level (b1 = 2: every block scale is 0 or v), whose residual W - Q changes far more
 *                 from one iteration to the next; used when larger than warm_power / warm_power_2.  lq_error_table
 *                 processes such configurations first, in batches of their own.  Default 4.
 *   warm_power_fine  subspace iterations per LQ iteration from the third on for configurations with codes of four or
 *                 more bits and block scales of eight or more (b0 >= 4, b1 >= 8), whose quantized component follows
 *                 W - L1 L2 closely enough that the residual hardly moves between iterations.  lq_error_table processes them last, in batches of their own where
 *                 the batch size allows; in a batch that mixes classes each configuration still does its own count.
 *                 Their second LQ iteration takes one more (at most warm_power_2).  Default 1.
 *   max_batch     lq_error_table advances up to this many configurations in lock step (more
 *                 workspace, better GPU occupancy).  Default 36.
 *   streams       lq_error_table splits a batch over this many HIP streams (1..4, all default priority, the
 *                 first is the caller's) and interleaves them so that latency-bound steps of one part overlap
 *                 throughput-bound kernels of another.  Default 3.
 *   gemm_mode     arithmetic of the large products against the d x k matrix: 1 = fp32 MFMA; 2 = both operands
 *                 split on the fly into bf16 hi + lo and multiplied by three bf16 MFMAs with fp32 accumulation
 *                 (products good to about 2^-16 relative, several times faster); 3 = as 2 for the first Factorize, and
 *                 the residual W - Q of the later ones is stored, scaled by a power of two, as an fp16 plane plus a
 *                 byte plane of what that rounding dropped (14 significant bits together): the products that steer the
 *                 subspace read the fp16 plane, the projection that the singular values and factors come from reads
 *                 both (warm_width <= 96, else as 2).
 *                 Default 3.
 *   init_quantized  lq_decompose only: 1 starts Algorithm 2 from Q(0) = Quantize(W) instead of Q(0) = 0 (the
 *                 variant of the footnote in Section 3.1: the first Factorize then sees W - Quantize(W)).
 *                 lq_error_table rejects it (LQ_ERR_ARG): its configurations share the first Factorize.
 */
typedef struct {
  int32_t first_width;
  float   first_tol;
  int32_t first_check;
  int32_t first_max;
  int32_t warm_width;
  int32_t warm_power;
  int32_t warm_power_2;
  int32_t max_batch;
  int32_t gemm_mode;
  int32_t streams;
  int32_t init_quantized;
  int32_t warm_power_coarse;
  int32_t warm_power_fine;
} lq_svd_params;

const char* lq_status_string(int status);
/* hipError_t of the most recent failing HIP call on this thread (0 if none). */
int lq_last_hip_error(void);
/* Destroys the idle streams of the pool that lq_error_table leases its extra streams from (all devices).  Streams that a
 * running call holds are not touched; later calls create what they need again.  LQ_ERR_HIP if a stream could not be
 * destroyed. */
int lq_release_streams(void);

/* NF-`bits` code book (Section 2.2): host_out[i] = value of code i, 2^bits ascending fp32 values
 * in [-1, 1] with host_out[2^(bits-1) - 1] == 0.  host pointer.  LQ_ERR_CONFIG for bits not in 2..8. */
int lq_nf_codebook(int bits, float* host_out);

/* Bytes of the packed code array for n weights: ceil(n * bits / 8).  Codes are packed as a
 * little-endian bit stream: code j occupies bits [j*bits, (j+1)*bits) (Appendix A: sub-8-bit codes
 * are packed into int8 containers). */
size_t lq_codes_bytes(int64_t n, int bits);
/* storage(A, c) of Eq. 3 in bits: n * (b0 + b1/B0 + bits(b2)/(B0*B1)).  Negative on a bad config. */
double lq_storage_bits(int64_t n, lq_config c);

/*
 * Quantize(x, c) of Section 3.2: Quantize-NF(x, b0, B0) -> codes and absmax s per block of B0
 * consecutive weights; Quantize-INT(s, b1, B1) -> integer scale indices and one scale v per group
 * of B1 consecutive blocks; cast(v, b2).
 *   x            n fp32 weights (row-major flattening of the matrix); n % B0 == 0, n > 0
 *   codes_packed lq_codes_bytes(n, b0) bytes
 *   scale_idx    n / B0 bytes, one index in [0, 2^(b1-1) - 1] per block
 *   v            ceil(n / (B0*B1)) fp32 values (already rounded to b2); the last group may be short
 * Arithmetic (fixed, so that results are reproducible bit for bit): the normalised weight is
 * fl32(u * fl32(1/s)); the code is the nearest code-book value, ties to the lower code; a block
 * with s == 0 gets the code of value 0; sigma = fl32(v/(2^(b1-1)-1)),
 * index = clamp(round_half_even(fl32(s/sigma)), 0, 2^(b1-1)-1).
 */
int lq_nf_quantize(const float* x, int64_t n, lq_config c, uint8_t* codes_packed, uint8_t* scale_idx,
                   float* v, void* stream);

/* The scale indices of a quantized matrix as the b1-bit integers that Eq. 3 counts (Section 3.2: the absmax
 * vector is quantized to b1 bits): `count` one-byte indices <-> a little-endian bit stream of scale_bits bits each,
 * lq_codes_bytes(count, scale_bits) bytes, index j in bits [j*scale_bits, (j+1)*scale_bits).  scale_bits 2..8
 * (LQ_ERR_CONFIG otherwise), count > 0 (LQ_ERR_SHAPE).  Both only enqueue work on `stream`. */
int lq_pack_scale_indices(const uint8_t* scale_idx, int64_t count, int scale_bits, uint8_t* packed, void* stream);
int lq_unpack_scale_indices(const uint8_t* packed, int64_t count, int scale_bits, uint8_t* scale_idx, void* stream);

/* Dequantize (Section 3.2, the reverse of the above): out[j] = fl32(codebook[code_j] *
 * fl32(scale_idx[block] * fl32(v[group] / (2^(b1-1)-1)))).  out: n fp32 values. */
int lq_nf_dequantize(const uint8_t* codes_packed, const uint8_t* scale_idx, const float* v, int64_t n,
                     lq_config c, float* out, void* stream);

/*
 * Factorize(A, F, r) of Algorithm 4 / Eq. 5 by randomized subspace iteration from a cold start.
 *   A      d x k
 *   row_w, col_w  Fisher-scale positive weights (d and k values) or both NULL.  The SVD is taken of
 *          diag(sqrt(row_w)) A diag(sqrt(col_w)) and the factors are un-scaled (Eq. 5).
 *   seed   seeds the Gaussian sketch; equal seeds give bit-identical results
 *   L1     d x rank  = D_row^-1 U sqrt(Sigma)        L2  rank x k = sqrt(Sigma) V^T D_col^-1
 *   sigma  host, rank doubles: the singular values found (descending); may be NULL
 */
size_t lq_factorize_workspace_bytes(int64_t d, int64_t k, int rank, const lq_svd_params* p);
int lq_factorize(const float* A, int64_t d, int64_t k, int rank, const float* row_w, const float* col_w,
                 uint64_t seed, const lq_svd_params* p, float* L1, float* L2, double* sigma,
                 void* workspace, size_t workspace_bytes, void* stream);

/*
 * LQ(W, F, c, r) of Algorithm 2 (Eq. 2): Q <- 0; repeat `iters` times
 *   L1, L2 <- Factorize(W - Q, F, r);  Q <- Quantize(W - L1 L2, c);
 *   eps_t = || sqrt(F) .* (W - Q - L1 L2) ||_F  with F_ij = row_w[i]*col_w[j] (Eq. 4), or F = 1.
 * With early_stop == 1 the loop ends after the first iteration whose eps exceeds the previous one and
 * returns that iterate, as Algorithm 2 prints it (this mode synchronizes once per iteration).  early_stop == 2 stops
 * by the same rule but returns the iterate before it, the one with the smallest eps seen (a variant, not the
 * paper's listing): L1, L2, the quantized component, sigma and err then belong to iteration iters_done - 1, or to
 * iteration iters when the error never went up.  Other values: LQ_ERR_ARG.
 *   W            d x k
 *   L1, L2       d x rank, rank x k (balanced factors of the last Factorize)
 *   q_codes, q_scale_idx, q_v   the quantized component, laid out as for lq_nf_quantize (n = d*k)
 *   Q_dense      d x k dequantized Q, or NULL
 *   err          host, 1 double: eps of the returned iterate          (may be NULL)
 *   err_trace    host, iters doubles: eps_1..; entries past iters_done are NaN   (may be NULL)
 *   iters_done   host, 1 int32: iterations run                         (may be NULL)
 *   sigma        host, rank doubles: singular values of the last Factorize (may be NULL)
 */
size_t lq_decompose_workspace_bytes(int64_t d, int64_t k, int rank, const lq_svd_params* p);
int lq_decompose(const float* W, int64_t d, int64_t k, int rank, lq_config c, int iters, int early_stop,
                 const float* row_w, const float* col_w, uint64_t seed, const lq_svd_params* p,
                 float* L1, float* L2, uint8_t* q_codes, uint8_t* q_scale_idx, float* q_v, float* Q_dense,
                 double* err, double* err_trace, int32_t* iters_done, double* sigma,
                 void* workspace, size_t workspace_bytes, void* stream);

/*
 * Inner loops of GetConfig (Algorithm 3) for one matrix: for every configuration c of `cfgs`,
 * err_sq[c] = eps^2 of LQ(W, F, c, rank) and storage_bits[c] = storage(W, c) (Eq. 3).
 * The first Factorize (Q = 0) does not depend on c and is computed once; the configurations then
 * advance in lock step, `max_batch` at a time.  early_stop as for lq_decompose: err_sq is that of the iterate
 * lq_decompose would return (the rule is applied to the finished traces, every configuration runs `iters` iterations).
 *   cfgs          host, n_cfgs entries           err_sq, storage_bits   host, n_cfgs doubles each
 *   err_trace     host, n_cfgs * iters doubles (row per configuration), or NULL
 */
size_t lq_error_table_workspace_bytes(int64_t d, int64_t k, int rank, int n_cfgs, const lq_svd_params* p);
int lq_error_table(const float* W, int64_t d, int64_t k, int rank, const lq_config* cfgs, int n_cfgs,
                   int iters, int early_stop, const float* row_w, const float* col_w, uint64_t seed,
                   const lq_svd_params* p, double* err_sq, double* storage_bits, double* err_trace,
                   void* workspace, size_t workspace_bytes, void* stream);

/*
 * ILPSolve of Algorithm 3 (the integer program of Section 3.2, "Dynamic quantization configurations"): one
 * configuration per matrix, minimising the summed error under a storage budget,
 *     min sum_i err[i][c_i]   s.t.   sum_i storage[i][c_i] <= budget_bits.
 * Host-only (all pointers are host pointers, no GPU is touched): the paper calls an external solver here.  The
 * problem is a multiple-choice knapsack; it is solved by branch and bound on its linear relaxation.
 *   err, storage   n_matrices x n_cfgs doubles, row per matrix (the err_sq / storage_bits rows of lq_error_table);
 *                  finite and non-negative
 *   node_limit     0 = search to proven optimality; otherwise stop after this many nodes with the best assignment found
 *   choice         n_matrices configuration indices            total_err, total_storage   sums of the chosen cells
 *   lower_bound    a proven lower bound on the optimum: equal to *total_err when the search completed
 * Any of total_err, total_storage, lower_bound may be NULL.  LQ_ERR_ARG when even the cheapest configuration of
 * every matrix exceeds the budget, or on non-finite / negative inputs.
 */
int lq_assign_configs(const double* err, const double* storage, int n_matrices, int n_cfgs, double budget_bits,
                      int64_t node_limit, int32_t* choice, double* total_err, double* total_storage,
                      double* lower_bound);

/*
 * RowAverage / ColAverage of Algorithm 4 (Section 3.3) from a full diagonal Fisher matrix F (d x k fp32, positive):
 * with a_i, b_j the row and column means of sqrt(F), row_w[i] = a_i^2 and col_w[j] = (b_j / mean(sqrt F))^2, so that
 * row_w[i] * col_w[j] reproduces F exactly when F has rank one.  Sums are taken in fp64 in a fixed order.  The two
 * vectors are what lq_factorize / lq_decompose / lq_error_table take as row_w, col_w.  Only enqueues work.
 *   row_w  d fp32    col_w  k fp32    workspace  lq_fisher_row_col_workspace_bytes(d, k) bytes
 */
size_t lq_fisher_row_col_workspace_bytes(int64_t d, int64_t k);
int lq_fisher_row_col(const float* F, int64_t d, int64_t k, float* row_w, float* col_w, void* workspace,
                      size_t workspace_bytes, void* stream);

/*
 * Forward product with a decomposed weight (Section 3.2 "Implementation" and Appendix A: products between fp32
 * inputs and quantized matrices with the matrix dequantized just in time):
 *     Y = X (Q + L1 L2)  computed as  X Q + (X L1) L2,
 * Q given in the quantized form that lq_decompose / lq_nf_quantize produce; its weights are decoded inside the
 * GEMM's load stage and never written to memory.
 *   X        m x d fp32, 16-byte aligned          Y        m x k fp32, 16-byte aligned (so is L2)
 *   codes_packed, scale_idx, v    Quantize(Q, c) of the d x k matrix Q (row-major flattening); k % B0 == 0
 *   L1, L2   d x rank and rank x k fp32, or rank == 0 (then both may be NULL): Y = X Q
 *   precision  0: every operand is split into bf16 hi + lo and each product takes three bf16 MFMAs with fp32
 *                 accumulation (error of an output about 2^-16 of sum |x||w|);  1: bf16 operands, one MFMA
 *                 (about 2^-8), for callers that train in bf16
 *              With m <= 8 and rank <= 512 the product is bound by reading the weights once; it then runs in plain
 *              fp32 on the vector ALU (exact products, fp32 accumulation) and `precision` is ignored.
 *   workspace  lq_matmul_workspace_bytes(m, d, k, rank) bytes: the bf16 hi / lo planes of X (rows padded to a
 *              multiple of 256), X L1 and its planes and, for small m, partial sums
 * d must be a multiple of 32 and ceil(m / 256) * 256 * d below 2^31 (LQ_ERR_SHAPE), rank <= 1024 (LQ_ERR_RANK).  Only enqueues work on `stream`; the
 * result is deterministic (partial sums are added in a fixed order).
 */
size_t lq_matmul_workspace_bytes(int64_t m, int64_t d, int64_t k, int rank);
int lq_matmul(const float* X, int64_t m, int64_t d, int64_t k, const uint8_t* codes_packed, const uint8_t* scale_idx,
              const float* v, lq_config c, const float* L1, const float* L2, int rank, int precision, float* Y,
              void* workspace, size_t workspace_bytes, void* stream);

/*
 * The few-row forward product for callers that cannot allocate or size a workspace (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): Y = X (Q + L1 L2) as lq_matmul computes it for m <= 8 rows and
 * rank <= 512 (plain fp32 on the vector ALU, deterministic), with the partial sums in a fixed array of
 * lq_matmul_few_rows_static_scratch_bytes() = 4 MiB of device memory that the library owns (one copy per GPU, held until
 * the process ends) instead of a caller's workspace.  The call allocates nothing and only enqueues kernels on `stream`.
 * Arguments as for lq_matmul.  A shape whose partial sums do not fit (the LLaMA-2-7B shapes fit at 8 rows, 8192 x 8192
 * at 4, 8192 x 28672 at 2) is refused with LQ_ERR_WORKSPACE before anything is launched; m > 8: LQ_ERR_SHAPE; rank > 512:
 * LQ_ERR_RANK.  Every call on a GPU uses that GPU's one array: calls that overlap in time on one GPU (different streams or
 * threads) race and must be serialized by the caller.  The array keeps the previous call's contents; the kernels write
 * every partial sum they later read, so nothing needs clearing.
 */
size_t lq_matmul_few_rows_static_scratch_bytes(void);
int lq_matmul_few_rows_static(const float* X, int64_t m, int64_t d, int64_t k, const uint8_t* codes_packed,
                              const uint8_t* scale_idx, const float* v, lq_config c, const float* L1, const float* L2,
                              int rank, float* Y, void* stream);

/*
 * Per-kernel timing for benchmarks (off by default).  While enabled, every kernel launch of the library
 * is bracketed by two HIP events on the launch stream; lq_profile_read synchronizes the device and returns,
 * for one kernel class, the summed event time, the number of launches and the summed algorithmic work
 * (flops for the GEMM classes, bytes otherwise: what the operation has to move, not what the kernel moved) since the last lq_profile_reset.  Class names are the
 * kernels' names.  Not thread-safe against concurrent library calls.
 */
int lq_profile_enable(int on);
int lq_profile_reset(void);
int lq_profile_num_classes(void);
const char* lq_profile_class_name(int cls);
int lq_profile_read(int cls, double* total_ms, int64_t* launches, double* work);

#ifdef __cplusplus
}
#endif
#endif /* LQ_H_ */
