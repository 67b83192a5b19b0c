// C ABI, part 2: Factorize (Algorithm 4), the LQ loop (Algorithm 2) and the error-table sweep
// (Algorithm 3).  Host orchestration only: validation, workspace carving, kernel sequencing.
//
// Data layout.  Every skinny matrix of the randomized SVD is kept "wide": l rows (the subspace
// dimension) by d or k columns, row-major, leading dimension padded to a multiple of 32 with zeros.
//   Y (l x d): orthonormal rows spanning the left subspace;   B = Y A (l x k): projected matrix.
// After the Rayleigh-Ritz rotation the rows are ordered by descending singular value, so the first
// `rank` rows give L1 L2 = Y_r^T B_r, and the first `warm_width` rows seed the next iteration.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <mutex>
#include <vector>

#include "kernels.h"
#include "nf_device.h"
#ifdef LQ_TESTING_HOOKS
#include "testing_capture.h"
#endif

namespace lq {

int check_quant_args(int64_t n, lq_config& c);

constexpr int MAX_ITERS = 1024;
constexpr int MAX_RANK = 128;
constexpr int MAX_DEVICES = 64;

static int64_t up32(int64_t x) { return (x + 31) / 32 * 32; }
static int64_t up64(int64_t x) { return (x + 63) / 64 * 64; }
static size_t up256(size_t x) { return (x + 255) / 256 * 256; }

struct Params {
  int l1, check, maxit, lw, qw, qw2, qw_coarse, qw_fine, max_batch, prec, streams, init_quantized;
  double tol;
};

static int resolve_params(int rank, const lq_svd_params* p, Params& out) {
  lq_svd_params z;
  std::memset(&z, 0, sizeof(z));
  if (p) z = *p;
  out.l1 = z.first_width ? z.first_width : (int)std::min<int64_t>(256, up32(std::max(2 * rank, rank + 56)));
  out.tol = z.first_tol > 0 ? z.first_tol : 2e-6;
  out.check = z.first_check ? z.first_check : 8;
  out.maxit = z.first_max ? z.first_max : 600;
  out.lw = z.warm_width ? z.warm_width : (int)std::min<int64_t>(out.l1, up32(rank + std::max(rank / 2, 24)));
  out.qw = z.warm_power ? z.warm_power : 2;
  out.qw2 = z.warm_power_2 ? z.warm_power_2 : 3;
  out.qw_coarse = z.warm_power_coarse ? z.warm_power_coarse : 4;
  out.qw_fine = z.warm_power_fine ? z.warm_power_fine : 1;
  out.max_batch = z.max_batch ? z.max_batch : 36;
  if (z.gemm_mode < 0 || z.gemm_mode > 3) return LQ_ERR_ARG;
  // 0: fp32 MFMA everywhere; 1: large products on bf16 hi/lo splits; 2: as 1, and the residual W - Q of the warm
  // iterations is kept in fp16 (products against it: fp16 hi/lo split of the skinny operand)
  out.prec = z.gemm_mode == 1 ? 0 : (z.gemm_mode == 2 ? 1 : 2);
  out.streams = z.streams ? z.streams : 3;
  if (out.streams < 1 || out.streams > 4) return LQ_ERR_ARG;
  if (z.init_quantized != 0 && z.init_quantized != 1) return LQ_ERR_ARG;
  out.init_quantized = z.init_quantized;
  if (out.l1 % 32 || out.l1 <= rank || out.l1 > 256) return LQ_ERR_ARG;
  if (out.lw % 32 || out.lw <= rank || out.lw > out.l1) return LQ_ERR_ARG;
  if (out.prec == 2 && !wide_gemm_f16_supported(out.lw)) out.prec = 1;
  if (out.check < 1 || out.maxit < 1 || out.qw < 1 || out.qw2 < 1 || out.qw_coarse < 1 || out.qw_fine < 1 || out.max_batch < 1) return LQ_ERR_ARG;
  return LQ_OK;
}

static int check_matrix_args(int64_t d, int64_t k, int rank) {
  if (d <= 0 || k <= 0 || d > (1 << 30) || k > (1 << 30)) return LQ_ERR_SHAPE;
  if (d * k >= (1ll << 30)) return LQ_ERR_SHAPE;     // the large products address the matrix with 32-bit byte offsets
  if (k % 16 != 0) return LQ_ERR_SHAPE;       // rows are whole 16-weight runs (every block size divides k)
  if (rank < 1 || rank > MAX_RANK || rank >= std::min(d, k)) return LQ_ERR_RANK;
  return LQ_OK;
}

// ---- workspace plan ---------------------------------------------------------------------------------
struct Plan {
  int64_t d, k, ldd, ldk, n;
  int rank, batch, lmax;
  Params prm;
  // shared
  size_t sr, sc, rsr, rsc;              // floats: d, k, d, k
  size_t Ya, Yb, Yc, Yd, Ba, Bb;        // cold-start wide bases (l1 rows)
  size_t gpart, gram_part, G, Vt, Ut, lam, lam_cold, prob, errs;
  // per problem (offset of problem 0, stride)
  size_t R, strideR;
  size_t Yw, Yw2, strideYw;             // floats
  size_t Bw, Bw2, strideBw;
  size_t codes, strideCodes, blk, strideBlk, sidx, strideSidx, v, strideV, epart, strideEpart;
  size_t packed, stridePacked;          // bf16 elements per problem (0: fp32 phase 1)
  size_t gpart_floats;
  size_t total;
};

static void make_plan(int64_t d, int64_t k, int rank, const Params& prm, int batch, Plan& pl) {
  pl.d = d; pl.k = k; pl.ldd = up64(d); pl.ldk = up64(k); pl.n = d * k;
  pl.rank = rank; pl.batch = batch; pl.prm = prm; pl.lmax = prm.l1;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += up256(bytes); return o; };
  const int l1 = prm.l1, lw = prm.lw;
  pl.sr = take(d * 4); pl.sc = take(k * 4); pl.rsr = take(d * 4); pl.rsc = take(k * 4);
  pl.Ya = take((size_t)l1 * pl.ldd * 4); pl.Yb = take((size_t)l1 * pl.ldd * 4);
  pl.Yc = take((size_t)l1 * pl.ldd * 4); pl.Yd = take((size_t)l1 * pl.ldd * 4);
  pl.Ba = take((size_t)l1 * pl.ldk * 4); pl.Bb = take((size_t)l1 * pl.ldk * 4);
  pl.gpart_floats = std::max(gemm_part_floats(l1, 0), gemm_part_floats(lw, 0));
  pl.gpart = take(pl.gpart_floats * 4);
  const size_t ll = (size_t)l1 * l1;
  pl.gram_part = take((size_t)batch * GRAM_CHUNKS * ll * 8);
  pl.G = take((size_t)batch * ll * 8);
  pl.Vt = take((size_t)batch * ll * 8);
  pl.Ut = take((size_t)batch * ll * 4);
  pl.lam = take((size_t)batch * l1 * 8);
  pl.lam_cold = take((size_t)l1 * 8);
  pl.prob = take((size_t)batch * sizeof(LoopProblem));
  pl.errs = take((size_t)batch * MAX_ITERS * 8);
  const size_t n = (size_t)pl.n;
  if (prm.prec == 2) {      // fp16 residuals; the area also has to hold one fp32 matrix (input of the first Factorize)
    pl.strideR = up256(n * 2) / 2;          pl.R = take(std::max(pl.strideR * 3 * batch, up256(n * 4)));   // fp16 planes, then byte planes
  } else {
    pl.strideR = up256(n * 4) / 4;          pl.R = take(pl.strideR * 4 * batch);
  }
  pl.strideYw = (size_t)lw * pl.ldd;        pl.Yw = take(pl.strideYw * 4 * batch); pl.Yw2 = take(pl.strideYw * 4 * batch);
  pl.strideBw = (size_t)lw * pl.ldk;        pl.Bw = take(pl.strideBw * 4 * batch); pl.Bw2 = take(pl.strideBw * 4 * batch);
  pl.strideCodes = up256(n);                pl.codes = take(pl.strideCodes * batch);
  pl.strideBlk = up256(n / 16 * sizeof(BlockRec)) / sizeof(BlockRec); pl.blk = take(pl.strideBlk * sizeof(BlockRec) * batch);
  pl.strideSidx = up256(n / 16);            pl.sidx = take(pl.strideSidx * batch);
  pl.strideV = up256(n / 256 * 4 + 4) / 4;  pl.v = take(pl.strideV * 4 * batch);
  pl.strideEpart = up256((size_t)err_partials_per_problem(pl.n, 16) * 8) / 8; pl.epart = take(pl.strideEpart * 8 * batch);
  pl.stridePacked = prm.prec ? up256(packed_factor_elems(d, k, rank) * 2) / 2 : 0;
  pl.packed = take(pl.stridePacked * 2 * batch);
  pl.total = off;
}

// ---- execution context --------------------------------------------------------------------------------
struct Ctx {
  Plan pl;
  char* ws;
  hipStream_t st;
  const float* W;
  const float* row_w;
  const float* col_w;
  bool weighted;
  const DevTables* tables;
  // set once per call and shared by the per-stream contexts of a sweep
  const float* sr; const float* sc; const float* rsr; const float* rsc;   // sqrt / 1/sqrt of the Fisher weights
  const double* lam_cold;                                                   // Ritz values of the cold start
  float a_scale;            // power of two the fp16 residual is multiplied by (residual_scale)
  template <typename T> T* at(size_t off) const { return reinterpret_cast<T*>(ws + off); }
};

// Cholesky-QR: the rows of X (l x m) are replaced by an orthonormal basis of their span.  With the factor in
// LDS the result is written to Xalt by the MFMA GEMM (C^-1 X) and the two pointers are exchanged; otherwise
// X is solved in place.
static int orthonormalize(const Ctx& c, float*& X, float*& Xalt, int l, int64_t m, int64_t ldx, size_t strideX,
                          int batch) {
  double* G = c.at<double>(c.pl.G);
  LQ_TRY(launch_gram(X, l, m, ldx, strideX, c.at<double>(c.pl.gram_part), G, batch, c.st));
  if (cholinv_supported(l)) {
    float* Cinv = c.at<float>(c.pl.Ut);
    LQ_TRY(launch_cholinv(G, l, Cinv, batch, c.st));
    LQ_TRY(launch_wide_gemm(MODE_NN, l, ldx, l, Cinv, l, (size_t)l * l, X, ldx, strideX, Xalt, ldx, strideX, batch,
                            nullptr, 0, c.st));
    std::swap(X, Xalt);
    return LQ_OK;
  }
  LQ_TRY(launch_cholesky(G, l, batch, c.st));
  return launch_trsm(G, l, X, m, ldx, strideX, batch, c.st);
}

static int gemm(const Ctx& c, int mode, int l, int64_t big, int64_t K, const float* X, int64_t ldx, size_t sX,
                const float* A, int64_t lda, size_t sA, float* C, int64_t ldc, size_t sC, int batch) {
  return launch_wide_gemm(mode, l, big, K, X, ldx, sX, A, lda, sA, C, ldc, sC, batch, c.at<float>(c.pl.gpart),
                          c.pl.gpart_floats, c.st, c.pl.prm.prec ? 1 : 0);
}

// Rayleigh-Ritz on the subspace spanned by the rows of Y (orthonormal) with B = Y A:
// eigen-decomposition of B B^T, then both bases are rotated into Ritz order.  Y2 / B2 receive the result.
static int ritz_rotate(const Ctx& c, int l, const float* Y, float* Y2, size_t sY, const float* B, float* B2, size_t sB,
                       double* lambda, int batch) {
  const Plan& pl = c.pl;
  double* G = c.at<double>(pl.G);
  float* Ut = c.at<float>(pl.Ut);
  LQ_TRY(launch_gram(B, l, pl.k, pl.ldk, sB, c.at<double>(pl.gram_part), G, batch, c.st));
  const bool fast = jacobi_fast_supported(l);
  if (fast) LQ_TRY(launch_jacobi_fast(G, l, Ut, lambda, batch, c.st));
  else LQ_TRY(launch_jacobi_eig(G, l, c.at<double>(pl.Vt), Ut, lambda, batch, c.st));
  LQ_TRY(launch_wide_gemm(MODE_NN, l, pl.ldd, l, Ut, l, (size_t)l * l, Y, pl.ldd, sY, Y2, pl.ldd, sY, batch, nullptr, 0,
                          c.st));
  LQ_TRY(launch_wide_gemm(MODE_NN, l, pl.ldk, l, Ut, l, (size_t)l * l, B, pl.ldk, sB, B2, pl.ldk, sB, batch, nullptr, 0,
                          c.st));
  // Ritz values from the rotated projection itself: sigma_i^2 = |row i of B2|^2
  if (fast) LQ_TRY(launch_row_sumsq(B2, l, pl.k, pl.ldk, sB, lambda, batch, c.st));
  return LQ_OK;
}

// Cold-start randomized SVD of A (d x k): on return *Yout / *Bout (l1 rows, Ritz order) and lam_cold.
//
// Chebyshev-filtered subspace iteration on M = A A^T.  With theta_1 >= .. >= theta_l the Ritz values of the block, the
// part of the spectrum below b = theta_l is what the block must lose; T_m mapped to [0, b] stays within +-1 there and
// grows like cosh(m acosh(2 lambda / b - 1)) above, so on the flat spectra of weight matrices m filter steps separate
// the wanted directions like ~m^2 / 2 power iterations would.  Any cut-off is stable (the interval starts at 0, below
// the whole spectrum); a poor b only costs speed.  A cycle is m steps of the three-term recurrence
//   Y_1 = (2/b) Y_0 M - Y_0,   Y_{j+1} = (4/b) Y_j M - 2 Y_j - Y_{j-1}
// from an orthonormal Y_0, then one Cholesky-QR.  The rows are independent under the recurrence, and after a
// Rayleigh-Ritz the rows that matter for convergence (around theta_rank) are orthogonal to the dominant directions up
// to rounding, ~1e-6; the recurrence amplifies that leak by T_m(2 theta_1 / b - 1) / T_m(2 theta_rank / b - 1), and m is
// limited so that this stays below `growth` = 1e5 (the leak stays a small part of the row).
// Dominant directions that would hold the degree down are locked once converged (a direction theta_i has converged to
// (b / theta_i)^it after `it` applications of M; 1e-5 is asked for): their rows stay as the last Rayleigh-Ritz left them
// and every filter step ends by removing their components from the other rows (deflate_rows_kernel), so the recurrence
// runs on the deflated operator and theta_1 above is the largest unlocked Ritz value.  Spectra with a dominant part
// that is neither locked yet nor small get m = 1, which is subspace iteration on M - (b/2) I.  Before the first
// Rayleigh-Ritz there is no b: plain power steps.
// Convergence is judged on the top-`rank` Ritz values.  Each Rayleigh-Ritz costs an l x l eigen-solve, so they are
// scheduled: after 2 applications (to get b), when lock candidates will have converged, and then where the error is
// predicted to reach the tolerance, by the decay rate measured over two equal gaps if there is one, else by the
// filter's own rate for theta_rank (derated by 0.7).  The iteration only stops on measured quantities: the change over
// the last gap, divided by the measured decay over that gap where available.
static int cold_factorize(const Ctx& c, const float* A, uint64_t seed, const float** Yout, const float** Bout) {
  const Plan& pl = c.pl;
  const int l = pl.prm.l1, r = pl.rank;
  float* const all[4] = {c.at<float>(pl.Ya), c.at<float>(pl.Yb), c.at<float>(pl.Yc), c.at<float>(pl.Yd)};
  float* Y0 = all[0];                                         // orthonormal rows: start of the cycle
  float* P[3] = {all[1], all[2], all[3]};                     // the other three of the four row blocks
  float* Ba = c.at<float>(pl.Ba); float* Bb = c.at<float>(pl.Bb);
  double* lam = c.at<double>(pl.lam_cold);
  const int64_t ycount = (int64_t)l * pl.ldd;
  for (float* p : all) LQ_HIP_TRY(hipMemsetAsync(p, 0, ycount * 4, c.st));
  LQ_HIP_TRY(hipMemsetAsync(Bb, 0, (size_t)l * pl.ldk * 4, c.st));
  LQ_TRY(launch_gaussian_fill(Ba, l, pl.k, pl.ldk, seed, c.st));
  LQ_TRY(gemm(c, MODE_NT, l, pl.d, pl.k, Ba, pl.ldk, 0, A, pl.k, 0, Y0, pl.ldd, 0, 1));
  LQ_TRY(orthonormalize(c, Y0, P[0], l, pl.d, pl.ldd, 0, 1));
  std::vector<double> prev(r, 0.0), cur(l, 0.0);
  bool have_prev = false;
  double bcut = 0.0;          // filter cut-off: theta_l of a Rayleigh-Ritz (0: none yet)
  double free_top = 0.0;      // largest unlocked Ritz value
  double wanted = 0.0;        // theta_rank
  int locked = 0;             // leading rows of Y0 that the filter leaves alone
  double kappa = 0.0;         // measured decay rate of the error per application of M (natural log), 0 = unknown
  const int first_gap = std::min(2, pl.prm.check);
  int next_check = first_gap, last_check = 0, m_prev = 1;
  bool rate_ok = false;       // last_est was measured with the current filter
  const double rounding = 1.0e-6, crowding = 10.0, lock_accuracy = 1.0e-5;
  const int m_max = 8;
  auto cheb = [](int deg, double x) { return std::cosh(deg * std::acosh(std::max(x, 1.0))); };
  // Degree of the next cycle by the leak rule (before the caps that depend on the schedule).  A direction theta_i above
  // theta_rank is present in the other rows at a level of about (b / theta_i)^it (its convergence so far), at least
  // 1e-6 (rounding); a cycle multiplies that by T_m(x_i) / T_m(x_rank), and the product, the factor by which such a
  // direction can come to outweigh a row's own content, has to stay below `crowding`: the Cholesky-QR that follows and
  // the fp32 rows themselves lose that many digits of the rest.
  auto filter_degree = [&](int it_now) {
    if (!(bcut > 0.0)) return 1;
    const double xr = 2.0 * wanted / bcut - 1.0;
    int m = 1;
    while (m < m_max) {
      // the largest unlocked direction grows by T_m(x) in a cycle: the rows of a block stay within 1e8 of each other
      bool ok = cheb(m + 1, 2.0 * cur[locked] / bcut - 1.0) <= 1.0e8;
      for (int i = locked; i < r - 1 && ok; ++i) {
        const double ratio = cur[i] / bcut;
        if (!(ratio > 1.0)) break;
        const double leak = std::max(rounding, std::exp(-it_now * std::log(ratio)));
        ok = leak * cheb(m + 1, 2.0 * ratio - 1.0) <= crowding * cheb(m + 1, xr);
      }
      if (!ok) break;
      ++m;
    }
    return m;
  };
  double* res_dev = c.at<double>(pl.lam);     // squared residual norms of the top-r Ritz pairs (free until the warm passes)
  std::vector<double> res(r, 0.0);
  double last_est = 0.0;      // residual-based error estimate of the previous Rayleigh-Ritz (valid when rate_ok)
  for (int it = 0;;) {        // it: applications of M so far
    LQ_TRY(gemm(c, MODE_NN, l, pl.k, pl.d, Y0, pl.ldd, 0, A, pl.k, 0, Ba, pl.ldk, 0, 1));
    bool have_g = false;      // P[0] = Ba A^T = Y0 M already computed (by the residual check)
    if (it >= next_check || it >= pl.prm.maxit) {
      LQ_TRY(ritz_rotate(c, l, Y0, P[0], 0, Ba, Bb, 0, lam, 1));
      std::swap(Y0, P[0]); std::swap(Ba, Bb);
      // residuals of the top-r Ritz pairs, |y_j M - theta_j y_j|: y_j M = (y_j A) A^T is the first product of the next
      // cycle anyway
      LQ_TRY(gemm(c, MODE_NT, l, pl.d, pl.k, Ba, pl.ldk, 0, A, pl.k, 0, P[0], pl.ldd, 0, 1));
      LQ_TRY(launch_ritz_residual(P[0], Y0, lam, r, pl.d, pl.ldd, res_dev, c.st));
      have_g = true;
      LQ_HIP_TRY(hipMemcpyAsync(cur.data(), lam, sizeof(double) * l, hipMemcpyDeviceToHost, c.st));
      LQ_HIP_TRY(hipMemcpyAsync(res.data(), res_dev, sizeof(double) * r, hipMemcpyDeviceToHost, c.st));
      LQ_HIP_TRY(hipStreamSynchronize(c.st));
      double delta = 0.0;
      for (int j = 0; j < r; ++j) {
        const double a = std::sqrt(cur[j]), b = std::sqrt(prev[j]);
        const double rel = a > 0 ? std::fabs(a - b) / a : 0.0;
        if (!(rel <= delta)) delta = rel;      // NaN-safe maximum
      }
      const int gap = it - last_check;
      const bool usable = cur[0] > 0 && cur[l - 1] > 1e-12 * cur[0] && std::isfinite(cur[0]);
      // Error of sigma_j = sqrt(theta_j) from the residual rho_j of its Ritz pair: theta_j misses the eigenvalue by at
      // most rho_j^2 / gap_j, gap_j = distance from theta_j to the spectrum outside the block.  That spectrum ends near
      // theta_l; half of theta_j - theta_l is used for the gap (theta_l is itself an underestimate), so
      // d sigma / sigma = d theta / (2 theta) <= rho_j^2 / (theta_j (theta_j - theta_l)).
      double est = INFINITY;
      if (usable) {
        est = 0.0;
        for (int j = 0; j < r; ++j) {
          const double gapj = cur[j] - cur[l - 1];
          const double e = gapj > 1e-9 * cur[j] ? res[j] / (cur[j] * gapj) : INFINITY;
          if (!(e <= est)) est = e;
        }
      }
      // measured decay rate per application of M between two Rayleigh-Ritz steps under the same filter, derated by 0.7
      if (rate_ok && last_est > 0 && est > 0 && est < last_est && std::isfinite(last_est) && gap > 0)
        kappa = 0.7 * std::log(last_est / est) / gap;
      // the change over the last gap, as a second witness: err(it) ~ exp(-kappa it), so the change is err(it) (exp(kappa gap) - 1)
      double change_est = delta;
      if (kappa > 0) change_est = std::min(delta, delta / std::expm1(kappa * gap));
      const bool done = est <= pl.prm.tol || (have_prev && change_est <= pl.prm.tol);
      if (done || it >= pl.prm.maxit) break;
      rate_ok = usable;
      // the cut-off follows theta_l upwards; a noticeable change of the filter invalidates the measured rate
      if (usable && cur[l - 1] > bcut) {
        if (cur[l - 1] > 1.03 * bcut) { rate_ok = false; kappa = 0.0; }
        bcut = cur[l - 1];
      }
      int lock_at = 0;        // application count at which the next lock candidate will have converged (0: none waiting)
      if (usable) {
        wanted = cur[r - 1];
        const double xr = 2.0 * wanted / bcut - 1.0;
        int n = 0;
        while (n < std::min(DEFLATE_ROWS_MAX, l - 1)) {
          const double th = cur[n];
          if (!(rounding * cheb(m_max, 2.0 * th / bcut - 1.0) > crowding * cheb(m_max, xr))) break;   // would not hold the degree down
          const double per_step = std::log(th / bcut);
          if (it * per_step < std::log(1.0 / lock_accuracy)) {
            lock_at = (int)std::ceil(std::log(1.0 / lock_accuracy) / per_step);
            break;
          }
          ++n;
        }
        if (n != locked) { rate_ok = false; kappa = 0.0; }
        locked = n;
        free_top = cur[locked];
      }
      // next Rayleigh-Ritz where the error is predicted to reach the tolerance: by the measured rate, else by the
      // filter's own rate for theta_rank, derated by 0.5 (theta_l below the true edge of the unwanted spectrum and the
      // shorter first cycles both make the real decay slower)
      double rate = kappa;
      if (!(rate > 0) && bcut > 0.0 && lock_at == 0) {
        const int m = filter_degree(it);
        rate = 0.5 * 2.0 * std::log(cheb(m, 2.0 * wanted / bcut - 1.0)) / m;   // values converge like squared angles
      }
      int next_gap = pl.prm.check;
      if (rate > 0 && std::isfinite(est) && est > 0) {
        const double need = std::log(est / pl.prm.tol) / rate;
        next_gap = (int)std::min<double>(std::max<double>(std::ceil(need), (pl.prm.check + 1) / 2), 8.0 * pl.prm.check);
      }
      last_est = est; last_check = it; next_check = it + next_gap;
      if (lock_at > it) next_check = std::min(next_check, lock_at);
      for (int j = 0; j < r; ++j) prev[j] = cur[j];
      have_prev = true;
    }
    // one cycle: m filter steps from Y0, then Cholesky-QR
    int m = std::min(filter_degree(it), 4 * m_prev);
    m = std::max(1, std::min(m, std::min(next_check, pl.prm.maxit) - it));
    m_prev = m;
    // step 1 (Ba = Y0 A is at hand)
    if (!have_g) LQ_TRY(gemm(c, MODE_NT, l, pl.d, pl.k, Ba, pl.ldk, 0, A, pl.k, 0, P[0], pl.ldd, 0, 1));
    if (bcut > 0.0) LQ_TRY(launch_lincomb3(P[0], (float)(2.0 / bcut), Y0, -1.0f, nullptr, 0.0f, ycount, c.st));
    LQ_TRY(launch_deflate_rows(P[0], Y0, l, locked, pl.d, pl.ldd, c.st));
    // Y0 keeps the locked rows for the whole cycle: the recurrence rotates through the other three blocks
    float* Yj = P[0]; float* Yjm1 = Y0; float* Ynew = P[1]; float* third = P[2];
    for (int j = 1; j < m; ++j) {
      LQ_TRY(gemm(c, MODE_NN, l, pl.k, pl.d, Yj, pl.ldd, 0, A, pl.k, 0, Bb, pl.ldk, 0, 1));
      LQ_TRY(gemm(c, MODE_NT, l, pl.d, pl.k, Bb, pl.ldk, 0, A, pl.k, 0, Ynew, pl.ldd, 0, 1));
      LQ_TRY(launch_lincomb3(Ynew, (float)(4.0 / bcut), Yj, -2.0f, Yjm1, -1.0f, ycount, c.st));
      LQ_TRY(launch_deflate_rows(Ynew, Y0, l, locked, pl.d, pl.ldd, c.st));
      float* freed = Yjm1 == Y0 ? third : Yjm1;
      Yjm1 = Yj; Yj = Ynew; Ynew = freed;
    }
    float* alt = Y0;                                                 // its locked rows are in Yj by now
    LQ_TRY(orthonormalize(c, Yj, alt, l, pl.d, pl.ldd, 0, 1));       // Yj now names the orthonormal block
    Y0 = Yj;
    for (int q = 0, n = 0; q < 4; ++q)
      if (all[q] != Y0) P[n++] = all[q];
    it += m;
  }
  *Yout = Y0; *Bout = Ba;
  return LQ_OK;
}

// One warm-started Factorize for every problem of the batch: power[b] subspace iterations on R_b starting from the
// rows of Bsrc, then Rayleigh-Ritz.  Results land in Yw / Bw (swapped with Yw2 / Bw2).
// power[] does not increase with b: the iterations are counted down, step j runs for the problems that have at least j
// left (a prefix of the batch), so every problem's last iteration is the batch's last, which is the one that reads both
// planes of the residual.  A problem enters at its first step with X = its rows of Bsrc and continues with X = the
// projection B of the step before.
struct WideSet { float* Yw; float* Yw2; float* Bw; float* Bw2; };

static int batch_planes(const Ctx& c) { return c.pl.batch; }      // problems per plane set of the fp16 residual area

static int warm_factorize(const Ctx& c, WideSet& w, const float* Bsrc, size_t sBsrc, const double* lamsrc, size_t sLam,
                          const int* power, int batch) {
  const Plan& pl = c.pl;
  const int l = pl.prm.lw;
  const float* R = c.at<float>(pl.R);
  const uint16_t* R16 = c.at<uint16_t>(pl.R);
  const uint8_t* R16lo = reinterpret_cast<const uint8_t*>(R16 + pl.strideR * (size_t)batch_planes(c));   // one byte per element
  const bool half = pl.prm.prec == 2;
  float* part = c.at<float>(pl.gpart);
  // fp16 residual: the rows of X = B (norms at most sigma_1, taken from the Ritz values the rows of Bsrc came with;
  // the products Y A of the later iterations have rows no longer than sigma_1 of the new residual, which the headroom
  // of the scale covers) are scaled per problem; an orthonormal X by 2^13.  Both products come back in true scale.
  const float ys = 8192.0f;
  // problems first .. first + n - 1: Yw = X A^T with X = their rows of Xb (stride sX)
  auto project_back = [&](const float* Xb, size_t sX, int first, int n) -> int {
    if (n <= 0) return LQ_OK;
    float* Y = w.Yw + pl.strideYw * (size_t)first;
    if (half)
      return launch_wide_gemm_f16(MODE_NT, l, pl.d, pl.k, Xb, pl.ldk, sX, R16 + pl.strideR * (size_t)first, nullptr, pl.k,
                                  pl.strideR, Y, pl.ldd, pl.strideYw, n, part, pl.gpart_floats, 1.0f,
                                  lamsrc + sLam * (size_t)first, sLam, 1.0f / c.a_scale, c.st);
    return gemm(c, MODE_NT, l, pl.d, pl.k, Xb, pl.ldk, sX, R + pl.strideR * (size_t)first, pl.k, pl.strideR, Y, pl.ldd,
                pl.strideYw, n);
  };
  auto active = [&](int j) { int n = 0; while (n < batch && power[n] >= j) ++n; return n; };
  for (int j = power[0]; j >= 1; --j) {
    const int n = active(j), carried = j < power[0] ? active(j + 1) : 0;
    LQ_TRY(project_back(w.Bw, pl.strideBw, 0, carried));
    LQ_TRY(project_back(Bsrc + sBsrc * (size_t)carried, sBsrc, carried, n - carried));
    LQ_TRY(orthonormalize(c, w.Yw, w.Yw2, l, pl.d, pl.ldd, pl.strideYw, n));
    if (half)
      // the last product is the projection B = Y A that the Ritz values and the factors are read from: it takes both
      // planes of the residual (a rounding of A to fp16 would show in sigma to first order wherever a few entries carry a
      // singular vector); the products before it only steer the subspace and take the hi plane
      LQ_TRY(launch_wide_gemm_f16(MODE_NN, l, pl.k, pl.d, w.Yw, pl.ldd, pl.strideYw, R16, j == 1 ? R16lo : nullptr,
                                  pl.k, pl.strideR, w.Bw, pl.ldk, pl.strideBw, n, part, pl.gpart_floats, ys, nullptr, 0,
                                  1.0f / (ys * c.a_scale), c.st));
    else
      LQ_TRY(gemm(c, MODE_NN, l, pl.k, pl.d, w.Yw, pl.ldd, pl.strideYw, R, pl.k, pl.strideR, w.Bw, pl.ldk, pl.strideBw, n));
  }
  LQ_TRY(ritz_rotate(c, l, w.Yw, w.Yw2, pl.strideYw, w.Bw, w.Bw2, pl.strideBw, c.at<double>(pl.lam), batch));
  std::swap(w.Yw, w.Yw2); std::swap(w.Bw, w.Bw2);
  return LQ_OK;
}

static int setup_common(Ctx& c, const float* W, const float* row_w, const float* col_w, void* workspace,
                        hipStream_t st) {
  c.ws = (char*)workspace; c.st = st; c.W = W; c.row_w = row_w; c.col_w = col_w; c.weighted = row_w != nullptr;
  LQ_TRY(device_tables(&c.tables));
  const Plan& pl = c.pl;
  c.sr = c.sc = c.rsr = c.rsc = nullptr;
  c.a_scale = 1.0f;
  c.lam_cold = c.at<double>(pl.lam_cold);
  if (c.weighted) {
    c.sr = c.at<float>(pl.sr); c.sc = c.at<float>(pl.sc); c.rsr = c.at<float>(pl.rsr); c.rsc = c.at<float>(pl.rsc);
    LQ_TRY(launch_sqrt_vecs(row_w, pl.d, c.at<float>(pl.sr), c.at<float>(pl.rsr), st));
    LQ_TRY(launch_sqrt_vecs(col_w, pl.k, c.at<float>(pl.sc), c.at<float>(pl.rsc), st));
  }
  return LQ_OK;
}

// Power of two that puts the entries of D_row (W - Q) D_col in the middle of the fp16 range: the largest |w| times the
// largest square roots of the weights lands in [2^9, 2^10), which leaves a factor of 64 for |W - Q| to exceed |W| by
// (beyond that the residual kernel saturates) and keeps everything above 2^-24 of the largest entry a normal number.
// Synchronizes the stream.
static int residual_scale(Ctx& c) {
  const Plan& pl = c.pl;
  if (pl.prm.prec != 2) return LQ_OK;
  float* scratch = c.at<float>(pl.gram_part);
  LQ_TRY(launch_absmax(c.W, pl.n, scratch, c.st));
  if (c.weighted) {
    LQ_TRY(launch_absmax(c.sr, pl.d, scratch + 1056, c.st));
    LQ_TRY(launch_absmax(c.sc, pl.k, scratch + 2112, c.st));
  }
  float m[3] = {0.f, 1.f, 1.f};
  LQ_HIP_TRY(hipMemcpyAsync(&m[0], scratch + 1024, sizeof(float), hipMemcpyDeviceToHost, c.st));
  if (c.weighted) {
    LQ_HIP_TRY(hipMemcpyAsync(&m[1], scratch + 1056 + 1024, sizeof(float), hipMemcpyDeviceToHost, c.st));
    LQ_HIP_TRY(hipMemcpyAsync(&m[2], scratch + 2112 + 1024, sizeof(float), hipMemcpyDeviceToHost, c.st));
  }
  LQ_HIP_TRY(hipStreamSynchronize(c.st));
  const double top = (double)m[0] * m[1] * m[2];
  c.a_scale = (top > 0.0 && std::isfinite(top)) ? (float)std::ldexp(1.0, 9 - std::ilogb(top)) : 1.0f;
  if (!(c.a_scale > 0.0f) || !std::isfinite(c.a_scale)) c.a_scale = 1.0f;
  return LQ_OK;
}

// Input of the first Factorize: W itself, or D_row W D_col staged in problem 0's residual buffer.
static int first_input(const Ctx& c, const float** A) {
  const Plan& pl = c.pl;
  if (!c.weighted) { *A = c.W; return LQ_OK; }
  float* As = c.at<float>(pl.R);
  LQ_TRY(launch_scale_matrix(c.W, pl.d, pl.k, c.sr, c.sc, As, c.st));
  *A = As;
  return LQ_OK;
}

static bool is_coarse(const lq_config& c) { return c.scale_bits != 0 && c.scale_bits <= 2; }
// Codes of four or more bits on block scales of eight or more: Q follows W - L1 L2 closely, so W - Q changes little
// from one pass to the next and the warm-started subspace is nearly invariant already.  (With 3-bit scales a 4-bit
// configuration's error after a single subspace iteration was measured 1.3e-3 off.)
static bool is_fine(const lq_config& c) { return c.bits >= 4 && (c.scale_bits == 0 || c.scale_bits >= 8); }
// Order in which lq_error_table processes configurations: those that need the most subspace iterations first.
static int power_class(const lq_config& c) { return is_coarse(c) ? 0 : (is_fine(c) ? 2 : 1); }

struct LoopOut {          // batch == 1 only: user buffers that receive the quantized component directly
  uint8_t* codes; uint8_t* sidx; float* v; float* Qd;
  float* L1; float* L2; double* sigma;      // only used when the best iterate is kept (early_stop == 2)
};

static int emit_factors(const Ctx& c, const float* Y, const float* B, const double* lam, float* L1, float* L2,
                        double* sigma_host);

// Algorithm 2 for `batch` configurations in lock step from the shared first factorization (Y1, B1, lam_cold),
// as a sequence of asynchronous steps on the context's stream so that several such loops (one per stream) can
// be interleaved by the host: begin(), step(t) for t = 1.., finish().
struct Loop {
  Ctx* c = nullptr;
  const lq_config* cfgs = nullptr;
  int batch = 0, iters = 0, early_stop = 0;
  bool want_trace = false;
  const float* Y1 = nullptr; const float* B1 = nullptr;
  const LoopOut* direct = nullptr;
  const int* cfg_ids = nullptr;             // position of each configuration in the caller's list (NULL: 0, 1, ..)
  std::vector<int> qw, qw2;                 // subspace iterations per Factorize and problem (second pass: qw2), set by begin()
  // state
  std::vector<LoopProblem> probs;
  std::vector<double> host_err;
  std::vector<uint8_t> bits_host;
  int min_block = 1 << 30, done = 0;
  PhaseArgs a;
  WideSet w;
  const float* Ycur = nullptr; const float* Bcur = nullptr;
  size_t sY = 0, sB = 0;
  const double* lamcur = nullptr; size_t sLam = 0;   // Ritz values the rows of Bcur came with (stride per problem)
  double* errs = nullptr;
  double prev_eps = INFINITY;
  bool stopped = false;
  // early_stop == 2 (batch == 1): the iterate before the error went up is the one returned.  Its quantized component is
  // kept by writing the iterations alternately into the caller's buffers and into the workspace's, its factors by
  // assembling L1, L2 after every iteration that did not make the error worse.
  bool keep_best() const { return early_stop == 2 && direct != nullptr; }
  int returned = 0;                         // iteration whose pieces the outputs hold
  void point_codes(int t) {
    const Plan& pl = c->pl;
    if (!keep_best() || (t & 1)) { a.codes = direct->codes; a.sidx = direct->sidx; a.v = direct->v; }
    else { a.codes = c->at<uint8_t>(pl.codes); a.sidx = c->at<uint8_t>(pl.sidx); a.v = c->at<float>(pl.v); }
  }

  int begin() {
    const Plan& pl = c->pl;
    probs.assign(batch, LoopProblem());
    for (int b = 0; b < batch; ++b) {
      std::memset(&probs[b], 0, sizeof(LoopProblem));
      probs[b].cfg = cfgs[b];
      probs[b].levels = scale_levels(cfgs[b]);
      min_block = std::min(min_block, (int)cfgs[b].block);
    }
    // A scale quantizer with a single level (b1 = 2: every block scale is 0 or v) leaves a residual W - Q that moves a lot
    // from pass to pass, and the warm-started subspace needs more iterations to follow it.
    // Codes of at least four bits need fewer (one) from the third pass on.  warm_factorize wants counts that do not
    // increase along the batch (lq_error_table orders the configurations that way): otherwise all take the largest.
    qw.assign(batch, 0); qw2.assign(batch, 0);
    for (int b = 0; b < batch; ++b) {
      const bool coarse = is_coarse(cfgs[b]);
      qw[b] = coarse ? std::max(pl.prm.qw, pl.prm.qw_coarse) : (is_fine(cfgs[b]) ? pl.prm.qw_fine : pl.prm.qw);
      qw2[b] = coarse ? std::max(pl.prm.qw2, pl.prm.qw_coarse) : (is_fine(cfgs[b]) ? std::min(pl.prm.qw2, pl.prm.qw_fine + 1) : pl.prm.qw2);
    }
    for (std::vector<int>* q : {&qw, &qw2})
      if (!std::is_sorted(q->rbegin(), q->rend())) q->assign(batch, *std::max_element(q->begin(), q->end()));
    LoopProblem* dprob = c->at<LoopProblem>(pl.prob);
    LQ_HIP_TRY(hipMemcpyAsync(dprob, probs.data(), sizeof(LoopProblem) * batch, hipMemcpyHostToDevice, c->st));
    w = WideSet{c->at<float>(pl.Yw), c->at<float>(pl.Yw2), c->at<float>(pl.Bw), c->at<float>(pl.Bw2)};
    LQ_HIP_TRY(hipMemsetAsync(w.Yw, 0, pl.strideYw * 4 * batch, c->st));
    LQ_HIP_TRY(hipMemsetAsync(w.Yw2, 0, pl.strideYw * 4 * batch, c->st));
    LQ_HIP_TRY(hipMemsetAsync(w.Bw, 0, pl.strideBw * 4 * batch, c->st));
    LQ_HIP_TRY(hipMemsetAsync(w.Bw2, 0, pl.strideBw * 4 * batch, c->st));
    std::memset(&a, 0, sizeof(a));
    a.W = c->W; a.d = pl.d; a.k = pl.k; a.rank = pl.rank; a.ldy = pl.ldd; a.ldb = pl.ldk;
    if (c->weighted) {
      a.rsr = c->rsr; a.rsc = c->rsc; a.sr = c->sr; a.sc = c->sc;
      a.row_w = c->row_w; a.col_w = c->col_w;
    }
    a.prob = dprob; a.tables = c->tables; a.batch = batch;
    bits_host.resize(batch);
    for (int b = 0; b < batch; ++b) bits_host[b] = (uint8_t)cfgs[b].bits;
    a.bits_host = bits_host.data();
    for (int b = 0; b < batch; ++b)
      a.quant_bytes_per_weight += cfgs[b].bits / 8.0 + 1.0 / cfgs[b].block +
                                  (v_bits(cfgs[b]) / 8.0) / ((double)cfgs[b].block * cfgs[b].scale_block);
    if (direct) {
      a.codes = direct->codes; a.sidx = direct->sidx; a.v = direct->v;
    } else {
      a.codes = c->at<uint8_t>(pl.codes); a.strideCodes = pl.strideCodes;
      a.sidx = c->at<uint8_t>(pl.sidx); a.strideSidx = pl.strideSidx;
      a.v = c->at<float>(pl.v); a.strideV = pl.strideV;
    }
    a.blk = c->at<BlockRec>(pl.blk); a.strideBlk = pl.strideBlk;
    a.err_part = c->at<double>(pl.epart); a.strideErrPart = pl.strideEpart;
    errs = c->at<double>(pl.errs);
    a.strideErrOut = MAX_ITERS;
    set_first(Y1, B1);
    return LQ_OK;
  }

  // The factors of the first Factorize (cold start): shared by every problem of the batch.
  void set_first(const float* Yfirst, const float* Bfirst) {
    Y1 = Yfirst; B1 = Bfirst;
    Ycur = Y1; Bcur = B1; sY = 0; sB = 0;
    lamcur = c->lam_cold; sLam = 0;
  }

  // Q(0) = Quantize(W) (Section 3.1, footnote on the initialisation): quantizes W - 0 with the zeroed warm bases as
  // factors and leaves the input of the first Factorize, W - Q(0) (scaled when weighted), in the residual buffer.
  int init_quantized(const float** A0) {
    const Plan& pl = c->pl;
    a.Y = w.Yw; a.B = w.Bw; a.strideY = pl.strideYw; a.strideB = pl.strideBw;
    a.R = nullptr; a.Qd = nullptr; a.err_out = errs;
    if (pl.stridePacked) {
      a.packed = c->at<uint16_t>(pl.packed); a.stridePacked = pl.stridePacked;
      LQ_TRY(launch_pack_factors(a, c->st));
    } else {
      a.packed = nullptr; a.stridePacked = 0;
    }
    LQ_TRY(launch_lowrank_blockquant(a, false, c->st));
    LQ_TRY(launch_scalequant_error(a, min_block, false, c->st));
    a.R = c->at<float>(pl.R); a.strideR = pl.strideR;
    LQ_TRY(launch_residual(a, c->st));
    *A0 = a.R;
    return LQ_OK;
  }

  // Iteration t: Quantize(W - L1 L2) and its error, then (unless it is the last) the next Factorize.
  int step(int t) {
    if (stopped || t > iters) return LQ_OK;
    const Plan& pl = c->pl;
    a.Y = Ycur; a.B = Bcur; a.strideY = sY; a.strideB = sB;
    a.R = nullptr; a.Qd = nullptr; a.err_out = errs + (t - 1);
    if (direct) point_codes(t);
    // the error of an iteration costs extra arithmetic per weight: only computed when somebody looks at it
    const bool with_err = want_trace || early_stop || t == iters;
    if (pl.stridePacked) {
      a.packed = c->at<uint16_t>(pl.packed); a.stridePacked = pl.stridePacked;
      LQ_TRY(launch_pack_factors(a, c->st));
    } else {
      a.packed = nullptr; a.stridePacked = 0;
    }
    LQ_TRY(launch_lowrank_blockquant(a, with_err, c->st));
    LQ_TRY(launch_scalequant_error(a, min_block, with_err, c->st));
#ifdef LQ_TESTING_HOOKS
    LQ_TRY(capture_iterate(t));
#endif
    done = t;
    bool last = t == iters;
    returned = t;
    if (early_stop && batch == 1) {        // Algorithm 2's stopping rule needs eps_t on the host
      double eps = 0.0;
      LQ_HIP_TRY(hipMemcpyAsync(&eps, errs + (t - 1), sizeof(double), hipMemcpyDeviceToHost, c->st));
      LQ_HIP_TRY(hipStreamSynchronize(c->st));
      if (eps > prev_eps) {
        last = true;
        if (early_stop == 2) returned = t - 1;     // also without output buffers: the sweep reports that iterate's error
      } else if (keep_best()) {
        LQ_TRY(emit_factors(*c, Ycur, Bcur, lamcur, direct->L1, direct->L2, direct->sigma));
      }
      prev_eps = eps;
    }
    if (last) { stopped = true; return LQ_OK; }
    a.strideR = pl.strideR;
    if (pl.prm.prec == 2) {
      a.R16 = c->at<uint16_t>(pl.R); a.R16lo = reinterpret_cast<uint8_t*>(a.R16 + pl.strideR * (size_t)pl.batch); a.r_scale = c->a_scale;
    }
    else a.R = c->at<float>(pl.R);
    LQ_TRY(launch_residual(a, c->st));
    a.R16 = nullptr; a.R16lo = nullptr;
    LQ_TRY(warm_factorize(*c, w, Bcur, sB, lamcur, sLam, (t == 1 ? qw2 : qw).data(), batch));
    Ycur = w.Yw; Bcur = w.Bw; sY = pl.strideYw; sB = pl.strideBw;
    lamcur = c->at<double>(pl.lam); sLam = pl.prm.lw;
#ifdef LQ_TESTING_HOOKS
    LQ_TRY(capture_sigma(t));
#endif
    return LQ_OK;
  }

#ifdef LQ_TESTING_HOOKS
  // Testing build: the sweep copies out one configuration's quantized component after a chosen iteration (dense) and
  // the singular values the next Factorize finds for W - Q of that iterate, so that a test can redo that single step
  // from the very same Q on the CPU.
  int capture_slot(int t) const {
    const testing::Capture& cap = testing::capture();
    if (!cap.armed || direct || t != cap.iter) return -1;
    for (int b = 0; b < batch; ++b)
      if ((cfg_ids ? cfg_ids[b] : b) == cap.cfg) return b;
    return -1;
  }
  int capture_iterate(int t) {
    const int b = capture_slot(t);
    if (b < 0) return LQ_OK;
    PhaseArgs one = a;
    one.batch = 1; one.prob = a.prob + b; one.bits_host = a.bits_host + b; one.quant_bytes_per_weight = a.quant_bytes_per_weight / batch;
    one.codes = a.codes + (size_t)b * a.strideCodes; one.sidx = a.sidx + (size_t)b * a.strideSidx;
    one.v = a.v + (size_t)b * a.strideV;
    one.R = nullptr; one.Qd = testing::capture().Q; one.strideQd = 0;
    return launch_residual(one, c->st);
  }
  int capture_sigma(int t) {
    const int b = capture_slot(t);
    const testing::Capture& cap = testing::capture();
    if (b < 0 || !cap.sigma) return LQ_OK;
    const Plan& pl = c->pl;
    std::vector<double> lamh(pl.rank);
    LQ_HIP_TRY(hipMemcpyAsync(lamh.data(), c->at<double>(pl.lam) + (size_t)b * pl.prm.lw, sizeof(double) * pl.rank,
                              hipMemcpyDeviceToHost, c->st));
    LQ_HIP_TRY(hipStreamSynchronize(c->st));
    for (int j = 0; j < pl.rank; ++j) cap.sigma[j] = std::sqrt(lamh[j]);
    return LQ_OK;
  }
#endif

  // Dense Q if asked for, then the error trace comes to the host (synchronizes the stream).
  // Host outputs: trace[b * iters + t] (NaN where not computed), iters_done[b].
  int finish(double* trace, int32_t* iters_done, int32_t* best_iter = nullptr) {
    if (keep_best() && returned > 0) {       // outputs = the pieces of iteration `returned`
      const Plan& pl = c->pl;
      point_codes(returned);
      if (a.codes != direct->codes) {
        const int64_t n = pl.d * pl.k;
        const lq_config& cf = cfgs[0];
        LQ_HIP_TRY(hipMemcpyAsync(direct->codes, a.codes, lq_codes_bytes(n, cf.bits), hipMemcpyDeviceToDevice, c->st));
        LQ_HIP_TRY(hipMemcpyAsync(direct->sidx, a.sidx, (size_t)num_blocks(n, cf), hipMemcpyDeviceToDevice, c->st));
        LQ_HIP_TRY(hipMemcpyAsync(direct->v, a.v, sizeof(float) * (size_t)num_groups(n, cf), hipMemcpyDeviceToDevice,
                                  c->st));
        point_codes(1);                      // the caller's buffers
      }
    }
    if (direct && direct->Qd) {
      a.R = nullptr; a.Qd = direct->Qd; a.strideQd = 0;
      LQ_TRY(launch_residual(a, c->st));
    }
    host_err.assign((size_t)batch * MAX_ITERS, 0.0);
    for (int b = 0; b < batch; ++b)   // only the used prefix of every row
      LQ_HIP_TRY(hipMemcpyAsync(host_err.data() + (size_t)b * MAX_ITERS, errs + (size_t)b * MAX_ITERS,
                                sizeof(double) * done, hipMemcpyDeviceToHost, c->st));
    LQ_HIP_TRY(hipStreamSynchronize(c->st));
    for (int b = 0; b < batch; ++b) {
      int nd = done;
      int best = done;
      if (early_stop && batch > 1) {         // lock-step batches apply the rule after the fact
        for (int t = 1; t < done; ++t)
          if (host_err[(size_t)b * MAX_ITERS + t] > host_err[(size_t)b * MAX_ITERS + t - 1]) {
            nd = t + 1;
            best = early_stop == 2 ? t : t + 1;
            break;
          }
      } else if (batch == 1) {
        best = returned;
      }
      if (best_iter) best_iter[b] = best;
      if (iters_done) iters_done[b] = nd;
      if (trace)
        for (int t = 0; t < iters; ++t)
          trace[(size_t)b * iters + t] =
              (t < nd && (want_trace || early_stop || t == iters - 1)) ? host_err[(size_t)b * MAX_ITERS + t] : NAN;
    }
    return LQ_OK;
  }
};

// Extra streams for lq_error_table's interleaved sub-batches (default priority).  One process-wide pool per device:
// a call leases what it needs and hands it back on every exit path, so the number of streams the library ever creates
// is the largest number in use at one time (concurrent calls x (streams - 1)), whatever the number of host threads
// that come and go.  lq_release_streams destroys the idle ones.
struct StreamPool {
  std::mutex mu;
  std::vector<hipStream_t> idle[MAX_DEVICES];
};
static StreamPool& stream_pool() { static StreamPool p; return p; }

struct StreamLease {            // also owns the event the sub-batches wait for
  int dev = -1;
  std::vector<hipStream_t> held;
  hipEvent_t ready = nullptr;
  int take(hipStream_t* out) {
    if (dev < 0) {
      LQ_HIP_TRY(hipGetDevice(&dev));
      if (dev < 0 || dev >= MAX_DEVICES) { dev = -1; return LQ_ERR_HIP; }
    }
    StreamPool& p = stream_pool();
    hipStream_t s = nullptr;
    {
      std::lock_guard<std::mutex> lock(p.mu);
      if (!p.idle[dev].empty()) { s = p.idle[dev].back(); p.idle[dev].pop_back(); }
    }
    if (!s) LQ_HIP_TRY(hipStreamCreateWithFlags(&s, hipStreamNonBlocking));
    held.push_back(s);
    *out = s;
    return LQ_OK;
  }
  ~StreamLease() {
    if (ready) (void)hipEventDestroy(ready);
    if (held.empty()) return;
    StreamPool& p = stream_pool();
    std::lock_guard<std::mutex> lock(p.mu);
    for (hipStream_t s : held) p.idle[dev].push_back(s);
  }
};

static int emit_factors(const Ctx& c, const float* Y, const float* B, const double* lam, float* L1, float* L2,
                        double* sigma_host) {
  const Plan& pl = c.pl;
  LQ_TRY(launch_assemble_factors(Y, pl.ldd, B, pl.ldk, lam, pl.rank, pl.d, pl.k,
                                 c.rsr, c.rsc, L1, L2, c.st));
  std::vector<double> lamh(pl.rank);
  LQ_HIP_TRY(hipMemcpyAsync(lamh.data(), lam, sizeof(double) * pl.rank, hipMemcpyDeviceToHost, c.st));
  LQ_HIP_TRY(hipStreamSynchronize(c.st));
  if (sigma_host)
    for (int j = 0; j < pl.rank; ++j) sigma_host[j] = std::sqrt(lamh[j]);
  return LQ_OK;
}

static bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

static int check_workspace(const void* ws, size_t have, size_t need) {
  if (!ws || ((uintptr_t)ws & 255) != 0 || have < need) return LQ_ERR_WORKSPACE;
  return LQ_OK;
}

}  // namespace lq

using namespace lq;

extern "C" {

size_t lq_factorize_workspace_bytes(int64_t d, int64_t k, int rank, const lq_svd_params* p) {
  return lq_decompose_workspace_bytes(d, k, rank, p);
}

size_t lq_decompose_workspace_bytes(int64_t d, int64_t k, int rank, const lq_svd_params* p) {
  Params prm;
  if (check_matrix_args(d, k, rank) != LQ_OK || resolve_params(rank, p, prm) != LQ_OK) return 0;
  Plan pl;
  make_plan(d, k, rank, prm, 1, pl);
  return pl.total;
}

size_t lq_error_table_workspace_bytes(int64_t d, int64_t k, int rank, int n_cfgs, const lq_svd_params* p) {
  Params prm;
  if (n_cfgs < 1 || check_matrix_args(d, k, rank) != LQ_OK || resolve_params(rank, p, prm) != LQ_OK) return 0;
  const int batch_max = std::min(n_cfgs, prm.max_batch);
  const int nsub = std::max(1, std::min(prm.streams, batch_max / 4));
  Plan pl;
  make_plan(d, k, rank, prm, (batch_max + nsub - 1) / nsub, pl);
  return up256(pl.total) * nsub;
}

int lq_factorize(const float* A, int64_t d, int64_t k, int rank, const float* row_w, const float* col_w,
                 uint64_t seed, const lq_svd_params* p, float* L1, float* L2, double* sigma, void* workspace,
                 size_t workspace_bytes, void* stream) {
  if (!A || !L1 || !L2) return LQ_ERR_NULL;
  LQ_TRY(check_matrix_args(d, k, rank));
  if ((row_w == nullptr) != (col_w == nullptr)) return LQ_ERR_WEIGHT;
  if (!aligned16(A) || !aligned16(L1) || !aligned16(L2)) return LQ_ERR_ARG;
  Params prm;
  LQ_TRY(resolve_params(rank, p, prm));
  Ctx c;
  make_plan(d, k, rank, prm, 1, c.pl);
  LQ_TRY(check_workspace(workspace, workspace_bytes, c.pl.total));
  LQ_TRY(setup_common(c, A, row_w, col_w, workspace, (hipStream_t)stream));
  const float* A0; const float* Y; const float* B;
  LQ_TRY(first_input(c, &A0));
  LQ_TRY(cold_factorize(c, A0, seed, &Y, &B));
  return emit_factors(c, Y, B, c.at<double>(c.pl.lam_cold), L1, L2, sigma);
}

int lq_decompose(const float* W, int64_t d, int64_t k, int rank, lq_config cfg, int iters, int early_stop,
                 const float* row_w, const float* col_w, uint64_t seed, const lq_svd_params* p, float* L1, float* L2,
                 uint8_t* q_codes, uint8_t* q_scale_idx, float* q_v, float* Q_dense, double* err, double* err_trace,
                 int32_t* iters_done, double* sigma, void* workspace, size_t workspace_bytes, void* stream) {
  if (!W || !L1 || !L2 || !q_codes || !q_scale_idx || !q_v) return LQ_ERR_NULL;
  LQ_TRY(check_matrix_args(d, k, rank));
  LQ_TRY(check_quant_args(d * k, cfg));
  if (cfg.block > 128 || k % cfg.block != 0) return cfg.block > 128 ? LQ_ERR_CONFIG : LQ_ERR_SHAPE;
  if ((row_w == nullptr) != (col_w == nullptr)) return LQ_ERR_WEIGHT;
  if (iters < 1 || iters > MAX_ITERS || early_stop < 0 || early_stop > 2) return LQ_ERR_ARG;
  if (!aligned16(W) || !aligned16(L1) || !aligned16(L2) || !aligned16(q_codes) || (Q_dense && !aligned16(Q_dense)))
    return LQ_ERR_ARG;
  Params prm;
  LQ_TRY(resolve_params(rank, p, prm));
  Ctx c;
  make_plan(d, k, rank, prm, 1, c.pl);
  LQ_TRY(check_workspace(workspace, workspace_bytes, c.pl.total));
  LQ_TRY(setup_common(c, W, row_w, col_w, workspace, (hipStream_t)stream));
  LQ_TRY(residual_scale(c));
  const float* A0; const float* Y1; const float* B1;
  LoopOut direct{q_codes, q_scale_idx, q_v, Q_dense, L1, L2, sigma};
  std::vector<double> trace(iters, NAN);
  int32_t done = 0;
  Loop lp;
  lp.c = &c; lp.cfgs = &cfg; lp.batch = 1; lp.iters = iters; lp.early_stop = early_stop;
  lp.want_trace = err_trace != nullptr; lp.direct = &direct;
  LQ_TRY(lp.begin());
  if (prm.init_quantized) LQ_TRY(lp.init_quantized(&A0));
  else LQ_TRY(first_input(c, &A0));
  LQ_TRY(cold_factorize(c, A0, seed, &Y1, &B1));
  lp.set_first(Y1, B1);
  for (int t = 1; t <= iters; ++t) LQ_TRY(lp.step(t));
  int32_t best = 0;
  LQ_TRY(lp.finish(trace.data(), &done, &best));
  if (!lp.keep_best()) LQ_TRY(emit_factors(c, lp.Ycur, lp.Bcur, lp.lamcur, L1, L2, sigma));
  if (err) *err = trace[best - 1];
  if (err_trace) std::memcpy(err_trace, trace.data(), sizeof(double) * iters);
  if (iters_done) *iters_done = done;
  return LQ_OK;
}

size_t lq_fisher_row_col_workspace_bytes(int64_t d, int64_t k) {
  if (d <= 0 || k <= 0 || d > (1 << 30) || k > (1 << 30)) return 0;
  return fisher_scratch_doubles(d, k) * sizeof(double) + 256;
}

int lq_fisher_row_col(const float* F, int64_t d, int64_t k, float* row_w, float* col_w, void* workspace,
                      size_t workspace_bytes, void* stream) {
  if (!F || !row_w || !col_w) return LQ_ERR_NULL;
  if (d <= 0 || k <= 0 || d > (1 << 30) || k > (1 << 30)) return LQ_ERR_SHAPE;
  LQ_TRY(check_workspace(workspace, workspace_bytes, lq_fisher_row_col_workspace_bytes(d, k)));
  return launch_fisher_row_col(F, d, k, reinterpret_cast<double*>(workspace), row_w, col_w, (hipStream_t)stream);
}

int lq_error_table(const float* W, int64_t d, int64_t k, int rank, const lq_config* cfgs, int n_cfgs, int iters,
                   int early_stop, const float* row_w, const float* col_w, uint64_t seed, const lq_svd_params* p,
                   double* err_sq, double* storage_bits, double* err_trace, void* workspace, size_t workspace_bytes,
                   void* stream) {
  if (!W || !cfgs || !err_sq || !storage_bits) return LQ_ERR_NULL;
  if (n_cfgs < 1 || iters < 1 || iters > MAX_ITERS || early_stop < 0 || early_stop > 2) return LQ_ERR_ARG;
  LQ_TRY(check_matrix_args(d, k, rank));
  std::vector<lq_config> cf(cfgs, cfgs + n_cfgs);
  for (auto& cc : cf) {
    LQ_TRY(check_quant_args(d * k, cc));
    if (cc.block > 128) return LQ_ERR_CONFIG;
    if (k % cc.block != 0) return LQ_ERR_SHAPE;
  }
  // The number of subspace iterations per pass depends on the configuration (see Loop::begin: most for a single-level
  // scale quantizer, fewest for codes of four or more bits): configurations are processed by class, keeping the
  // caller's order within a class, so that lock-step batches are as uniform as possible.  order[i] is the caller's
  // index of the i-th configuration processed.
  std::vector<int> order(n_cfgs);
  for (int i = 0; i < n_cfgs; ++i) order[i] = i;
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return power_class(cf[a]) < power_class(cf[b]); });
  {
    std::vector<lq_config> sorted(n_cfgs);
    for (int i = 0; i < n_cfgs; ++i) sorted[i] = cf[order[i]];
    cf.swap(sorted);
  }
  if ((row_w == nullptr) != (col_w == nullptr)) return LQ_ERR_WEIGHT;
  if (!aligned16(W)) return LQ_ERR_ARG;
  Params prm;
  LQ_TRY(resolve_params(rank, p, prm));
  if (prm.init_quantized) return LQ_ERR_ARG;   // the sweep shares the first Factorize between configurations
  // The configurations of a batch are split over `streams` sub-batches, each with its own stream and workspace
  // slice; the host enqueues their iterations alternately, so the latency-bound single-workgroup steps of one
  // sub-batch (Cholesky, Jacobi) overlap the bandwidth- and MFMA-bound kernels of the other.
  const int batch_max = std::min(n_cfgs, prm.max_batch);
  const int nsub = std::max(1, std::min(prm.streams, batch_max / 4));
  const int per_sub = (batch_max + nsub - 1) / nsub;
  std::vector<Ctx> cs(nsub);
  make_plan(d, k, rank, prm, per_sub, cs[0].pl);
  const size_t slice = up256(cs[0].pl.total);
  LQ_TRY(check_workspace(workspace, workspace_bytes, slice * nsub));
  Ctx& c = cs[0];
  LQ_TRY(setup_common(c, W, row_w, col_w, workspace, (hipStream_t)stream));
  LQ_TRY(residual_scale(c));
  const float* A0; const float* Y1; const float* B1;
  LQ_TRY(first_input(c, &A0));
  LQ_TRY(cold_factorize(c, A0, seed, &Y1, &B1));
  StreamLease lease;             // streams go back to the pool and the event is destroyed on every return below
  if (nsub > 1) {
    LQ_HIP_TRY(hipEventCreateWithFlags(&lease.ready, hipEventDisableTiming));
    LQ_HIP_TRY(hipEventRecord(lease.ready, c.st));
  }
  for (int s1 = 1; s1 < nsub; ++s1) {
    cs[s1] = c;
    cs[s1].ws = (char*)workspace + slice * s1;
    LQ_TRY(lease.take(&cs[s1].st));
    LQ_HIP_TRY(hipStreamWaitEvent(cs[s1].st, lease.ready, 0));
  }
  int rc = LQ_OK;
#ifdef LQ_TESTING_HOOKS
  struct Disarm { ~Disarm() { testing::capture().armed = false; } } disarm;     // a capture request serves one call
#endif
  std::vector<double> trace((size_t)per_sub * iters);
  std::vector<int32_t> done(per_sub), best(per_sub);
  for (int c0 = 0; c0 < n_cfgs && rc == LQ_OK; c0 += batch_max) {
    const int nb = std::min(batch_max, n_cfgs - c0);
    std::vector<Loop> loops(nsub);
    int used = 0;
    for (int s1 = 0; s1 < nsub; ++s1) {
      const int b0 = s1 * per_sub, b1 = std::min(nb, b0 + per_sub);
      if (b0 >= b1) break;
      Loop& lp = loops[s1];
      lp.c = &cs[s1]; lp.cfgs = cf.data() + c0 + b0; lp.batch = b1 - b0; lp.iters = iters; lp.early_stop = early_stop;
      lp.want_trace = err_trace != nullptr; lp.Y1 = Y1; lp.B1 = B1; lp.direct = nullptr; lp.cfg_ids = order.data() + c0 + b0;
      if ((rc = lp.begin()) != LQ_OK) break;
      ++used;
    }
    for (int t = 1; t <= iters && rc == LQ_OK; ++t)
      for (int s1 = 0; s1 < used && rc == LQ_OK; ++s1) rc = loops[s1].step(t);
    for (int s1 = 0; s1 < used; ++s1) {           // always drain every stream, even after an error
      const int frc = loops[s1].finish(trace.data(), done.data(), best.data());
      if (rc == LQ_OK) rc = frc;
      if (frc != LQ_OK) continue;
      const int b0 = s1 * per_sub;
      for (int b = 0; b < loops[s1].batch; ++b) {
        const int ci = order[c0 + b0 + b];                            // the caller's index of this configuration
        const double eps = trace[(size_t)b * iters + best[b] - 1];   // the iterate that would be returned
        err_sq[ci] = eps * eps;
        storage_bits[ci] = lq_storage_bits(d * k, cf[c0 + b0 + b]);
        if (err_trace) std::memcpy(err_trace + (size_t)ci * iters, trace.data() + (size_t)b * iters, sizeof(double) * iters);
      }
    }
  }
  return rc;
}

int lq_release_streams(void) {
  StreamPool& p = stream_pool();
  std::lock_guard<std::mutex> lock(p.mu);
  int rc = LQ_OK;
  for (int dev = 0; dev < MAX_DEVICES; ++dev) {
    for (hipStream_t st : p.idle[dev])
      if (hipStreamDestroy(st) != hipSuccess) rc = LQ_ERR_HIP;
    p.idle[dev].clear();
  }
  return rc;
}

}  // extern "C"
