/*
 * CPU oracle for the LQ decomposition path  --  TEST INFRASTRUCTURE, not the product.
 *
 * Plain, slow, obviously-correct C written from the paper (LQ-LoRA, arxiv 2311.12023).  It shares
 * no code with the GPU library and is only ever called by the tests, the smoke check and the
 * benchmark's CPU-baseline leg.  Nothing here is blocked, fused or reordered beyond what the cited
 * passage states.  Floating point: fp32 where the quantizer's result depends on it (stated per
 * function), float64 everywhere else.  Compile with -ffp-contract=off and without fast-math.
 *
 * Readings taken where the paper is silent are marked "reading:" at the point of use.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <float.h>

#define OQ_OK 0
#define OQ_ERR (-1)

typedef struct {
  int32_t bits;        /* b0: NF code bits                      (Section 3.2, config tuple)  */
  int32_t block;       /* B0: weights per absmax block                                        */
  int32_t scale_block; /* B1: absmax values per second-level group                            */
  int32_t scale_bits;  /* b1: bits of the integer-quantized absmax values                     */
  int32_t v_dtype;     /* b2: 0 = fp32, 1 = bf16, 2 = fp16                                    */
} oq_config;

/* ------------------------------------------------------------------------------------------ */
/* Gaussian quantile by bisection on Phi(x) = erfc(-x/sqrt2)/2 (Section 2.2: q_i = Phi^-1(p_i)). */
static double oq_phi(double x) { return 0.5 * erfc(-x / sqrt(2.0)); }

double oq_norm_ppf(double p) {
  double lo = -40.0, hi = 40.0;
  for (int it = 0; it < 400; ++it) {
    double mid = 0.5 * (lo + hi);
    if (oq_phi(mid) < p) lo = mid; else hi = mid;
  }
  return 0.5 * (lo + hi);
}

/* NF-b codebook (Section 2.2).  2^(b-1) evenly spaced probabilities on [delta, 1/2] and
 * 2^(b-1)+1 on [1/2, 1-delta], delta = (1/30 + 1/32)/2.
 * reading: the two sets share 1/2, which is kept once, so that 2^b values result; the quantile at
 * 1/2 is exactly 0.  Quantiles are divided by the last one and rounded once to fp32.
 * out[i] is the value of code i; codes ascend with value. */
int oq_codebook(int bits, float* out) {
  if (bits < 2 || bits > 8) return OQ_ERR;
  const int half = 1 << (bits - 1);
  const int ncode = 1 << bits;
  const double delta = 0.5 * (1.0 / 30.0 + 1.0 / 32.0);
  double q[256];
  for (int i = 0; i < half; ++i) {               /* [delta, 1/2], last one is 1/2 itself */
    double p = delta + (double)i * (0.5 - delta) / (double)(half - 1);
    q[i] = (i == half - 1) ? 0.0 : oq_norm_ppf(p);
  }
  for (int i = 1; i <= half; ++i) {              /* (1/2, 1-delta] */
    double p = 0.5 + (double)i * (0.5 - delta) / (double)half;
    q[half - 1 + i] = oq_norm_ppf(p);
  }
  for (int i = 0; i < ncode; ++i) out[i] = (float)(q[i] / q[ncode - 1]);
  return OQ_OK;
}

/* ------------------------------------------------------------------------------------------ */
/* cast(v, b2) (Section 3.2): round-to-nearest-even to the storage type, returned as fp32.     */
static float oq_round_bf16(float x) {
  uint32_t u; memcpy(&u, &x, 4);
  if ((u & 0x7f800000u) == 0x7f800000u) return x;            /* inf / nan unchanged */
  uint32_t lsb = (u >> 16) & 1u;
  u += 0x7fffu + lsb;
  u &= 0xffff0000u;
  float r; memcpy(&r, &u, 4); return r;
}
static float oq_round_fp16(float x) {
  /* value-level rounding to binary16 (11-bit significand, exponents -14..15, subnormals). */
  if (x == 0.0f || isnan(x) || isinf(x)) return x;
  double a = fabs((double)x);
  int e; frexp(a, &e);                   /* a = m * 2^e, m in [0.5,1) */
  int ex = e - 1;                        /* a in [2^ex, 2^(ex+1)) */
  if (ex < -14) ex = -14;                /* subnormal spacing */
  double ulp = ldexp(1.0, ex - 10);
  double r = nearbyint(a / ulp) * ulp;   /* default rounding mode: ties to even */
  if (r > 65504.0) r = INFINITY;
  return (float)(x < 0 ? -r : r);
}
float oq_cast_v(float v, int v_dtype) {
  if (v_dtype == 1) return oq_round_bf16(v);
  if (v_dtype == 2) return oq_round_fp16(v);
  return v;
}
int oq_v_bits(int v_dtype) { return v_dtype == 0 ? 32 : 16; }

static int oq_config_ok(oq_config c) {
  if (c.bits < 2 || c.bits > 8) return 0;
  if (c.block < 1 || c.scale_block < 1) return 0;
  if (c.scale_bits < 2 || c.scale_bits > 8) return 0;
  if (c.v_dtype < 0 || c.v_dtype > 2) return 0;
  return 1;
}

/* ------------------------------------------------------------------------------------------ */
/* Quantize (Section 3.2): Quantize-NF(x, b0, B0) -> codes, s;  Quantize-INT(s, b1, B1) -> s^, v;
 * cast(v, b2).  x is the row-major flattening, n a multiple of B0; the last group may be short.
 * Outputs: codes[n] one code per byte (unpacked), scale_idx[n/B0], v[ceil(n/(B0*B1))] (already
 * cast to b2, held as fp32), s_exact[n/B0] optional (the un-quantized absmax values).
 *
 * readings:
 *  - u/s is taken as fl32(u * fl32(1/s)): one correctly rounded reciprocal per block, one
 *    correctly rounded product per weight.  A block with s = 0 (or whose reciprocal overflows)
 *    uses reciprocal 0, so all its codes are the code of value 0.
 *  - argmin ties go to the lower code index.  Distances are taken in double: both operands are
 *    fp32 numbers, so the differences are exact and the comparison is exact.
 *  - integer scale quantizer: levels n1 = 2^(b1-1)-1; sigma = fl32(v/n1);
 *    idx = clamp(rne(fl32(s/sigma)), 0, n1) (round half to even); v = 0 gives idx = 0.
 *  - the codes are chosen against the exact absmax s; only dequantization sees the
 *    reconstructed scale.  idx is computed from the un-cast v; the stored v is cast(v, b2). */
int oq_quantize(const float* x, int64_t n, oq_config c, uint8_t* codes, uint8_t* scale_idx,
                float* v, float* s_exact) {
  if (!oq_config_ok(c) || n < 0 || n % c.block != 0) return OQ_ERR;
  float q[256];
  oq_codebook(c.bits, q);
  const int ncode = 1 << c.bits;
  const int64_t nb = n / c.block;
  float* s = (float*)malloc(sizeof(float) * (size_t)(nb > 0 ? nb : 1));
  if (!s) return OQ_ERR;
#pragma omp parallel for schedule(static)
  for (int64_t b = 0; b < nb; ++b) {
    const float* u = x + b * c.block;
    float amax = 0.0f;
    for (int j = 0; j < c.block; ++j) { float a = fabsf(u[j]); if (a > amax) amax = a; }
    s[b] = amax;
    float rcp = 0.0f;
    if (amax > 0.0f) { rcp = 1.0f / amax; if (isinf(rcp)) rcp = 0.0f; }
    for (int j = 0; j < c.block; ++j) {
      volatile float xn = u[j] * rcp;           /* fl32 product, kept out of any wider register */
      int best = 0;
      double bestd = fabs((double)q[0] - (double)xn);
      for (int i = 1; i < ncode; ++i) {
        double dist = fabs((double)q[i] - (double)xn);
        if (dist < bestd) { bestd = dist; best = i; }
      }
      codes[b * c.block + j] = (uint8_t)best;
    }
  }
  const int n1 = (1 << (c.scale_bits - 1)) - 1;
  const int64_t ng = (nb + c.scale_block - 1) / c.scale_block;
  for (int64_t g = 0; g < ng; ++g) {
    int64_t b0 = g * c.scale_block, b1 = b0 + c.scale_block; if (b1 > nb) b1 = nb;
    float vmax = 0.0f;
    for (int64_t b = b0; b < b1; ++b) if (s[b] > vmax) vmax = s[b];
    volatile float sigma = vmax / (float)n1;
    for (int64_t b = b0; b < b1; ++b) {
      int idx = 0;
      if (sigma > 0.0f) {
        volatile float ratio = s[b] / sigma;
        float r = nearbyintf(ratio);
        if (r < 0.0f) r = 0.0f;
        if (r > (float)n1) r = (float)n1;
        idx = (int)r;
      }
      scale_idx[b] = (uint8_t)idx;
    }
    v[g] = oq_cast_v(vmax, c.v_dtype);
  }
  if (s_exact) memcpy(s_exact, s, sizeof(float) * (size_t)nb);
  free(s);
  return OQ_OK;
}

/* Reconstructed block scale: s^_b = fl32(idx_b * fl32(v^_g / n1)). */
static float oq_block_scale(uint8_t idx, float vhat, int scale_bits) {
  const int n1 = (1 << (scale_bits - 1)) - 1;
  volatile float sigma = vhat / (float)n1;
  volatile float sh = (float)idx * sigma;
  return sh;
}

/* Dequantize (Section 3.2, "simply reverses this process"): out_j = fl32(q~[code_j] * s^_block). */
int oq_dequantize(const uint8_t* codes, const uint8_t* scale_idx, const float* v, int64_t n,
                  oq_config c, float* out) {
  if (!oq_config_ok(c) || n < 0 || n % c.block != 0) return OQ_ERR;
  float q[256];
  oq_codebook(c.bits, q);
  const int64_t nb = n / c.block;
  for (int64_t b = 0; b < nb; ++b) {
    float sh = oq_block_scale(scale_idx[b], v[b / c.scale_block], c.scale_bits);
    for (int j = 0; j < c.block; ++j) {
      volatile float val = q[codes[b * c.block + j]] * sh;
      out[b * c.block + j] = val;
    }
  }
  return OQ_OK;
}

/* Forward product with a decomposed weight (Section 3.2 "Implementation", Appendix A): the plain definition
 * Y = X (Q + L1 L2) in double, with Q = Dequantize of the stored codes (unpacked, one per byte).
 * X: m x d, L1: d x r, L2: r x k (r may be 0), Y: m x k doubles.  absY, if not NULL, receives |X| (|Q| + |L1 L2|'s
 * entrywise bound |L1| |L2|) -- the scale that floating-point error bounds of a product are stated against. */
int oq_matmul(const float* X, int m, int d, int k, const uint8_t* codes, const uint8_t* scale_idx, const float* v,
              oq_config c, const float* L1, const float* L2, int r, double* Y, double* absY) {
  const int64_t n = (int64_t)d * k;
  float* q = (float*)malloc((size_t)n * sizeof(float));
  double* w = (double*)malloc((size_t)n * sizeof(double));
  double* wa = (double*)malloc((size_t)n * sizeof(double));
  if (!q || !w || !wa || oq_dequantize(codes, scale_idx, v, n, c, q) != OQ_OK) { free(q); free(w); free(wa); return OQ_ERR; }
  for (int i = 0; i < d; ++i)
    for (int j = 0; j < k; ++j) {
      double low = 0.0, lowa = 0.0;
      for (int t = 0; t < r; ++t) {
        low += (double)L1[(int64_t)i * r + t] * (double)L2[(int64_t)t * k + j];
        lowa += fabs((double)L1[(int64_t)i * r + t]) * fabs((double)L2[(int64_t)t * k + j]);
      }
      w[(int64_t)i * k + j] = (double)q[(int64_t)i * k + j] + low;
      wa[(int64_t)i * k + j] = fabs((double)q[(int64_t)i * k + j]) + lowa;
    }
  for (int a = 0; a < m; ++a)
    for (int j = 0; j < k; ++j) {
      double y = 0.0, ya = 0.0;
      for (int i = 0; i < d; ++i) {
        y += (double)X[(int64_t)a * d + i] * w[(int64_t)i * k + j];
        ya += fabs((double)X[(int64_t)a * d + i]) * wa[(int64_t)i * k + j];
      }
      Y[(int64_t)a * k + j] = y;
      if (absY) absY[(int64_t)a * k + j] = ya;
    }
  free(q); free(w); free(wa);
  return OQ_OK;
}

/* Packed code layout (the paper packs sub-8-bit codes into int8 containers, Appendix A, and gives
 * no layout).  reading: little-endian bit stream, code j occupies bits [j*b, (j+1)*b). */
int64_t oq_packed_bytes(int64_t n, int bits) { return (n * bits + 7) / 8; }
void oq_pack(const uint8_t* codes, int64_t n, int bits, uint8_t* packed) {
  memset(packed, 0, (size_t)oq_packed_bytes(n, bits));
  for (int64_t j = 0; j < n; ++j)
    for (int t = 0; t < bits; ++t)
      if ((codes[j] >> t) & 1) { int64_t pos = j * bits + t; packed[pos >> 3] |= (uint8_t)(1u << (pos & 7)); }
}
void oq_unpack(const uint8_t* packed, int64_t n, int bits, uint8_t* codes) {
  for (int64_t j = 0; j < n; ++j) {
    unsigned cval = 0;
    for (int t = 0; t < bits; ++t) { int64_t pos = j * bits + t; cval |= (unsigned)((packed[pos >> 3] >> (pos & 7)) & 1) << t; }
    codes[j] = (uint8_t)cval;
  }
}

/* storage(A, c) = sizeof(A) * (b0 + b1/B0 + b2/(B0*B1)) bits  (Eq. 3). */
double oq_storage_bits(int64_t n, oq_config c) {
  return (double)n * ((double)c.bits + (double)c.scale_bits / (double)c.block +
                      (double)oq_v_bits(c.v_dtype) / ((double)c.block * (double)c.scale_block));
}

/* ------------------------------------------------------------------------------------------ */
/* Exact SVD by one-sided (Hestenes) Jacobi in double.
 * X holds nv vectors of length len, one per row (row-major, overwritten).  Rows are rotated
 * pairwise until mutually orthogonal: on return X = Sigma * Vt (row j has norm sigma_j) and
 * R (nv x nv, row-major) holds the accumulated rotations with X_in = R * X_out, i.e. column j of R
 * is the j-th left singular vector of X_in.  Pairs are visited in round-robin tournament order;
 * the pairs of one round are disjoint, so the result does not depend on the thread count.
 * Returns the number of sweeps. */
int oq_jacobi_rows(double* X, int nv, int len, double* R) {
  for (int i = 0; i < nv; ++i)
    for (int j = 0; j < nv; ++j) R[(size_t)i * nv + j] = (i == j) ? 1.0 : 0.0;
  /* R is accumulated transposed (row p of Rt <-> vector p) so that the same row rotation applies. */
  const int np = (nv + 1) & ~1;                  /* players, padded to even */
  int* who = (int*)malloc(sizeof(int) * (size_t)np);
  int sweeps = 0;
  for (; sweeps < 60; ++sweeps) {
    int rotated = 0;
    for (int i = 0; i < np; ++i) who[i] = i;
    for (int round = 0; round < np - 1; ++round) {
#pragma omp parallel for schedule(static) reduction(+ : rotated)
      for (int m = 0; m < np / 2; ++m) {
        int p = who[m], qq = who[np - 1 - m];
        if (p >= nv || qq >= nv) continue;
        if (p > qq) { int t = p; p = qq; qq = t; }
        double* xp = X + (size_t)p * len;
        double* xq = X + (size_t)qq * len;
        double alpha = 0, beta = 0, gamma = 0;
        for (int t = 0; t < len; ++t) { alpha += xp[t] * xp[t]; beta += xq[t] * xq[t]; gamma += xp[t] * xq[t]; }
        if (gamma == 0.0 || fabs(gamma) <= 1e-15 * sqrt(alpha * beta)) continue;
        rotated += 1;
        double zeta = (beta - alpha) / (2.0 * gamma);
        double tt = (zeta >= 0 ? 1.0 : -1.0) / (fabs(zeta) + sqrt(1.0 + zeta * zeta));
        double cs = 1.0 / sqrt(1.0 + tt * tt), sn = cs * tt;
        for (int t = 0; t < len; ++t) {
          double a = xp[t], b = xq[t];
          xp[t] = cs * a - sn * b;
          xq[t] = sn * a + cs * b;
        }
        double* rp = R + (size_t)p * nv;
        double* rq = R + (size_t)qq * nv;
        for (int t = 0; t < nv; ++t) {
          double a = rp[t], b = rq[t];
          rp[t] = cs * a - sn * b;
          rq[t] = sn * a + cs * b;
        }
      }
      /* rotate the tournament: player 0 fixed */
      int last = who[np - 1];
      for (int i = np - 1; i > 1; --i) who[i] = who[i - 1];
      who[1] = last;
    }
    if (!rotated) { ++sweeps; break; }
  }
  free(who);
  /* rows of R currently hold the transposed accumulation: row p of Rt = coefficients of the
   * rotated vector p in terms of the input vectors.  X_out = Rt * X_in, so X_in = Rt^T * X_out;
   * transpose in place so that column j of R is the left singular vector. */
  for (int i = 0; i < nv; ++i)
    for (int j = i + 1; j < nv; ++j) {
      double t = R[(size_t)i * nv + j]; R[(size_t)i * nv + j] = R[(size_t)j * nv + i]; R[(size_t)j * nv + i] = t;
    }
  return sweeps;
}

/* Full SVD of a row-major d x k double matrix: A = U diag(S) Vt, singular values descending.
 * U is d x m, Vt is m x k, m = min(d,k).  (Section 3.1, Eq. 2: the SVD step.) */
int oq_svd(const double* A, int d, int k, double* U, double* S, double* Vt) {
  const int m = d < k ? d : k;
  const int transposed = d > k;              /* rotate the shorter set of vectors */
  const int nv = m, len = transposed ? d : k;
  double* X = (double*)malloc(sizeof(double) * (size_t)nv * len);
  double* R = (double*)malloc(sizeof(double) * (size_t)nv * nv);
  int* order = (int*)malloc(sizeof(int) * (size_t)nv);
  double* nrm = (double*)malloc(sizeof(double) * (size_t)nv);
  if (!X || !R || !order || !nrm) return OQ_ERR;
  if (!transposed) memcpy(X, A, sizeof(double) * (size_t)d * k);
  else
    for (int i = 0; i < d; ++i)
      for (int j = 0; j < k; ++j) X[(size_t)j * d + i] = A[(size_t)i * k + j];
  oq_jacobi_rows(X, nv, len, R);
  for (int i = 0; i < nv; ++i) {
    double s2 = 0;
    for (int t = 0; t < len; ++t) s2 += X[(size_t)i * len + t] * X[(size_t)i * len + t];
    nrm[i] = sqrt(s2); order[i] = i;
  }
  for (int i = 1; i < nv; ++i) {             /* insertion sort, descending, stable */
    int o = order[i]; int j = i - 1;
    while (j >= 0 && nrm[order[j]] < nrm[o]) { order[j + 1] = order[j]; --j; }
    order[j + 1] = o;
  }
  for (int jn = 0; jn < nv; ++jn) {
    int j = order[jn];
    double sg = nrm[j];
    S[jn] = sg;
    /* unit row of X (length len) and column j of R (length nv) */
    if (!transposed) {       /* rows of A rotated: X = Sigma Vt, R = U (d x d) */
      for (int t = 0; t < k; ++t) Vt[(size_t)jn * k + t] = sg > 0 ? X[(size_t)j * len + t] / sg : 0.0;
      for (int t = 0; t < d; ++t) U[(size_t)t * m + jn] = R[(size_t)t * nv + j];
    } else {                 /* columns of A rotated: X = Sigma U^T, R = V (k x k) */
      for (int t = 0; t < d; ++t) U[(size_t)t * m + jn] = sg > 0 ? X[(size_t)j * len + t] / sg : 0.0;
      for (int t = 0; t < k; ++t) Vt[(size_t)jn * k + t] = R[(size_t)t * nv + j];
    }
  }
  free(X); free(R); free(order); free(nrm);
  return OQ_OK;
}

/* Factorize(A, F, r)  (Algorithm 4, Eq. 5).  A is d x k fp32.  Unweighted (row_w == NULL):
 * U,S,Vt <- SVD(A, r); L1 = U sqrt(S); L2 = sqrt(S) Vt.  Weighted: D_row = diag(sqrt(row_w)),
 * D_col = diag(sqrt(col_w)); SVD of D_row A D_col; L1 = D_row^-1 U sqrt(S); L2 = sqrt(S) Vt D_col^-1.
 * reading: the library receives Fisher-scale vectors row_w, col_w > 0 whose square roots are the
 * diagonal scalings.  L1 (d x r), L2 (r x k) are rounded to fp32; sigma_out[r] (optional, double). */
int oq_factorize(const float* A, int d, int k, const float* row_w, const float* col_w, int r,
                 float* L1, float* L2, double* sigma_out) {
  const int m = d < k ? d : k;
  if (r < 1 || r > m) return OQ_ERR;
  double* Ad = (double*)malloc(sizeof(double) * (size_t)d * k);
  double* U = (double*)malloc(sizeof(double) * (size_t)d * m);
  double* S = (double*)malloc(sizeof(double) * (size_t)m);
  double* Vt = (double*)malloc(sizeof(double) * (size_t)m * k);
  if (!Ad || !U || !S || !Vt) return OQ_ERR;
  for (int i = 0; i < d; ++i)
    for (int j = 0; j < k; ++j) {
      double a = (double)A[(size_t)i * k + j];
      if (row_w) a = sqrt((double)row_w[i]) * a * sqrt((double)col_w[j]);
      Ad[(size_t)i * k + j] = a;
    }
  int rc = oq_svd(Ad, d, k, U, S, Vt);
  if (rc == OQ_OK) {
    for (int p = 0; p < r; ++p) {
      double rs = sqrt(S[p]);
      if (sigma_out) sigma_out[p] = S[p];
      for (int i = 0; i < d; ++i) {
        double val = U[(size_t)i * m + p] * rs;
        if (row_w) val /= sqrt((double)row_w[i]);
        L1[(size_t)i * r + p] = (float)val;
      }
      for (int j = 0; j < k; ++j) {
        double val = rs * Vt[(size_t)p * k + j];
        if (col_w) val /= sqrt((double)col_w[j]);
        L2[(size_t)p * k + j] = (float)val;
      }
    }
  }
  free(Ad); free(U); free(S); free(Vt);
  return rc;
}

/* (W - L1 L2)_ij with the product accumulated in double. */
static double oq_lowrank_residual(const float* W, const float* L1, const float* L2, int k, int r,
                                  int i, int j) {
  double acc = 0.0;
  for (int p = 0; p < r; ++p) acc += (double)L1[(size_t)i * r + p] * (double)L2[(size_t)p * k + j];
  return (double)W[(size_t)i * k + j] - acc;
}

/* One pass through the loop body of Algorithm 2 from a given Q(t-1):
 *   L1, L2 <- Factorize(W - Q(t-1), F, r);  Q(t) <- Quantize(W - L1 L2, c);  eps_t (Eq. 4 when weighted).
 * Q holds Q(t-1) on entry and Q(t) on return; A and T are n-element work arrays; cd, si, vv receive the codes, scale
 * indices and group scales of Q(t). */
static int oq_lq_iteration(const float* W, int d, int k, int r, oq_config c, const float* row_w, const float* col_w,
                           float* Q, float* A, float* T, float* L1, float* L2, uint8_t* cd, uint8_t* si, float* vv,
                           double* sigma, double* eps_out) {
  const int64_t n = (int64_t)d * k;
  int rc;
  for (int64_t e = 0; e < n; ++e) A[e] = W[e] - Q[e];
  rc = oq_factorize(A, d, k, row_w, col_w, r, L1, L2, sigma);
  if (rc != OQ_OK) return rc;
#pragma omp parallel for schedule(static)
  for (int i = 0; i < d; ++i)
    for (int j = 0; j < k; ++j) T[(size_t)i * k + j] = (float)oq_lowrank_residual(W, L1, L2, k, r, i, j);
  rc = oq_quantize(T, n, c, cd, si, vv, NULL);
  if (rc != OQ_OK) return rc;
  oq_dequantize(cd, si, vv, n, c, Q);
  double acc = 0.0;
  for (int i = 0; i < d; ++i) {
    double rowacc = 0.0;
    for (int j = 0; j < k; ++j) {
      double diff = oq_lowrank_residual(W, L1, L2, k, r, i, j) - (double)Q[(size_t)i * k + j];
      double w = row_w ? (double)row_w[i] * (double)col_w[j] : 1.0;
      rowacc += w * diff * diff;
    }
    acc += rowacc;
  }
  *eps_out = sqrt(acc);
  return OQ_OK;
}

/* The same single iteration for callers: Algorithm 2's loop body applied once to a given Q(t-1) (Qprev, d x k fp32,
 * any matrix; all zeros gives the first iteration).  Outputs as for oq_lq_init; any of codes, scale_idx, v, Qd,
 * sigma may be NULL. */
int oq_lq_step(const float* W, int d, int k, int r, oq_config c, const float* row_w, const float* col_w,
               const float* Qprev, float* L1, float* L2, uint8_t* codes, uint8_t* scale_idx, float* v, float* Qd,
               double* err, double* sigma) {
  const int64_t n = (int64_t)d * k;
  if (!oq_config_ok(c) || n % c.block != 0) return OQ_ERR;
  if ((row_w == NULL) != (col_w == NULL)) return OQ_ERR;
  const int64_t nb = n / c.block, ng = (nb + c.scale_block - 1) / c.scale_block;
  float* Q = (float*)malloc(sizeof(float) * (size_t)n);
  float* A = (float*)malloc(sizeof(float) * (size_t)n);
  float* T = (float*)malloc(sizeof(float) * (size_t)n);
  uint8_t* cd = (uint8_t*)malloc((size_t)n);
  uint8_t* si = (uint8_t*)malloc((size_t)nb);
  float* vv = (float*)malloc(sizeof(float) * (size_t)ng);
  if (!Q || !A || !T || !cd || !si || !vv) return OQ_ERR;
  memcpy(Q, Qprev, sizeof(float) * (size_t)n);
  double eps = INFINITY;
  int rc = oq_lq_iteration(W, d, k, r, c, row_w, col_w, Q, A, T, L1, L2, cd, si, vv, sigma, &eps);
  if (err) *err = eps;
  if (codes) memcpy(codes, cd, (size_t)n);
  if (scale_idx) memcpy(scale_idx, si, (size_t)nb);
  if (v) memcpy(v, vv, sizeof(float) * (size_t)ng);
  if (Qd) memcpy(Qd, Q, sizeof(float) * (size_t)n);
  free(Q); free(A); free(T); free(cd); free(si); free(vv);
  return rc;
}

/* LQ(W, F, c, r)  (Algorithm 2; Eq. 2; stopping rule of Section 3.1).
 * Q <- 0, eps_0 <- inf; for t = 1..iters: L1,L2 <- Factorize(W - Q); Q <- Quantize(W - L1 L2, c);
 * eps_t = || sqrt(w) .* (W - Q - L1 L2) ||_F with w = 1 or row_w[i]*col_w[j]  (Eq. 4);
 * if early_stop and eps_t > eps_{t-1}: stop (the current, worse, iterate is what is returned,
 * as printed in Algorithm 2).
 * The quantizer never sees the weights.  The quantizer's input is the fp32 rounding of W - L1 L2.
 * Outputs (any may be NULL except L1, L2): codes[n] unpacked, scale_idx, v, Qd (dense Q, fp32),
 * err (eps of the last executed iteration), trace[iters], iters_done, sigma[r] of the last
 * Factorize. */
int oq_lq_init(const float* W, int d, int k, int r, oq_config c, int iters, int early_stop,
          const float* row_w, const float* col_w, float* L1, float* L2, uint8_t* codes,
          uint8_t* scale_idx, float* v, float* Qd, double* err, double* trace, int32_t* iters_done,
          double* sigma, int init_quantized) {
  const int64_t n = (int64_t)d * k;
  if (!oq_config_ok(c) || n % c.block != 0 || iters < 1) return OQ_ERR;
  if ((row_w == NULL) != (col_w == NULL)) return OQ_ERR;
  const int64_t nb = n / c.block, ng = (nb + c.scale_block - 1) / c.scale_block;
  float* Q = (float*)calloc((size_t)n, sizeof(float));
  float* A = (float*)malloc(sizeof(float) * (size_t)n);
  float* T = (float*)malloc(sizeof(float) * (size_t)n);
  uint8_t* cd = (uint8_t*)malloc((size_t)n);
  uint8_t* si = (uint8_t*)malloc((size_t)nb);
  float* vv = (float*)malloc(sizeof(float) * (size_t)ng);
  if (!Q || !A || !T || !cd || !si || !vv) return OQ_ERR;
  if (init_quantized) {   /* Section 3.1, footnote on the initialisation: Q(0) = Quantize(W) instead of 0 */
    if (oq_quantize(W, n, c, cd, si, vv, NULL) != OQ_OK) return OQ_ERR;
    oq_dequantize(cd, si, vv, n, c, Q);
  }
  /* early_stop == 2 (a variant, not the listing): the iterate before the error went up is returned, so a copy of
   * the previous iterate's pieces is kept */
  const int keep = early_stop == 2;
  float* pL1 = keep ? (float*)malloc(sizeof(float) * (size_t)d * r) : NULL;
  float* pL2 = keep ? (float*)malloc(sizeof(float) * (size_t)r * k) : NULL;
  float* pQ = keep ? (float*)malloc(sizeof(float) * (size_t)n) : NULL;
  uint8_t* pcd = keep ? (uint8_t*)malloc((size_t)n) : NULL;
  uint8_t* psi = keep ? (uint8_t*)malloc((size_t)nb) : NULL;
  float* pvv = keep ? (float*)malloc(sizeof(float) * (size_t)ng) : NULL;
  double* psg = keep ? (double*)malloc(sizeof(double) * (size_t)r) : NULL;
  if (keep && (!pL1 || !pL2 || !pQ || !pcd || !psi || !pvv || !psg)) return OQ_ERR;
  double prev = INFINITY, eps = INFINITY;
  int t = 0, rc = OQ_OK;
  for (t = 1; t <= iters; ++t) {
    if (keep && t > 1) {
      memcpy(pL1, L1, sizeof(float) * (size_t)d * r); memcpy(pL2, L2, sizeof(float) * (size_t)r * k);
      memcpy(pQ, Q, sizeof(float) * (size_t)n); memcpy(pcd, cd, (size_t)n); memcpy(psi, si, (size_t)nb);
      memcpy(pvv, vv, sizeof(float) * (size_t)ng);
      if (sigma) memcpy(psg, sigma, sizeof(double) * (size_t)r);
    }
    rc = oq_lq_iteration(W, d, k, r, c, row_w, col_w, Q, A, T, L1, L2, cd, si, vv, sigma, &eps);
    if (rc != OQ_OK) break;
    if (trace) trace[t - 1] = eps;
    if (early_stop && eps > prev) {
      if (keep) {           /* hand back iterate t - 1 */
        memcpy(L1, pL1, sizeof(float) * (size_t)d * r); memcpy(L2, pL2, sizeof(float) * (size_t)r * k);
        memcpy(Q, pQ, sizeof(float) * (size_t)n); memcpy(cd, pcd, (size_t)n); memcpy(si, psi, (size_t)nb);
        memcpy(vv, pvv, sizeof(float) * (size_t)ng);
        if (sigma) memcpy(sigma, psg, sizeof(double) * (size_t)r);
        eps = prev;
      }
      ++t;
      break;
    }
    prev = eps;
  }
  free(pL1); free(pL2); free(pQ); free(pcd); free(psi); free(pvv); free(psg);
  if (iters_done) *iters_done = t - 1;
  if (err) *err = eps;
  if (codes) memcpy(codes, cd, (size_t)n);
  if (scale_idx) memcpy(scale_idx, si, (size_t)nb);
  if (v) memcpy(v, vv, sizeof(float) * (size_t)ng);
  if (Qd) memcpy(Qd, Q, sizeof(float) * (size_t)n);
  free(Q); free(A); free(T); free(cd); free(si); free(vv);
  return rc;
}

/* Algorithm 2 as printed: Q(0) = 0. */
int oq_lq(const float* W, int d, int k, int r, oq_config c, int iters, int early_stop,
          const float* row_w, const float* col_w, float* L1, float* L2, uint8_t* codes,
          uint8_t* scale_idx, float* v, float* Qd, double* err, double* trace, int32_t* iters_done,
          double* sigma) {
  return oq_lq_init(W, d, k, r, c, iters, early_stop, row_w, col_w, L1, L2, codes, scale_idx, v, Qd, err, trace, iters_done, sigma, 0);
}

/* Inner loops of GetConfig (Algorithm 3): E[c] = eps^2, S[c] = storage(W, c) for every config. */
int oq_error_table(const float* W, int d, int k, int r, const oq_config* cfgs, int n_cfgs, int iters,
                   int early_stop, const float* row_w, const float* col_w, double* err_sq,
                   double* storage_bits) {
  float* L1 = (float*)malloc(sizeof(float) * (size_t)d * r);
  float* L2 = (float*)malloc(sizeof(float) * (size_t)r * k);
  if (!L1 || !L2) return OQ_ERR;
  int rc = OQ_OK;
  for (int ci = 0; ci < n_cfgs && rc == OQ_OK; ++ci) {
    double eps = 0.0;
    rc = oq_lq(W, d, k, r, cfgs[ci], iters, early_stop, row_w, col_w, L1, L2, NULL, NULL, NULL, NULL,
               &eps, NULL, NULL, NULL);
    err_sq[ci] = eps * eps;
    storage_bits[ci] = oq_storage_bits((int64_t)d * k, cfgs[ci]);
  }
  free(L1); free(L2);
  return rc;
}

/* RowAverage / ColAverage of sqrt(F)  (Section 3.3; Algorithm 4): D_row = diag(row means of
 * sqrt F), D_col = diag(column means of sqrt F).
 * reading: the vectors handed to the decomposition are on the Fisher scale, row_w = a^2 and
 * col_w = (b / mean(sqrt F))^2 with a, b the row / column means, so that row_w[i]*col_w[j]
 * reproduces F exactly when F has rank one (the identity of Section 3.3 drops this constant; it
 * changes the error's scale, not the minimiser). */
void oq_fisher_row_col(const double* F, int d, int k, float* row_w, float* col_w) {
  double* a = (double*)calloc((size_t)d, sizeof(double));
  double* b = (double*)calloc((size_t)k, sizeof(double));
  double total = 0.0;
  for (int i = 0; i < d; ++i)
    for (int j = 0; j < k; ++j) {
      double s = sqrt(F[(size_t)i * k + j]);
      a[i] += s; b[j] += s; total += s;
    }
  double mean = total / ((double)d * (double)k);
  for (int i = 0; i < d; ++i) { double ai = a[i] / k; row_w[i] = (float)(ai * ai); }
  for (int j = 0; j < k; ++j) { double bj = b[j] / d / mean; col_w[j] = (float)(bj * bj); }
  free(a); free(b);
}
