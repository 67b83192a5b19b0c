// Small dense kernels of the randomized SVD: Gram matrices in fp64, Cholesky-QR orthonormalisation,
// the l x l symmetric eigenproblem of the Rayleigh-Ritz step (parallel Jacobi), sketch generation and
// factor assembly (Algorithm 4).  These run on the ALUs with their working set in LDS when it fits;
// they are latency-, not throughput-critical, and batched over the configurations of a sweep.
#include <cmath>

#include "kernels.h"

namespace lq {

// ------------------------------------------------------------------------------------------------
// Gram matrix: one workgroup per (column chunk, 32x32 output block, problem).  Inputs are fp32, products
// and sums fp64 (the Gram matrix of a basis whose singular values span two decades loses what the SVD
// tolerance needs if it is accumulated in fp32).
__global__ __launch_bounds__(256) void gram_partial_kernel(const float* __restrict__ X, int l, int64_t m, int64_t ldx,
                                                           size_t strideX, int64_t cols_per_chunk,
                                                           double* __restrict__ part) {
  __shared__ float xa[32][33];
  __shared__ float xb[32][33];
  const int chunk = blockIdx.x, nblk = l / 32;
  const int bi = blockIdx.y / nblk, bj = blockIdx.y % nblk;
  const int z = blockIdx.z;
  const float* Xz = X + (size_t)z * strideX;
  const int tid = threadIdx.x, ty = tid >> 4, tx = tid & 15;
  const int64_t c0 = (int64_t)chunk * cols_per_chunk;
  const int64_t c1 = c0 + cols_per_chunk < m ? c0 + cols_per_chunk : m;
  double acc00 = 0, acc01 = 0, acc10 = 0, acc11 = 0;
  for (int64_t cb = c0; cb < c1; cb += 32) {
    __syncthreads();
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int idx = tid + q * 256;
      const int r = idx >> 5, cc = idx & 31;
      const int64_t col = cb + cc;
      const bool ok = col < c1;
      xa[r][cc] = ok ? Xz[(size_t)(32 * bi + r) * ldx + col] : 0.0f;
      xb[r][cc] = ok ? Xz[(size_t)(32 * bj + r) * ldx + col] : 0.0f;
    }
    __syncthreads();
#pragma unroll 8
    for (int cc = 0; cc < 32; ++cc) {
      const double a0 = xa[ty][cc], a1 = xa[ty + 16][cc], b0 = xb[tx][cc], b1 = xb[tx + 16][cc];
      acc00 = fma(a0, b0, acc00); acc01 = fma(a0, b1, acc01);
      acc10 = fma(a1, b0, acc10); acc11 = fma(a1, b1, acc11);
    }
  }
  double* P = part + ((size_t)z * GRAM_CHUNKS + chunk) * (size_t)l * l;
  const int r0 = 32 * bi + ty, q0 = 32 * bj + tx;
  P[(size_t)r0 * l + q0] = acc00; P[(size_t)r0 * l + q0 + 16] = acc01;
  P[(size_t)(r0 + 16) * l + q0] = acc10; P[(size_t)(r0 + 16) * l + q0 + 16] = acc11;
}

__global__ __launch_bounds__(256) void gram_reduce_kernel(const double* __restrict__ part, double* __restrict__ G,
                                                          int ll) {
  const int z = blockIdx.y;
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= ll) return;
  const double* P = part + (size_t)z * GRAM_CHUNKS * ll;
  double s = 0;
  for (int c = 0; c < GRAM_CHUNKS; ++c) s += P[(size_t)c * ll + i];
  G[(size_t)z * ll + i] = s;
}

int launch_gram(const float* X, int l, int64_t m, int64_t ldx, size_t strideX, double* part, double* G, int batch,
                hipStream_t st) {
  int64_t cpc = (m + GRAM_CHUNKS - 1) / GRAM_CHUNKS;
  cpc = (cpc + 31) / 32 * 32;
  const int nblk = l / 32;
  hipLaunchKernelGGL(gram_partial_kernel, dim3(GRAM_CHUNKS, nblk * nblk, batch), dim3(256), 0, st, X, l, m, ldx,
                     strideX, cpc, part);
  LQ_HIP_TRY(hipGetLastError());
  hipLaunchKernelGGL(gram_reduce_kernel, dim3((l * l + 255) / 256, batch), dim3(256), 0, st, (const double*)part, G,
                     l * l);
  LQ_HIP_TRY(hipGetLastError());
  return LQ_OK;
}

// ------------------------------------------------------------------------------------------------
// Cholesky, right-looking, one workgroup per problem.  PACKED: the lower triangle is worked on in LDS
// (row-packed); otherwise in place in global memory.
template <bool PACKED>
__global__ __launch_bounds__(256) void cholesky_kernel(double* __restrict__ Gall, int l) {
  extern __shared__ double lds[];
  __shared__ double s_inv;
  __shared__ double s_tol;
  double* G = Gall + (size_t)blockIdx.x * l * l;
  const int tid = threadIdx.x, ty = tid >> 4, tx = tid & 15;
  double* Lw = PACKED ? lds : G;
  auto at = [&](int i, int j) -> double& { return PACKED ? Lw[(size_t)i * (i + 1) / 2 + j] : Lw[(size_t)i * l + j]; };
  if (PACKED) {
    for (int idx = tid; idx < l * l; idx += 256) {
      const int i = idx / l, j = idx % l;
      if (j <= i) at(i, j) = G[idx];
    }
  }
  if (tid == 0) {
    double mx = 0;
    for (int i = 0; i < l; ++i) mx = fmax(mx, G[(size_t)i * l + i]);
    s_tol = 1e-12 * mx;
  }
  for (int j = 0; j < l; ++j) {
    __syncthreads();
    const double piv = at(j, j);
    const bool ok = piv > s_tol;
    const double cjj = ok ? sqrt(piv) : 0.0;
    const double inv = ok ? 1.0 / cjj : 0.0;
    for (int i = j + 1 + tid; i < l; i += 256) at(i, j) *= inv;
    __syncthreads();
    if (tid == 0) at(j, j) = cjj;
    for (int i = j + 1 + ty; i < l; i += 16) {
      const double cij = at(i, j);
      for (int kk = j + 1 + tx; kk <= i; kk += 16) at(i, kk) -= cij * at(kk, j);
    }
  }
  __syncthreads();
  if (PACKED) {
    for (int idx = tid; idx < l * l; idx += 256) {
      const int i = idx / l, j = idx % l;
      if (j <= i) G[idx] = at(i, j);
    }
  }
  (void)s_inv;
}

static size_t g_max_lds = 0;
static size_t max_lds_bytes() {
  if (g_max_lds == 0) {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) == hipSuccess && v > 0)
      g_max_lds = (size_t)v;
    else
      g_max_lds = 65536;
  }
  return g_max_lds;
}
size_t lds_limit_for_tests() { return max_lds_bytes(); }

int launch_cholesky(double* G, int l, int batch, hipStream_t st) {
  const size_t need = (size_t)l * (l + 1) / 2 * sizeof(double);
  if (need + 64 <= 65536 && need + 64 <= max_lds_bytes())
    hipLaunchKernelGGL(cholesky_kernel<true>, dim3(batch), dim3(256), need, st, G, l);
  else
    hipLaunchKernelGGL(cholesky_kernel<false>, dim3(batch), dim3(256), 0, st, G, l);
  LQ_HIP_TRY(hipGetLastError());
  return LQ_OK;
}

// ------------------------------------------------------------------------------------------------
// Forward substitution X <- C^-1 X, one lane per column of X, the column kept in LDS.
__global__ __launch_bounds__(64) void trsm_kernel(const double* __restrict__ Call, int l, float* __restrict__ Xall,
                                                  int64_t m, int64_t ldx, size_t strideX) {
  extern __shared__ float ys[];   // [l][64]
  const int z = blockIdx.y, lane = threadIdx.x;
  const double* __restrict__ Cf = Call + (size_t)z * l * l;
  float* X = Xall + (size_t)z * strideX;
  const int64_t col = (int64_t)blockIdx.x * 64 + lane;
  const bool live = col < m;
  for (int i = 0; i < l; ++i) {
    float acc = live ? X[(size_t)i * ldx + col] : 0.0f;
    const double* __restrict__ crow = Cf + (size_t)i * l;
    for (int kk = 0; kk < i; ++kk) acc = fmaf(-(float)crow[kk], ys[kk * 64 + lane], acc);
    const double cii = crow[i];
    const float y = cii > 0.0 ? acc / (float)cii : 0.0f;
    ys[i * 64 + lane] = y;
    if (live) X[(size_t)i * ldx + col] = y;
  }
}

int launch_trsm(const double* Cfac, int l, float* X, int64_t m, int64_t ldx, size_t strideX, int batch,
                hipStream_t st) {
  hipLaunchKernelGGL(trsm_kernel, dim3((unsigned)((m + 63) / 64), batch), dim3(64), (size_t)l * 64 * sizeof(float), st,
                     Cfac, l, X, m, ldx, strideX);
  LQ_HIP_TRY(hipGetLastError());
  return LQ_OK;
}

// ------------------------------------------------------------------------------------------------
// Symmetric eigen-decomposition, two-sided Jacobi with a round-robin ordering: every round applies
// l/2 disjoint rotations at once, M <- J^T M J as independent 2x2 blocks, Vt <- J^T Vt as row pairs.
constexpr int JT = 512;

__device__ inline void rr_pair(int a, int round, int n, int& p, int& q) {
  if (a == 0) { p = n - 1; q = round; }
  else { p = (round + a) % (n - 1); q = (round - a + (n - 1)) % (n - 1); }
  if (p > q) { const int t = p; p = q; q = t; }
}

template <bool INLDS>
__global__ __launch_bounds__(JT) void jacobi_eig_kernel(double* __restrict__ Gall, int l, double* __restrict__ Vall,
                                                        float* __restrict__ Utall, double* __restrict__ lamall) {
  extern __shared__ double lds[];
  __shared__ double s_c[128], s_s[128];
  __shared__ int s_p[128], s_q[128];
  __shared__ int s_rot;
  const int z = blockIdx.x, tid = threadIdx.x;
  double* G = Gall + (size_t)z * l * l;
  double* Vt = Vall + (size_t)z * l * l;
  double* M = INLDS ? lds : G;
  const int ll = l * l, half = l / 2;
  for (int idx = tid; idx < ll; idx += JT) {
    if (INLDS) M[idx] = G[idx];
    Vt[idx] = (idx / l == idx % l) ? 1.0 : 0.0;
  }
  __syncthreads();
  for (int sweep = 0; sweep < 40; ++sweep) {
    if (tid == 0) s_rot = 0;
    __syncthreads();
    for (int round = 0; round < l - 1; ++round) {
      if (tid < half) {
        int p, q;
        rr_pair(tid, round, l, p, q);
        const double mpp = M[(size_t)p * l + p], mqq = M[(size_t)q * l + q], mpq = M[(size_t)p * l + q];
        double c = 1.0, s = 0.0;
        if (mpq != 0.0 && fabs(mpq) > 1e-11 * sqrt(fabs(mpp * mqq))) {
          const double tau = (mqq - mpp) / (2.0 * mpq);
          const double t = (tau >= 0 ? 1.0 : -1.0) / (fabs(tau) + sqrt(1.0 + tau * tau));
          c = 1.0 / sqrt(1.0 + t * t);
          s = t * c;
          s_rot = 1;
        }
        s_c[tid] = c; s_s[tid] = s; s_p[tid] = p; s_q[tid] = q;
      }
      __syncthreads();
      // M <- J^T M J, block (a, b): rows (p,q) of pair a, columns (p2,q2) of pair b
      for (int blk = tid; blk < half * half; blk += JT) {
        const int a = blk / half, b = blk % half;
        const double c1 = s_c[a], s1 = s_s[a], c2 = s_c[b], s2 = s_s[b];
        if (s1 == 0.0 && s2 == 0.0) continue;
        const int p = s_p[a], q = s_q[a], p2 = s_p[b], q2 = s_q[b];
        const double m00 = M[(size_t)p * l + p2], m01 = M[(size_t)p * l + q2];
        const double m10 = M[(size_t)q * l + p2], m11 = M[(size_t)q * l + q2];
        const double r00 = c1 * m00 - s1 * m10, r01 = c1 * m01 - s1 * m11;   // rows: J^T from the left
        const double r10 = s1 * m00 + c1 * m10, r11 = s1 * m01 + c1 * m11;
        M[(size_t)p * l + p2] = c2 * r00 - s2 * r01; M[(size_t)p * l + q2] = s2 * r00 + c2 * r01;
        M[(size_t)q * l + p2] = c2 * r10 - s2 * r11; M[(size_t)q * l + q2] = s2 * r10 + c2 * r11;
      }
      // Vt <- J^T Vt
      for (int it = tid; it < half * l; it += JT) {
        const int a = it / l, col = it % l;
        const double c1 = s_c[a], s1 = s_s[a];
        if (s1 == 0.0) continue;
        const int p = s_p[a], q = s_q[a];
        const double vp = Vt[(size_t)p * l + col], vq = Vt[(size_t)q * l + col];
        Vt[(size_t)p * l + col] = c1 * vp - s1 * vq;
        Vt[(size_t)q * l + col] = s1 * vp + c1 * vq;
      }
      __syncthreads();
    }
    if (s_rot == 0) break;   // every thread reads the flag after the round's closing barrier
    __syncthreads();
  }
  // descending sort by rank counting, then emit fp32 eigenvectors as rows
  __shared__ int s_rank[256];
  for (int i = tid; i < l; i += JT) {
    const double li = M[(size_t)i * l + i];
    int r = 0;
    for (int j = 0; j < l; ++j) {
      const double lj = M[(size_t)j * l + j];
      r += (lj > li || (lj == li && j < i)) ? 1 : 0;
    }
    s_rank[i] = r;
    lamall[(size_t)z * l + r] = li > 0.0 ? li : 0.0;
  }
  __syncthreads();
  float* Ut = Utall + (size_t)z * l * l;
  for (int idx = tid; idx < ll; idx += JT) {
    const int i = idx / l, col = idx % l;
    Ut[(size_t)s_rank[i] * l + col] = (float)Vt[idx];
  }
}

int launch_jacobi_eig(double* G, int l, double* vt, float* Ut, double* lambda, int batch, hipStream_t st) {
  if (l > 256) return LQ_ERR_ARG;
  const size_t need = (size_t)l * l * sizeof(double);
  if (need + 4096 <= 65536 && need + 4096 <= max_lds_bytes())
    hipLaunchKernelGGL(jacobi_eig_kernel<true>, dim3(batch), dim3(JT), need, st, G, l, vt, Ut, lambda);
  else
    hipLaunchKernelGGL(jacobi_eig_kernel<false>, dim3(batch), dim3(JT), 0, st, G, l, vt, Ut, lambda);
  LQ_HIP_TRY(hipGetLastError());
  return LQ_OK;
}

// ------------------------------------------------------------------------------------------------
__device__ inline uint64_t mix64(uint64_t x) {
  x += 0x9e3779b97f4a7c15ull;
  x = (x ^ (x >> 30)) * 0xbf58476d1ce4e5b9ull;
  x = (x ^ (x >> 27)) * 0x94d049bb133111ebull;
  return x ^ (x >> 31);
}

__global__ __launch_bounds__(256) void gaussian_fill_kernel(float* __restrict__ X, int l, int64_t m, int64_t ldx,
                                                            uint64_t seed) {
  const int64_t total = (int64_t)l * ldx;
  for (int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * 256) {
    const int64_t row = idx / ldx, col = idx % ldx;
    float val = 0.0f;
    if (col < m) {
      const uint64_t h = mix64(mix64(seed) ^ (uint64_t)(row * m + col));
      const float u1 = ((float)(uint32_t)(h >> 40) + 0.5f) * (1.0f / 16777216.0f);   // (0,1)
      const float u2 = ((float)(uint32_t)((h >> 8) & 0xffffffu)) * (1.0f / 16777216.0f);
      val = sqrtf(-2.0f * logf(u1)) * cosf(6.28318530717958647692f * u2);
    }
    X[idx] = val;
  }
}

int launch_gaussian_fill(float* X, int l, int64_t m, int64_t ldx, uint64_t seed, hipStream_t st) {
  const int64_t total = (int64_t)l * ldx;
  const int64_t want = (total + 255) / 256;
  hipLaunchKernelGGL(gaussian_fill_kernel, dim3((unsigned)(want < 4096 ? want : 4096)), dim3(256), 0, st, X, l, m, ldx,
                     seed);
  LQ_HIP_TRY(hipGetLastError());
  return LQ_OK;
}

__global__ __launch_bounds__(256) void scale_matrix_kernel(const float* __restrict__ A, int64_t d, int64_t k,
                                                           const float* __restrict__ sr,
                                                           const float* __restrict__ sc, float* __restrict__ out) {
  const int64_t total = d * k;
  for (int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * 256) {
    const int64_t i = idx / k, j = idx % k;
    out[idx] = sr[i] * A[idx] * sc[j];
  }
}

int launch_scale_matrix(const float* A, int64_t d, int64_t k, const float* sr, const float* sc, float* out,
                        hipStream_t st) {
  const int64_t want = (d * k + 255) / 256;
  hipLaunchKernelGGL(scale_matrix_kernel, dim3((unsigned)(want < 8192 ? want : 8192)), dim3(256), 0, st, A, d, k,
                     sr, sc, out);
  LQ_HIP_TRY(hipGetLastError());
  return LQ_OK;
}

__global__ void sqrt_vecs_kernel(const float* __restrict__ w, int64_t n, float* __restrict__ s, float* __restrict__ rs) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) {
    const float r = sqrtf(w[i]);
    s[i] = r;
    rs[i] = 1.0f / r;
  }
}

int launch_sqrt_vecs(const float* w, int64_t n, float* s, float* rs, hipStream_t st) {
  hipLaunchKernelGGL(sqrt_vecs_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, w, n, s, rs);
  LQ_HIP_TRY(hipGetLastError());
  return LQ_OK;
}

// L1 (d x rank) and L2 (rank x k) from the Ritz-ordered bases.
__global__ __launch_bounds__(256) void assemble_factors_kernel(const float* __restrict__ Y, int64_t ldy,
                                                               const float* __restrict__ B, int64_t ldb,
                                                               const double* __restrict__ lambda, int rank, int64_t d,
                                                               int64_t k, const float* __restrict__ rsr,
                                                               const float* __restrict__ rsc, float* __restrict__ L1,
                                                               float* __restrict__ L2) {
  const int64_t n1 = d * rank, n2 = (int64_t)rank * k;
  for (int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x; idx < n1 + n2; idx += (int64_t)gridDim.x * 256) {
    if (idx < n1) {
      const int64_t i = idx / rank;
      const int p = (int)(idx % rank);
      const float rs = (float)sqrt(sqrt(lambda[p]));           // sqrt(sigma)
      float val = Y[(size_t)p * ldy + i] * rs;
      if (rsr) val *= rsr[i];
      L1[idx] = val;
    } else {
      const int64_t e = idx - n1;
      const int p = (int)(e / k);
      const int64_t j = e % k;
      const double sg = sqrt(lambda[p]);
      const float inv = sg > 0.0 ? (float)(1.0 / sqrt(sg)) : 0.0f;
      float val = B[(size_t)p * ldb + j] * inv;
      if (rsc) val *= rsc[j];
      L2[e] = val;
    }
  }
}

int launch_assemble_factors(const float* Y, int64_t ldy, const float* B, int64_t ldb, const double* lambda, int rank,
                            int64_t d, int64_t k, const float* rsr, const float* rsc, float* L1, float* L2,
                            hipStream_t st) {
  const int64_t want = ((d + k) * rank + 255) / 256;
  hipLaunchKernelGGL(assemble_factors_kernel, dim3((unsigned)(want < 4096 ? want : 4096)), dim3(256), 0, st, Y, ldy, B,
                     ldb, lambda, rank, d, k, rsr, rsc, L1, L2);
  LQ_HIP_TRY(hipGetLastError());
  return LQ_OK;
}

}  // namespace lq
