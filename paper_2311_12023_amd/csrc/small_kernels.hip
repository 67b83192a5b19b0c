// Small dense kernels of the randomized SVD: Gram matrices in fp64, Cholesky-QR orthonormalisation,
// the l x l symmetric eigenproblem of the Rayleigh-Ritz step (parallel Jacobi), sketch generation and
// factor assembly (Algorithm 4).  These run on the ALUs with their working set in LDS when it fits;
// they are latency-, not throughput-critical, and batched over the configurations of a sweep.
#include <cmath>

#include "kernels.h"
#include "profiler.h"

namespace lq {

// ------------------------------------------------------------------------------------------------
// Gram matrix: one workgroup per (column chunk, 32x32 output block of the lower triangle, problem).  Inputs are
// fp32, products and sums fp64 (the Gram matrix of a basis whose singular values span two decades loses what the
// SVD tolerance needs if it is accumulated in fp32), which makes the kernel fp64-FMA bound: only the blocks on and
// below the diagonal are computed and gram_reduce_kernel mirrors them.
__global__ __launch_bounds__(256) void gram_partial_kernel(const float* __restrict__ X, int l, int64_t m, int64_t ldx,
                                                           size_t strideX, int64_t cols_per_chunk,
                                                           double* __restrict__ part) {
  __shared__ float xa[32][33];
  __shared__ float xb[32][33];
  const int chunk = blockIdx.x;
  int bi = 0, bj = blockIdx.y;                    // blockIdx.y enumerates the pairs bj <= bi row by row
  while (bj > bi) { bj -= bi + 1; ++bi; }
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
                                                          int l) {
  const int z = blockIdx.y, ll = l * l;
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= ll) return;
  const int r = i / l, q = i - r * l;
  const int src = (r >> 5) >= (q >> 5) ? i : q * l + r;       // blocks above the diagonal: the transposed entry
  const double* P = part + (size_t)z * GRAM_CHUNKS * ll;
  double s = 0;
  for (int c = 0; c < GRAM_CHUNKS; ++c) s += P[(size_t)c * ll + src];
  G[(size_t)z * ll + i] = s;
}

int launch_gram(const float* X, int l, int64_t m, int64_t ldx, size_t strideX, double* part, double* G, int batch,
                hipStream_t st) {
  int64_t cpc = (m + GRAM_CHUNKS - 1) / GRAM_CHUNKS;
  cpc = (cpc + 31) / 32 * 32;
  const int nblk = l / 32;
  prof::Scope ps(prof::GRAM, st, (double)l * m * 4.0 * batch);
  hipLaunchKernelGGL(gram_partial_kernel, dim3(GRAM_CHUNKS, nblk * (nblk + 1) / 2, batch), dim3(256), 0, st, X, l, m, ldx,
                     strideX, cpc, part);
  LQ_HIP_TRY(hipGetLastError());
  hipLaunchKernelGGL(gram_reduce_kernel, dim3((l * l + 255) / 256, batch), dim3(256), 0, st, (const double*)part, G,
                     l);
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
  // A pivot is compared with the row's own squared norm (what is left of row j after the rows before it have been
  // taken out is negligible below 1e-6 of its length), not with the largest one: the rows of a block may differ in
  // length by many orders of magnitude (filtered rows beside rows kept at unit length).
  __shared__ double s_diag[256];
  for (int i = tid; i < l; i += 256) s_diag[i] = G[(size_t)i * l + i];
  for (int j = 0; j < l; ++j) {
    __syncthreads();
    const double piv = at(j, j);
    const bool ok = piv > 1e-12 * s_diag[j];
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
  prof::Scope ps(prof::CHOLESKY, st, (double)l * l * 8.0 * batch);
  if (need + 64 <= 65536 && need + 64 <= max_lds_bytes())
    hipLaunchKernelGGL(cholesky_kernel<true>, dim3(batch), dim3(256), need, st, G, l);
  else
    hipLaunchKernelGGL(cholesky_kernel<false>, dim3(batch), dim3(256), 0, st, G, l);
  LQ_HIP_TRY(hipGetLastError());
  return LQ_OK;
}

// ------------------------------------------------------------------------------------------------
// Cholesky factor and its inverse in one kernel (l = 32*NB <= 128), fp64.  G = C C^T; out = C^-1 as a
// dense fp32 l x l matrix (zeros above the diagonal) that the MFMA GEMM then applies to the basis.
// 1024 threads form a 32 x 32 grid; thread (ty, tx) keeps the elements (i, k) with i = ty (mod 32),
// k = tx (mod 32) of both the matrix being factored and the inverse being built in registers.
// Right-looking: step j broadcasts column j of the matrix and row j of the inverse through LDS
// (double-buffered, one barrier per step) and every thread updates its own elements:
//   a(i,k) -= c_ij c_kj,   T(i,k) -= c_ij T(j,k)   (Gauss-Jordan on [C | I]).
// A non-positive pivot (dependent direction) zeroes that row of C^-1, which removes the direction.
// 1 / sqrt(x) for positive finite x: fp32 seed on the mantissa (so that the seed exists whatever the magnitude of x),
// three Newton steps in fp64, exponent put back.
__device__ inline double fast_rsqrt(double x) {
  int e;
  double m = frexp(x, &e);                    // x = m 2^e, m in [0.5, 1)
  if (e & 1) { m *= 2.0; e -= 1; }            // even exponent, m in [0.5, 2)
  double r = (double)rsqrtf((float)m);
  r = r * (1.5 - 0.5 * m * r * r);
  r = r * (1.5 - 0.5 * m * r * r);
  r = r * (1.5 - 0.5 * m * r * r);
  return ldexp(r, -(e / 2));
}

template <int NB>
__global__ __launch_bounds__(1024) void cholinv_kernel(const double* __restrict__ Gall, float* __restrict__ Cinvall) {
  constexpr int l = 32 * NB;
  __shared__ double colbuf[2][l];
  __shared__ double rowbuf[2][l];
  const int tid = threadIdx.x, ty = tid >> 5, tx = tid & 31;
  const double* G = Gall + (size_t)blockIdx.x * l * l;
  double a[NB][NB], t[NB][NB];
#pragma unroll
  for (int ei = 0; ei < NB; ++ei)
#pragma unroll
    for (int ek = 0; ek < NB; ++ek) {
      const int i = ty + 32 * ei, k = tx + 32 * ek;
      a[ei][ek] = G[(size_t)i * l + k];
      t[ei][ek] = (i == k) ? 1.0 : 0.0;
    }
  // A pivot is compared with the row's own squared norm, not with the largest one (see cholesky_kernel).
  __shared__ double s_diag[l];
  if (ty == tx) {
#pragma unroll
    for (int e = 0; e < NB; ++e) s_diag[ty + 32 * e] = a[e][e];
  }
  __syncthreads();

#pragma unroll
  for (int jb = 0; jb < NB; ++jb) {
    for (int jt = 0; jt < 32; ++jt) {
      const int j = 32 * jb + jt, buf = j & 1;
      if (tx == jt) {
#pragma unroll
        for (int ei = 0; ei < NB; ++ei) colbuf[buf][ty + 32 * ei] = a[ei][jb];
      }
      if (ty == jt) {
#pragma unroll
        for (int ek = 0; ek < NB; ++ek) rowbuf[buf][tx + 32 * ek] = t[jb][ek];
      }
      __syncthreads();
      const double piv = colbuf[buf][j];
      const bool ok = piv > 1e-12 * s_diag[j];
      const double inv = ok ? fast_rsqrt(piv) : 0.0;
      double ci[NB], ck[NB], tr[NB];
#pragma unroll
      for (int e = 0; e < NB; ++e) {
        const int i = ty + 32 * e, k = tx + 32 * e;
        ci[e] = i > j ? colbuf[buf][i] * inv : 0.0;      // c_ij for this thread's rows
        ck[e] = k > j ? colbuf[buf][k] * inv : 0.0;      // c_kj for this thread's columns
        tr[e] = k <= j ? rowbuf[buf][k] * inv : 0.0;     // scaled row j of the inverse
      }
      // only row blocks that reach below row j change; the matrix part needs columns > j, the inverse part
      // columns <= j (uniform conditions: whole 32-wide blocks are skipped)
#pragma unroll
      for (int ei = 0; ei < NB; ++ei) {
        if (32 * ei + 31 <= j) continue;
#pragma unroll
        for (int ek = 0; ek < NB; ++ek) {
          if (32 * ek + 31 > j) a[ei][ek] = fma(-ci[ei], ck[ek], a[ei][ek]);
          if (32 * ek <= j) t[ei][ek] = fma(-ci[ei], tr[ek], t[ei][ek]);
        }
      }
      if (ty == jt) {
#pragma unroll
        for (int ek = 0; ek < NB; ++ek) t[jb][ek] = tr[ek];
      }
    }
  }
  float* out = Cinvall + (size_t)blockIdx.x * l * l;
#pragma unroll
  for (int ei = 0; ei < NB; ++ei)
#pragma unroll
    for (int ek = 0; ek < NB; ++ek) {
      const int i = ty + 32 * ei, k = tx + 32 * ek;
      out[(size_t)i * l + k] = k <= i ? (float)t[ei][ek] : 0.0f;
    }
}

bool cholinv_supported(int l) { return l % 32 == 0 && l >= 32 && l <= 128; }

int launch_cholinv(const double* G, int l, float* Cinv, int batch, hipStream_t st) {
  prof::Scope ps(prof::CHOLESKY, st, (double)l * l * 12.0 * batch);
  switch (l / 32) {
    case 1: hipLaunchKernelGGL(cholinv_kernel<1>, dim3(batch), dim3(1024), 0, st, G, Cinv); break;
    case 2: hipLaunchKernelGGL(cholinv_kernel<2>, dim3(batch), dim3(1024), 0, st, G, Cinv); break;
    case 3: hipLaunchKernelGGL(cholinv_kernel<3>, dim3(batch), dim3(1024), 0, st, G, Cinv); break;
    case 4: hipLaunchKernelGGL(cholinv_kernel<4>, dim3(batch), dim3(1024), 0, st, G, Cinv); break;
    default: return LQ_ERR_ARG;
  }
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
  prof::Scope ps(prof::TRSM, st, (double)l * m * 8.0 * batch);
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
  // circle method: round < n-1, a < n/2, so both sums stay below 2(n-1) and one conditional subtraction
  // replaces the modulo
  if (a == 0) { p = n - 1; q = round; }
  else {
    p = round + a; if (p >= n - 1) p -= n - 1;
    q = round - a + (n - 1); if (q >= n - 1) q -= n - 1;
  }
  if (p > q) { const int t = p; p = q; q = t; }
}

// STORE: 0 = M and Vt in global memory, 1 = M in LDS, 2 = M and Vt in LDS.
template <int STORE>
__global__ __launch_bounds__(JT) void jacobi_eig_kernel(double* __restrict__ Gall, int l, double* __restrict__ Vall,
                                                        float* __restrict__ Utall, double* __restrict__ lamall) {
  extern __shared__ double lds[];
  __shared__ double s_c[128], s_s[128];
  __shared__ int s_p[128], s_q[128];
  __shared__ int s_rot;
  __shared__ int s_rank[256];
  const int z = blockIdx.x, tid = threadIdx.x;
  double* G = Gall + (size_t)z * l * l;
  const int pm = STORE >= 1 ? l + 1 : l;       // row pitch of M
  const int pv = STORE == 2 ? l + 1 : l;       // row pitch of Vt
  double* M = STORE >= 1 ? lds : G;
  double* Vt = STORE == 2 ? lds + (size_t)l * (l + 1) : Vall + (size_t)z * l * l;
  const int ll = l * l, half = l / 2;
  for (int idx = tid; idx < ll; idx += JT) {
    const int r = idx / l, cidx = idx % l;
    if (STORE >= 1) M[r * pm + cidx] = G[idx];
    Vt[r * pv + cidx] = (r == cidx) ? 1.0 : 0.0;
  }
  __syncthreads();
  for (int sweep = 0; sweep < 40; ++sweep) {
    if (tid == 0) s_rot = 0;
    __syncthreads();
    for (int round = 0; round < l - 1; ++round) {
      if (tid < half) {
        int p, q;
        rr_pair(tid, round, l, p, q);
        const double mpp = M[p * pm + p], mqq = M[q * pm + q], mpq = M[p * pm + q];
        double c = 1.0, s = 0.0;
        if (mpq != 0.0 && fabs(mpq) > 1e-10 * sqrt(fabs(mpp * mqq))) {
          const double tau = (mqq - mpp) / (2.0 * mpq);
          const double t = (tau >= 0 ? 1.0 : -1.0) / (fabs(tau) + sqrt(1.0 + tau * tau));
          c = 1.0 / sqrt(1.0 + t * t);
          s = t * c;
          s_rot = 1;
        }
        s_c[tid] = c; s_s[tid] = s; s_p[tid] = p; s_q[tid] = q;
      }
      __syncthreads();
      // M <- J^T M J on the blocks a <= b (rows of pair a, columns of pair b); the mirror block is written too
      for (int blk = tid; blk < half * half; blk += JT) {
        const int a = blk / half, b = blk % half;
        if (b < a) continue;
        const double c1 = s_c[a], s1 = s_s[a], c2 = s_c[b], s2 = s_s[b];
        if (s1 == 0.0 && s2 == 0.0) continue;
        const int p = s_p[a], q = s_q[a], p2 = s_p[b], q2 = s_q[b];
        const double m00 = M[p * pm + p2], m01 = M[p * pm + q2];
        const double m10 = M[q * pm + p2], m11 = M[q * pm + q2];
        const double r00 = c1 * m00 - s1 * m10, r01 = c1 * m01 - s1 * m11;   // rows: J^T from the left
        const double r10 = s1 * m00 + c1 * m10, r11 = s1 * m01 + c1 * m11;
        const double n00 = c2 * r00 - s2 * r01, n01 = s2 * r00 + c2 * r01;
        const double n10 = c2 * r10 - s2 * r11, n11 = s2 * r10 + c2 * r11;
        M[p * pm + p2] = n00; M[p * pm + q2] = n01; M[q * pm + p2] = n10; M[q * pm + q2] = n11;
        if (a != b) { M[p2 * pm + p] = n00; M[q2 * pm + p] = n01; M[p2 * pm + q] = n10; M[q2 * pm + q] = n11; }
      }
      // Vt <- J^T Vt
      for (int it = tid; it < half * l; it += JT) {
        const int a = it / l, col = it % l;
        const double c1 = s_c[a], s1 = s_s[a];
        if (s1 == 0.0) continue;
        const int p = s_p[a], q = s_q[a];
        const double vp = Vt[p * pv + col], vq = Vt[q * pv + col];
        Vt[p * pv + col] = c1 * vp - s1 * vq;
        Vt[q * pv + col] = s1 * vp + c1 * vq;
      }
      __syncthreads();
    }
    if (s_rot == 0) break;   // every thread reads the flag after the round's closing barrier
    __syncthreads();
  }
  // descending sort by rank counting, then emit fp32 eigenvectors as rows
  for (int i = tid; i < l; i += JT) {
    const double li = M[i * pm + i];
    int r = 0;
    for (int j = 0; j < l; ++j) {
      const double lj = M[j * pm + j];
      r += (lj > li || (lj == li && j < i)) ? 1 : 0;
    }
    s_rank[i] = r;
    lamall[(size_t)z * l + r] = li > 0.0 ? li : 0.0;
  }
  __syncthreads();
  float* Ut = Utall + (size_t)z * l * l;
  for (int idx = tid; idx < ll; idx += JT) {
    const int i = idx / l, col = idx % l;
    Ut[(size_t)s_rank[i] * l + col] = (float)Vt[i * pv + col];
  }
}

// Sum over the LP = 16 lanes of a DPP row, or over its 8-lane halves (quad swaps, then the mirrors); every lane gets the
// total, bit-identical in all of them (each step adds the same two numbers in both lanes); no LDS traffic.
template <int LP>
__device__ __forceinline__ float lanes_sum(float x) {
  x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0xB1, 0xf, 0xf, false));    // quad_perm [1,0,3,2]
  x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x4E, 0xf, 0xf, false));    // quad_perm [2,3,0,1]
  x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x141, 0xf, 0xf, false));   // row_half_mirror
  if constexpr (LP == 16)
    x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x140, 0xf, 0xf, false)); // row_mirror
  return x;
}

// CE consecutive floats between LDS and registers with the widest accesses the chunk allows (16-byte aligned).
template <int CE>
__device__ __forceinline__ void chunk_load(const float* src, float (&v)[CE]) {
  if constexpr (CE % 4 == 0) {
#pragma unroll
    for (int e = 0; e < CE; e += 4) {
      const float4 t = *reinterpret_cast<const float4*>(src + e);
      v[e] = t.x; v[e + 1] = t.y; v[e + 2] = t.z; v[e + 3] = t.w;
    }
  } else {
#pragma unroll
    for (int e = 0; e < CE; e += 2) {
      const float2 t = *reinterpret_cast<const float2*>(src + e);
      v[e] = t.x; v[e + 1] = t.y;
    }
  }
}
template <int CE>
__device__ __forceinline__ void chunk_store(float* dst, const float (&v)[CE]) {
  if constexpr (CE % 4 == 0) {
#pragma unroll
    for (int e = 0; e < CE; e += 4) *reinterpret_cast<float4*>(dst + e) = make_float4(v[e], v[e + 1], v[e + 2], v[e + 3]);
  } else {
#pragma unroll
    for (int e = 0; e < CE; e += 2) *reinterpret_cast<float2*>(dst + e) = make_float2(v[e], v[e + 1]);
  }
}

// One-sided (Hestenes) Jacobi in fp32, everything in LDS (l = 16*NE <= 128).  Works on X = M itself:
// rotating the columns of X = M J until they are mutually orthogonal makes J^T M^2 J diagonal, so J holds
// the eigenvectors of the symmetric M and the column norms are the eigenvalues.  fp32 rotations give
// eigenvectors good to about 1e-6; the Ritz values are not taken from here but recomputed in fp64 from
// the rotated basis (row_sumsq_kernel), which is second-order accurate in the eigenvector error.
// LP lanes per column pair, each lane owning l / LP consecutive entries of both columns (128-bit LDS accesses); a round
// handles l/2 disjoint pairs, one barrier per round.  The squared column norms are kept in LDS and updated with the
// rotation (|x_p|^2 -= t g, |x_q|^2 += t g), so a round computes one inner product instead of three; they are
// recomputed from the columns at the start of every sweep, and they only enter the angle and the skip test (the inner
// product that a rotation annihilates is always computed from the columns themselves).
template <int NE, int LP>
__global__ __launch_bounds__(LP * 8 * NE) void jacobi_onesided_kernel(const double* __restrict__ Gall,
                                                                    float* __restrict__ Utall,
                                                                    double* __restrict__ lamall) {
  constexpr int l = 16 * NE, P = l + 4;     // pitch a multiple of 4: every lane's chunk starts on a 16-byte boundary
  constexpr int CE = l / LP;                // entries of a column per lane
  static_assert(LP == 8 || LP == 16, "a pair's lanes are a DPP row or half of one");
  static_assert(CE % 2 == 0, "chunks move as 64- or 128-bit accesses");
  extern __shared__ __attribute__((aligned(16))) float fl[];   // X[l][P] then V[l][P], column c at row c
  __shared__ int s_rot;
  __shared__ float s_big;
  __shared__ float s_norm[128];
  __shared__ float s_n2[128];
  __shared__ int s_rank[128];
  float* X = fl;
  float* V = fl + l * P;
  const int z = blockIdx.x, tid = threadIdx.x, nthr = LP * l / 2;
  const double* G = Gall + (size_t)z * l * l;
  // M is brought to unit scale by a power of two first: the rotations work with products of four of its entries, which
  // leave the fp32 range for matrices whose singular values are below 1e-5 or above 1e4 otherwise
  __shared__ double s_scale;
  if (tid == 0) {
    double mx = 0.0;
    for (int i = 0; i < l; ++i) mx = fmax(mx, fabs(G[(size_t)i * l + i]));
    s_scale = (mx > 0.0 && mx < 1.0e300) ? ldexp(1.0, -ilogb(mx)) : 1.0;
  }
  __syncthreads();
  const double mscale = s_scale;
  for (int idx = tid; idx < l * l; idx += nthr) {
    const int c = idx / l, i = idx % l;
    X[c * P + i] = (float)(G[idx] * mscale);  // symmetric: row c of M is column c
    V[c * P + i] = (c == i) ? 1.0f : 0.0f;
  }
  const int g = tid / LP, sub = tid % LP;
  const int eo = CE * sub;                    // this lane's entries of a column: eo .. eo + CE - 1
  __syncthreads();
  for (int sweep = 0; sweep < 30; ++sweep) {
    if (tid == 0) { s_rot = 0; s_big = 0.0f; }
    // squared norms of the columns, fresh from the columns: group g takes columns g and g + l/2
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int c = g + h * (l / 2);
      float x[CE];
      chunk_load<CE>(X + c * P + eo, x);
      float n2 = 0.f;
#pragma unroll
      for (int e = 0; e < CE; ++e) n2 = fmaf(x[e], x[e], n2);
      n2 = lanes_sum<LP>(n2);
      if (sub == 0) s_n2[c] = n2;
    }
    __syncthreads();
    float worst = 0.0f;
    bool rotated = false;
    for (int round = 0; round < l - 1; ++round) {
      int p, q;
      rr_pair(g, round, l, p, q);
      float xp[CE], xq[CE], vp[CE], vq[CE];
      chunk_load<CE>(X + p * P + eo, xp);
      chunk_load<CE>(X + q * P + eo, xq);
      const float al = s_n2[p], be = s_n2[q];
      // the eigenvector entries are fetched now, whether or not the pair rotates: their latency passes behind the
      // reduction and the angle
      chunk_load<CE>(V + p * P + eo, vp);
      chunk_load<CE>(V + q * P + eo, vq);
      float ga = 0.f;
#pragma unroll
      for (int e = 0; e < CE; ++e) ga = fmaf(xp[e], xq[e], ga);
      ga = lanes_sum<LP>(ga);
      // hardware reciprocal / square-root approximations (1 ulp) are enough here: a rotation that is orthogonal
      // to 1e-7 and an angle that misses the exact one by 1e-7 change nothing in the convergence, and the
      // eigenvector rows are renormalised at the end
      const float ab = al * be;
      if (ga != 0.0f && ga * ga > 4e-12f * ab) {
        rotated = true;
        worst = fmaxf(worst, fabsf(ga) * __builtin_amdgcn_rsqf(ab));
        const float zeta = (be - al) * 0.5f * __builtin_amdgcn_rcpf(ga);
        const float tt = copysignf(__builtin_amdgcn_rcpf(fabsf(zeta) + __builtin_amdgcn_sqrtf(1.0f + zeta * zeta)), zeta);
        const float cs = __builtin_amdgcn_rsqf(1.0f + tt * tt), sn = cs * tt;
        float np[CE], nq[CE];
#pragma unroll
        for (int e = 0; e < CE; ++e) { np[e] = cs * xp[e] - sn * xq[e]; nq[e] = sn * xp[e] + cs * xq[e]; }
        chunk_store<CE>(X + p * P + eo, np);
        chunk_store<CE>(X + q * P + eo, nq);
#pragma unroll
        for (int e = 0; e < CE; ++e) { np[e] = cs * vp[e] - sn * vq[e]; nq[e] = sn * vp[e] + cs * vq[e]; }
        chunk_store<CE>(V + p * P + eo, np);
        chunk_store<CE>(V + q * P + eo, nq);
        if (sub == 0) {                          // the pairs of a round are disjoint: nobody else touches these two
          s_n2[p] = fmaxf(al - tt * ga, 0.0f);
          s_n2[q] = be + tt * ga;
        }
      }
      __syncthreads();
    }
    if (rotated) { s_rot = 1; }
    if (worst > 1e-4f) s_big = 1.0f;           // benign race: every writer stores the same value
    __syncthreads();
    const bool more = s_rot != 0 && s_big != 0.0f;   // quadratic convergence: a sweep whose worst pair was
    __syncthreads();                                 // below 1e-4 leaves nothing above ~1e-7 behind
    if (!more) break;
  }
  // eigenvalue estimates = column norms; rank them (descending) and emit eigenvectors as rows
  __shared__ float s_vscale[128];
  for (int c = tid; c < l; c += nthr) {
    float n2 = 0.f;
    double v2 = 0.0;
    for (int i = 0; i < l; ++i) {
      n2 = fmaf(X[c * P + i], X[c * P + i], n2);
      const double vv = V[c * P + i];
      v2 = fma(vv, vv, v2);
    }
    s_norm[c] = sqrtf(n2);
    s_vscale[c] = (float)(1.0 / sqrt(v2));    // accumulated rotations drift from unit norm by ~1e-6
  }
  __syncthreads();
  for (int c = tid; c < l; c += nthr) {
    const float li = s_norm[c];
    int r = 0;
    for (int j = 0; j < l; ++j) r += (s_norm[j] > li || (s_norm[j] == li && j < c)) ? 1 : 0;
    s_rank[c] = r;
    lamall[(size_t)z * l + r] = (double)li / mscale;
  }
  __syncthreads();
  float* Ut = Utall + (size_t)z * l * l;
  for (int idx = tid; idx < l * l; idx += nthr) {
    const int c = idx / l, i = idx % l;
    Ut[(size_t)s_rank[c] * l + i] = V[c * P + i] * s_vscale[c];
  }
}

template <int NE, int LP>
static int launch_onesided(const double* G, float* Ut, double* lambda, int batch, hipStream_t st) {
  constexpr int l = 16 * NE;
  const size_t need = (size_t)2 * l * (l + 4) * sizeof(float);
  static bool attr_set = false;
  if (!attr_set) {
    LQ_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(jacobi_onesided_kernel<NE, LP>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)need));
    attr_set = true;
  }
  hipLaunchKernelGGL((jacobi_onesided_kernel<NE, LP>), dim3(batch), dim3(LP * l / 2), need, st, G, Ut, lambda);
  LQ_HIP_TRY(hipGetLastError());
  return LQ_OK;
}

// lam[z][i] = sum_j X[z][i][j]^2 in fp64: the Ritz values sigma_i^2 as the squared row norms of the rotated
// projected matrix.
__global__ __launch_bounds__(256) void row_sumsq_kernel(const float* __restrict__ X, int64_t m, int64_t ldx,
                                                        size_t strideX, int l, double* __restrict__ lam) {
  __shared__ double s_sum[4];
  const int row = blockIdx.x, z = blockIdx.y, tid = threadIdx.x;
  const float* x = X + (size_t)z * strideX + (size_t)row * ldx;
  double s = 0.0;
  for (int64_t j = tid; j < m; j += 256) { const double v = x[j]; s = fma(v, v, s); }
  for (int off = 1; off < 64; off <<= 1) s += __shfl_xor(s, off);
  if ((tid & 63) == 0) s_sum[tid >> 6] = s;
  __syncthreads();
  if (tid == 0) lam[(size_t)z * l + row] = (s_sum[0] + s_sum[1]) + (s_sum[2] + s_sum[3]);
}

// res[i] = |G_i - lam[i] Y_i|^2 for the first `rows` rows: squared residual norms of the Ritz pairs (lam_i, Y_i) of the
// operator that G = Y M was formed with.
__global__ __launch_bounds__(256) void ritz_residual_kernel(const float* __restrict__ G, const float* __restrict__ Y,
                                                            const double* __restrict__ lam, int64_t m, int64_t ldx,
                                                            double* __restrict__ res) {
  __shared__ double s_sum[4];
  const int row = blockIdx.x, tid = threadIdx.x;
  const float* g = G + (size_t)row * ldx;
  const float* y = Y + (size_t)row * ldx;
  const double th = lam[row];
  double s = 0.0;
  for (int64_t j = tid; j < m; j += 256) { const double v = (double)g[j] - th * (double)y[j]; s = fma(v, v, s); }
  for (int off = 1; off < 64; off <<= 1) s += __shfl_xor(s, off);
  if ((tid & 63) == 0) s_sum[tid >> 6] = s;
  __syncthreads();
  if (tid == 0) res[row] = (s_sum[0] + s_sum[1]) + (s_sum[2] + s_sum[3]);
}

int launch_ritz_residual(const float* G, const float* Y, const double* lam, int rows, int64_t m, int64_t ldx, double* res,
                         hipStream_t st) {
  prof::Scope ps(prof::MISC, st, (double)rows * m * 8.0);
  hipLaunchKernelGGL(ritz_residual_kernel, dim3(rows), dim3(256), 0, st, G, Y, lam, m, ldx, res);
  LQ_HIP_TRY(hipGetLastError());
  return LQ_OK;
}

int launch_row_sumsq(const float* X, int l, int64_t m, int64_t ldx, size_t strideX, double* lam, int batch,
                     hipStream_t st) {
  prof::Scope ps(prof::MISC, st, (double)l * m * 4.0 * batch);
  hipLaunchKernelGGL(row_sumsq_kernel, dim3(l, batch), dim3(256), 0, st, X, m, ldx, strideX, l, lam);
  LQ_HIP_TRY(hipGetLastError());
  return LQ_OK;
}

int launch_jacobi_fast(const double* G, int l, float* Ut, double* lambda, int batch, hipStream_t st) {
  prof::Scope ps(prof::JACOBI, st, (double)l * l * 8.0 * batch);
  // 16 lanes per column pair: 8 lanes with twice the entries each measured 30 % slower
  switch (l / 16) {
    case 2: return launch_onesided<2, 16>(G, Ut, lambda, batch, st);
    case 4: return launch_onesided<4, 16>(G, Ut, lambda, batch, st);
    case 6: return launch_onesided<6, 16>(G, Ut, lambda, batch, st);
    case 8: return launch_onesided<8, 16>(G, Ut, lambda, batch, st);
    default: return LQ_ERR_ARG;
  }
}

bool jacobi_fast_supported(int l) { return l % 32 == 0 && l >= 32 && l <= 128; }

int launch_jacobi_eig(double* G, int l, double* vt, float* Ut, double* lambda, int batch, hipStream_t st) {
  if (l > 256 || l % 2) return LQ_ERR_ARG;
  const size_t lim = max_lds_bytes() - 8192;          // static arrays of the kernel
  const size_t one = (size_t)l * (l + 1) * sizeof(double);
  static bool attr_set = false;
  if (!attr_set) {
    LQ_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(jacobi_eig_kernel<1>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lim));
    LQ_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(jacobi_eig_kernel<2>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lim));
    attr_set = true;
  }
  prof::Scope ps(prof::JACOBI, st, (double)l * l * 8.0 * batch);
  if (2 * one <= lim)
    hipLaunchKernelGGL(jacobi_eig_kernel<2>, dim3(batch), dim3(JT), 2 * one, st, G, l, vt, Ut, lambda);
  else if (one <= lim)
    hipLaunchKernelGGL(jacobi_eig_kernel<1>, dim3(batch), dim3(JT), one, st, G, l, vt, Ut, lambda);
  else
    hipLaunchKernelGGL(jacobi_eig_kernel<0>, dim3(batch), dim3(JT), 0, st, G, l, vt, Ut, lambda);
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

// Largest finite |x[i]|: 1024 workgroups leave their maxima in out[0..1023], then one workgroup reduces them into
// out[1024] (two launches; a maximum does not depend on the order it is taken in).
__global__ __launch_bounds__(256) void absmax_kernel(const float* __restrict__ x, int64_t n, float* __restrict__ out,
                                                     int stage) {
  __shared__ float s_max[256];
  const int tid = threadIdx.x;
  float m = 0.0f;
  if (stage == 0) {
    for (int64_t i = (int64_t)blockIdx.x * 256 + tid; i < n; i += (int64_t)gridDim.x * 256) {
      const float a = fabsf(x[i]);
      if (a < __builtin_inff()) m = fmaxf(m, a);     // false for NaN as well
    }
  } else {
    for (int i = tid; i < 1024; i += 256) m = fmaxf(m, out[i]);
  }
  s_max[tid] = m;
  __syncthreads();
  for (int w = 128; w >= 1; w >>= 1) {
    if (tid < w) s_max[tid] = fmaxf(s_max[tid], s_max[tid + w]);
    __syncthreads();
  }
  if (tid == 0) out[stage == 0 ? blockIdx.x : 1024] = s_max[0];
}

int launch_absmax(const float* x, int64_t n, float* out, hipStream_t st) {
  prof::Scope ps(prof::ABSMAX, st, (double)n * 4.0);
  hipLaunchKernelGGL(absmax_kernel, dim3(1024), dim3(256), 0, st, x, n, out, 0);
  LQ_HIP_TRY(hipGetLastError());
  hipLaunchKernelGGL(absmax_kernel, dim3(1), dim3(256), 0, st, x, n, out, 1);
  LQ_HIP_TRY(hipGetLastError());
  return LQ_OK;
}

// X <- a X + b Y + c Z over `count` floats (count a multiple of 4; Z may be NULL: no third term).
__global__ __launch_bounds__(256) void lincomb3_kernel(float* __restrict__ X, float a, const float* __restrict__ Y, float b,
                                                       const float* __restrict__ Z, float c, int64_t count4) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < count4; i += (int64_t)gridDim.x * 256) {
    float4 x = reinterpret_cast<float4*>(X)[i];
    const float4 y = reinterpret_cast<const float4*>(Y)[i];
    x.x = fmaf(a, x.x, b * y.x); x.y = fmaf(a, x.y, b * y.y); x.z = fmaf(a, x.z, b * y.z); x.w = fmaf(a, x.w, b * y.w);
    if (Z != nullptr) {
      const float4 z = reinterpret_cast<const float4*>(Z)[i];
      x.x = fmaf(c, z.x, x.x); x.y = fmaf(c, z.y, x.y); x.z = fmaf(c, z.z, x.z); x.w = fmaf(c, z.w, x.w);
    }
    reinterpret_cast<float4*>(X)[i] = x;
  }
}

int launch_lincomb3(float* X, float a, const float* Y, float b, const float* Z, float c, int64_t count, hipStream_t st) {
  const int64_t count4 = count / 4;
  const int64_t want = (count4 + 255) / 256;
  prof::Scope ps(prof::MISC, st, (double)count * (Z ? 16.0 : 12.0));
  hipLaunchKernelGGL(lincomb3_kernel, dim3((unsigned)(want < 2048 ? want : 2048)), dim3(256), 0, st, X, a, Y, b, Z, c, count4);
  LQ_HIP_TRY(hipGetLastError());
  return LQ_OK;
}

// Rows of X against the first `locked` rows of L (orthonormal): rows i >= locked lose their components along them,
// x_i <- x_i - sum_o (x_i . l_o) l_o; rows i < locked become copies of l_i.  One workgroup per row; inner products in
// fp32 with a fixed summation order.  locked <= DEFLATE_MAX.
constexpr int DEFLATE_MAX = 16;

__global__ __launch_bounds__(256) void deflate_rows_kernel(float* __restrict__ X, const float* __restrict__ L, int locked,
                                                           int64_t m4, int64_t ldx) {
  __shared__ float s_part[4][DEFLATE_MAX];
  __shared__ float s_dot[DEFLATE_MAX];
  const int row = blockIdx.x, tid = threadIdx.x;
  float4* x = reinterpret_cast<float4*>(X + (size_t)row * ldx);
  if (row < locked) {
    const float4* src = reinterpret_cast<const float4*>(L + (size_t)row * ldx);
    for (int64_t j = tid; j < m4; j += 256) x[j] = src[j];
    return;
  }
  float dot[DEFLATE_MAX];
#pragma unroll
  for (int o = 0; o < DEFLATE_MAX; ++o) dot[o] = 0.f;
  for (int64_t j = tid; j < m4; j += 256) {
    const float4 v = x[j];
#pragma unroll
    for (int o = 0; o < DEFLATE_MAX; ++o)
      if (o < locked) {
        const float4 u = reinterpret_cast<const float4*>(L + (size_t)o * ldx)[j];
        dot[o] = fmaf(v.x, u.x, fmaf(v.y, u.y, fmaf(v.z, u.z, fmaf(v.w, u.w, dot[o]))));
      }
  }
#pragma unroll
  for (int o = 0; o < DEFLATE_MAX; ++o) {
    float t = dot[o];
    for (int off = 1; off < 64; off <<= 1) t += __shfl_xor(t, off);
    if ((tid & 63) == 0) s_part[tid >> 6][o] = t;
  }
  __syncthreads();
  if (tid < DEFLATE_MAX) s_dot[tid] = (s_part[0][tid] + s_part[1][tid]) + (s_part[2][tid] + s_part[3][tid]);
  __syncthreads();
  for (int64_t j = tid; j < m4; j += 256) {
    float4 v = x[j];
#pragma unroll
    for (int o = 0; o < DEFLATE_MAX; ++o)
      if (o < locked) {
        const float4 u = reinterpret_cast<const float4*>(L + (size_t)o * ldx)[j];
        const float c = s_dot[o];
        v.x = fmaf(-c, u.x, v.x); v.y = fmaf(-c, u.y, v.y); v.z = fmaf(-c, u.z, v.z); v.w = fmaf(-c, u.w, v.w);
      }
    x[j] = v;
  }
}

int launch_deflate_rows(float* X, const float* L, int l, int locked, int64_t m, int64_t ldx, hipStream_t st) {
  if (locked < 0 || locked > DEFLATE_MAX || ldx % 4 != 0) return LQ_ERR_ARG;
  if (locked == 0) return LQ_OK;
  prof::Scope ps(prof::MISC, st, (double)l * m * 4.0 * 2.0 * (1 + locked));
  hipLaunchKernelGGL(deflate_rows_kernel, dim3(l), dim3(256), 0, st, X, L, locked, (m + 3) / 4, ldx);
  LQ_HIP_TRY(hipGetLastError());
  return LQ_OK;
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

// ---- RowAverage / ColAverage of sqrt(F) (Section 3.3, Algorithm 4) ----------------------------------------------
// Pass 1: a workgroup takes FISHER_ROWS rows; thread t walks the columns t, t + 256, ...: it adds sqrt(F) down its
// column into one partial column sum per workgroup and across into FISHER_ROWS row sums, all in fp64.
constexpr int FISHER_ROWS = 16;

__global__ __launch_bounds__(256) void fisher_partial_kernel(const float* __restrict__ F, int64_t d, int64_t k,
                                                             double* __restrict__ rowsum,
                                                             double* __restrict__ colpart) {
  __shared__ double s_red[4][FISHER_ROWS];
  const int64_t row0 = (int64_t)blockIdx.x * FISHER_ROWS;
  const int tid = threadIdx.x;
  double racc[FISHER_ROWS];
#pragma unroll
  for (int r = 0; r < FISHER_ROWS; ++r) racc[r] = 0.0;
  for (int64_t c = tid; c < k; c += 256) {
    double cacc = 0.0;
#pragma unroll
    for (int r = 0; r < FISHER_ROWS; ++r) {
      const double s = row0 + r < d ? sqrt((double)F[(row0 + r) * k + c]) : 0.0;
      cacc += s;
      racc[r] += s;
    }
    colpart[(size_t)blockIdx.x * k + c] = cacc;
  }
#pragma unroll
  for (int r = 0; r < FISHER_ROWS; ++r) {
    double x = racc[r];
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
    if ((tid & 63) == 0) s_red[tid >> 6][r] = x;
  }
  __syncthreads();
  if (tid < FISHER_ROWS && row0 + tid < d) rowsum[row0 + tid] = (s_red[0][tid] + s_red[1][tid]) + (s_red[2][tid] + s_red[3][tid]);
}

// Pass 2: every workgroup forms the grand total from the row sums in the same fixed order, then finishes its share
// of the outputs: row_w = a^2, col_w = (b / mean)^2 with a, b the row and column means of sqrt(F).
__global__ __launch_bounds__(256) void fisher_finalize_kernel(const double* __restrict__ rowsum,
                                                              const double* __restrict__ colpart, int64_t d, int64_t k,
                                                              int chunks, float* __restrict__ row_w,
                                                              float* __restrict__ col_w) {
  __shared__ double s_red[4];
  const int tid = threadIdx.x;
  double tot = 0.0;
  for (int64_t i = tid; i < d; i += 256) tot += rowsum[i];
  for (int o = 32; o > 0; o >>= 1) tot += __shfl_xor(tot, o);
  if ((tid & 63) == 0) s_red[tid >> 6] = tot;
  __syncthreads();
  const double mean = ((s_red[0] + s_red[1]) + (s_red[2] + s_red[3])) / ((double)d * (double)k);
  const int64_t gid = (int64_t)blockIdx.x * 256 + tid, stride = (int64_t)gridDim.x * 256;
  for (int64_t i = gid; i < d; i += stride) {
    const double a = rowsum[i] / (double)k;
    row_w[i] = (float)(a * a);
  }
  for (int64_t j = gid; j < k; j += stride) {
    double b = 0.0;
    for (int ch = 0; ch < chunks; ++ch) b += colpart[(size_t)ch * k + j];
    b = b / (double)d / mean;
    col_w[j] = (float)(b * b);
  }
}

size_t fisher_scratch_doubles(int64_t d, int64_t k) {
  return (size_t)d + (size_t)((d + FISHER_ROWS - 1) / FISHER_ROWS) * (size_t)k;
}

int launch_fisher_row_col(const float* F, int64_t d, int64_t k, double* scratch, float* row_w, float* col_w,
                          hipStream_t st) {
  const int64_t chunks = (d + FISHER_ROWS - 1) / FISHER_ROWS;
  if (chunks >= (1ll << 31)) return LQ_ERR_SHAPE;
  double* rowsum = scratch;
  double* colpart = scratch + d;
  hipLaunchKernelGGL(fisher_partial_kernel, dim3((unsigned)chunks), dim3(256), 0, st, F, d, k, rowsum, colpart);
  LQ_HIP_TRY(hipGetLastError());
  const int64_t want = (std::max(d, k) + 255) / 256;
  hipLaunchKernelGGL(fisher_finalize_kernel, dim3((unsigned)std::min<int64_t>(want, 256)), dim3(256), 0, st, rowsum,
                     colpart, d, k, (int)chunks, row_w, col_w);
  LQ_HIP_TRY(hipGetLastError());
  return LQ_OK;
}

}  // namespace lq
