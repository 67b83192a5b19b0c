// Fused kernels of one LQ iteration (Algorithm 2):  Q <- Quantize(W - L1 L2, c)  and the error
// eps_t = || sqrt(F) .* (W - Q - L1 L2) ||_F, for a lock-step batch of configurations that share W.
//
// The residual T = W - L1 L2 is never written to memory.  Three phases, because the reconstructed block
// scale needs the absmax of a whole scale group (B0*B1 consecutive weights, which in general straddles
// rows) while T is produced in 2-D MFMA tiles:
//   1  per 64x128 tile: L1 L2 by MFMA (K = rank), T, block absmax s, codes against s (the codes depend on
//      the exact block absmax only), and three sums per block from which the error follows for any
//      reconstructed scale s^ = s + delta:  sum w (t - q s^)^2 = e2 - 2 delta eq + delta^2 q2.
//   2  per scale group: v = max s, scale indices, cast of v, and the error of the iteration.
//   3  per weight: R = D_row (W - Q) D_col, the input of the next Factorize (and / or dense Q).
#include "kernels.h"
#include "nf_device.h"
#include "profiler.h"

namespace lq {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int TM = 64;     // tile rows
constexpr int TN = 128;    // tile columns
constexpr int PP = TN + 4; // pitch of the product tile in LDS
constexpr int KC = 32;     // rank chunk staged in LDS

template <int BITS>
__device__ inline void phase1_epilogue(const PhaseArgs& a, const LoopProblem& pr, int z, const float* pt,
                                       const float* s_code, const float* s_thr, int64_t r0, int64_t c0,
                                       const float4 (&wreg)[2][4]) {
  Thresholds<BITS> thr(s_thr);
  const int tid = threadIdx.x;
  const int rpb = pr.cfg.block / 16;
  uint8_t* codes = a.codes + (size_t)z * a.strideCodes;
  BlockRec* blk = a.blk + (size_t)z * a.strideBlk;
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int rid = tid + 256 * u;            // run inside the tile: 8 runs per row
    const int lr = rid >> 3, rc = rid & 7;
    const int64_t row = r0 + lr, col = c0 + 16 * rc;
    const bool live = row < a.d && col < a.k;
    float t[16], w[16];
    if (live) {
      const float rs = a.rsr ? a.rsr[row] : 1.0f;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float4 f = wreg[u][q];
        const float4 p = *reinterpret_cast<const float4*>(pt + lr * PP + 16 * rc + 4 * q);
        float pv[4] = {p.x, p.y, p.z, p.w};
        const float fv[4] = {f.x, f.y, f.z, f.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          float cwj = 1.0f;
          if (a.rsc) {
            pv[e] = pv[e] * (rs * a.rsc[col + 4 * q + e]);
            cwj = a.col_w[col + 4 * q + e];
          }
          t[4 * q + e] = fv[e] - pv[e];
          w[4 * q + e] = cwj;
        }
      }
    } else {
#pragma unroll
      for (int j = 0; j < 16; ++j) { t[j] = 0.0f; w[j] = 0.0f; }
    }
    float amax = run_absmax(t);
    for (int off = 1; off < rpb; off <<= 1) amax = fmaxf(amax, __shfl_xor(amax, off));
    const float rcp = safe_reciprocal(amax);
    uint32_t c[16];
    float e2 = 0.f, eq = 0.f, q2 = 0.f;
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      c[j] = thr.nearest(t[j] * rcp);
      const float q = s_code[c[j]];
      const float e = t[j] - q * amax;
      e2 = fmaf(w[j] * e, e, e2);
      eq = fmaf(w[j] * e, q, eq);
      q2 = fmaf(w[j] * q, q, q2);
    }
    for (int off = 1; off < rpb; off <<= 1) {
      e2 += __shfl_xor(e2, off); eq += __shfl_xor(eq, off); q2 += __shfl_xor(q2, off);
    }
    if (live) {
      const int64_t run = ((int64_t)row * a.k + col) >> 4;
      store_codes<BITS>(codes, run, c);
      if ((run & (rpb - 1)) == 0) {
        BlockRec rec; rec.s = amax; rec.e2 = e2; rec.eq = eq; rec.q2 = q2;
        blk[run / rpb] = rec;
      }
    }
  }
}

__global__ __launch_bounds__(256) void lowrank_blockquant_kernel(PhaseArgs a) {
  // The operand chunks (Y: KC x TM, B: KC x TN) and the product tile share one LDS buffer: the product is
  // written after the last MFMA has read its operands.
  __shared__ __attribute__((aligned(16))) float smem[TM * PP];
  __shared__ float s_code[256];
  __shared__ float s_thr[256];
  float (*ys)[TM] = reinterpret_cast<float (*)[TM]>(smem);
  float (*bs)[TN] = reinterpret_cast<float (*)[TN]>(smem + KC * TM);
  float* pt = smem;
  static_assert(KC * TM + KC * TN <= TM * PP, "operand chunks must fit in the product tile");
  // problem index fastest: the workgroups that share a tile of W run together and hit it in L2
  const int z = blockIdx.x, tid = threadIdx.x;
  const LoopProblem pr = a.prob[z];
  const int64_t r0 = (int64_t)blockIdx.z * TM, c0 = (int64_t)blockIdx.y * TN;
  // this lane's two runs of W, fetched now so that the loads overlap the MFMA stage
  float4 wreg[2][4];
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int rid = tid + 256 * u;
    const int64_t row = r0 + (rid >> 3), col = c0 + 16 * (rid & 7);
    if (row < a.d && col < a.k) {
      const float4* wp = reinterpret_cast<const float4*>(a.W + (size_t)row * a.k + col);
#pragma unroll
      for (int q = 0; q < 4; ++q) wreg[u][q] = wp[q];
    } else {
#pragma unroll
      for (int q = 0; q < 4; ++q) wreg[u][q] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
  }
  const float* __restrict__ Y = a.Y + (size_t)z * a.strideY;
  const float* __restrict__ B = a.B + (size_t)z * a.strideB;
  const int wave = tid >> 6, lane = tid & 63, ln = lane & 31, lh = lane >> 5;
  const int wr = wave >> 1, wc = wave & 1;

  floatx16 acc[2];
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[j][e] = 0.0f;

  for (int k0 = 0; k0 < a.rank; k0 += KC) {
    __syncthreads();
    // stage Y[k0..k0+32)[r0..r0+64) and B[k0..k0+32)[c0..c0+128); rows past rank and columns past the
    // matrix are zero (the wide bases hold more than `rank` rows; only the leading ones form L1 L2)
    for (int idx = tid; idx < KC * TM; idx += 256) {
      const int kk = idx / TM, rr = idx % TM;
      float val = 0.0f;
      if (k0 + kk < a.rank && r0 + rr < a.d) val = Y[(size_t)(k0 + kk) * a.ldy + r0 + rr];
      ys[kk][rr] = val;
    }
    for (int idx = tid; idx < KC * TN; idx += 256) {
      const int kk = idx / TN, cc = idx % TN;
      float val = 0.0f;
      if (k0 + kk < a.rank && c0 + cc < a.k) val = B[(size_t)(k0 + kk) * a.ldb + c0 + cc];
      bs[kk][cc] = val;
    }
    __syncthreads();
#pragma unroll
    for (int s = 0; s < KC / 2; ++s) {
      const float av = ys[2 * s + lh][32 * wr + ln];
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const float bv = bs[2 * s + lh][64 * wc + 32 * j + ln];
        acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc[j], 0, 0, 0);
      }
    }
  }
  __syncthreads();          // all operand reads done before the product overwrites the buffer
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int row = 32 * wr + 8 * (e >> 2) + 4 * lh + (e & 3);
      pt[row * PP + 64 * wc + 32 * j + ln] = acc[j][e];
    }
  // code-book for this problem's bit width
  const int slot = pr.cfg.bits == 2 ? 0 : pr.cfg.bits == 3 ? 1 : pr.cfg.bits == 4 ? 2 : 3;
  s_code[tid] = a.tables->code[slot][tid];
  s_thr[tid] = a.tables->thr[slot][tid];
  __syncthreads();
  switch (pr.cfg.bits) {
    case 2: phase1_epilogue<2>(a, pr, z, pt, s_code, s_thr, r0, c0, wreg); break;
    case 3: phase1_epilogue<3>(a, pr, z, pt, s_code, s_thr, r0, c0, wreg); break;
    case 4: phase1_epilogue<4>(a, pr, z, pt, s_code, s_thr, r0, c0, wreg); break;
    default: phase1_epilogue<8>(a, pr, z, pt, s_code, s_thr, r0, c0, wreg); break;
  }
}

int launch_lowrank_blockquant(const PhaseArgs& a, hipStream_t st) {
  const dim3 grid((unsigned)a.batch, (unsigned)((a.k + TN - 1) / TN), (unsigned)((a.d + TM - 1) / TM));
  prof::Scope ps(prof::LOWRANK_BLOCKQUANT, st, (double)a.d * a.k * 4.0 * a.batch);
  hipLaunchKernelGGL(lowrank_blockquant_kernel, grid, dim3(256), 0, st, a);
  LQ_HIP_TRY(hipGetLastError());
  return LQ_OK;
}

// ------------------------------------------------------------------------------------------------
// Phase 2: one lane per block.
__global__ __launch_bounds__(256) void scalequant_error_kernel(PhaseArgs a) {
  __shared__ float s_wave[4];
  __shared__ double s_sum[4];
  const int z = blockIdx.y, tid = threadIdx.x;
  const LoopProblem pr = a.prob[z];
  const int64_t nb = (a.d * a.k) / pr.cfg.block;
  const int64_t b = (int64_t)blockIdx.x * 256 + tid;
  double* part = a.err_part + (size_t)z * a.strideErrPart;
  if ((int64_t)blockIdx.x * 256 >= nb) {           // whole workgroup past this problem's blocks
    if (tid == 0) part[blockIdx.x] = 0.0;
    return;
  }
  BlockRec rec; rec.s = 0.f; rec.e2 = 0.f; rec.eq = 0.f; rec.q2 = 0.f;
  if (b < nb) rec = a.blk[(size_t)z * a.strideBlk + b];
  const float vmax = group_max(rec.s, pr.cfg.scale_block, s_wave);
  const float sigma = vmax / (float)pr.levels;
  const float vhat = cast_group_scale(vmax, pr.cfg.v_dtype);
  double err = 0.0;
  if (b < nb) {
    const uint32_t idx = scale_index(rec.s, sigma, pr.levels);
    a.sidx[(size_t)z * a.strideSidx + b] = (uint8_t)idx;
    if ((b & (pr.cfg.scale_block - 1)) == 0) a.v[(size_t)z * a.strideV + b / pr.cfg.scale_block] = vhat;
    const float shat = block_scale(idx, vhat, pr.levels);
    const double delta = (double)shat - (double)rec.s;
    err = (double)rec.e2 - 2.0 * delta * (double)rec.eq + delta * delta * (double)rec.q2;
    if (a.row_w) err *= (double)a.row_w[(b * pr.cfg.block) / a.k];
  }
  for (int off = 1; off < 64; off <<= 1) err += __shfl_xor(err, off);
  if ((tid & 63) == 0) s_sum[tid >> 6] = err;
  __syncthreads();
  if (tid == 0) part[blockIdx.x] = (s_sum[0] + s_sum[1]) + (s_sum[2] + s_sum[3]);
}

// eps = sqrt(sum of the partials), one workgroup per problem, fixed summation order.
__global__ __launch_bounds__(256) void error_finalize_kernel(const double* __restrict__ part, size_t stride,
                                                             int64_t count, double* __restrict__ out,
                                                             size_t out_stride) {
  __shared__ double s_sum[256];
  const int z = blockIdx.x, tid = threadIdx.x;
  const double* p = part + (size_t)z * stride;
  double s = 0.0;
  for (int64_t i = tid; i < count; i += 256) s += p[i];
  s_sum[tid] = s;
  __syncthreads();
  for (int w = 128; w >= 1; w >>= 1) {
    if (tid < w) s_sum[tid] += s_sum[tid + w];
    __syncthreads();
  }
  if (tid == 0) out[(size_t)z * out_stride] = sqrt(s_sum[0] > 0.0 ? s_sum[0] : 0.0);
}

int64_t err_partials_per_problem(int64_t n, int block) { return (n / block + 255) / 256; }

int launch_scalequant_error(const PhaseArgs& a, int min_block, hipStream_t st) {
  const int64_t nwg = err_partials_per_problem(a.d * a.k, min_block);
  prof::Scope ps(prof::SCALEQUANT_ERROR, st, (double)(a.d * a.k / min_block) * 17.0 * a.batch);
  hipLaunchKernelGGL(scalequant_error_kernel, dim3((unsigned)nwg, (unsigned)a.batch), dim3(256), 0, st, a);
  LQ_HIP_TRY(hipGetLastError());
  hipLaunchKernelGGL(error_finalize_kernel, dim3((unsigned)a.batch), dim3(256), 0, st, (const double*)a.err_part,
                     a.strideErrPart, nwg, a.err_out, a.strideErrOut);
  LQ_HIP_TRY(hipGetLastError());
  return LQ_OK;
}

// ------------------------------------------------------------------------------------------------
// Phase 3: one quad (4 consecutive weights) per lane and step, so each wavefront instruction reads / writes
// 1 KB of contiguous fp32.
template <int BITS>
__device__ inline void phase3_body(const PhaseArgs& a, const LoopProblem& pr, int z, const float* s_code) {
  const int64_t nquads = (a.d * a.k) >> 2;
  const int qpb_shift = __builtin_ctz(pr.cfg.block / 4), sb_shift = __builtin_ctz(pr.cfg.scale_block);
  const uint8_t* codes = a.codes + (size_t)z * a.strideCodes;
  const uint8_t* sidx = a.sidx + (size_t)z * a.strideSidx;
  const float* v = a.v + (size_t)z * a.strideV;
  float* R = a.R ? a.R + (size_t)z * a.strideR : nullptr;
  float* Qd = a.Qd ? a.Qd + (size_t)z * a.strideQd : nullptr;
  for (int64_t quad = (int64_t)blockIdx.y * 256 + threadIdx.x; quad < nquads; quad += (int64_t)gridDim.y * 256) {
    const int64_t blk = quad >> qpb_shift;
    const float sh = block_scale(sidx[blk], v[blk >> sb_shift], pr.levels);
    uint32_t c[4];
    load_quad_codes<BITS>(codes, quad, c);
    const int64_t e0 = quad << 2;
    const float4 f = *reinterpret_cast<const float4*>(a.W + e0);
    float4 qv, rv;
    qv.x = s_code[c[0]] * sh; qv.y = s_code[c[1]] * sh; qv.z = s_code[c[2]] * sh; qv.w = s_code[c[3]] * sh;
    rv.x = f.x - qv.x; rv.y = f.y - qv.y; rv.z = f.z - qv.z; rv.w = f.w - qv.w;
    if (a.sr) {
      const int64_t row = e0 / a.k, col = e0 % a.k;
      const float srow = a.sr[row];
      const float4 cs = *reinterpret_cast<const float4*>(a.sc + col);
      rv.x = srow * rv.x * cs.x; rv.y = srow * rv.y * cs.y; rv.z = srow * rv.z * cs.z; rv.w = srow * rv.w * cs.w;
    }
    if (R) *reinterpret_cast<float4*>(R + e0) = rv;
    if (Qd) *reinterpret_cast<float4*>(Qd + e0) = qv;
  }
}

__global__ __launch_bounds__(256) void residual_kernel(PhaseArgs a) {
  __shared__ float s_code[256];
  const int z = blockIdx.x;          // problem index fastest: W is fetched from HBM once per batch
  const LoopProblem pr = a.prob[z];
  const int slot = pr.cfg.bits == 2 ? 0 : pr.cfg.bits == 3 ? 1 : pr.cfg.bits == 4 ? 2 : 3;
  s_code[threadIdx.x] = a.tables->code[slot][threadIdx.x];
  __syncthreads();
  switch (pr.cfg.bits) {
    case 2: phase3_body<2>(a, pr, z, s_code); break;
    case 3: phase3_body<3>(a, pr, z, s_code); break;
    case 4: phase3_body<4>(a, pr, z, s_code); break;
    default: phase3_body<8>(a, pr, z, s_code); break;
  }
}

int launch_residual(const PhaseArgs& a, hipStream_t st) {
  const int64_t nquads = (a.d * a.k) >> 2;
  const int64_t want = (nquads + 255) / 256;
  const int64_t cap = 8192;
  prof::Scope ps(prof::RESIDUAL, st, (double)a.d * a.k * 8.0 * a.batch);
  hipLaunchKernelGGL(residual_kernel, dim3((unsigned)a.batch, (unsigned)(want < cap ? want : cap)), dim3(256), 0, st,
                     a);
  LQ_HIP_TRY(hipGetLastError());
  return LQ_OK;
}

}  // namespace lq
