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
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int TM = 64;     // tile rows
constexpr int TN = 128;    // tile columns
constexpr int PP = TN + 4; // pitch of the product tile in LDS
constexpr int KC = 32;     // rank chunk staged in LDS
constexpr int NTHR1 = 512; // threads of the phase-1 workgroup: 8 wavefronts, one 32x32 MFMA tile each
constexpr int KC2 = 64;    // rank chunk of the split-precision product
constexpr int KP = KC2 + 8;// LDS row pitch of its operand planes in bf16 elements (144 B: conflict-free b128 reads)

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 halfx4 __attribute__((ext_vector_type(4)));

// ------------------------------------------------------------------------------------------------
// Split-precision operands of L1 L2 = Y_r^T B_r: every factor entry x is stored as bf16 hi + bf16 lo
// (x = hi + lo + O(2^-17 x)), transposed so that the reduction index is contiguous:
//   plane[i][p], i < rows_pad (zero rows past the matrix), p < RK = round_up16(rank) (zeros past the rank);
// per problem: Y hi, Y lo (dpad x RK each), then B hi, B lo (kpad x RK each).
int64_t packed_rows_y(int64_t d) { return (d + TM - 1) / TM * TM; }
int64_t packed_rows_b(int64_t k) { return (k + TN - 1) / TN * TN; }
int packed_rank(int rank) { return (rank + 15) / 16 * 16; }
size_t packed_factor_elems(int64_t d, int64_t k, int rank) {
  return (size_t)2 * (packed_rows_y(d) + packed_rows_b(k)) * packed_rank(rank);
}

__global__ __launch_bounds__(256) void pack_factors_kernel(PhaseArgs a, int64_t dpad, int64_t kpad, int rk) {
  const int z = blockIdx.y;
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;          // row of the packed planes, Y rows first
  if (i >= dpad + kpad) return;
  const bool isy = i < dpad;
  const int64_t r = isy ? i : i - dpad, lim = isy ? a.d : a.k, ld = isy ? a.ldy : a.ldb;
  const float* src = isy ? a.Y + (size_t)z * a.strideY : a.B + (size_t)z * a.strideB;
  __bf16* base = reinterpret_cast<__bf16*>(a.packed) + (size_t)z * a.stridePacked + (isy ? 0 : (size_t)2 * dpad * rk);
  __bf16* hi = base + (size_t)r * rk;
  __bf16* lo = hi + (size_t)(isy ? dpad : kpad) * rk;
  for (int p0 = 0; p0 < rk; p0 += 8) {
    bf16x8 h, l;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float x = (r < lim && p0 + e < a.rank) ? src[(size_t)(p0 + e) * ld + r] : 0.0f;
      const __bf16 xh = (__bf16)x;
      h[e] = xh;
      l[e] = (__bf16)(x - (float)xh);
    }
    *reinterpret_cast<bf16x8*>(hi + p0) = h;
    *reinterpret_cast<bf16x8*>(lo + p0) = l;
  }
}

int launch_pack_factors(const PhaseArgs& a, hipStream_t st) {
  const int64_t dpad = packed_rows_y(a.d), kpad = packed_rows_b(a.k);
  prof::Scope ps(prof::MISC, st, (double)(a.d + a.k) * a.rank * 8.0 * a.batch);
  hipLaunchKernelGGL(pack_factors_kernel, dim3((unsigned)((dpad + kpad + 255) / 256), (unsigned)a.batch), dim3(256), 0,
                     st, a, dpad, kpad, packed_rank(a.rank));
  LQ_HIP_TRY(hipGetLastError());
  return LQ_OK;
}

// Stores the 4 codes of one quad.  `base`: address of the codes of a quad whose index is a multiple of 4 (uniform across
// the wavefront in phase 1), `lq`: this lane's quad index relative to it.  2, 4, 8 bits: 1, 2, 4 bytes per lane,
// contiguous across lanes.  3 bits: the four lanes of a 16-weight run gather their 12-bit pieces into the run's 48-bit
// word and three of them store 16 bits each.  All 64 lanes must call (cross-lane exchange inside).
template <int BITS>
__device__ __forceinline__ void store_quad_codes(uint8_t* __restrict__ base, uint32_t lq, const uint32_t (&c)[4],
                                                 bool live) {
  const uint32_t w = c[0] | (c[1] << BITS) | (c[2] << (2 * BITS)) | (c[3] << (3 * BITS));
  if constexpr (BITS == 8) {
    if (live) *reinterpret_cast<uint32_t*>(base + lq * 4u) = w;
  } else if constexpr (BITS == 4) {
    if (live) *reinterpret_cast<uint16_t*>(base + lq * 2u) = (uint16_t)w;
  } else if constexpr (BITS == 2) {
    if (live) base[lq] = (uint8_t)w;
  } else {
    const int sub = threadIdx.x & 3;
    uint32_t lo = sub < 2 ? (w << (12 * sub)) : (sub == 2 ? (w << 24) : 0u);        // bits 0..31 of the run word
    uint32_t hi = sub == 2 ? (w >> 8) : (sub == 3 ? (w << 4) : 0u);                 // bits 32..47
    lo |= dpp_move_u32<DPP_QUAD_XOR1>(lo); hi |= dpp_move_u32<DPP_QUAD_XOR1>(hi);
    lo |= dpp_move_u32<DPP_QUAD_XOR2>(lo); hi |= dpp_move_u32<DPP_QUAD_XOR2>(hi);
    if (live && sub < 3) {
      const uint16_t piece = sub == 0 ? (uint16_t)lo : (sub == 1 ? (uint16_t)(lo >> 16) : (uint16_t)hi);
      *reinterpret_cast<uint16_t*>(base + (lq >> 2) * 6u + 2u * sub) = piece;
    }
  }
}

// Code search of phase 1.  One 16-byte LDS entry per bucket j = floor((x + 1) * 256), j = 0..513 (x lies in
// [-1, 1] up to rounding; the index is clamped all the same): {thr[c0], c0, thr[c0 + 1]} with c0 = the number of
// thresholds safely below the bucket.  The code of x is c0 + (x >= thr[c0]) (+ (x >= thr[c0 + 1]) for 8 bits, where two
// thresholds can fall into one bucket): one LDS read and one or two comparisons per weight for every bit width.
struct SearchEntry { float ta; uint32_t c0; float tb; uint32_t pad; };
constexpr int SEARCH_ENTRIES = 514;

__device__ __forceinline__ void build_search_nosync(const DevTables* __restrict__ tab, int slot, SearchEntry* s_search) {
  for (int j = threadIdx.x; j < SEARCH_ENTRIES; j += blockDim.x) {
    const uint32_t c0 = tab->lut[slot][j < 511 ? j : 511];
    SearchEntry e;
    e.ta = tab->thr[slot][c0]; e.c0 = c0; e.tb = tab->thr[slot][c0 + 1]; e.pad = 0;
    s_search[j] = e;
  }
}

template <int BITS>
__device__ __forceinline__ uint32_t search_code(const SearchEntry* s_search, float x) {
  int j = (int)fmaf(x, 256.0f, 256.0f);                         // NaN -> 0
  j = j < 0 ? 0 : (j > SEARCH_ENTRIES - 1 ? SEARCH_ENTRIES - 1 : j);
  if constexpr (BITS == 8) {
    const float4 e = *reinterpret_cast<const float4*>(s_search + j);
    return __float_as_uint(e.y) + ((x >= e.x) ? 1u : 0u) + ((x >= e.z) ? 1u : 0u);
  } else {
    const float2 e = *reinterpret_cast<const float2*>(s_search + j);
    return __float_as_uint(e.y) + ((x >= e.x) ? 1u : 0u);
  }
}

// max |t| of a quad, as the bit pattern of a non-negative float (unsigned order = numeric order).
__device__ __forceinline__ uint32_t quad_absmax_bits(const float (&t)[4]) {
  float m;
  asm("v_max3_f32 %0, |%1|, |%2|, |%3|\n\tv_max_f32 %0, |%4|, %0" : "=&v"(m) : "v"(t[0]), "v"(t[1]), "v"(t[2]), "v"(t[3]));
  return __float_as_uint(m);
}
template <int CTRL>
__device__ __forceinline__ uint32_t umax_dpp(uint32_t x) {
  const uint32_t y = (uint32_t)__builtin_amdgcn_update_dpp((int)x, (int)x, CTRL, 0xf, 0xf, false);
  return x > y ? x : y;
}
// Maximum over the QPB consecutive lanes that hold one block (see group_max_lanes), on bit patterns.
template <int QPB>
__device__ __forceinline__ uint32_t block_umax(uint32_t x) {
  x = umax_dpp<DPP_QUAD_XOR1>(x);
  x = umax_dpp<DPP_QUAD_XOR2>(x);
  if constexpr (QPB >= 8) x = umax_dpp<DPP_ROW_HALF_MIRROR>(x);
  if constexpr (QPB >= 16) x = umax_dpp<DPP_ROW_MIRROR>(x);
  if constexpr (QPB >= 32) { const uint32_t y = (uint32_t)__shfl_xor((int)x, 16); x = x > y ? x : y; }
  return x;
}

// Epilogue of phase 1 in quad layout: lane `tid` handles quads tid, tid+512, ... of the 64 x 128 tile (32 quads
// per row), so W loads, LDS reads of the product and code stores are all contiguous across lanes.  QPB = B0/4
// lanes hold one block.  The four quads of a lane lie in four different blocks; their block maxima are found first,
// then one division serves all four (lane i of every hardware quad divides for quad i, the quotients go back by quad
// broadcasts: the four lanes of a hardware quad always share their blocks), then the codes.
template <int BITS, int QPB, bool WITH_ERR>
__device__ __forceinline__ void phase1_epilogue(const PhaseArgs& a, int z, const float* pt, const SearchEntry* s_search,
                                                const float* s_code, int64_t r0, int64_t c0, const float4 (&wreg)[4]) {
  const int tid = threadIdx.x;
  uint8_t* codes = a.codes + (size_t)z * a.strideCodes;
  BlockRec* blk = a.blk + (size_t)z * a.strideBlk;
  // quad indices: a uniform part per quad u (first quad of the tile, NTHR1 / 32 rows further down for each u) plus a
  // 32-bit lane part; both are multiples of QPB where a block starts, so block indices split the same way
  const int cq = tid & 31;
  const int64_t col = c0 + 4 * cq;
  const int64_t tq0 = (r0 * a.k + c0) >> 2, quad_step = (NTHR1 / 32) * (a.k >> 2);
  const uint32_t lq = (uint32_t)((tid >> 5) * (a.k >> 2) + cq);
  constexpr int CODE_BYTES_X2 = BITS;            // bytes per quad = BITS / 2
  const bool col_live = col < a.k;
  float4 rc = make_float4(1.f, 1.f, 1.f, 1.f), cw = make_float4(1.f, 1.f, 1.f, 1.f);
  if (a.rsc && col_live) {
    rc = *reinterpret_cast<const float4*>(a.rsc + col);
    if (WITH_ERR) cw = *reinterpret_cast<const float4*>(a.col_w + col);
  }
  float t[4][4];
  uint32_t mbits[4];
  bool live[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int lr = (tid >> 5) + (NTHR1 / 32) * u;
    const int64_t row = r0 + lr;
    live[u] = row < a.d && col_live;
    const float4 p = *reinterpret_cast<const float4*>(pt + lr * PP + 4 * cq);
    float pv[4] = {p.x, p.y, p.z, p.w};
    const float fv[4] = {wreg[u].x, wreg[u].y, wreg[u].z, wreg[u].w};
    if (a.rsc) {
      const float rs = live[u] ? a.rsr[row] : 0.0f;
      pv[0] *= rs * rc.x; pv[1] *= rs * rc.y; pv[2] *= rs * rc.z; pv[3] *= rs * rc.w;
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) t[u][e] = live[u] ? fv[e] - pv[e] : 0.0f;
    mbits[u] = block_umax<QPB>(quad_absmax_bits(t[u]));
  }
  // lane i of each hardware quad divides for quad i
  const int sub = tid & 3;
  const uint32_t mine = sub == 0 ? mbits[0] : sub == 1 ? mbits[1] : sub == 2 ? mbits[2] : mbits[3];
  const int rmine = (int)__float_as_uint(safe_reciprocal(__uint_as_float(mine)));
  const float rcp[4] = {__int_as_float(__builtin_amdgcn_mov_dpp(rmine, 0x00, 0xf, 0xf, true)),
                        __int_as_float(__builtin_amdgcn_mov_dpp(rmine, 0x55, 0xf, 0xf, true)),
                        __int_as_float(__builtin_amdgcn_mov_dpp(rmine, 0xAA, 0xf, 0xf, true)),
                        __int_as_float(__builtin_amdgcn_mov_dpp(rmine, 0xFF, 0xf, 0xf, true))};
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const float amax = __uint_as_float(mbits[u]);
    uint32_t c[4];
    float e2 = 0.f, eq = 0.f, q2 = 0.f;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      c[e] = search_code<BITS>(s_search, t[u][e] * rcp[u]);
      if (WITH_ERR) {
        const float w = a.rsc ? (e == 0 ? cw.x : e == 1 ? cw.y : e == 2 ? cw.z : cw.w) : 1.0f;
        const float q = s_code[c[e]];
        const float err = t[u][e] - q * amax;
        e2 = fmaf(w * err, err, e2);
        eq = fmaf(w * err, q, eq);
        q2 = fmaf(w * q, q, q2);
      }
    }
    if (WITH_ERR) {
      if (!live[u]) { e2 = 0.f; eq = 0.f; q2 = 0.f; }
      e2 = group_sum_lanes<QPB>(e2); eq = group_sum_lanes<QPB>(eq); q2 = group_sum_lanes<QPB>(q2);
    }
    const int64_t quad_u = tq0 + (int64_t)u * quad_step;                   // uniform
    store_quad_codes<BITS>(codes + ((quad_u * CODE_BYTES_X2) >> 1), lq, c, live[u]);
    if (live[u] && (cq & (QPB - 1)) == 0) {
      if (WITH_ERR) {
        BlockRec rec; rec.s = amax; rec.e2 = e2; rec.eq = eq; rec.q2 = q2;
        (blk + quad_u / QPB)[lq / QPB] = rec;
      } else {
        (reinterpret_cast<float*>(blk) + quad_u / QPB)[lq / QPB] = amax;   // without error sums a record is the absmax alone
      }
    }
  }
}

template <int BITS, bool WITH_ERR>
__device__ __forceinline__ void phase1_dispatch_block(const PhaseArgs& a, int block, int z, const float* pt,
                                                      const SearchEntry* s_search, const float* s_code, int64_t r0,
                                                      int64_t c0, const float4 (&wreg)[4]) {
  switch (block) {
    case 16: phase1_epilogue<BITS, 4, WITH_ERR>(a, z, pt, s_search, s_code, r0, c0, wreg); break;
    case 32: phase1_epilogue<BITS, 8, WITH_ERR>(a, z, pt, s_search, s_code, r0, c0, wreg); break;
    case 64: phase1_epilogue<BITS, 16, WITH_ERR>(a, z, pt, s_search, s_code, r0, c0, wreg); break;
    default: phase1_epilogue<BITS, 32, WITH_ERR>(a, z, pt, s_search, s_code, r0, c0, wreg); break;
  }
}

// SPLIT: L1 L2 from the packed bf16 hi/lo planes with three v_mfma_f32_32x32x16_bf16 per 16-deep group
// (hi*hi + hi*lo + lo*hi, fp32 accumulation; products good to about 2^-16 relative) instead of fp32 MFMAs.
// Launch: one-dimensional, batch * tiles8 workgroups (tiles8 = number of 64 x 128 tiles rounded up to a multiple
// of 8).  Workgroups go to the 8 XCDs round-robin by index; the index is decoded as (tile mod 8, problem, tile div 8),
// so the problems of a batch that share a tile of W run on one XCD and fetch it into that XCD's L2 once.
template <bool WITH_ERR, bool SPLIT>
__global__ __launch_bounds__(NTHR1) void lowrank_blockquant_kernel(PhaseArgs a, int tiles, int tiles_n) {
  // The operand chunks and the product tile share one LDS buffer: the product is written after the last MFMA has
  // read its operands.  fp32: Y chunk KC x TM, B chunk KC x TN.  Split: four planes (Y hi, Y lo: TM rows; B hi, B lo:
  // TN rows) of KC2 reduction indices, pitch KP.
  constexpr int SMEM_FLOATS = SPLIT ? ((2 * (TM + TN) * KP * 2 + 3) / 4 > TM * PP ? (2 * (TM + TN) * KP * 2 + 3) / 4 : TM * PP)
                                    : TM * PP;
  __shared__ __attribute__((aligned(16))) float smem[SMEM_FLOATS];
  __shared__ __attribute__((aligned(16))) SearchEntry s_search[SEARCH_ENTRIES];
  __shared__ float s_code[WITH_ERR ? 256 : 1];
  float* pt = smem;
  static_assert(KC * TM + KC * TN <= TM * PP, "operand chunks must fit in the product tile");
  const int tid = threadIdx.x;
  const int slot8 = blockIdx.x >> 3;
  const int z = slot8 % a.batch;
  const int tile = (int)(blockIdx.x & 7) + 8 * (slot8 / a.batch);
  if (tile >= tiles) return;                   // padding of the tile count to a multiple of 8
  const LoopProblem pr = a.prob[z];
  const int64_t r0 = (int64_t)(tile / tiles_n) * TM, c0 = (int64_t)(tile % tiles_n) * TN;
  const int wave = tid >> 6, lane = tid & 63, ln = lane & 31, lh = lane >> 5;
  const int wr = wave >> 2, wc = wave & 3;      // 2 x 4 grid of 32x32 tiles

  // search table (and, for the error sums, the code book) of this problem's bit width, visible after the barriers of
  // the product stage
  const int slot = pr.cfg.bits == 2 ? 0 : pr.cfg.bits == 3 ? 1 : pr.cfg.bits == 4 ? 2 : 3;
  build_search_nosync(a.tables, slot, s_search);
  if constexpr (WITH_ERR)
    for (int i = tid; i < 256; i += NTHR1) s_code[i] = a.tables->code[slot][i];
  // this lane's 4 quads of W, fetched now so that the loads overlap the MFMA stage.  Addresses are a uniform base per
  // quad plus one 32-bit lane offset (rows of a tile are at most 63 apart).
  float4 wreg[4];
  const uint32_t w_lane = (uint32_t)(((tid >> 5) * a.k + 4 * (tid & 31)) * 4);
  const bool w_col_live = c0 + 4 * (tid & 31) < a.k;
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int64_t row_u = r0 + (NTHR1 / 32) * u;                       // uniform
    const char* base = reinterpret_cast<const char*>(a.W + (size_t)row_u * a.k + c0);
    wreg[u] = (row_u + (tid >> 5) < a.d && w_col_live) ? *reinterpret_cast<const float4*>(base + w_lane)
                                                         : make_float4(0.f, 0.f, 0.f, 0.f);
  }

  floatx16 acc;
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[e] = 0.0f;

  if constexpr (SPLIT) {
    __bf16* planes = reinterpret_cast<__bf16*>(smem);          // [Yh | Yl | Bh | Bl], rows x KP
    const int rk = (a.rank + 15) / 16 * 16;
    const int64_t dpad = (a.d + TM - 1) / TM * TM, kpad = (a.k + TN - 1) / TN * TN;
    const __bf16* gy = reinterpret_cast<const __bf16*>(a.packed) + (size_t)z * a.stridePacked;
    const __bf16* gb = gy + (size_t)2 * dpad * rk;
    // piece idx = tid + 512 i, i < 6: 16 bytes (8 reduction indices) of one row of one plane.  Rows tid / 8 + 64 i of the
    // stacked planes [Yh | Yl | Bh | Bl]: piece i always falls into the same plane, at row (tid / 8) (+ 64 for the second
    // half of a B plane), so its address is a uniform base plus the lane offset all pieces share.
    constexpr int PIECES = 2 * (TM + TN) * (KC2 / 8) / NTHR1;
    static_assert(PIECES == 6 && TM == 64 && TN == 128 && NTHR1 == 512, "piece-to-plane map below");
    floatx4 st[PIECES];
    const floatx4 zero4 = {0.f, 0.f, 0.f, 0.f};
    const uint32_t p_lane = (uint32_t)(((tid >> 3) * rk + 8 * (tid & 7)) * 2);
    const char* pbase[PIECES] = {
        reinterpret_cast<const char*>(gy + (size_t)r0 * rk),                   // Y hi
        reinterpret_cast<const char*>(gy + (size_t)(dpad + r0) * rk),          // Y lo
        reinterpret_cast<const char*>(gb + (size_t)c0 * rk),                   // B hi, rows 0..63
        reinterpret_cast<const char*>(gb + (size_t)(c0 + 64) * rk),            // B hi, rows 64..127
        reinterpret_cast<const char*>(gb + (size_t)(kpad + c0) * rk),          // B lo, rows 0..63
        reinterpret_cast<const char*>(gb + (size_t)(kpad + c0 + 64) * rk)};    // B lo, rows 64..127
    auto fetch_planes = [&](int k0) {
      const bool ok = k0 + 8 * (tid & 7) < rk;
#pragma unroll
      for (int i = 0; i < PIECES; ++i)
        st[i] = ok ? *reinterpret_cast<const floatx4*>(pbase[i] + p_lane + 2 * k0) : zero4;
    };
    fetch_planes(0);
    for (int k0 = 0; k0 < rk; k0 += KC2) {
      __syncthreads();
#pragma unroll
      for (int i = 0; i < PIECES; ++i) {
        const int idx = tid + NTHR1 * i;
        *reinterpret_cast<floatx4*>(planes + (size_t)(idx >> 3) * KP + 8 * (idx & 7)) = st[i];
      }
      __syncthreads();
      if (k0 + KC2 < rk) fetch_planes(k0 + KC2);
      const __bf16* yh = planes + (size_t)(32 * wr + ln) * KP + 8 * lh;
      const __bf16* yl = yh + (size_t)TM * KP;
      const __bf16* bh = planes + (size_t)(2 * TM + 32 * wc + ln) * KP + 8 * lh;
      const __bf16* bl = bh + (size_t)TN * KP;
#pragma unroll
      for (int kg = 0; kg < KC2 / 16; ++kg) {
        if (k0 + 16 * kg < rk) {
          const bf16x8 ah = *reinterpret_cast<const bf16x8*>(yh + 16 * kg), al = *reinterpret_cast<const bf16x8*>(yl + 16 * kg);
          const bf16x8 vh = *reinterpret_cast<const bf16x8*>(bh + 16 * kg), vl = *reinterpret_cast<const bf16x8*>(bl + 16 * kg);
          acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, vh, acc, 0, 0, 0);
          acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, vl, acc, 0, 0, 0);
          acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, vh, acc, 0, 0, 0);
        }
      }
    }
  } else {
    float (*ys)[TM] = reinterpret_cast<float (*)[TM]>(smem);
    float (*bs)[TN] = reinterpret_cast<float (*)[TN]>(smem + KC * TM);
    const float* __restrict__ Y = a.Y + (size_t)z * a.strideY;
    const float* __restrict__ B = a.B + (size_t)z * a.strideB;
    // operand chunk staging through registers, 128-bit pieces: piece idx = tid + 512*i of the chunk.  The wide
    // bases have at least round_up32(rank) rows and zero-padded leading dimensions, so only the column offset
    // needs clamping; rows past `rank` and columns past the matrix are replaced by zeros after the load.
    floatx4 yst[KC * TM / (4 * NTHR1)], bst[KC * TN / (4 * NTHR1)];
    const floatx4 zero4 = {0.f, 0.f, 0.f, 0.f};
    auto fetch_chunk = [&](int k0) {
#pragma unroll
      for (int i = 0; i < KC * TM / (4 * NTHR1); ++i) {
        const int idx = tid + NTHR1 * i, kk = idx / (TM / 4), rr = 4 * (idx % (TM / 4));
        const int64_t off = r0 + rr;
        const bool ok = k0 + kk < a.rank && off < a.d;
        const floatx4 v = *reinterpret_cast<const floatx4*>(Y + (size_t)(k0 + kk) * a.ldy + (off + 4 <= a.ldy ? off : a.ldy - 4));
        yst[i] = ok ? v : zero4;
      }
#pragma unroll
      for (int i = 0; i < KC * TN / (4 * NTHR1); ++i) {
        const int idx = tid + NTHR1 * i, kk = idx / (TN / 4), cc = 4 * (idx % (TN / 4));
        const int64_t off = c0 + cc;
        const bool ok = k0 + kk < a.rank && off < a.k;
        const floatx4 v = *reinterpret_cast<const floatx4*>(B + (size_t)(k0 + kk) * a.ldb + (off + 4 <= a.ldb ? off : a.ldb - 4));
        bst[i] = ok ? v : zero4;
      }
    };
    fetch_chunk(0);
    for (int k0 = 0; k0 < a.rank; k0 += KC) {
      __syncthreads();
#pragma unroll
      for (int i = 0; i < KC * TM / (4 * NTHR1); ++i) {
        const int idx = tid + NTHR1 * i;
        *reinterpret_cast<floatx4*>(&ys[idx / (TM / 4)][4 * (idx % (TM / 4))]) = yst[i];
      }
#pragma unroll
      for (int i = 0; i < KC * TN / (4 * NTHR1); ++i) {
        const int idx = tid + NTHR1 * i;
        *reinterpret_cast<floatx4*>(&bs[idx / (TN / 4)][4 * (idx % (TN / 4))]) = bst[i];
      }
      __syncthreads();
      if (k0 + KC < a.rank) fetch_chunk(k0 + KC);
#pragma unroll
      for (int s = 0; s < KC / 2; ++s) {
        const float av = ys[2 * s + lh][32 * wr + ln];
        const float bv = bs[2 * s + lh][32 * wc + ln];
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc, 0, 0, 0);
      }
    }
  }
  __syncthreads();          // all operand reads done before the product overwrites the buffer
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    const int row = 32 * wr + 8 * (e >> 2) + 4 * lh + (e & 3);
    pt[row * PP + 32 * wc + ln] = acc[e];
  }
  __syncthreads();
  switch (pr.cfg.bits) {
    case 2: phase1_dispatch_block<2, WITH_ERR>(a, pr.cfg.block, z, pt, s_search, s_code, r0, c0, wreg); break;
    case 3: phase1_dispatch_block<3, WITH_ERR>(a, pr.cfg.block, z, pt, s_search, s_code, r0, c0, wreg); break;
    case 4: phase1_dispatch_block<4, WITH_ERR>(a, pr.cfg.block, z, pt, s_search, s_code, r0, c0, wreg); break;
    default: phase1_dispatch_block<8, WITH_ERR>(a, pr.cfg.block, z, pt, s_search, s_code, r0, c0, wreg); break;
  }
}

// The split-precision variant used by default: a workgroup keeps the planes of one 128-column stretch of B in LDS and
// walks `nb` consecutive 64-row bands of W with them, so the B planes (half of what a tile needs from memory) are
// fetched once per `nb` tiles, and the W quads and Y planes of band i + 1 are fetched while band i is being quantized.
// Launch: one-dimensional, batch * units8 workgroups, units = column stretches x groups of bands, rounded up to a
// multiple of 8; index decoded as (unit mod 8, problem, unit div 8) so that the problems of a batch that share a
// stretch of W run on one XCD at the same time.
template <bool WITH_ERR>
__global__ __launch_bounds__(NTHR1) void lowrank_blockquant_bands_kernel(PhaseArgs a, int units, int tiles_n, int nb) {
  constexpr int BPLANE = 2 * TN * KP;                     // bf16 elements: B hi, B lo
  constexpr int YPLANE = 2 * TM * KP;                     // Y hi, Y lo; shares its space with the product tile
  constexpr int PT_BYTES = TM * PP * 4 > YPLANE * 2 ? TM * PP * 4 : YPLANE * 2;
  __shared__ __attribute__((aligned(16))) __bf16 s_b[BPLANE];
  __shared__ __attribute__((aligned(16))) char s_yp[PT_BYTES];
  __shared__ __attribute__((aligned(16))) SearchEntry s_search[SEARCH_ENTRIES];
  __shared__ float s_code[WITH_ERR ? 256 : 1];
  __bf16* s_y = reinterpret_cast<__bf16*>(s_yp);
  float* pt = reinterpret_cast<float*>(s_yp);
  const int tid = threadIdx.x;
  const int slot8 = blockIdx.x >> 3;
  const int z = slot8 % a.batch;
  const int unit = (int)(blockIdx.x & 7) + 8 * (slot8 / a.batch);
  if (unit >= units) return;                   // padding of the unit count to a multiple of 8
  const LoopProblem pr = a.prob[z];
  const int nbands = (int)((a.d + TM - 1) / TM);
  const int band0 = (unit / tiles_n) * nb;
  const int band1 = band0 + nb < nbands ? band0 + nb : nbands;
  const int64_t c0 = (int64_t)(unit % tiles_n) * TN;
  const int wave = tid >> 6, lane = tid & 63, ln = lane & 31, lh = lane >> 5;
  const int wr = wave >> 2, wc = wave & 3;      // 2 x 4 grid of 32x32 tiles

  const int slot = pr.cfg.bits == 2 ? 0 : pr.cfg.bits == 3 ? 1 : pr.cfg.bits == 4 ? 2 : 3;
  build_search_nosync(a.tables, slot, s_search);
  if constexpr (WITH_ERR)
    for (int i = tid; i < 256; i += NTHR1) s_code[i] = a.tables->code[slot][i];

  const int rk = (a.rank + 15) / 16 * 16;
  const int64_t dpad = (a.d + TM - 1) / TM * TM, kpad = (a.k + TN - 1) / TN * TN;
  const __bf16* gy = reinterpret_cast<const __bf16*>(a.packed) + (size_t)z * a.stridePacked;
  const __bf16* gb = gy + (size_t)2 * dpad * rk;
  const floatx4 zero4 = {0.f, 0.f, 0.f, 0.f};
  // lane parts of the addresses: 16-byte piece (tid & 7) of row tid / 8 of a plane; quad tid & 31 of row tid / 32 of W
  const uint32_t p_lane = (uint32_t)(((tid >> 3) * rk + 8 * (tid & 7)) * 2);
  const bool p_ok = 8 * (tid & 7) < rk;         // the rank fits one 64-deep chunk (checked by the launcher)
  const uint32_t w_lane = (uint32_t)(((tid >> 5) * a.k + 4 * (tid & 31)) * 4);
  const bool w_col_live = c0 + 4 * (tid & 31) < a.k;

  // B planes of this column stretch: rows 0..63 and 64..127 of hi and of lo, one piece each per thread
  {
    const char* bbase[4] = {reinterpret_cast<const char*>(gb + (size_t)c0 * rk),
                            reinterpret_cast<const char*>(gb + (size_t)(c0 + 64) * rk),
                            reinterpret_cast<const char*>(gb + (size_t)(kpad + c0) * rk),
                            reinterpret_cast<const char*>(gb + (size_t)(kpad + c0 + 64) * rk)};
    floatx4 bp[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) bp[i] = p_ok ? *reinterpret_cast<const floatx4*>(bbase[i] + p_lane) : zero4;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      *reinterpret_cast<floatx4*>(s_b + (size_t)((tid >> 3) + 64 * i) * KP + 8 * (tid & 7)) = bp[i];
  }

  float4 wnext[4];
  floatx4 ynext[2];
  auto prefetch = [&](int band) {
    const int64_t r0 = (int64_t)band * TM;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int64_t row_u = r0 + (NTHR1 / 32) * u;                       // uniform
      const char* base = reinterpret_cast<const char*>(a.W + (size_t)row_u * a.k + c0);
      wnext[u] = (row_u + (tid >> 5) < a.d && w_col_live) ? *reinterpret_cast<const float4*>(base + w_lane)
                                                           : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    const char* ybase[2] = {reinterpret_cast<const char*>(gy + (size_t)r0 * rk),
                            reinterpret_cast<const char*>(gy + (size_t)(dpad + r0) * rk)};
#pragma unroll
    for (int i = 0; i < 2; ++i) ynext[i] = p_ok ? *reinterpret_cast<const floatx4*>(ybase[i] + p_lane) : zero4;
  };
  prefetch(band0);

  for (int band = band0; band < band1; ++band) {
    const int64_t r0 = (int64_t)band * TM;
    __syncthreads();          // the previous band's epilogue is done with the product tile (first band: nothing)
#pragma unroll
    for (int i = 0; i < 2; ++i)
      *reinterpret_cast<floatx4*>(s_y + (size_t)((tid >> 3) + 64 * i) * KP + 8 * (tid & 7)) = ynext[i];
    float4 wcur[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) wcur[u] = wnext[u];
    __syncthreads();          // Y planes (and, first band, B planes and tables) visible
    if (band + 1 < band1) prefetch(band + 1);

    floatx16 acc;
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = 0.0f;
    const __bf16* yh = s_y + (size_t)(32 * wr + ln) * KP + 8 * lh;
    const __bf16* yl = yh + (size_t)TM * KP;
    const __bf16* bh = s_b + (size_t)(32 * wc + ln) * KP + 8 * lh;
    const __bf16* bl = bh + (size_t)TN * KP;
#pragma unroll
    for (int kg = 0; kg < KC2 / 16; ++kg) {
      if (16 * kg < rk) {
        const bf16x8 ah = *reinterpret_cast<const bf16x8*>(yh + 16 * kg), al = *reinterpret_cast<const bf16x8*>(yl + 16 * kg);
        const bf16x8 vh = *reinterpret_cast<const bf16x8*>(bh + 16 * kg), vl = *reinterpret_cast<const bf16x8*>(bl + 16 * kg);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, vh, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, vl, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, vh, acc, 0, 0, 0);
      }
    }
    __syncthreads();          // all reads of the Y planes done before the product overwrites them
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int row = 32 * wr + 8 * (e >> 2) + 4 * lh + (e & 3);
      pt[row * PP + 32 * wc + ln] = acc[e];
    }
    __syncthreads();
    switch (pr.cfg.bits) {
      case 2: phase1_dispatch_block<2, WITH_ERR>(a, pr.cfg.block, z, pt, s_search, s_code, r0, c0, wcur); break;
      case 3: phase1_dispatch_block<3, WITH_ERR>(a, pr.cfg.block, z, pt, s_search, s_code, r0, c0, wcur); break;
      case 4: phase1_dispatch_block<4, WITH_ERR>(a, pr.cfg.block, z, pt, s_search, s_code, r0, c0, wcur); break;
      default: phase1_dispatch_block<8, WITH_ERR>(a, pr.cfg.block, z, pt, s_search, s_code, r0, c0, wcur); break;
    }
  }
}

int launch_lowrank_blockquant(const PhaseArgs& a, bool with_err, hipStream_t st) {
  const int tiles_n = (int)((a.k + TN - 1) / TN);
  const int64_t nbands = (a.d + TM - 1) / TM;
  const int64_t tiles = (int64_t)tiles_n * nbands;
  if ((tiles + 7) / 8 * 8 * a.batch >= (1ll << 31)) return LQ_ERR_SHAPE;
  if (a.k > (1ll << 25)) return LQ_ERR_SHAPE;      // lane offsets within a tile (up to 63 rows apart) are 32-bit byte offsets
  // algorithmic bytes: W and the factors in, the quantized form out, per configuration (the scale part of the latter is
  // finished by the scale kernel that follows)
  prof::Scope ps(prof::LOWRANK_BLOCKQUANT, st,
                 (double)a.d * a.k * (4.0 * a.batch + a.quant_bytes_per_weight) + 4.0 * a.rank * (double)(a.d + a.k) * a.batch);
  const bool split = a.packed != nullptr;
  if (split && a.rank <= KC2) {
    // bands per workgroup: as many as leave a few thousand workgroups, at most 8
    int64_t nb = tiles * a.batch / 4096;
    nb = nb < 1 ? 1 : (nb > 8 ? 8 : nb);
    if (nb > nbands) nb = nbands;
    const int64_t units = (int64_t)tiles_n * ((nbands + nb - 1) / nb);
    const dim3 grid((unsigned)((units + 7) / 8 * 8 * a.batch));
    if (with_err) hipLaunchKernelGGL(lowrank_blockquant_bands_kernel<true>, grid, dim3(NTHR1), 0, st, a, (int)units, tiles_n, (int)nb);
    else hipLaunchKernelGGL(lowrank_blockquant_bands_kernel<false>, grid, dim3(NTHR1), 0, st, a, (int)units, tiles_n, (int)nb);
    LQ_HIP_TRY(hipGetLastError());
    return LQ_OK;
  }
  const dim3 grid((unsigned)((tiles + 7) / 8 * 8 * a.batch));
  if (split) {
    if (with_err) hipLaunchKernelGGL((lowrank_blockquant_kernel<true, true>), grid, dim3(NTHR1), 0, st, a, (int)tiles, tiles_n);
    else hipLaunchKernelGGL((lowrank_blockquant_kernel<false, true>), grid, dim3(NTHR1), 0, st, a, (int)tiles, tiles_n);
  } else {
    if (with_err) hipLaunchKernelGGL((lowrank_blockquant_kernel<true, false>), grid, dim3(NTHR1), 0, st, a, (int)tiles, tiles_n);
    else hipLaunchKernelGGL((lowrank_blockquant_kernel<false, false>), grid, dim3(NTHR1), 0, st, a, (int)tiles, tiles_n);
  }
  LQ_HIP_TRY(hipGetLastError());
  return LQ_OK;
}

// ------------------------------------------------------------------------------------------------
// Phase 2: one lane per block.
// WITH_ERR: phase 1 left full block records {s, e2, eq, q2}; otherwise only the block absmax values (4 B per block)
// and the error output is zero.
template <bool WITH_ERR>
__global__ __launch_bounds__(256) void scalequant_error_kernel(PhaseArgs a) {
  __shared__ float s_wave[4];
  __shared__ double s_sum[4];
  const int z = blockIdx.y, tid = threadIdx.x;
  const LoopProblem pr = a.prob[z];
  const int64_t nb = (a.d * a.k) / pr.cfg.block;
  const int64_t b = (int64_t)blockIdx.x * 256 + tid;
  double* part = a.err_part + (size_t)z * a.strideErrPart;
  if ((int64_t)blockIdx.x * 256 >= nb) {           // whole workgroup past this problem's blocks
    if (WITH_ERR && tid == 0) part[blockIdx.x] = 0.0;
    return;
  }
  BlockRec rec; rec.s = 0.f; rec.e2 = 0.f; rec.eq = 0.f; rec.q2 = 0.f;
  if (b < nb) {
    if (WITH_ERR) rec = a.blk[(size_t)z * a.strideBlk + b];
    else rec.s = reinterpret_cast<const float*>(a.blk + (size_t)z * a.strideBlk)[b];
  }
  const float vmax = group_max(rec.s, pr.cfg.scale_block, s_wave);
  const float sigma = vmax / (float)pr.levels;
  const float vhat = cast_group_scale(vmax, pr.cfg.v_dtype);
  double err = 0.0;
  if (b < nb) {
    const uint32_t idx = scale_index(rec.s, sigma, pr.levels);
    a.sidx[(size_t)z * a.strideSidx + b] = (uint8_t)idx;
    if ((b & (pr.cfg.scale_block - 1)) == 0) a.v[(size_t)z * a.strideV + b / pr.cfg.scale_block] = vhat;
    if constexpr (WITH_ERR) {
      const float shat = block_scale(idx, vhat, pr.levels);
      const double delta = (double)shat - (double)rec.s;
      err = (double)rec.e2 - 2.0 * delta * (double)rec.eq + delta * delta * (double)rec.q2;
      if (a.row_w) err *= (double)a.row_w[(b * pr.cfg.block) / a.k];
    }
  }
  if constexpr (WITH_ERR) {
    for (int off = 1; off < 64; off <<= 1) err += __shfl_xor(err, off);
    if ((tid & 63) == 0) s_sum[tid >> 6] = err;
    __syncthreads();
    if (tid == 0) part[blockIdx.x] = (s_sum[0] + s_sum[1]) + (s_sum[2] + s_sum[3]);
  }
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

int launch_scalequant_error(const PhaseArgs& a, int min_block, bool with_err, hipStream_t st) {
  const int64_t nwg = err_partials_per_problem(a.d * a.k, min_block);
  prof::Scope ps(prof::SCALEQUANT_ERROR, st, (double)(a.d * a.k / min_block) * (with_err ? 17.0 : 5.0) * a.batch);
  if (with_err) hipLaunchKernelGGL(scalequant_error_kernel<true>, dim3((unsigned)nwg, (unsigned)a.batch), dim3(256), 0, st, a);
  else hipLaunchKernelGGL(scalequant_error_kernel<false>, dim3((unsigned)nwg, (unsigned)a.batch), dim3(256), 0, st, a);
  LQ_HIP_TRY(hipGetLastError());
  if (with_err) {
    hipLaunchKernelGGL(error_finalize_kernel, dim3((unsigned)a.batch), dim3(256), 0, st, (const double*)a.err_part,
                       a.strideErrPart, nwg, a.err_out, a.strideErrOut);
    LQ_HIP_TRY(hipGetLastError());
  }
  return LQ_OK;
}

// ------------------------------------------------------------------------------------------------
// Phase 3: one quad (4 consecutive weights) per lane and step, so each wavefront instruction reads / writes
// 1 KB of contiguous fp32.
// A workgroup takes a stretch of 512 quads (RES_U = 2 per lane) of W and keeps it in registers for several problems of
// the batch, so W crosses the L2 / L1 fabric a few times per batch instead of once per problem (R is 4 B per weight
// out; W would be another 4 B per weight in).
constexpr int RES_U = 2;

struct ResidualFetch {                 // what one lane needs of one problem besides W
  uint32_t cw[RES_U];                  // packed codes of the quad (4 * bits bits)
  uint32_t si[RES_U];
  float vv[RES_U];
};

__device__ __forceinline__ uint32_t load_quad_word(const uint8_t* __restrict__ codes, int64_t quad, int bits) {
  if (bits == 8) return *reinterpret_cast<const uint32_t*>(codes + quad * 4);
  if (bits == 4) return *reinterpret_cast<const uint16_t*>(codes + quad * 2);
  if (bits == 2) return codes[quad];
  const int64_t byte = (quad * 3) >> 1;     // 3 bits: 12 bits starting at bit 12*quad, nibble-aligned
  return (((uint32_t)codes[byte] | ((uint32_t)codes[byte + 1] << 8)) >> ((quad & 1) * 4)) & 0xfffu;
}

__device__ __forceinline__ void residual_fetch(const PhaseArgs& a, const LoopProblem& pr, int z, const int64_t (&qq)[RES_U],
                                               ResidualFetch& f) {
  const int qpb_shift = __builtin_ctz(pr.cfg.block / 4), sb_shift = __builtin_ctz(pr.cfg.scale_block);
  const uint8_t* codes = a.codes + (size_t)z * a.strideCodes;
  const uint8_t* sidx = a.sidx + (size_t)z * a.strideSidx;
  const float* v = a.v + (size_t)z * a.strideV;
#pragma unroll
  for (int u = 0; u < RES_U; ++u) {
    const int64_t blk = qq[u] >> qpb_shift;
    f.cw[u] = load_quad_word(codes, qq[u], pr.cfg.bits);
    f.si[u] = sidx[blk];
    f.vv[u] = v[blk >> sb_shift];
  }
}

// A workgroup serves RES_G problems for its stretch of W: every load is issued first, then everything is computed
// and stored, and the wavefront ends without ever waiting for a store.  (Loads and stores share one in-order
// counter on this architecture, so a wait for a load also waits for every store issued before it: a loop that
// alternates loads and stores runs at the pace of the store latency.)  Measured on 36 x 4096 x 11008: 3.7 TB/s
// written; a kernel that only stores reaches 5.7 - 6.9 TB/s, one that loads 2 B per quad before storing 3.8 TB/s.  The problem group is the fastest launch
// index, so the groups of a batch that read the same stretch of W run together and share it in L2.
// The lo plane of the fp16 residual: what the rounding of sv to hi dropped, times 2^11, rounded to the upper byte of
// its fp16 form (sign, five exponent bits, two fraction bits; round to nearest even on the bit pattern, which carries
// into the exponent where it has to).  |sv - hi| <= 16 for |sv| <= 65504, so the scaled value stays below 2^15 + 1.
__device__ __forceinline__ uint32_t lo_plane_byte(float sv, _Float16 hi) {
  const _Float16 l = (_Float16)((sv - (float)hi) * 2048.0f);
  const uint32_t b = (uint32_t)__builtin_bit_cast(uint16_t, l);
  return (b + 0x7Fu + ((b >> 8) & 1u)) >> 8;
}

constexpr int RES_G = 6;

__global__ __launch_bounds__(256) void residual_kernel(PhaseArgs a, int groups) {
  __shared__ float s_code[4][256];
  const int tid = threadIdx.x;
  for (int i = tid; i < 1024; i += 256) s_code[i >> 8][i & 255] = a.tables->code[i >> 8][i & 255];
  const int zfirst = (int)(blockIdx.x % groups) * RES_G;
  const int64_t nquads = (a.d * a.k) >> 2;
  const int64_t q0 = (int64_t)(blockIdx.x / groups) * (256 * RES_U) + tid;
  int64_t qq[RES_U];                   // clamped quad indices (loads stay in bounds; stores are guarded)
  float4 w[RES_U];
#pragma unroll
  for (int u = 0; u < RES_U; ++u) {
    const int64_t quad = q0 + 256 * u;
    qq[u] = quad < nquads ? quad : nquads - 1;
    w[u] = *reinterpret_cast<const float4*>(a.W + (qq[u] << 2));
  }
  LoopProblem pr[RES_G];
  ResidualFetch f[RES_G];
#pragma unroll
  for (int gI = 0; gI < RES_G; ++gI) {
    const int z = zfirst + gI < a.batch ? zfirst + gI : a.batch - 1;      // clamped: loaded, never stored
    pr[gI] = a.prob[z];
    residual_fetch(a, pr[gI], z, qq, f[gI]);
  }
  float srow[RES_U];
  float4 cs[RES_U];
  if (a.sr) {
#pragma unroll
    for (int u = 0; u < RES_U; ++u) {
      const int64_t e0 = qq[u] << 2;
      srow[u] = a.sr[e0 / a.k];
      cs[u] = *reinterpret_cast<const float4*>(a.sc + e0 % a.k);
    }
  }
  __syncthreads();                     // code books in LDS
#pragma unroll
  for (int gI = 0; gI < RES_G; ++gI) {
    const int z = zfirst + gI;
    if (z >= a.batch) break;
    const int bits = pr[gI].cfg.bits, levels = pr[gI].levels;
    const float* code = s_code[bits == 2 ? 0 : bits == 3 ? 1 : bits == 4 ? 2 : 3];
    const uint32_t mask = (1u << bits) - 1u;
    float* R = a.R ? a.R + (size_t)z * a.strideR : nullptr;
    _Float16* R16 = a.R16 ? reinterpret_cast<_Float16*>(a.R16) + (size_t)z * a.strideR : nullptr;
    uint8_t* R16lo = a.R16lo ? a.R16lo + (size_t)z * a.strideR : nullptr;
    float* Qd = a.Qd ? a.Qd + (size_t)z * a.strideQd : nullptr;
#pragma unroll
    for (int u = 0; u < RES_U; ++u) {
      const int64_t quad = q0 + 256 * u;
      if (quad >= nquads) break;
      const float sh = block_scale(f[gI].si[u], f[gI].vv[u], levels);
      const uint32_t cw = f[gI].cw[u];
      float4 qv, rv;
      qv.x = code[cw & mask] * sh; qv.y = code[(cw >> bits) & mask] * sh;
      qv.z = code[(cw >> (2 * bits)) & mask] * sh; qv.w = code[(cw >> (3 * bits)) & mask] * sh;
      rv.x = w[u].x - qv.x; rv.y = w[u].y - qv.y; rv.z = w[u].z - qv.z; rv.w = w[u].w - qv.w;
      if (a.sr) {
        rv.x = srow[u] * rv.x * cs[u].x; rv.y = srow[u] * rv.y * cs[u].y;
        rv.z = srow[u] * rv.z * cs[u].z; rv.w = srow[u] * rv.w * cs[u].w;
      }
      if (R) __builtin_nontemporal_store(floatx4{rv.x, rv.y, rv.z, rv.w}, reinterpret_cast<floatx4*>(R + (quad << 2)));
      if (R16) {
        const float lim = 65504.0f;        // largest fp16: out-of-range entries saturate instead of becoming infinite
        const float sv[4] = {__builtin_amdgcn_fmed3f(rv.x * a.r_scale, -lim, lim), __builtin_amdgcn_fmed3f(rv.y * a.r_scale, -lim, lim),
                             __builtin_amdgcn_fmed3f(rv.z * a.r_scale, -lim, lim), __builtin_amdgcn_fmed3f(rv.w * a.r_scale, -lim, lim)};
        halfx4 h;
        uint32_t l = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          h[e] = (_Float16)sv[e];
          l |= lo_plane_byte(sv[e], h[e]) << (8 * e);
        }
        // streamed out: nothing reads these lines before they have left the caches anyway
        __builtin_nontemporal_store(h, reinterpret_cast<halfx4*>(R16 + (quad << 2)));
        if (R16lo) __builtin_nontemporal_store(l, reinterpret_cast<uint32_t*>(R16lo + (quad << 2)));
      }
      if (Qd) __builtin_nontemporal_store(floatx4{qv.x, qv.y, qv.z, qv.w}, reinterpret_cast<floatx4*>(Qd + (quad << 2)));
    }
  }
}

// The form of phase 3 that the warm iterations use: only the scaled fp16 planes of the residual are written.  A
// workgroup owns one stretch of W (RP_U runs of 8 consecutive weights per lane, kept in registers) and walks through the
// problems of the batch with it, so W is read once per batch; the codes and scales of problem z + 1 are fetched before
// problem z is computed and stored, so no load ever waits behind a store; every store of a plane is 16 bytes per lane,
// 1 KB contiguous per wavefront, and is streamed past the caches (measured: the kernel is bound by the bytes it moves;
// per-problem workgroups that re-read W, in either launch order, took 1.29 - 1.36 ms per 36 problems where this takes
// less).
constexpr int RP_U = 2;
typedef _Float16 halfx8r __attribute__((ext_vector_type(8)));
typedef uint32_t uintx2r __attribute__((ext_vector_type(2)));

struct PlaneFetch { uint32_t cw[RP_U][2]; uint32_t si[RP_U]; float vv[RP_U]; };

template <int BITS>
__device__ __forceinline__ void residual_planes_fetch(const PhaseArgs& a, int blk_shift, int sb_shift, int z,
                                                      const int64_t (&oct)[RP_U], PlaneFetch& f) {
  const uint8_t* codes = a.codes + (size_t)z * a.strideCodes;
  const uint8_t* sidx = a.sidx + (size_t)z * a.strideSidx;
  const float* v = a.v + (size_t)z * a.strideV;
#pragma unroll
  for (int u = 0; u < RP_U; ++u) {
    const int64_t o = oct[u];
    f.cw[u][1] = 0;
    if constexpr (BITS == 8) {
      const uint2 c2 = *reinterpret_cast<const uint2*>(codes + o * 8);
      f.cw[u][0] = c2.x; f.cw[u][1] = c2.y;
    } else if constexpr (BITS == 4) {
      f.cw[u][0] = *reinterpret_cast<const uint32_t*>(codes + o * 4);
    } else if constexpr (BITS == 2) {
      f.cw[u][0] = *reinterpret_cast<const uint16_t*>(codes + o * 2);
    } else {       // 24 bits at byte 3 * oct: a 16-bit and an 8-bit piece, the 16-bit one at the even address
      const int64_t b = o * 3;
      const uint32_t h = *reinterpret_cast<const uint16_t*>(codes + b + (o & 1));
      const uint32_t q = codes[b + ((o & 1) ? 0 : 2)];
      f.cw[u][0] = (o & 1) ? (q | (h << 8)) : (h | (q << 16));
    }
    const int64_t blk = o >> blk_shift;
    f.si[u] = sidx[blk];
    f.vv[u] = v[blk >> sb_shift];
  }
}

// zmask: the problems of the batch (bit z) this launch serves; all of them have BITS code bits.
// The loop over them is unrolled twice over two fetch buffers and has no conditional load or store inside (past the
// last problem it fetches the last one again; lanes past the end of the matrix work on the last run of 8 weights again
// and store the same values as its owner), so the compiler's wait for the loads of problem i + 1 never includes the
// stores of problem i that were issued after them.
template <int BITS, bool WEIGHTED>
__global__ __launch_bounds__(256) void residual_planes_kernel(PhaseArgs a, uint64_t zmask) {
  __shared__ float s_code[1 << BITS];
  __shared__ int s_list[64];
  __shared__ int s_par[64][4];         // per problem: log2(B0 / 8), log2(B1), levels
  const int tid = threadIdx.x;
  for (int i = tid; i < (1 << BITS); i += 256) s_code[i] = a.tables->code[Slot<BITS>::value][i];
  if (tid < 64 && ((zmask >> tid) & 1)) {
    const LoopProblem p = a.prob[tid];
    s_list[__builtin_popcountll(zmask & ((1ull << tid) - 1ull))] = tid;
    s_par[tid][0] = __builtin_ctz(p.cfg.block / 8); s_par[tid][1] = __builtin_ctz(p.cfg.scale_block); s_par[tid][2] = p.levels;
  }
  const int count = __builtin_popcountll(zmask);
  const int64_t nocts = (a.d * a.k) >> 3;
  const int64_t oct0 = (int64_t)blockIdx.x * (256 * RP_U) + tid;
  int64_t oct[RP_U];
  float wv[RP_U][8], cv[RP_U][8], srow[RP_U];
#pragma unroll
  for (int u = 0; u < RP_U; ++u) {
    oct[u] = oct0 + 256 * u < nocts ? oct0 + 256 * u : nocts - 1;
    const float4 w0 = *reinterpret_cast<const float4*>(a.W + (oct[u] << 3));
    const float4 w1 = *reinterpret_cast<const float4*>(a.W + (oct[u] << 3) + 4);
    wv[u][0] = w0.x; wv[u][1] = w0.y; wv[u][2] = w0.z; wv[u][3] = w0.w;
    wv[u][4] = w1.x; wv[u][5] = w1.y; wv[u][6] = w1.z; wv[u][7] = w1.w;
    if constexpr (WEIGHTED) {
      const int64_t e0 = oct[u] << 3;
      srow[u] = a.sr[e0 / a.k];
      const float4 c0 = *reinterpret_cast<const float4*>(a.sc + e0 % a.k);
      const float4 c1 = *reinterpret_cast<const float4*>(a.sc + e0 % a.k + 4);
      cv[u][0] = c0.x; cv[u][1] = c0.y; cv[u][2] = c0.z; cv[u][3] = c0.w;
      cv[u][4] = c1.x; cv[u][5] = c1.y; cv[u][6] = c1.z; cv[u][7] = c1.w;
    }
  }
  __syncthreads();                     // code book, problem list and parameters in LDS
  const float lim = 65504.0f;          // largest fp16: out-of-range entries saturate instead of becoming infinite
  constexpr uint32_t mask = (1u << BITS) - 1u;
  auto fetch = [&](int i, PlaneFetch& f) {
    const int z = s_list[i < count ? i : count - 1];
    residual_planes_fetch<BITS>(a, s_par[z][0], s_par[z][1], z, oct, f);
  };
  auto emit = [&](int i, const PlaneFetch& f) {
    const int z = s_list[i];
    const int levels = s_par[z][2];
    _Float16* hi = reinterpret_cast<_Float16*>(a.R16) + (size_t)z * a.strideR;
    uint8_t* lo = a.R16lo + (size_t)z * a.strideR;
#pragma unroll
    for (int u = 0; u < RP_U; ++u) {
      const float sh = block_scale(f.si[u], f.vv[u], levels);
      halfx8r h;
      uint32_t l[2] = {0u, 0u};
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const uint32_t c = BITS == 8 ? (f.cw[u][e >> 2] >> (8 * (e & 3))) & mask : (f.cw[u][0] >> (BITS * e)) & mask;
        float r = wv[u][e] - s_code[c] * sh;
        if constexpr (WEIGHTED) r = srow[u] * r * cv[u][e];
        const float sv = __builtin_amdgcn_fmed3f(r * a.r_scale, -lim, lim);
        h[e] = (_Float16)sv;
        l[e >> 2] |= lo_plane_byte(sv, h[e]) << (8 * (e & 3));
      }
      __builtin_nontemporal_store(h, reinterpret_cast<halfx8r*>(hi + (oct[u] << 3)));
      __builtin_nontemporal_store(uintx2r{l[0], l[1]}, reinterpret_cast<uintx2r*>(lo + (oct[u] << 3)));
    }
  };
  PlaneFetch fa, fb;
  fetch(0, fa);
  for (int i = 0;;) {
    fetch(i + 1, fb);
    emit(i, fa);
    if (++i >= count) break;
    fetch(i + 1, fa);
    emit(i, fb);
    if (++i >= count) break;
  }
}

template <int BITS>
static void launch_residual_planes(const PhaseArgs& a, uint64_t zmask, dim3 grid, hipStream_t st) {
  if (a.sr) hipLaunchKernelGGL((residual_planes_kernel<BITS, true>), grid, dim3(256), 0, st, a, zmask);
  else hipLaunchKernelGGL((residual_planes_kernel<BITS, false>), grid, dim3(256), 0, st, a, zmask);
}

int launch_residual(const PhaseArgs& a, hipStream_t st) {
  const int64_t nquads = (a.d * a.k) >> 2;
  const int groups = (a.batch + RES_G - 1) / RES_G;
  const int64_t nwg = (nquads + 256 * RES_U - 1) / (256 * RES_U) * groups;
  if (nwg >= (1ll << 31)) return LQ_ERR_SHAPE;
  // R (or dense Q) out per problem, the quantized form in per problem, W in once
  const double out_bytes = (a.R ? 4.0 : 0.0) + (a.R16 ? 2.0 : 0.0) + (a.R16 && a.R16lo ? 1.0 : 0.0) + (a.Qd ? 4.0 : 0.0);
  prof::Scope ps(prof::RESIDUAL, st, (double)a.d * a.k * (out_bytes * a.batch + 4.0 + a.quant_bytes_per_weight));
  if (a.R16 && a.R16lo && !a.R && !a.Qd && ((a.d * a.k) & 7) == 0 && a.batch <= 64 && a.bits_host) {
    const int64_t nwg2 = (((a.d * a.k) >> 3) + 256 * RP_U - 1) / (256 * RP_U);
    if (nwg2 >= (1ll << 31)) return LQ_ERR_SHAPE;
    const dim3 grid((unsigned)nwg2);
    // one launch per code width present in the batch (the kernel's loads depend on it)
    uint64_t m[4] = {0, 0, 0, 0};
    for (int z = 0; z < a.batch; ++z) {
      const int b = a.bits_host[z];
      m[b == 2 ? 0 : b == 3 ? 1 : b == 4 ? 2 : 3] |= 1ull << z;
    }
    if (m[0]) launch_residual_planes<2>(a, m[0], grid, st);
    if (m[1]) launch_residual_planes<3>(a, m[1], grid, st);
    if (m[2]) launch_residual_planes<4>(a, m[2], grid, st);
    if (m[3]) launch_residual_planes<8>(a, m[3], grid, st);
    LQ_HIP_TRY(hipGetLastError());
    return LQ_OK;
  }
  hipLaunchKernelGGL(residual_kernel, dim3((unsigned)nwg), dim3(256), 0, st, a, groups);
  LQ_HIP_TRY(hipGetLastError());
  return LQ_OK;
}

}  // namespace lq
