// Device-side building blocks of the NF quantizer (Sections 2.2 and 3.2), shared by the stand-alone
// quantize / dequantize kernels and by the fused kernels of the decomposition loop.
//
// All arithmetic that decides a code or a scale index is written as single correctly rounded fp32
// operations (the library is compiled with -ffp-contract=off), so results are reproducible bit for bit:
//   normalised weight  fl32(u * fl32(1/s))           code = #{i : x >= thr[i]}
//   sigma = fl32(v / levels)   index = clamp(rne(fl32(s / sigma)), 0, levels)   s^ = fl32(index * sigma)
#pragma once

#include <hip/hip_fp16.h>

#include "lq_internal.h"

namespace lq {

typedef NfTables DevTables;
// Device address of the tables on the current device (uploads them on first use).
int device_tables(const DevTables** out);

template <int BITS>
struct Slot;
template <> struct Slot<2> { static constexpr int value = 0; };
template <> struct Slot<3> { static constexpr int value = 1; };
template <> struct Slot<4> { static constexpr int value = 2; };
template <> struct Slot<8> { static constexpr int value = 3; };

// LDS copy of one bit width's tables.
struct LdsTables {
  float code[256];
  float thr[260];
  uint8_t lut[512];
};

// Copies the tables of one bit width (slot) into LDS.  The caller places a barrier before the first use.
__device__ inline void load_tables_slot_nosync(const DevTables* __restrict__ tab, int slot, LdsTables& t) {
  for (int i = threadIdx.x; i < 256; i += blockDim.x) t.code[i] = tab->code[slot][i];
  for (int i = threadIdx.x; i < 260; i += blockDim.x) t.thr[i] = tab->thr[slot][i];
  for (int i = threadIdx.x; i < 128; i += blockDim.x)
    reinterpret_cast<uint32_t*>(t.lut)[i] = reinterpret_cast<const uint32_t*>(tab->lut[slot])[i];
}
__device__ inline void load_tables_slot(const DevTables* __restrict__ tab, int slot, LdsTables& t) {
  load_tables_slot_nosync(tab, slot, t);
  __syncthreads();
}
template <int BITS>
__device__ inline void load_tables(const DevTables* __restrict__ tab, LdsTables& t) {
  load_tables_slot(tab, Slot<BITS>::value, t);
}

// Nearest code with ties to the lower index = number of thresholds <= x.
// 2 and 3 bits: the thresholds live in registers and are counted.  4 and 8 bits: a 512-bucket table in LDS
// gives the count of thresholds safely below x's bucket; at most two thresholds (8 bits) or one (4 bits, whose
// thresholds are more than twenty buckets apart) remain to be compared.  NaN compares false everywhere and lands
// on code 0 either way.
template <int BITS>
struct Thresholds {
  float r[(1 << BITS) - 1];
  __device__ explicit Thresholds(const LdsTables& t) {
#pragma unroll
    for (int i = 0; i < (1 << BITS) - 1; ++i) r[i] = t.thr[i];
  }
  __device__ inline uint32_t nearest(float x) const {
    uint32_t c = 0;
#pragma unroll
    for (int i = 0; i < (1 << BITS) - 1; ++i) c += (x >= r[i]) ? 1u : 0u;
    return c;
  }
};
template <int COMPARES>
struct BucketSearch {
  const LdsTables& t;
  __device__ explicit BucketSearch(const LdsTables& tt) : t(tt) {}
  __device__ inline uint32_t nearest(float x) const {
    int j = (int)fmaf(x, 256.0f, 256.0f);
    j = j < 0 ? 0 : (j > 511 ? 511 : j);
    const uint32_t c0 = t.lut[j];
    uint32_t c = c0 + ((x >= t.thr[c0]) ? 1u : 0u);
    if constexpr (COMPARES == 2) c += (x >= t.thr[c0 + 1]) ? 1u : 0u;
    return c;
  }
};
template <> struct Thresholds<4> : BucketSearch<1> { __device__ explicit Thresholds(const LdsTables& tt) : BucketSearch<1>(tt) {} };
template <> struct Thresholds<8> : BucketSearch<2> { __device__ explicit Thresholds(const LdsTables& tt) : BucketSearch<2>(tt) {} };

// ---- reductions over the QPB = 4, 8, 16 or 32 consecutive lanes that hold one block (aligned groups) ----
// Cross-lane moves by DPP: quad_perm for the two steps inside a quad; after those every quad is uniform, so the
// mirror of a half row swaps the two quads of an 8-lane group and the mirror of a row the two halves of a 16-lane
// group.  Only the last step of a 32-lane group goes through the LDS crossbar.
constexpr int DPP_QUAD_XOR1 = 0xB1, DPP_QUAD_XOR2 = 0x4E, DPP_ROW_HALF_MIRROR = 0x141, DPP_ROW_MIRROR = 0x140;
template <int CTRL>
__device__ __forceinline__ float dpp_move(float x) {
  return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, x), CTRL, 0xf, 0xf, true));
}
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_move_u32(uint32_t x) {
  return (uint32_t)__builtin_amdgcn_mov_dpp((int)x, CTRL, 0xf, 0xf, true);
}

template <int QPB>
__device__ __forceinline__ float group_max_lanes(float x) {
  x = fmaxf(x, dpp_move<DPP_QUAD_XOR1>(x));
  x = fmaxf(x, dpp_move<DPP_QUAD_XOR2>(x));
  if constexpr (QPB >= 8) x = fmaxf(x, dpp_move<DPP_ROW_HALF_MIRROR>(x));
  if constexpr (QPB >= 16) x = fmaxf(x, dpp_move<DPP_ROW_MIRROR>(x));
  if constexpr (QPB >= 32) x = fmaxf(x, __shfl_xor(x, 16));
  return x;
}
template <int QPB>
__device__ __forceinline__ float group_sum_lanes(float x) {
  x += dpp_move<DPP_QUAD_XOR1>(x);
  x += dpp_move<DPP_QUAD_XOR2>(x);
  if constexpr (QPB >= 8) x += dpp_move<DPP_ROW_HALF_MIRROR>(x);
  if constexpr (QPB >= 16) x += dpp_move<DPP_ROW_MIRROR>(x);
  if constexpr (QPB >= 32) x += __shfl_xor(x, 16);
  return x;
}

__device__ inline float run_absmax(const float (&t)[16]) {
  float m = 0.0f;
#pragma unroll
  for (int j = 0; j < 16; ++j) m = fmaxf(m, fabsf(t[j]));
  return m;
}

// fl32(1/s); 0 for an all-zero block or when the reciprocal overflows.
__device__ inline float safe_reciprocal(float s) {
  float r = 0.0f;
  if (s > 0.0f) {
    r = 1.0f / s;
    if (isinf(r)) r = 0.0f;
  }
  return r;
}

// ---- packed code stream: code j of run `run` occupies bits [(16*run + j)*BITS, +BITS) ------------
template <int BITS>
__device__ inline void store_codes(uint8_t* __restrict__ codes, int64_t run, const uint32_t (&c)[16]) {
  if constexpr (BITS == 8) {
    uint4 w;
    w.x = c[0] | (c[1] << 8) | (c[2] << 16) | (c[3] << 24);
    w.y = c[4] | (c[5] << 8) | (c[6] << 16) | (c[7] << 24);
    w.z = c[8] | (c[9] << 8) | (c[10] << 16) | (c[11] << 24);
    w.w = c[12] | (c[13] << 8) | (c[14] << 16) | (c[15] << 24);
    *reinterpret_cast<uint4*>(codes + run * 16) = w;
  } else {
    uint64_t w = 0;
#pragma unroll
    for (int j = 0; j < 16; ++j) w |= (uint64_t)c[j] << (j * BITS);
    if constexpr (BITS == 4) {
      *reinterpret_cast<uint2*>(codes + run * 8) = make_uint2((uint32_t)w, (uint32_t)(w >> 32));
    } else if constexpr (BITS == 2) {
      *reinterpret_cast<uint32_t*>(codes + run * 4) = (uint32_t)w;
    } else {   // 3 bits: 48 bits, 2-byte aligned
      uint16_t* p = reinterpret_cast<uint16_t*>(codes + run * 6);
      p[0] = (uint16_t)w; p[1] = (uint16_t)(w >> 16); p[2] = (uint16_t)(w >> 32);
    }
  }
}

template <int BITS>
__device__ inline void load_codes(const uint8_t* __restrict__ codes, int64_t run, uint32_t (&c)[16]) {
  if constexpr (BITS == 8) {
    const uint4 w = *reinterpret_cast<const uint4*>(codes + run * 16);
    const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
    for (int j = 0; j < 16; ++j) c[j] = (ww[j >> 2] >> ((j & 3) * 8)) & 0xffu;
  } else {
    uint64_t w;
    if constexpr (BITS == 4) {
      const uint2 u = *reinterpret_cast<const uint2*>(codes + run * 8);
      w = (uint64_t)u.x | ((uint64_t)u.y << 32);
    } else if constexpr (BITS == 2) {
      w = *reinterpret_cast<const uint32_t*>(codes + run * 4);
    } else {
      const uint16_t* p = reinterpret_cast<const uint16_t*>(codes + run * 6);
      w = (uint64_t)p[0] | ((uint64_t)p[1] << 16) | ((uint64_t)p[2] << 32);
    }
#pragma unroll
    for (int j = 0; j < 16; ++j) c[j] = (uint32_t)(w >> (j * BITS)) & ((1u << BITS) - 1u);
  }
}

// ---- quad layout: one lane holds 4 consecutive weights, 4 lanes a 16-weight run, so that every wavefront
// load / store covers one contiguous stretch.  Codes of quad `quad` occupy bits [quad*4*BITS, +4*BITS).
template <int BITS>
__device__ inline void load_quad_codes(const uint8_t* __restrict__ codes, int64_t quad, uint32_t (&c)[4]) {
  uint32_t w;
  if constexpr (BITS == 8) w = *reinterpret_cast<const uint32_t*>(codes + quad * 4);
  else if constexpr (BITS == 4) w = *reinterpret_cast<const uint16_t*>(codes + quad * 2);
  else if constexpr (BITS == 2) w = codes[quad];
  else {   // 3 bits: 12 bits starting at bit 12*quad = byte floor(1.5*quad), nibble-aligned
    const int64_t byte = (quad * 3) >> 1;
    w = ((uint32_t)codes[byte] | ((uint32_t)codes[byte + 1] << 8)) >> ((quad & 1) * 4);
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) c[j] = (w >> (j * BITS)) & ((1u << BITS) - 1u);
}

// ---- second-level (integer) scale quantization -------------------------------------------------
// Maximum over the `width` (power of two, <= 64, aligned) consecutive lanes of a wavefront: DPP moves up to 16 lanes
// (quad permutes, then half-row and row mirrors, which act as xor 4 and xor 8 on quad-uniform values), the LDS
// crossbar beyond.  `width` is uniform, so the branches are too.
__device__ __forceinline__ float lanes_max(float x, int width) {
  if (width > 1) x = fmaxf(x, dpp_move<DPP_QUAD_XOR1>(x));
  if (width > 2) x = fmaxf(x, dpp_move<DPP_QUAD_XOR2>(x));
  if (width > 4) x = fmaxf(x, dpp_move<DPP_ROW_HALF_MIRROR>(x));
  if (width > 8) x = fmaxf(x, dpp_move<DPP_ROW_MIRROR>(x));
  if (width > 16) x = fmaxf(x, __shfl_xor(x, 16));
  if (width > 32) x = fmaxf(x, __shfl_xor(x, 32));
  return x;
}

// Maximum over the `width` consecutive lanes (power of two, 16..256, aligned) that hold one scale
// group; the workgroup has 256 threads.  s_wave: 4 floats of LDS.  Contains barriers when
// width > 64, so every thread of the workgroup must call it.
__device__ inline float group_max(float x, int width, float* s_wave) {
  x = lanes_max(x, width < 64 ? width : 64);
  if (width > 64) {
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) s_wave[wave] = x;
    __syncthreads();
    const int per = width >> 6;             // waves per group: 2 or 4
    const int base = wave & ~(per - 1);
    float m = s_wave[base];
    for (int i = 1; i < per; ++i) m = fmaxf(m, s_wave[base + i]);
    x = m;
    __syncthreads();
  }
  return x;
}

__device__ inline uint32_t scale_index(float s, float sigma, int levels) {
  if (!(sigma > 0.0f)) return 0u;
  float r = rintf(s / sigma);
  r = fminf(fmaxf(r, 0.0f), (float)levels);
  return (uint32_t)r;
}

__device__ inline float block_scale(uint32_t idx, float v_stored, int levels) {
  const float sigma = v_stored / (float)levels;
  return (float)idx * sigma;
}

// cast(v, b2): round to nearest even into the storage type, returned as fp32.
__device__ inline float cast_group_scale(float v, int v_dtype) {
  if (v_dtype == LQ_V_BF16) {
    uint32_t u = __float_as_uint(v);
    if ((u & 0x7f800000u) != 0x7f800000u) {
      u += 0x7fffu + ((u >> 16) & 1u);
      u &= 0xffff0000u;
    }
    return __uint_as_float(u);
  }
  if (v_dtype == LQ_V_FP16) return __half2float(__float2half_rn(v));
  return v;
}

}  // namespace lq
