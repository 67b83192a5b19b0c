// Internal declarations shared by the host orchestration and the HIP kernels of the LQ library.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/lq.h"

namespace lq {

// ---- error plumbing -------------------------------------------------------------------------
void set_last_hip_error(int e);
#define LQ_HIP_TRY(expr)                                   \
  do {                                                     \
    hipError_t e__ = (expr);                               \
    if (e__ != hipSuccess) {                               \
      ::lq::set_last_hip_error((int)e__);                  \
      return LQ_ERR_HIP;                                   \
    }                                                      \
  } while (0)
#define LQ_TRY(expr)                 \
  do {                               \
    int s__ = (expr);                \
    if (s__ != LQ_OK) return s__;    \
  } while (0)

// ---- configuration helpers ------------------------------------------------------------------
// Normalised copy (scale_bits 0 -> 8) and validity (Section 3.2 tuple, supported subset).
lq_config normalized(lq_config c);
bool config_supported(const lq_config& c);
inline int scale_levels(const lq_config& c) { return (1 << (c.scale_bits - 1)) - 1; }
inline int v_bits(const lq_config& c) { return c.v_dtype == LQ_V_FP32 ? 32 : 16; }
inline int64_t num_blocks(int64_t n, const lq_config& c) { return n / c.block; }
inline int64_t num_groups(int64_t n, const lq_config& c) {
  return (num_blocks(n, c) + c.scale_block - 1) / c.scale_block;
}

// ---- code-book tables (host side, Section 2.2) ----------------------------------------------
// Slot of a supported bit width in the device tables: 2->0, 3->1, 4->2, 8->3, otherwise -1.
int bits_slot(int bits);
// code[i]: value of code i.  thr[i], i < 2^bits-1: smallest fp32 strictly above the midpoint of
// code i and code i+1, so that (number of thr <= x) is the nearest code with ties to the lower one.
// lut[j], j = floor((x + 1) * 256) clamped to [0, 511]: number of thresholds that lie safely below bucket j,
// built so that at most two further thresholds can be <= any x that lands in the bucket.  The code of x is
// then lut[j] + (x >= thr[lut[j]]) + (x >= thr[lut[j] + 1]).  thr is padded with +inf.
struct NfTables {
  float code[4][256];
  float thr[4][260];
  uint8_t lut[4][512];
};
typedef NfTables HostTables;
const HostTables& host_tables();
int host_codebook(int bits, float* out);   // any bits in 2..8
// Uploads the tables to the current device once.  Returns lq_status.
int ensure_device_tables();

// ---- kernel launchers: NF quantization (nf_kernels.hip) -------------------------------------
// Per-block record written by the block-quantization pass: absmax and the three weighted sums
// needed to evaluate sum w (t - q s^)^2 once the reconstructed scale s^ is known.
struct BlockRec {
  float s;    // exact absmax of the block
  float e2;   // sum_j w_j (t_j - q_j s)^2
  float eq;   // sum_j w_j (t_j - q_j s) q_j
  float q2;   // sum_j w_j q_j^2
};

// Stand-alone Quantize(x, c) in one pass (requires B0*B1 <= 16384).
int launch_quantize(const float* x, int64_t n, const lq_config& c, uint8_t* codes, uint8_t* sidx, float* v,
                    hipStream_t st);
// idx -> packed (unpack = false) or packed (first argument) -> idx (last pointer argument), `bits` bits per index.
int launch_pack_bits(const uint8_t* src, int64_t count, int bits, uint8_t* dst, bool unpack, hipStream_t st);
int launch_dequant(const uint8_t* codes, const uint8_t* sidx, const float* v, int64_t n, const lq_config& c,
                   float* out, hipStream_t st);

}  // namespace lq
