// C ABI, part 1: status strings, code-book, storage cost, Quantize / Dequantize entry points.
#include <cmath>

#include "lq_internal.h"

namespace lq {
int last_hip_error();

int check_quant_args(int64_t n, lq_config& c) {
  c = normalized(c);
  if (!config_supported(c)) return LQ_ERR_CONFIG;
  if (n <= 0 || n % c.block != 0) return LQ_ERR_SHAPE;
  return LQ_OK;
}
}  // namespace lq

using namespace lq;

extern "C" {

const char* lq_status_string(int status) {
  switch (status) {
    case LQ_OK: return "ok";
    case LQ_ERR_NULL: return "a required pointer is NULL";
    case LQ_ERR_SHAPE: return "bad shape: non-positive size, or size not a multiple of the block size";
    case LQ_ERR_CONFIG: return "unsupported quantization configuration";
    case LQ_ERR_RANK: return "rank must satisfy 1 <= rank < min(d, k) and rank <= 128";
    case LQ_ERR_WEIGHT: return "row_w and col_w must both be given or both be NULL";
    case LQ_ERR_WORKSPACE: return "workspace is NULL, misaligned or too small";
    case LQ_ERR_HIP: return "a HIP runtime call failed";
    case LQ_ERR_ARG: return "bad argument";
    default: return "unknown status";
  }
}

int lq_last_hip_error(void) { return last_hip_error(); }

int lq_nf_codebook(int bits, float* host_out) {
  if (!host_out) return LQ_ERR_NULL;
  return host_codebook(bits, host_out);
}

size_t lq_codes_bytes(int64_t n, int bits) {
  if (n <= 0 || bits <= 0) return 0;
  return (size_t)((n * bits + 7) / 8);
}

double lq_storage_bits(int64_t n, lq_config c) {
  c = normalized(c);
  if (!config_supported(c) || n < 0) return -1.0;
  return (double)n * ((double)c.bits + (double)c.scale_bits / (double)c.block +
                      (double)v_bits(c) / ((double)c.block * (double)c.scale_block));
}

int lq_nf_quantize(const float* x, int64_t n, lq_config c, uint8_t* codes_packed, uint8_t* scale_idx, float* v,
                   void* stream) {
  if (!x || !codes_packed || !scale_idx || !v) return LQ_ERR_NULL;
  LQ_TRY(check_quant_args(n, c));
  return launch_quantize(x, n, c, codes_packed, scale_idx, v, (hipStream_t)stream);
}

int lq_nf_dequantize(const uint8_t* codes_packed, const uint8_t* scale_idx, const float* v, int64_t n, lq_config c,
                     float* out, void* stream) {
  if (!codes_packed || !scale_idx || !v || !out) return LQ_ERR_NULL;
  LQ_TRY(check_quant_args(n, c));
  return launch_dequant(codes_packed, scale_idx, v, n, c, out, (hipStream_t)stream);
}

int lq_pack_scale_indices(const uint8_t* scale_idx, int64_t count, int scale_bits, uint8_t* packed, void* stream) {
  if (!scale_idx || !packed) return LQ_ERR_NULL;
  if (count <= 0 || count >= ((int64_t)1 << 40)) return LQ_ERR_SHAPE;
  if (scale_bits < 2 || scale_bits > 8) return LQ_ERR_CONFIG;
  return launch_pack_bits(scale_idx, count, scale_bits, packed, false, (hipStream_t)stream);
}

int lq_unpack_scale_indices(const uint8_t* packed, int64_t count, int scale_bits, uint8_t* scale_idx, void* stream) {
  if (!scale_idx || !packed) return LQ_ERR_NULL;
  if (count <= 0 || count >= ((int64_t)1 << 40)) return LQ_ERR_SHAPE;
  if (scale_bits < 2 || scale_bits > 8) return LQ_ERR_CONFIG;
  return launch_pack_bits(packed, count, scale_bits, scale_idx, true, (hipStream_t)stream);
}

}  // extern "C"
