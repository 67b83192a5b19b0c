// Host-side NF code-book and decision thresholds (Section 2.2), plus configuration checks.
#include <cmath>
#include <cstring>
#include <mutex>

#include "lq_internal.h"

namespace lq {

static thread_local int tl_last_hip_error = 0;
void set_last_hip_error(int e) { tl_last_hip_error = e; }
int last_hip_error() { return tl_last_hip_error; }

lq_config normalized(lq_config c) {
  if (c.scale_bits == 0) c.scale_bits = 8;
  return c;
}

static bool is_pow2(int x) { return x > 0 && (x & (x - 1)) == 0; }

bool config_supported(const lq_config& c) {
  if (bits_slot(c.bits) < 0) return false;
  if (!is_pow2(c.block) || c.block < 16 || c.block > 1024) return false;
  if (!is_pow2(c.scale_block) || c.scale_block < 16 || c.scale_block > 256) return false;
  if ((int64_t)c.block * c.scale_block > 16384) return false;   // one workgroup holds a whole scale group
  if (c.scale_bits < 2 || c.scale_bits > 8) return false;
  if (c.v_dtype != LQ_V_FP32 && c.v_dtype != LQ_V_BF16 && c.v_dtype != LQ_V_FP16) return false;
  return true;
}

int bits_slot(int bits) {
  switch (bits) {
    case 2: return 0;
    case 3: return 1;
    case 4: return 2;
    case 8: return 3;
    default: return -1;
  }
}

// Standard normal CDF and its inverse.  The inverse starts from the logistic approximation of the
// probit and is polished by Newton steps on Phi(x) - p, which converge to double precision for
// the probabilities used here (all inside [0.03, 0.97]).
static double normal_cdf(double x) { return 0.5 * std::erfc(-x * 0.70710678118654752440); }

static double normal_quantile(double p) {
  double x = std::log(p / (1.0 - p)) / 1.702;
  for (int it = 0; it < 100; ++it) {
    const double pdf = 0.39894228040143267794 * std::exp(-0.5 * x * x);
    const double step = (normal_cdf(x) - p) / pdf;
    x -= step;
    if (std::fabs(step) <= 1e-17 * (1.0 + std::fabs(x))) break;
  }
  return x;
}

int host_codebook(int bits, float* out) {
  if (bits < 2 || bits > 8 || !out) return LQ_ERR_CONFIG;
  const int half = 1 << (bits - 1), ncode = 1 << bits;
  const double delta = 0.5 * (1.0 / 30.0 + 1.0 / 32.0);
  // 2^(b-1) probabilities evenly spaced on [delta, 1/2], 2^(b-1)+1 on [1/2, 1-delta]; the shared
  // 1/2 is kept once and its quantile is exactly zero.
  double q[256];
  const double span = 0.5 - delta;
  for (int i = 0; i < half - 1; ++i) q[i] = normal_quantile(delta + span * i / (half - 1));
  q[half - 1] = 0.0;
  for (int i = 1; i <= half; ++i) q[half - 1 + i] = normal_quantile(0.5 + span * i / half);
  const double top = q[ncode - 1];
  for (int i = 0; i < ncode; ++i) out[i] = (float)(q[i] / top);
  return LQ_OK;
}

static void build_tables(HostTables& t) {
  std::memset(&t, 0, sizeof(t));
  const int widths[4] = {2, 3, 4, 8};
  for (int s = 0; s < 4; ++s) {
    const int ncode = 1 << widths[s];
    host_codebook(widths[s], t.code[s]);
    for (int i = 0; i < 260; ++i) t.thr[s][i] = INFINITY;
    for (int i = 0; i + 1 < ncode; ++i) {
      const double mid = 0.5 * ((double)t.code[s][i] + (double)t.code[s][i + 1]);   // exact
      float f = (float)mid;
      if (!((double)f > mid)) f = std::nextafterf(f, INFINITY);
      t.thr[s][i] = f;
    }
    // bucket table; the margin covers the rounding of (x + 1) * 256 in fp32
    const double margin = 4e-6;
    for (int j = 0; j < 512; ++j) {
      const double lo = -1.0 + j / 256.0 - margin, hi = -1.0 + (j + 1) / 256.0 + margin;
      int below = 0, upto = 0;
      for (int i = 0; i + 1 < ncode; ++i) {
        if ((double)t.thr[s][i] <= lo) ++below;
        if ((double)t.thr[s][i] <= hi || j == 511) ++upto;
      }
      // the search compares one threshold (4 bits) or two (8 bits) after the table; more candidates per bucket
      // cannot happen for NF code-books (checked by the tests)
      const int compares = widths[s] == 4 ? 1 : 2;
      if (upto - below > compares) below = upto - compares;
      t.lut[s][j] = (uint8_t)below;
    }
  }
}

const HostTables& host_tables() {
  static HostTables tables;
  static std::once_flag once;
  std::call_once(once, [] { build_tables(tables); });
  return tables;
}

}  // namespace lq
