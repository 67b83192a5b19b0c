// NormalFloat block quantization kernels for gfx950 (Sections 2.2 and 3.2).
//
// Work unit: a "run" of 16 consecutive weights held by one lane (64 B of fp32 in, 2*bits bytes of
// packed codes out).  A block of B0 weights is B0/16 consecutive runs, i.e. consecutive lanes of one
// wavefront, so the block absmax is a few cross-lane maxima and never touches LDS.  Code-book and
// thresholds sit in LDS (8-bit) or registers (2..4-bit).
#include <hip/hip_fp16.h>

#include <mutex>

#include "nf_device.h"
#include "profiler.h"

namespace lq {

__device__ DevTables g_nf_tables;

static std::mutex g_tables_mutex;
static const DevTables* g_tables_ptr[64] = {nullptr};

int device_tables(const DevTables** out) {
  int dev = 0;
  LQ_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= 64) return LQ_ERR_HIP;
  std::lock_guard<std::mutex> lock(g_tables_mutex);
  if (!g_tables_ptr[dev]) {
        void* p = nullptr;
    LQ_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(g_nf_tables)));
    LQ_HIP_TRY(hipMemcpy(p, &host_tables(), sizeof(HostTables), hipMemcpyHostToDevice));
    g_tables_ptr[dev] = (const DevTables*)p;
  }
  *out = g_tables_ptr[dev];
  return LQ_OK;
}

int ensure_device_tables() {
  const DevTables* t;
  return device_tables(&t);
}

// ---------------------------------------------------------------------------------------------
// Quantize(x, c) in one pass.  A workgroup of 256 lanes walks chunks of 4096*U weights that hold whole
// scale groups (B0*B1 <= 4096*U); lane t owns runs t, t+256, ... of the chunk, so every load
// instruction of a wavefront covers one contiguous 4 KB stretch.  Block absmax: cross-lane maxima over
// B0/16 lanes.  Group absmax: cross-lane / LDS maxima over B0*B1/16 runs.  Nothing but the inputs and
// outputs touches memory.

template <int BITS, int U>
__global__ __launch_bounds__(256) void quantize_fused_kernel(const float* __restrict__ x, int64_t nruns,
                                                             int runs_per_block, int scale_block, int levels,
                                                             int v_dtype, const DevTables* __restrict__ tab,
                                                             uint8_t* __restrict__ codes, uint8_t* __restrict__ sidx,
                                                             float* __restrict__ v) {
  __shared__ LdsTables s_tab;
  __shared__ float s_wave[4];
  load_tables<BITS>(tab, s_tab);
  Thresholds<BITS> thr(s_tab);

  const int runs_per_group = runs_per_block * scale_block;          // 16 .. 256*U
  const int slabs_per_group = runs_per_group > 256 ? runs_per_group / 256 : 1;
  const int lane_width = runs_per_group > 256 ? 256 : runs_per_group;
  const int block_lanes = runs_per_block < 64 ? runs_per_block : 64;   // B0 <= 1024: a block never leaves a wavefront
  const int64_t chunk_runs = 256 * U;
  const int64_t nchunks = (nruns + chunk_runs - 1) / chunk_runs;

  for (int64_t chunk = blockIdx.x; chunk < nchunks; chunk += gridDim.x) {
    // Codes need the block absmax only, so each slab of 256 runs is searched and its codes stored as soon as it is
    // loaded (the next slab's loads are already in flight); what waits for the whole chunk is the group absmax.
    float amax[U];
    int64_t run[U];
    float4 nxt[4];
    auto fetch = [&](int u) {
      const int64_t r = chunk * chunk_runs + u * 256 + threadIdx.x;
      const float4* p = reinterpret_cast<const float4*>(x + (r < nruns ? r : nruns - 1) * 16);   // clamped, masked below
#pragma unroll
      for (int q = 0; q < 4; ++q) nxt[q] = p[q];
    };
    fetch(0);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      run[u] = chunk * chunk_runs + u * 256 + threadIdx.x;
      const bool live = run[u] < nruns;
      float t[16];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        t[4 * q] = live ? nxt[q].x : 0.0f; t[4 * q + 1] = live ? nxt[q].y : 0.0f;
        t[4 * q + 2] = live ? nxt[q].z : 0.0f; t[4 * q + 3] = live ? nxt[q].w : 0.0f;
      }
      if (u + 1 < U) fetch(u + 1);
      amax[u] = lanes_max(run_absmax(t), block_lanes);
      const float rcp = safe_reciprocal(amax[u]);
      uint32_t c[16];
#pragma unroll
      for (int j = 0; j < 16; ++j) c[j] = thr.nearest(t[j] * rcp);
      if (live) store_codes<BITS>(codes, run[u], c);
    }
    // group maxima: first across the slabs that belong to one group, then across lanes
    float gmax[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float m = amax[u];
      const int g0 = u - (u % slabs_per_group);
#pragma unroll
      for (int w = 0; w < U; ++w)
        if (w >= g0 && w < g0 + slabs_per_group) m = fmaxf(m, amax[w]);
      gmax[u] = m;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) gmax[u] = group_max(gmax[u], lane_width, s_wave);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (run[u] < nruns) {
        if ((run[u] & (runs_per_block - 1)) == 0) {
          const float sigma = gmax[u] / (float)levels;
          sidx[run[u] / runs_per_block] = (uint8_t)scale_index(amax[u], sigma, levels);
        }
        if (run[u] % runs_per_group == 0) v[run[u] / runs_per_group] = cast_group_scale(gmax[u], v_dtype);
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Dequantize: one quad (4 consecutive weights) per lane and step, DQ_U steps per lane, so every wavefront store is
// 1 KB contiguous.  A workgroup owns one stretch of 256 * DQ_U quads: every load is issued first, then everything is
// computed and stored, and the wavefront ends without waiting for a store (loads and stores retire through one in-order
// counter, so a loop that alternates them runs at the pace of the store latency).
constexpr int DQ_U = 4;
typedef float floatx4n __attribute__((ext_vector_type(4)));

template <int BITS>
__global__ __launch_bounds__(256) void dequant_kernel(const uint8_t* __restrict__ codes,
                                                      const uint8_t* __restrict__ sidx, const float* __restrict__ v,
                                                      int64_t nquads, int qpb_shift, int sb_shift, int levels,
                                                      const DevTables* __restrict__ tab, float* __restrict__ out) {
  __shared__ float s_code[1 << BITS];
  for (int i = threadIdx.x; i < (1 << BITS); i += 256) s_code[i] = tab->code[Slot<BITS>::value][i];
  const int64_t q0 = (int64_t)blockIdx.x * (256 * DQ_U) + threadIdx.x;
  uint32_t cw[DQ_U], si[DQ_U];
  float vv[DQ_U];
#pragma unroll
  for (int u = 0; u < DQ_U; ++u) {
    const int64_t quad = q0 + 256 * u < nquads ? q0 + 256 * u : nquads - 1;      // clamped: loaded, never stored
    const int64_t blk = quad >> qpb_shift;
    if constexpr (BITS == 8) cw[u] = *reinterpret_cast<const uint32_t*>(codes + quad * 4);
    else if constexpr (BITS == 4) cw[u] = *reinterpret_cast<const uint16_t*>(codes + quad * 2);
    else if constexpr (BITS == 2) cw[u] = codes[quad];
    else {   // 3 bits: 12 bits starting at bit 12*quad = byte floor(1.5*quad), nibble-aligned
      const int64_t byte = (quad * 3) >> 1;
      cw[u] = (((uint32_t)codes[byte] | ((uint32_t)codes[byte + 1] << 8)) >> ((quad & 1) * 4)) & 0xfffu;
    }
    si[u] = sidx[blk];
    vv[u] = v[blk >> sb_shift];
  }
  __syncthreads();                     // code book in LDS
  constexpr uint32_t mask = (1u << BITS) - 1u;
#pragma unroll
  for (int u = 0; u < DQ_U; ++u) {
    const int64_t quad = q0 + 256 * u;
    if (quad >= nquads) break;
    const float sh = block_scale(si[u], vv[u], levels);
    floatx4n f;
    f[0] = s_code[cw[u] & mask] * sh; f[1] = s_code[(cw[u] >> BITS) & mask] * sh;
    f[2] = s_code[(cw[u] >> (2 * BITS)) & mask] * sh; f[3] = s_code[(cw[u] >> (3 * BITS)) & mask] * sh;
    __builtin_nontemporal_store(f, reinterpret_cast<floatx4n*>(out + (quad << 2)));
  }
}

// ---------------------------------------------------------------------------------------------
// Scale indices as a little-endian bit stream of `bits` bits each (the b1 bits per block that the storage formula
// of Eq. 3 counts): one lane packs / unpacks 8 indices = `bits` bytes.
__global__ __launch_bounds__(256) void pack_bits_kernel(const uint8_t* __restrict__ idx, int64_t count, int bits,
                                                        uint8_t* __restrict__ packed) {
  const int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;       // group of 8 indices
  if (g * 8 >= count) return;
  uint64_t w = 0;
  for (int j = 0; j < 8; ++j) {
    const int64_t i = g * 8 + j;
    const uint64_t c = i < count ? (uint64_t)(idx[i] & ((1u << bits) - 1u)) : 0u;
    w |= c << (j * bits);
  }
  const int64_t total = (count * bits + 7) / 8;
  for (int b = 0; b < bits; ++b)
    if (g * bits + b < total) packed[g * bits + b] = (uint8_t)(w >> (8 * b));
}

__global__ __launch_bounds__(256) void unpack_bits_kernel(const uint8_t* __restrict__ packed, int64_t count, int bits,
                                                          uint8_t* __restrict__ idx) {
  const int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (g * 8 >= count) return;
  const int64_t total = (count * bits + 7) / 8;
  uint64_t w = 0;
  for (int b = 0; b < bits; ++b)
    if (g * bits + b < total) w |= (uint64_t)packed[g * bits + b] << (8 * b);
  for (int j = 0; j < 8; ++j) {
    const int64_t i = g * 8 + j;
    if (i < count) idx[i] = (uint8_t)((w >> (j * bits)) & ((1u << bits) - 1u));
  }
}

int launch_pack_bits(const uint8_t* idx, int64_t count, int bits, uint8_t* packed, bool unpack, hipStream_t st) {
  const int64_t groups = (count + 7) / 8;
  const dim3 grid((unsigned)((groups + 255) / 256)), block(256);
  prof::Scope ps(prof::MISC, st, (double)count * (1.0 + bits / 8.0));
  if (unpack) hipLaunchKernelGGL(unpack_bits_kernel, grid, block, 0, st, idx, count, bits, packed);
  else hipLaunchKernelGGL(pack_bits_kernel, grid, block, 0, st, idx, count, bits, packed);
  LQ_HIP_TRY(hipGetLastError());
  return LQ_OK;
}

// ---------------------------------------------------------------------------------------------
template <int BITS>
static void launch_quantize_bits(const float* x, int64_t nruns, const lq_config& c, const DevTables* tab,
                                 uint8_t* codes, uint8_t* sidx, float* v, hipStream_t st) {
  const int rpb = c.block / 16;
  const int lv = scale_levels(c);
  const bool big = (int64_t)c.block * c.scale_block > 8192;
  const int64_t chunk_runs = big ? 1024 : 512;
  const int64_t nchunks = (nruns + chunk_runs - 1) / chunk_runs;
  const int64_t cap = (int64_t)1 << 22;       // one chunk per workgroup: the loads of the many resident workgroups overlap
  const dim3 grid((unsigned)(nchunks < cap ? nchunks : cap)), block(256);
  if (big)
    hipLaunchKernelGGL((quantize_fused_kernel<BITS, 4>), grid, block, 0, st, x, nruns, rpb, c.scale_block, lv,
                       c.v_dtype, tab, codes, sidx, v);
  else
    hipLaunchKernelGGL((quantize_fused_kernel<BITS, 2>), grid, block, 0, st, x, nruns, rpb, c.scale_block, lv,
                       c.v_dtype, tab, codes, sidx, v);
}

int launch_quantize(const float* x, int64_t n, const lq_config& c, uint8_t* codes, uint8_t* sidx, float* v,
                    hipStream_t st) {
  const DevTables* tab;
  LQ_TRY(device_tables(&tab));
  const int64_t nruns = n / 16;
  prof::Scope ps(prof::QUANTIZE, st,
                 (double)n * (4.0 + c.bits / 8.0 + 1.0 / c.block + 4.0 / ((double)c.block * c.scale_block)));
  switch (c.bits) {
    case 2: launch_quantize_bits<2>(x, nruns, c, tab, codes, sidx, v, st); break;
    case 3: launch_quantize_bits<3>(x, nruns, c, tab, codes, sidx, v, st); break;
    case 4: launch_quantize_bits<4>(x, nruns, c, tab, codes, sidx, v, st); break;
    case 8: launch_quantize_bits<8>(x, nruns, c, tab, codes, sidx, v, st); break;
    default: return LQ_ERR_CONFIG;
  }
  LQ_HIP_TRY(hipGetLastError());
  return LQ_OK;
}

int launch_dequant(const uint8_t* codes, const uint8_t* sidx, const float* v, int64_t n, const lq_config& c,
                   float* out, hipStream_t st) {
  const DevTables* tab;
  LQ_TRY(device_tables(&tab));
  const int64_t nruns = n / 4;            // quads
  const int rpb = __builtin_ctz(c.block / 4);            // log2(quads per block)
  const int64_t want = (nruns + 256 * DQ_U - 1) / (256 * DQ_U);
  if (want >= (1ll << 31)) return LQ_ERR_SHAPE;
  const dim3 grid((unsigned)want), block(256);
  const int lv = scale_levels(c);
  prof::Scope ps(prof::DEQUANTIZE, st,
                 (double)n * (4.0 + c.bits / 8.0 + 1.0 / c.block + 4.0 / ((double)c.block * c.scale_block)));
  switch (c.bits) {
    case 2: hipLaunchKernelGGL(dequant_kernel<2>, grid, block, 0, st, codes, sidx, v, nruns, rpb, __builtin_ctz(c.scale_block), lv, tab, out); break;
    case 3: hipLaunchKernelGGL(dequant_kernel<3>, grid, block, 0, st, codes, sidx, v, nruns, rpb, __builtin_ctz(c.scale_block), lv, tab, out); break;
    case 4: hipLaunchKernelGGL(dequant_kernel<4>, grid, block, 0, st, codes, sidx, v, nruns, rpb, __builtin_ctz(c.scale_block), lv, tab, out); break;
    case 8: hipLaunchKernelGGL(dequant_kernel<8>, grid, block, 0, st, codes, sidx, v, nruns, rpb, __builtin_ctz(c.scale_block), lv, tab, out); break;
    default: return LQ_ERR_CONFIG;
  }
  LQ_HIP_TRY(hipGetLastError());
  return LQ_OK;
}

}  // namespace lq
