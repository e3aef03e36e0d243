// libhif8: HiF8 (HiFloat8, arXiv 2409.16626) conversion kernels for MI355X (gfx950).
// This file holds the C ABI declared in include/hif8.h, the per-device lookup tables and
// their initialisation, the launch-shape tuning, and a few small utility kernels; the
// conversion kernels themselves live in hif8_conv.hpp (one translation unit per tensor kind).
#include <hip/hip_runtime.h>

#include <atomic>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <mutex>

#include "hif8.h"
#include "hif8_diag.h"
#include "hif8_conv_api.hpp"
#include "hif8_device.hpp"
#include "hif8_host.hpp"
#include "hif8_stream.hpp"

using namespace hif8dev;

// ------------------------------------------------------------------------------------
// static device tables (written once per device by k_build_tables)
// ------------------------------------------------------------------------------------
static __device__ __attribute__((aligned(16))) uint8_t g_enc_lut[2][2][3][8192];  // [NaN -> 0][sat][TA, TE ties, truncating][pattern >> 19]
static __device__ __attribute__((aligned(16))) uint16_t g_val_lut[2][2][3][8192];  // layout of g_enc_lut: upper half of the binary32 pattern of the entry's value
static __device__ __attribute__((aligned(16))) uint8_t g_hr16_lut[2][2][2][8192];  // HR, 16-bit sources: [NaN -> 0][sat][source LSB][pattern >> 19]
static __device__ __attribute__((aligned(16))) uint32_t g_dec_lut[256];        // code -> binary32 bits

// Scratch of hif8_quantize_tensor_static: the per-workgroup partial maxima that hif8_quantize_tensor_* keeps in a
// caller's workspace.  One copy per GPU, held until the process ends.  In host code this name is only a handle
// for hipGetSymbolAddress: ensure_init() resolves the address of the current device's copy once and every
// launch is given that pointer.
static __device__ __align__(256) uint32_t scratch[hif8conv::kMaxParts];

__global__ void k_build_tables() {
  const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < 8192u) {
#pragma unroll
    for (uint32_t z = 0; z < 2u; ++z)
#pragma unroll
      for (uint32_t sat = 0; sat < 2u; ++sat) {
        const uint32_t flags = (z ? kFlagNan2Zero : 0u) | (sat ? kFlagSat : 0u);
        g_enc_lut[z][sat][0][i] = (uint8_t)encode_alu<false, kSrcF32>(i << 19, flags);
        g_enc_lut[z][sat][1][i] = (uint8_t)encode_any<kSrcF32>(i << 19, kRmTE | flags, 0u);
        // code of the pattern with the bits below its exponent's kept mantissa cleared: the lookup of the
        // 16-bit HR path, which adds its per-exponent addend and leaves the truncation to this table
        g_enc_lut[z][sat][2][i] = (uint8_t)encode_alu<false, kSrcF32>(trunc_table_pattern(i), flags);
        // HR of the pattern as a BF16-sourced value (source LSB = bit 16); the bits below 19 that the
        // index drops do not enter the decision
#pragma unroll
        for (uint32_t k = 0; k < 3u; ++k) g_val_lut[z][sat][k][i] = (uint16_t)(decode_bits(g_enc_lut[z][sat][k][i]) >> 16);
        g_hr16_lut[z][sat][0][i] = (uint8_t)encode_any<kSrcBF16>(i << 19, kRmHR | flags, 0u);
        g_hr16_lut[z][sat][1][i] = (uint8_t)encode_any<kSrcBF16>((i << 19) | 0x10000u, kRmHR | flags, 0u);
      }
  }
  if (i < 256u) g_dec_lut[i] = decode_bits(i);
}

__global__ void k_fill_u32(uint32_t* p, uint32_t v, uint32_t count) {
  const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < count) p[i] = v;
}

// scale = fl32(target / amax) (optionally floored to a power of two), inverse = fl32(1 / scale)
__global__ void k_scale_from_amax(const float* d_amax, float* d_scale2, uint32_t count, float target,
                                  int pow2) {
  const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= count) return;
  d_amax += i;
  d_scale2 += 2 * i;
  const float s = scale_from_amax_value(*d_amax, target, pow2);
  d_scale2[0] = s;
  d_scale2[1] = 1.0f / s;
}

// diagnostic stream kernel: read 16 B per lane, write the first OUT bytes of it (OUT = 0: read only)
template <int U, int OUT>
__global__ void __launch_bounds__(1024)
k_diag_stream(const uint4* __restrict__ src, void* __restrict__ dst, size_t nvec, Walk walk) {
  uint32_t acc = 0;
  tile_loop<U, uint4>(
      nvec, walk, [&](size_t idx) { return ld_stream(src + idx); },
      [&](size_t idx, const uint4& v) {
        if (OUT == 0) acc |= (v.x ^ v.y) & (v.z ^ v.w);
        else if (OUT == 4) st_stream(reinterpret_cast<uint32_t*>(dst) + idx, v.x);
        else if (OUT == 8) st_stream(reinterpret_cast<uint2*>(dst) + idx, make_uint2(v.x, v.y));
        else st_stream(reinterpret_cast<uint4*>(dst) + idx, v);
      },
      []() {});
  if (OUT == 0 && dst && acc == 0x9E3779B9u) *reinterpret_cast<uint32_t*>(dst) = acc;  // keeps the loads alive (dst is null in practice)
}

// ====================================================================================
// host side
// ====================================================================================
namespace hif8host {

namespace {

thread_local int t_last_hip_error = 0;

// Defaults from a sweep on MI355X under sustained load (hundreds of back-to-back launches on
// 64 Mi-element tensors; short bursts rank the shapes differently): one-shot grids of
// 256- or 512-lane workgroups with 16-32 KiB of source per staged table win for the read+write
// kernels, a persistent grid of one 1024-lane workgroup per CU wins for the read-only reduction.
// FP32 TA encode: 256 lanes x 4 loads, one tile per workgroup (16 KiB of source) -- 6.48 TB/s on 2^26
// and 6.5 TB/s on 2^30 elements against 6.39 / 6.2 TB/s for 512 lanes x 2 loads x 2 tiles.
const Shape kDefaultShape[FAM_COUNT] = {
    {256, 4, 1, 4},   // FP32 encode, TA
    {512, 4, 1, 4},   // FP32 encode, HR
    {512, 2, 2, 4},   // 16-bit encode
    {512, 2, 2, 4},   // fake-quant
    {512, 2, 1, 4},   // decode
    {1024, 2, 0, 1},  // amax
    {512, 1, 2, 4},   // diagnostic stream
    {512, 2, 2, 4},   // calibration sweeps
    {1024, 2, 0, 1},  // amax that leaves per-workgroup maxima (hif8_quantize_tensor_*)
    {512, 8, 0, 1},   // group-wise multi-tensor cast: only wg_per_cu (amax workgroups per CU of a stage) is used
};

// user overrides; -1 = use the family default
struct Tuning {
  int block = -1;
  int wg_per_cu = -1;
  int unroll = -1;
  int ta_impl = 0;
  int tiles_per_wg = -1;
  int amax_nt = -1;  // -1: by size
  int group_mib = 192;
  int family = -1;  // kernel family the shape overrides apply to; -1: all
  int stage_overlap = 1;
};
// Process-wide; written only by hif8_set_tuning (a benchmarking call, documented as not thread-safe).
Tuning g_tune;
std::atomic<uint64_t> g_sr_seed{0};

constexpr int kMaxDevices = 64;
std::mutex g_init_mutex;
bool g_inited[kMaxDevices] = {};
int g_cu_count[kMaxDevices] = {};
DevTables g_tables[kMaxDevices] = {};
uint32_t* g_scratch[kMaxDevices] = {};  // device address of `scratch` on each device

}  // namespace

Shape shape_for(Family f) {
  Shape s = kDefaultShape[f];
  if (g_tune.family >= 0 && g_tune.family != (int)f) return s;
  if (g_tune.block >= 0) s.block = g_tune.block;
  if (g_tune.unroll >= 0) s.unroll = g_tune.unroll;
  if (g_tune.tiles_per_wg >= 0) s.tiles_per_wg = g_tune.tiles_per_wg;
  if (g_tune.wg_per_cu >= 0) s.wg_per_cu = g_tune.wg_per_cu;
  return s;
}
int tune_ta_impl() { return g_tune.ta_impl; }
int tune_amax_nt() { return g_tune.amax_nt; }
uint64_t multi_group_bytes() { return (uint64_t)g_tune.group_mib << 20; }
bool multi_stage_overlap() { return g_tune.stage_overlap != 0; }
uint64_t sr_seed() { return g_sr_seed.load(std::memory_order_relaxed); }

bool hip_ok(hipError_t e) {
  if (e == hipSuccess) return true;
  t_last_hip_error = (int)e;
  return false;
}

hif8_status finish_launch() { return hip_ok(hipGetLastError()) ? HIF8_OK : HIF8_ERR_HIP; }

hif8_status ensure_init(int* cu_count_out, DevTables* tables_out) {
  int dev = 0;
  if (!hip_ok(hipGetDevice(&dev))) return HIF8_ERR_HIP;
  if (dev < 0 || dev >= kMaxDevices) return HIF8_ERR_ARG;
  std::lock_guard<std::mutex> lock(g_init_mutex);
  if (!g_inited[dev]) {
    int cus = 0;
    if (!hip_ok(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev)))
      return HIF8_ERR_HIP;
    if (cus <= 0) cus = 256;
    void* p_enc = nullptr;
    void* p_dec = nullptr;
    void* p_hr16 = nullptr;
    void* p_val = nullptr;
    if (!hip_ok(hipGetSymbolAddress(&p_enc, HIP_SYMBOL(g_enc_lut)))) return HIF8_ERR_HIP;
    if (!hip_ok(hipGetSymbolAddress(&p_dec, HIP_SYMBOL(g_dec_lut)))) return HIF8_ERR_HIP;
    if (!hip_ok(hipGetSymbolAddress(&p_hr16, HIP_SYMBOL(g_hr16_lut)))) return HIF8_ERR_HIP;
    if (!hip_ok(hipGetSymbolAddress(&p_val, HIP_SYMBOL(g_val_lut)))) return HIF8_ERR_HIP;
    void* p_scratch = nullptr;
    if (!hip_ok(hipGetSymbolAddress(&p_scratch, HIP_SYMBOL(scratch))) || !p_scratch) return HIF8_ERR_HIP;
    hipLaunchKernelGGL(k_build_tables, dim3(8192 / 256), dim3(256), 0, (hipStream_t)0);
    if (!hip_ok(hipGetLastError())) return HIF8_ERR_HIP;
    // the null stream synchronises with every blocking stream; wait on the host as well so
    // that non-blocking streams also see the tables
    if (!hip_ok(hipStreamSynchronize((hipStream_t)0))) return HIF8_ERR_HIP;
    g_cu_count[dev] = cus;
    g_tables[dev].enc_lut = reinterpret_cast<const uint8_t*>(p_enc);
    g_tables[dev].dec_lut = reinterpret_cast<const uint32_t*>(p_dec);
    g_tables[dev].hr16_lut = reinterpret_cast<const uint8_t*>(p_hr16);
    g_tables[dev].val_lut = reinterpret_cast<const uint16_t*>(p_val);
    g_scratch[dev] = reinterpret_cast<uint32_t*>(p_scratch);
    g_inited[dev] = true;
  }
  if (cu_count_out) *cu_count_out = g_cu_count[dev];
  if (tables_out) *tables_out = g_tables[dev];
  return HIF8_OK;
}

// device address of the static scratch array on the current device (after ensure_init)
static uint32_t* static_scratch() {
  int dev = 0;
  if (!hip_ok(hipGetDevice(&dev)) || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(g_init_mutex);
  return g_inited[dev] ? g_scratch[dev] : nullptr;
}

bool valid_mode(uint32_t mode) {
  if ((mode & ~(HIF8_RM_MASK | HIF8_FLAG_SAT | HIF8_FLAG_NAN2ZERO)) != 0) return false;
  return (mode & HIF8_RM_MASK) <= HIF8_RM_SR;
}

bool valid_scale(float scale, float* inv_out) {
  if (!(scale > 0.0f) || std::isinf(scale)) return false;
  volatile float inv = 1.0f / scale;
  if (!(inv > 0.0f) || std::isinf((float)inv)) return false;
  *inv_out = inv;
  return true;
}

unsigned grid_for(size_t nvec, int cus, const Shape& sh, Walk* walk, unsigned max_grid) {
  const size_t tile = (size_t)sh.block * (size_t)sh.unroll;
  size_t tiles = (nvec + tile - 1) / tile;
  if (tiles == 0) tiles = 1;  // block 0 still handles a ragged tail
  size_t grid;
  if (sh.tiles_per_wg > 0) {
    size_t tpw = (size_t)sh.tiles_per_wg;
    if (max_grid != 0 && (tiles + tpw - 1) / tpw > max_grid) tpw = (tiles + max_grid - 1) / max_grid;
    grid = (tiles + tpw - 1) / tpw;
    *walk = Walk{(uint32_t)tpw, 1u, (uint32_t)tpw};
  } else {
    size_t cap = (size_t)cus * (size_t)sh.wg_per_cu;
    if (max_grid != 0 && cap > max_grid) cap = max_grid;
    grid = tiles < cap ? tiles : cap;
    *walk = Walk{1u, (uint32_t)grid, (uint32_t)((tiles + grid - 1) / grid)};
  }
  return (unsigned)grid;
}

unsigned grid_elem(size_t n, int cus) {
  size_t blocks = (n + 255) / 256;
  const size_t cap = (size_t)cus * 16;
  if (blocks == 0) blocks = 1;
  return (unsigned)(blocks < cap ? blocks : cap);
}

hif8_status launch_fill_u32(uint32_t* p, uint32_t v, uint32_t count, hipStream_t st) {
  hipLaunchKernelGGL(k_fill_u32, dim3((count + 255) / 256), dim3(256), 0, st, p, v, count);
  return finish_launch();
}

hif8_status launch_scale_from_amax(const float* d_amax, float* d_scale2, uint32_t count, float target,
                                   int pow2, hipStream_t st) {
  hipLaunchKernelGGL(k_scale_from_amax, dim3((count + 255) / 256), dim3(256), 0, st, d_amax, d_scale2,
                     count, target, pow2);
  return finish_launch();
}

}  // namespace hif8host

using namespace hif8host;
using namespace hif8conv;

extern "C" {

int hif8_version(void) { return 400; }
int hif8_last_hip_error(void) { return t_last_hip_error; }
hif8_status hif8_init(void) { return ensure_init(nullptr, nullptr); }

hif8_status hif8_set_sr_seed(uint64_t seed) {
  g_sr_seed.store(seed, std::memory_order_relaxed);
  return HIF8_OK;
}
uint64_t hif8_get_sr_seed(void) { return sr_seed(); }
uint32_t hif8_sr_threshold(uint64_t seed, uint64_t index) { return sr_threshold(seed, index); }

hif8_status hif8_set_tuning(int key, int value) {
  switch (key) {
    case HIF8_TUNE_BLOCK:
      if (value != -1 && (value < 64 || value > 1024 || (value % 64) != 0)) return HIF8_ERR_ARG;
      g_tune.block = value;
      return HIF8_OK;
    case HIF8_TUNE_WG_PER_CU:
      if (value != -1 && (value < 1 || value > 64)) return HIF8_ERR_ARG;
      g_tune.wg_per_cu = value;
      return HIF8_OK;
    case HIF8_TUNE_UNROLL:
      if (value != -1 && value != 1 && value != 2 && value != 4 && value != 8) return HIF8_ERR_ARG;
      g_tune.unroll = value;
      return HIF8_OK;
    case HIF8_TUNE_TA_IMPL:
      if (value != 0 && value != 1) return HIF8_ERR_ARG;
      g_tune.ta_impl = value;
      return HIF8_OK;
    case HIF8_TUNE_TILES_PER_WG:
      if (value < -1 || value > 4096) return HIF8_ERR_ARG;
      g_tune.tiles_per_wg = value;
      return HIF8_OK;
    case HIF8_TUNE_AMAX_NT:
      if (value < -1 || value > 1) return HIF8_ERR_ARG;
      g_tune.amax_nt = value;
      return HIF8_OK;
    case HIF8_TUNE_GROUP_MIB:
      if (value < 1 || value > 4096) return HIF8_ERR_ARG;
      g_tune.group_mib = value;
      return HIF8_OK;
    case HIF8_TUNE_FAMILY:
      if (value < -1 || value >= (int)FAM_COUNT) return HIF8_ERR_ARG;
      g_tune.family = value;
      return HIF8_OK;
    case HIF8_TUNE_STAGE_OVERLAP:
      if (value != 0 && value != 1) return HIF8_ERR_ARG;
      g_tune.stage_overlap = value;
      return HIF8_OK;
    default:
      return HIF8_ERR_ARG;
  }
}

int hif8_get_tuning(int key) {
  switch (key) {
    case HIF8_TUNE_BLOCK: return g_tune.block;
    case HIF8_TUNE_WG_PER_CU: return g_tune.wg_per_cu;
    case HIF8_TUNE_UNROLL: return g_tune.unroll;
    case HIF8_TUNE_TA_IMPL: return g_tune.ta_impl;
    case HIF8_TUNE_TILES_PER_WG: return g_tune.tiles_per_wg;
    case HIF8_TUNE_AMAX_NT: return g_tune.amax_nt;
    case HIF8_TUNE_GROUP_MIB: return g_tune.group_mib;
    case HIF8_TUNE_FAMILY: return g_tune.family;
    case HIF8_TUNE_STAGE_OVERLAP: return g_tune.stage_overlap;
    default: return -1;
  }
}

hif8_status hif8_scale_from_amax(const float* d_amax, float* d_scale2, float target, int pow2,
                                 hif8_stream_t stream) {
  if (!d_amax || !d_scale2) return HIF8_ERR_NULL;
  if (!(target > 0.0f) || std::isinf(target)) return HIF8_ERR_ARG;
  return launch_scale_from_amax(d_amax, d_scale2, 1u, target, pow2, (hipStream_t)stream);
}

// One block of entry points per tensor kind: NAME suffix, element type, kind constant.
#define HIF8_DEFINE_KIND(SFX, T, K)                                                                      \
  hif8_status hif8_amax_##SFX(const T* src, size_t n, float* d_amax, hif8_stream_t stream) {             \
    return conv_amax<K>(src, n, d_amax, (hipStream_t)stream);                                            \
  }                                                                                                      \
  hif8_status hif8_encode_##SFX(const T* src, uint8_t* dst, size_t n, float scale, uint32_t mode,        \
                                hif8_stream_t stream) {                                                  \
    return conv_encode<K>(src, dst, n, scale, nullptr, nullptr, mode, nullptr, (hipStream_t)stream);     \
  }                                                                                                      \
  hif8_status hif8_decode_##SFX(const uint8_t* src, T* dst, size_t n, float scale,                       \
                                hif8_stream_t stream) {                                                  \
    return conv_decode<K>(src, dst, n, scale, nullptr, (hipStream_t)stream);                             \
  }                                                                                                      \
  hif8_status hif8_fake_quant_##SFX(const T* src, T* dst, uint8_t* codes, size_t n, float scale,         \
                                    uint32_t mode, hif8_stream_t stream) {                               \
    return conv_fake_quant<K>(src, dst, codes, n, scale, nullptr, nullptr, mode, nullptr,                \
                              (hipStream_t)stream);                                                      \
  }                                                                                                      \
  hif8_status hif8_encode_##SFX##_ds(const T* src, uint8_t* dst, size_t n, const float* d_scale2,        \
                                     float* d_amax_acc, uint32_t mode, hif8_stream_t stream) {           \
    if (!d_scale2) return HIF8_ERR_NULL;                                                                 \
    return conv_encode<K>(src, dst, n, 1.0f, d_scale2, d_amax_acc, mode, nullptr, (hipStream_t)stream);  \
  }                                                                                                      \
  hif8_status hif8_decode_##SFX##_ds(const uint8_t* src, T* dst, size_t n, const float* d_scale2,        \
                                     hif8_stream_t stream) {                                             \
    if (!d_scale2) return HIF8_ERR_NULL;                                                                 \
    return conv_decode<K>(src, dst, n, 1.0f, d_scale2, (hipStream_t)stream);                             \
  }                                                                                                      \
  hif8_status hif8_fake_quant_##SFX##_ds(const T* src, T* dst, uint8_t* codes, size_t n,                 \
                                         const float* d_scale2, float* d_amax_acc, uint32_t mode,        \
                                         hif8_stream_t stream) {                                         \
    if (!d_scale2) return HIF8_ERR_NULL;                                                                 \
    return conv_fake_quant<K>(src, dst, codes, n, 1.0f, d_scale2, d_amax_acc, mode, nullptr,             \
                              (hipStream_t)stream);                                                      \
  }                                                                                                      \
  hif8_status hif8_encode_##SFX##_sr(const T* src, uint8_t* dst, size_t n, float scale, uint32_t mode,   \
                                     uint64_t seed, uint64_t index_base, hif8_stream_t stream) {         \
    const SrArg sr{seed, index_base};                                                                    \
    return conv_encode<K>(src, dst, n, scale, nullptr, nullptr, mode, &sr, (hipStream_t)stream);         \
  }                                                                                                      \
  hif8_status hif8_fake_quant_##SFX##_sr(const T* src, T* dst, uint8_t* codes, size_t n, float scale,    \
                                         uint32_t mode, uint64_t seed, uint64_t index_base,              \
                                         hif8_stream_t stream) {                                         \
    const SrArg sr{seed, index_base};                                                                    \
    return conv_fake_quant<K>(src, dst, codes, n, scale, nullptr, nullptr, mode, &sr,                    \
                              (hipStream_t)stream);                                                      \
  }                                                                                                      \
  hif8_status hif8_quantize_tensor_##SFX(const T* src, T* dst, uint8_t* codes, size_t n, float target,   \
                                         int pow2, uint32_t mode, float* d_amax, float* d_scale2,        \
                                         void* workspace, size_t workspace_bytes,                        \
                                         hif8_stream_t stream) {                                         \
    if (workspace && (workspace_bytes < hif8_quantize_workspace_bytes() || !aligned_to(workspace, 4)))   \
      return HIF8_ERR_ARG;                                                                               \
    return conv_quantize_tensor<K>(src, dst, codes, n, target, pow2, mode, d_amax, d_scale2,             \
                                   reinterpret_cast<uint32_t*>(workspace), nullptr, (hipStream_t)stream);\
  }                                                                                                      \
  hif8_status hif8_multi_cast_##SFX(const hif8_cast_item* host_items, const hif8_cast_item* d_items,     \
                                    size_t count, uint64_t total_tiles, float* d_amax, float* d_scale2,  \
                                    float target, int pow2, uint32_t mode, hif8_stream_t stream) {       \
    return conv_multi_cast<K>(host_items, d_items, count, total_tiles, d_amax, d_scale2, target, pow2,   \
                              mode, (hipStream_t)stream);                                                \
  }                                                                                                      \
  hif8_status hif8_multi_encode_##SFX##_ds(const hif8_cast_item* d_items, size_t count,                  \
                                           uint64_t total_tiles, const float* d_scale2,                  \
                                           float* d_amax_acc, uint32_t mode, hif8_stream_t stream) {     \
    return conv_multi_encode_ds<K>(d_items, count, total_tiles, d_scale2, d_amax_acc, mode,              \
                                   (hipStream_t)stream);                                                 \
  }

HIF8_DEFINE_KIND(f32, float, kSrcF32)
HIF8_DEFINE_KIND(bf16, uint16_t, kSrcBF16)
HIF8_DEFINE_KIND(f16, uint16_t, kSrcF16)
#undef HIF8_DEFINE_KIND

size_t hif8_quantize_workspace_bytes(void) { return (size_t)kMaxParts * sizeof(uint32_t); }

hif8_status hif8_quantize_tensor_static(const void* src, void* dst, uint8_t* codes, size_t n, int src_kind, float target,
                                        int pow2, uint32_t mode, float* d_amax, float* d_scale2, hif8_stream_t stream) {
  if (src_kind != HIF8_KIND_F32 && src_kind != HIF8_KIND_BF16 && src_kind != HIF8_KIND_F16) return HIF8_ERR_ARG;
  if (n > HIF8_STATIC_MAX_ELEMENTS) return HIF8_ERR_ARG;
  if (!valid_mode(mode)) return HIF8_ERR_MODE;
  if (!(target > 0.0f) || std::isinf(target)) return HIF8_ERR_ARG;
  if (!d_amax || !d_scale2 || (n != 0 && (!src || (!dst && !codes)))) return HIF8_ERR_NULL;
  hif8_status s = ensure_init(nullptr, nullptr);  // resolves the scratch address of this device on first use
  if (s != HIF8_OK) return s;
  uint32_t* parts = hif8host::static_scratch();
  if (!parts) return HIF8_ERR_HIP;
  hipStream_t st = (hipStream_t)stream;
  switch (src_kind) {
    case HIF8_KIND_F32: return conv_quantize_tensor<kSrcF32>(src, dst, codes, n, target, pow2, mode, d_amax, d_scale2, parts, nullptr, st);
    case HIF8_KIND_BF16: return conv_quantize_tensor<kSrcBF16>(src, dst, codes, n, target, pow2, mode, d_amax, d_scale2, parts, nullptr, st);
    default: return conv_quantize_tensor<kSrcF16>(src, dst, codes, n, target, pow2, mode, d_amax, d_scale2, parts, nullptr, st);
  }
}

hif8_status hif8_multi_plan(hif8_cast_item* host_items, size_t count, int src_is_16bit,
                            uint64_t* total_tiles_out) {
  if (!total_tiles_out || (!host_items && count != 0)) return HIF8_ERR_NULL;
  if (count > 0xFFFFFFu) return HIF8_ERR_ARG;
  uint64_t tiles = 0;
  for (size_t i = 0; i < count; ++i) {
    hif8_cast_item& it = host_items[i];
    if (it.n != 0 && (!it.src || !it.dst)) return HIF8_ERR_NULL;
    if (!aligned_to(it.src, 16) || !aligned_to(it.dst, src_is_16bit ? 8 : 4)) return HIF8_ERR_ARG;
    it.first_tile = tiles;
    tiles += plan_item_tiles(it.n, src_is_16bit != 0);
  }
  *total_tiles_out = tiles;
  return HIF8_OK;
}

hif8_status hif8_diag_stream(const void* src, void* dst, size_t n_groups, int out_bytes,
                             hif8_stream_t stream) {
  if (!src || (!dst && out_bytes != 0)) return HIF8_ERR_NULL;
  if (out_bytes != 0 && out_bytes != 4 && out_bytes != 8 && out_bytes != 16) return HIF8_ERR_ARG;
  if (!aligned_to(src, 16) || (out_bytes != 0 && !aligned_to(dst, (size_t)out_bytes))) return HIF8_ERR_ARG;
  if (n_groups == 0) return HIF8_OK;
  int cus = 0;
  hif8_status s = ensure_init(&cus, nullptr);
  if (s != HIF8_OK) return s;
  const Shape shape = shape_for(FAM_DIAG);
  Walk walk;
  const dim3 grid(grid_for(n_groups, cus, shape, &walk)), block(shape.block);
  const uint4* s4 = reinterpret_cast<const uint4*>(src);
  hipStream_t st = (hipStream_t)stream;
  dispatch_unroll(shape.unroll, [&](auto u_c) {
    constexpr int U = decltype(u_c)::value;
    if (out_bytes == 0) hipLaunchKernelGGL((k_diag_stream<U, 0>), grid, block, 0, st, s4, dst, n_groups, walk);
    else if (out_bytes == 4) hipLaunchKernelGGL((k_diag_stream<U, 4>), grid, block, 0, st, s4, dst, n_groups, walk);
    else if (out_bytes == 8) hipLaunchKernelGGL((k_diag_stream<U, 8>), grid, block, 0, st, s4, dst, n_groups, walk);
    else hipLaunchKernelGGL((k_diag_stream<U, 16>), grid, block, 0, st, s4, dst, n_groups, walk);
  });
  return finish_launch();
}

}  // extern "C"
