// libhif8: HiF8 (HiFloat8, arXiv 2409.16626) conversion kernels for MI355X (gfx950) and the
// C ABI declared in include/hif8.h.
//
// All kernels are HBM-streaming scans: every lane moves 16 bytes per load, a persistent
// grid (a few workgroups per compute unit) strides over the tensor, U independent loads
// are in flight per lane.  There is no contraction anywhere, hence no MFMA.
//
//   encode, TA   : the TA code of a non-NaN binary32 value depends only on its top 13 bits
//                  (sign, exponent, 3 kept + 1 rounding mantissa bit), so the hot loop is one
//                  shift and one byte lookup in an 8 KiB table staged in LDS.  The table
//                  itself is produced on the device, once, by the integer encoder below.
//   encode, HR   : integer rounding in registers (round_mag), then the same byte lookup.
//   decode       : 256-entry binary32 table staged in LDS, one multiply by 1/scale.
//   fake-quant   : encode and decode fused; the value never leaves registers.
//   amax         : unsigned max of magnitude patterns; DPP reduction inside a wavefront,
//                  LDS across wavefronts, one atomic max per workgroup.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstring>
#include <mutex>

#include "hif8.h"
#include "hif8_device.hpp"

using namespace hif8dev;

// ------------------------------------------------------------------------------------
// static device tables (written once per device by k_build_tables)
// ------------------------------------------------------------------------------------
static __device__ __attribute__((aligned(16))) uint8_t g_enc_lut[2][8192];  // [sat][pattern >> 19]
static __device__ __attribute__((aligned(16))) uint32_t g_dec_lut[256];     // code -> binary32 bits

__global__ void k_build_tables() {
  const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < 8192u) {
    g_enc_lut[0][i] = (uint8_t)encode_alu<false, false>(i << 19, 0u);
    g_enc_lut[1][i] = (uint8_t)encode_alu<false, false>(i << 19, kFlagSat);
  }
  if (i < 256u) g_dec_lut[i] = decode_bits(i);
}

// ------------------------------------------------------------------------------------
// small device helpers
// ------------------------------------------------------------------------------------
enum : int { IMPL_TA_LUT = 0, IMPL_TA_ALU = 1, IMPL_HR = 2 };

__device__ __forceinline__ void stage_enc_lut(uint8_t* lut, uint32_t mode) {
  const uint4* g = reinterpret_cast<const uint4*>(g_enc_lut[(mode & kFlagSat) ? 1 : 0]);
  uint4* l = reinterpret_cast<uint4*>(lut);
  for (uint32_t i = threadIdx.x; i < 8192u / 16u; i += blockDim.x) l[i] = g[i];
}
__device__ __forceinline__ void stage_hr_table(HrExp* hrt) {
  for (uint32_t i = threadIdx.x; i < 256u; i += blockDim.x) hrt[i] = hr_exp_entry(i);
}
__device__ __forceinline__ void stage_dec_lut(uint32_t* lut) {
  for (uint32_t i = threadIdx.x; i < 256u; i += blockDim.x) lut[i] = g_dec_lut[i];
}

// One element: scaled pattern -> code.  `lut` is the staged TA table (unused for IMPL_TA_ALU).
template <int IMPL, bool SRC16>
__device__ __forceinline__ uint32_t encode_one(uint32_t ybits, const uint8_t* lut, const HrExp* hrt,
                                              uint32_t mode) {
  if (IMPL == IMPL_TA_LUT) {
    uint32_t c = lut[ybits >> 19];
    // NaNs whose payload sits only in the low 19 bits index the Inf entry; fix them here.
    if ((ybits & 0x7FFFFFFFu) > 0x7F800000u) c = nan_code(mode);
    return c;
  } else if (IMPL == IMPL_TA_ALU) {
    return encode_alu<false, SRC16>(ybits, mode);
  } else {
    // HR: table-driven rounding to the grid, then the byte of the (now representable)
    // pattern from the TA table
    const uint32_t r = hr_round_bits<SRC16>(ybits, hrt[(ybits >> 23) & 0xFFu]);
    uint32_t c = lut[r >> 19];
    if ((ybits & 0x7FFFFFFFu) > 0x7F800000u) c = nan_code(mode);
    return c;
  }
}

__device__ __forceinline__ uint32_t scaled_bits(uint32_t xbits, float scale) {
  return __float_as_uint(__fmul_rn(__uint_as_float(xbits), scale));
}

template <int IMPL>
__device__ __forceinline__ uint32_t encode4_f32(const uint4& v, float scale, const uint8_t* lut,
                                               const HrExp* hrt, uint32_t mode) {
  const uint32_t c0 = encode_one<IMPL, false>(scaled_bits(v.x, scale), lut, hrt, mode);
  const uint32_t c1 = encode_one<IMPL, false>(scaled_bits(v.y, scale), lut, hrt, mode);
  const uint32_t c2 = encode_one<IMPL, false>(scaled_bits(v.z, scale), lut, hrt, mode);
  const uint32_t c3 = encode_one<IMPL, false>(scaled_bits(v.w, scale), lut, hrt, mode);
  return c0 | (c1 << 8) | (c2 << 16) | (c3 << 24);
}

// two bfloat16 in one dword -> two codes in the low 16 bits
template <int IMPL>
__device__ __forceinline__ uint32_t encode2_bf16(uint32_t w, float scale, const uint8_t* lut,
                                                const HrExp* hrt, uint32_t mode) {
  const uint32_t c0 = encode_one<IMPL, true>(scaled_bits(w << 16, scale), lut, hrt, mode);
  const uint32_t c1 = encode_one<IMPL, true>(scaled_bits(w & 0xFFFF0000u, scale), lut, hrt, mode);
  return c0 | (c1 << 8);
}

template <int IMPL>
__device__ __forceinline__ uint2 encode8_bf16(const uint4& v, float scale, const uint8_t* lut,
                                              const HrExp* hrt, uint32_t mode) {
  uint2 o;
  o.x = encode2_bf16<IMPL>(v.x, scale, lut, hrt, mode) | (encode2_bf16<IMPL>(v.y, scale, lut, hrt, mode) << 16);
  o.y = encode2_bf16<IMPL>(v.z, scale, lut, hrt, mode) | (encode2_bf16<IMPL>(v.w, scale, lut, hrt, mode) << 16);
  return o;
}

__device__ __forceinline__ uint32_t descale_bits(uint32_t code, const uint32_t* dec, float inv) {
  return __float_as_uint(__fmul_rn(__uint_as_float(dec[code & 0xFFu]), inv));
}

// two codes -> two descaled bfloat16 in one dword; the narrowing is the hardware's packed
// round-to-nearest-even conversion (v_cvt_pk_bf16_f32)
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t descale2_bf16(uint32_t c0, uint32_t c1, const uint32_t* dec,
                                                  float inv) {
  const f32x2_t f = {__uint_as_float(descale_bits(c0, dec, inv)),
                     __uint_as_float(descale_bits(c1, dec, inv))};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2_t));
}

// ------------------------------------------------------------------------------------
// streaming kernels.  Vector unit = one 16-byte source load per lane (decode: one lane's
// worth of codes).  A tile is blockDim.x * U vector units; blocks stride over tiles.
// The ragged tail (n modulo the vector width) is done element-wise by block 0.
// ------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t umax(uint32_t a, uint32_t b) { return a > b ? a : b; }

// Maximum over the 64 lanes of a wavefront with DPP row shifts and row broadcasts; the
// result is valid in lane 63 and returned to every lane through a scalar read of that lane.
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
  v = umax(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x111, 0xF, 0xF, false));  // row_shr:1
  v = umax(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x112, 0xF, 0xF, false));  // row_shr:2
  v = umax(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x114, 0xF, 0xF, false));  // row_shr:4
  v = umax(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x118, 0xF, 0xF, false));  // row_shr:8
  v = umax(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x142, 0xF, 0xF, false));  // row_bcast:15
  v = umax(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x143, 0xF, 0xF, false));  // row_bcast:31
  return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}

__device__ __forceinline__ void block_max_to_global(uint32_t m, uint32_t* out) {
  __shared__ uint32_t wave_m[16];
  m = wave_max_u32(m);
  const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
  if (lane == 0) wave_m[wave] = m;
  __syncthreads();
  if (threadIdx.x == 0) {
    const uint32_t nw = (blockDim.x + 63u) >> 6;
    uint32_t r = wave_m[0];
    for (uint32_t w = 1; w < nw; ++w) r = umax(r, wave_m[w]);
    if (r) atomicMax(out, r);
  }
}

// running magnitude maximum of one 16-byte vector: FP32 -> binary32 magnitude pattern;
// BF16 -> two 15-bit magnitudes, one per 16-bit half (folded by fold_amax_bf16 at the end)
typedef uint16_t u16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t vec_amax_f32(uint32_t m, const uint4& v) {
  return umax(m, umax(umax(v.x & 0x7FFFFFFFu, v.y & 0x7FFFFFFFu),
                      umax(v.z & 0x7FFFFFFFu, v.w & 0x7FFFFFFFu)));
}
__device__ __forceinline__ uint32_t vec_amax_bf16(uint32_t m, const uint4& v) {
  u16x2_t mm = __builtin_bit_cast(u16x2_t, m);
  mm = __builtin_elementwise_max(mm, __builtin_bit_cast(u16x2_t, v.x & 0x7FFF7FFFu));
  mm = __builtin_elementwise_max(mm, __builtin_bit_cast(u16x2_t, v.y & 0x7FFF7FFFu));
  mm = __builtin_elementwise_max(mm, __builtin_bit_cast(u16x2_t, v.z & 0x7FFF7FFFu));
  mm = __builtin_elementwise_max(mm, __builtin_bit_cast(u16x2_t, v.w & 0x7FFF7FFFu));
  return __builtin_bit_cast(uint32_t, mm);
}
__device__ __forceinline__ uint32_t fold_amax_bf16(uint32_t m) { return umax(m & 0xFFFFu, m >> 16) << 16; }

// How a workgroup walks the tiles of a tensor (tile t = vector units [t*tile, (t+1)*tile)):
// workgroup b visits tiles b*first_mul + i*stride for i in [0, count).
//   persistent grid : first_mul = 1, stride = gridDim.x, count = ceil(tiles / gridDim.x)
//   one-shot chunks : first_mul = count = tiles per workgroup, stride = 1; the hardware
//                     dispatcher hands out chunks in address order as workgroups retire, which
//                     keeps the set of DRAM pages being streamed compact.
struct Walk {
  uint32_t first_mul;
  uint32_t stride;
  uint32_t count;
};

// Streaming (non-temporal) 16 / 8 / 4-byte accesses: the data is touched once.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint4 ld_stream(const uint4* p) {
  const u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
  return make_uint4(t.x, t.y, t.z, t.w);
}
__device__ __forceinline__ uint2 ld_stream(const uint2* p) {
  const u32x2 t = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(p));
  return make_uint2(t.x, t.y);
}
__device__ __forceinline__ uint32_t ld_stream(const uint32_t* p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ void st_stream(uint4* p, const uint4& v) {
  const u32x4 t = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(t, reinterpret_cast<u32x4*>(p));
}
__device__ __forceinline__ void st_stream(uint2* p, const uint2& v) {
  const u32x2 t = {v.x, v.y};
  __builtin_nontemporal_store(t, reinterpret_cast<u32x2*>(p));
}
__device__ __forceinline__ void st_stream(uint32_t* p, uint32_t v) { __builtin_nontemporal_store(v, p); }

// The first tile's loads are issued before `prologue` (table staging + barrier) runs, so the
// staging latency overlaps with the first HBM round trip.
template <int U, typename V, typename LoadF, typename StoreF, typename PrologueF>
__device__ __forceinline__ void tile_loop(size_t nvec, const Walk w, LoadF load, StoreF store,
                                          PrologueF prologue) {
  const size_t tile = (size_t)blockDim.x * U;
  size_t base = (size_t)blockIdx.x * w.first_mul * tile;
  V v[U];
  auto load_tile = [&](size_t b) {
    const size_t first = b + threadIdx.x;
    if (b + tile <= nvec) {
#pragma unroll
      for (int j = 0; j < U; ++j) v[j] = load(first + (size_t)j * blockDim.x);
    } else {
#pragma unroll
      for (int j = 0; j < U; ++j) {
        const size_t idx = first + (size_t)j * blockDim.x;
        if (idx < nvec) v[j] = load(idx);
      }
    }
  };
  auto store_tile = [&](size_t b) {
    const size_t first = b + threadIdx.x;
    if (b + tile <= nvec) {
#pragma unroll
      for (int j = 0; j < U; ++j) store(first + (size_t)j * blockDim.x, v[j]);
    } else {
#pragma unroll
      for (int j = 0; j < U; ++j) {
        const size_t idx = first + (size_t)j * blockDim.x;
        if (idx < nvec) store(idx, v[j]);
      }
    }
  };
  if (w.count > 0 && base < nvec) load_tile(base);
  prologue();
  for (uint32_t i = 0; i < w.count && base < nvec; ++i) {
    store_tile(base);
    base += (size_t)w.stride * tile;
    if (i + 1 < w.count && base < nvec) load_tile(base);
  }
}

template <int U, int IMPL>
__global__ void __launch_bounds__(1024)
k_encode_f32(const float* __restrict__ src, uint8_t* __restrict__ dst, size_t n, float scale_arg,
             const float* __restrict__ d_scale2, uint32_t* __restrict__ amax_acc, uint32_t mode,
             Walk walk) {
  __shared__ __attribute__((aligned(16))) uint8_t lut[IMPL == IMPL_TA_ALU ? 16 : 8192];
  __shared__ __attribute__((aligned(8))) HrExp hrt[IMPL == IMPL_HR ? 256 : 1];
  const float scale = d_scale2 ? d_scale2[0] : scale_arg;
  const uint4* __restrict__ src4 = reinterpret_cast<const uint4*>(src);
  uint32_t* __restrict__ dst4 = reinterpret_cast<uint32_t*>(dst);
  const size_t nvec = n >> 2;
  uint32_t m = 0;  // amax of the unscaled input, only tracked when amax_acc != nullptr
  tile_loop<U, uint4>(
      nvec, walk, [&](size_t idx) { return ld_stream(src4 + idx); },
      [&](size_t idx, const uint4& v) {
        if (amax_acc) m = vec_amax_f32(m, v);
        st_stream(dst4 + idx, encode4_f32<IMPL>(v, scale, lut, hrt, mode));
      },
      [&]() {
        if (IMPL != IMPL_TA_ALU) {
          stage_enc_lut(lut, mode);
          if (IMPL == IMPL_HR) stage_hr_table(hrt);
          __syncthreads();
        }
      });
  const size_t t = (nvec << 2) + threadIdx.x;
  if (blockIdx.x == 0 && t < n) {
    const uint32_t xb = __float_as_uint(src[t]);
    m = umax(m, xb & 0x7FFFFFFFu);
    dst[t] = (uint8_t)encode_one<IMPL, false>(scaled_bits(xb, scale), lut, hrt, mode);
  }
  if (amax_acc) block_max_to_global(m, amax_acc);
}

template <int U, int IMPL>
__global__ void __launch_bounds__(1024)
k_encode_bf16(const uint16_t* __restrict__ src, uint8_t* __restrict__ dst, size_t n,
              float scale_arg, const float* __restrict__ d_scale2,
              uint32_t* __restrict__ amax_acc, uint32_t mode, Walk walk) {
  __shared__ __attribute__((aligned(16))) uint8_t lut[IMPL == IMPL_TA_ALU ? 16 : 8192];
  __shared__ __attribute__((aligned(8))) HrExp hrt[IMPL == IMPL_HR ? 256 : 1];
  const float scale = d_scale2 ? d_scale2[0] : scale_arg;
  const uint4* __restrict__ src4 = reinterpret_cast<const uint4*>(src);
  uint2* __restrict__ dst8 = reinterpret_cast<uint2*>(dst);
  const size_t nvec = n >> 3;
  uint32_t m = 0;
  tile_loop<U, uint4>(
      nvec, walk, [&](size_t idx) { return ld_stream(src4 + idx); },
      [&](size_t idx, const uint4& v) {
        if (amax_acc) m = vec_amax_bf16(m, v);
        st_stream(dst8 + idx, encode8_bf16<IMPL>(v, scale, lut, hrt, mode));
      },
      [&]() {
        if (IMPL != IMPL_TA_ALU) {
          stage_enc_lut(lut, mode);
          if (IMPL == IMPL_HR) stage_hr_table(hrt);
          __syncthreads();
        }
      });
  const size_t t = (nvec << 3) + threadIdx.x;
  m = fold_amax_bf16(m);
  if (blockIdx.x == 0 && t < n) {
    const uint32_t xb = (uint32_t)src[t] << 16;
    m = umax(m, xb & 0x7FFFFFFFu);
    dst[t] = (uint8_t)encode_one<IMPL, true>(scaled_bits(xb, scale), lut, hrt, mode);
  }
  if (amax_acc) block_max_to_global(m, amax_acc);
}

template <int U>
__global__ void __launch_bounds__(1024)
k_decode_f32(const uint8_t* __restrict__ src, float* __restrict__ dst, size_t n, float inv_arg,
             const float* __restrict__ d_scale2, Walk walk) {
  __shared__ uint32_t dec[256];
  const float inv = d_scale2 ? d_scale2[1] : inv_arg;  // fl32(1/scale), computed by the host
  const uint32_t* __restrict__ src4 = reinterpret_cast<const uint32_t*>(src);
  uint4* __restrict__ dst4 = reinterpret_cast<uint4*>(dst);
  const size_t nvec = n >> 2;
  tile_loop<U, uint32_t>(
      nvec, walk, [&](size_t idx) { return ld_stream(src4 + idx); },
      [&](size_t idx, uint32_t w) {
        uint4 o;
        o.x = descale_bits(w, dec, inv);
        o.y = descale_bits(w >> 8, dec, inv);
        o.z = descale_bits(w >> 16, dec, inv);
        o.w = descale_bits(w >> 24, dec, inv);
        st_stream(dst4 + idx, o);
      },
      [&]() {
        stage_dec_lut(dec);
        __syncthreads();
      });
  const size_t t = (nvec << 2) + threadIdx.x;
  if (blockIdx.x == 0 && t < n) dst[t] = __uint_as_float(descale_bits(src[t], dec, inv));
}

template <int U>
__global__ void __launch_bounds__(1024)
k_decode_bf16(const uint8_t* __restrict__ src, uint16_t* __restrict__ dst, size_t n,
              float inv_arg, const float* __restrict__ d_scale2, Walk walk) {
  __shared__ uint32_t dec[256];
  const float inv = d_scale2 ? d_scale2[1] : inv_arg;
  const uint2* __restrict__ src8 = reinterpret_cast<const uint2*>(src);
  uint4* __restrict__ dst16 = reinterpret_cast<uint4*>(dst);
  const size_t nvec = n >> 3;
  tile_loop<U, uint2>(
      nvec, walk, [&](size_t idx) { return ld_stream(src8 + idx); },
      [&](size_t idx, const uint2& w) {
        uint4 o;
        o.x = descale2_bf16(w.x, w.x >> 8, dec, inv);
        o.y = descale2_bf16(w.x >> 16, w.x >> 24, dec, inv);
        o.z = descale2_bf16(w.y, w.y >> 8, dec, inv);
        o.w = descale2_bf16(w.y >> 16, w.y >> 24, dec, inv);
        st_stream(dst16 + idx, o);
      },
      [&]() {
        stage_dec_lut(dec);
        __syncthreads();
      });
  const size_t t = (nvec << 3) + threadIdx.x;
  if (blockIdx.x == 0 && t < n) dst[t] = (uint16_t)narrow_bf16(descale_bits(src[t], dec, inv));
}

// fake-quant: src and dst may alias (each lane reads its own vectors before it writes them)
template <int U, int IMPL, bool CODES>
__global__ void __launch_bounds__(1024)
k_fake_quant_f32(const float* src, float* dst, uint8_t* codes, size_t n, float scale_arg,
                 float inv_arg, const float* __restrict__ d_scale2, uint32_t* amax_acc,
                  uint32_t mode, Walk walk) {
  __shared__ __attribute__((aligned(16))) uint8_t lut[IMPL == IMPL_TA_ALU ? 16 : 8192];
  __shared__ __attribute__((aligned(8))) HrExp hrt[IMPL == IMPL_HR ? 256 : 1];
  __shared__ uint32_t dec[256];
  const float scale = d_scale2 ? d_scale2[0] : scale_arg;
  const float inv = d_scale2 ? d_scale2[1] : inv_arg;
  auto prologue = [&]() {
    if (IMPL != IMPL_TA_ALU) stage_enc_lut(lut, mode);
    if (IMPL == IMPL_HR) stage_hr_table(hrt);
    stage_dec_lut(dec);
    __syncthreads();
  };
  const uint4* src4 = reinterpret_cast<const uint4*>(src);
  uint4* dst4 = reinterpret_cast<uint4*>(dst);
  uint32_t* codes4 = reinterpret_cast<uint32_t*>(codes);
  const size_t nvec = n >> 2;
  uint32_t m = 0;
  tile_loop<U, uint4>(
      nvec, walk, [&](size_t idx) { return ld_stream(src4 + idx); },
      [&](size_t idx, const uint4& v) {
        if (amax_acc) m = vec_amax_f32(m, v);
        const uint32_t w = encode4_f32<IMPL>(v, scale, lut, hrt, mode);
        uint4 o;
        o.x = descale_bits(w, dec, inv);
        o.y = descale_bits(w >> 8, dec, inv);
        o.z = descale_bits(w >> 16, dec, inv);
        o.w = descale_bits(w >> 24, dec, inv);
        st_stream(dst4 + idx, o);
        if (CODES) st_stream(codes4 + idx, w);
      },
      prologue);
  const size_t t = (nvec << 2) + threadIdx.x;
  if (blockIdx.x == 0 && t < n) {
    const uint32_t xb = __float_as_uint(src[t]);
    m = umax(m, xb & 0x7FFFFFFFu);
    const uint32_t c = encode_one<IMPL, false>(scaled_bits(xb, scale), lut, hrt, mode);
    dst[t] = __uint_as_float(descale_bits(c, dec, inv));
    if (CODES) codes[t] = (uint8_t)c;
  }
  if (amax_acc) block_max_to_global(m, amax_acc);
}

template <int U, int IMPL, bool CODES>
__global__ void __launch_bounds__(1024)
k_fake_quant_bf16(const uint16_t* src, uint16_t* dst, uint8_t* codes, size_t n, float scale_arg,
                  float inv_arg, const float* __restrict__ d_scale2, uint32_t* amax_acc,
                  uint32_t mode, Walk walk) {
  __shared__ __attribute__((aligned(16))) uint8_t lut[IMPL == IMPL_TA_ALU ? 16 : 8192];
  __shared__ __attribute__((aligned(8))) HrExp hrt[IMPL == IMPL_HR ? 256 : 1];
  __shared__ uint32_t dec[256];
  const float scale = d_scale2 ? d_scale2[0] : scale_arg;
  const float inv = d_scale2 ? d_scale2[1] : inv_arg;
  auto prologue = [&]() {
    if (IMPL != IMPL_TA_ALU) stage_enc_lut(lut, mode);
    if (IMPL == IMPL_HR) stage_hr_table(hrt);
    stage_dec_lut(dec);
    __syncthreads();
  };
  const uint4* src4 = reinterpret_cast<const uint4*>(src);
  uint4* dst4 = reinterpret_cast<uint4*>(dst);
  uint2* codes8 = reinterpret_cast<uint2*>(codes);
  const size_t nvec = n >> 3;
  uint32_t m = 0;
  tile_loop<U, uint4>(
      nvec, walk, [&](size_t idx) { return ld_stream(src4 + idx); },
      [&](size_t idx, const uint4& v) {
        if (amax_acc) m = vec_amax_bf16(m, v);
        const uint2 w = encode8_bf16<IMPL>(v, scale, lut, hrt, mode);
        uint4 o;
        o.x = descale2_bf16(w.x, w.x >> 8, dec, inv);
        o.y = descale2_bf16(w.x >> 16, w.x >> 24, dec, inv);
        o.z = descale2_bf16(w.y, w.y >> 8, dec, inv);
        o.w = descale2_bf16(w.y >> 16, w.y >> 24, dec, inv);
        st_stream(dst4 + idx, o);
        if (CODES) st_stream(codes8 + idx, w);
      },
      prologue);
  const size_t t = (nvec << 3) + threadIdx.x;
  m = fold_amax_bf16(m);
  if (blockIdx.x == 0 && t < n) {
    const uint32_t xb = (uint32_t)src[t] << 16;
    m = umax(m, xb & 0x7FFFFFFFu);
    const uint32_t c = encode_one<IMPL, true>(scaled_bits(xb, scale), lut, hrt, mode);
    dst[t] = (uint16_t)narrow_bf16(descale_bits(c, dec, inv));
    if (CODES) codes[t] = (uint8_t)c;
  }
  if (amax_acc) block_max_to_global(m, amax_acc);
}

// ------------------------------------------------------------------------------------
// element-per-lane kernels for pointers that do not meet the fast path's alignment
// ------------------------------------------------------------------------------------
template <bool SRC16>
__device__ __forceinline__ uint32_t load_bits(const void* src, size_t i) {
  return SRC16 ? ((uint32_t) reinterpret_cast<const uint16_t*>(src)[i] << 16)
               : __float_as_uint(reinterpret_cast<const float*>(src)[i]);
}
template <bool SRC16>
__device__ __forceinline__ uint32_t encode_any(uint32_t yb, uint32_t mode) {
  return ((mode & 0xFu) == HIF8_RM_HR) ? encode_alu<true, SRC16>(yb, mode)
                                       : encode_alu<false, SRC16>(yb, mode);
}

template <bool SRC16>
__global__ void __launch_bounds__(256)
k_encode_elem(const void* src, uint8_t* dst, size_t n, float scale_arg, const float* d_scale2,
              uint32_t* amax_acc, uint32_t mode) {
  const float scale = d_scale2 ? d_scale2[0] : scale_arg;
  uint32_t m = 0;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
       i += (size_t)gridDim.x * blockDim.x) {
    const uint32_t xb = load_bits<SRC16>(src, i);
    m = umax(m, xb & 0x7FFFFFFFu);
    dst[i] = (uint8_t)encode_any<SRC16>(scaled_bits(xb, scale), mode);
  }
  if (amax_acc) block_max_to_global(m, amax_acc);
}

template <bool DST16>
__global__ void __launch_bounds__(256)
k_decode_elem(const uint8_t* src, void* dst, size_t n, float inv_arg, const float* d_scale2) {
  const float inv = d_scale2 ? d_scale2[1] : inv_arg;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
       i += (size_t)gridDim.x * blockDim.x) {
    const uint32_t b = __float_as_uint(__fmul_rn(__uint_as_float(decode_bits(src[i])), inv));
    if (DST16) reinterpret_cast<uint16_t*>(dst)[i] = (uint16_t)narrow_bf16(b);
    else reinterpret_cast<uint32_t*>(dst)[i] = b;
  }
}

template <bool T16>
__global__ void __launch_bounds__(256)
k_fake_quant_elem(const void* src, void* dst, uint8_t* codes, size_t n, float scale_arg,
                  float inv_arg, const float* d_scale2, uint32_t* amax_acc, uint32_t mode) {
  const float scale = d_scale2 ? d_scale2[0] : scale_arg;
  const float inv = d_scale2 ? d_scale2[1] : inv_arg;
  uint32_t m = 0;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
       i += (size_t)gridDim.x * blockDim.x) {
    const uint32_t xb = load_bits<T16>(src, i);
    m = umax(m, xb & 0x7FFFFFFFu);
    const uint32_t c = encode_any<T16>(scaled_bits(xb, scale), mode);
    const uint32_t b = __float_as_uint(__fmul_rn(__uint_as_float(decode_bits(c)), inv));
    if (T16) reinterpret_cast<uint16_t*>(dst)[i] = (uint16_t)narrow_bf16(b);
    else reinterpret_cast<uint32_t*>(dst)[i] = b;
    if (codes) codes[i] = (uint8_t)c;
  }
  if (amax_acc) block_max_to_global(m, amax_acc);
}

// ------------------------------------------------------------------------------------
// amax
// ------------------------------------------------------------------------------------
__global__ void k_fill_u32(uint32_t* p, uint32_t v, uint32_t count) {
  const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < count) p[i] = v;
}

// magnitude patterns as binary32 bits: FP32 -> bits & 0x7FFFFFFF; BF16 -> (bits & 0x7FFF) << 16
template <int U, bool SRC16, bool NT>
__global__ void __launch_bounds__(1024)
k_amax(const void* __restrict__ src, size_t n, uint32_t* __restrict__ out, Walk walk) {
  const uint4* __restrict__ src4 = reinterpret_cast<const uint4*>(src);
  const size_t nvec = SRC16 ? (n >> 3) : (n >> 2);
  uint32_t m = 0;  // FP32: magnitude pattern; BF16: two 15-bit magnitudes, one per half
  tile_loop<U, uint4>(
      nvec, walk, [&](size_t idx) { return NT ? ld_stream(src4 + idx) : src4[idx]; },
      [&](size_t, const uint4& v) { m = SRC16 ? vec_amax_bf16(m, v) : vec_amax_f32(m, v); },
      []() {});
  if (SRC16) m = fold_amax_bf16(m);
  const size_t t = (SRC16 ? (nvec << 3) : (nvec << 2)) + threadIdx.x;
  if (blockIdx.x == 0 && t < n) {
    const uint32_t a = SRC16 ? (((uint32_t) reinterpret_cast<const uint16_t*>(src)[t] & 0x7FFFu) << 16)
                             : (__float_as_uint(reinterpret_cast<const float*>(src)[t]) & 0x7FFFFFFFu);
    m = umax(m, a);
  }
  block_max_to_global(m, out);
}

template <bool SRC16>
__global__ void __launch_bounds__(256)
k_amax_elem(const void* __restrict__ src, size_t n, uint32_t* __restrict__ out) {
  uint32_t m = 0;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
       i += (size_t)gridDim.x * blockDim.x) {
    const uint32_t a = SRC16 ? (((uint32_t) reinterpret_cast<const uint16_t*>(src)[i] & 0x7FFFu) << 16)
                             : (__float_as_uint(reinterpret_cast<const float*>(src)[i]) & 0x7FFFFFFFu);
    m = umax(m, a);
  }
  block_max_to_global(m, out);
}

// scale = fl32(target / amax) (optionally floored to a power of two), inverse = fl32(1 / scale)
__global__ void k_scale_from_amax(const float* d_amax, float* d_scale2, uint32_t count, float target,
                                  int pow2) {
  const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= count) return;
  d_amax += i;
  d_scale2 += 2 * i;
  const float amax = *d_amax;
  const uint32_t ab = __float_as_uint(amax);
  float s = 1.0f;
  if (ab != 0u && ab < 0x7F800000u) {  // positive, finite, non-zero
    const float q = target / amax;     // correctly rounded divide
    const uint32_t qb = __float_as_uint(q);
    if (qb != 0u && qb < 0x7F800000u) {
      s = q;
      if (pow2) {
        if ((qb >> 23) != 0u) s = __uint_as_float(qb & 0x7F800000u);
        else s = __uint_as_float(1u << (31 - __clz((int)qb)));  // subnormal quotient
      }
    }
  }
  d_scale2[0] = s;
  d_scale2[1] = 1.0f / s;
}

// ------------------------------------------------------------------------------------
// multi-tensor cast: many tensors per launch (amax, then scale, then encode), so that a
// list of small tensors is not bound by launch gaps.  All tensors share one global tile
// index space; items[i].first_tile is the prefix sum of tile counts.  A tile is
// kMultiBlock * kMultiUnroll vector units of one tensor.
// ------------------------------------------------------------------------------------
constexpr int kMultiBlock = 512;
constexpr int kMultiUnroll = 2;
constexpr uint32_t kMultiTileVec = kMultiBlock * kMultiUnroll;
constexpr uint32_t kMultiTpwEncode = 2;
constexpr uint32_t kMultiTpwAmax = 8;

// largest i with items[i].first_tile <= tile (zero-size items are skipped by construction)
__device__ __forceinline__ uint32_t multi_find_item(const hif8_cast_item* __restrict__ items,
                                                    uint32_t count, uint64_t tile) {
  uint32_t lo = 0, hi = count;
  while (hi - lo > 1u) {
    const uint32_t mid = (lo + hi) >> 1;
    if (items[mid].first_tile <= tile) lo = mid; else hi = mid;
  }
  return lo;
}

template <bool SRC16>
__device__ __forceinline__ uint64_t multi_item_tiles(uint64_t n) {
  const uint64_t nvec = SRC16 ? (n >> 3) : (n >> 2);
  const uint64_t t = (nvec + kMultiTileVec - 1) / kMultiTileVec;
  return (t == 0 && n != 0) ? 1 : t;
}

template <bool SRC16>
__global__ void __launch_bounds__(kMultiBlock)
k_multi_amax(const hif8_cast_item* __restrict__ items, uint32_t count, uint64_t total_tiles,
             uint32_t* __restrict__ amax_out) {
  uint32_t m = 0;
  uint32_t cur = 0xFFFFFFFFu;
  for (uint32_t i = 0; i < kMultiTpwAmax; ++i) {
    const uint64_t tile = (uint64_t)blockIdx.x * kMultiTpwAmax + i;
    if (tile >= total_tiles) break;
    const uint32_t it = multi_find_item(items, count, tile);
    if (it != cur) {
      if (cur != 0xFFFFFFFFu) {
        block_max_to_global(SRC16 ? (umax(m & 0xFFFFu, m >> 16) << 16) : m, amax_out + cur);
        __syncthreads();
      }
      cur = it;
      m = 0;
    }
    const uint64_t n = items[it].n;
    const uint64_t nvec = SRC16 ? (n >> 3) : (n >> 2);
    const uint64_t local = tile - items[it].first_tile;
    const uint4* __restrict__ src4 = reinterpret_cast<const uint4*>(items[it].src);
    const uint64_t first = local * kMultiTileVec + threadIdx.x;
    uint4 v[kMultiUnroll];
#pragma unroll
    for (int j = 0; j < kMultiUnroll; ++j) {
      const uint64_t idx = first + (uint64_t)j * kMultiBlock;
      v[j] = (idx < nvec) ? ld_stream(src4 + idx) : make_uint4(0u, 0u, 0u, 0u);
    }
#pragma unroll
    for (int j = 0; j < kMultiUnroll; ++j) {
      if (SRC16) {
        typedef uint16_t u16x2 __attribute__((ext_vector_type(2)));
        u16x2 mm = __builtin_bit_cast(u16x2, m);
        mm = __builtin_elementwise_max(mm, __builtin_bit_cast(u16x2, v[j].x & 0x7FFF7FFFu));
        mm = __builtin_elementwise_max(mm, __builtin_bit_cast(u16x2, v[j].y & 0x7FFF7FFFu));
        mm = __builtin_elementwise_max(mm, __builtin_bit_cast(u16x2, v[j].z & 0x7FFF7FFFu));
        mm = __builtin_elementwise_max(mm, __builtin_bit_cast(u16x2, v[j].w & 0x7FFF7FFFu));
        m = __builtin_bit_cast(uint32_t, mm);
      } else {
        m = umax(m, umax(umax(v[j].x & 0x7FFFFFFFu, v[j].y & 0x7FFFFFFFu),
                         umax(v[j].z & 0x7FFFFFFFu, v[j].w & 0x7FFFFFFFu)));
      }
    }
    // ragged tail of the tensor, done with its last tile
    if (local + 1 == multi_item_tiles<SRC16>(n)) {
      const uint64_t t = (SRC16 ? (nvec << 3) : (nvec << 2)) + threadIdx.x;
      if (t < n) {
        // BF16: m holds two 15-bit running maxima; a 15-bit value can join either half
        if (SRC16) m = (m & 0xFFFF0000u) | umax(m & 0xFFFFu, (uint32_t) reinterpret_cast<const uint16_t*>(items[it].src)[t] & 0x7FFFu);
        else m = umax(m, __float_as_uint(reinterpret_cast<const float*>(items[it].src)[t]) & 0x7FFFFFFFu);
      }
    }
  }
  if (cur != 0xFFFFFFFFu) block_max_to_global(SRC16 ? (umax(m & 0xFFFFu, m >> 16) << 16) : m, amax_out + cur);
}

template <int IMPL, bool SRC16>
__global__ void __launch_bounds__(kMultiBlock)
k_multi_encode(const hif8_cast_item* __restrict__ items, uint32_t count, uint64_t total_tiles,
               const float* __restrict__ d_scale2, uint32_t mode) {
  __shared__ __attribute__((aligned(16))) uint8_t lut[8192];
  __shared__ __attribute__((aligned(8))) HrExp hrt[IMPL == IMPL_HR ? 256 : 1];
  stage_enc_lut(lut, mode);
  if (IMPL == IMPL_HR) stage_hr_table(hrt);
  __syncthreads();
  for (uint32_t i = 0; i < kMultiTpwEncode; ++i) {
    const uint64_t tile = (uint64_t)blockIdx.x * kMultiTpwEncode + i;
    if (tile >= total_tiles) break;
    const uint32_t it = multi_find_item(items, count, tile);
    const uint64_t n = items[it].n;
    const uint64_t nvec = SRC16 ? (n >> 3) : (n >> 2);
    const uint64_t local = tile - items[it].first_tile;
    const float scale = d_scale2 ? d_scale2[2 * it] : 1.0f;
    const uint4* __restrict__ src4 = reinterpret_cast<const uint4*>(items[it].src);
    uint8_t* __restrict__ dst = items[it].dst;
    const uint64_t first = local * kMultiTileVec + threadIdx.x;
    uint4 v[kMultiUnroll];
#pragma unroll
    for (int j = 0; j < kMultiUnroll; ++j) {
      const uint64_t idx = first + (uint64_t)j * kMultiBlock;
      if (idx < nvec) v[j] = ld_stream(src4 + idx);
    }
#pragma unroll
    for (int j = 0; j < kMultiUnroll; ++j) {
      const uint64_t idx = first + (uint64_t)j * kMultiBlock;
      if (idx < nvec) {
        if (SRC16) st_stream(reinterpret_cast<uint2*>(dst) + idx, encode8_bf16<IMPL>(v[j], scale, lut, hrt, mode));
        else st_stream(reinterpret_cast<uint32_t*>(dst) + idx, encode4_f32<IMPL>(v[j], scale, lut, hrt, mode));
      }
    }
    if (local + 1 == multi_item_tiles<SRC16>(n)) {
      const uint64_t t = (SRC16 ? (nvec << 3) : (nvec << 2)) + threadIdx.x;
      if (t < n) {
        const uint32_t xb = SRC16 ? ((uint32_t) reinterpret_cast<const uint16_t*>(items[it].src)[t] << 16)
                                  : __float_as_uint(reinterpret_cast<const float*>(items[it].src)[t]);
        dst[t] = (uint8_t)encode_one<IMPL, SRC16>(scaled_bits(xb, scale), lut, hrt, mode);
      }
    }
  }
}

// diagnostic stream kernel: read 16 B per lane, write the first OUT bytes of it
template <int U, int OUT>
__global__ void __launch_bounds__(1024)
k_diag_stream(const uint4* __restrict__ src, void* __restrict__ dst, size_t nvec, Walk walk) {
  tile_loop<U, uint4>(
      nvec, walk, [&](size_t idx) { return ld_stream(src + idx); },
      [&](size_t idx, const uint4& v) {
        if (OUT == 4) st_stream(reinterpret_cast<uint32_t*>(dst) + idx, v.x);
        else if (OUT == 8) st_stream(reinterpret_cast<uint2*>(dst) + idx, make_uint2(v.x, v.y));
        else st_stream(reinterpret_cast<uint4*>(dst) + idx, v);
      },
      []() {});
}

// ====================================================================================
// host side: C ABI
// ====================================================================================
namespace {

thread_local int t_last_hip_error = 0;

// Launch shape of one kernel family.  tiles_per_wg == 0 selects the persistent grid.
struct Shape {
  int block;
  int unroll;
  int tiles_per_wg;
  int wg_per_cu;
};
enum Family { FAM_ENC32_TA, FAM_ENC32_HR, FAM_ENC16, FAM_FQ, FAM_DEC, FAM_AMAX, FAM_DIAG, FAM_COUNT };
// Defaults from a sweep on MI355X under sustained load (hundreds of back-to-back launches on
// 64 Mi-element tensors; short bursts rank the shapes differently): one-shot grids of
// 512-lane workgroups with 16-32 KiB of source per staged table win for the read+write
// kernels, a persistent grid of one 1024-lane workgroup per CU wins for the read-only reduction.
const Shape kDefaultShape[FAM_COUNT] = {
    {512, 2, 2, 4},   // FP32 encode, TA
    {512, 4, 1, 4},   // FP32 encode, HR
    {512, 2, 2, 4},   // BF16 encode
    {512, 2, 2, 4},   // fake-quant
    {512, 2, 1, 4},   // decode
    {1024, 2, 0, 1},  // amax
    {512, 1, 2, 4},   // diagnostic stream
};

// user overrides; -1 = use the family default
struct Tuning {
  int block = -1;
  int wg_per_cu = -1;
  int unroll = -1;
  int ta_impl = 0;
  int tiles_per_wg = -1;
  int amax_nt = 1;
};
Tuning g_tune;

Shape shape_for(Family f) {
  Shape s = kDefaultShape[f];
  if (g_tune.block >= 0) s.block = g_tune.block;
  if (g_tune.unroll >= 0) s.unroll = g_tune.unroll;
  if (g_tune.tiles_per_wg >= 0) s.tiles_per_wg = g_tune.tiles_per_wg;
  if (g_tune.wg_per_cu >= 0) s.wg_per_cu = g_tune.wg_per_cu;
  return s;
}

constexpr int kMaxDevices = 64;
std::mutex g_init_mutex;
bool g_inited[kMaxDevices] = {};
int g_cu_count[kMaxDevices] = {};

bool hip_ok(hipError_t e) {
  if (e == hipSuccess) return true;
  t_last_hip_error = (int)e;
  return false;
}

hif8_status ensure_init(int* cu_count_out) {
  int dev = 0;
  if (!hip_ok(hipGetDevice(&dev))) return HIF8_ERR_HIP;
  if (dev < 0 || dev >= kMaxDevices) return HIF8_ERR_ARG;
  std::lock_guard<std::mutex> lock(g_init_mutex);
  if (!g_inited[dev]) {
    int cus = 0;
    if (!hip_ok(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev)))
      return HIF8_ERR_HIP;
    if (cus <= 0) cus = 256;
    hipLaunchKernelGGL(k_build_tables, dim3(8192 / 256), dim3(256), 0, (hipStream_t)0);
    if (!hip_ok(hipGetLastError())) return HIF8_ERR_HIP;
    // the null stream synchronises with every blocking stream; wait on the host as well so
    // that non-blocking streams also see the tables
    if (!hip_ok(hipStreamSynchronize((hipStream_t)0))) return HIF8_ERR_HIP;
    g_cu_count[dev] = cus;
    g_inited[dev] = true;
  }
  if (cu_count_out) *cu_count_out = g_cu_count[dev];
  return HIF8_OK;
}

bool aligned_to(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

bool valid_mode(uint32_t mode) {
  if ((mode & ~(HIF8_RM_MASK | HIF8_FLAG_SAT | HIF8_FLAG_NAN2ZERO)) != 0) return false;
  const uint32_t rm = mode & HIF8_RM_MASK;
  return rm == HIF8_RM_TA || rm == HIF8_RM_HR;
}

// scale and fl32(1/scale) both finite and positive
bool valid_scale(float scale, float* inv_out) {
  if (!(scale > 0.0f) || std::isinf(scale)) return false;
  volatile float inv = 1.0f / scale;
  if (!(inv > 0.0f) || std::isinf((float)inv)) return false;
  *inv_out = inv;
  return true;
}

// grid size and tile walk for nvec vector units under the current tuning
unsigned grid_for(size_t nvec, int cus, const Shape& sh, Walk* walk) {
  const size_t tile = (size_t)sh.block * (size_t)sh.unroll;
  size_t tiles = (nvec + tile - 1) / tile;
  if (tiles == 0) tiles = 1;  // block 0 still handles a ragged tail
  size_t grid;
  if (sh.tiles_per_wg > 0) {
    const size_t tpw = (size_t)sh.tiles_per_wg;
    grid = (tiles + tpw - 1) / tpw;
    *walk = Walk{(uint32_t)tpw, 1u, (uint32_t)tpw};
  } else {
    const size_t cap = (size_t)cus * (size_t)sh.wg_per_cu;
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

int impl_for(uint32_t mode) {
  if ((mode & HIF8_RM_MASK) == HIF8_RM_HR) return IMPL_HR;
  return g_tune.ta_impl ? IMPL_TA_ALU : IMPL_TA_LUT;
}

#define HIF8_DISPATCH_U(CALL)             \
  switch (shape.unroll) {                 \
    case 1: { constexpr int U = 1; CALL; } break; \
    case 2: { constexpr int U = 2; CALL; } break; \
    case 8: { constexpr int U = 8; CALL; } break; \
    default: { constexpr int U = 4; CALL; } break; \
  }

#define HIF8_DISPATCH_IMPL(IMPLV, CALL)                                   \
  switch (IMPLV) {                                                        \
    case IMPL_TA_ALU: { constexpr int IMPL = IMPL_TA_ALU; CALL; } break;  \
    case IMPL_HR: { constexpr int IMPL = IMPL_HR; CALL; } break;          \
    default: { constexpr int IMPL = IMPL_TA_LUT; CALL; } break;           \
  }

hif8_status finish_launch() { return hip_ok(hipGetLastError()) ? HIF8_OK : HIF8_ERR_HIP; }

// ---- common implementations (scale either by value or from device memory) ----
template <bool SRC16>
hif8_status do_encode(const void* src, uint8_t* dst, size_t n, float scale, const float* d_scale2,
                      float* d_amax_acc, uint32_t mode, hipStream_t st) {
  uint32_t* amax_acc = reinterpret_cast<uint32_t*>(d_amax_acc);
  if (!valid_mode(mode)) return HIF8_ERR_MODE;
  float inv = 1.0f;
  if (!d_scale2 && !valid_scale(scale, &inv)) return HIF8_ERR_SCALE;
  if (n == 0) return HIF8_OK;
  if (!src || !dst) return HIF8_ERR_NULL;
  int cus = 0;
  hif8_status s = ensure_init(&cus);
  if (s != HIF8_OK) return s;
  const bool fast = aligned_to(src, 16) && aligned_to(dst, SRC16 ? 8 : 4);
  if (!fast) {
    hipLaunchKernelGGL(k_encode_elem<SRC16>, dim3(grid_elem(n, cus)), dim3(256), 0, st, src, dst, n,
                       scale, d_scale2, amax_acc, mode);
    return finish_launch();
  }
  const size_t nvec = SRC16 ? (n >> 3) : (n >> 2);
  const int impl = impl_for(mode);
  const Shape shape = shape_for(SRC16 ? FAM_ENC16 : (impl == IMPL_HR ? FAM_ENC32_HR : FAM_ENC32_TA));
  Walk walk;
  const dim3 grid(grid_for(nvec, cus, shape, &walk)), block(shape.block);
  if (SRC16) {
    HIF8_DISPATCH_U(HIF8_DISPATCH_IMPL(impl, hipLaunchKernelGGL((k_encode_bf16<U, IMPL>), grid, block, 0, st,
        reinterpret_cast<const uint16_t*>(src), dst, n, scale, d_scale2, amax_acc, mode, walk)))
  } else {
    HIF8_DISPATCH_U(HIF8_DISPATCH_IMPL(impl, hipLaunchKernelGGL((k_encode_f32<U, IMPL>), grid, block, 0, st,
        reinterpret_cast<const float*>(src), dst, n, scale, d_scale2, amax_acc, mode, walk)))
  }
  return finish_launch();
}

template <bool DST16>
hif8_status do_decode(const uint8_t* src, void* dst, size_t n, float scale, const float* d_scale2,
                      hipStream_t st) {
  float inv = 1.0f;
  if (!d_scale2 && !valid_scale(scale, &inv)) return HIF8_ERR_SCALE;
  if (n == 0) return HIF8_OK;
  if (!src || !dst) return HIF8_ERR_NULL;
  int cus = 0;
  hif8_status s = ensure_init(&cus);
  if (s != HIF8_OK) return s;
  const bool fast = aligned_to(src, DST16 ? 8 : 4) && aligned_to(dst, 16);
  if (!fast) {
    hipLaunchKernelGGL(k_decode_elem<DST16>, dim3(grid_elem(n, cus)), dim3(256), 0, st, src, dst, n,
                       inv, d_scale2);
    return finish_launch();
  }
  const size_t nvec = DST16 ? (n >> 3) : (n >> 2);
  const Shape shape = shape_for(FAM_DEC);
  Walk walk;
  const dim3 grid(grid_for(nvec, cus, shape, &walk)), block(shape.block);
  if (DST16) {
    HIF8_DISPATCH_U(hipLaunchKernelGGL((k_decode_bf16<U>), grid, block, 0, st, src,
                                       reinterpret_cast<uint16_t*>(dst), n, inv, d_scale2, walk))
  } else {
    HIF8_DISPATCH_U(hipLaunchKernelGGL((k_decode_f32<U>), grid, block, 0, st, src,
                                       reinterpret_cast<float*>(dst), n, inv, d_scale2, walk))
  }
  return finish_launch();
}

template <bool T16>
hif8_status do_fake_quant(const void* src, void* dst, uint8_t* codes, size_t n, float scale,
                          const float* d_scale2, float* d_amax_acc, uint32_t mode, hipStream_t st) {
  uint32_t* amax_acc = reinterpret_cast<uint32_t*>(d_amax_acc);
  if (!valid_mode(mode)) return HIF8_ERR_MODE;
  float inv = 1.0f;
  if (!d_scale2 && !valid_scale(scale, &inv)) return HIF8_ERR_SCALE;
  if (n == 0) return HIF8_OK;
  if (!src || !dst) return HIF8_ERR_NULL;
  int cus = 0;
  hif8_status s = ensure_init(&cus);
  if (s != HIF8_OK) return s;
  const bool fast = aligned_to(src, 16) && aligned_to(dst, 16) && (!codes || aligned_to(codes, T16 ? 8 : 4));
  if (!fast) {
    hipLaunchKernelGGL(k_fake_quant_elem<T16>, dim3(grid_elem(n, cus)), dim3(256), 0, st, src, dst,
                       codes, n, scale, inv, d_scale2, amax_acc, mode);
    return finish_launch();
  }
  const size_t nvec = T16 ? (n >> 3) : (n >> 2);
  const Shape shape = shape_for(FAM_FQ);
  Walk walk;
  const dim3 grid(grid_for(nvec, cus, shape, &walk)), block(shape.block);
  const int impl = impl_for(mode);
#define HIF8_FQ_LAUNCH(KERNEL, TS, TD, CODESV)                                                        \
  HIF8_DISPATCH_U(HIF8_DISPATCH_IMPL(impl, hipLaunchKernelGGL((KERNEL<U, IMPL, CODESV>), grid, block, \
      0, st, reinterpret_cast<TS>(src), reinterpret_cast<TD>(dst), codes, n, scale, inv, d_scale2, amax_acc, mode, walk)))
  if (T16) {
    if (codes) { HIF8_FQ_LAUNCH(k_fake_quant_bf16, const uint16_t*, uint16_t*, true) }
    else { HIF8_FQ_LAUNCH(k_fake_quant_bf16, const uint16_t*, uint16_t*, false) }
  } else {
    if (codes) { HIF8_FQ_LAUNCH(k_fake_quant_f32, const float*, float*, true) }
    else { HIF8_FQ_LAUNCH(k_fake_quant_f32, const float*, float*, false) }
  }
#undef HIF8_FQ_LAUNCH
  return finish_launch();
}

template <bool SRC16>
hif8_status do_amax(const void* src, size_t n, float* d_amax, hipStream_t st) {
  if (!d_amax || (!src && n != 0)) return HIF8_ERR_NULL;
  int cus = 0;
  hif8_status s = ensure_init(&cus);
  if (s != HIF8_OK) return s;
  uint32_t* out = reinterpret_cast<uint32_t*>(d_amax);
  hipLaunchKernelGGL(k_fill_u32, dim3(1), dim3(64), 0, st, out, 0u, 1u);
  if (!hip_ok(hipGetLastError())) return HIF8_ERR_HIP;
  if (n == 0) return HIF8_OK;
  if (!aligned_to(src, 16)) {
    hipLaunchKernelGGL(k_amax_elem<SRC16>, dim3(grid_elem(n, cus)), dim3(256), 0, st, src, n, out);
    return finish_launch();
  }
  const size_t nvec = SRC16 ? (n >> 3) : (n >> 2);
  const Shape shape = shape_for(FAM_AMAX);
  Walk walk;
  const dim3 grid(grid_for(nvec, cus, shape, &walk)), block(shape.block);
  if (g_tune.amax_nt) { HIF8_DISPATCH_U(hipLaunchKernelGGL((k_amax<U, SRC16, true>), grid, block, 0, st, src, n, out, walk)) }
  else { HIF8_DISPATCH_U(hipLaunchKernelGGL((k_amax<U, SRC16, false>), grid, block, 0, st, src, n, out, walk)) }
  return finish_launch();
}

}  // namespace

extern "C" {

int hif8_version(void) { return 100; }
int hif8_last_hip_error(void) { return t_last_hip_error; }
hif8_status hif8_init(void) { return ensure_init(nullptr); }

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
      if (value != 0 && value != 1) return HIF8_ERR_ARG;
      g_tune.amax_nt = value;
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
    default: return -1;
  }
}

hif8_status hif8_amax_f32(const float* src, size_t n, float* d_amax, hif8_stream_t stream) {
  return do_amax<false>(src, n, d_amax, (hipStream_t)stream);
}
hif8_status hif8_amax_bf16(const uint16_t* src, size_t n, float* d_amax, hif8_stream_t stream) {
  return do_amax<true>(src, n, d_amax, (hipStream_t)stream);
}

hif8_status hif8_scale_from_amax(const float* d_amax, float* d_scale2, float target, int pow2,
                                 hif8_stream_t stream) {
  if (!d_amax || !d_scale2) return HIF8_ERR_NULL;
  if (!(target > 0.0f) || std::isinf(target)) return HIF8_ERR_ARG;
  hipLaunchKernelGGL(k_scale_from_amax, dim3(1), dim3(64), 0, (hipStream_t)stream, d_amax, d_scale2,
                     1u, target, pow2);
  return finish_launch();
}

hif8_status hif8_encode_f32(const float* src, uint8_t* dst, size_t n, float scale, uint32_t mode,
                            hif8_stream_t stream) {
  return do_encode<false>(src, dst, n, scale, nullptr, nullptr, mode, (hipStream_t)stream);
}
hif8_status hif8_encode_bf16(const uint16_t* src, uint8_t* dst, size_t n, float scale,
                             uint32_t mode, hif8_stream_t stream) {
  return do_encode<true>(src, dst, n, scale, nullptr, nullptr, mode, (hipStream_t)stream);
}
hif8_status hif8_decode_f32(const uint8_t* src, float* dst, size_t n, float scale,
                            hif8_stream_t stream) {
  return do_decode<false>(src, dst, n, scale, nullptr, (hipStream_t)stream);
}
hif8_status hif8_decode_bf16(const uint8_t* src, uint16_t* dst, size_t n, float scale,
                             hif8_stream_t stream) {
  return do_decode<true>(src, dst, n, scale, nullptr, (hipStream_t)stream);
}
hif8_status hif8_fake_quant_f32(const float* src, float* dst, uint8_t* codes, size_t n, float scale,
                                uint32_t mode, hif8_stream_t stream) {
  return do_fake_quant<false>(src, dst, codes, n, scale, nullptr, nullptr, mode, (hipStream_t)stream);
}
hif8_status hif8_fake_quant_bf16(const uint16_t* src, uint16_t* dst, uint8_t* codes, size_t n,
                                 float scale, uint32_t mode, hif8_stream_t stream) {
  return do_fake_quant<true>(src, dst, codes, n, scale, nullptr, nullptr, mode, (hipStream_t)stream);
}

hif8_status hif8_encode_f32_ds(const float* src, uint8_t* dst, size_t n, const float* d_scale2,
                               float* d_amax_acc, uint32_t mode, hif8_stream_t stream) {
  if (!d_scale2) return HIF8_ERR_NULL;
  return do_encode<false>(src, dst, n, 1.0f, d_scale2, d_amax_acc, mode, (hipStream_t)stream);
}
hif8_status hif8_encode_bf16_ds(const uint16_t* src, uint8_t* dst, size_t n, const float* d_scale2,
                                float* d_amax_acc, uint32_t mode, hif8_stream_t stream) {
  if (!d_scale2) return HIF8_ERR_NULL;
  return do_encode<true>(src, dst, n, 1.0f, d_scale2, d_amax_acc, mode, (hipStream_t)stream);
}
hif8_status hif8_decode_f32_ds(const uint8_t* src, float* dst, size_t n, const float* d_scale2,
                               hif8_stream_t stream) {
  if (!d_scale2) return HIF8_ERR_NULL;
  return do_decode<false>(src, dst, n, 1.0f, d_scale2, (hipStream_t)stream);
}
hif8_status hif8_decode_bf16_ds(const uint8_t* src, uint16_t* dst, size_t n, const float* d_scale2,
                                hif8_stream_t stream) {
  if (!d_scale2) return HIF8_ERR_NULL;
  return do_decode<true>(src, dst, n, 1.0f, d_scale2, (hipStream_t)stream);
}
hif8_status hif8_fake_quant_f32_ds(const float* src, float* dst, uint8_t* codes, size_t n,
                                   const float* d_scale2, float* d_amax_acc, uint32_t mode,
                                   hif8_stream_t stream) {
  if (!d_scale2) return HIF8_ERR_NULL;
  return do_fake_quant<false>(src, dst, codes, n, 1.0f, d_scale2, d_amax_acc, mode, (hipStream_t)stream);
}
hif8_status hif8_fake_quant_bf16_ds(const uint16_t* src, uint16_t* dst, uint8_t* codes, size_t n,
                                    const float* d_scale2, float* d_amax_acc, uint32_t mode,
                                    hif8_stream_t stream) {
  if (!d_scale2) return HIF8_ERR_NULL;
  return do_fake_quant<true>(src, dst, codes, n, 1.0f, d_scale2, d_amax_acc, mode, (hipStream_t)stream);
}

hif8_status hif8_multi_plan(hif8_cast_item* host_items, size_t count, int src_is_bf16,
                            uint64_t* total_tiles_out) {
  if (!total_tiles_out || (!host_items && count != 0)) return HIF8_ERR_NULL;
  if (count > 0xFFFFFFu) return HIF8_ERR_ARG;
  uint64_t tiles = 0;
  for (size_t i = 0; i < count; ++i) {
    hif8_cast_item& it = host_items[i];
    if (it.n != 0 && (!it.src || !it.dst)) return HIF8_ERR_NULL;
    if (!aligned_to(it.src, 16) || !aligned_to(it.dst, src_is_bf16 ? 8 : 4)) return HIF8_ERR_ARG;
    it.first_tile = tiles;
    const uint64_t nvec = src_is_bf16 ? (it.n >> 3) : (it.n >> 2);
    uint64_t t = (nvec + kMultiTileVec - 1) / kMultiTileVec;
    if (t == 0 && it.n != 0) t = 1;
    tiles += t;
  }
  *total_tiles_out = tiles;
  return HIF8_OK;
}

static hif8_status multi_cast(const hif8_cast_item* d_items, size_t count, uint64_t total_tiles,
                              float* d_amax, float* d_scale2, float target, int pow2, uint32_t mode,
                              bool bf16, hipStream_t st) {
  if (!valid_mode(mode)) return HIF8_ERR_MODE;
  if (!(target > 0.0f) || std::isinf(target)) return HIF8_ERR_ARG;
  if (count == 0) return HIF8_OK;
  if (!d_items || !d_amax || !d_scale2) return HIF8_ERR_NULL;
  if (count > 0xFFFFFFu) return HIF8_ERR_ARG;
  hif8_status s = ensure_init(nullptr);
  if (s != HIF8_OK) return s;
  const uint32_t cnt = (uint32_t)count;
  uint32_t* am = reinterpret_cast<uint32_t*>(d_amax);
  hipLaunchKernelGGL(k_fill_u32, dim3((cnt + 255) / 256), dim3(256), 0, st, am, 0u, cnt);
  if (total_tiles != 0) {
    const unsigned g1 = (unsigned)((total_tiles + kMultiTpwAmax - 1) / kMultiTpwAmax);
    if (bf16) hipLaunchKernelGGL(k_multi_amax<true>, dim3(g1), dim3(kMultiBlock), 0, st, d_items, cnt, total_tiles, am);
    else hipLaunchKernelGGL(k_multi_amax<false>, dim3(g1), dim3(kMultiBlock), 0, st, d_items, cnt, total_tiles, am);
  }
  hipLaunchKernelGGL(k_scale_from_amax, dim3((cnt + 255) / 256), dim3(256), 0, st, d_amax, d_scale2, cnt,
                     target, pow2);
  if (total_tiles != 0) {
    const unsigned g2 = (unsigned)((total_tiles + kMultiTpwEncode - 1) / kMultiTpwEncode);
    const bool hr = (mode & HIF8_RM_MASK) == HIF8_RM_HR;
    if (bf16) {
      if (hr) hipLaunchKernelGGL((k_multi_encode<IMPL_HR, true>), dim3(g2), dim3(kMultiBlock), 0, st, d_items, cnt, total_tiles, d_scale2, mode);
      else hipLaunchKernelGGL((k_multi_encode<IMPL_TA_LUT, true>), dim3(g2), dim3(kMultiBlock), 0, st, d_items, cnt, total_tiles, d_scale2, mode);
    } else {
      if (hr) hipLaunchKernelGGL((k_multi_encode<IMPL_HR, false>), dim3(g2), dim3(kMultiBlock), 0, st, d_items, cnt, total_tiles, d_scale2, mode);
      else hipLaunchKernelGGL((k_multi_encode<IMPL_TA_LUT, false>), dim3(g2), dim3(kMultiBlock), 0, st, d_items, cnt, total_tiles, d_scale2, mode);
    }
  }
  return finish_launch();
}

hif8_status hif8_multi_cast_bf16(const hif8_cast_item* d_items, size_t count, uint64_t total_tiles,
                                 float* d_amax, float* d_scale2, float target, int pow2,
                                 uint32_t mode, hif8_stream_t stream) {
  return multi_cast(d_items, count, total_tiles, d_amax, d_scale2, target, pow2, mode, true,
                    (hipStream_t)stream);
}
hif8_status hif8_multi_cast_f32(const hif8_cast_item* d_items, size_t count, uint64_t total_tiles,
                                float* d_amax, float* d_scale2, float target, int pow2,
                                uint32_t mode, hif8_stream_t stream) {
  return multi_cast(d_items, count, total_tiles, d_amax, d_scale2, target, pow2, mode, false,
                    (hipStream_t)stream);
}

hif8_status hif8_diag_stream(const void* src, void* dst, size_t n_groups, int out_bytes,
                             hif8_stream_t stream) {
  if (!src || !dst) return HIF8_ERR_NULL;
  if (out_bytes != 4 && out_bytes != 8 && out_bytes != 16) return HIF8_ERR_ARG;
  if (!aligned_to(src, 16) || !aligned_to(dst, (size_t)out_bytes)) return HIF8_ERR_ARG;
  if (n_groups == 0) return HIF8_OK;
  int cus = 0;
  hif8_status s = ensure_init(&cus);
  if (s != HIF8_OK) return s;
  const Shape shape = shape_for(FAM_DIAG);
  Walk walk;
  const dim3 grid(grid_for(n_groups, cus, shape, &walk)), block(shape.block);
  const uint4* s4 = reinterpret_cast<const uint4*>(src);
  hipStream_t st = (hipStream_t)stream;
  if (out_bytes == 4) { HIF8_DISPATCH_U(hipLaunchKernelGGL((k_diag_stream<U, 4>), grid, block, 0, st, s4, dst, n_groups, walk)) }
  else if (out_bytes == 8) { HIF8_DISPATCH_U(hipLaunchKernelGGL((k_diag_stream<U, 8>), grid, block, 0, st, s4, dst, n_groups, walk)) }
  else { HIF8_DISPATCH_U(hipLaunchKernelGGL((k_diag_stream<U, 16>), grid, block, 0, st, s4, dst, n_groups, walk)) }
  return finish_launch();
}

}  // extern "C"
