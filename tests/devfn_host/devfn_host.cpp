// CPU build of the HIP library's device-side bit logic (hif8_device.hpp), for tests that
// run where there is no GPU.  Test infrastructure: it lets the encode / decode bit
// manipulation be compared with the oracle on the CPU before (and besides) the GPU parity
// tests.  Not part of the product and never loaded by it.
#include <stdint.h>
#include <stddef.h>
#define HIF8_DEVICE_HOST_SHIM 1
#define __device__
#define __host__
#define __forceinline__ inline
static inline int __clz(int x) { return x == 0 ? 32 : __builtin_clz((unsigned)x); }
#include "../../paper_2409_16626_amd/csrc/hif8_device.hpp"
#include "../../paper_2409_16626_amd/csrc/hif8_gemm_split.hpp"

extern "C" {
// per-tensor scale from an amax (the arithmetic of the scale kernels)
void devfn_scale_from_amax(const float* amax, float* out, size_t n, float target, int pow2) {
  for (size_t i = 0; i < n; ++i) out[i] = hif8dev::scale_from_amax_value(amax[i], target, pow2);
}
// generic element-wise form (any rounding method, any source kind)
void devfn_encode_bits(const uint32_t* ybits, uint8_t* dst, size_t n, uint32_t mode, int srck,
                       uint64_t seed) {
  for (size_t i = 0; i < n; ++i) {
    const uint32_t t = hif8dev::sr_threshold(seed, (uint64_t)i);
    uint32_t c;
    if (srck == 0) c = hif8dev::encode_any<0>(ybits[i], mode, t);
    else if (srck == 1) c = hif8dev::encode_any<1>(ybits[i], mode, t);
    else c = hif8dev::encode_any<2>(ybits[i], mode, t);
    dst[i] = (uint8_t)c;
  }
}
// table-driven hybrid rounding (or simplified SR everywhere) of binary32 sources, then the TA code of
// the (representable) result
void devfn_encode_bits_hr_table(const uint32_t* ybits, uint8_t* dst, size_t n, uint32_t mode) {
  const bool ssr = (mode & 0xF) == hif8dev::kRmSSR;
  for (size_t i = 0; i < n; ++i) {
    const uint32_t y = ybits[i];
    if ((y & 0x7FFFFFFFu) > 0x7F800000u) { dst[i] = (uint8_t)hif8dev::nan_code(mode); continue; }
    const uint32_t r = hif8dev::hr_round_bits<0>(y, hif8dev::hr_exp_entry((y >> 23) & 0xFFu, ssr));
    dst[i] = (uint8_t)hif8dev::encode_alu<false, 0>(r & 0xFFF80000u, mode);
  }
}
// 16-bit sources, streaming form: clamped sum, then the truncating table's entry (the TA code of
// trunc_table_pattern())
void devfn_encode_bits_hr16_stream(const uint32_t* ybits, uint8_t* dst, size_t n, uint32_t mode, int srck) {
  const bool ssr = (mode & 0xF) == hif8dev::kRmSSR;
  for (size_t i = 0; i < n; ++i) {
    const uint32_t y = ybits[i];
    const hif8dev::HrExp16 p = hif8dev::hr16_exp_entry((y >> 23) & 0xFFu, ssr);
    const uint32_t lsb = srck == 1 ? hif8dev::hr16_lsb<1>(y) : hif8dev::hr16_lsb<2>(y);
    const uint32_t r = hif8dev::hr16_round_sum(y, lsb ? p.add1 : p.add0);
    dst[i] = (uint8_t)hif8dev::encode_alu<false, 0>(hif8dev::trunc_table_pattern(r >> 19), mode);
  }
}
// standard SR, streaming form: per-exponent table entry, add-and-truncate, then the TA code of the
// (representable) result
void devfn_encode_bits_sr_table(const uint32_t* ybits, uint8_t* dst, size_t n, uint32_t mode, uint64_t seed) {
  for (size_t i = 0; i < n; ++i) {
    const uint32_t y = ybits[i];
    if ((y & 0x7FFFFFFFu) > 0x7F800000u) { dst[i] = (uint8_t)hif8dev::nan_code(mode); continue; }
    const uint32_t r = hif8dev::sr_round_bits(y, hif8dev::sr_threshold(seed, (uint64_t)i), hif8dev::sr_exp_entry((y >> 23) & 0xFFu));
    dst[i] = (uint8_t)hif8dev::encode_alu<false, 0>(r & 0xFFF80000u, mode);
  }
}
void devfn_decode_bits(const uint8_t* codes, uint32_t* dst, size_t n) {
  for (size_t i = 0; i < n; ++i) dst[i] = hif8dev::decode_bits(codes[i]);
}
void devfn_narrow_bf16(const uint32_t* bits, uint16_t* dst, size_t n) {
  for (size_t i = 0; i < n; ++i) dst[i] = (uint16_t)hif8dev::narrow_bf16(bits[i]);
}
// workgroup -> tile of the expanded-operand GEMM: tile_m * tiles_n + tile_n, or 0xFFFFFFFF for a workgroup without a tile
uint32_t devfn_tile_order(uint32_t b, uint32_t tiles_m, uint32_t tiles_n) {
  uint32_t tm = 0, tn = 0;
  return hif8gemm::tile_order(b, tiles_m, tiles_n, &tm, &tn) ? tm * tiles_n + tn : 0xFFFFFFFFu;
}
uint32_t devfn_tile_order_grid(uint32_t n_tiles) { return hif8gemm::tile_order_grid(n_tiles); }
// host-side launch planning of the GEMM kernels: returns the split column, or 0 for a single launch
uint32_t devfn_ragged_round_split(size_t M, size_t N, size_t cus) {
  uint32_t split = 0;
  return hif8gemm::ragged_round_split(M, N, cus, &split) ? split : 0u;
}
}
