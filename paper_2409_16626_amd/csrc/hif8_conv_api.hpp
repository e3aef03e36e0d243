// Host entry points of the conversion kernels, one instantiation per source / destination
// kind (hif8dev::kSrcF32, kSrcBF16, kSrcF16).  Defined in hif8_conv.hpp and instantiated in
// hif8_conv_f32.hip, hif8_conv_bf16.hip and hif8_conv_f16.hip; called by the C ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "hif8.h"

namespace hif8conv {

// Seed of the standard-SR thresholds of one call and the index its element 0 has in the threshold stream
// (a slice of a tensor, or the second tensor of a training step, continues the stream instead of
// restarting it).
struct SrArg {
  uint64_t seed;
  uint64_t base;
};

// scale by value (d_scale2 == nullptr) or from device memory {scale, 1/scale}; sr_or_null == nullptr: the
// process-wide seed, index base 0
template <int SRCK>
hif8_status conv_encode(const void* src, uint8_t* dst, size_t n, float scale, const float* d_scale2,
                        float* d_amax_acc, uint32_t mode, const SrArg* sr_or_null, hipStream_t st);
template <int DSTK>
hif8_status conv_decode(const uint8_t* src, void* dst, size_t n, float scale, const float* d_scale2,
                        hipStream_t st);
template <int SRCK>
hif8_status conv_fake_quant(const void* src, void* dst, uint8_t* codes, size_t n, float scale,
                            const float* d_scale2, float* d_amax_acc, uint32_t mode, const SrArg* sr_or_null,
                            hipStream_t st);
template <int SRCK>
hif8_status conv_amax(const void* src, size_t n, float* d_amax, hipStream_t st);
// dst == nullptr: codes only; else the fused round trip into dst, codes optional.  parts: kMaxParts words of
// device scratch for the per-workgroup maxima.
template <int SRCK>
hif8_status conv_quantize_tensor(const void* src, void* dst, uint8_t* codes, size_t n, float target, int pow2,
                                 uint32_t mode, float* d_amax, float* d_scale2, uint32_t* parts, const SrArg* sr_or_null,
                                 hipStream_t st);
template <int SRCK>
hif8_status conv_multi_cast(const hif8_cast_item* host_items_or_null, const hif8_cast_item* d_items, size_t count,
                            uint64_t total_tiles, float* d_amax, float* d_scale2, float target, int pow2, uint32_t mode,
                            hipStream_t st);
template <int SRCK>
hif8_status conv_multi_encode_ds(const hif8_cast_item* d_items, size_t count, uint64_t total_tiles,
                                 const float* d_scale2, float* d_amax_acc, uint32_t mode, hipStream_t st);

// vector units per tile of the multi-tensor kernels (shared with hif8_multi_plan)
constexpr int kMultiBlock = 512;
constexpr int kMultiUnroll = 2;
constexpr uint32_t kMultiTileVec = kMultiBlock * kMultiUnroll;
// tiles of an item of n elements (an item shorter than one vector still owns a tile for its ragged tail)
inline uint64_t plan_item_tiles(uint64_t n, bool src_is_16bit) {
  const uint64_t nvec = src_is_16bit ? (n >> 3) : (n >> 2);
  const uint64_t t = (nvec + kMultiTileVec - 1) / kMultiTileVec;
  return (t == 0 && n != 0) ? 1 : t;
}
// most per-workgroup partial maxima conv_quantize_tensor writes (size of its scratch in 32-bit words)
constexpr uint32_t kMaxParts = 1024;

}  // namespace hif8conv
