// Training-side scale state of the HiF8 method (arXiv 2409.16626, Sec. 5.1):
//   per-tensor scaling (PTS)      device-resident {scale, 1/scale} pairs for a list of GEMM input
//                                 tensors, refreshed from amax accumulators every `interval`
//                                 iterations by one small kernel (no host round trip);
//   adaptive loss scaling (ALS)   host state machine: dynamic loss scale whose growth window moves
//                                 along {1, 20, 50, 100, 200, 500, 1000}.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>

#include "hif8.h"
#include "hif8_host.hpp"

using namespace hif8host;

// scale = largest power of two with amax * scale <= target; a degenerate amax (0, Inf, NaN)
// keeps the previous pair.  The accumulator is cleared for the next window.
__global__ void k_pts_update(float* __restrict__ d_amax, float* __restrict__ d_scale2, uint32_t count,
                             float target) {
  const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= count) return;
  const uint32_t ab = __float_as_uint(d_amax[i]);
  d_amax[i] = 0.0f;
  if (ab == 0u || ab >= 0x7F800000u) return;
  const float q = target / __uint_as_float(ab);  // correctly rounded divide: floor(log2) is that of the exact quotient
  uint32_t qb = __float_as_uint(q);
  if (qb >= 0x7F800000u) qb = 0x7F000000u;       // quotient overflowed: largest power of two, 2^127
  uint32_t sb = qb & 0x7F800000u;
  if (sb == 0u) sb = 1u << 23;                    // subnormal quotient: smallest normal power of two
  if (sb > (253u << 23)) sb = 253u << 23;         // keep 1/scale normal as well (2^126 at most)
  const float s = __uint_as_float(sb);
  d_scale2[2 * i] = s;
  d_scale2[2 * i + 1] = 1.0f / s;
}

__global__ void k_pts_reset(float* __restrict__ d_amax, float* __restrict__ d_scale2, uint32_t count) {
  const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= count) return;
  d_amax[i] = 0.0f;
  d_scale2[2 * i] = 1.0f;
  d_scale2[2 * i + 1] = 1.0f;
}

namespace {
constexpr int kAlsWindows[7] = {1, 20, 50, 100, 200, 500, 1000};
constexpr float kAlsMinScale = 1.0f;
constexpr float kAlsMaxScale = 8.507059173023462e37f;  // 2^126
}  // namespace

extern "C" {

hif8_status hif8_pts_init(hif8_pts_state* st, float* d_amax, float* d_scale2, size_t count,
                          uint32_t interval, float target, hif8_stream_t stream) {
  if (!st || ((!d_amax || !d_scale2) && count != 0)) return HIF8_ERR_NULL;
  if (interval == 0 || count > 0x7FFFFFFFu || !(target > 0.0f) || std::isinf(target)) return HIF8_ERR_ARG;
  int ex = 0;
  if (std::frexp(target, &ex) != 0.5f) return HIF8_ERR_ARG;  // power of two: the floor below is then exact
  st->d_amax = d_amax;
  st->d_scale2 = d_scale2;
  st->count = (uint32_t)count;
  st->interval = interval;
  st->target = target;
  st->iteration = 0;
  if (count == 0) return HIF8_OK;
  hipLaunchKernelGGL(k_pts_reset, dim3(((uint32_t)count + 255) / 256), dim3(256), 0, (hipStream_t)stream,
                     d_amax, d_scale2, (uint32_t)count);
  return finish_launch();
}

int hif8_pts_collects(const hif8_pts_state* st) {
  return (st && st->interval != 0 && st->iteration % st->interval == 0) ? 1 : 0;
}

hif8_status hif8_pts_end_iteration(hif8_pts_state* st, hif8_stream_t stream) {
  if (!st) return HIF8_ERR_NULL;
  if (st->interval == 0) return HIF8_ERR_ARG;
  hif8_status rc = HIF8_OK;
  if (st->iteration % st->interval == 0 && st->count != 0) {
    hipLaunchKernelGGL(k_pts_update, dim3((st->count + 255) / 256), dim3(256), 0, (hipStream_t)stream,
                       st->d_amax, st->d_scale2, st->count, st->target);
    rc = finish_launch();
  }
  st->iteration += 1;
  return rc;
}

void hif8_als_init(hif8_als_state* st) {
  if (!st) return;
  st->scale = 4294967296.0f;  // 2^32
  st->window_index = 1;       // window 20
  st->good_steps = 0;
  st->increases = 0;
  st->decrease_streak = 0;
}

int hif8_als_window(const hif8_als_state* st) {
  if (!st || st->window_index < 0 || st->window_index > 6) return -1;
  return kAlsWindows[st->window_index];
}

hif8_status hif8_als_update(hif8_als_state* st, int found_overflow) {
  if (!st) return HIF8_ERR_NULL;
  if (st->window_index < 0 || st->window_index > 6) return HIF8_ERR_ARG;
  if (found_overflow) {
    const float h = st->scale * 0.5f;
    st->scale = h < kAlsMinScale ? kAlsMinScale : h;
    st->good_steps = 0;
    if (++st->decrease_streak == 3) {
      if (st->window_index > 0) --st->window_index;
      st->decrease_streak = 0;
      st->increases = 0;
    }
  } else if (++st->good_steps >= kAlsWindows[st->window_index]) {
    const float d = st->scale * 2.0f;
    st->scale = d > kAlsMaxScale ? kAlsMaxScale : d;
    st->good_steps = 0;
    st->decrease_streak = 0;
    if (++st->increases == 3) {
      if (st->window_index < 6) ++st->window_index;
      st->increases = 0;
    }
  }
  return HIF8_OK;
}

}  // extern "C"
