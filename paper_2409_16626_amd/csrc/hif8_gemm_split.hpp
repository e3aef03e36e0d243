// Host-side launch planning of the HiF8 GEMM kernels (plain C++, no HIP types).
#pragma once

#include <stddef.h>
#include <stdint.h>

namespace hif8gemm {

// A ragged last round of 256 x 256 tiles leaves most compute units idle for a whole tile time.  When that
// round would be at most half full, the large tiles get as many whole tile columns as fill complete rounds
// (columns [0, *split)) and the remaining columns go to 128 x 128 tiles -- a quarter of the work each, two
// workgroups per compute unit, one round -- in a second launch.  Returns false where one launch is better.
inline bool ragged_round_split(size_t M, size_t N, size_t cus, uint32_t* split) {
  const size_t tm = (M + 255) / 256, tn = (N + 255) / 256, tiles = tm * tn;
  if (cus == 0 || tiles <= cus || tiles % cus == 0) return false;
  const size_t cols_big = tiles / cus * cus / tm;  // whole tile columns within the complete rounds
  if (cols_big < 1 || cols_big >= tn || (tn - cols_big) * tm * 2 > cus) return false;
  *split = (uint32_t)(cols_big * 256);
  return true;
}

}  // namespace hif8gemm
