// Launch planning of the HiF8 GEMM kernels: which launches cover a problem, and which tile a workgroup takes
// (plain C++, no HIP types; `__host__ __device__` are the only annotations, defined away in host-only builds).
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

// Workgroup -> tile of the expanded-operand kernel.  The hardware deals consecutive workgroups round-robin over the
// kXcds accelerator dies (XCDs), each with its own L2.  Workgroup b therefore takes tile number
// (b % kXcds) * per_xcd + b / kXcds of a tile order that walks groups of kGroupM tile rows column by column: the
// workgroups resident on one die at a time then cover a compact kGroupM x (a few) block of tiles and share their
// operand panels in that die's L2, whatever tiles_n is.  The launch has tile_order_grid() workgroups; returns false
// for the few at the end of the last die's share that have no tile.
constexpr uint32_t kXcds = 8;    // accelerator dies, each with an L2 of its own
constexpr uint32_t kGroupM = 8;  // tile rows per group of the tile order
__host__ __device__ inline uint32_t tile_order_grid(uint32_t n_tiles) { return (n_tiles + kXcds - 1u) / kXcds * kXcds; }
__host__ __device__ inline bool tile_order(uint32_t b, uint32_t tiles_m, uint32_t tiles_n, uint32_t* tile_m, uint32_t* tile_n) {
  const uint32_t n_tiles = tiles_m * tiles_n, per_xcd = (n_tiles + kXcds - 1u) / kXcds;
  const uint32_t t = (b % kXcds) * per_xcd + b / kXcds;
  if (t >= n_tiles) return false;
  const uint32_t grp = t / (kGroupM * tiles_n), first_m = grp * kGroupM;
  const uint32_t grp_rows = tiles_m - first_m < kGroupM ? tiles_m - first_m : kGroupM;
  const uint32_t in_grp = t - grp * (kGroupM * tiles_n);
  *tile_n = in_grp / grp_rows;
  *tile_m = first_m + (in_grp - *tile_n * grp_rows);
  return true;
}

}  // namespace hif8gemm
