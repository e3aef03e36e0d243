/*
 * hif8_diag.h -- benchmarking and profiling surface of libhif8.  Nothing here is part of the
 * method (arXiv 2409.16626): the calls in hif8.h compute the same results whatever these knobs say.
 * For the bench harness and the tests that sweep launch shapes; not thread-safe (set the knobs
 * before other threads call into the library).
 */
#ifndef HIF8_DIAG_H_
#define HIF8_DIAG_H_

#include "hif8.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Launch-shape tuning knobs (process-wide).  The first, second, third, fifth and sixth default
 * to -1 = "use the built-in choice of each kernel family".
 *   HIF8_TUNE_BLOCK        threads per workgroup of the streaming kernels (64..1024, multiple of 64)
 *   HIF8_TUNE_WG_PER_CU    persistent mode: workgroups launched per compute unit (1..64)
 *   HIF8_TUNE_UNROLL       16-byte loads in flight per lane (1, 2, 4 or 8); a tile is
 *                          block * unroll lanes' worth of data
 *   HIF8_TUNE_TA_IMPL      0 = TA encode through the LDS lookup table, 1 = TA encode in ALU only
 *                          (the integer encoder the table is built from; about half the speed)
 *   HIF8_TUNE_TILES_PER_WG 0 = persistent grid (grid-stride over tiles); k >= 1 = one-shot grid in
 *                          which every workgroup handles k consecutive tiles (0..4096)
 *   HIF8_TUNE_AMAX_NT      1 = hif8_amax_* reads with non-temporal loads, 0 = ordinary (cached)
 *                          loads, -1 (default) = ordinary loads for tensors up to 192 MiB (a cast of
 *                          the same tensor usually follows and then finds it in the last-level
 *                          cache), non-temporal loads above
 *   HIF8_TUNE_GROUP_MIB    source MiB per group of the group-wise hif8_multi_cast_* (1..4096, default 192)
 *   HIF8_TUNE_FAMILY       kernel family the four shape knobs (block, workgroups per CU, unroll, tiles
 *                          per workgroup) apply to; -1 (default) = all.  0 = FP32 encode TA, 1 = FP32
 *                          encode HR, 2 = 16-bit encode, 3 = fake-quant, 4 = decode, 5 = amax,
 *                          6 = diagnostic stream, 7 = calibration sweeps, 8 = first pass of
 *                          hif8_quantize_tensor_*, 9 = group-wise hif8_multi_cast_* (only the workgroups
 *                          per CU apply: amax workgroups of a stage)
 *   HIF8_TUNE_STAGE_OVERLAP  group-wise hif8_multi_cast_*: 1 (default) = one launch casts a group and gathers
 *                          the amax of the next one, 0 = two launches, one after the other
 * Returns HIF8_ERR_ARG for an unknown key or a value outside the stated range.
 */
enum {
  HIF8_TUNE_BLOCK = 0,
  HIF8_TUNE_WG_PER_CU = 1,
  HIF8_TUNE_UNROLL = 2,
  HIF8_TUNE_TA_IMPL = 3,
  HIF8_TUNE_TILES_PER_WG = 4,
  HIF8_TUNE_AMAX_NT = 5,
  HIF8_TUNE_GROUP_MIB = 6,
  HIF8_TUNE_FAMILY = 7,
  HIF8_TUNE_STAGE_OVERLAP = 8
};
hif8_status hif8_set_tuning(int key, int value);
int hif8_get_tuning(int key); /* -1 for an unknown key */

/*
 * Tile shape of the simulated HiF8 GEMMs, for benchmarking (default 0 = chosen by problem size).
 *   code-operand kernel (hif8_gemm_*):         5 = 256 x 256 x 32 workgroup tile, 8 wavefronts as 4 x 2 (the
 *                                              choice when there is such a tile for every compute unit);
 *                                              6 = 128 x 128 x 32, 4 wavefronts, two workgroups per CU
 *   expanded-operand kernel (hif8_gemm_expanded_*): 9 = 128 x 128 x 64, 4 wavefronts (the choice below one large
 *                                              tile per compute unit); 10 = 256 x 256 x 64, 4 wavefronts as 2 x 2,
 *                                              memory instructions placed one by one between the MFMAs (the choice
 *                                              from two rounds of tiles on); 11 = the same placement with 8
 *                                              wavefronts as 2 x 4 (the choice for a single round)
 * 0 resets both choices.  Other values: HIF8_ERR_ARG.
 */
hif8_status hif8_gemm_set_variant(int variant);

/*
 * Diagnostic stream kernel with the same read:write mix as a conversion
 * (read in_bytes_per_lane = 16 per lane, write out_bytes_per_lane in {0, 4, 8, 16}; 0 = read only),
 * launched with the shape the tuning knobs select: a same-mix copy for comparison with the
 * conversion kernels.  Copies the low bytes of each 16-byte group: dst group g = first out_bytes
 * of src group g.  n_groups 16-byte groups are read.  src 16-byte aligned, dst aligned to
 * out_bytes (dst may be NULL for out_bytes = 0).
 */
hif8_status hif8_diag_stream(const void* src, void* dst, size_t n_groups, int out_bytes_per_lane,
                             hif8_stream_t stream);

#ifdef __cplusplus
}
#endif
#endif /* HIF8_DIAG_H_ */
