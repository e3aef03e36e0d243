// Host-side plumbing shared by the translation units of libhif8: error capture, per-device
// initialisation, launch shapes and argument checks.  Defined in hif8_lib.hip.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <type_traits>

#include "hif8.h"
#include "hif8_stream.hpp"

namespace hif8host {

// Read-only lookup tables in static device memory of one device (addresses of that device's
// copy, resolved once by ensure_init()).
struct DevTables {
  // [NaN -> 0 option 0/1][sat 0/1][kind 0/1][8192] bytes.  kind 0: TA code of pattern (i << 19); kind 1: TE
  // code of the same pattern (used only when the low 19 bits of the converted pattern are all zero).
  const uint8_t* enc_lut;
  const uint8_t* hr16_lut;
  const uint16_t* val_lut;  // layout of enc_lut, values instead of codes
  const uint32_t* dec_lut;  // [256] code -> binary32 pattern
};

// Launch shape of one kernel family.  tiles_per_wg == 0 selects the persistent grid.
struct Shape {
  int block;
  int unroll;
  int tiles_per_wg;
  int wg_per_cu;
};
enum Family { FAM_ENC32_TA, FAM_ENC32_HR, FAM_ENC16, FAM_FQ, FAM_DEC, FAM_AMAX, FAM_DIAG, FAM_CALIB, FAM_AMAX_PARTS, FAM_MULTI_STAGE, FAM_COUNT };

Shape shape_for(Family f);
int tune_ta_impl();   // 0 = table, 1 = ALU
int tune_amax_nt();   // 1 = non-temporal loads in amax, 0 = cached loads, -1 = by tensor size
uint64_t multi_group_bytes();  // source bytes per group of the group-wise multi-tensor cast
bool multi_stage_overlap();  // true: one launch gathers the amax of a group and casts the previous one
uint64_t sr_seed();   // seed of the standard-SR threshold generator in effect now

bool hip_ok(hipError_t e);  // records a failure for hif8_last_hip_error()
hif8_status finish_launch();
hif8_status ensure_init(int* cu_count_out, DevTables* tables_out);

inline bool aligned_to(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
bool valid_mode(uint32_t mode);
bool valid_scale(float scale, float* inv_out);  // scale and fl32(1/scale) both finite and positive

// grid size and tile walk for nvec vector units under a launch shape; max_grid != 0 caps the number of
// workgroups (a one-shot grid then gives every workgroup more consecutive tiles)
unsigned grid_for(size_t nvec, int cus, const Shape& sh, hif8dev::Walk* walk, unsigned max_grid = 0);
unsigned grid_elem(size_t n, int cus);

// small utility launches shared by the translation units
hif8_status launch_fill_u32(uint32_t* p, uint32_t v, uint32_t count, hipStream_t st);
// per item i < count: d_scale2[2i] = scale from d_amax[i], d_scale2[2i+1] = fl32(1/scale)
hif8_status launch_scale_from_amax(const float* d_amax, float* d_scale2, uint32_t count, float target,
                                   int pow2, hipStream_t st);

}  // namespace hif8host

namespace hif8host {
// Calls f(std::integral_constant<int, U>) for the unroll factor chosen at run time.
template <typename F>
inline void dispatch_unroll(int unroll, F&& f) {
  switch (unroll) {
    case 1: f(std::integral_constant<int, 1>{}); break;
    case 2: f(std::integral_constant<int, 2>{}); break;
    case 8: f(std::integral_constant<int, 8>{}); break;
    default: f(std::integral_constant<int, 4>{}); break;
  }
}
}  // namespace hif8host
