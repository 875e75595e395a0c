// Internal helpers shared by the library's translation units (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "../../include/rv.h"

#define RV_HIP_TRY(expr)                         \
  do {                                           \
    hipError_t _e = (expr);                      \
    if (_e != hipSuccess) return RV_E_DEVICE;    \
  } while (0)

#define RV_TRY(expr)                 \
  do {                               \
    rv_status _s = (expr);           \
    if (_s != RV_OK) return _s;      \
  } while (0)

static inline rv_status rv_launch_status() {
  return hipGetLastError() == hipSuccess ? RV_OK : RV_E_DEVICE;
}

// fp32 -> bf16 bits, round to nearest even (finite inputs).
__device__ __forceinline__ uint16_t rv_f32_to_bf16(float x) {
  uint32_t b = __float_as_uint(x);
  b += 0x7FFFu + ((b >> 16) & 1u);
  return (uint16_t)(b >> 16);
}
__device__ __forceinline__ float rv_bf16_to_f32(uint16_t h) {
  return __uint_as_float(((uint32_t)h) << 16);
}
// two fp32 -> packed bf16x2, round to nearest even: one v_cvt_pk_bf16_f32 on gfx950
__device__ __forceinline__ uint32_t rv_pack_bf16x2(float lo, float hi) {
  typedef __bf16 rv_bf16x2 __attribute__((ext_vector_type(2)));
  typedef float rv_f32x2 __attribute__((ext_vector_type(2)));
  const rv_f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, rv_bf16x2));
}

// Sum of v over the 32 lanes of each half wave, left in every lane of the half, in a fixed
// butterfly order: four steps inside a row of 16 lanes as DPP operands of the additions
// themselves (quad swaps, then the two mirrors - after each step every lane of the group holds
// the group's sum), one cross-row exchange at the end.
template <int CTRL>
__device__ __forceinline__ float rv_dpp_add(float v) {
  return v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}
__device__ __forceinline__ float rv_half_wave_sum(float v) {
  v = rv_dpp_add<0xB1>(v);    // quad_perm [1,0,3,2]
  v = rv_dpp_add<0x4E>(v);    // quad_perm [2,3,0,1]
  v = rv_dpp_add<0x141>(v);   // row_half_mirror: the other quad of each 8
  v = rv_dpp_add<0x140>(v);   // row_mirror: the other 8 of each 16
  return v + __shfl_xor(v, 16, 64);
}
