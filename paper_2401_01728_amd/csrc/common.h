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
