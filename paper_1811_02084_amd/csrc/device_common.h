// Small device/host helpers shared by the HIP translation units (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

#include "mtf_internal.h"

namespace mtf {

typedef uint16_t bf16_t;  // raw bfloat16 bits in memory

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float((uint32_t)v << 16); }

// Round-to-nearest-even; NaN stays NaN (hardware conversion).
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  return __builtin_bit_cast(bf16_t, (__bf16)f);
}

// Two floats -> packed bf16 pair with the hardware converter (v_cvt_pk_bf16_f32: round to
// nearest even, NaN stays NaN), lo in bits 0..15.
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  typedef __attribute__((ext_vector_type(2))) float f32x2_t;
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

inline int hip_fail(hipError_t e, const char* what) {
  return fail(MTF_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

// Checks the launch that was just issued.
inline int launch_status(const char* kernel) {
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? MTF_OK : hip_fail(e, kernel);
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

}  // namespace mtf
