// Small device/host helpers shared by the HIP translation units (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

#include "mtf_internal.h"

namespace mtf {

typedef uint16_t bf16_t;  // raw bfloat16 bits in memory

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float((uint32_t)v << 16); }

// Round-to-nearest-even; NaN stays NaN.
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16);
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
