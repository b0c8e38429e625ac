// Device-side helpers shared by the HIP kernels of the jagged HSTU attention library (gfx950).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "hstu_geometry.h"

namespace hstu {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef int32_t i32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kWave = 64;
constexpr int kNumXcd = 8;          // MI355X: 8 accelerator dies, workgroups are dealt to them round-robin
constexpr int kXcdGroup = 4;        // consecutive schedule entries kept on one die (the scheduler writes them as runs of one head)

__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// round-to-nearest-even fp32 -> bf16 (NaN kept quiet); inputs here are finite
__device__ __forceinline__ uint16_t float_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
  typedef float v2f __attribute__((ext_vector_type(2)));
  v2f x = {lo, hi};
  v2bf y = __builtin_convertvector(x, v2bf);                 // v_cvt_pk_bf16_f32 on gfx950 (RNE)
  return __builtin_bit_cast(uint32_t, y);
}

}  // namespace hstu
