// Shared device-side helpers for the population-step kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pbt {

typedef uint16_t bf16_t;  // raw bfloat16 bits

// Round-to-nearest-even float -> bfloat16 (NaN kept quiet).
__device__ __forceinline__ bf16_t f2bf(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}
__device__ __forceinline__ float bf2f(bf16_t h) { return __uint_as_float(((uint32_t)h) << 16); }

enum { ACT_NONE = 0, ACT_RELU = 1, ACT_GELU = 2, ACT_LEAKY_RELU = 3, ACT_TANH = 4 };

// Activation and its derivative as functions of the pre-activation z.
__device__ __forceinline__ float act_fwd(float z, int kind) {
  switch (kind) {
    case ACT_RELU: return z > 0.f ? z : 0.f;
    case ACT_GELU: return 0.5f * z * (1.f + erff(z * 0.70710678118654752f));
    case ACT_LEAKY_RELU: return z > 0.f ? z : 0.2f * z;
    case ACT_TANH: return tanhf(z);
    default: return z;
  }
}
__device__ __forceinline__ float act_bwd(float z, int kind) {
  switch (kind) {
    case ACT_RELU: return z > 0.f ? 1.f : 0.f;
    case ACT_GELU:
      return 0.5f * (1.f + erff(z * 0.70710678118654752f)) + z * 0.39894228040143268f * __expf(-0.5f * z * z);
    case ACT_LEAKY_RELU: return z > 0.f ? 1.f : 0.2f;
    case ACT_TANH: { float t = tanhf(z); return 1.f - t * t; }
    default: return 1.f;
  }
}

// Sum over the 64 lanes of a wavefront; every lane receives the total.  The
// butterfly order is fixed, so the result does not depend on scheduling.
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
  return v;
}

}  // namespace pbt
