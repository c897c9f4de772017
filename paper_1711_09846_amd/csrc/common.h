// Shared device-side helpers for the population-step kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pbt {

typedef uint16_t bf16_t;  // raw bfloat16 bits

// Round-to-nearest-even float -> bfloat16 (NaN kept quiet).
// float -> bf16, round to nearest even: the matrix-core generation has a conversion instruction
// (v_cvt_pk_bf16_f32), which the compiler emits for these casts
__device__ __forceinline__ bf16_t f2bf(float f) { return __builtin_bit_cast(bf16_t, (__bf16)f); }
// two at once: lo in bits 0..15, hi in bits 16..31
__device__ __forceinline__ uint32_t f2bf_pair(float lo, float hi) {
  typedef __attribute__((ext_vector_type(2))) float f32x2_t;
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
__device__ __forceinline__ float bf2f(bf16_t h) { return __uint_as_float(((uint32_t)h) << 16); }
// double -> bf16 with a single round-to-nearest-even: first to float with round-to-odd (truncate
// toward zero, then set the last bit if anything was lost), which the final rounding cannot mistake.
__device__ __forceinline__ bf16_t d2bf(double v) {
  float f = (float)v;
  const double back = (double)f;
  if (back != v) {
    uint32_t b = __float_as_uint(f);
    if (fabs(back) > fabs(v)) b -= 1u;  // step toward zero (f is finite and non-zero here)
    f = __uint_as_float(b | 1u);
  }
  return f2bf(f);
}

// bf16(x * s) with a single round-to-nearest-even of the exact product, in float arithmetic: hi = fl(x s) and the
// exact remainder lo = x s - hi (one fma).  Rounding hi to bf16 can only differ from rounding the exact product
// when hi sits exactly half way between two bf16 values; the sign of lo then says on which side the product lies.
// (Products so small that lo could underflow take the double route.)
__device__ __forceinline__ bf16_t bf16_times_float(bf16_t x, float s) {
  const float xf = bf2f(x);
  const float hi = xf * s;
  const uint32_t b = __float_as_uint(hi);
  if ((b & 0xffffu) != 0x8000u) return f2bf(hi);
  if ((b & 0x7f800000u) < (40u << 23)) return d2bf((double)xf * (double)s);
  const float lo = fmaf(xf, s, -hi);
  if (lo == 0.f) return f2bf(hi);                                  // a true tie: to even
  const bool away = (lo > 0.f) == (hi > 0.f);                      // the product is larger in magnitude than hi
  return (bf16_t)((b >> 16) + (away ? 1u : 0u));
}

enum { ACT_NONE = 0, ACT_RELU = 1, ACT_GELU = 2, ACT_LEAKY_RELU = 3, ACT_TANH = 4 };

// Standard normal CDF Phi(z) and density phi(z) for GELU and its derivative, from ONE exponential:
// erf(x) = 1 - (a1 t + ... + a5 t^5) exp(-x^2), t = 1/(1 + p x), x >= 0 (Abramowitz & Stegun
// 7.1.26, |error| <= 1.5e-7), with x = |z|/sqrt(2) so that exp(-x^2) = exp(-z^2/2) is also what
// phi(z) needs.  About a dozen instructions instead of a library erff call per element, which
// matters in GEMM epilogues that touch 8 million elements per layer.
__device__ __forceinline__ void normal_cdf_pdf(float z, float& cdf, float& pdf) {
  const float x = fabsf(z) * 0.70710678118654752f;
  const float t = __frcp_rn(fmaf(0.3275911f, x, 1.f));
  const float e = __expf(-x * x);
  float poly = fmaf(1.061405429f, t, -1.453152027f);
  poly = fmaf(poly, t, 1.421413741f);
  poly = fmaf(poly, t, -0.284496736f);
  poly = fmaf(poly, t, 0.254829592f);
  const float half_erfc = 0.5f * poly * t * e;          // 0.5 * erfc(|z| / sqrt 2)
  cdf = z >= 0.f ? 1.f - half_erfc : half_erfc;
  pdf = 0.39894228040143268f * e;
}

// Activation and its derivative as functions of the pre-activation z.
__device__ __forceinline__ float act_fwd(float z, int kind) {
  switch (kind) {
    case ACT_RELU: return z > 0.f ? z : 0.f;
    case ACT_GELU: { float c, p; normal_cdf_pdf(z, c, p); return z * c; }
    case ACT_LEAKY_RELU: return z > 0.f ? z : 0.2f * z;
    case ACT_TANH: return tanhf(z);
    default: return z;
  }
}
__device__ __forceinline__ float act_bwd(float z, int kind) {
  switch (kind) {
    case ACT_RELU: return z > 0.f ? 1.f : 0.f;
    case ACT_GELU: { float c, p; normal_cdf_pdf(z, c, p); return fmaf(z, p, c); }
    case ACT_LEAKY_RELU: return z > 0.f ? 1.f : 0.2f;
    case ACT_TANH: { float t = tanhf(z); return 1.f - t * t; }
    default: return 1.f;
  }
}

// The same for eight values with the choice of the activation taken once, outside the element loop (inside
// it the compiler keeps a branch ladder per element).
__device__ __forceinline__ void act_fwd8(const float* z, float* a, int kind) {
  switch (kind) {
    case ACT_RELU:
#pragma unroll
      for (int e = 0; e < 8; ++e) a[e] = z[e] > 0.f ? z[e] : 0.f;
      break;
    case ACT_GELU:
#pragma unroll
      for (int e = 0; e < 8; ++e) { float c, p; normal_cdf_pdf(z[e], c, p); a[e] = z[e] * c; }
      break;
    case ACT_LEAKY_RELU:
#pragma unroll
      for (int e = 0; e < 8; ++e) a[e] = z[e] > 0.f ? z[e] : 0.2f * z[e];
      break;
    case ACT_TANH:
#pragma unroll
      for (int e = 0; e < 8; ++e) a[e] = tanhf(z[e]);
      break;
    default:
#pragma unroll
      for (int e = 0; e < 8; ++e) a[e] = z[e];
  }
}
// d[e] = v[e] * act'(z[e])
__device__ __forceinline__ void act_bwd_scale8(const float* v, const float* z, float* d, int kind) {
  switch (kind) {
    case ACT_RELU:
#pragma unroll
      for (int e = 0; e < 8; ++e) d[e] = v[e] * (z[e] > 0.f ? 1.f : 0.f);
      break;
    case ACT_GELU:
#pragma unroll
      for (int e = 0; e < 8; ++e) { float c, p; normal_cdf_pdf(z[e], c, p); d[e] = v[e] * fmaf(z[e], p, c); }
      break;
    case ACT_LEAKY_RELU:
#pragma unroll
      for (int e = 0; e < 8; ++e) d[e] = v[e] * (z[e] > 0.f ? 1.f : 0.2f);
      break;
    case ACT_TANH:
#pragma unroll
      for (int e = 0; e < 8; ++e) { const float t = tanhf(z[e]); d[e] = v[e] * (1.f - t * t); }
      break;
    default:
#pragma unroll
      for (int e = 0; e < 8; ++e) d[e] = v[e] * 1.f;
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
