// GeLU of the recurrent block's second branch (Section 2.3): z * Phi(z) with Phi the standard
// normal CDF, or the tanh form 0.5 z (1 + tanh(sqrt(2/pi) (z + 0.044715 z^3))) = z * sigmoid(2k).
// FAST = false: accurate library functions (fp32 storage); FAST = true: hardware exp2 and
// reciprocal, enough for results that are rounded to bf16.
#pragma once
#include <hip/hip_runtime.h>

namespace rglru {

constexpr float GELU_C0 = 0.7978845608028654f;   // sqrt(2 / pi)
constexpr float GELU_C1 = 0.044715f;
constexpr float INV_SQRT2 = 0.7071067811865476f;
constexpr float INV_SQRT_2PI = 0.3989422804014327f;

// Phi(z) for the fast path, branch-free: the rational approximation of erfc (Abramowitz and
// Stegun 7.1.26, absolute error below 1.5e-7) evaluated on |z|, which also keeps the negative
// tail free of cancellation. `e` returns exp(-z^2 / 2).
__device__ __forceinline__ float normal_cdf_fast(float z, float &e) {
  const float az = fabsf(z) * INV_SQRT2;
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, az, 1.f));
  float pl = fmaf(1.061405429f, t, -1.453152027f);
  pl = fmaf(pl, t, 1.421413741f);
  pl = fmaf(pl, t, -0.284496736f);
  pl = fmaf(pl, t, 0.254829592f);
  e = __builtin_amdgcn_exp2f(-0.5f * 1.4426950408889634f * z * z);
  const float q = 0.5f * pl * t * e;     // Phi(-|z|)
  return z < 0.f ? q : 1.f - q;
}

template <bool TANH, bool FAST>
__device__ __forceinline__ float gelu(float z) {
  if (TANH) {
    const float k2 = 2.f * GELU_C0 * (z + GELU_C1 * z * z * z);
    if (FAST) return z * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-1.4426950408889634f * k2));
    return z / (1.f + expf(-k2));
  }
  // erfc keeps its relative accuracy in the negative tail, where 1 + erf cancels
  if (FAST) {
    float e;
    return z * normal_cdf_fast(z, e);
  }
  return 0.5f * z * erfcf(-z * INV_SQRT2);
}

// value and derivative together
template <bool TANH, bool FAST>
__device__ __forceinline__ void gelu_and_grad(float z, float &val, float &grad) {
  if (TANH) {
    const float k2 = 2.f * GELU_C0 * (z + GELU_C1 * z * z * z);
    const float s = FAST ? __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-1.4426950408889634f * k2))
                         : 1.f / (1.f + expf(-k2));
    val = z * s;
    // d/dz [z s(2k)] = s + z s (1 - s) 2 k', 2 k' = 2 c0 (1 + 3 c1 z^2)
    grad = s + z * s * (1.f - s) * (2.f * GELU_C0) * (1.f + 3.f * GELU_C1 * z * z);
    return;
  }
  float phi, e;
  if (FAST) {
    phi = normal_cdf_fast(z, e);
  } else {
    phi = 0.5f * erfcf(-z * INV_SQRT2);
    e = expf(-0.5f * z * z);
  }
  val = z * phi;
  grad = phi + z * INV_SQRT_2PI * e;
}

}  // namespace rglru
