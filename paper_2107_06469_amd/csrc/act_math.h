// Activation functions and their derivatives as the GEMM epilogues apply them; shared by every kernel that applies
// one, so that all of them compute the same values.
#pragma once
#include <hip/hip_runtime.h>

#include "kernels.h"

namespace hydra {

// GeLU(z) = z Phi(z) where only the value is needed (forward epilogues apply it to every output, and the workgroup's
// MFMAs wait meanwhile): Phi(-a) = 2^(a Q(a) - 1) on a = min(|z|, 6) with Q of degree 6, fitted to the normal CDF for
// the smallest maximal absolute error of Phi (4e-8; 8e-8 as evaluated in fp32), and z Phi(z) = max(z, 0) - a Phi(-a).
// One exponential and no reciprocal: 13 instructions per element with the bias and the two conversions of the
// epilogue around it, against 17 with the rational erf below; the error of z Phi(z) in fp32 is 3.8e-7 at most (with
// the rational erf: 4.7e-7).  Past |z| = 6 Phi(-6) = 1e-9 stands for the smaller true value.
__device__ __forceinline__ float gelu_fwd(float z) {
  const float a = fminf(fabsf(z), 6.0f);
  float q = 8.60450347e-06f;
  q = __fmaf_rn(q, a, -5.54861494e-05f);
  q = __fmaf_rn(q, a, -0.000414218041f);
  q = __fmaf_rn(q, a, 0.00737433818f);
  q = __fmaf_rn(q, a, -0.0526751051f);
  q = __fmaf_rn(q, a, -0.459161409f);
  q = __fmaf_rn(q, a, -1.15110918f);
  const float w = __builtin_amdgcn_exp2f(__fmaf_rn(a, q, -1.0f));
  return __fmaf_rn(-a, w, fmaxf(z, 0.f));
}
__device__ __forceinline__ float act_fwd(float v, int act) {
  if (act == EPI_ACT_RELU) return v > 0.f ? v : 0.f;
  if (act == EPI_ACT_GELU) return gelu_fwd(v);
  return v;
}
// GeLU'(z) = Phi(z) + z phi(z) for the gate epilogues (which apply it to every output).  erf by the rational
// approximation of Abramowitz & Stegun 7.1.26 (|error| <= 1.5e-7, below fp32 rounding of the surrounding arithmetic):
// erfc(x) = t (a1 + t (a2 + ...)) exp(-x^2), t = 1 / (1 + p x).  With x = |z| / sqrt(2) the exponential is the
// density's as well; the 1/sqrt(2) is folded into p and the 1/2 of the CDF into the a's, so that
// Phi(-|z|) = e t (a1/2 + t (a2/2 + ...)), e = exp(-z^2/2): 16 instructions.
__device__ __forceinline__ float gelu_grad(float z) {
  const float a = fabsf(z);
  const float t = __builtin_amdgcn_rcpf(__fmaf_rn(0.3275911f * 0.70710678118654752f, a, 1.0f));
  const float e = __builtin_amdgcn_exp2f((z * z) * (-0.5f * 1.4426950408889634f));  // exp(-z^2/2)
  float p = 0.5f * 1.061405429f;
  p = __fmaf_rn(p, t, 0.5f * -1.453152027f);
  p = __fmaf_rn(p, t, 0.5f * 1.421413741f);
  p = __fmaf_rn(p, t, 0.5f * -0.284496736f);
  p = __fmaf_rn(p, t, 0.5f * 0.254829592f);
  const float h = (p * t) * e;                  // Phi(-|z|)
  const float cdf = z > 0.f ? 1.0f - h : h;
  return __fmaf_rn(z * e, 0.39894228040143268f, cdf);
}
__device__ __forceinline__ float act_grad(float z, int act) {
  if (act == EPI_ACT_RELU) return z > 0.f ? 1.f : 0.f;
  if (act == EPI_ACT_GELU) return gelu_grad(z);
  return 1.f;
}

}  // namespace hydra
