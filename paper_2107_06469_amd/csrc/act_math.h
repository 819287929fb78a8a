// Activation functions and their derivatives as the GEMM epilogues apply them; shared by every kernel that applies
// one, so that all of them compute the same values.
#pragma once
#include <hip/hip_runtime.h>

#include "kernels.h"

namespace hydra {

// Normal CDF and density for GeLU's derivative (and wherever both are needed).  erf by the rational approximation of
// Abramowitz & Stegun 7.1.26 (|error| <= 1.5e-7, below fp32 rounding of the surrounding arithmetic): a dozen VALU
// operations, a reciprocal and an exponential per element instead of a library erf, which matters because the
// epilogue applies it to every output.
__device__ __forceinline__ void normal_cdf_pdf(float z, float& cdf, float& pdf) {
  const float x = fabsf(z) * 0.70710678118654752f;
  const float t = __builtin_amdgcn_rcpf(1.0f + 0.3275911f * x);
  const float e = __expf(-x * x);  // = exp(-z^2/2)
  const float poly = t * (0.254829592f + t * (-0.284496736f + t * (1.421413741f + t * (-1.453152027f + t * 1.061405429f))));
  const float erf_abs = 1.0f - poly * e;
  cdf = 0.5f * (1.0f + (z < 0.f ? -erf_abs : erf_abs));
  pdf = e * 0.39894228040143268f;
}
// GeLU(z) = z Phi(z) where only the value is needed (forward epilogues apply it to every output, and the workgroup's
// MFMAs wait meanwhile): Phi(-a) = 2^(a Q(a) - 1) on a = min(|z|, 6) with Q of degree 6, fitted to the normal CDF for
// the smallest maximal absolute error of Phi (4e-8; 8e-8 as evaluated in fp32), and z Phi(z) = max(z, 0) - a Phi(-a).
// One exponential and no reciprocal: 16 VALU issue slots per element with the bias and the two conversions of the
// epilogue around it, against 23 through normal_cdf_pdf; the error of z Phi(z) in fp32 is 3.8e-7 at most (the other
// form: 4.7e-7).  Past |z| = 6 Phi(-6) = 1e-9 stands for the smaller true value.
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
__device__ __forceinline__ float act_grad(float z, int act) {
  if (act == EPI_ACT_RELU) return z > 0.f ? 1.f : 0.f;
  if (act == EPI_ACT_GELU) {
    float cdf, pdf;
    normal_cdf_pdf(z, cdf, pdf);
    return cdf + z * pdf;
  }
  return 1.f;
}

}  // namespace hydra
