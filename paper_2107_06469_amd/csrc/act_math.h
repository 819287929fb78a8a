// Activation functions and their derivatives as the GEMM epilogues apply them; shared by every kernel that applies
// one, so that all of them compute the same values.
#pragma once
#include <hip/hip_runtime.h>

#include "kernels.h"

namespace hydra {

// Normal CDF and density for GeLU.  erf by the rational approximation of Abramowitz & Stegun 7.1.26
// (|error| <= 1.5e-7, below fp32 rounding of the surrounding arithmetic): a dozen VALU operations per
// element instead of a library erf, which matters because the epilogue applies it to every output.
__device__ __forceinline__ void normal_cdf_pdf(float z, float& cdf, float& pdf) {
  const float x = fabsf(z) * 0.70710678118654752f;
  const float t = __builtin_amdgcn_rcpf(1.0f + 0.3275911f * x);
  const float e = __expf(-x * x);  // = exp(-z^2/2)
  const float poly = t * (0.254829592f + t * (-0.284496736f + t * (1.421413741f + t * (-1.453152027f + t * 1.061405429f))));
  const float erf_abs = 1.0f - poly * e;
  cdf = 0.5f * (1.0f + (z < 0.f ? -erf_abs : erf_abs));
  pdf = e * 0.39894228040143268f;
}
__device__ __forceinline__ float act_fwd(float v, int act) {
  if (act == EPI_ACT_RELU) return v > 0.f ? v : 0.f;
  if (act == EPI_ACT_GELU) {
    float cdf, pdf;
    normal_cdf_pdf(v, cdf, pdf);
    return v * cdf;
  }
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
