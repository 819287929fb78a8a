// Per-model parameter update over a shard's flat parameter block (paper, Approach, "Desiderata":
// the gradient update of every model must be exactly the one unsharded training applies).
//   SGD:  p <- p - lr g
//   Adam: m <- b1 m + (1-b1) g;  v <- b2 v + (1-b2) g^2;
//         p <- p - lr * (m * bc1) / (sqrt(v * bc2) + eps),  bc1 = 1/(1-b1^t), bc2 = 1/(1-b2^t)
// and, for bf16 models, the working copy w16 <- bf16(p).
// The kernel is a pure stream over HBM: 16 B/elem read + 4 written (SGD); 16 read + 12 written (+2 for
// the bf16 copy) for Adam.  Each lane moves 16-byte vectors; G models share a grid (blockIdx.y), each
// with its own hyper-parameters.
#include "kernels.h"

namespace hydra {
namespace {

__device__ __forceinline__ bf16_t f2bf(float v) {
  __bf16 h = (__bf16)v;
  return __builtin_bit_cast(bf16_t, h);
}

template <int OPT, bool W16>
__global__ __launch_bounds__(256) void optim_kernel(const OptimArgs a) {
  const int g = blockIdx.y;
  const size_t n4 = a.n >> 2;
  float4* __restrict__ p = reinterpret_cast<float4*>(a.p[g]);
  const float4* __restrict__ gr = reinterpret_cast<const float4*>(a.g[g]);
  float4* __restrict__ m = reinterpret_cast<float4*>(a.m[g]);
  float4* __restrict__ v = reinterpret_cast<float4*>(a.v[g]);
  uint2* __restrict__ w16 = reinterpret_cast<uint2*>(a.w16[g]);
  const float lr = a.lr[g], b1 = a.b1[g], b2 = a.b2[g], eps = a.eps[g], bc1 = a.bc1[g], bc2 = a.bc2[g];
  const float c1 = a.c1[g], c2 = a.c2[g];
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += stride) {
    float4 pv = p[i];
    const float4 gv = gr[i];
    float pe[4] = {pv.x, pv.y, pv.z, pv.w};
    const float ge[4] = {gv.x, gv.y, gv.z, gv.w};
    if (OPT == 0) {
#pragma unroll
      for (int e = 0; e < 4; ++e) pe[e] = pe[e] - lr * ge[e];
    } else {
      float4 mv = m[i], vv = v[i];
      float me[4] = {mv.x, mv.y, mv.z, mv.w}, ve[4] = {vv.x, vv.y, vv.z, vv.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        me[e] = b1 * me[e] + c1 * ge[e];
        ve[e] = b2 * ve[e] + c2 * ge[e] * ge[e];
        pe[e] = pe[e] - lr * (me[e] * bc1) / (sqrtf(ve[e] * bc2) + eps);
      }
      m[i] = make_float4(me[0], me[1], me[2], me[3]);
      v[i] = make_float4(ve[0], ve[1], ve[2], ve[3]);
    }
    p[i] = make_float4(pe[0], pe[1], pe[2], pe[3]);
    if (W16)
      w16[i] = make_uint2((uint32_t)f2bf(pe[0]) | ((uint32_t)f2bf(pe[1]) << 16),
                          (uint32_t)f2bf(pe[2]) | ((uint32_t)f2bf(pe[3]) << 16));
  }
}

}  // namespace

hipError_t launch_optim(const OptimArgs& a, hipStream_t s) {
  if (a.G < 1 || a.G > MAXG || (a.n & 3)) return hipErrorInvalidValue;
  if (a.n == 0) return hipSuccess;
  const bool w16 = a.w16[0] != nullptr;
  for (int g = 0; g < a.G; ++g) {
    if (!a.p[g] || !a.g[g] || (w16 != (a.w16[g] != nullptr))) return hipErrorInvalidValue;
    if (a.opt == 1 && (!a.m[g] || !a.v[g])) return hipErrorInvalidValue;
  }
  size_t n4 = a.n >> 2;
  size_t bx = (n4 + 255) / 256;
  // at most 8 vectors per lane per grid pass keeps the grid large enough to fill 256 CUs
  size_t cap = (bx + 7) / 8;
  if (cap < 1) cap = 1;
  if (cap > 65535) cap = 65535;
  dim3 grid((unsigned)cap, a.G);
  if (a.opt == 0) {
    if (w16) hipLaunchKernelGGL((optim_kernel<0, true>), grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL((optim_kernel<0, false>), grid, dim3(256), 0, s, a);
  } else {
    if (w16) hipLaunchKernelGGL((optim_kernel<1, true>), grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL((optim_kernel<1, false>), grid, dim3(256), 0, s, a);
  }
  return hipGetLastError();
}

}  // namespace hydra
