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
#include "optim_math.h"

namespace hydra {
namespace {

__device__ __forceinline__ bf16_t f2bf(float v) {
  __bf16 h = (__bf16)v;
  return __builtin_bit_cast(bf16_t, h);
}

// one 16-byte vector of each state array
template <int OPT, bool W16>
__device__ __forceinline__ void update4(const OptimArgs& a, int g, size_t i, const OptimHp& h) {
  // every array is read once and written once per launch: streaming (non-temporal) accesses
  typedef __attribute__((ext_vector_type(4))) float f32x4;
  f32x4* __restrict__ p = reinterpret_cast<f32x4*>(a.p[g]);
  const f32x4* __restrict__ gr = reinterpret_cast<const f32x4*>(a.g[g]);
  const f32x4 pv = __builtin_nontemporal_load(p + i);
  const f32x4 gv = __builtin_nontemporal_load(gr + i);
  float pe[4] = {pv.x, pv.y, pv.z, pv.w};
  const float ge[4] = {gv.x, gv.y, gv.z, gv.w};
  float me[4] = {0.f, 0.f, 0.f, 0.f}, ve[4] = {0.f, 0.f, 0.f, 0.f};
  if (OPT == 1) {
    const f32x4 mv = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(a.m[g]) + i);
    const f32x4 vv = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(a.v[g]) + i);
    me[0] = mv.x; me[1] = mv.y; me[2] = mv.z; me[3] = mv.w;
    ve[0] = vv.x; ve[1] = vv.y; ve[2] = vv.z; ve[3] = vv.w;
  }
#pragma unroll
  for (int e = 0; e < 4; ++e) optim_step<OPT>(pe[e], me[e], ve[e], ge[e], h);
  if (OPT == 1) {
    const f32x4 mo = {me[0], me[1], me[2], me[3]}, vo = {ve[0], ve[1], ve[2], ve[3]};
    __builtin_nontemporal_store(mo, reinterpret_cast<f32x4*>(a.m[g]) + i);
    __builtin_nontemporal_store(vo, reinterpret_cast<f32x4*>(a.v[g]) + i);
  }
  const f32x4 po = {pe[0], pe[1], pe[2], pe[3]};
  __builtin_nontemporal_store(po, p + i);
  if (W16)
    reinterpret_cast<uint2*>(a.w16[g])[i] = make_uint2((uint32_t)f2bf(pe[0]) | ((uint32_t)f2bf(pe[1]) << 16),
                                                       (uint32_t)f2bf(pe[2]) | ((uint32_t)f2bf(pe[3]) << 16));
}

// One vector per lane, workgroup b the b-th run of 256 vectors: the launch sweeps every array once, front to back
// (measured against a grid-stride loop over an eighth of the workgroups: 5.6 -> 5.9 TB/s on 8 x 16.8 M parameters;
// writes in particular run faster the fewer separate address streams are open at a time).
template <int OPT, bool W16>
__global__ __launch_bounds__(256) void optim_kernel(const OptimArgs a) {
  const int g = blockIdx.y;
  const OptimHp h = a.hp[g];
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < (a.n >> 2)) update4<OPT, W16>(a, g, i, h);
}

// one chunk of at most 256 vectors per workgroup
template <int OPT, bool W16>
__global__ __launch_bounds__(256) void optim_chunks_kernel(const OptimArgs a) {
  const int g = blockIdx.y;
  const OptimHp h = a.hp[g];
  const uint2 ch = a.chunks[blockIdx.x];
  if (threadIdx.x < ch.y) update4<OPT, W16>(a, g, (size_t)ch.x + threadIdx.x, h);
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
  if (a.chunks) {
    if (a.n_chunks < 1) return a.n_chunks == 0 ? hipSuccess : hipErrorInvalidValue;
    dim3 grid((unsigned)a.n_chunks, a.G);
    if (a.opt == 0) {
      if (w16) hipLaunchKernelGGL((optim_chunks_kernel<0, true>), grid, dim3(256), 0, s, a);
      else hipLaunchKernelGGL((optim_chunks_kernel<0, false>), grid, dim3(256), 0, s, a);
    } else {
      if (w16) hipLaunchKernelGGL((optim_chunks_kernel<1, true>), grid, dim3(256), 0, s, a);
      else hipLaunchKernelGGL((optim_chunks_kernel<1, false>), grid, dim3(256), 0, s, a);
    }
    return hipGetLastError();
  }
  size_t n4 = a.n >> 2;
  size_t bx = (n4 + 255) / 256;
  if (bx > 0x7fffffffu) return hipErrorInvalidValue;
  dim3 grid((unsigned)bx, a.G);
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
