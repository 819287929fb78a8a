// Fused softmax cross-entropy, forward and gradient, over rows of fp32 logits.
//   rowloss[m] = logsumexp(z_m) - z_m[y_m]
//   dz[m,c]    = (exp(z_mc - lse_m) - [c == y_m]) * inv_n
//   loss       = inv_n * sum_m rowloss[m]
// One workgroup per row; maxima and sums are reduced wavefront-first, then across the four
// wavefronts in a fixed order, so the result depends on the row only.
#include "kernels.h"

namespace hydra {
namespace {

__device__ __forceinline__ bf16_t f2bf(float v) {
  __bf16 h = (__bf16)v;
  return __builtin_bit_cast(bf16_t, h);
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

template <typename T>
__global__ __launch_bounds__(256) void softmax_ce_kernel(const SoftmaxCeArgs a) {
  __shared__ float red[4];
  const int m = blockIdx.x, g = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float* z = a.logits[g] + (size_t)m * a.ldz;
  T* dz = static_cast<T*>(a.dz[g]) + (size_t)m * a.lddz;
  const int y = a.labels[m];

  float mx = -INFINITY;
  for (int c = tid; c < a.C; c += 256) mx = fmaxf(mx, z[c]);
  mx = wave_max(mx);
  if (lane == 0) red[wave] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  __syncthreads();

  float sum = 0.f;
  for (int c = tid; c < a.C; c += 256) sum += expf(z[c] - mx);
  sum = wave_sum(sum);
  if (lane == 0) red[wave] = sum;
  __syncthreads();
  sum = (red[0] + red[1]) + (red[2] + red[3]);
  const float lse = logf(sum) + mx;
  const float inv_sum = 1.f / sum;

  for (int c = tid; c < a.lddz; c += 256) {
    float d = 0.f;
    if (c < a.C) d = (expf(z[c] - mx) * inv_sum - (c == y ? 1.f : 0.f)) * a.inv_n;
    if (sizeof(T) == 4) reinterpret_cast<float*>(dz)[c] = d;
    else reinterpret_cast<bf16_t*>(dz)[c] = f2bf(d);
  }
  if (tid == 0) a.rowloss[g][m] = lse - z[y];
}

// loss = inv_n * sum of rowloss[0..M): each thread adds every 256th row in ascending order, then a
// fixed tree over the 256 partial sums.
__global__ __launch_bounds__(256) void loss_reduce_kernel(const SoftmaxCeArgs a) {
  __shared__ float red[256];
  const int g = blockIdx.x, tid = threadIdx.x;
  float s = 0.f;
  for (int m = tid; m < a.M; m += 256) s += a.rowloss[g][m];
  red[tid] = s;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if (tid < o) red[tid] += red[tid + o];
    __syncthreads();
  }
  if (tid == 0) a.loss_out[g][0] = red[0] * a.inv_n;
}

}  // namespace

hipError_t launch_softmax_ce(const SoftmaxCeArgs& a, hipStream_t s) {
  if (a.G < 1 || a.G > MAXG || a.M < 1 || a.C < 1 || a.ldz < a.C || a.lddz < a.C) return hipErrorInvalidValue;
  dim3 grid(a.M, a.G);
  if (a.dtype == GEMM_F32) hipLaunchKernelGGL(softmax_ce_kernel<float>, grid, dim3(256), 0, s, a);
  else hipLaunchKernelGGL(softmax_ce_kernel<bf16_t>, grid, dim3(256), 0, s, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(loss_reduce_kernel, dim3(a.G), dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace hydra
