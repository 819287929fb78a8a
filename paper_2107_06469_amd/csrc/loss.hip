// Fused softmax cross-entropy, forward and gradient, over rows of fp32 logits.
//   rowloss[m] = logsumexp(z_m) - z_m[y_m]
//   dz[m,c]    = (exp(z_mc - lse_m) - [c == y_m]) * inv_n
//   loss       = inv_n * sum_m rowloss[m]
// One workgroup per row; maxima and sums are reduced wavefront-first, then across the four
// wavefronts in a fixed order, so the result depends on the row only.
// Rows of up to 32768 logits whose storage is 16-byte aligned are held in registers: the logits are read once
// (6 bytes per logit with a bf16 gradient) and each exponential is evaluated once.  Other rows take three passes.
#include <stdint.h>

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

// Row held in registers: thread t of NT owns the float4 groups t, t + NT, ..., NV of them.
template <typename T, int NV, int NT>
__global__ __launch_bounds__(NT) void softmax_ce_row_kernel(const SoftmaxCeArgs a) {
  constexpr int NWV = NT / 64;
  __shared__ float red[NWV];
  const int m = blockIdx.x, g = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float* z = a.logits[g] + (size_t)m * a.ldz;
  T* dz = static_cast<T*>(a.dz[g]) + (size_t)m * a.lddz;
  const int y = a.labels[m];
  const int C = a.C;
  float v[NV][4];
  float mx = -INFINITY;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = 4 * (tid + NT * i);
    if (c + 4 <= C) {
      const float4 q = *reinterpret_cast<const float4*>(z + c);
      v[i][0] = q.x; v[i][1] = q.y; v[i][2] = q.z; v[i][3] = q.w;
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) v[i][e] = c + e < C ? z[c + e] : -INFINITY;
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) mx = fmaxf(mx, v[i][e]);
  }
  mx = wave_max(mx);
  if (lane == 0) red[wave] = mx;
  __syncthreads();
  mx = red[0];
#pragma unroll
  for (int w = 1; w < NWV; ++w) mx = fmaxf(mx, red[w]);
  __syncthreads();
  // the label's logit, picked up by the thread that holds it
  float zy = 0.f;
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = 4 * (tid + NT * i);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      if (c + e == y) zy = v[i][e];
      v[i][e] = expf(v[i][e] - mx);  // exp(-inf) = 0 past the end of the row
      sum += v[i][e];
    }
  }
  sum = wave_sum(sum);
  if (lane == 0) red[wave] = sum;
  __syncthreads();
  sum = red[0];
#pragma unroll
  for (int w = 1; w < NWV; ++w) sum += red[w];  // fixed order
  const float inv_sum = 1.f / sum;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = 4 * (tid + NT * i);
    if (c >= a.lddz) continue;
    float d[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) d[e] = c + e < C ? (v[i][e] * inv_sum - (c + e == y ? 1.f : 0.f)) * a.inv_n : 0.f;
    if (c + 4 <= a.lddz) {
      if (sizeof(T) == 4) *reinterpret_cast<float4*>(reinterpret_cast<float*>(dz) + c) = make_float4(d[0], d[1], d[2], d[3]);
      else
        *reinterpret_cast<uint2*>(reinterpret_cast<bf16_t*>(dz) + c) =
            make_uint2((uint32_t)f2bf(d[0]) | ((uint32_t)f2bf(d[1]) << 16), (uint32_t)f2bf(d[2]) | ((uint32_t)f2bf(d[3]) << 16));
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (c + e < a.lddz) {
          if (sizeof(T) == 4) reinterpret_cast<float*>(dz)[c + e] = d[e];
          else reinterpret_cast<bf16_t*>(dz)[c + e] = f2bf(d[e]);
        }
    }
  }
  // exactly one thread holds column y
  if ((y >> 2) % NT == tid) a.rowloss[g][m] = (logf(sum) + mx) - zy;
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
  // register path: every row starts on a 16-byte boundary (8 for a bf16 gradient) and the padded row fits
  bool vec = a.ldz % 4 == 0 && a.lddz % 4 == 0 && a.lddz <= 32768;
  for (int g = 0; g < a.G && vec; ++g)
    vec = (reinterpret_cast<uintptr_t>(a.logits[g]) & 15) == 0 && (reinterpret_cast<uintptr_t>(a.dz[g]) & 15) == 0;
  if (vec) {
    const bool f32 = a.dtype == GEMM_F32;
    if (a.lddz <= 1024) {
      if (f32) hipLaunchKernelGGL((softmax_ce_row_kernel<float, 1, 256>), grid, dim3(256), 0, s, a);
      else hipLaunchKernelGGL((softmax_ce_row_kernel<bf16_t, 1, 256>), grid, dim3(256), 0, s, a);
    } else if (a.lddz <= 8192) {
      if (f32) hipLaunchKernelGGL((softmax_ce_row_kernel<float, 8, 256>), grid, dim3(256), 0, s, a);
      else hipLaunchKernelGGL((softmax_ce_row_kernel<bf16_t, 8, 256>), grid, dim3(256), 0, s, a);
    } else {
      if (f32) hipLaunchKernelGGL((softmax_ce_row_kernel<float, 16, 512>), grid, dim3(512), 0, s, a);
      else hipLaunchKernelGGL((softmax_ce_row_kernel<bf16_t, 16, 512>), grid, dim3(512), 0, s, a);
    }
  } else if (a.dtype == GEMM_F32) hipLaunchKernelGGL(softmax_ce_kernel<float>, grid, dim3(256), 0, s, a);
  else hipLaunchKernelGGL(softmax_ce_kernel<bf16_t>, grid, dim3(256), 0, s, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(loss_reduce_kernel, dim3(a.G), dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace hydra
