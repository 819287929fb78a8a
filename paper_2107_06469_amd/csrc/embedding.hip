// Token/position embedding and its adjoint, row gather/scatter for the target rows, and the
// element-wise pieces of the gated feed-forward block.  All memory-bound.
//   embed:      x[t,:] = tok[ids[t],:] + pos[t mod S,:]
//   dtok[v,:]   = sum over tokens t with ids[t] == v of dx[t,:]   (tokens of one id are listed in
//                 ascending order in a CSR built from the data, so the sum has a fixed order and
//                 duplicates need no atomics; rows of unused ids are written as zero)
//   dpos[s,:]   = sum_b dx[b*S+s,:]  (b ascending); rows s >= S of the table get zero
//   gather:     out[r,:] = src[rows[r],:];  scatter: dst = 0, dst[rows[r],:] = src[r,:] (rows distinct)
#include "kernels.h"

namespace hydra {
namespace {

__device__ __forceinline__ bf16_t f2bf(float v) {
  __bf16 h = (__bf16)v;
  return __builtin_bit_cast(bf16_t, h);
}
__device__ __forceinline__ float bf2f(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

template <typename T> __device__ __forceinline__ float to_f(T v);
template <> __device__ __forceinline__ float to_f<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f<bf16_t>(bf16_t v) { return bf2f(v); }
template <typename T> __device__ __forceinline__ T from_f(float v);
template <> __device__ __forceinline__ float from_f<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f<bf16_t>(float v) { return f2bf(v); }

template <typename T>
__global__ __launch_bounds__(256) void embed_fwd_kernel(const EmbedArgs a) {
  const int g = blockIdx.y, t = blockIdx.x;
  const T* tok = static_cast<const T*>(a.tok[g]) + (size_t)a.ids[t] * a.d;
  const T* pos = static_cast<const T*>(a.pos[g]) + (size_t)(t % a.S) * a.d;
  T* x = static_cast<T*>(a.x[g]) + (size_t)t * a.ld;
  for (int c = threadIdx.x; c < a.d; c += 256) x[c] = from_f<T>(to_f<T>(tok[c]) + to_f<T>(pos[c]));
}

// one workgroup per vocabulary row and 256 columns
template <typename T>
__global__ __launch_bounds__(256) void embed_bwd_tok_kernel(const EmbedBwdArgs a) {
  const int g = blockIdx.y, v = blockIdx.x, c = blockIdx.z * 256 + threadIdx.x;
  if (c >= a.d) return;
  const int beg = a.row_ptr[v], end = a.row_ptr[v + 1];
  const T* dx = static_cast<const T*>(a.dx[g]) + c;
  // A frequent id (the mask token holds 15 % of an encoder batch) makes this a long sequential sum: the
  // loads of 16 occurrences are issued together, the additions keep the ascending order.
  float s = 0.f;
  int i = beg;
  for (; i + 16 <= end; i += 16) {
    float w[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) w[u] = to_f<T>(dx[(size_t)a.positions[i + u] * a.ld]);
#pragma unroll
    for (int u = 0; u < 16; ++u) s += w[u];
  }
  for (; i < end; ++i) s += to_f<T>(dx[(size_t)a.positions[i] * a.ld]);
  a.dtok[g][(size_t)v * a.d + c] = s;
}

// one workgroup per row of the position table
template <typename T>
__global__ __launch_bounds__(256) void embed_bwd_pos_kernel(const EmbedBwdArgs a) {
  const int g = blockIdx.y, s = blockIdx.x;
  const T* dx = static_cast<const T*>(a.dx[g]);
  float* out = a.dpos[g] + (size_t)s * a.d;
  for (int c = threadIdx.x; c < a.d; c += 256) {
    float t = 0.f;
    if (s < a.S)
      for (int b = 0; b < a.B; ++b) t += to_f<T>(dx[((size_t)b * a.S + s) * a.ld + c]);
    out[c] = t;
  }
}

template <typename T>
__global__ __launch_bounds__(256) void gather_rows_kernel(const RowsArgs a) {
  const int g = blockIdx.y, r = blockIdx.x;
  const T* src = static_cast<const T*>(a.src[g]) + (size_t)a.rows[r] * a.ld_src;
  T* dst = static_cast<T*>(a.dst[g]) + (size_t)r * a.ld_dst;
  for (int c = threadIdx.x; c < a.d; c += 256) dst[c] = src[c];
}

template <typename T>
__global__ __launch_bounds__(256) void scatter_rows_kernel(const RowsArgs a) {
  const int g = blockIdx.y, r = blockIdx.x;
  const T* src = static_cast<const T*>(a.src[g]) + (size_t)r * a.ld_src;
  T* dst = static_cast<T*>(a.dst[g]) + (size_t)a.rows[r] * a.ld_dst;
  for (int c = threadIdx.x; c < a.d; c += 256) dst[c] = src[c];
}

// gated feed-forward, backward: given dh (gradient of hmid = gelu(zg) * z1)
//   dz1 = dh * gelu(zg);  dzg = dh * z1 * gelu'(zg)
template <typename T>
__global__ __launch_bounds__(256) void gated_bwd_kernel(const GatedBwdArgs a) {
  const int g = blockIdx.y;
  const T* dh = static_cast<const T*>(a.dh[g]);
  const T* z1 = static_cast<const T*>(a.z1[g]);
  const T* zg = static_cast<const T*>(a.zg[g]);
  T* dz1 = static_cast<T*>(a.dz1[g]);
  T* dzg = static_cast<T*>(a.dzg[g]);
  const size_t n = (size_t)a.rows * a.ld, stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) {
    const float d = to_f<T>(dh[i]), u = to_f<T>(z1[i]), z = to_f<T>(zg[i]);
    // normal CDF/density as in the GEMM epilogue (Abramowitz & Stegun 7.1.26 for erf)
    const float xa = fabsf(z) * 0.70710678118654752f, tt = __builtin_amdgcn_rcpf(1.0f + 0.3275911f * xa), ee = __expf(-xa * xa);
    const float er = 1.0f - tt * (0.254829592f + tt * (-0.284496736f + tt * (1.421413741f + tt * (-1.453152027f + tt * 1.061405429f)))) * ee;
    const float cdf = 0.5f * (1.0f + (z < 0.f ? -er : er));
    const float pdf = ee * 0.39894228040143268f;
    dz1[i] = from_f<T>(d * z * cdf);
    dzg[i] = from_f<T>(d * u * (cdf + z * pdf));
  }
}

#define DISPATCH(kernel, grid, args)                                                           \
  do {                                                                                         \
    if ((args).dtype == GEMM_F32) hipLaunchKernelGGL(kernel<float>, grid, dim3(256), 0, s, args); \
    else hipLaunchKernelGGL(kernel<bf16_t>, grid, dim3(256), 0, s, args);                        \
    return hipGetLastError();                                                                  \
  } while (0)

}  // namespace

hipError_t launch_embed_fwd(const EmbedArgs& a, hipStream_t s) {
  if (a.G < 1 || a.G > MAXG || a.tokens < 1 || a.S < 1 || a.d < 1 || a.ld < a.d) return hipErrorInvalidValue;
  DISPATCH(embed_fwd_kernel, dim3(a.tokens, a.G), a);
}
hipError_t launch_embed_bwd(const EmbedBwdArgs& a, hipStream_t s) {
  if (a.G < 1 || a.G > MAXG || a.V < 1 || a.S < 1 || a.B < 1 || a.S_table < a.S || a.ld < a.d) return hipErrorInvalidValue;
  if (a.dtype == GEMM_F32) {
    hipLaunchKernelGGL(embed_bwd_tok_kernel<float>, dim3(a.V, a.G, (a.d + 255) / 256), dim3(256), 0, s, a);
    hipLaunchKernelGGL(embed_bwd_pos_kernel<float>, dim3(a.S_table, a.G), dim3(256), 0, s, a);
  } else {
    hipLaunchKernelGGL(embed_bwd_tok_kernel<bf16_t>, dim3(a.V, a.G, (a.d + 255) / 256), dim3(256), 0, s, a);
    hipLaunchKernelGGL(embed_bwd_pos_kernel<bf16_t>, dim3(a.S_table, a.G), dim3(256), 0, s, a);
  }
  return hipGetLastError();
}
hipError_t launch_gather_rows(const RowsArgs& a, hipStream_t s) {
  if (a.G < 1 || a.G > MAXG || a.n < 1 || a.d < 1) return hipErrorInvalidValue;
  DISPATCH(gather_rows_kernel, dim3(a.n, a.G), a);
}
hipError_t launch_scatter_rows(const RowsArgs& a, hipStream_t s) {
  if (a.G < 1 || a.G > MAXG || a.n < 1 || a.d < 1) return hipErrorInvalidValue;
  DISPATCH(scatter_rows_kernel, dim3(a.n, a.G), a);
}
hipError_t launch_gated_bwd(const GatedBwdArgs& a, hipStream_t s) {
  if (a.G < 1 || a.G > MAXG || a.rows < 1 || a.ld < 1) return hipErrorInvalidValue;
  size_t n = (size_t)a.rows * a.ld;
  size_t b = (n + 255) / 256;
  if (b > 8192) b = 8192;
  DISPATCH(gated_bwd_kernel, dim3((unsigned)b, a.G), a);
}

}  // namespace hydra
