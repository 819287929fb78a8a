// Small memory-bound kernels: seeded initialisation, fills, casts, batch staging, column sums.
#include <mutex>

#include "../../include/hydra.h"
#include "../../include/hydra_ops.h"
#include "kernels.h"

// Partial column sums of hydra_op_colsum_noalloc: one array per GPU, held until the process ends.  In host code
// this name is only a handle for hipGetSymbolAddress; kernels get the address that call returns.
constexpr size_t COLSUM_SCRATCH_FLOATS = (size_t)1 << 20;  // 4 MiB
static __device__ __align__(256) float scratch[COLSUM_SCRATCH_FLOATS];

namespace hydra {
namespace {

__device__ __forceinline__ bf16_t f2bf(float v) {
  __bf16 h = (__bf16)v;  // round to nearest even
  return __builtin_bit_cast(bf16_t, h);
}
__device__ __forceinline__ float bf2f(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

// SplitMix64 (Steele, Lea, Flood 2014): output n of the generator started at `key` is the
// finaliser applied to key + (n+1)*golden.  24 high bits -> u in [0,1); value = u*2a - a, one rounding.
__global__ void init_uniform_kernel(float* dst, size_t n, uint64_t key, float a) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) {
    uint64_t z = key + (i + 1) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    z ^= z >> 31;
    float u = (float)(uint32_t)(z >> 40) * 5.9604644775390625e-08f;  // exact: 24 bits * 2^-24
    dst[i] = __fmaf_rn(u, 2.0f * a, -a);
  }
}

__global__ void fill_u32_kernel(uint32_t* dst, size_t n, uint32_t v) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) dst[i] = v;
}

__global__ void cast_bf16_kernel(const float* __restrict__ src, bf16_t* __restrict__ dst, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) dst[i] = f2bf(src[i]);
}

__global__ void stage_rows_kernel(const float* __restrict__ src, void* __restrict__ dst, int rows, int cols, int ld,
                                  int to_bf16) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t n = (size_t)rows * cols, stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) {
    size_t r = i / cols, c = i % cols;
    float v = src[i];
    if (to_bf16) static_cast<bf16_t*>(dst)[r * ld + c] = f2bf(v);
    else static_cast<float*>(dst)[r * ld + c] = v;
  }
}

// Column sums in two fixed-order stages.  Stage 1: a block owns 64 columns and a chunk of 256 rows;
// its 16 row lanes each add every 16th row of the chunk in ascending order, then the 16 partial sums
// are added in lane order.  Stage 2 (only when there is more than one chunk) adds the chunk sums in
// chunk order.  The order depends on (M, column) only, never on timing or on the group.
constexpr int COLSUM_CHUNK = 256;

template <typename T>
__global__ __launch_bounds__(1024) void colsum_kernel(const ColsumArgs a, int nch) {
  __shared__ float part[16][64];
  const int g = blockIdx.z, ch = blockIdx.y, col = blockIdx.x * 64 + (threadIdx.x & 63), rl = threadIdx.x >> 6;
  const T* src = static_cast<const T*>(a.src[g]);
  const int m_end = min(a.M, (ch + 1) * COLSUM_CHUNK);
  float s = 0.f;
  if (col < a.N) {
    for (int m = ch * COLSUM_CHUNK + rl; m < m_end; m += 16) {
      T v = src[(size_t)m * a.ld + col];
      s += sizeof(T) == 4 ? *reinterpret_cast<const float*>(&v) : bf2f(*reinterpret_cast<const bf16_t*>(&v));
    }
  }
  part[rl][threadIdx.x & 63] = s;
  __syncthreads();
  if (rl == 0 && col < a.N) {
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) t += part[i][threadIdx.x];
    if (nch == 1) a.out[g][col] = t;
    else a.part[g][(size_t)ch * a.N + col] = t;
  }
}

__global__ __launch_bounds__(256) void colsum_reduce_kernel(const ColsumArgs a, int nch) {
  const int g = blockIdx.y, col = blockIdx.x * 256 + threadIdx.x;
  if (col >= a.N) return;
  float t = 0.f;
  for (int ch = 0; ch < nch; ++ch) t += a.part[g][(size_t)ch * a.N + col];
  a.out[g][col] = t;
}

inline int blocks_for(size_t n, int threads, int cap = 4096) {
  size_t b = (n + threads - 1) / threads;
  return (int)(b < 1 ? 1 : (b > (size_t)cap ? cap : b));
}

}  // namespace

hipError_t launch_init_uniform(float* dst, size_t n, uint64_t key, float a, hipStream_t s) {
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(init_uniform_kernel, dim3(blocks_for(n, 256)), dim3(256), 0, s, dst, n, key, a);
  return hipGetLastError();
}
hipError_t launch_fill_u32(uint32_t* dst, size_t n, uint32_t v, hipStream_t s) {
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(fill_u32_kernel, dim3(blocks_for(n, 256)), dim3(256), 0, s, dst, n, v);
  return hipGetLastError();
}
hipError_t launch_fill_f32(float* dst, size_t n, float v, hipStream_t s) {
  uint32_t bits;
  __builtin_memcpy(&bits, &v, 4);
  return launch_fill_u32(reinterpret_cast<uint32_t*>(dst), n, bits, s);
}
hipError_t launch_cast_bf16(const float* src, bf16_t* dst, size_t n, hipStream_t s) {
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(cast_bf16_kernel, dim3(blocks_for(n, 256)), dim3(256), 0, s, src, dst, n);
  return hipGetLastError();
}
hipError_t launch_stage_rows(const float* src, void* dst, int rows, int cols, int ld, int to_bf16, hipStream_t s) {
  if (rows <= 0 || cols <= 0 || ld < cols) return hipErrorInvalidValue;
  hipLaunchKernelGGL(stage_rows_kernel, dim3(blocks_for((size_t)rows * cols, 256)), dim3(256), 0, s, src, dst, rows,
                     cols, ld, to_bf16);
  return hipGetLastError();
}
size_t colsum_part_floats(int M, int N) {
  const int nch = (M + COLSUM_CHUNK - 1) / COLSUM_CHUNK;
  return nch > 1 ? (size_t)nch * N : 0;
}

hipError_t launch_colsum(const ColsumArgs& a, hipStream_t s) {
  if (a.G < 1 || a.G > MAXG || a.M < 1 || a.N < 1 || a.ld < a.N) return hipErrorInvalidValue;
  const int nch = (a.M + COLSUM_CHUNK - 1) / COLSUM_CHUNK;
  if (nch > 1)
    for (int g = 0; g < a.G; ++g)
      if (!a.part[g]) return hipErrorInvalidValue;
  dim3 grid((a.N + 63) / 64, nch, a.G);
  if (a.dtype == GEMM_F32) hipLaunchKernelGGL(colsum_kernel<float>, grid, dim3(1024), 0, s, a, nch);
  else hipLaunchKernelGGL(colsum_kernel<bf16_t>, grid, dim3(1024), 0, s, a, nch);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || nch == 1) return e;
  hipLaunchKernelGGL(colsum_reduce_kernel, dim3((a.N + 255) / 256, a.G), dim3(256), 0, s, a, nch);
  return hipGetLastError();
}

}  // namespace hydra

// ---- measurement aid: the cost of a kernel launch that does nothing ------------------------------------------
namespace {
__global__ void empty_kernel() {}
}  // namespace

extern "C" int hydra_op_empty_launches(int n, void* stream) {
  if (n < 0) return hydra::ops_fail(HYDRA_ERR_INVALID_ARG, "hydra_op_empty_launches: n < 0");
  for (int i = 0; i < n; ++i) hipLaunchKernelGGL(empty_kernel, dim3(1), dim3(64), 0, static_cast<hipStream_t>(stream));
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? HYDRA_OK : hydra::ops_fail(HYDRA_ERR_DEVICE, "hydra_op_empty_launches", hipGetErrorString(e));
}

// ---- column sums for callers that cannot allocate ---------------------------------------------------------
namespace {
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
float* g_scratch_ptr[MAX_DEVICES] = {};  // device address of `scratch` on every GPU seen so far

// address of the current device's copy of the scratch array (looked up once per device)
hipError_t scratch_of_current_device(float** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = static_cast<float*>(p);
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}
}  // namespace

extern "C" size_t hydra_op_colsum_noalloc_max_floats(void) { return COLSUM_SCRATCH_FLOATS; }

extern "C" int hydra_op_colsum_noalloc(int dtype, int M, int N, int ld, int G, const void* const* src, float* const* out,
                                       void* stream) {
  using namespace hydra;
  if (!src || !out || G < 1 || G > MAXG) return ops_fail(HYDRA_ERR_INVALID_ARG, "hydra_op_colsum_noalloc: NULL table or G out of range");
  if (M < 1 || N < 1 || ld < N) return ops_fail(HYDRA_ERR_INVALID_ARG, "hydra_op_colsum_noalloc: need M, N >= 1 and ld >= N");
  const size_t per = colsum_part_floats(M, N);
  if (per * (size_t)G > COLSUM_SCRATCH_FLOATS)
    return ops_fail(HYDRA_ERR_INVALID_ARG,
                    "hydra_op_colsum_noalloc: the partial sums of this call (G * ceil(M/256) * N floats) exceed the built-in "
                    "scratch of 1048576 floats; use hydra_op_colsum with caller scratch");
  float* base = nullptr;
  hipError_t e = scratch_of_current_device(&base);
  if (e != hipSuccess) return ops_fail(HYDRA_ERR_DEVICE, "hydra_op_colsum_noalloc: scratch lookup failed", hipGetErrorString(e));
  ColsumArgs a{};
  a.dtype = dtype == HYDRA_OPS_F32 ? GEMM_F32 : GEMM_BF16;
  a.M = M; a.N = N; a.ld = ld; a.G = G;
  for (int g = 0; g < G; ++g) {
    if (!src[g] || !out[g]) return ops_fail(HYDRA_ERR_INVALID_ARG, "hydra_op_colsum_noalloc: NULL entry");
    a.src[g] = src[g];
    a.out[g] = out[g];
    a.part[g] = base + (size_t)g * per;  // every partial sum that stage 2 reads is written by stage 1 first: nothing to clear
  }
  e = launch_colsum(a, static_cast<hipStream_t>(stream));
  if (e != hipSuccess)
    return ops_fail(e == hipErrorInvalidValue ? HYDRA_ERR_INVALID_ARG : HYDRA_ERR_DEVICE, "hydra_op_colsum_noalloc", hipGetErrorString(e));
  return HYDRA_OK;
}
