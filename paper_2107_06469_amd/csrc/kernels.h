// Launchers of the device kernels.  Every launcher enqueues on the given stream and returns the
// HIP status of the launch; none allocates or synchronises.  Pointers are device pointers.
//
// "Grouped" launches run the same operation for G independent problems of identical shape, one
// per model, in a single grid: this is how ready shards of different models that share a shape
// fill the device together (paper, Approach: the unit of parallel work is the shard, and shards
// of different models are independent).  Results of a problem never depend on G or on its
// position in the group.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hydra {

constexpr int MAXG = 16;  // problems per grouped launch

typedef uint16_t bf16_t;  // storage type of bf16 values (top half of an fp32, round-to-nearest-even)

enum { EPI_ACT_NONE = 0, EPI_ACT_RELU = 1, EPI_ACT_GELU = 2 };
enum { GEMM_F32 = 0, GEMM_BF16 = 1 };

// C[M,N] = sum_k X(m,k) * W(n,k) followed by the epilogue
//   v = acc (+ bias[n]);  pre[m,n] = v (optional);
//   v = gate ? v * act'(gate[m,n]) : act(v);  v += resid[m,n] (optional);  out[m,n] = v.
// x_kmajor: X stored [M, ldx] with k contiguous, else stored [K, ldx] with m contiguous.
// w_kmajor: W stored [N, ldw] with k contiguous, else stored [K, ldw] with n contiguous.
// Leading dimensions are in elements and must be multiples of 16 bytes worth of elements, and at
// least the contiguous extent rounded up to that; base pointers 16-byte aligned.
struct GemmArgs {
  int dtype;  // GEMM_F32: operands fp32; GEMM_BF16: operands bf16.  Accumulation is fp32.
  int M, N, K;
  int x_kmajor, w_kmajor;
  int ldx, ldw;
  int G;
  const void* X[MAXG];
  const void* W[MAXG];
  const float* bias[MAXG];  // fp32 [N] or null (all-or-none across the group)
  void* out[MAXG];          // [M, ldo], operand dtype, or fp32 when out_f32
  void* pre[MAXG];          // nullable, [M, ldo], operand dtype
  const void* gate[MAXG];   // nullable, [M, ldg], operand dtype
  const void* resid[MAXG];  // nullable, [M, ldr], operand dtype
  int ldo, ldg, ldr;
  int act;
  int out_f32;
  int tile;  // 0 = choose by problem size; 1 = 256x256, 2 = 128x128, 3 = 32x128 (tests, tuning)
};
hipError_t launch_gemm(const GemmArgs& a, hipStream_t s);
// Must be called once per process before the first launch_gemm (sets the kernels' LDS limits).
hipError_t gemm_init();

// ---- elementwise / reductions (see each .hip file for definitions) ---------------------------------

struct PtrGroup {
  int G;
  void* p[MAXG];
};

// dst[i] = uniform on [-a, a): counter RNG keyed by key, index i.  a2 = 2a.
hipError_t launch_init_uniform(float* dst, size_t n, uint64_t key, float a, hipStream_t s);
hipError_t launch_fill_f32(float* dst, size_t n, float v, hipStream_t s);
hipError_t launch_fill_u32(uint32_t* dst, size_t n, uint32_t v, hipStream_t s);
// dst[i] = bf16(src[i]) for i < n
hipError_t launch_cast_bf16(const float* src, bf16_t* dst, size_t n, hipStream_t s);
// rows x cols (fp32, contiguous) -> rows x ld (fp32 or bf16), padding columns untouched
hipError_t launch_stage_rows(const float* src, void* dst, int rows, int cols, int ld, int to_bf16, hipStream_t s);

// Column sums: out_g[n] = sum_m src_g[m,n] for m < M (fp32 accumulation in a fixed order).
struct ColsumArgs {
  int dtype, M, N, ld, G;
  const void* src[MAXG];
  float* out[MAXG];
};
hipError_t launch_colsum(const ColsumArgs& a, hipStream_t s);

// Softmax cross-entropy over rows of fp32 logits [M, ldz] with C classes:
//   rowloss[m] = logsumexp(z_m) - z_m[y_m];  dz[m,c] = (softmax(z_m)[c] - [c == y_m]) * inv_n
// then loss_out_g[0] = inv_n * sum_m rowloss[m] (fixed order).  dz has dtype `dtype`, leading dim lddz;
// padding columns [C, lddz) are written as zero.
struct SoftmaxCeArgs {
  int dtype, M, C, ldz, lddz, G;
  float inv_n;
  const float* logits[MAXG];
  const int32_t* labels;  // shared by the group, [M]
  void* dz[MAXG];
  float* rowloss[MAXG];   // scratch [M]
  float* loss_out[MAXG];  // one float each
};
hipError_t launch_softmax_ce(const SoftmaxCeArgs& a, hipStream_t s);

// Optimizer over flat fp32 blocks of n elements (n multiple of 4).
//   SGD:  p -= lr * g
//   Adam: m = b1 m + (1-b1) g; v = b2 v + (1-b2) g^2; p -= lr * (m*bc1) / (sqrt(v*bc2) + eps)
// with bc1 = 1/(1-b1^t), bc2 = 1/(1-b2^t) precomputed by the host.  When w16 is non-null the bf16
// working copy is refreshed: w16 = bf16(p).
struct OptimArgs {
  int opt, G;
  size_t n;
  float* p[MAXG];
  const float* g[MAXG];
  float* m[MAXG];
  float* v[MAXG];
  bf16_t* w16[MAXG];
  float lr[MAXG], b1[MAXG], b2[MAXG], c1[MAXG], c2[MAXG], eps[MAXG], bc1[MAXG], bc2[MAXG];  // c = 1 - b, rounded from double
};
hipError_t launch_optim(const OptimArgs& a, hipStream_t s);

}  // namespace hydra
