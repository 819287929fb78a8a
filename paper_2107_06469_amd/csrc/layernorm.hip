// LayerNorm forward and backward over rows of width d (bf16 or fp32 rows, fp32 statistics).
//   forward:  mu = mean(x), var = mean((x-mu)^2) (biased), rstd = 1/sqrt(var+eps),
//             y = (x-mu)*rstd*gamma + beta; mu and rstd are saved per row.
//   backward: g = dy*gamma; dx = rstd*(g - mean(g) - xhat*mean(g*xhat)) (+ add);
//             dgamma = sum_rows dy*xhat; dbeta = sum_rows dy.
// One wavefront owns a row (in the backward pass only up to 1024 elements; wider rows are shared by the four
// waves of a workgroup): each lane keeps its 16-byte chunks of the row in registers, statistics are
// butterfly reductions over the 64 lanes (fixed order).  The column sums of the backward pass are
// accumulated per workgroup over a fixed range of rows, written as partial sums, and added over
// workgroups in index order by a second kernel: no atomics, so results do not depend on timing.
#include "kernels.h"

namespace hydra {
namespace {

// MAXC = 8-element chunks a lane may own: d <= 8*64*MAXC (2 -> 1024, 4 -> 2048, 8 -> 4096)
constexpr int LN_ROWS_PER_WG = 64;  // rows per workgroup in the backward pass (4 waves x 16 rows)
// Rows wider than this are taken by a whole workgroup at a time (ln_bwd_wide_kernel), 32 rows per workgroup.
constexpr int LN_WAVE_ROW_MAX = 1024;
constexpr int LN_WIDE_ROWS_PER_WG = 32;

__device__ __forceinline__ bf16_t f2bf(float v) {
  __bf16 h = (__bf16)v;
  return __builtin_bit_cast(bf16_t, h);
}
// two floats -> two bf16 in one word (round to nearest even): one v_cvt_pk_bf16_f32
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  typedef __attribute__((ext_vector_type(2))) float f32x2_t;
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

template <typename T>
__device__ __forceinline__ void ld8(const T* p, float (&v)[8]);
template <>
__device__ __forceinline__ void ld8<float>(const float* p, float (&v)[8]) {
  float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
  v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
template <>
__device__ __forceinline__ void ld8<bf16_t>(const bf16_t* p, float (&v)[8]) {
  uint4 a = *reinterpret_cast<const uint4*>(p);
  uint32_t w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    v[2 * i] = __uint_as_float(w[i] << 16);
    v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
  }
}
template <typename T>
__device__ __forceinline__ void st8(T* p, const float (&v)[8]);
template <>
__device__ __forceinline__ void st8<float>(float* p, const float (&v)[8]) {
  *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
  *reinterpret_cast<float4*>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
}
template <>
__device__ __forceinline__ void st8<bf16_t>(bf16_t* p, const float (&v)[8]) {
  uint32_t w[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) w[i] = pack_bf16x2(v[2 * i], v[2 * i + 1]);
  *reinterpret_cast<uint4*>(p) = make_uint4(w[0], w[1], w[2], w[3]);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

template <typename T, int LN_MAXC>
__global__ __launch_bounds__(256) void ln_fwd_kernel(const LnArgs a) {
  const int g = blockIdx.y, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int row = blockIdx.x * 4 + wave;
  if (row >= a.rows) return;
  const T* x = static_cast<const T*>(a.x[g]) + (size_t)row * a.ld;
  T* y = static_cast<T*>(a.y[g]) + (size_t)row * a.ld;
  const int nch = a.d >> 3;
  float v[LN_MAXC][8];
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < LN_MAXC; ++i) {
    const int c = lane + 64 * i;
    if (c < nch) {
      ld8<T>(x + 8 * c, v[i]);
#pragma unroll
      for (int e = 0; e < 8; ++e) s += v[i][e];
    }
  }
  const float mu = wave_sum(s) / (float)a.d;
  float q = 0.f;
#pragma unroll
  for (int i = 0; i < LN_MAXC; ++i) {
    const int c = lane + 64 * i;
    if (c < nch) {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float t = v[i][e] - mu;
        q += t * t;
      }
    }
  }
  const float rstd = 1.0f / sqrtf(wave_sum(q) / (float)a.d + a.eps);
  const float* gamma = a.gamma[g];
  const float* beta = a.beta[g];
#pragma unroll
  for (int i = 0; i < LN_MAXC; ++i) {
    const int c = lane + 64 * i;
    if (c < nch) {
      float ga[8], be[8], o[8];
      ld8<float>(gamma + 8 * c, ga);
      ld8<float>(beta + 8 * c, be);
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e] = (v[i][e] - mu) * rstd * ga[e] + be[e];
      st8<T>(y + 8 * c, o);
    }
  }
  if (lane == 0) {
    a.mean[g][row] = mu;
    a.rstd[g][row] = rstd;
  }
}

// dx and per-workgroup partial column sums, rows of up to 1024 elements.  Workgroup b owns rows [b*64, b*64+64); wave w takes rows
// b*64 + w, +4, +8, ...; partial sums go to part[g][b][2][d].
template <typename T, int LN_MAXC>
__global__ __launch_bounds__(256) void ln_bwd_kernel(const LnBwdArgs a) {
  extern __shared__ float red[];  // [4][2][d]
  const int g = blockIdx.y, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nch = a.d >> 3;
  const float* gamma = a.gamma[g];
  float ga[LN_MAXC][8], sg[LN_MAXC][8], sb[LN_MAXC][8];
#pragma unroll
  for (int i = 0; i < LN_MAXC; ++i) {
    const int c = lane + 64 * i;
#pragma unroll
    for (int e = 0; e < 8; ++e) sg[i][e] = sb[i][e] = ga[i][e] = 0.f;
    if (c < nch) ld8<float>(gamma + 8 * c, ga[i]);
  }
  const int row0 = blockIdx.x * LN_ROWS_PER_WG;
  // A wave's rows are software-pipelined: the loads of its next row (x, dy, the additive term, the statistics) are
  // issued before the current row is reduced, and stay in flight as raw registers until that row's turn.
  // Only where the extra registers cost no spill and little occupancy: 16-bit rows of at most 1024 elements.  The
  // other shapes fetch each row at its own turn (and its additive term after the reductions).
  constexpr bool PF = sizeof(T) == 2 && LN_MAXC <= 2;
  constexpr int RW = sizeof(T) == 2 ? 1 : 2;  // 16-byte pieces per 8 elements
  uint4 nx[LN_MAXC][RW], ndy[LN_MAXC][RW], nadd[LN_MAXC][RW];
  float nmu = 0.f, nrstd = 0.f;
  auto fetch_row = [&](int row) {
    const uint4* x = reinterpret_cast<const uint4*>(static_cast<const T*>(a.x[g]) + (size_t)row * a.ld);
    const uint4* dy = reinterpret_cast<const uint4*>(static_cast<const T*>(a.dy[g]) + (size_t)row * a.ld);
    const uint4* add = a.add[g] ? reinterpret_cast<const uint4*>(static_cast<const T*>(a.add[g]) + (size_t)row * a.ld) : nullptr;
#pragma unroll
    for (int i = 0; i < LN_MAXC; ++i) {
      const int c = lane + 64 * i;
      if (c < nch) {
#pragma unroll
        for (int q = 0; q < RW; ++q) {
          nx[i][q] = x[c * RW + q];
          ndy[i][q] = dy[c * RW + q];
          if (PF && add) nadd[i][q] = add[c * RW + q];
        }
      }
    }
    nmu = a.mean[g][row];
    nrstd = a.rstd[g][row];
  };
  auto unpack = [&](const uint4 (&raw)[RW], float (&v)[8]) {
    if constexpr (sizeof(T) == 2) {
      const uint32_t w[4] = {raw[0].x, raw[0].y, raw[0].z, raw[0].w};
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        v[2 * q] = __uint_as_float(w[q] << 16);
        v[2 * q + 1] = __uint_as_float(w[q] & 0xffff0000u);
      }
    } else {
      v[0] = __uint_as_float(raw[0].x); v[1] = __uint_as_float(raw[0].y); v[2] = __uint_as_float(raw[0].z); v[3] = __uint_as_float(raw[0].w);
      v[4] = __uint_as_float(raw[RW - 1].x); v[5] = __uint_as_float(raw[RW - 1].y); v[6] = __uint_as_float(raw[RW - 1].z); v[7] = __uint_as_float(raw[RW - 1].w);
    }
  };
  if (PF && row0 + wave < a.rows) fetch_row(row0 + wave);
  for (int r = wave; r < LN_ROWS_PER_WG; r += 4) {
    const int row = row0 + r;
    if (row >= a.rows) break;
    // this row's values move out of the prefetch registers; then the next row's loads are issued
    uint4 cx[LN_MAXC][RW], cdy[LN_MAXC][RW], cadd[LN_MAXC][RW];
#pragma unroll
    for (int i = 0; i < LN_MAXC; ++i)
#pragma unroll
      for (int q = 0; q < RW; ++q) { cx[i][q] = nx[i][q]; cdy[i][q] = ndy[i][q]; cadd[i][q] = nadd[i][q]; }
    const float mu = PF ? nmu : a.mean[g][row], rstd = PF ? nrstd : a.rstd[g][row];
    if (PF && r + 4 < LN_ROWS_PER_WG && row + 4 < a.rows) fetch_row(row + 4);
    float xh[LN_MAXC][8], gg[LN_MAXC][8];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int i = 0; i < LN_MAXC; ++i) {
      const int c = lane + 64 * i;
      if (c < nch) {
        float xv[8], dv[8];
        if constexpr (PF) {
          unpack(cx[i], xv);
          unpack(cdy[i], dv);
        } else {
          ld8<T>(static_cast<const T*>(a.x[g]) + (size_t)row * a.ld + 8 * c, xv);
          ld8<T>(static_cast<const T*>(a.dy[g]) + (size_t)row * a.ld + 8 * c, dv);
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          xh[i][e] = (xv[e] - mu) * rstd;
          gg[i][e] = dv[e] * ga[i][e];
          s1 += gg[i][e];
          s2 += gg[i][e] * xh[i][e];
          sg[i][e] += dv[e] * xh[i][e];
          sb[i][e] += dv[e];
        }
      }
    }
    const float c1 = wave_sum(s1) / (float)a.d, c2 = wave_sum(s2) / (float)a.d;
    T* dx = static_cast<T*>(a.dx[g]) + (size_t)row * a.ld;
    const bool add = a.add[g] != nullptr;
#pragma unroll
    for (int i = 0; i < LN_MAXC; ++i) {
      const int c = lane + 64 * i;
      if (c < nch) {
        float o[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = rstd * (gg[i][e] - c1 - xh[i][e] * c2);
        if (add) {
          float av[8];
          if constexpr (PF) {
            unpack(cadd[i], av);
          } else {
            ld8<T>(static_cast<const T*>(a.add[g]) + (size_t)row * a.ld + 8 * c, av);
          }
#pragma unroll
          for (int e = 0; e < 8; ++e) o[e] += av[e];
        }
        st8<T>(dx + 8 * c, o);
      }
    }
  }
  // the four waves' partial sums are added in wave order
#pragma unroll
  for (int i = 0; i < LN_MAXC; ++i) {
    const int c = lane + 64 * i;
    if (c < nch) {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        red[(wave * 2 + 0) * a.d + 8 * c + e] = sg[i][e];
        red[(wave * 2 + 1) * a.d + 8 * c + e] = sb[i][e];
      }
    }
  }
  __syncthreads();
  float* part = a.part[g] + (size_t)blockIdx.x * 2 * a.d;
  for (int j = threadIdx.x; j < 2 * a.d; j += 256) {
    const int which = j / a.d, col = j % a.d;
    float t = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) t += red[(w * 2 + which) * a.d + col];
    part[which * a.d + col] = t;
  }
}

// Rows of more than 1024 elements: a wave per row would need 32 or 64 values of x-hat and g per lane (one or two waves
// per SIMD, and up to 128 KB of LDS for the cross-wave column sums).  Here the four waves of a workgroup share each
// row: thread t owns chunks t, t + 256 (MAXW of them), the two row sums cross the waves through LDS (added in wave
// order), and every column belongs to exactly one thread, which adds its dgamma/dbeta terms over the workgroup's 32
// rows in row order and writes them to part[g][b][2][d] itself.  16-bit rows are prefetched one row ahead.
template <typename T, int MAXW>
__global__ __launch_bounds__(256) void ln_bwd_wide_kernel(const LnBwdArgs a) {
  __shared__ float xs[2][4][2];  // [row parity][wave][s1, s2]
  const int g = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int nch = a.d >> 3;
  constexpr bool PF = sizeof(T) == 2;
  constexpr int RW = sizeof(T) == 2 ? 1 : 2;  // 16-byte pieces per 8 elements
  const float* gamma = a.gamma[g];
  float ga[MAXW][8], sg[MAXW][8], sb[MAXW][8];
#pragma unroll
  for (int i = 0; i < MAXW; ++i) {
    const int c = tid + 256 * i;
#pragma unroll
    for (int e = 0; e < 8; ++e) sg[i][e] = sb[i][e] = ga[i][e] = 0.f;
    if (c < nch) ld8<float>(gamma + 8 * c, ga[i]);
  }
  uint4 nx[MAXW][RW], ndy[MAXW][RW], nadd[MAXW][RW];
  float nmu = 0.f, nrstd = 0.f;
  const bool has_add = a.add[g] != nullptr;
  auto fetch_row = [&](int row) {
    const uint4* x = reinterpret_cast<const uint4*>(static_cast<const T*>(a.x[g]) + (size_t)row * a.ld);
    const uint4* dy = reinterpret_cast<const uint4*>(static_cast<const T*>(a.dy[g]) + (size_t)row * a.ld);
    const uint4* add = has_add ? reinterpret_cast<const uint4*>(static_cast<const T*>(a.add[g]) + (size_t)row * a.ld) : nullptr;
#pragma unroll
    for (int i = 0; i < MAXW; ++i) {
      const int c = tid + 256 * i;
      if (c < nch) {
#pragma unroll
        for (int q = 0; q < RW; ++q) {
          nx[i][q] = x[c * RW + q];
          ndy[i][q] = dy[c * RW + q];
          if (has_add) nadd[i][q] = add[c * RW + q];
        }
      }
    }
    nmu = a.mean[g][row];
    nrstd = a.rstd[g][row];
  };
  auto unpack = [&](const uint4 (&raw)[RW], float (&v)[8]) {
    if constexpr (sizeof(T) == 2) {
      const uint32_t w[4] = {raw[0].x, raw[0].y, raw[0].z, raw[0].w};
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        v[2 * q] = __uint_as_float(w[q] << 16);
        v[2 * q + 1] = __uint_as_float(w[q] & 0xffff0000u);
      }
    } else {
      v[0] = __uint_as_float(raw[0].x); v[1] = __uint_as_float(raw[0].y); v[2] = __uint_as_float(raw[0].z); v[3] = __uint_as_float(raw[0].w);
      v[4] = __uint_as_float(raw[RW - 1].x); v[5] = __uint_as_float(raw[RW - 1].y); v[6] = __uint_as_float(raw[RW - 1].z); v[7] = __uint_as_float(raw[RW - 1].w);
    }
  };
  const int row0 = blockIdx.x * LN_WIDE_ROWS_PER_WG;
  const int nrow = min(LN_WIDE_ROWS_PER_WG, a.rows - row0);  // the same for every thread: the barriers below are uniform
  if (PF && nrow > 0) fetch_row(row0);
  for (int r = 0; r < nrow; ++r) {
    const int row = row0 + r;
    if (!PF) fetch_row(row);
    uint4 cx[MAXW][RW], cdy[MAXW][RW], cadd[MAXW][RW];
#pragma unroll
    for (int i = 0; i < MAXW; ++i)
#pragma unroll
      for (int q = 0; q < RW; ++q) { cx[i][q] = nx[i][q]; cdy[i][q] = ndy[i][q]; cadd[i][q] = nadd[i][q]; }
    const float mu = nmu, rstd = nrstd;
    if (PF && r + 1 < nrow) fetch_row(row + 1);
    float xh[MAXW][8], gg[MAXW][8];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int i = 0; i < MAXW; ++i) {
      const int c = tid + 256 * i;
      if (c < nch) {
        float xv[8], dv[8];
        unpack(cx[i], xv);
        unpack(cdy[i], dv);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          xh[i][e] = (xv[e] - mu) * rstd;
          gg[i][e] = dv[e] * ga[i][e];
          s1 += gg[i][e];
          s2 += gg[i][e] * xh[i][e];
          sg[i][e] += dv[e] * xh[i][e];
          sb[i][e] += dv[e];
        }
      }
    }
    // Two LDS slots by row parity and one barrier per row: a wave can write the slot of row r + 2 only after the
    // barrier of row r + 1, which every wave reaches after it has read the slot of row r.
    s1 = wave_sum(s1);
    s2 = wave_sum(s2);
    if (lane == 0) {
      xs[r & 1][wave][0] = s1;
      xs[r & 1][wave][1] = s2;
    }
    __syncthreads();
    float t1 = 0.f, t2 = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      t1 += xs[r & 1][w][0];
      t2 += xs[r & 1][w][1];
    }
    const float c1 = t1 / (float)a.d, c2 = t2 / (float)a.d;
    T* dx = static_cast<T*>(a.dx[g]) + (size_t)row * a.ld;
#pragma unroll
    for (int i = 0; i < MAXW; ++i) {
      const int c = tid + 256 * i;
      if (c < nch) {
        float o[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = rstd * (gg[i][e] - c1 - xh[i][e] * c2);
        if (has_add) {
          float av[8];
          unpack(cadd[i], av);
#pragma unroll
          for (int e = 0; e < 8; ++e) o[e] += av[e];
        }
        st8<T>(dx + 8 * c, o);
      }
    }
  }
  float* part = a.part[g] + (size_t)blockIdx.x * 2 * a.d;
#pragma unroll
  for (int i = 0; i < MAXW; ++i) {
    const int c = tid + 256 * i;
    if (c < nch) {
      st8<float>(part + 8 * c, sg[i]);
      st8<float>(part + a.d + 8 * c, sb[i]);
    }
  }
}

// dgamma[col] = sum_b part[b][0][col], dbeta[col] = sum_b part[b][1][col].  A workgroup owns 16 columns; thread
// (w, col) adds the w-th of 16 contiguous ranges of b in ascending order and the 16 range sums are then added in
// ascending w: a fixed order that depends on the number of row blocks only.
__global__ __launch_bounds__(256) void ln_reduce_kernel(const LnBwdArgs a, int nblocks) {
  __shared__ float sh[16][17];
  const int g = blockIdx.y, cl = threadIdx.x & 15, w = threadIdx.x >> 4;
  const int j = blockIdx.x * 16 + cl, n2 = 2 * a.d;
  const int per = (nblocks + 15) / 16, b0 = w * per, b1 = min(nblocks, b0 + per);
  const float* part = a.part[g];
  float t = 0.f;
  if (j < n2)
    for (int b = b0; b < b1; ++b) t += part[(size_t)b * n2 + j];
  sh[w][cl] = t;
  __syncthreads();
  if (w == 0 && j < n2) {
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += sh[i][cl];
    if (j < a.d) a.dgamma[g][j] = s;
    else a.dbeta[g][j - a.d] = s;
  }
}

}  // namespace

int ln_bwd_blocks(int rows, int d) {
  const int per = d > LN_WAVE_ROW_MAX ? LN_WIDE_ROWS_PER_WG : LN_ROWS_PER_WG;
  return (rows + per - 1) / per;
}

static bool ln_shape_ok(int G, int rows, int d, int ld) {
  return G >= 1 && G <= MAXG && rows >= 1 && d >= 8 && !(d & 7) && d <= 4096 && ld >= d && !(ld & 7);
}

template <typename T, int C>
static hipError_t ln_fwd_run(const LnArgs& a, hipStream_t s) {
  hipLaunchKernelGGL((ln_fwd_kernel<T, C>), dim3((a.rows + 3) / 4, a.G), dim3(256), 0, s, a);
  return hipGetLastError();
}
template <typename T>
static hipError_t ln_fwd_pick(const LnArgs& a, hipStream_t s) {
  if (a.d <= 1024) return ln_fwd_run<T, 2>(a, s);
  if (a.d <= 2048) return ln_fwd_run<T, 4>(a, s);
  return ln_fwd_run<T, 8>(a, s);
}

hipError_t launch_ln_fwd(const LnArgs& a, hipStream_t s) {
  if (!ln_shape_ok(a.G, a.rows, a.d, a.ld)) return hipErrorInvalidValue;
  return a.dtype == GEMM_F32 ? ln_fwd_pick<float>(a, s) : ln_fwd_pick<bf16_t>(a, s);
}

template <typename T>
static hipError_t ln_bwd_pick(const LnBwdArgs& a, hipStream_t s) {
  const dim3 grid(ln_bwd_blocks(a.rows, a.d), a.G);
  if (a.d <= LN_WAVE_ROW_MAX) {
    const size_t lds = (size_t)4 * 2 * a.d * sizeof(float);
    hipLaunchKernelGGL((ln_bwd_kernel<T, 2>), grid, dim3(256), lds, s, a);
  } else if (a.d <= 2048) {
    hipLaunchKernelGGL((ln_bwd_wide_kernel<T, 1>), grid, dim3(256), 0, s, a);
  } else {
    hipLaunchKernelGGL((ln_bwd_wide_kernel<T, 2>), grid, dim3(256), 0, s, a);
  }
  return hipGetLastError();
}

hipError_t launch_ln_bwd(const LnBwdArgs& a, hipStream_t s) {
  if (!ln_shape_ok(a.G, a.rows, a.d, a.ld)) return hipErrorInvalidValue;
  hipError_t e = a.dtype == GEMM_F32 ? ln_bwd_pick<float>(a, s) : ln_bwd_pick<bf16_t>(a, s);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(ln_reduce_kernel, dim3((2 * a.d + 15) / 16, a.G), dim3(256), 0, s, a, ln_bwd_blocks(a.rows, a.d));
  return hipGetLastError();
}

// nothing to set up: the wave-per-row kernel needs at most 32 KB of LDS
hipError_t ln_init() { return hipSuccess; }

}  // namespace hydra
