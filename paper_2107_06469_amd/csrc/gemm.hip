// Grouped matrix-core GEMM for gfx950: C[M,N] = sum_k X(m,k) W(n,k) with a fused epilogue.
//
// It serves the three contractions of a Linear layer (forward Y = X W^T; input gradient
// dX = dY W; weight gradient dW = dY^T X) for bf16 and fp32 operands with fp32 accumulation, for G
// same-shaped problems of different models in one grid.
//
// Design (64-wide wavefronts, v_mfma_f32_32x32x16_bf16 / v_mfma_f32_32x32x2_f32):
//  * A workgroup of WM x WN waves owns a (WM*FM*32) x (WN*FN*32) tile of C; each wave keeps FM x FN
//    accumulators of 32x32 in registers.
//  * Both operand tiles are kept in LDS as rows of 128 bytes of k (64 bf16 or 32 fp32), i.e. eight
//    16-byte chunks per row, whatever the layout in memory: a k-contiguous operand is copied chunk
//    by chunk, an operand stored with k as the slow index is transposed in registers (E x E element
//    blocks, E = elements per 16 bytes) on its way in.  The chunk position inside a row is XOR-ed
//    with (row ^ row>>3)&7 so that fragment reads (32 consecutive rows, one chunk) and transposed
//    writes (rows E apart) both spread over all banks.
//  * The W tile feeds the MFMA "A" operand and the X tile the "B" operand, so a lane ends up holding
//    four consecutive n for one m: epilogue accesses are 8- or 16-byte vectors.
//  * LDS is double buffered: global loads of tile t+1 are issued before the MFMAs of tile t and
//    land in the other buffer afterwards; one barrier per k-tile.
//  * The sum over k runs in ascending order with one MFMA chain per output element, no split-K and
//    no atomics, so a result does not depend on tile shape, grid placement or group size.
//  * Workgroup ids are dealt round-robin to the 8 XCDs by the hardware; the tile index is remapped
//    so each XCD gets a contiguous run of tiles (m fastest) and the M-tiles that share a W tile hit
//    the same L2.
#include "kernels.h"

namespace hydra {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

namespace {

__device__ __forceinline__ int swz(int row) { return (row ^ (row >> 3)) & 7; }

template <typename T>
struct Elem;
template <>
struct Elem<float> {
  static constexpr int E = 4;
  static __device__ __forceinline__ float to_f(float v) { return v; }
  static __device__ __forceinline__ float from_f(float v) { return v; }
};
template <>
struct Elem<bf16_t> {
  static constexpr int E = 8;
  static __device__ __forceinline__ float to_f(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }
  static __device__ __forceinline__ bf16_t from_f(float v) {
    __bf16 h = (__bf16)v;  // round to nearest even (v_cvt_pk_bf16_f32)
    return __builtin_bit_cast(bf16_t, h);
  }
};

// zero the elements of a 16-byte chunk at positions >= valid
template <typename T>
__device__ __forceinline__ uint4 mask_tail(uint4 v, int valid) {
  uint32_t w[4] = {v.x, v.y, v.z, v.w};
  if (sizeof(T) == 4) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (i >= valid) w[i] = 0;
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (2 * i >= valid) w[i] = 0;
      else if (2 * i + 1 >= valid) w[i] &= 0xffffu;
    }
  }
  return make_uint4(w[0], w[1], w[2], w[3]);
}

__device__ __forceinline__ float act_fwd(float v, int act) {
  if (act == EPI_ACT_RELU) return v > 0.f ? v : 0.f;
  if (act == EPI_ACT_GELU) return 0.5f * v * (1.f + erff(v * 0.70710678118654752f));
  return v;
}
__device__ __forceinline__ float act_grad(float z, int act) {
  if (act == EPI_ACT_RELU) return z > 0.f ? 1.f : 0.f;
  if (act == EPI_ACT_GELU)
    return 0.5f * (1.f + erff(z * 0.70710678118654752f)) + z * expf(-0.5f * z * z) * 0.39894228040143268f;
  return 1.f;
}

// ---- global -> register loaders ---------------------------------------------------------------------

// k-contiguous operand: tile rows [row0, row0+ROWS), k in [k0, k0+BK).  Chunk c = tid + NT*i covers
// row c/8, k-chunk c%8.
template <typename T, int ROWS, int NT>
struct LoaderK {
  static constexpr int E = Elem<T>::E;
  static constexpr int NCH = ROWS * 8 / NT;
  static_assert(ROWS * 8 % NT == 0 && NCH >= 1, "tile too small for the workgroup");
  uint4 r[NCH];
  __device__ __forceinline__ void load(const T* base, int ld, int row0, int nrows, int k0, int K, int tid) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      int c = tid + NT * i, row = c >> 3, kc = c & 7;
      int gr = row0 + row, gk = k0 + kc * E;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (gr < nrows && gk < K) {
        v = *reinterpret_cast<const uint4*>(base + (size_t)gr * ld + gk);
        if (gk + E > K) v = mask_tail<T>(v, K - gk);
      }
      r[i] = v;
    }
  }
  __device__ __forceinline__ void store(uint4* tile, int tid) const {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      int c = tid + NT * i, row = c >> 3, kc = c & 7;
      tile[row * 8 + (kc ^ swz(row))] = r[i];
    }
  }
};

// operand stored with k as the slow index: memory is [K, ld] with the tile's row index contiguous.
// Block b = tid + NT*i covers rows [mb*E, mb*E+E) x k [kb*E, kb*E+E), mb = b % (ROWS/E), kb = b / (ROWS/E);
// it is read as E chunks along the row index and written as E chunks along k.
template <typename T, int ROWS, int NT>
struct LoaderT {
  static constexpr int E = Elem<T>::E;
  static constexpr int NB = (ROWS / E) * 8;
  static constexpr int NBT = (NB + NT - 1) / NT;
  uint4 r[NBT][E];
  __device__ __forceinline__ void load(const T* base, int ld, int row0, int nrows, int k0, int K, int tid) {
#pragma unroll
    for (int i = 0; i < NBT; ++i) {
      int b = tid + NT * i;
      int mb = b % (ROWS / E), kb = b / (ROWS / E);
      int gr = row0 + mb * E;
#pragma unroll
      for (int j = 0; j < E; ++j) {
        int gk = k0 + kb * E + j;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (b < NB && gr < nrows && gk < K) v = *reinterpret_cast<const uint4*>(base + (size_t)gk * ld + gr);
        r[i][j] = v;
      }
    }
  }
  __device__ __forceinline__ void store(uint4* tile, int tid) const {
#pragma unroll
    for (int i = 0; i < NBT; ++i) {
      int b = tid + NT * i;
      if (b >= NB) continue;
      int mb = b % (ROWS / E), kb = b / (ROWS / E);
      uint32_t in[E][4];
#pragma unroll
      for (int j = 0; j < E; ++j) {
        in[j][0] = r[i][j].x; in[j][1] = r[i][j].y; in[j][2] = r[i][j].z; in[j][3] = r[i][j].w;
      }
#pragma unroll
      for (int m = 0; m < E; ++m) {
        uint32_t o[4];
        if (sizeof(T) == 4) {
#pragma unroll
          for (int q = 0; q < 4; ++q) o[q] = in[q][m];
        } else {
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            uint32_t lo = (in[2 * q][m >> 1] >> (16 * (m & 1))) & 0xffffu;
            uint32_t hi = (in[2 * q + 1][m >> 1] >> (16 * (m & 1))) & 0xffffu;
            o[q] = lo | (hi << 16);
          }
        }
        int row = mb * E + m;
        tile[row * 8 + (kb ^ swz(row))] = make_uint4(o[0], o[1], o[2], o[3]);
      }
    }
  }
};

template <typename T, int ROWS, int NT, bool KMAJ>
struct LoaderSel { typedef LoaderK<T, ROWS, NT> type; };
template <typename T, int ROWS, int NT>
struct LoaderSel<T, ROWS, NT, false> { typedef LoaderT<T, ROWS, NT> type; };

// ---- one 32x32 MFMA step over 16 bytes of k per lane ----------------------------------------------
template <typename T>
__device__ __forceinline__ void mma(f32x16& acc, const uint4& wfrag, const uint4& xfrag);
template <>
__device__ __forceinline__ void mma<bf16_t>(f32x16& acc, const uint4& wfrag, const uint4& xfrag) {
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, wfrag), __builtin_bit_cast(bf16x8, xfrag),
                                                acc, 0, 0, 0);
}
template <>
__device__ __forceinline__ void mma<float>(f32x16& acc, const uint4& wfrag, const uint4& xfrag) {
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(wfrag.x), __uint_as_float(xfrag.x), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(wfrag.y), __uint_as_float(xfrag.y), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(wfrag.z), __uint_as_float(xfrag.z), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(wfrag.w), __uint_as_float(xfrag.w), acc, 0, 0, 0);
}

// 8 consecutive elements of operand type T <-> 8 floats (16-byte aligned for bf16, 32-byte for fp32)
template <typename T>
__device__ __forceinline__ void load8(const T* p, float (&v)[8]);
template <>
__device__ __forceinline__ void load8<float>(const float* p, float (&v)[8]) {
  float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
  v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
template <>
__device__ __forceinline__ void load8<bf16_t>(const bf16_t* p, float (&v)[8]) {
  uint4 a = *reinterpret_cast<const uint4*>(p);
  uint32_t w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    v[2 * i] = __uint_as_float(w[i] << 16);
    v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
  }
}
template <typename T>
__device__ __forceinline__ void store8(T* p, const float (&v)[8]);
template <>
__device__ __forceinline__ void store8<float>(float* p, const float (&v)[8]) {
  *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
  *reinterpret_cast<float4*>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
}
template <>
__device__ __forceinline__ void store8<bf16_t>(bf16_t* p, const float (&v)[8]) {
  uint32_t w[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
    w[i] = (uint32_t)Elem<bf16_t>::from_f(v[2 * i]) | ((uint32_t)Elem<bf16_t>::from_f(v[2 * i + 1]) << 16);
  *reinterpret_cast<uint4*>(p) = make_uint4(w[0], w[1], w[2], w[3]);
}

template <typename T, int WM, int WN, int FM, int FN, bool X_KMAJ, bool W_KMAJ>
__global__ __launch_bounds__(WM* WN * 64) void gemm_kernel(const GemmArgs a) {
  constexpr int E = Elem<T>::E;
  constexpr int BK = 8 * E;
  constexpr int BM = WM * FM * 32, BN = WN * FN * 32;
  constexpr int NT = WM * WN * 64;
  extern __shared__ uint4 lds[];  // [2][(BM + BN) * 8] chunks
  constexpr int STAGE = (BM + BN) * 8;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;

  // tile index, remapped so that each XCD works on a contiguous run of tiles
  const int tiles_m = (a.M + BM - 1) / BM, tiles_n = (a.N + BN - 1) / BN;
  const int n_tiles = tiles_m * tiles_n * a.G;
  const int per_xcd = (n_tiles + 7) >> 3;
  const int t_id = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (t_id >= n_tiles) return;
  const int tm = t_id % tiles_m, tn = (t_id / tiles_m) % tiles_n, g = t_id / (tiles_m * tiles_n);
  const int m0 = tm * BM, n0 = tn * BN;

  const T* X = static_cast<const T*>(a.X[g]);
  const T* W = static_cast<const T*>(a.W[g]);

  typename LoaderSel<T, BM, NT, X_KMAJ>::type lx;
  typename LoaderSel<T, BN, NT, W_KMAJ>::type lw;

  f32x16 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int nk = (a.K + BK - 1) / BK;
  lx.load(X, a.ldx, m0, a.M, 0, a.K, tid);
  lw.load(W, a.ldw, n0, a.N, 0, a.K, tid);
  lx.store(lds, tid);
  lw.store(lds + BM * 8, tid);
  __syncthreads();

  const int lrow = lane & 31, lgrp = lane >> 5;
  for (int kt = 0; kt < nk; ++kt) {
    const uint4* tx = lds + (kt & 1) * STAGE;
    const uint4* tw = tx + BM * 8;
    if (kt + 1 < nk) {
      lx.load(X, a.ldx, m0, a.M, (kt + 1) * BK, a.K, tid);
      lw.load(W, a.ldw, n0, a.N, (kt + 1) * BK, a.K, tid);
    }
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const int kc = 2 * s + lgrp;
      uint4 xf[FM], wf[FN];
#pragma unroll
      for (int i = 0; i < FM; ++i) {
        int row = (wm * FM + i) * 32 + lrow;
        xf[i] = tx[row * 8 + (kc ^ swz(row))];
      }
#pragma unroll
      for (int j = 0; j < FN; ++j) {
        int row = (wn * FN + j) * 32 + lrow;
        wf[j] = tw[row * 8 + (kc ^ swz(row))];
      }
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) mma<T>(acc[i][j], wf[j], xf[i]);
    }
    if (kt + 1 < nk) {
      uint4* nx = lds + ((kt + 1) & 1) * STAGE;
      lx.store(nx, tid);
      lw.store(nx + BM * 8, tid);
    }
    __syncthreads();
  }

  // ---- epilogue -----------------------------------------------------------------------------------
  // Each wave passes its accumulators through its own LDS patch, one 32-row band (32 x FN*32 fp32)
  // at a time, and reads them back row-wise so that a lane owns 8 consecutive n of one m: global
  // accesses are 16/32-byte vectors and a row band is written as FN*32 contiguous elements.
  constexpr int SP = FN * 32 + 4;          // patch pitch in floats (+4: spreads rows over banks)
  constexpr int LPR = FN * 4;              // lanes per row (8 elements each)
  constexpr int RPP = 64 / LPR;            // rows per pass
  static_assert((size_t)WM * WN * 32 * SP * 4 <= 2 * (size_t)STAGE * 16, "epilogue patch exceeds LDS");
  float* patch = reinterpret_cast<float*>(lds) + wave * (32 * SP);
  const float* bias = a.bias[g];
  T* pre = static_cast<T*>(a.pre[g]);
  const T* gate = static_cast<const T*>(a.gate[g]);
  const T* resid = static_cast<const T*>(a.resid[g]);
  const T* mul = static_cast<const T*>(a.mul[g]);
  const int act = a.act;
#pragma unroll
  for (int i = 0; i < FM; ++i) {
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q)
        *reinterpret_cast<float4*>(&patch[lrow * SP + j * 32 + 8 * q + 4 * lgrp]) =
            make_float4(acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
    __syncthreads();
    for (int p = 0; p < 32 / RPP; ++p) {
      const int r = p * RPP + lane / LPR, c = (lane % LPR) * 8;
      const int m = m0 + (wm * FM + i) * 32 + r, n = n0 + wn * FN * 32 + c;
      if (m >= a.M || n >= a.N) continue;
      float v[8];
      load8<float>(&patch[r * SP + c], v);
      const int cnt = a.N - n;  // >= 8: full vector
      if (cnt >= 8) {
        if (bias) {
          float b[8];
          load8<float>(bias + n, b);
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] += b[e];
        }
        if (pre) store8<T>(pre + (size_t)m * a.ldo + n, v);
        if (gate) {
          float z[8];
          load8<T>(gate + (size_t)m * a.ldg + n, z);
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] *= act_grad(z[e], act);
        } else if (act != EPI_ACT_NONE) {
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] = act_fwd(v[e], act);
        }
        if (mul) {
          float z[8];
          load8<T>(mul + (size_t)m * a.ldo + n, z);
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] *= z[e];
        }
        if (resid) {
          float z[8];
          load8<T>(resid + (size_t)m * a.ldr + n, z);
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] += z[e];
        }
        if (a.out_f32) store8<float>(static_cast<float*>(a.out[g]) + (size_t)m * a.ldo + n, v);
        else store8<T>(static_cast<T*>(a.out[g]) + (size_t)m * a.ldo + n, v);
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          if (e < cnt) {
            float t = v[e];
            if (bias) t += bias[n + e];
            if (pre) pre[(size_t)m * a.ldo + n + e] = Elem<T>::from_f(t);
            if (gate) t *= act_grad(Elem<T>::to_f(gate[(size_t)m * a.ldg + n + e]), act);
            else t = act_fwd(t, act);
            if (mul) t *= Elem<T>::to_f(mul[(size_t)m * a.ldo + n + e]);
            if (resid) t += Elem<T>::to_f(resid[(size_t)m * a.ldr + n + e]);
            if (a.out_f32) static_cast<float*>(a.out[g])[(size_t)m * a.ldo + n + e] = t;
            else static_cast<T*>(a.out[g])[(size_t)m * a.ldo + n + e] = Elem<T>::from_f(t);
          }
        }
      }
    }
    __syncthreads();
  }
}

template <typename T, int WM, int WN, int FM, int FN>
struct Cfg {
  static constexpr int BM = WM * FM * 32, BN = WN * FN * 32, NT = WM * WN * 64;
  static constexpr size_t LDS = 2 * (size_t)(BM + BN) * 8 * 16;
  template <bool XK, bool WK>
  static hipError_t run1(const GemmArgs& a, hipStream_t s) {
    int tiles = ((a.M + BM - 1) / BM) * ((a.N + BN - 1) / BN) * a.G;
    int grid = ((tiles + 7) / 8) * 8;
    hipLaunchKernelGGL((gemm_kernel<T, WM, WN, FM, FN, XK, WK>), dim3(grid), dim3(NT), LDS, s, a);
    return hipGetLastError();
  }
  static hipError_t run(const GemmArgs& a, hipStream_t s) {
    if (a.x_kmajor) return a.w_kmajor ? run1<true, true>(a, s) : run1<true, false>(a, s);
    return a.w_kmajor ? run1<false, true>(a, s) : run1<false, false>(a, s);
  }
  template <bool XK, bool WK>
  static hipError_t attr1() {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_kernel<T, WM, WN, FM, FN, XK, WK>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS);
  }
  static hipError_t attr() {
    hipError_t e;
    if ((e = attr1<true, true>()) != hipSuccess) return e;
    if ((e = attr1<true, false>()) != hipSuccess) return e;
    if ((e = attr1<false, true>()) != hipSuccess) return e;
    return attr1<false, false>();
  }
};

template <typename T>
hipError_t dispatch(const GemmArgs& a, hipStream_t s) {
  typedef Cfg<T, 2, 2, 4, 4> Big;   // 256 x 256
  typedef Cfg<T, 2, 2, 2, 2> Mid;   // 128 x 128
  typedef Cfg<T, 1, 4, 1, 1> Small; // 32 x 128
  int tile = a.tile;
  if (tile == 0) {
    auto tiles = [&](int bm, int bn) { return (long)((a.M + bm - 1) / bm) * ((a.N + bn - 1) / bn) * a.G; };
    if (a.M >= 192 && tiles(256, 256) >= 192) tile = 1;
    else if (a.M >= 96 && tiles(128, 128) >= 64) tile = 2;
    else tile = 3;
  }
  if (tile == 1) return Big::run(a, s);
  if (tile == 2) return Mid::run(a, s);
  return Small::run(a, s);
}

}  // namespace

hipError_t gemm_init() {
  hipError_t e;
  if ((e = Cfg<bf16_t, 2, 2, 4, 4>::attr()) != hipSuccess) return e;
  if ((e = Cfg<bf16_t, 2, 2, 2, 2>::attr()) != hipSuccess) return e;
  if ((e = Cfg<bf16_t, 1, 4, 1, 1>::attr()) != hipSuccess) return e;
  if ((e = Cfg<float, 2, 2, 4, 4>::attr()) != hipSuccess) return e;
  if ((e = Cfg<float, 2, 2, 2, 2>::attr()) != hipSuccess) return e;
  return Cfg<float, 1, 4, 1, 1>::attr();
}

hipError_t kernels_init() {
  hipError_t e;
  if ((e = gemm_init()) != hipSuccess) return e;
  if ((e = ln_init()) != hipSuccess) return e;
  return attn_init();
}

hipError_t launch_gemm(const GemmArgs& a, hipStream_t s) {
  const int E = a.dtype == GEMM_F32 ? 4 : 8;
  auto rup = [&](int v) { return (v + E - 1) / E * E; };
  if (a.G < 1 || a.G > MAXG || a.M < 1 || a.N < 1 || a.K < 1) return hipErrorInvalidValue;
  if (a.ldx % E || a.ldw % E) return hipErrorInvalidValue;
  if (a.ldx < rup(a.x_kmajor ? a.K : a.M) || a.ldw < rup(a.w_kmajor ? a.K : a.N)) return hipErrorInvalidValue;
  if (a.ldo < a.N) return hipErrorInvalidValue;
  // the epilogue moves 8 consecutive outputs as 16/32-byte vectors
  if (a.ldo % 8 || (a.gate[0] && a.ldg % 8) || (a.resid[0] && a.ldr % 8)) return hipErrorInvalidValue;
  for (int g = 0; g < a.G; ++g) {
    if (!a.X[g] || !a.W[g] || !a.out[g]) return hipErrorInvalidValue;
    if (((uintptr_t)a.X[g] | (uintptr_t)a.W[g] | (uintptr_t)a.out[g] | (uintptr_t)a.bias[g] | (uintptr_t)a.pre[g] |
         (uintptr_t)a.gate[g] | (uintptr_t)a.resid[g] | (uintptr_t)a.mul[g]) & 15)
      return hipErrorInvalidValue;
    if ((a.bias[g] == nullptr) != (a.bias[0] == nullptr) || (a.pre[g] == nullptr) != (a.pre[0] == nullptr) ||
        (a.mul[g] == nullptr) != (a.mul[0] == nullptr) ||
        (a.gate[g] == nullptr) != (a.gate[0] == nullptr) || (a.resid[g] == nullptr) != (a.resid[0] == nullptr))
      return hipErrorInvalidValue;
  }
  if (a.gate[0] && a.ldg < a.N) return hipErrorInvalidValue;
  if (a.resid[0] && a.ldr < a.N) return hipErrorInvalidValue;
  return a.dtype == GEMM_F32 ? dispatch<float>(a, s) : dispatch<bf16_t>(a, s);
}

}  // namespace hydra
