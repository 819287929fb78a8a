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
//    so each XCD gets a contiguous run of tiles, ordered in bands of 8 tile rows so that the tiles
//    resident on an XCD at one time share a few X and W panels in its L2.
//  * With a GemmUpdate the kernel is the weight-gradient GEMM of a Linear layer and its epilogue
//    applies the optimizer step to the parameters, moments and bf16 working copy of the elements
//    it holds (optim_math.h): the gradient never goes to memory (paper, Approach, "Desiderata":
//    same update as unsharded training, so the arithmetic is shared with the optimizer kernel).
#include <algorithm>

#include "act_math.h"
#include "kernels.h"
#include "optim_math.h"

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
// two floats -> two bf16 in one word (round to nearest even): one v_cvt_pk_bf16_f32
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  typedef __attribute__((ext_vector_type(2))) float f32x2_t;
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

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

typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

// Buffer descriptor covering bytes [first, total) of a matrix (empty when first >= total).  Reads beyond
// it return zero, which is what pads ragged tiles.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t tile_rsrc(const void* base, long first, long total) {
  long rem = total - first;
  rem = rem < 0 ? 0 : (rem > 0x7fffffffL ? 0x7fffffffL : rem);
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(static_cast<const char*>(base)) + (rem > 0 ? first : 0), 0,
                                           (int)rem, 0x00020000);
}

// ---- global -> register loaders ---------------------------------------------------------------------

// k-contiguous operand: tile rows [row0, row0+ROWS), k in [k0, k0+BK).  Chunk c = tid + NT*i covers
// row c/8, k-chunk c%8.
template <typename T, int ROWS, int NT>
struct LoaderK {
  static constexpr int E = Elem<T>::E;
  static constexpr int NCH = ROWS * 8 / NT;
  static_assert(ROWS * 8 % NT == 0 && NCH >= 1, "tile too small for the workgroup");
  static constexpr int N_LOAD = NCH, N_STORE = NCH;  // global loads / LDS writes per thread and tile
  uint4 r[NCH];
  // Buffer loads: the descriptor starts at the tile's first element and ends with the matrix, so rows
  // past the matrix read as zero without a guard; a chunk past the end of k is sent out of range.
  __device__ __forceinline__ void load(const T* base, int ld, int row0, int nrows, int k0, int K, int tid) {
    const long first = ((long)row0 * ld + k0) * (long)sizeof(T);
    const __amdgpu_buffer_rsrc_t rs = tile_rsrc(base, first, (long)nrows * ld * (long)sizeof(T));
    const int kc = tid & 7, gk = k0 + kc * E;
    const unsigned voff = ((unsigned)(tid >> 3) * (unsigned)ld + (unsigned)(kc * E)) * (unsigned)sizeof(T);
    const unsigned step = (unsigned)(NT / 8) * (unsigned)ld * (unsigned)sizeof(T);
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const unsigned off = gk < K ? voff + step * i : 0xfffffff0u;
      const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rs, (int)off, 0, 0);
      r[i] = make_uint4(v.x, v.y, v.z, v.w);
      if (gk < K && gk + E > K) r[i] = mask_tail<T>(r[i], K - gk);
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
// Block b covers rows [mb*E, mb*E+E) x k [kb*E, kb*E+E), mb = b % (ROWS/E), kb = b / (ROWS/E); it is read as E
// chunks along the row index and written as E chunks along k.  When the tile has fewer blocks than the
// workgroup has threads, SPLIT = 2 threads share a block (each takes half of its k rows, i.e. half of every
// 16-byte chunk it writes).  Work unit u maps to (mb, half, kb) with 16 consecutive lanes on consecutive mb
// (256 contiguous bytes per global load) and the next 16 lanes on the other half: a 32-lane group then writes
// both halves of 8 distinct chunks, i.e. all LDS banks, instead of one half of them four times over.
template <typename T, int ROWS, int NT>
struct LoaderT {
  static constexpr int E = Elem<T>::E;
  static constexpr int RB = ROWS / E;                           // blocks along the row index
  static constexpr int LO = RB < 16 ? RB : 16;                  // consecutive lanes on consecutive blocks
  static_assert(RB % LO == 0, "tile rows must be a multiple of 16 blocks (or fewer than 16)");
  static constexpr int NB = RB * 8;                             // E x E blocks in the tile
  static constexpr int SPLIT = (2 * NB <= NT) ? 2 : 1;          // threads sharing a block (halves of its k rows)
  static constexpr int KR = E / SPLIT;                          // k rows per thread
  static constexpr int NU = NB * SPLIT;                         // work units
  static constexpr int NBT = (NU + NT - 1) / NT;
  static constexpr int N_LOAD = NBT * KR, N_STORE = NBT * E;
  static constexpr int OW = KR * (int)sizeof(T) / 4;            // dwords written per output row (4, 2 or 1)
  uint4 r[NBT][KR];
  // Buffer loads: the descriptor starts at element (k0, row0) and ends after k row K-1, so k rows past K
  // read as zero without a guard.  Tile rows past the matrix read whatever follows (padding or the next
  // k row); they only feed outputs that are never stored.
  __device__ __forceinline__ void load(const T* base, int ld, int row0, int nrows, int k0, int K, int tid) {
    const long first = ((long)k0 * ld + row0) * (long)sizeof(T);
    const __amdgpu_buffer_rsrc_t rs = tile_rsrc(base, first, (long)K * ld * (long)sizeof(T));
    (void)nrows;
#pragma unroll
    for (int i = 0; i < NBT; ++i) {
      const int u = tid + NT * i, half = (u / LO) % SPLIT, rest = u / (LO * SPLIT);
      const int mb = u % LO + LO * (rest % (RB / LO)), kb = rest / (RB / LO);
      const unsigned voff = ((unsigned)(kb * E + half * KR) * (unsigned)ld + (unsigned)(mb * E)) * (unsigned)sizeof(T);
#pragma unroll
      for (int j = 0; j < KR; ++j) {
        const unsigned off = u < NU ? voff + (unsigned)j * (unsigned)ld * (unsigned)sizeof(T) : 0xfffffff0u;
        const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rs, (int)off, 0, 0);
        r[i][j] = make_uint4(v.x, v.y, v.z, v.w);
      }
    }
  }
  __device__ __forceinline__ void store(uint4* tile, int tid) const {
#pragma unroll
    for (int i = 0; i < NBT; ++i) {
      const int u = tid + NT * i, half = (u / LO) % SPLIT, rest = u / (LO * SPLIT);
      if (u >= NU) continue;
      const int mb = u % LO + LO * (rest % (RB / LO)), kb = rest / (RB / LO);
      uint32_t in[KR][4];
#pragma unroll
      for (int j = 0; j < KR; ++j) {
        in[j][0] = r[i][j].x; in[j][1] = r[i][j].y; in[j][2] = r[i][j].z; in[j][3] = r[i][j].w;
      }
#pragma unroll
      for (int m = 0; m < E; ++m) {
        uint32_t o[OW];
        if (sizeof(T) == 4) {
#pragma unroll
          for (int q = 0; q < OW; ++q) o[q] = in[q][m];
        } else {
#pragma unroll
          for (int q = 0; q < OW; ++q) {
            uint32_t lo = (in[2 * q][m >> 1] >> (16 * (m & 1))) & 0xffffu;
            uint32_t hi = (in[2 * q + 1][m >> 1] >> (16 * (m & 1))) & 0xffffu;
            o[q] = lo | (hi << 16);
          }
        }
        const int row = mb * E + m;
        uint32_t* dst = reinterpret_cast<uint32_t*>(tile + row * 8 + (kb ^ swz(row))) + half * OW;
        if (OW == 4) *reinterpret_cast<uint4*>(dst) = make_uint4(o[0], o[1 % OW], o[2 % OW], o[3 % OW]);
        else if (OW == 2) *reinterpret_cast<uint2*>(dst) = make_uint2(o[0], o[1 % OW]);
        else *dst = o[0];
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

// c + the sum of the elements of one 16-byte operand chunk, added in a fixed order
template <typename T>
__device__ __forceinline__ float chunk_sum(const uint4& f, float c);
template <>
__device__ __forceinline__ float chunk_sum<bf16_t>(const uint4& f, float c) {
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
  const bf16x2 one = {(__bf16)1.0f, (__bf16)1.0f};
  c = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, f.x), one, c, false);
  c = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, f.y), one, c, false);
  c = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, f.z), one, c, false);
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, f.w), one, c, false);
}
template <>
__device__ __forceinline__ float chunk_sum<float>(const uint4& f, float c) {
#pragma clang fp contract(off)
  c = c + __uint_as_float(f.x);
  c = c + __uint_as_float(f.y);
  c = c + __uint_as_float(f.z);
  return c + __uint_as_float(f.w);
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
// 8 bf16 held in a 16-byte register group -> 8 floats
__device__ __forceinline__ void unpack8(const uint4& a, float (&v)[8]) {
  const uint32_t w[4] = {a.x, a.y, a.z, a.w};
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
    w[i] = pack_bf16x2(v[2 * i], v[2 * i + 1]);
  *reinterpret_cast<uint4*>(p) = make_uint4(w[0], w[1], w[2], w[3]);
}

// Streaming (non-temporal) store of 8 outputs: a large activation tensor is written once and read by a later
// launch, long after these lines would have left the caches
template <typename T>
__device__ __forceinline__ void store8_stream(T* p, const float (&v)[8]);
template <>
__device__ __forceinline__ void store8_stream<float>(float* p, const float (&v)[8]) {
  const f32x4 a = {v[0], v[1], v[2], v[3]}, b = {v[4], v[5], v[6], v[7]};
  __builtin_nontemporal_store(a, reinterpret_cast<f32x4*>(p));
  __builtin_nontemporal_store(b, reinterpret_cast<f32x4*>(p) + 1);
}
template <>
__device__ __forceinline__ void store8_stream<bf16_t>(bf16_t* p, const float (&v)[8]) {
  u32x4 w;
#pragma unroll
  for (int i = 0; i < 4; ++i)
    w[i] = pack_bf16x2(v[2 * i], v[2 * i + 1]);
  __builtin_nontemporal_store(w, reinterpret_cast<u32x4*>(p));
}

// Scheduling hint for one MFMA step: spread NR LDS reads and NMEM memory operations (mask MEMMASK:
// 0x200 = LDS write, 0x020 = global read) evenly between the step's NM MFMAs.
template <int NM, int NR, int NMEM, int MEMMASK>
__device__ __forceinline__ void sched_interleave() {
  constexpr int want = NR > NMEM ? NR : NMEM;
  constexpr int groups = want < NM ? want : NM;
  if constexpr (groups > 0) {
    constexpr int per = NM / groups;
    constexpr int rd = (NR + groups - 1) / groups, mem = (NMEM + groups - 1) / groups;
#pragma unroll
    for (int i = 0; i < groups; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, per, 0);
      if constexpr (rd > 0) __builtin_amdgcn_sched_group_barrier(0x100, rd, 0);
      if constexpr (mem > 0) __builtin_amdgcn_sched_group_barrier(MEMMASK, mem, 0);
    }
    if constexpr (NM - per * groups > 0) __builtin_amdgcn_sched_group_barrier(0x008, NM - per * groups, 0);
  }
}

// PF (W operand) and PFX <= PF (X operand) = k-tiles kept in flight in registers (1 or 2 register sets).  With one wave per SIMD
// (4-wave workgroups) fragments are double buffered so LDS latency hides behind the previous step's MFMAs;
// with two waves per SIMD the other wave's MFMAs hide it and the registers are saved.
struct NoUpdate {};
template <bool UPD> struct UpdSel { typedef NoUpdate type; };
template <> struct UpdSel<true> { typedef GemmUpdate type; };

// Orders a wave's own LDS writes before its own later LDS reads (and the reverse): a wave's LDS instructions
// execute in order, so no hardware barrier is needed, only that the compiler keeps the order.
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Epilogue of a wave of a weight-gradient product with the parameter update in it.  The optimizer state of a pass (8
// rows of a 32-row band) depends on addresses only, so the loads of LA passes are issued together, ahead of the values
// they will be combined with: more bytes in flight per wave while the accumulators still travel through the patch.
// A lane takes 4 consecutive columns in two rows (RPP/2 apart) rather than 8 in one, so that each 16-byte load or
// store instruction of the wave covers whole contiguous row segments (FN*128 bytes per row).  The state is read once
// and written once per launch: loads and fp32 stores carry the non-temporal hint, so that the lines do not displace
// the operand panels that other workgroups' k-loops still re-read from L2.  OPT (the optimizer) and INSIDE (the
// wave's block lies inside the matrix: no bounds tests) are fixed at compile time and every pointer is read from the
// argument block once, so that the passes are straight-line code.
template <int FM, int FN, int OPT, bool INSIDE>
__device__ __forceinline__ void update_bands(f32x16 (&acc)[FM][FN], float* patch, const GemmArgs& a, const GemmUpdate& upd,
                                             int g, int mrow0, int ncol0, int lane) {
  constexpr int SP = FN * 32 + 4, LPR = FN * 4, RPP = 64 / LPR, NP = 32 / RPP;
  constexpr int LA = FM * FN <= 4 ? NP : 2;  // passes in flight (registers permitting)
  constexpr int LPR4 = FN * 8, RPH = 64 / LPR4;  // lanes per row with 4 columns each; rows per instruction
  static_assert(NP % LA == 0 && RPH * 2 == RPP, "passes per band");
  const int lrow = lane & 31, lgrp = lane >> 5;
  const bool adam = OPT < 0 ? upd.opt == 1 : OPT == 1;  // OPT = -1: decided at run time (one copy of the code)
  const OptimHp h = upd.hp[g];
  float* const P = upd.p[g];
  float* const Mo = upd.m[g];
  float* const Vo = upd.v[g];
  bf16_t* const W16 = upd.w16[g];
  float* const G = static_cast<float*>(a.out[g]);
  const int M = a.M, N = a.N;
  const size_t ldo = (size_t)a.ldo;
#pragma unroll
  for (int i = 0; i < FM; ++i) {
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q)
        *reinterpret_cast<float4*>(&patch[lrow * SP + j * 32 + 8 * q + 4 * lgrp]) =
            make_float4(acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
    wave_lds_sync();
#pragma unroll
    for (int p0 = 0; p0 < NP; p0 += LA) {
      f32x4 pe[LA][2], me[LA][2], ve[LA][2];
      size_t idx[LA][2];
      bool ok[LA][2];
#pragma unroll
      for (int q = 0; q < LA; ++q)
#pragma unroll
        for (int hf = 0; hf < 2; ++hf) {
          const int r = (p0 + q) * RPP + hf * RPH + lane / LPR4, n = ncol0 + (lane % LPR4) * 4;
          const int m = mrow0 + i * 32 + r;
          ok[q][hf] = INSIDE || (m < M && n < N);  // N is a multiple of 8 here (checked by the launcher): full vectors only
          idx[q][hf] = (size_t)m * ldo + n;
          if (ok[q][hf]) {
            pe[q][hf] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(P + idx[q][hf]));
            if (adam) {
              me[q][hf] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(Mo + idx[q][hf]));
              ve[q][hf] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(Vo + idx[q][hf]));
            }
          }
        }
#pragma unroll
      for (int q = 0; q < LA; ++q)
#pragma unroll
        for (int hf = 0; hf < 2; ++hf) {
          if (!ok[q][hf]) continue;
          const int r = (p0 + q) * RPP + hf * RPH + lane / LPR4, c = (lane % LPR4) * 4;
          const float4 gv = *reinterpret_cast<const float4*>(&patch[r * SP + c]);
          const float v[4] = {gv.x, gv.y, gv.z, gv.w};
          float pp[4] = {pe[q][hf].x, pe[q][hf].y, pe[q][hf].z, pe[q][hf].w};
          float mm[4] = {0.f, 0.f, 0.f, 0.f}, vv[4] = {0.f, 0.f, 0.f, 0.f};
          const size_t ix = idx[q][hf];
          if (adam) {
            mm[0] = me[q][hf].x; mm[1] = me[q][hf].y; mm[2] = me[q][hf].z; mm[3] = me[q][hf].w;
            vv[0] = ve[q][hf].x; vv[1] = ve[q][hf].y; vv[2] = ve[q][hf].z; vv[3] = ve[q][hf].w;
#pragma unroll
            for (int e = 0; e < 4; ++e) optim_step<1>(pp[e], mm[e], vv[e], v[e], h);
            const f32x4 mo = {mm[0], mm[1], mm[2], mm[3]}, vo = {vv[0], vv[1], vv[2], vv[3]};
            __builtin_nontemporal_store(mo, reinterpret_cast<f32x4*>(Mo + ix));
            __builtin_nontemporal_store(vo, reinterpret_cast<f32x4*>(Vo + ix));
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) optim_step<0>(pp[e], mm[e], vv[e], v[e], h);
          }
          const f32x4 po = {pp[0], pp[1], pp[2], pp[3]};
          __builtin_nontemporal_store(po, reinterpret_cast<f32x4*>(P + ix));
          if (W16) *reinterpret_cast<uint2*>(W16 + ix) = make_uint2(pack_bf16x2(pp[0], pp[1]), pack_bf16x2(pp[2], pp[3]));
          if (G) *reinterpret_cast<float4*>(G + ix) = gv;
        }
    }
    wave_lds_sync();
  }
}

// Epilogue of a wave that stores its fp32 sums as they are (a gradient, or a partial sum of a split one) and whose
// block lies inside the matrix: 4 consecutive columns per lane in two rows, so that each 16-byte store instruction of
// the wave covers contiguous row segments; no tests per element.
template <int FM, int FN>
__device__ __forceinline__ void plain_f32_bands(f32x16 (&acc)[FM][FN], float* patch, float* out, size_t ldo, int mrow0,
                                                int ncol0, int lane) {
  constexpr int SP = FN * 32 + 4, LPR = FN * 4, RPP = 64 / LPR, LPR4 = FN * 8, RPH = 64 / LPR4;
  const int lrow = lane & 31, lgrp = lane >> 5;
  const int c = (lane % LPR4) * 4, rl = lane / LPR4;
  float* const o = out + (size_t)(mrow0 + rl) * ldo + ncol0 + c;
#pragma unroll
  for (int i = 0; i < FM; ++i) {
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q)
        *reinterpret_cast<float4*>(&patch[lrow * SP + j * 32 + 8 * q + 4 * lgrp]) =
            make_float4(acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
    wave_lds_sync();
#pragma unroll
    for (int p = 0; p < 32 / RPP; ++p)
#pragma unroll
      for (int hf = 0; hf < 2; ++hf) {
        const int r = p * RPP + hf * RPH;
        *reinterpret_cast<float4*>(o + (size_t)(i * 32 + r) * ldo) = *reinterpret_cast<const float4*>(&patch[(r + rl) * SP + c]);
      }
    wave_lds_sync();
  }
}

// Epilogue of a wave whose 32 FM x 32 FN block lies inside the matrix, bf16 operands, no update: no bounds checks, the
// bias is read once, and per 32-row band everything the band reads from memory (gate, multiplier, residual) is
// requested before the band's first store, so that a wait for a load is not also a wait for the stores in front of
// it.  MODE >= 0 fixes which operands exist (EPI_* bits) and ACT the activation at compile time: straight-line code,
// where the version that tests them at run time (MODE = -1) spends much of its time in taken branches.  Per element
// the same operations in the same order as the general path of tile_epilogue.
enum { EPI_BIAS = 1, EPI_PRE = 2, EPI_GATE = 4, EPI_RESID = 8, EPI_ACTF = 16 };
template <typename T, int FM, int FN, int MODE, int ACT>
__device__ __forceinline__ void fast_bands(f32x16 (&acc)[FM][FN], float* patch, const GemmArgs& a, int g, int mrow0,
                                           int ncol0, int lane, size_t out_off) {
  constexpr bool CT = MODE >= 0;
  constexpr int SP = FN * 32 + 4, LPR = FN * 4, RPP = 64 / LPR, NP = 32 / RPP;
  const int lrow = lane & 31, lgrp = lane >> 5;
  const float* bias = a.bias[g];
  T* pre = static_cast<T*>(a.pre[g]);
  const T* gate = static_cast<const T*>(a.gate[g]);
  const T* resid = static_cast<const T*>(a.resid[g]);
  const T* mul = static_cast<const T*>(a.mul[g]);
  void* const outp = a.out[g];
  const bool has_bias = CT ? (MODE & EPI_BIAS) != 0 : bias != nullptr;
  const bool has_pre = CT ? (MODE & EPI_PRE) != 0 : pre != nullptr;
  const bool has_gate = CT ? (MODE & EPI_GATE) != 0 : gate != nullptr;
  const bool has_resid = CT ? (MODE & EPI_RESID) != 0 : resid != nullptr;
  const bool has_mul = CT ? false : mul != nullptr;
  const bool out_f32 = CT ? false : a.out_f32 != 0;
  const int act = CT ? ACT : a.act;
  const bool has_actf = CT ? (MODE & EPI_ACTF) != 0 : (!has_gate && act != EPI_ACT_NONE);
  const int c = (lane % LPR) * 8, r0 = lane / LPR, n = ncol0 + c;
  float bv[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (has_bias) load8<float>(bias + n, bv);
#pragma unroll
  for (int i = 0; i < FM; ++i) {
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q)
        *reinterpret_cast<float4*>(&patch[lrow * SP + j * 32 + 8 * q + 4 * lgrp]) =
            make_float4(acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
    wave_lds_sync();
    uint4 gz[NP], mz[NP], rz[NP];
#pragma unroll
    for (int p = 0; p < NP; ++p) {
      const size_t m = (size_t)(mrow0 + i * 32 + p * RPP + r0);
      if (has_gate) gz[p] = *reinterpret_cast<const uint4*>(gate + m * a.ldg + n);
      if (has_mul) mz[p] = *reinterpret_cast<const uint4*>(mul + m * a.ldo + n);
      if (has_resid) rz[p] = *reinterpret_cast<const uint4*>(resid + m * a.ldr + n);
    }
#pragma unroll
    for (int p = 0; p < NP; ++p) {
      const size_t m = (size_t)(mrow0 + i * 32 + p * RPP + r0);
      float v[8], z[8];
      load8<float>(&patch[(p * RPP + r0) * SP + c], v);
      if (has_bias) {
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] += bv[e];
      }
      if (has_pre) store8_stream<T>(pre + m * a.ldo + n, v);
      if (has_gate) {
        unpack8(gz[p], z);
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] *= act_grad(z[e], act);
      } else if (has_actf) {
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = act_fwd(v[e], act);
      }
      if (has_mul) {
        unpack8(mz[p], z);
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] *= z[e];
      }
      if (has_resid) {
        unpack8(rz[p], z);
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] += z[e];
      }
      if (out_f32) store8<float>(static_cast<float*>(outp) + out_off + m * a.ldo + n, v);
      else store8_stream<T>(static_cast<T*>(outp) + m * a.ldo + n, v);
    }
    wave_lds_sync();
  }
}

// Epilogue of one wave: its FM x FN accumulators (rows mrow0.., columns ncol0.. of problem g) pass through the
// wave's own LDS patch (32 x (FN*32+4) floats), one 32-row band at a time, and are read back row-wise so that a
// lane owns 8 consecutive n of one m: global accesses are 16/32-byte vectors and a row band is written as FN*32
// contiguous elements.  Only the wave itself touches its patch, so the waves of a workgroup run their epilogues
// independently.
// SPEC: which versions of the fast path a kernel carries (each costs compile time and code size): -1 none, 0 the one
// that tests the operands at run time, 1 also the straight-line ones of forward products (bias; bias + residual;
// bias + activation + stored pre-activation), 2 also those of input gradients (nothing; residual; gate; gate +
// residual).
template <typename T, int FM, int FN, bool UPD, int SPEC = -1>
__device__ __forceinline__ void tile_epilogue(f32x16 (&acc)[FM][FN], float* patch, const GemmArgs& a,
                                              const typename UpdSel<UPD>::type& upd, int g, int mrow0, int ncol0, int lane,
                                              size_t out_off = 0) {
  constexpr int SP = FN * 32 + 4;          // patch pitch in floats (+4: spreads rows over banks)
  constexpr int LPR = FN * 4;              // lanes per row (8 elements each)
  constexpr int RPP = 64 / LPR;            // rows per pass
  const int lrow = lane & 31, lgrp = lane >> 5;
  const float* bias = a.bias[g];
  T* pre = static_cast<T*>(a.pre[g]);
  const T* gate = static_cast<const T*>(a.gate[g]);
  const T* resid = static_cast<const T*>(a.resid[g]);
  const T* mul = static_cast<const T*>(a.mul[g]);
  const int act = a.act;
  const bool plain_f32 = !UPD && a.out_f32 && !pre && !gate && !resid && !mul && act == EPI_ACT_NONE;
  const bool vec4_ok = a.ldo % 4 == 0 && (reinterpret_cast<uintptr_t>(a.out[g]) & 15) == 0 && out_off % 4 == 0 &&
                      (reinterpret_cast<uintptr_t>(bias) & 15) == 0;
  if constexpr (!UPD) {
    if (plain_f32 && !bias && vec4_ok && mrow0 + FM * 32 <= a.M && ncol0 + FN * 32 <= a.N) {
      plain_f32_bands<FM, FN>(acc, patch, static_cast<float*>(a.out[g]) + out_off, (size_t)a.ldo, mrow0, ncol0, lane);
      return;
    }
  }
  if constexpr (UPD) {
    if constexpr (SPEC >= 0) {
      const bool inside = mrow0 + FM * 32 <= a.M && ncol0 + FN * 32 <= a.N;
      if (upd.opt == 1) {
        if (inside) update_bands<FM, FN, 1, true>(acc, patch, a, upd, g, mrow0, ncol0, lane);
        else update_bands<FM, FN, 1, false>(acc, patch, a, upd, g, mrow0, ncol0, lane);
      } else {
        if (inside) update_bands<FM, FN, 0, true>(acc, patch, a, upd, g, mrow0, ncol0, lane);
        else update_bands<FM, FN, 0, false>(acc, patch, a, upd, g, mrow0, ncol0, lane);
      }
    } else {  // the register-staged kernel's 256x256 tile has no registers to spare for more than one copy
      update_bands<FM, FN, -1, false>(acc, patch, a, upd, g, mrow0, ncol0, lane);
    }
    return;
  }
  // A wave whose 32 FM x 32 FN block lies inside the matrix (bf16 operands) takes the path without bounds checks
  // (fast_bands above); the combinations of epilogue operands that the trainers use have straight-line versions.
  if constexpr (!UPD && sizeof(T) == 2 && SPEC >= 0) {
    if (!plain_f32 && mrow0 + FM * 32 <= a.M && ncol0 + FN * 32 <= a.N) {
      const int mode = (bias ? EPI_BIAS : 0) | (pre ? EPI_PRE : 0) | (gate ? EPI_GATE : 0) | (resid ? EPI_RESID : 0) |
                       (!gate && act != EPI_ACT_NONE ? EPI_ACTF : 0);
      bool done = false;
      if constexpr (SPEC > 0) {
        if (!mul && !a.out_f32 && (mode & (EPI_GATE | EPI_ACTF) ? (act == EPI_ACT_GELU || act == EPI_ACT_RELU) : true)) {
          done = true;
#define HYDRA_EPI_CASE(M)                                                                                              \
  case M:                                                                                                              \
    if ((M) & (EPI_GATE | EPI_ACTF)) {                                                                                 \
      if (act == EPI_ACT_GELU) fast_bands<T, FM, FN, M, EPI_ACT_GELU>(acc, patch, a, g, mrow0, ncol0, lane, out_off);   \
      else fast_bands<T, FM, FN, M, EPI_ACT_RELU>(acc, patch, a, g, mrow0, ncol0, lane, out_off);                      \
    } else {                                                                                                           \
      fast_bands<T, FM, FN, M, EPI_ACT_NONE>(acc, patch, a, g, mrow0, ncol0, lane, out_off);                           \
    }                                                                                                                  \
    break;
          if constexpr (SPEC == 1) {
            switch (mode) {
              HYDRA_EPI_CASE(EPI_BIAS)
              HYDRA_EPI_CASE(EPI_BIAS | EPI_RESID)
              HYDRA_EPI_CASE(EPI_BIAS | EPI_PRE | EPI_ACTF)
              default: done = false;
            }
          } else {
            switch (mode) {
              HYDRA_EPI_CASE(0)
              HYDRA_EPI_CASE(EPI_RESID)
              HYDRA_EPI_CASE(EPI_GATE)
              HYDRA_EPI_CASE(EPI_GATE | EPI_RESID)
              default: done = false;
            }
          }
#undef HYDRA_EPI_CASE
        }
      }
      if (!done) fast_bands<T, FM, FN, -1, 0>(acc, patch, a, g, mrow0, ncol0, lane, out_off);
      return;
    }
  }
#pragma unroll
  for (int i = 0; i < FM; ++i) {
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q)
        *reinterpret_cast<float4*>(&patch[lrow * SP + j * 32 + 8 * q + 4 * lgrp]) =
            make_float4(acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
    wave_lds_sync();
    if (plain_f32) {
      // fp32 sums stored as they are (a gradient, or a partial sum of a split one): 4 consecutive columns per lane in
      // two rows, so that each 16-byte store instruction of the wave covers contiguous row segments
      constexpr int LPR4 = FN * 8, RPH = 64 / LPR4;
      float* o = static_cast<float*>(a.out[g]) + out_off;
#pragma unroll
      for (int p = 0; p < 32 / RPP; ++p)
#pragma unroll
        for (int hf = 0; hf < 2; ++hf) {
          const int r = p * RPP + hf * RPH + lane / LPR4, c = (lane % LPR4) * 4;
          const int m = mrow0 + i * 32 + r, n = ncol0 + c;
          if (m >= a.M || n >= a.N) continue;
          float4 v = *reinterpret_cast<const float4*>(&patch[r * SP + c]);
          if (n + 4 <= a.N && vec4_ok) {
            if (bias) {
              const float4 bv = *reinterpret_cast<const float4*>(bias + n);
              v.x += bv.x; v.y += bv.y; v.z += bv.z; v.w += bv.w;
            }
            *reinterpret_cast<float4*>(o + (size_t)m * a.ldo + n) = v;
          } else {
            const float e4[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (n + e < a.N) o[(size_t)m * a.ldo + n + e] = e4[e] + (bias ? bias[n + e] : 0.f);
          }
        }
      wave_lds_sync();
      continue;
    }
    for (int p = 0; p < 32 / RPP; ++p) {
      const int r = p * RPP + lane / LPR, c = (lane % LPR) * 8;
      const int m = mrow0 + i * 32 + r, n = ncol0 + c;
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
        if (pre) store8_stream<T>(pre + (size_t)m * a.ldo + n, v);
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
        if (a.out_f32) store8<float>(static_cast<float*>(a.out[g]) + out_off + (size_t)m * a.ldo + n, v);
        else store8_stream<T>(static_cast<T*>(a.out[g]) + (size_t)m * a.ldo + n, v);
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
            if (a.out_f32) static_cast<float*>(a.out[g])[out_off + (size_t)m * a.ldo + n + e] = t;
            else static_cast<T*>(a.out[g])[(size_t)m * a.ldo + n + e] = Elem<T>::from_f(t);
          }
        }
      }
    }
    wave_lds_sync();
  }
}



// UPD: the accumulators are weight gradients and the epilogue applies the parameter update to the
// elements it holds instead of (or besides) storing them.
template <typename T, int WM, int WN, int FM, int FN, int PFX, int PF, bool X_KMAJ, bool W_KMAJ, bool UPD>
__global__ __launch_bounds__(WM* WN * 64) void gemm_kernel(const GemmArgs a, const typename UpdSel<UPD>::type upd) {
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
  // Tile order inside a problem: bands of GM tile rows; inside a band the column index is the slow
  // one.  The few dozen tiles an XCD runs at a time then form a GM x (a few columns) block that shares
  // GM X panels and a few W panels in its L2, instead of one long row or column of tiles whose other
  // operand is streamed from memory again for every tile.
  constexpr int GM = 8;
  const int g = t_id / (tiles_m * tiles_n), t_in = t_id % (tiles_m * tiles_n);
  const int band = t_in / (GM * tiles_n), r_in = t_in % (GM * tiles_n);
  const int band_rows = min(GM, tiles_m - band * GM);
  const int tm = band * GM + r_in % band_rows, tn = r_in / band_rows;
  const int m0 = tm * BM, n0 = tn * BN;

  const T* X = static_cast<const T*>(a.X[g]);
  const T* W = static_cast<const T*>(a.W[g]);

  typedef typename LoaderSel<T, BM, NT, X_KMAJ>::type LX;
  typedef typename LoaderSel<T, BN, NT, W_KMAJ>::type LW;
  LX lx[PFX];
  LW lw[PF];

  f32x16 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // ---- main loop ---------------------------------------------------------------------------------------
  // Software pipeline over k-tiles.  While the MFMAs of k-tile t run out of LDS buffer t&1, the register
  // set holding k-tile t+1 is written to the other buffer (first half of the tile's MFMAs) and the global
  // loads of k-tile t+1+PF are issued into that set (second half): with PF = 2 a load has a whole k-tile
  // of MFMAs to arrive.  Inside a k-tile the fragments of MFMA step s+1 are read from LDS while step s
  // computes.  Loads past the end of K return zeros, so the pipeline needs no tail handling.
  const int nk = (a.K + BK - 1) / BK;
  const int lrow = lane & 31, lgrp = lane >> 5;
  lx[0].load(X, a.ldx, m0, a.M, 0, a.K, tid);
  lw[0].load(W, a.ldw, n0, a.N, 0, a.K, tid);
  lx[0].store(lds, tid);
  lw[0].store(lds + BM * 8, tid);
#pragma unroll
  for (int p = 0; p < PFX; ++p) lx[p].load(X, a.ldx, m0, a.M, (1 + p) * BK, a.K, tid);
#pragma unroll
  for (int p = 0; p < PF; ++p) lw[p].load(W, a.ldw, n0, a.N, (1 + p) * BK, a.K, tid);
  __syncthreads();

  constexpr bool FDB = WM * WN <= 4;  // fragment double buffering
  constexpr int NFB = FDB ? 2 : 1;
  uint4 xf[NFB][FM], wf[NFB][FN];
  auto read_frags = [&](const uint4* tx, int s, uint4(&xo)[FM], uint4(&wo)[FN]) {
    const uint4* tw = tx + BM * 8;
    const int kc = 2 * s + lgrp;
#pragma unroll
    for (int i = 0; i < FM; ++i) {
      const int row = (wm * FM + i) * 32 + lrow;
      xo[i] = tx[row * 8 + (kc ^ swz(row))];
    }
#pragma unroll
    for (int j = 0; j < FN; ++j) {
      const int row = (wn * FN + j) * 32 + lrow;
      wo[j] = tw[row * 8 + (kc ^ swz(row))];
    }
  };
  constexpr int NM = FM * FN * (sizeof(T) == 4 ? 4 : 1);  // MFMA instructions per step
  // Row sums of the X operand, sum_k X(m,k): in the weight-gradient layout X is dY, so this is the bias
  // gradient of the layer.  Every lane (row, half) adds up the 16-byte chunks it feeds to the MFMAs anyway,
  // in ascending k (a handful of VALU operations per step, hidden behind the MFMAs); the two halves are added
  // at the end and the tiles of the first tile column store the result.  The order depends on nothing but
  // k, like the GEMM's own sums.
  constexpr bool RS = !X_KMAJ && !W_KMAJ;
  const bool do_rs = RS && a.rowsum[g] != nullptr && tn == 0;  // uniform over the workgroup
  float rs[FM];
#pragma unroll
  for (int i = 0; i < FM; ++i) rs[i] = 0.f;
  if (FDB) read_frags(lds, 0, xf[0], wf[0]);
  for (int kt = 0; kt < nk; kt += PF) {
#pragma unroll
    for (int u = 0; u < PF; ++u) {
      const int t = kt + u;
      if (t < nk) {  // uniform over the workgroup
        const uint4* tx = lds + (t & 1) * STAGE;
        uint4* nx = lds + ((t + 1) & 1) * STAGE;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
          if (FDB && s < 3) read_frags(tx, s + 1, xf[(s + 1) & 1], wf[(s + 1) & 1]);
          if (!FDB) read_frags(tx, s, xf[0], wf[0]);
          if (s == 0) lx[u % PFX].store(nx, tid);
          if (s == 1) lw[u].store(nx + BM * 8, tid);
          if (s == 2) lx[u % PFX].load(X, a.ldx, m0, a.M, (t + 1 + PFX) * BK, a.K, tid);
          if (s == 3) lw[u].load(W, a.ldw, n0, a.N, (t + 1 + PF) * BK, a.K, tid);
#pragma unroll
          for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j) mma<T>(acc[i][j], wf[FDB ? (s & 1) : 0][j], xf[FDB ? (s & 1) : 0][i]);
          if constexpr (RS) {
#pragma unroll
            for (int i = 0; i < FM; ++i) rs[i] = chunk_sum<T>(xf[FDB ? (s & 1) : 0][i], rs[i]);
          }
          // interleave the step's LDS reads and memory operations between its MFMAs
          if (s == 0) sched_interleave<NM, FM + FN, LX::N_STORE, 0x200>();
          if (s == 1) sched_interleave<NM, FM + FN, LW::N_STORE, 0x200>();
          if (s == 2) sched_interleave<NM, FM + FN, LX::N_LOAD, 0x020>();
          if (s == 3) sched_interleave<NM, FDB ? 0 : FM + FN, LW::N_LOAD, 0x020>();
        }
        __syncthreads();
        if (FDB && t + 1 < nk) read_frags(nx, 0, xf[0], wf[0]);
      }
    }
  }
  if (do_rs && wn == 0) {
#pragma unroll
    for (int i = 0; i < FM; ++i) {
      const float total = rs[i] + __shfl_xor(rs[i], 32, 64);  // even chunks + odd chunks
      const int m = m0 + (wm * FM + i) * 32 + lrow;
      if (lgrp == 0 && m < a.M) a.rowsum[g][m] = total;
    }
  }

  // ---- epilogue -----------------------------------------------------------------------------------
  // (the k-loop ended with a barrier: every wave is done with the operand tiles, whose LDS the patches reuse)
  constexpr int SP = FN * 32 + 4;
  static_assert((size_t)WM * WN * 32 * SP * 4 <= 2 * (size_t)STAGE * 16, "epilogue patch exceeds LDS");
  float* patch = reinterpret_cast<float*>(lds) + wave * (32 * SP);
  tile_epilogue<T, FM, FN, UPD>(acc, patch, a, upd, g, m0 + wm * FM * 32, n0 + wn * FN * 32, lane);
}

// ---- bf16: operand tiles go from memory straight into LDS ----------------------------------------------------
//
// The k-loop advances in sub-tiles of 32 k through a ring of NS LDS stages.  Every wave issues its share of a
// sub-tile as wave-wide buffer loads whose destination is LDS (lane l of a load fills the 16-byte slot base + l),
// NS-1 sub-tiles ahead of the one being multiplied, so no operand passes through registers on its way in and a
// load has NS-2 sub-tiles of MFMAs to arrive.  A tile keeps the layout it has in memory:
//  * k-contiguous operand: rows of 64 bytes (four 16-byte chunks); the chunk position inside a row is XOR-ed with
//    ((row>>2)&3)^(row&2).  The lanes pick their global chunk accordingly (a row's four lanes still cover its 64
//    contiguous bytes); a fragment is one 16-byte read per lane and 32-row fragment reads spread over all banks.
//  * operand with k as the slow index: 32 k-rows of ROWS elements (ROWS/8 chunks); the chunk position inside a
//    k-row is XOR-ed with (k&3)<<2.  A fragment is two transposing 8-byte LDS reads (ds_read_b64_tr_b16): within
//    a group of 16 lanes, source lane j supplies four consecutive row elements of k-row j/4 at row offset 4(j%4),
//    and lane i receives element i%4 of source lanes i/4, 4+i/4, 8+i/4, 12+i/4, i.e. four consecutive k for one
//    row.  The XOR puts the four k-rows a half-wave reads into four different 64-byte bank groups.
// One barrier per sub-tile sits between its two MFMA steps: before it a wave has the step-1 fragments of the
// current stage in registers and waits until all but its newest (NS-2) groups of loads have landed; after it the
// step-0 fragments of the next stage are read while step 1 computes.  The sum over k is the same ascending chain of
// 16-wide MFMA steps as in gemm_kernel, with the same k values in every lane, so both kernels give the same bits.
__device__ __forceinline__ int swz4(int row) { return ((row >> 2) & 3) ^ (row & 2); }
// chunk permutation of a 128-byte row (8 chunks): 16 consecutive rows, read at one chunk index, spread over all banks
__device__ __forceinline__ int swz8(int row) { return ((row >> 1) & 3) | (((row & 1) ^ ((row >> 3) & 1)) << 2); }

// 128-bit buffer descriptor (base, stride 0, size in bytes, raw dword format) for bytes [first, total) of a matrix;
// reads beyond it return zero
__device__ __forceinline__ u32x4 rsrc_words(const void* base, long first, long total) {
  long rem = total - first;
  rem = rem < 0 ? 0 : (rem > 0x7fffffffL ? 0x7fffffffL : rem);
  const uint64_t p = (uint64_t)(uintptr_t)base + (uint64_t)(rem > 0 ? first : 0);
  u32x4 r;
  r.x = __builtin_amdgcn_readfirstlane((unsigned)p);
  r.y = __builtin_amdgcn_readfirstlane((unsigned)(p >> 32) & 0xffffu);
  r.z = __builtin_amdgcn_readfirstlane((unsigned)rem);
  r.w = 0x00020000u;
  return r;
}
// One wave-wide load of 16 bytes per lane from a buffer into LDS: lane l's bytes land at lds_addr + 16 l (lds_addr is
// a byte address inside the workgroup's LDS, uniform over the wave).  The compiler does not see the LDS write:
// callers order it against LDS reads with an explicit vmcnt wait and a barrier.
__device__ __forceinline__ void load_to_lds_b128(u32x4 rs, unsigned lds_addr, unsigned voff) {
  asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds" ::"s"(lds_addr), "v"(voff), "s"(rs) : "m0");
}

// One operand tile of ROWS rows in the ring: what a lane contributes to the direct loads of a sub-tile and where it
// reads its MFMA fragments.  NW = waves of the workgroup; load i of wave w fills slots [(i*NW + w)*64, +64).
// BKW = k per sub-tile: 32, or 64 (a k-contiguous row is then 128 contiguous bytes per load: whole cache lines).
template <bool KMAJ, int ROWS, int NW, int BKW = 32>
struct RingOperand {
  static constexpr int CPR = BKW / 8;                 // 16-byte chunks per k-contiguous row
  static constexpr int NLD = ROWS * CPR / 64 / NW;    // loads per wave and sub-tile (a sub-tile is ROWS*CPR slots either way)
  static_assert(ROWS * CPR % (64 * NW) == 0, "tile rows must divide over the waves");
  static_assert(BKW == 32 || BKW == 64, "sub-tile depth");
  static __device__ __forceinline__ int swz(int row) { return BKW == 32 ? swz4(row) : swz8(row); }
  u32x4 rs;
  unsigned voff[NLD];   // byte offset of the lane's chunk in sub-tile 0, relative to the descriptor's base
  int kofs[NLD];        // k (inside a sub-tile) of the lane's chunk: a chunk at or past K is loaded as zeros
  unsigned step;        // bytes from one sub-tile to the next
  // base/ld/row0/nrows: the matrix, its leading dimension, the tile's first row and the matrix's row count
  __device__ __forceinline__ void init(const bf16_t* base, int ld, int row0, int nrows, int K, int wave, int lane) {
    if (KMAJ) {
      rs = rsrc_words(base, (long)row0 * ld * 2, (long)nrows * ld * 2);  // rows past the matrix read as zero
      step = 2u * BKW;
    } else {
      rs = rsrc_words(base, (long)row0 * 2, (long)K * ld * 2);           // k-rows past K read as zero
      step = 2u * BKW * (unsigned)ld;
    }
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int sl = (i * NW + wave) * 64 + lane;
      if (KMAJ) {
        const int row = sl / CPR;
        kofs[i] = ((sl % CPR) ^ swz(row)) * 8;
        voff[i] = ((unsigned)row * (unsigned)ld + (unsigned)kofs[i]) * 2u;
      } else {
        const int k = sl / (ROWS / 8), rc = (sl % (ROWS / 8)) ^ ((k & 3) << 2);
        kofs[i] = k;
        voff[i] = ((unsigned)k * (unsigned)ld + (unsigned)rc * 8u) * 2u;
      }
    }
  }
  // nd-th load of sub-tile t into the operand's part of a stage at LDS byte address st
  __device__ __forceinline__ void issue(int nd, int t, unsigned st, int K, int wave) const {
    const int i = nd < NLD ? nd : 0;
    load_to_lds_b128(rs, st + (unsigned)((i * NW + wave) * 64 * 16), t * BKW + kofs[i] < K ? voff[i] + (unsigned)t * step : 0xfffffff0u);
  }
  // byte offset inside the operand's part of a stage of the lane's fragment of rows [rowbase, rowbase+32) for MFMA step
  // mfma_step of the sub-tile (k-contiguous: every step has its own offset because of the XOR; k-slow: 16 k-rows each)
  static __device__ __forceinline__ int frag_offset(int rowbase, int lane, int mfma_step) {
    if (KMAJ) {
      const int row = rowbase + (lane & 31);
      return (row * CPR + ((2 * mfma_step + (lane >> 5)) ^ swz(row))) * 16;
    }
    const int j = lane & 15, grp = lane >> 4, k = 16 * mfma_step + 8 * (grp >> 1) + (j >> 2);
    const int rc = rowbase / 8 + 2 * (grp & 1) + ((j & 3) >> 1);
    return (k * (ROWS / 8) + (rc ^ ((k & 3) << 2))) * 16 + (j & 1) * 8;
  }
  static __device__ __forceinline__ uint4 read_frag(const char* stage_part, int off) {
    if (KMAJ) return *reinterpret_cast<const uint4*>(stage_part + off);
    typedef __attribute__((ext_vector_type(4))) short s16x4;
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    const unsigned a0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) const char*)(stage_part + off);
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(uintptr_t)a0);
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(uintptr_t)(a0 + 4u * (ROWS / 8) * 16u));  // k + 4
    uint2 l = __builtin_bit_cast(uint2, lo), h = __builtin_bit_cast(uint2, hi);
    return make_uint4(l.x, l.y, h.x, h.y);
  }
};

// SPLITK: the grid holds a.split_k copies of every tile; copy sp sums the sp-th contiguous range of sub-tiles and
// stores its fp32 partial tile at element offset sp*M*ldo of out (row sums at sp*M); splitk_finish_kernel adds them.
// BK = 64 (with NS = 2): sub-tiles of 64 k, so that a load of a k-contiguous operand covers 128 contiguous bytes per
// row; one barrier per sub-tile, before its last MFMA step, and the loads of sub-tile t+2 follow that barrier.
template <int WM, int WN, int FM, int FN, int NS, bool X_KMAJ, bool W_KMAJ, bool UPD, bool SPLITK = false, int BK = 32>
__global__ __launch_bounds__(WM* WN * 64) void gemm_dma_kernel(const GemmArgs a, const typename UpdSel<UPD>::type upd) {
  static_assert(!SPLITK || !UPD, "partial sums are stored plainly");
  static_assert(BK == 32 || (BK == 64 && NS == 2), "ring shape");
  typedef bf16_t T;
  constexpr int BM = WM * FM * 32, BN = WN * FN * 32, NW = WM * WN;
  constexpr int XPART = BM * (BK / 8) * 16;          // bytes of the X part of a stage
  constexpr int STAGE = (BM + BN) * (BK / 8) * 16;   // bytes per stage: X part, then W part
  typedef RingOperand<X_KMAJ, BM, NW, BK> RX;
  typedef RingOperand<W_KMAJ, BN, NW, BK> RW;
  constexpr int NL = RX::NLD + RW::NLD;
  extern __shared__ uint4 lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WN, wn = wave % WN;

  const int tiles_m = (a.M + BM - 1) / BM, tiles_n = (a.N + BN - 1) / BN;
  const int n_tiles = tiles_m * tiles_n * a.G;
  const int n_work = SPLITK ? n_tiles * a.split_k : n_tiles;
  const int per_xcd = (n_work + 7) >> 3;
  const int w_id = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (w_id >= n_work) return;
  const int sp = SPLITK ? w_id / n_tiles : 0, t_id = SPLITK ? w_id % n_tiles : w_id;  // neighbouring ids: same k range
  constexpr int GM = 8;  // tile order as in gemm_kernel: contiguous runs per XCD, bands of GM tile rows
  const int g = t_id / (tiles_m * tiles_n), t_in = t_id % (tiles_m * tiles_n);
  const int band = t_in / (GM * tiles_n), r_in = t_in % (GM * tiles_n);
  const int band_rows = min(GM, tiles_m - band * GM);
  const int tm = band * GM + r_in % band_rows, tn = r_in / band_rows;
  const int m0 = tm * BM, n0 = tn * BN;
  const int K = a.K;

  RX ox_;
  RW ow_;
  ox_.init(static_cast<const T*>(a.X[g]), a.ldx, m0, a.M, K, wave, lane);
  ow_.init(static_cast<const T*>(a.W[g]), a.ldw, n0, a.N, K, wave, lane);
  const char* lds_c = reinterpret_cast<const char*>(lds);
  const unsigned lds_base = (unsigned)(uintptr_t)(__attribute__((address_space(3))) void*)lds;
  // this workgroup's range of sub-tiles
  const int nk_all = (K + BK - 1) / BK;
  const int nk_per = SPLITK ? (nk_all + a.split_k - 1) / a.split_k : nk_all;
  const int kb = sp * nk_per;
  const int nk = max(0, min(nk_all, kb + nk_per) - kb);
  const int K_end = min(K, (kb + nk) * BK);  // chunks at or past it load as zeros
  auto load_one = [&](int t, int nd) {  // nd-th direct load of the range's sub-tile t
    const unsigned st = lds_base + (unsigned)((t % NS) * STAGE);
    if (nd < RX::NLD) ox_.issue(nd, kb + t, st, K_end, wave);
    else ow_.issue(nd - RX::NLD, kb + t, st + (unsigned)XPART, K_end, wave);
  };

  f32x16 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  const int lrow = lane & 31, lgrp = lane >> 5;
  constexpr int NSTEP = BK / 16;   // MFMA steps per sub-tile
  int fx[NSTEP][FM], fw[NSTEP][FN];  // fragment byte offsets inside a stage per MFMA step
#pragma unroll
  for (int s = 0; s < NSTEP; ++s) {
#pragma unroll
    for (int i = 0; i < FM; ++i) fx[s][i] = RX::frag_offset((wm * FM + i) * 32, lane, s);
#pragma unroll
    for (int j = 0; j < FN; ++j) fw[s][j] = XPART + RW::frag_offset((wn * FN + j) * 32, lane, s);
  }
  // loads of this wave that may still be in flight when the next sub-tile must have landed (BK = 64: none, the loads
  // of the sub-tile after it are issued behind the barrier); in the prologue sub-tile 0 must have landed
  constexpr int ALLOW = BK == 32 ? (NS - 2) * NL : 0;
  constexpr int ALLOW0 = BK == 32 ? ALLOW : NL;
  static_assert(ALLOW < 64 && ALLOW0 < 64, "vmcnt field");
  constexpr int WAIT_VM = (ALLOW & 15) | ((ALLOW >> 4) << 14) | (7 << 4);  // s_waitcnt vmcnt(ALLOW) lgkmcnt(0)
  constexpr int WAIT_VM0 = (ALLOW0 & 15) | ((ALLOW0 >> 4) << 14) | (7 << 4) | (15 << 8);  // vmcnt(ALLOW0) only
#pragma unroll
  for (int t = 0; t < (BK == 32 ? NS - 1 : 2); ++t)
#pragma unroll
    for (int nd = 0; nd < NL; ++nd) load_one(t, nd);
  __builtin_amdgcn_s_waitcnt(WAIT_VM0);
  __builtin_amdgcn_s_barrier();
  uint4 xa[FM], wa[FN], xb[FM], wb[FN];
#pragma unroll
  for (int i = 0; i < FM; ++i) xa[i] = RX::read_frag(lds_c, fx[0][i]);
#pragma unroll
  for (int j = 0; j < FN; ++j) wa[j] = RW::read_frag(lds_c, fw[0][j]);
  // Row sums of the X operand (the bias gradient when X = dY), as in gemm_kernel: every lane adds up the chunks it
  // feeds to the MFMAs, in ascending k
  constexpr bool RS = !X_KMAJ && !W_KMAJ;
  const bool do_rs = RS && a.rowsum[g] != nullptr && tn == 0;
  float rs[FM];
#pragma unroll
  for (int i = 0; i < FM; ++i) rs[i] = 0.f;
  // One MFMA step on the fragments (xc, wc) while the fragments of the following step are read from stage sn into
  // (xn, wn) and, with tl >= 0, the loads of sub-tile tl are issued; the order is pinned so that LDS reads and
  // loads sit between the MFMAs that hide them.
  auto step = [&](uint4(&xc)[FM], uint4(&wc)[FN], uint4(&xn)[FM], uint4(&wn_)[FN], const char* sn, int s, int tl) {
    int nr = 0, nd = 0;
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
      for (int j = 0; j < FN; ++j) {
        const int q = i * FN + j;
        if (tl >= 0 && nd < NL && nd * (FM * FN) <= q * NL) {
          load_one(tl, nd);
          ++nd;
        }
        if (nr < FM + FN) {
          if (nr < FM) xn[nr] = RX::read_frag(sn, fx[s][nr]);
          else wn_[nr - FM] = RW::read_frag(sn, fw[s][nr - FM]);
          ++nr;
        }
        mma<T>(acc[i][j], wc[j], xc[i]);
        if (RS && j == 0) rs[i] = chunk_sum<T>(xc[i], rs[i]);
        __builtin_amdgcn_sched_barrier(0);
      }
  };
  for (int t = 0; t < nk; ++t) {
    const char* st = lds_c + (t % NS) * STAGE;
    const char* sn = lds_c + ((t + 1) % NS) * STAGE;
    if constexpr (BK == 32) {
      step(xa, wa, xb, wb, st, 1, t + NS - 1);
      __builtin_amdgcn_s_waitcnt(WAIT_VM);
      __builtin_amdgcn_s_barrier();
      step(xb, wb, xa, wa, sn, 0, -1);
    } else {
      step(xa, wa, xb, wb, st, 1, -1);
      step(xb, wb, xa, wa, st, 2, -1);
      step(xa, wa, xb, wb, st, 3, -1);
      __builtin_amdgcn_s_waitcnt(WAIT_VM);  // sub-tile t+1 (issued one sub-tile ago) has landed; own reads of stage t are done
      __builtin_amdgcn_s_barrier();
      step(xb, wb, xa, wa, sn, 0, t + 2);    // stage t is free: sub-tile t+2 goes there
    }
  }
  if (do_rs && wn == 0) {
#pragma unroll
    for (int i = 0; i < FM; ++i) {
      const float total = rs[i] + __shfl_xor(rs[i], 32, 64);  // even chunks + odd chunks
      const int m = m0 + (wm * FM + i) * 32 + lrow;
      if (lgrp == 0 && m < a.M) a.rowsum[g][(size_t)sp * a.M + m] = total;
    }
  }
  // the trailing (all-zero) loads must have landed and every wave must be done with the ring before patches reuse it
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();
  constexpr int SP = FN * 32 + 4;
  static_assert((size_t)NW * 32 * SP * 4 <= (size_t)NS * STAGE, "epilogue patch exceeds LDS");
  float* patch = reinterpret_cast<float*>(lds) + wave * (32 * SP);
  constexpr int SPEC = SPLITK ? -1 : (UPD || FM != 4 || FN != 2 || !X_KMAJ) ? 0 : (W_KMAJ ? 1 : 2);
  tile_epilogue<T, FM, FN, UPD, SPEC>(acc, patch, a, upd, g, m0 + wm * FM * 32, n0 + wn * FN * 32, lane,
                                      SPLITK ? (size_t)sp * a.M * a.ldo : 0);
}

// Second launch of a split weight gradient: element (m, n) of problem g = the S partial sums added in ascending
// order, then stored (fp32) and/or fed to the parameter update exactly as the one-launch epilogue would.
struct SplitFinishArgs {
  int M, N, ldo, S, G, opt, upd;
  const float* ws[MAXG];      // [S][M][ldo] partial sums, then [S][M] partial row sums
  float* out[MAXG];           // nullable
  float* rowsum[MAXG];        // nullable
  float* p[MAXG];
  float* m[MAXG];
  float* v[MAXG];
  bf16_t* w16[MAXG];
  OptimHp hp[MAXG];
};
// A thread takes 4 consecutive columns, so that every 16-byte access of a wave covers contiguous memory; the S
// partial sums are all requested before the first is used and added in ascending order of s.
constexpr int SPLIT_MAX = 8;
// MODE: 0 = store the sums, 1 = SGD, 2 = Adam (then `out` also receives the sums when it is given).  A wave takes 64
// consecutive 16-byte pieces of a row, a workgroup four rows at a time: no index division, and the problem's pointers
// are read from the argument block once.
template <int MODE>
__global__ __launch_bounds__(256) void splitk_finish_kernel(const SplitFinishArgs a) {
  const int g = blockIdx.y;
  const size_t plane = (size_t)a.M * a.ldo;
  const int n4 = a.N / 4;  // N is a multiple of 8
  const int S = a.S;
  const float* const WS = a.ws[g];
  float* const P = a.p[g];
  float* const Mo = a.m[g];
  float* const Vo = a.v[g];
  bf16_t* const W16 = a.w16[g];
  float* const OUT = a.out[g];
  const OptimHp h = a.hp[g];
  const int lx = threadIdx.x & 63, ly = threadIdx.x >> 6;
  for (int m = blockIdx.x * 4 + ly; m < a.M; m += gridDim.x * 4) {
    for (int c = lx; c < n4; c += 64) {
      const size_t idx = (size_t)m * a.ldo + 4 * c;
      f32x4 part[SPLIT_MAX];
#pragma unroll
      for (int s = 0; s < SPLIT_MAX; ++s)
        if (s < S) part[s] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(WS + (size_t)s * plane + idx));
      f32x4 pv, mv, vv;
      if (MODE >= 1) pv = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(P + idx));
      if (MODE == 2) {
        mv = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(Mo + idx));
        vv = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(Vo + idx));
      }
      float v[4] = {part[0].x, part[0].y, part[0].z, part[0].w};
#pragma unroll
      for (int s = 1; s < SPLIT_MAX; ++s)
        if (s < S) {
          v[0] += part[s].x; v[1] += part[s].y; v[2] += part[s].z; v[3] += part[s].w;
        }
      if (MODE >= 1) {
        float pe[4] = {pv.x, pv.y, pv.z, pv.w}, me[4] = {0.f, 0.f, 0.f, 0.f}, ve[4] = {0.f, 0.f, 0.f, 0.f};
        if (MODE == 2) {
          me[0] = mv.x; me[1] = mv.y; me[2] = mv.z; me[3] = mv.w;
          ve[0] = vv.x; ve[1] = vv.y; ve[2] = vv.z; ve[3] = vv.w;
#pragma unroll
          for (int e = 0; e < 4; ++e) optim_step<1>(pe[e], me[e], ve[e], v[e], h);
          const f32x4 mo = {me[0], me[1], me[2], me[3]}, vo = {ve[0], ve[1], ve[2], ve[3]};
          __builtin_nontemporal_store(mo, reinterpret_cast<f32x4*>(Mo + idx));
          __builtin_nontemporal_store(vo, reinterpret_cast<f32x4*>(Vo + idx));
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e) optim_step<0>(pe[e], me[e], ve[e], v[e], h);
        }
        const f32x4 po = {pe[0], pe[1], pe[2], pe[3]};
        __builtin_nontemporal_store(po, reinterpret_cast<f32x4*>(P + idx));
        if (W16) *reinterpret_cast<uint2*>(W16 + idx) = make_uint2(pack_bf16x2(pe[0], pe[1]), pack_bf16x2(pe[2], pe[3]));
      }
      if (OUT) *reinterpret_cast<float4*>(OUT + idx) = make_float4(v[0], v[1], v[2], v[3]);
    }
  }
  if (a.rowsum[g] && blockIdx.x == 0) {
    const float* rs = a.ws[g] + (size_t)a.S * plane;
    for (int m = threadIdx.x; m < a.M; m += 256) {
      float t = rs[m];
      for (int s = 1; s < a.S; ++s) t += rs[(size_t)s * a.M + m];
      a.rowsum[g][m] = t;
    }
  }
}

struct DmaBig {  // 256 x 256, 8 waves (2 x 4, each 128 x 64), ring of 4 stages of 32 KB (or 2 of 64 KB)
  static constexpr int WM = 2, WN = 4, FM = 4, FN = 2, NS = 4;
  static constexpr int BM = WM * FM * 32, BN = WN * FN * 32, NT = WM * WN * 64;
  static constexpr size_t LDS = (size_t)NS * (BM + BN) * 4 * 16;
  static int grid_of(const GemmArgs& a) {
    int tiles = ((a.M + BM - 1) / BM) * ((a.N + BN - 1) / BN) * a.G;
    return ((tiles + 7) / 8) * 8;
  }
  // with both operands k-contiguous (forward) the ring is two stages of 64 k (same LDS bytes): measured 3-7 % faster;
  // with one of them k-slow (its rows are 512 contiguous bytes already) the deeper ring of 32 k is level or better
  template <bool XK, bool WK>
  static hipError_t run1(const GemmArgs& a, hipStream_t s) {
    if constexpr (XK && WK)
      hipLaunchKernelGGL((gemm_dma_kernel<WM, WN, FM, FN, 2, XK, WK, false, false, 64>), dim3(grid_of(a)), dim3(NT), LDS, s, a, NoUpdate());
    else
      hipLaunchKernelGGL((gemm_dma_kernel<WM, WN, FM, FN, NS, XK, WK, false>), dim3(grid_of(a)), dim3(NT), LDS, s, a, NoUpdate());
    return hipGetLastError();
  }
  static hipError_t run(const GemmArgs& a, hipStream_t s) {
    if (a.x_kmajor) return a.w_kmajor ? run1<true, true>(a, s) : run1<true, false>(a, s);
    return a.w_kmajor ? run1<false, true>(a, s) : run1<false, false>(a, s);
  }
  static hipError_t run_update(const GemmArgs& a, const GemmUpdate& u, hipStream_t s) {
    hipLaunchKernelGGL((gemm_dma_kernel<WM, WN, FM, FN, NS, false, false, true>), dim3(grid_of(a)), dim3(NT), LDS, s, a, u);
    return hipGetLastError();
  }
  static hipError_t run_split(const GemmArgs& a, hipStream_t s) {
    hipLaunchKernelGGL((gemm_dma_kernel<WM, WN, FM, FN, NS, false, false, false, true>), dim3(grid_of(a) * a.split_k), dim3(NT), LDS,
                       s, a, NoUpdate());
    return hipGetLastError();
  }
  template <bool XK, bool WK, bool UPD>
  static hipError_t attr1() {
    if constexpr (XK && WK && !UPD)
      return hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_dma_kernel<WM, WN, FM, FN, 2, XK, WK, false, false, 64>),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS);
    else
      return hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_dma_kernel<WM, WN, FM, FN, NS, XK, WK, UPD>),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS);
  }
  static hipError_t attr() {
    hipError_t e;
    if ((e = attr1<true, true, false>()) != hipSuccess) return e;
    if ((e = attr1<true, false, false>()) != hipSuccess) return e;
    if ((e = attr1<false, true, false>()) != hipSuccess) return e;
    if ((e = attr1<false, false, false>()) != hipSuccess) return e;
    if ((e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_dma_kernel<WM, WN, FM, FN, NS, false, false, false, true>),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS)) != hipSuccess)
      return e;
    return attr1<false, false, true>();
  }
};
// Measured against the register-staged 128 x 128 tile on one model's 8192-token products (d = 1024): forward 8-11 %
// faster, input gradient 21-31 %, weight gradient 23-46 %; with the update in the epilogue (8 x [4096 x 4096], 512
// tokens) 720 -> 663 us per launch.
struct DmaMid {  // 128 x 128, 4 waves (2 x 2, each 64 x 64), ring of 4 stages of 16 KB: two workgroups per CU
  static constexpr int WM = 2, WN = 2, FM = 2, FN = 2, NS = 4;
  static constexpr int BM = WM * FM * 32, BN = WN * FN * 32, NT = WM * WN * 64;
  static constexpr size_t LDS = (size_t)NS * (BM + BN) * 4 * 16;
  template <bool XK, bool WK>
  static hipError_t run1(const GemmArgs& a, hipStream_t s) {
    const int tiles = ((a.M + BM - 1) / BM) * ((a.N + BN - 1) / BN) * a.G;
    hipLaunchKernelGGL((gemm_dma_kernel<WM, WN, FM, FN, NS, XK, WK, false>), dim3((tiles + 7) / 8 * 8), dim3(NT), LDS, s, a, NoUpdate());
    return hipGetLastError();
  }
  static hipError_t run(const GemmArgs& a, hipStream_t s) {
    if (a.x_kmajor) return a.w_kmajor ? run1<true, true>(a, s) : run1<true, false>(a, s);
    return a.w_kmajor ? run1<false, true>(a, s) : run1<false, false>(a, s);
  }
  static hipError_t run_update(const GemmArgs& a, const GemmUpdate& u, hipStream_t s) {
    const int tiles = ((a.M + BM - 1) / BM) * ((a.N + BN - 1) / BN) * a.G;
    hipLaunchKernelGGL((gemm_dma_kernel<WM, WN, FM, FN, NS, false, false, true>), dim3((tiles + 7) / 8 * 8), dim3(NT), LDS, s, a, u);
    return hipGetLastError();
  }
  template <bool XK, bool WK>
  static hipError_t attr1() {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_dma_kernel<WM, WN, FM, FN, NS, XK, WK, false>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS);
  }
  static hipError_t attr() {
    hipError_t e;
    if ((e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_dma_kernel<WM, WN, FM, FN, NS, false, false, true>),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS)) != hipSuccess)
      return e;
    if ((e = attr1<true, true>()) != hipSuccess) return e;
    if ((e = attr1<true, false>()) != hipSuccess) return e;
    if ((e = attr1<false, true>()) != hipSuccess) return e;
    return attr1<false, false>();
  }
};
// The direct-to-LDS kernel takes bf16 problems.  A k-contiguous operand needs K to be a multiple of 8 (a 16-byte
// chunk is then entirely inside or outside the matrix); an operand with k as the slow index is addressed from the
// tile's first element with 32-bit offsets, so its K x ld bytes must stay below 2 GiB.
inline bool dma_eligible(const GemmArgs& a) {
  if (a.dtype != GEMM_BF16) return false;
  if ((a.x_kmajor || a.w_kmajor) && a.K % 8 != 0) return false;
  if (!a.x_kmajor && (long)a.K * a.ldx * 2 >= 0x7fffffffL) return false;
  if (!a.w_kmajor && (long)a.K * a.ldw * 2 >= 0x7fffffffL) return false;
  return true;
}

template <typename T, int WM, int WN, int FM, int FN, int PFX, int PF>
struct Cfg {
  static constexpr int BM = WM * FM * 32, BN = WN * FN * 32, NT = WM * WN * 64;
  static constexpr size_t LDS = 2 * (size_t)(BM + BN) * 8 * 16;
  template <bool XK, bool WK>
  static hipError_t run1(const GemmArgs& a, hipStream_t s) {
    int tiles = ((a.M + BM - 1) / BM) * ((a.N + BN - 1) / BN) * a.G;
    int grid = ((tiles + 7) / 8) * 8;
    hipLaunchKernelGGL((gemm_kernel<T, WM, WN, FM, FN, PFX, PF, XK, WK, false>), dim3(grid), dim3(NT), LDS, s, a, NoUpdate());
    return hipGetLastError();
  }
  static hipError_t run_update(const GemmArgs& a, const GemmUpdate& u, hipStream_t s) {
    int tiles = ((a.M + BM - 1) / BM) * ((a.N + BN - 1) / BN) * a.G;
    int grid = ((tiles + 7) / 8) * 8;
    hipLaunchKernelGGL((gemm_kernel<T, WM, WN, FM, FN, PFX, PF, false, false, true>), dim3(grid), dim3(NT), LDS, s, a, u);
    return hipGetLastError();
  }
  static hipError_t run(const GemmArgs& a, hipStream_t s) {
    if (a.x_kmajor) return a.w_kmajor ? run1<true, true>(a, s) : run1<true, false>(a, s);
    return a.w_kmajor ? run1<false, true>(a, s) : run1<false, false>(a, s);
  }
  template <bool XK, bool WK>
  static hipError_t attr1() {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_kernel<T, WM, WN, FM, FN, PFX, PF, XK, WK, false>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS);
  }
  static hipError_t attr() {
    hipError_t e;
    if ((e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_kernel<T, WM, WN, FM, FN, PFX, PF, false, false, true>),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS)) != hipSuccess)
      return e;
    if ((e = attr1<true, true>()) != hipSuccess) return e;
    if ((e = attr1<true, false>()) != hipSuccess) return e;
    if ((e = attr1<false, true>()) != hipSuccess) return e;
    return attr1<false, false>();
  }
};

template <typename T> struct Tiles {
  // 256 x 256 with 8 waves (2 x 4, each 128 x 64): two waves per SIMD, so one wave's MFMAs run while the
  // other waits for its loads, LDS reads or the barrier.  (A 4-wave 256 x 256 tile with 4 x 4 accumulators
  // per wave reads less LDS per MFMA but leaves every wait exposed: measured 8-30 % slower.)
  typedef Cfg<T, 2, 4, 4, 2, 1, 1> Big;
  typedef Cfg<T, 2, 2, 2, 2, 2, 2> Mid;    // 128 x 128, two k-tiles in flight, two workgroups per CU
  typedef Cfg<T, 1, 4, 1, 1, 1, 1> Small;  // 32 x 128
};

// A weight gradient whose output has few 256x256 tiles leaves most of the device idle while its sum over k is long.
// The split depends on the shape alone (never on the group), so it cannot make a result depend on the schedule.
int split_of(int M, int N, int K) {
  const long tiles = (long)((M + 255) / 256) * ((N + 255) / 256);
  if (tiles >= 64 || N % 8) return 1;
  // about half the device's compute units for one problem: a group of a few models then fills it, and the partial
  // sums (S fp32 copies of the gradient, written and read once) stay a small part of the traffic
  long s = std::min<long>(8, 128 / tiles);
  s = std::min<long>(s, K / 1024);  // at least 1024 k per range
  return s < 2 ? 1 : (int)s;
}

// the two launches of a split problem; u = nullptr: plain store
hipError_t run_split(const GemmArgs& a, const GemmUpdate* u, int S, hipStream_t s) {
  GemmArgs b = a;
  SplitFinishArgs f{};
  if (S > SPLIT_MAX) return hipErrorInvalidValue;
  f.M = a.M; f.N = a.N; f.ldo = a.ldo; f.S = S; f.G = a.G; f.upd = u != nullptr; f.opt = u ? u->opt : 0;
  const size_t plane = (size_t)a.M * a.ldo;
  for (int g = 0; g < a.G; ++g) {
    float* ws = static_cast<float*>(a.ws[g]);
    b.out[g] = ws;
    b.rowsum[g] = a.rowsum[g] ? ws + (size_t)S * plane : nullptr;
    f.ws[g] = ws;
    f.out[g] = static_cast<float*>(a.out[g]);
    f.rowsum[g] = a.rowsum[g];
    if (u) { f.p[g] = u->p[g]; f.m[g] = u->m[g]; f.v[g] = u->v[g]; f.w16[g] = u->w16[g]; f.hp[g] = u->hp[g]; }
  }
  b.out_f32 = 1;
  b.split_k = S;
  hipError_t e = DmaBig::run_split(b, s);
  if (e != hipSuccess) return e;
  // a workgroup takes four rows at a time; enough workgroups to fill the device several times over
  const unsigned bx = (unsigned)std::min<size_t>(((size_t)a.M + 3) / 4, 4096);
  if (!u) hipLaunchKernelGGL(splitk_finish_kernel<0>, dim3(bx, a.G), dim3(256), 0, s, f);
  else if (u->opt == 1) hipLaunchKernelGGL(splitk_finish_kernel<2>, dim3(bx, a.G), dim3(256), 0, s, f);
  else hipLaunchKernelGGL(splitk_finish_kernel<1>, dim3(bx, a.G), dim3(256), 0, s, f);
  return hipGetLastError();
}

// S > 1 when the problem is to be split: weight-gradient layout, bf16, plain fp32 output (or the update), scratch given
int split_for(const GemmArgs& a) {
  if (!a.ws[0] || a.dtype != GEMM_BF16 || a.x_kmajor || a.w_kmajor || !a.out_f32 || !dma_eligible(a)) return 1;
  if (a.bias[0] || a.pre[0] || a.gate[0] || a.resid[0] || a.mul[0] || a.act != EPI_ACT_NONE) return 1;
  const int S = split_of(a.M, a.N, a.K);
  if (S > 1 && a.ws_bytes < ((size_t)S * a.M * a.ldo + (size_t)S * a.M) * 4) return 1;
  return S;
}

int choose_tile(const GemmArgs& a) {
  if (a.tile) return a.tile;
  auto tiles = [&](int bm, int bn) { return (long)((a.M + bm - 1) / bm) * ((a.N + bn - 1) / bn) * a.G; };
  const long big = tiles(256, 256), mid = tiles(128, 128);
  if (a.M >= 192 && big >= 192) return 1;  // the big tile fills the chip
  if (a.M >= 96 && mid >= 64) {
    // Too few big tiles for 256 CUs: 128 x 128 tiles win while they fit in one pass over the chip (two
    // workgroups per CU); beyond that a partly filled pass of big tiles is still the faster choice.
    return (a.M >= 192 && big >= 128 && mid > 512) ? 1 : 2;
  }
  return 3;
}

template <typename T>
hipError_t dispatch_update(const GemmArgs& a, const GemmUpdate& u, hipStream_t s) {
  if (const int S = split_for(a); S > 1) return run_split(a, &u, S, s);
  int tile = choose_tile(a);
  // With a short k-loop the state traffic of the epilogue dominates: with two workgroups per CU one streams
  // state while the other runs its k-loop, which the 256x256 tile (one workgroup per CU) cannot do.
  if (!a.tile && tile == 1 && a.K < 2048) tile = 2;
  if (tile == 1 && dma_eligible(a)) return DmaBig::run_update(a, u, s);
  if (tile == 2 && dma_eligible(a)) return DmaMid::run_update(a, u, s);
  switch (tile) {
    case 1:
    case 4: return Tiles<T>::Big::run_update(a, u, s);
    case 2: return Tiles<T>::Mid::run_update(a, u, s);
    case 3: return Tiles<T>::Small::run_update(a, u, s);
  }
  return hipErrorInvalidValue;
}

template <typename T>
hipError_t dispatch(const GemmArgs& a, hipStream_t s) {
  if (const int S = split_for(a); S > 1) return run_split(a, nullptr, S, s);
  const int tile = choose_tile(a);
  if (tile == 1 && dma_eligible(a)) return DmaBig::run(a, s);
  if (tile == 2 && dma_eligible(a)) return DmaMid::run(a, s);
  switch (tile) {
    case 1:
    case 4: return Tiles<T>::Big::run(a, s);
    case 2: return Tiles<T>::Mid::run(a, s);
    case 3: return Tiles<T>::Small::run(a, s);
  }
  return hipErrorInvalidValue;
}

template <typename T>
hipError_t init_tiles() {
  hipError_t e;
  if ((e = Tiles<T>::Big::attr()) != hipSuccess) return e;
  if ((e = Tiles<T>::Mid::attr()) != hipSuccess) return e;
  return Tiles<T>::Small::attr();
}

}  // namespace

hipError_t gemm_init() {
  hipError_t e = DmaBig::attr();
  if (e != hipSuccess) return e;
  if ((e = DmaMid::attr()) != hipSuccess) return e;
  e = init_tiles<bf16_t>();
  return e != hipSuccess ? e : init_tiles<float>();
}

hipError_t kernels_init() {
  hipError_t e;
  if ((e = gemm_init()) != hipSuccess) return e;
  if ((e = ln_init()) != hipSuccess) return e;
  return attn_init();
}

static hipError_t check_gemm(const GemmArgs& a, bool need_out) {
  const int E = a.dtype == GEMM_F32 ? 4 : 8;
  auto rup = [&](int v) { return (v + E - 1) / E * E; };
  if (a.G < 1 || a.G > MAXG || a.M < 1 || a.N < 1 || a.K < 1) return hipErrorInvalidValue;
  if (a.ldx % E || a.ldw % E) return hipErrorInvalidValue;
  if (a.ldx < rup(a.x_kmajor ? a.K : a.M) || a.ldw < rup(a.w_kmajor ? a.K : a.N)) return hipErrorInvalidValue;
  if (a.ldo < a.N) return hipErrorInvalidValue;
  // the epilogue moves 8 consecutive outputs as 16/32-byte vectors
  if (a.ldo % 8 || (a.gate[0] && a.ldg % 8) || (a.resid[0] && a.ldr % 8)) return hipErrorInvalidValue;
  for (int g = 0; g < a.G; ++g) {
    if (!a.X[g] || !a.W[g] || (need_out && !a.out[g])) return hipErrorInvalidValue;
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
  for (int g = 0; g < a.G; ++g)
    if ((a.rowsum[g] == nullptr) != (a.rowsum[0] == nullptr) || (a.ws[g] == nullptr) != (a.ws[0] == nullptr) ||
        ((uintptr_t)a.ws[g] & 31))
      return hipErrorInvalidValue;
  if (a.rowsum[0] && (a.x_kmajor || a.w_kmajor)) return hipErrorInvalidValue;
  return hipSuccess;
}

int gemm_split_k(int M, int N, int K) { return split_of(M, N, K); }
size_t gemm_split_ws_bytes(int M, int N, int K, int ldo) {
  const int S = split_of(M, N, K);
  return S > 1 ? ((size_t)S * M * ldo + (size_t)S * M) * 4 : 0;
}

hipError_t launch_gemm(const GemmArgs& a, hipStream_t s) {
  hipError_t e = check_gemm(a, true);
  if (e != hipSuccess) return e;
  return a.dtype == GEMM_F32 ? dispatch<float>(a, s) : dispatch<bf16_t>(a, s);
}

hipError_t launch_gemm_update(const GemmArgs& a, const GemmUpdate& u, hipStream_t s) {
  hipError_t e = check_gemm(a, false);
  if (e != hipSuccess) return e;
  if (a.x_kmajor || a.w_kmajor || !a.out_f32 || a.act != EPI_ACT_NONE) return hipErrorInvalidValue;
  if (a.bias[0] || a.pre[0] || a.gate[0] || a.resid[0] || a.mul[0]) return hipErrorInvalidValue;
  if (u.opt != 0 && u.opt != 1 || a.N % 8) return hipErrorInvalidValue;
  for (int g = 0; g < a.G; ++g) {
    if (!u.p[g] || (u.opt == 1 && (!u.m[g] || !u.v[g]))) return hipErrorInvalidValue;
    if ((u.w16[g] == nullptr) != (u.w16[0] == nullptr) || (a.out[g] == nullptr) != (a.out[0] == nullptr))
      return hipErrorInvalidValue;
    if (((uintptr_t)u.p[g] | (uintptr_t)u.m[g] | (uintptr_t)u.v[g]) & 31 || ((uintptr_t)u.w16[g] & 15) ||
        ((uintptr_t)a.out[g] & 31))
      return hipErrorInvalidValue;
  }
  return a.dtype == GEMM_F32 ? dispatch_update<float>(a, u, s) : dispatch_update<bf16_t>(a, u, s);
}

}  // namespace hydra
