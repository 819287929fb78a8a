// Scaled dot-product attention for bf16 activations, forward and backward, block-wise so the S x S
// score matrix never reaches HBM.
//   forward:   P = softmax(q k^T * scale [+ causal mask]),  o = P v,  lse = log sum exp (saved)
//   backward:  delta_i = sum_c do[i,c] o[i,c];  P recomputed from lse;
//              dv = P^T do;  dP = do v^T;  dS = P * (dP - delta);  dq = scale * dS k;  dk = scale * dS^T q
// Memory layout: qkv is [B*S, ld] with q of head h at columns [h*DH, h*DH+DH), k at d + ..., v at 2d + ...
// (d = H*DH); o/do are [B*S, ld_o] with head h at columns [h*DH, ...); dqkv has the layout of qkv.
//
// Matrix-core mapping (v_mfma_f32_32x32x16_bf16, 64-wide wavefronts).  A 32x32 accumulator gives lane l
// column l%32 and rows 8q+4(l/32)+e (q,e = 0..3).  Every product is arranged so that the accumulator of
// the first contraction is already in the lane layout the second contraction needs as its B operand
// (k index = accumulator row), i.e. probabilities never go through LDS:
//   forward and dq:  S^T[j,i] = K Q^T  (lane = query i, rows = keys j)  ->  O^T[c,i] += Vt[c,j] P^T[j,i]
//   dk/dv:           S[i,j]   = Q K^T  (lane = key j, rows = queries i) ->  dV^T[c,j] += dOt[c,i] P[i,j]
// The A operand of the second contraction walks a tile along its slow index (eight keys, or queries, of one
// column).  The tiles stay row-major in LDS (rows of DH values, 16-byte chunks XOR-swizzled by the row) and that
// operand comes from transposing LDS reads (ds_read_b64_tr_b16: within 16 lanes, source lane j supplies four
// consecutive columns of row j/4 and lane i receives column i of rows 0..3), two per fragment, so every tile is
// loaded once and nothing is transposed in memory.  Tile loads are software-pipelined: the global loads of tile
// t+1 are issued into registers before the products of tile t and stored to LDS after them.  Softmax statistics
// of a query live in the two lanes l and l^32 and are combined with one cross-lane exchange.  A wavefront owns 32
// queries (or 32 keys) and loops over tiles of 64 keys (queries) shared through LDS by the four wavefronts of the
// workgroup.  All sums run in a fixed order; dq and dk/dv are separate kernels so that no atomics are needed.
#include "kernels.h"

namespace hydra {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

namespace {

constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;
constexpr float NEG_BIG = -1.0e30f;

// 2^x by the hardware instruction alone: arguments here are <= 0 up to rounding, results below the normal
// range may flush to zero, which is what a softmax weight that small is worth.
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// two floats -> two bf16 in one word, round to nearest even: one v_cvt_pk_bf16_f32
__device__ __forceinline__ uint32_t pack2(float a, float b) {
  typedef __attribute__((ext_vector_type(2))) float f32x2;
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
  const f32x2 v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
__device__ __forceinline__ float bf_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

__device__ __forceinline__ f32x16 mfma(const uint4& a, const uint4& b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// ---- LDS tiles of 64 rows x DH columns ---------------------------------------------------------------
// uint4 chunk (row, kc) sits at row*NCH + (kc ^ swz(row)), NCH = DH/8.
// A tile load is split in two so that it can be pipelined: fetch (global -> registers, rows past nrows as zero)
// and put (registers -> LDS).
// Work item of a workgroup.  The hardware deals consecutive workgroup ids to the 8 XCDs in turn; items are numbered so
// that each XCD gets a contiguous run of them, and the 128-row blocks of one (batch, head) are consecutive items: the
// blocks that read the same K/V (or Q/dO) tiles then run on one XCD and share them through its L2, instead of
// each XCD fetching them from memory.  Returns false for the padding ids at the end of the grid.
struct AttnItem { int blk, bh, gi; };
__device__ __forceinline__ bool attn_item(int n_blk, int n_bh, int n_g, AttnItem& it) {
  const int total = n_blk * n_bh * n_g, per_xcd = (total + 7) >> 3;
  const int id = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (id >= total || (int)(blockIdx.x >> 3) >= per_xcd) return false;
  it.blk = id % n_blk;
  it.bh = (id / n_blk) % n_bh;
  it.gi = id / (n_blk * n_bh);
  return true;
}

// XOR term of a row's chunk index.  Two access patterns must each spread over all 64 banks: a 128-bit row read
// (16 consecutive rows at one chunk index per pass) and a transposing 64-bit read (per pass of 32 lanes: rows 4g..4g+3 x
// 4 neighbouring chunks x both halves).  A row of DH = 128 fills the banks once: the 16 rows need 16 different terms,
// and 4 consecutive rows must move the group of 4 chunks to the 4 different groups: 4*(row%4) + (row/4)%4.  A row of
// DH = 64 fills half of the banks and rows of equal parity share them: the 8 such rows among 16 need 8 different terms,
// and the 2 among 4 consecutive rows must move the group of 4 chunks to different groups: 4*((row/2)%2) + (row/4)%4.
template <int DH>
__device__ __forceinline__ int swz(int row) {
  if (DH == 128) return 4 * (row & 3) + ((row >> 2) & 3);
  return 4 * ((row >> 1) & 1) + ((row >> 2) & 3);
}

template <int DH>
struct TileRegs {
  static constexpr int NCH = DH / 8, N = 64 * NCH / 256;
  uint4 r[N];
  __device__ __forceinline__ void fetch(const bf16_t* src, int ld, int row0, int nrows, int tid) {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const int c = tid + 256 * i, row = c / NCH, kc = c % NCH;
      r[i] = make_uint4(0, 0, 0, 0);
      if (row0 + row < nrows) r[i] = *reinterpret_cast<const uint4*>(src + (size_t)(row0 + row) * ld + 8 * kc);
    }
  }
  __device__ __forceinline__ void put(uint4* tile, int tid) const {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const int c = tid + 256 * i, row = c / NCH, kc = c % NCH;
      tile[row * NCH + (kc ^ swz<DH>(row))] = r[i];
    }
  }
};

// A operand along the slow index of a row-major tile: lane l gets, for column col0 + l%32, the values of rows
// row0 + 4g + {0..3} and row0 + 8 + 4g + {0..3} (g = l/32), the k order the accumulator rows of the first product
// have.  Two transposing reads: in the 16-lane group, source lane j reads 8 bytes at row 4g + j/4, column
// 16*(group&1) + 4*(j%4) of the block.
template <int DH>
__device__ __forceinline__ uint4 read_cols(const uint4* tile, int col0, int row0, int lane) {
  constexpr int NCH = DH / 8;
  typedef __attribute__((ext_vector_type(4))) short s16x4;
  typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
  const int j = lane & 15, grp = lane >> 4;
  const int col = col0 + 16 * (grp & 1) + 4 * (j & 3), kc = col >> 3, half = (col >> 2) & 1;
  const int r0 = row0 + 4 * (grp >> 1) + (j >> 2), r1 = r0 + 8;
  const unsigned base = (unsigned)(uintptr_t)(__attribute__((address_space(3))) const char*)reinterpret_cast<const char*>(tile);
  const unsigned a0 = base + (unsigned)((r0 * NCH + (kc ^ swz<DH>(r0))) * 16 + half * 8);
  const unsigned a1 = base + (unsigned)((r1 * NCH + (kc ^ swz<DH>(r1))) * 16 + half * 8);
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(uintptr_t)a0);
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(uintptr_t)a1);
  const uint2 l = __builtin_bit_cast(uint2, lo), h = __builtin_bit_cast(uint2, hi);
  return make_uint4(l.x, l.y, h.x, h.y);
}

template <int DH>
__device__ __forceinline__ uint4 read_rows(const uint4* tile, int row, int kc) {
  constexpr int NCH = DH / 8;
  return tile[row * NCH + (kc ^ swz<DH>(row))];
}

// The same two reads with the lane's part of the address computed once: for rows row0 + l%32 (row0 a multiple of
// NCH) the XOR term depends on the lane alone, so a tile's later row blocks, and a second tile that follows the first
// in LDS, are constant offsets from one pointer per chunk (they go into the instruction's offset field).
template <int DH>
__device__ __forceinline__ const uint4* rows_base(const uint4* tile, int li, int kc) {
  constexpr int NCH = DH / 8;
  return tile + li * NCH + (kc ^ swz<DH>(li));
}
// byte addresses of read_cols' two reads (rows r0 and r0 + 8) for row0 = 0; row0 (a multiple of 16) adds
// row0 * NCH * 16 to both
struct ColsBase { unsigned a0, a1; };
template <int DH>
__device__ __forceinline__ ColsBase cols_base(const uint4* tile, int col0, int lane) {
  constexpr int NCH = DH / 8;
  const int j = lane & 15, grp = lane >> 4;
  const int col = col0 + 16 * (grp & 1) + 4 * (j & 3), kc = col >> 3, half = (col >> 2) & 1;
  const int r0 = 4 * (grp >> 1) + (j >> 2), r1 = r0 + 8;
  const unsigned base = (unsigned)(uintptr_t)(__attribute__((address_space(3))) const char*)reinterpret_cast<const char*>(tile);
  ColsBase b;
  b.a0 = base + (unsigned)((r0 * NCH + (kc ^ swz<DH>(r0))) * 16 + half * 8);
  b.a1 = base + (unsigned)((r1 * NCH + (kc ^ swz<DH>(r1))) * 16 + half * 8);
  return b;
}
template <int DH>
__device__ __forceinline__ uint4 read_cols_at(const ColsBase& b, unsigned off) {
  typedef __attribute__((ext_vector_type(4))) short s16x4;
  typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(uintptr_t)(b.a0 + off));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(uintptr_t)(b.a1 + off));
  const uint2 l = __builtin_bit_cast(uint2, lo), h = __builtin_bit_cast(uint2, hi);
  return make_uint4(l.x, l.y, h.x, h.y);
}

__device__ __forceinline__ uint4 pack_half(const f32x16& p, int x) {
  return make_uint4(pack2(p[8 * x], p[8 * x + 1]), pack2(p[8 * x + 2], p[8 * x + 3]), pack2(p[8 * x + 4], p[8 * x + 5]),
                    pack2(p[8 * x + 6], p[8 * x + 7]));
}

// ---- forward ---------------------------------------------------------------------------------------------
template <int DH>
__global__ __launch_bounds__(256, DH == 64 ? 3 : 2) void attn_fwd_kernel(const AttnArgs a) {
  constexpr int NK = DH / 16, NC = DH / 32, NCH = DH / 8;
  extern __shared__ uint4 lds[];
  uint4* tK = lds;             // [64][NCH]
  uint4* tV = lds + 64 * NCH;  // [64][NCH]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, li = lane & 31, g = lane >> 5;
  AttnItem item;
  if (!attn_item((a.S + 127) / 128, a.B * a.H, a.G, item)) return;
  const int gi = item.gi, bh = item.bh, b = bh / a.H, h = bh % a.H, blk = item.blk;
  const int d = a.H * DH;
  const bf16_t* base = a.qkv[gi] + (size_t)b * a.S * a.ld_qkv + h * DH;
  const int iq = blk * 128 + wave * 32 + li;  // this lane's query
  uint4 qf[NK];
#pragma unroll
  for (int kk = 0; kk < NK; ++kk) {
    qf[kk] = make_uint4(0, 0, 0, 0);
    if (iq < a.S) qf[kk] = *reinterpret_cast<const uint4*>(base + (size_t)iq * a.ld_qkv + 16 * kk + 8 * g);
  }
  f32x16 oacc[NC];
#pragma unroll
  for (int c = 0; c < NC; ++c)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[c][r] = 0.f;
  float m_run = NEG_BIG, l_run = 0.f;
  const float sc = a.scale * LOG2E;
  const int q_hi = min(a.S, blk * 128 + 128) - 1;          // last query of the workgroup
  const int n_tiles = a.causal ? (q_hi / 64 + 1) : (a.S + 63) / 64;
  TileRegs<DH> pk, pv;
  pk.fetch(base + d, a.ld_qkv, 0, a.S, tid);
  pv.fetch(base + 2 * d, a.ld_qkv, 0, a.S, tid);
  const uint4* kr[NK];   // K rows l%32, chunk 2kk + g
  ColsBase vc[NC];       // V columns c*32.., rows from 0
#pragma unroll
  for (int kk = 0; kk < NK; ++kk) kr[kk] = rows_base<DH>(tK, li, 2 * kk + g);
#pragma unroll
  for (int c = 0; c < NC; ++c) vc[c] = cols_base<DH>(tV, c * 32, lane);
  for (int t = 0; t < n_tiles; ++t) {
    const int j0 = t * 64;
    __syncthreads();
    pk.put(tK, tid);
    pv.put(tV, tid);
    __syncthreads();
    if (t + 1 < n_tiles) {  // in flight while this tile is multiplied
      pk.fetch(base + d, a.ld_qkv, j0 + 64, a.S, tid);
      pv.fetch(base + 2 * d, a.ld_qkv, j0 + 64, a.S, tid);
    }
    f32x16 s[2];
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
#pragma unroll
      for (int r = 0; r < 16; ++r) s[sub][r] = 0.f;
#pragma unroll
      for (int kk = 0; kk < NK; ++kk) s[sub] = mfma(kr[kk][sub * 32 * NCH], qf[kk], s[sub]);
    }
    // Masking is needed only in tiles that reach past the sequence end or, with a causal mask, past the
    // wave's first query; the scale is folded into the exponent's multiply-add.
    const bool edge = j0 + 64 > a.S || (a.causal && j0 + 63 > blk * 128 + wave * 32);
    float mx = NEG_BIG;
    if (edge) {
#pragma unroll
      for (int sub = 0; sub < 2; ++sub)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int j = j0 + sub * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
          if (j >= a.S || (a.causal && j > iq)) s[sub][r] = NEG_BIG;
        }
    }
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[sub][r]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx * sc);
    const float alpha = fast_exp2(m_run - m_new);
    float rs = 0.f;
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float p = fast_exp2(fmaf(s[sub][r], sc, -m_new));
        s[sub][r] = p;
        rs += p;
      }
    rs += __shfl_xor(rs, 32, 64);
    l_run = l_run * alpha + rs;
    m_run = m_new;
#pragma unroll
    for (int c = 0; c < NC; ++c)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[c][r] *= alpha;
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
      for (int x = 0; x < 2; ++x) {
        const uint4 pf = pack_half(s[sub], x);
#pragma unroll
        for (int c = 0; c < NC; ++c) oacc[c] = mfma(read_cols_at<DH>(vc[c], (unsigned)((sub * 32 + 16 * x) * NCH * 16)), pf, oacc[c]);
      }
  }
  if (iq < a.S) {
    const float inv = 1.f / l_run;
    bf16_t* o = a.o[gi] + ((size_t)b * a.S + iq) * a.ld_o + h * DH;
#pragma unroll
    for (int c = 0; c < NC; ++c)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int col = c * 32 + 8 * q + 4 * g;
        *reinterpret_cast<uint2*>(o + col) = make_uint2(pack2(oacc[c][4 * q] * inv, oacc[c][4 * q + 1] * inv),
                                                        pack2(oacc[c][4 * q + 2] * inv, oacc[c][4 * q + 3] * inv));
      }
    if (g == 0) a.lse[gi][(size_t)bh * a.S + iq] = (m_run + log2f(l_run)) * LN2;
  }
}

// ---- backward, dq (also writes delta) ------------------------------------------------------------------
template <int DH>
__global__ __launch_bounds__(256, DH == 64 ? 3 : 2) void attn_bwd_dq_kernel(const AttnBwdArgs a) {
  constexpr int NK = DH / 16, NC = DH / 32, NCH = DH / 8;
  extern __shared__ uint4 lds[];
  uint4* tK = lds;             // [64][NCH]
  uint4* tV = lds + 64 * NCH;  // [64][NCH]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, li = lane & 31, g = lane >> 5;
  AttnItem item;
  if (!attn_item((a.S + 127) / 128, a.B * a.H, a.G, item)) return;
  const int gi = item.gi, bh = item.bh, b = bh / a.H, h = bh % a.H, blk = item.blk;
  const int d = a.H * DH;
  const bf16_t* base = a.qkv[gi] + (size_t)b * a.S * a.ld_qkv + h * DH;
  const int iq = blk * 128 + wave * 32 + li;
  uint4 qf[NK], dof[NK];
  float delta = 0.f;
#pragma unroll
  for (int kk = 0; kk < NK; ++kk) {
    qf[kk] = dof[kk] = make_uint4(0, 0, 0, 0);
    if (iq < a.S) {
      qf[kk] = *reinterpret_cast<const uint4*>(base + (size_t)iq * a.ld_qkv + 16 * kk + 8 * g);
      const size_t off = ((size_t)b * a.S + iq) * a.ld_o + h * DH + 16 * kk + 8 * g;
      dof[kk] = *reinterpret_cast<const uint4*>(a.dout[gi] + off);
      const uint4 of = *reinterpret_cast<const uint4*>(a.o[gi] + off);
      const uint32_t dw[4] = {dof[kk].x, dof[kk].y, dof[kk].z, dof[kk].w}, ow[4] = {of.x, of.y, of.z, of.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) delta += bf_lo(dw[e]) * bf_lo(ow[e]) + bf_hi(dw[e]) * bf_hi(ow[e]);
    }
  }
  delta += __shfl_xor(delta, 32, 64);
  const float lse2 = iq < a.S ? a.lse[gi][(size_t)bh * a.S + iq] * LOG2E : 0.f;
  if (iq < a.S && g == 0) a.delta[gi][(size_t)bh * a.S + iq] = delta;
  f32x16 acc[NC];
#pragma unroll
  for (int c = 0; c < NC; ++c)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[c][r] = 0.f;
  const float sc = a.scale * LOG2E;
  const int q_hi = min(a.S, blk * 128 + 128) - 1;
  const int n_tiles = a.causal ? (q_hi / 64 + 1) : (a.S + 63) / 64;
  TileRegs<DH> pk, pv;
  pk.fetch(base + d, a.ld_qkv, 0, a.S, tid);
  pv.fetch(base + 2 * d, a.ld_qkv, 0, a.S, tid);
  const uint4* kr[NK];   // K rows l%32, chunk 2kk + g; V is 64 rows further on
  ColsBase kc_[NC];      // K columns c*32.., rows from 0
#pragma unroll
  for (int kk = 0; kk < NK; ++kk) kr[kk] = rows_base<DH>(tK, li, 2 * kk + g);
#pragma unroll
  for (int c = 0; c < NC; ++c) kc_[c] = cols_base<DH>(tK, c * 32, lane);
  for (int t = 0; t < n_tiles; ++t) {
    const int j0 = t * 64;
    __syncthreads();
    pk.put(tK, tid);
    pv.put(tV, tid);
    __syncthreads();
    if (t + 1 < n_tiles) {
      pk.fetch(base + d, a.ld_qkv, j0 + 64, a.S, tid);
      pv.fetch(base + 2 * d, a.ld_qkv, j0 + 64, a.S, tid);
    }
    const bool edge = j0 + 64 > a.S || (a.causal && j0 + 63 > blk * 128 + wave * 32);
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
      f32x16 s, dp;
#pragma unroll
      for (int r = 0; r < 16; ++r) s[r] = dp[r] = 0.f;
#pragma unroll
      for (int kk = 0; kk < NK; ++kk) {
        s = mfma(kr[kk][sub * 32 * NCH], qf[kk], s);
        dp = mfma(kr[kk][(64 + sub * 32) * NCH], dof[kk], dp);
      }
      if (edge) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int j = j0 + sub * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
          if (j >= a.S || (a.causal && j > iq)) s[r] = NEG_BIG;
        }
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) s[r] = fast_exp2(fmaf(s[r], sc, -lse2)) * (dp[r] - delta);
#pragma unroll
      for (int x = 0; x < 2; ++x) {
        const uint4 df = pack_half(s, x);
#pragma unroll
        for (int c = 0; c < NC; ++c) acc[c] = mfma(read_cols_at<DH>(kc_[c], (unsigned)((sub * 32 + 16 * x) * NCH * 16)), df, acc[c]);
      }
    }
  }
  if (iq < a.S) {
    bf16_t* o = a.dqkv[gi] + ((size_t)b * a.S + iq) * a.ld_qkv + h * DH;
#pragma unroll
    for (int c = 0; c < NC; ++c)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int col = c * 32 + 8 * q + 4 * g;
        *reinterpret_cast<uint2*>(o + col) =
            make_uint2(pack2(acc[c][4 * q] * a.scale, acc[c][4 * q + 1] * a.scale),
                       pack2(acc[c][4 * q + 2] * a.scale, acc[c][4 * q + 3] * a.scale));
      }
  }
}

// ---- backward, dk and dv -----------------------------------------------------------------------------------
template <int DH>
__global__ __launch_bounds__(256, DH == 64 ? 2 : 1) void attn_bwd_dkv_kernel(const AttnBwdArgs a) {
  constexpr int NK = DH / 16, NC = DH / 32, NCH = DH / 8;
  extern __shared__ uint4 lds[];
  uint4* tQ = lds;                                        // [64][NCH]
  uint4* tdO = lds + 64 * NCH;                            // [64][NCH]
  float* st = reinterpret_cast<float*>(lds + 2 * 64 * NCH);  // [2][64]: lse*log2e, delta
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, li = lane & 31, g = lane >> 5;
  AttnItem item;
  if (!attn_item((a.S + 127) / 128, a.B * a.H, a.G, item)) return;
  const int gi = item.gi, bh = item.bh, b = bh / a.H, h = bh % a.H, blk = item.blk;
  const int d = a.H * DH;
  const bf16_t* base = a.qkv[gi] + (size_t)b * a.S * a.ld_qkv + h * DH;
  const bf16_t* dobase = a.dout[gi] + (size_t)b * a.S * a.ld_o + h * DH;
  const int jk = blk * 128 + wave * 32 + li;  // this lane's key
  uint4 kf[NK], vf[NK];
#pragma unroll
  for (int kk = 0; kk < NK; ++kk) {
    kf[kk] = vf[kk] = make_uint4(0, 0, 0, 0);
    if (jk < a.S) {
      kf[kk] = *reinterpret_cast<const uint4*>(base + d + (size_t)jk * a.ld_qkv + 16 * kk + 8 * g);
      vf[kk] = *reinterpret_cast<const uint4*>(base + 2 * d + (size_t)jk * a.ld_qkv + 16 * kk + 8 * g);
    }
  }
  f32x16 dk[NC], dv[NC];
#pragma unroll
  for (int c = 0; c < NC; ++c)
#pragma unroll
    for (int r = 0; r < 16; ++r) dk[c][r] = dv[c][r] = 0.f;
  const float sc = a.scale * LOG2E;
  const int t0 = a.causal ? (blk * 128) / 64 : 0;  // queries before the workgroup's first key see none of its keys
  const int n_tiles = (a.S + 63) / 64;
  TileRegs<DH> pq, pdo;
  float pst = 0.f;
  auto fetch_stats = [&](int i0) {  // threads 0..63: lse*log2e, 64..127: delta of query i0 + tid%64
    pst = 0.f;
    const int i = i0 + (tid & 63);
    if (tid < 128 && i < a.S) pst = tid < 64 ? a.lse[gi][(size_t)bh * a.S + i] * LOG2E : a.delta[gi][(size_t)bh * a.S + i];
  };
  const uint4* qr[NK];   // Q rows l%32, chunk 2kk + g; dO is 64 rows further on
  ColsBase qc[NC];       // Q columns c*32.., rows from 0
#pragma unroll
  for (int kk = 0; kk < NK; ++kk) qr[kk] = rows_base<DH>(tQ, li, 2 * kk + g);
#pragma unroll
  for (int c = 0; c < NC; ++c) qc[c] = cols_base<DH>(tQ, c * 32, lane);
  if (t0 < n_tiles) {
    pq.fetch(base, a.ld_qkv, t0 * 64, a.S, tid);
    pdo.fetch(dobase, a.ld_o, t0 * 64, a.S, tid);
    fetch_stats(t0 * 64);
  }
  for (int t = t0; t < n_tiles; ++t) {
    const int i0 = t * 64;
    __syncthreads();
    pq.put(tQ, tid);
    pdo.put(tdO, tid);
    if (tid < 128) st[tid] = pst;
    __syncthreads();
    if (t + 1 < n_tiles) {
      pq.fetch(base, a.ld_qkv, i0 + 64, a.S, tid);
      pdo.fetch(dobase, a.ld_o, i0 + 64, a.S, tid);
      fetch_stats(i0 + 64);
    }
    // queries past the end, or (causal) queries that precede some key of this wave, need the mask
    const bool edge = i0 + 64 > a.S || (a.causal && i0 < blk * 128 + wave * 32 + 31);
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
      f32x16 s, dp;
#pragma unroll
      for (int r = 0; r < 16; ++r) s[r] = dp[r] = 0.f;
#pragma unroll
      for (int kk = 0; kk < NK; ++kk) {
        s = mfma(qr[kk][sub * 32 * NCH], kf[kk], s);
        dp = mfma(qr[kk][(64 + sub * 32) * NCH], vf[kk], dp);
      }
      f32x16 ds;
      if (edge) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int i = i0 + sub * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
          if (i >= a.S || (a.causal && jk > i)) s[r] = NEG_BIG;
        }
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int il = sub * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
        const float p = fast_exp2(fmaf(s[r], sc, -st[il]));
        s[r] = p;
        ds[r] = p * (dp[r] - st[64 + il]);
      }
#pragma unroll
      for (int x = 0; x < 2; ++x) {
        const uint4 pf = pack_half(s, x), df = pack_half(ds, x);
#pragma unroll
        for (int c = 0; c < NC; ++c) {
          dv[c] = mfma(read_cols_at<DH>(qc[c], (unsigned)((64 + sub * 32 + 16 * x) * NCH * 16)), pf, dv[c]);
          dk[c] = mfma(read_cols_at<DH>(qc[c], (unsigned)((sub * 32 + 16 * x) * NCH * 16)), df, dk[c]);
        }
      }
    }
  }
  if (jk < a.S) {
    bf16_t* ok = a.dqkv[gi] + ((size_t)b * a.S + jk) * a.ld_qkv + d + h * DH;
    bf16_t* ov = ok + d;
#pragma unroll
    for (int c = 0; c < NC; ++c)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int col = c * 32 + 8 * q + 4 * g;
        *reinterpret_cast<uint2*>(ok + col) =
            make_uint2(pack2(dk[c][4 * q] * a.scale, dk[c][4 * q + 1] * a.scale),
                       pack2(dk[c][4 * q + 2] * a.scale, dk[c][4 * q + 3] * a.scale));
        *reinterpret_cast<uint2*>(ov + col) = make_uint2(pack2(dv[c][4 * q], dv[c][4 * q + 1]),
                                                         pack2(dv[c][4 * q + 2], dv[c][4 * q + 3]));
      }
  }
}

template <int DH> constexpr size_t fwd_lds() { return (size_t)2 * 64 * (DH / 8) * 16; }
template <int DH> constexpr size_t dq_lds() { return (size_t)2 * 64 * (DH / 8) * 16; }
template <int DH> constexpr size_t dkv_lds() { return (size_t)2 * 64 * (DH / 8) * 16 + 128 * 4; }

bool attn_ok(int B, int S, int H, int DH, int ld_qkv, int ld_o, int G) {
  return G >= 1 && G <= MAXG && B >= 1 && S >= 1 && H >= 1 && (DH == 64 || DH == 128) && ld_qkv >= 3 * H * DH &&
         !(ld_qkv & 7) && ld_o >= H * DH && !(ld_o & 7);
}

}  // namespace

hipError_t attn_init() { return hipSuccess; }  // every kernel stays below the default LDS limit

hipError_t launch_attn_fwd(const AttnArgs& a, hipStream_t s) {
  if (!attn_ok(a.B, a.S, a.H, a.DH, a.ld_qkv, a.ld_o, a.G)) return hipErrorInvalidValue;
  dim3 grid(((((a.S + 127) / 128) * a.B * a.H * a.G + 7) / 8) * 8);
  if (a.DH == 64) hipLaunchKernelGGL(attn_fwd_kernel<64>, grid, dim3(256), fwd_lds<64>(), s, a);
  else hipLaunchKernelGGL(attn_fwd_kernel<128>, grid, dim3(256), fwd_lds<128>(), s, a);
  return hipGetLastError();
}

hipError_t launch_attn_bwd(const AttnBwdArgs& a, hipStream_t s) {
  if (!attn_ok(a.B, a.S, a.H, a.DH, a.ld_qkv, a.ld_o, a.G)) return hipErrorInvalidValue;
  dim3 grid(((((a.S + 127) / 128) * a.B * a.H * a.G + 7) / 8) * 8);
  if (a.DH == 64) {
    hipLaunchKernelGGL(attn_bwd_dq_kernel<64>, grid, dim3(256), dq_lds<64>(), s, a);
    hipLaunchKernelGGL(attn_bwd_dkv_kernel<64>, grid, dim3(256), dkv_lds<64>(), s, a);
  } else {
    hipLaunchKernelGGL(attn_bwd_dq_kernel<128>, grid, dim3(256), dq_lds<128>(), s, a);
    hipLaunchKernelGGL(attn_bwd_dkv_kernel<128>, grid, dim3(256), dkv_lds<128>(), s, a);
  }
  return hipGetLastError();
}

}  // namespace hydra
