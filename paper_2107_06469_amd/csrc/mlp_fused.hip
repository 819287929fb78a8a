// Whole shard phases of small fp32 MLPs in one launch each.
//
// A model whose step is a few megaflops (32 rows, layers up to 256 wide) is bound by the chain of dependent launches,
// not by arithmetic or memory: every Linear layer as a launch of its own costs a launch, a round trip to memory for its
// operands and a kernel boundary.  Here the forward pass of a shard (all its layers, and the rows' losses when the shard
// ends the model) is one launch; the backward pass is two: the chain of input gradients through the shard's layers,
// then every weight gradient of the shard at once, each with the parameter update in the same kernel (a workgroup per
// 32 output rows of a layer; the one that has the model's last layer also adds up the step's loss).  In the two chains
// a workgroup takes 16 rows of one model's batch through all the layers, activations staying in LDS between them:
// rows are independent there, and the fp32 matrix pipes of one compute unit are what bounds a layer, so two
// workgroups of 16 rows take half the time of one of 32.  A wave needs only its own 32 rows (forward) or columns (input
// gradient) of a weight matrix; it streams them through a private piece of LDS in chunks of 32 k, requested 128
// contiguous bytes per 8 lanes, four chunks ahead of the one being multiplied, with the data movement placed between
// the dependent MFMAs.
//
// The chains use v_mfma_f32_16x16x4_f32 (16 batch rows x 16 columns per tile), the weight gradients
// v_mfma_f32_32x32x2_f32; every sum runs in a fixed order that depends on the layer's shape alone, and the epilogues
// apply the same single-rounded operations as the tiled GEMM kernel's.  Results depend on nothing but the model: not
// on the group, the cut points or the schedule.
#include "act_math.h"
#include "kernels.h"
#include "optim_math.h"

namespace hydra {
namespace {

typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4a;
constexpr int XS = 260;            // LDS row pitch in floats (256 + 4: rows spread over the banks)
constexpr int RB = 16;             // batch rows of a workgroup of the two chain kernels

// acc += W-operand chunk (4 consecutive k of one row n) x X-operand chunk (the same k of one row m) for the weight-gradient
// kernel's 32 x 32 tiles: four instructions, each summing k and k+4 (the two half-waves hold chunks 4 apart)
__device__ __forceinline__ void mma4(f32x16& acc, const float4& w, const float4& x) {
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(w.x, x.x, acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(w.y, x.y, acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(w.z, x.z, acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(w.w, x.w, acc, 0, 0, 0);
}
// The chain kernels' 16 x 16 tiles (v_mfma_f32_16x16x4_f32): lane l supplies row l%16 of either operand at
// k = 4 (l/16) + e of a group of 16 k (a float4 holds e = 0..3), so instruction e sums k = e, 4+e, 8+e, 12+e, and
// receives, for column (batch row) l%16, rows 4 (l/16) + 0..3 of the tile.  Two tiles (two blocks of 16 output
// columns) alternate, so that a wave has two independent chains in the matrix pipe.
__device__ __forceinline__ void mma16x2(f32x4a (&acc)[2], const float4& w0, const float4& w1, const float4& x, int e0) {
  const float wa[4] = {w0.x, w0.y, w0.z, w0.w}, wb[4] = {w1.x, w1.y, w1.z, w1.w}, xv[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
  for (int e = e0; e < e0 + 2; ++e) {
    acc[0] = __builtin_amdgcn_mfma_f32_16x16x4f32(wa[e], xv[e], acc[0], 0, 0, 0);
    acc[1] = __builtin_amdgcn_mfma_f32_16x16x4f32(wb[e], xv[e], acc[1], 0, 0, 0);
  }
}

__device__ __forceinline__ float4 zero4() { return make_float4(0.f, 0.f, 0.f, 0.f); }

// A pointer read from the activation table in memory carries no address space, and through such a pointer the compiler
// emits flat instructions, which count against the LDS counter as well and may complete out of order: every wait
// after one is a wait for everything.  The table's pointers go to global memory; these types say so.
typedef __attribute__((address_space(1))) float gfloat;
typedef float f32x4v __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(1))) f32x4v gf32x4v;
__device__ __forceinline__ gfloat* global_ptr(float* p) { return (gfloat*)p; }
__device__ __forceinline__ const gfloat* global_ptr(const float* p) { return (const gfloat*)p; }
__device__ __forceinline__ float4 gload4(const gfloat* p) {
  const f32x4v v = *(const gf32x4v*)p;
  return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void gstore4(gfloat* p, float a, float b, float c, float d) {
  const f32x4v v = {a, b, c, d};
  *(gf32x4v*)p = v;
}

// rows [0, rows) x columns [0, cols) of a row-major matrix into the RB LDS rows of pitch XS; everything else in the
// RB x XS block is zero (the products run over k in groups of 16 and must not meet what an earlier kernel left in LDS)
__device__ __forceinline__ void stage_rows(float* xs, const gfloat* src, int ld, int rows, int cols, int tid, int nt) {
  constexpr int C4 = XS / 4;  // float4 groups per row
  for (int i = tid; i < RB * C4; i += nt) {
    const int m = i / C4, c = (i % C4) * 4;
    float4 v = zero4();
    if (m < rows && c < cols) {
      const gfloat* r = src + (size_t)m * ld + c;
      if (c + 4 <= cols) v = gload4(r);
      else {
        v.x = r[0];
        if (c + 1 < cols) v.y = r[1];
        if (c + 2 < cols) v.z = r[2];
      }
    }
    *reinterpret_cast<float4*>(&xs[m * XS + c]) = v;
  }
}

// ---- forward: units [u0, u1) of 16 batch rows of one model per workgroup (8 waves; wave w owns output columns
// [32w, 32w+32)) --------------------------------------------------------------------------------------------------
// Rows of the batch do not meet before the loss, so a model's rows are split over workgroups (the fp32 matrix pipes of
// one compute unit are what bounds a layer: 16 rows take half the time of 32).  A wave multiplies by its own 32 rows
// of W only, so it stages them for itself: chunks of 32 k x 32 rows pass through a piece of LDS that no other wave
// touches (8 lanes per row, 128 contiguous bytes each, so every line that travels is used in full), four chunks are in
// flight in registers while a fifth is multiplied, and the requests run ahead across layer ends (weights do not depend
// on activations).  Nothing inside a layer waits for another wave: the workgroup meets only where a layer's outputs
// replace its inputs in LDS.
constexpr int WP = 36;               // LDS pitch of a staged weight row: 32 k + 4 (16 rows read as float4 hit 16 bank groups)
constexpr int WCH = 32 * WP;         // floats of one staged chunk of one wave
constexpr size_t FWD_LDS = (RB * XS + 8 * 2 * WCH) * sizeof(float);

// the same value in every lane, told to the compiler (descriptors of buffer loads must sit in scalar registers)
__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ const float* uniform(const float* p) {
  const unsigned long long b = reinterpret_cast<unsigned long long>(p);
  const unsigned lo = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)b);
  const unsigned hi = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(b >> 32));
  return reinterpret_cast<const float*>(((unsigned long long)hi << 32) | lo);
}

// orders a wave's own LDS writes before its later LDS reads (the hardware keeps a wave's LDS operations in order; this
// keeps the compiler from moving them)
__device__ __forceinline__ void wave_lds_order() {
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
}
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

__device__ __forceinline__ void fwd_body(const MlpFusedArgs& a, float* smem) {
  float* xs = smem;                  // [RB][XS] the layer's input rows
  const int g = blockIdx.x % a.G, r0 = (blockIdx.x / a.G) * RB;  // model, first batch row
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lrow = lane & 15, lgrp = lane >> 4;
  const int rows = a.B - r0 < RB ? a.B - r0 : RB;  // >= 1: the grid has ceil(B / RB) workgroups per model
  const __attribute__((address_space(1))) MlpTab* tb = (const __attribute__((address_space(1))) MlpTab*)a.tab[g];
  const float* P = a.p[g];
  const int n0 = wave * 32;
  float* wb = smem + RB * XS + wave * 2 * WCH;  // [2][32][WP] this wave's weight chunks
  const int ldrow = lane >> 3, ldseg = lane & 7;  // this lane's part of a chunk: rows n0 + ldrow + 8 i, k 4 ldseg .. + 3
  // The next chunk to request: unit lu, chunk lc of it, and the unit's matrix (lW: lN x lK floats; past the shard's
  // last unit an empty one).  Buffer loads with the whole address in the checked offset: rows at or past lN lie behind
  // the end of the descriptor and read as zero, a chunk column at or past lK is sent out of range.
  int lu = a.u0, lc = 0, lK = 0, lN = 0;
  const float* lW = P;
  auto unit_to_request = [&]() {  // after lu has changed
    const bool live = lu < a.u1;
    lK = uniform(lu == 0 ? a.d_in : a.d);
    lN = uniform(!live ? 0 : (lu < a.L ? a.d : a.n_out));
    lW = uniform(P + a.w_off[live ? lu : a.u0]);
  };
  unit_to_request();
  auto advance = [&]() {
    if (++lc * 32 >= (lK + 127) / 128 * 128) {  // every unit takes a multiple of four chunks (the last ones may be empty)
      ++lu;
      lc = 0;
      unit_to_request();
    }
  };
  auto issue = [&](float4 (&st)[4]) {
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(lW), 0, lN * lK * 4, 0x00020000);
    const int col = 32 * lc + 4 * ldseg;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const unsigned off = col < lK ? (unsigned)((n0 + ldrow + 8 * i) * lK + col) * 4u : 0xfffffff0u;
      const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rs, (int)off, 0, 0);
      st[i] = make_float4(__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w));
    }
    advance();
  };
  auto commit = [&](const float4 (&st)[4], float* buf) {
#pragma unroll
    for (int i = 0; i < 4; ++i) *reinterpret_cast<float4*>(&buf[(ldrow + 8 * i) * WP + 4 * ldseg]) = st[i];
    wave_lds_order();
  };
  float4 s0[4], s1[4], s2[4], s3[4];
  issue(s0);  // chunk 0
  issue(s1);  // chunk 1
  issue(s2);  // chunk 2
  issue(s3);  // chunk 3
  stage_rows(xs, global_ptr(a.u0 == 0 ? a.x[g] : tb->h[a.u0 - 1]) + (size_t)r0 * (a.u0 == 0 ? a.ld_in : a.ldd),
             a.u0 == 0 ? a.ld_in : a.ldd, rows, a.u0 == 0 ? a.d_in : a.d, tid, 512);
  commit(s0, wb);
  issue(s0);  // chunk 4
  __syncthreads();  // the input rows are in place
  for (int u = a.u0; u < a.u1; ++u) {
    // here: buffer 0 holds the unit's chunk 0, s1, s2, s3 its chunks 1, 2, 3, s0 the chunk after those
    const int K = u == 0 ? a.d_in : a.d, N = u < a.L ? a.d : a.n_out;
    const float* bias = P + a.b_off[u];
    const bool active = n0 < N;  // uniform over the wave
    f32x4a acc[2];
#pragma unroll
    for (int q = 0; q < 2; ++q)
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[q][e] = 0.f;
    float bv[2][4];
    if (active) {
#pragma unroll
      for (int q = 0; q < 2; ++q)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int nn = n0 + 16 * q + 4 * lgrp + e;
          bv[q][e] = nn < N ? bias[nn] : 0.f;
        }
    }
    // where the unit's outputs go: read from the table now, not between the stores at the unit's end (a pointer read
    // there would wait for every store before it)
    gfloat* const zu = global_ptr(u < a.L ? tb->z[u] : tb->logits);
    gfloat* const hu = global_ptr(u < a.L ? tb->h[u] : nullptr);
    gfloat* const dlog = global_ptr(u == a.L ? tb->dlogits : nullptr);
    gfloat* const rowl = global_ptr(u == a.L ? tb->rowloss : nullptr);
    // One chunk: multiply by the chunk in `cur` while the chunk held in `st` moves into `other` and the next chunk to
    // request takes its place in `st`, a quarter after each quarter of the products.  A wave's dependent MFMAs leave
    // its issue slot idle; the data movement goes into those gaps instead of standing in front of the products.
    auto half = [&](float4 (&st)[4], float* other, const float* cur, int c) {
      const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(lW), 0, lN * lK * 4, 0x00020000);
      const int col = 32 * lc + 4 * ldseg;
      const bool inside = col < lK;
      const unsigned off0 = (unsigned)((n0 + ldrow) * lK + col) * 4u, step = (unsigned)(8 * lK) * 4u;
      auto move = [&](int s) {  // a quarter of the chunk in st goes to LDS, a quarter of the next request takes its place
        __builtin_amdgcn_sched_barrier(0);
        *reinterpret_cast<float4*>(&other[(ldrow + 8 * s) * WP + 4 * ldseg]) = st[s];
        const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rs, (int)(inside ? off0 + step * s : 0xfffffff0u), 0, 0);
        st[s] = make_float4(__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w));
        __builtin_amdgcn_sched_barrier(0);
      };
      if (active) {
        // all of the chunk's operands are requested from LDS before the first product, so that only the first of
        // them is waited for (a group of 16 k that starts at or past K is not multiplied; inside a group, k at or past
        // K meet staged zeros on both sides)
        float4 wq[2][2], xq[2];
#pragma unroll
        for (int s = 0; s < 2; ++s) {
#pragma unroll
          for (int q = 0; q < 2; ++q) wq[q][s] = *reinterpret_cast<const float4*>(&cur[(16 * q + lrow) * WP + 16 * s + 4 * lgrp]);
          xq[s] = *reinterpret_cast<const float4*>(&xs[lrow * XS + 32 * c + 16 * s + 4 * lgrp]);
        }
        if (32 * c + 32 <= K) {  // a whole chunk: straight-line code
#pragma unroll
          for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
              mma16x2(acc, wq[0][s], wq[1][s], xq[s], 2 * h);
              move(2 * s + h);
            }
        } else {
#pragma unroll
          for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
              if (32 * c + 16 * s < K) mma16x2(acc, wq[0][s], wq[1][s], xq[s], 2 * h);
              move(2 * s + h);
            }
        }
      } else {
#pragma unroll
        for (int s = 0; s < 4; ++s) move(s);
      }
      advance();
      wave_lds_order();
    };
    auto four_chunks = [&](int c) {
      // the wave has multiplied by the other buffer's last chunk (its operands are in registers): it is free
      half(s1, wb + WCH, wb, c);
      half(s2, wb, wb + WCH, c + 1);
      half(s3, wb + WCH, wb, c + 2);
      half(s0, wb, wb + WCH, c + 3);
    };
    // The first pair stands outside the loop: the previous unit's stores may still be on their way when it starts,
    // and a wait with loads and stores both outstanding is a wait for everything; inside the loop only loads are
    // outstanding, so the wait for a chunk leaves the younger chunk's requests in flight.
    four_chunks(0);
    for (int c = 4; c * 32 < K; c += 4) four_chunks(c);
    __syncthreads();  // every wave has read this layer's input from LDS
    // a lane holds, for batch row r0 + lrow, columns n0 + 16q + 4 lgrp + (0..3), q = 0, 1
    if (active) {
      const int m = r0 + lrow;
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        const int nq = n0 + 16 * q + 4 * lgrp;
        if (nq >= N) continue;
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          v[e] = acc[q][e];
          if (nq + e < N) v[e] += bv[q][e];
        }
        if (u < a.L) {
          float h[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) h[e] = act_fwd(v[e], a.act);
          if (m < a.B) {  // N = d is a multiple of 8: whole vectors
            gstore4(zu + (size_t)m * a.ldd + nq, v[0], v[1], v[2], v[3]);
            gstore4(hu + (size_t)m * a.ldd + nq, h[0], h[1], h[2], h[3]);
          }
          *reinterpret_cast<float4*>(&xs[lrow * XS + nq]) = make_float4(h[0], h[1], h[2], h[3]);
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (nq + e < N) {
              if (m < a.B) zu[(size_t)m * a.ldv + nq + e] = v[e];
              xs[lrow * XS + nq + e] = v[e];
            }
        }
      }
    }
    __syncthreads();
    if (u == a.L) {
      // softmax cross-entropy of the workgroup's rows: lane m of the first wave walks its row in ascending class order
      // (the step's loss is the sum of the rows' losses; the gradient kernel, which follows, adds them up)
      const int C = a.n_out;
      if (wave == 0 && lane < rows) {
        const int m = r0 + lane;
        const float* z = &xs[lane * XS];
        const int y = a.labels[m];
        float mx = -INFINITY;
        for (int c = 0; c < C; ++c) mx = fmaxf(mx, z[c]);
        float sum = 0.f;
        for (int c = 0; c < C; ++c) sum += expf(z[c] - mx);
        const float lse = logf(sum) + mx, inv_sum = 1.f / sum;
        gfloat* dz = dlog + (size_t)m * a.ldv;
        for (int c = 0; c < a.ldv; ++c) dz[c] = c < C ? (expf(z[c] - mx) * inv_sum - (c == y ? 1.f : 0.f)) * a.inv_n : 0.f;
        rowl[m] = lse - z[y];
      }
    }
  }
}

// ---- backward, part 1: dz_{u-1} = (dz_u W_u) * act'(z_{u-1}) for u = u1-1 ... max(u0, 1), 16 batch rows of one model
// per workgroup ---------------------------------------------------------------------------------------------------
// W_u is k-major for this product (its rows are the k of the sum); a wave stages its own 32 columns of a chunk of 32 k
// (8 lanes per row, 128 contiguous bytes each) through the same private pipeline as in the forward kernel.
constexpr int DP = 36;               // LDS pitch of a staged k-row: 32 columns + 4 (the four quarter-waves read rows 4 apart)
constexpr int DCH = 32 * DP;         // floats of one staged chunk of one wave: 32 k x 32 columns
constexpr size_t DGRAD_LDS = (RB * XS + 8 * 2 * DCH) * sizeof(float);

__device__ __forceinline__ void chain_body(const MlpFusedArgs& a, float* smem) {
  float* ds = smem;                  // [RB][XS] dz_u
  const int g = blockIdx.x % a.G, r0 = (blockIdx.x / a.G) * RB;  // model, first batch row
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lrow = lane & 15, lgrp = lane >> 4;
  const int rows = a.B - r0 < RB ? a.B - r0 : RB;
  const __attribute__((address_space(1))) MlpTab* tb = (const __attribute__((address_space(1))) MlpTab*)a.tab[g];
  const float* P = a.p[g];
  const int u_hi = a.u1 - 1, u_lo = a.u0 > 1 ? a.u0 : 1;
  if (u_hi < u_lo) return;
  const int n0 = wave * 32;
  float* wb = smem + RB * XS + wave * 2 * DCH;  // [2][32][DP] this wave's weight chunks
  const int ldrow = lane >> 3, ldseg = lane & 7;  // this lane's part of a chunk: k ldrow + 8 i, columns n0 + 4 ldseg .. + 3
  const int Kin = a.d;               // width of dz_{u-1} (u >= 1)
  const bool active = n0 < Kin;      // uniform over the wave
  // The next chunk to request: unit lu (descending), chunk lc of it, and the unit's matrix (lW: lK rows of Kin floats;
  // below the shard's first unit an empty one).  Buffer loads with the whole address in the checked offset: the
  // descriptor ends with row lK - 1, so rows at or past it read as zero; columns at or past Kin are sent out of range.
  int lu = u_hi, lc = 0, lK = 0, lrows = 0;
  const float* lW = P;
  auto unit_to_request = [&]() {  // after lu has changed
    const bool live = lu >= u_lo;
    lK = uniform(lu < a.L ? a.d : a.n_out);  // rows of W_lu: the k of its sum
    lrows = uniform(live ? lK : 0);
    lW = uniform(P + a.w_off[live ? lu : u_hi]);
  };
  unit_to_request();
  auto advance = [&]() {
    if (++lc * 32 >= (lK + 127) / 128 * 128) {  // every unit takes a multiple of four chunks (the last ones may be empty)
      --lu;
      lc = 0;
      unit_to_request();
    }
  };
  const bool inside = n0 + 4 * ldseg < Kin;
  auto issue = [&](float4 (&st)[4]) {
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(lW), 0, lrows * Kin * 4, 0x00020000);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const unsigned off = inside ? (unsigned)((32 * lc + ldrow + 8 * i) * Kin + n0 + 4 * ldseg) * 4u : 0xfffffff0u;
      const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rs, (int)off, 0, 0);
      st[i] = make_float4(__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w));
    }
    advance();
  };
  auto commit = [&](const float4 (&st)[4], float* buf) {
#pragma unroll
    for (int i = 0; i < 4; ++i) *reinterpret_cast<float4*>(&buf[(ldrow + 8 * i) * DP + 4 * ldseg]) = st[i];
    wave_lds_order();
  };
  float4 s0[4], s1[4], s2[4], s3[4];
  issue(s0);  // chunk 0
  issue(s1);  // chunk 1
  issue(s2);  // chunk 2
  issue(s3);  // chunk 3
  stage_rows(ds, global_ptr(u_hi < a.L ? tb->dz[u_hi] : tb->dlogits) + (size_t)r0 * (u_hi < a.L ? a.ldd : a.ldv),
             u_hi < a.L ? a.ldd : a.ldv, rows, u_hi < a.L ? a.d : a.n_out, tid, 512);
  commit(s0, wb);
  issue(s0);  // chunk 4
  __syncthreads();  // dz of the shard's last unit is in place
  for (int u = u_hi; u >= u_lo; --u) {
    // here: buffer 0 holds the unit's chunk 0, s1, s2, s3 its chunks 1, 2, 3, s0 the chunk after those
    const int K = u < a.L ? a.d : a.n_out;
    f32x4a acc[2];
#pragma unroll
    for (int q = 0; q < 2; ++q)
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[q][e] = 0.f;
    // read the table now: between the stores at the unit's end a pointer read would wait for each of them
    gfloat* const dzo = global_ptr(tb->dz[u - 1]);
    const gfloat* const zg = global_ptr(tb->z[u - 1]);
    const int m = r0 + lrow;
    float4 gate[2];  // z_{u-1} at the outputs this lane will hold
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      const int nq = n0 + 16 * q + 4 * lgrp;
      gate[q] = (active && m < a.B && nq < Kin) ? gload4(zg + (size_t)m * a.ldd + nq) : zero4();
    }
    auto half = [&](float4 (&st)[4], float* other, const float* cur, int c) {
      const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(lW), 0, lrows * Kin * 4, 0x00020000);
      const unsigned off0 = (unsigned)((32 * lc + ldrow) * Kin + n0 + 4 * ldseg) * 4u, step = (unsigned)(8 * Kin) * 4u;
      auto move = [&](int s) {  // a quarter of the chunk in st goes to LDS, a quarter of the next request takes its place
        __builtin_amdgcn_sched_barrier(0);
        *reinterpret_cast<float4*>(&other[(ldrow + 8 * s) * DP + 4 * ldseg]) = st[s];
        const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rs, (int)(inside ? off0 + step * s : 0xfffffff0u), 0, 0);
        st[s] = make_float4(__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w));
        __builtin_amdgcn_sched_barrier(0);
      };
      if (active) {
        // all of the chunk's operands are requested from LDS before the first product: this lane's W values are
        // k = 16 s + 4 lgrp + (0..3) of columns lrow and 16 + lrow of the wave's 32
        float4 wq[2][2], xq[2];
#pragma unroll
        for (int s = 0; s < 2; ++s) {
          const float* r = cur + (16 * s + 4 * lgrp) * DP + lrow;
#pragma unroll
          for (int q = 0; q < 2; ++q) wq[q][s] = make_float4(r[16 * q], r[DP + 16 * q], r[2 * DP + 16 * q], r[3 * DP + 16 * q]);
          xq[s] = *reinterpret_cast<const float4*>(&ds[lrow * XS + 32 * c + 16 * s + 4 * lgrp]);
        }
        if (32 * c + 32 <= K) {  // a whole chunk: straight-line code
#pragma unroll
          for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
              mma16x2(acc, wq[0][s], wq[1][s], xq[s], 2 * h);
              move(2 * s + h);
            }
        } else {
#pragma unroll
          for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
              if (32 * c + 16 * s < K) mma16x2(acc, wq[0][s], wq[1][s], xq[s], 2 * h);
              move(2 * s + h);
            }
        }
      } else {
#pragma unroll
        for (int s = 0; s < 4; ++s) move(s);
      }
      advance();
      wave_lds_order();
    };
    auto four_chunks = [&](int c) {
      half(s1, wb + DCH, wb, c);
      half(s2, wb, wb + DCH, c + 1);
      half(s3, wb + DCH, wb, c + 2);
      half(s0, wb, wb + DCH, c + 3);
    };
    four_chunks(0);  // outside the loop for the same reason as in the forward kernel
    for (int c = 4; c * 32 < K; c += 4) four_chunks(c);
    __syncthreads();  // every wave has read dz_u from LDS
    if (active) {
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        const int nq = n0 + 16 * q + 4 * lgrp;
        if (nq >= Kin) continue;
        const float gz[4] = {gate[q].x, gate[q].y, gate[q].z, gate[q].w};
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = acc[q][e] * act_grad(gz[e], a.act);
        const float4 o = make_float4(v[0], v[1], v[2], v[3]);
        if (m < a.B) gstore4(dzo + (size_t)m * a.ldd + nq, v[0], v[1], v[2], v[3]);
        *reinterpret_cast<float4*>(&ds[lrow * XS + nq]) = m < a.B ? o : zero4();
      }
    }
    __syncthreads();
  }
}

static_assert(FWD_LDS == DGRAD_LDS, "the two chains share one LDS layout");

__global__ __launch_bounds__(512) void mlp_fwd_fused_kernel(const MlpFusedArgs a) {
  extern __shared__ float smem[];
  fwd_body(a, smem);
}
__global__ __launch_bounds__(512) void mlp_dgrad_chain_kernel(const MlpFusedArgs a) {
  extern __shared__ float smem[];
  chain_body(a, smem);
}
// Forward through all of a model's units, then straight on into the chain of input gradients: a workgroup's 16 rows
// need nothing from other workgroups in between (the rows' losses and the gradient of the logits are its own), so
// the two phases of a step that the plan runs back to back are one launch.  What the forward phase wrote to memory
// (pre-activations, the logits' gradient) is read back by other waves of the workgroup: a workgroup-wide fence and
// barrier stand between the phases.
__global__ __launch_bounds__(512) void mlp_fwd_chain_kernel(const MlpFusedArgs a) {
  extern __shared__ float smem[];
  fwd_body(a, smem);
  __threadfence_block();
  __syncthreads();
  chain_body(a, smem);
}

// ---- backward, part 2: dW_u = dz_u^T x_u with the update of W_u and b_u, for every unit of the shard -----------------
// grid (strip of 32 output rows, unit, model); wave w takes the 32-column tiles w, w+4 of the strip
template <int OPT>
__global__ __launch_bounds__(256) void mlp_wgrad_update_kernel(const MlpFusedArgs a) {
  const int strip = blockIdx.x, u = a.u0 + blockIdx.y, g = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lrow = lane & 31, lgrp = lane >> 5;
  const int N = u < a.L ? a.d : a.n_out, Kin = u == 0 ? a.d_in : a.d;
  if (strip * 32 >= N) return;
  const __attribute__((address_space(1))) MlpTab* tb = (const __attribute__((address_space(1))) MlpTab*)a.tab[g];
  if (u == a.L && strip == 0 && tid == 0) {
    // the step's loss: the rows' losses, which the forward kernel's workgroups left, added in ascending order
    const gfloat* rl = global_ptr(tb->rowloss);
    float t = 0.f;
    for (int m = 0; m < a.B; ++m) t += rl[m];
    *a.loss[g] = t * a.inv_n;
  }
  const gfloat* dz = global_ptr(u < a.L ? tb->dz[u] : tb->dlogits);
  const int lddz = u < a.L ? a.ldd : a.ldv;
  const gfloat* xin = global_ptr(u == 0 ? a.x[g] : tb->h[u - 1]);
  const int ldx = u == 0 ? a.ld_in : a.ldd;
  const int n = strip * 32 + lrow;
  const OptimHp hp = a.hp[g];
  // the sum runs over the batch rows: 4 groups of 8; this lane's dz values: rows 8s + 4 lgrp + e of column n
  float4 dv[4];
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    const int m = 8 * s + 4 * lgrp;
    dv[s] = zero4();
    if (n < N) {
      if (m < a.B) dv[s].x = dz[(size_t)m * lddz + n];
      if (m + 1 < a.B) dv[s].y = dz[(size_t)(m + 1) * lddz + n];
      if (m + 2 < a.B) dv[s].z = dz[(size_t)(m + 2) * lddz + n];
      if (m + 3 < a.B) dv[s].w = dz[(size_t)(m + 3) * lddz + n];
    }
  }
  for (int kt = wave; kt * 32 < Kin; kt += 4) {
    const int k = kt * 32 + lrow;
    float4 xa[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const int m = 8 * s + 4 * lgrp;
      xa[s] = zero4();
      if (k < Kin) {
        if (m < a.B) xa[s].x = xin[(size_t)m * ldx + k];
        if (m + 1 < a.B) xa[s].y = xin[(size_t)(m + 1) * ldx + k];
        if (m + 2 < a.B) xa[s].z = xin[(size_t)(m + 2) * ldx + k];
        if (m + 3 < a.B) xa[s].w = xin[(size_t)(m + 3) * ldx + k];
      }
    }
    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
    for (int s = 0; s < 4; ++s) mma4(acc, xa[s], dv[s]);
    // a lane holds, for output row n = strip*32 + lrow, columns kt*32 + 8q + 4 lgrp + (0..3)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int kq = kt * 32 + 8 * q + 4 * lgrp;
      if (n >= N || kq >= Kin) continue;   // Kin is a multiple of 8: whole vectors
      const size_t ix = (size_t)a.w_off[u] + (size_t)n * Kin + kq;
      const float gr[4] = {acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]};
      if (a.keep_grads) {
        *reinterpret_cast<float4*>(a.g[g] + ix) = make_float4(gr[0], gr[1], gr[2], gr[3]);
        continue;
      }
      const float4 pv = *reinterpret_cast<const float4*>(a.p[g] + ix);
      float pe[4] = {pv.x, pv.y, pv.z, pv.w}, me[4] = {0.f, 0.f, 0.f, 0.f}, ve[4] = {0.f, 0.f, 0.f, 0.f};
      if (OPT == 1) {
        const float4 mv = *reinterpret_cast<const float4*>(a.m[g] + ix), vv = *reinterpret_cast<const float4*>(a.v[g] + ix);
        me[0] = mv.x; me[1] = mv.y; me[2] = mv.z; me[3] = mv.w;
        ve[0] = vv.x; ve[1] = vv.y; ve[2] = vv.z; ve[3] = vv.w;
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) optim_step<OPT>(pe[e], me[e], ve[e], gr[e], hp);
      if (OPT == 1) {
        *reinterpret_cast<float4*>(a.m[g] + ix) = make_float4(me[0], me[1], me[2], me[3]);
        *reinterpret_cast<float4*>(a.v[g] + ix) = make_float4(ve[0], ve[1], ve[2], ve[3]);
      }
      *reinterpret_cast<float4*>(a.p[g] + ix) = make_float4(pe[0], pe[1], pe[2], pe[3]);
    }
  }
  if (wave == 0) {
    // bias gradient: column sums of dz.  Each half-wave adds its chunks in ascending row order, element by element,
    // then the two halves are added (the order the tiled kernel uses for its row sums)
    float rs = 0.f;
    {
#pragma clang fp contract(off)
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        rs = rs + dv[s].x;
        rs = rs + dv[s].y;
        rs = rs + dv[s].z;
        rs = rs + dv[s].w;
      }
    }
    const float total = rs + __shfl_xor(rs, 32, 64);
    if (lgrp == 0 && n < N) {
      const size_t ix = (size_t)a.b_off[u] + n;
      if (a.keep_grads) {
        a.g[g][ix] = total;
      } else {
        float pe = a.p[g][ix], me = 0.f, ve = 0.f;
        if (OPT == 1) {
          me = a.m[g][ix];
          ve = a.v[g][ix];
        }
        optim_step<OPT>(pe, me, ve, total, hp);
        if (OPT == 1) {
          a.m[g][ix] = me;
          a.v[g][ix] = ve;
        }
        a.p[g][ix] = pe;
      }
    }
  }
}

hipError_t check(const MlpFusedArgs& a) {
  if (a.G < 1 || a.G > MAXG || a.B < 1 || a.B > 32 || a.d_in < 8 || a.d_in > 256 || a.d_in % 8 || a.d < 8 || a.d > 256 ||
      a.d % 8 || a.n_out < 1 || a.n_out > 256 || a.L < 0 || a.L + 1 > MLP_FUSED_MAX_UNITS || a.u0 < 0 || a.u1 > a.L + 1 ||
      a.u0 >= a.u1 || a.ld_in < a.d_in || a.ld_in % 4 || a.ldd < a.d || a.ldd % 4 || a.ldv < a.n_out)
    return hipErrorInvalidValue;
  for (int g = 0; g < a.G; ++g)
    if (!a.p[g] || !a.tab[g] || !a.x[g]) return hipErrorInvalidValue;
  return hipSuccess;
}

}  // namespace

bool mlp_fused_shape_ok(int B, int d_in, int d, int n_out, int n_units) {
  return B >= 1 && B <= 32 && d_in >= 8 && d_in <= 256 && d_in % 8 == 0 && d >= 8 && d <= 256 && d % 8 == 0 && n_out >= 1 &&
         n_out <= 256 && n_units <= MLP_FUSED_MAX_UNITS;
}

hipError_t mlp_fused_init() {
  const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&mlp_fwd_fused_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)FWD_LDS);
  if (e != hipSuccess) return e;
  const hipError_t e2 = hipFuncSetAttribute(reinterpret_cast<const void*>(&mlp_dgrad_chain_kernel),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)DGRAD_LDS);
  if (e2 != hipSuccess) return e2;
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&mlp_fwd_chain_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                             (int)FWD_LDS);
}

hipError_t launch_mlp_fwd_fused(const MlpFusedArgs& a, hipStream_t s) {
  hipError_t e = check(a);
  if (e != hipSuccess) return e;
  if (a.u1 == a.L + 1 && !a.labels) return hipErrorInvalidValue;
  hipLaunchKernelGGL(mlp_fwd_fused_kernel, dim3(a.G * ((a.B + RB - 1) / RB)), dim3(512), FWD_LDS, s, a);
  return hipGetLastError();
}

hipError_t launch_mlp_fwd_chain(const MlpFusedArgs& a, hipStream_t s) {
  hipError_t e = check(a);
  if (e != hipSuccess) return e;
  if (a.u0 != 0 || a.u1 != a.L + 1 || !a.labels) return hipErrorInvalidValue;  // the whole model, forward and back
  hipLaunchKernelGGL(mlp_fwd_chain_kernel, dim3(a.G * ((a.B + RB - 1) / RB)), dim3(512), FWD_LDS, s, a);
  return hipGetLastError();
}

hipError_t launch_mlp_dgrad_chain(const MlpFusedArgs& a, hipStream_t s) {
  hipError_t e = check(a);
  if (e != hipSuccess) return e;
  if (a.u1 - 1 < (a.u0 > 1 ? a.u0 : 1)) return hipSuccess;  // no unit of the shard has an input gradient to produce
  hipLaunchKernelGGL(mlp_dgrad_chain_kernel, dim3(a.G * ((a.B + RB - 1) / RB)), dim3(512), DGRAD_LDS, s, a);
  return hipGetLastError();
}

hipError_t launch_mlp_wgrad_update(const MlpFusedArgs& a, hipStream_t s) {
  hipError_t e = check(a);
  if (e != hipSuccess) return e;
  for (int g = 0; g < a.G; ++g) {
    if (a.keep_grads ? !a.g[g] : (a.opt == 1 && (!a.m[g] || !a.v[g]))) return hipErrorInvalidValue;
    if (a.u1 == a.L + 1 && !a.loss[g]) return hipErrorInvalidValue;  // the launch with the last unit writes the step's loss
  }
  const int widest = a.d > a.n_out ? a.d : a.n_out;
  const dim3 grid((widest + 31) / 32, a.u1 - a.u0, a.G);
  if (a.opt == 1) hipLaunchKernelGGL(mlp_wgrad_update_kernel<1>, grid, dim3(256), 0, s, a);
  else hipLaunchKernelGGL(mlp_wgrad_update_kernel<0>, grid, dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace hydra
