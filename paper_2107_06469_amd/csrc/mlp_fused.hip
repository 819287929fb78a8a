// Whole shard phases of small fp32 MLPs in one launch each.
//
// A model whose step is a few megaflops (32 rows, layers up to 256 wide) is bound by the chain of dependent launches,
// not by arithmetic or memory: every Linear layer as a launch of its own costs a launch, a round trip to memory for its
// operands and a kernel boundary.  Here the forward pass of a shard (all its layers, and the loss when the shard ends
// the model) is one launch with one workgroup per model; the backward pass is two: the chain of input gradients
// through the shard's layers (one workgroup per model), then every weight gradient of the shard at once, each with the
// parameter update in the same kernel (a workgroup per 32 output rows of a layer).  Activations stay in LDS between
// layers; weights go from memory straight into MFMA operand registers, all requests of a layer in flight together.
//
// The products use v_mfma_f32_32x32x2_f32 with the same operand roles, the same k pairing inside an instruction
// (k and k+4 of every group of 8) and the same ascending chain as the tiled fp32 GEMM kernel, and the epilogues apply
// the same single-rounded operations, so a layer computes the same values here as there.  Results depend on nothing
// but the model: not on the group, the cut points or the schedule.
#include "act_math.h"
#include "kernels.h"
#include "optim_math.h"

namespace hydra {
namespace {

typedef __attribute__((ext_vector_type(16))) float f32x16;
constexpr int XS = 260;            // LDS row pitch in floats (256 + 4: rows spread over the banks)
constexpr int MAXK8 = 32;          // groups of 8 k in the widest layer (256)

// acc += W-operand chunk (4 consecutive k of one row n) x X-operand chunk (the same k of one row m): four instructions,
// each summing k and k+4 (the two half-waves hold chunks 4 apart), in ascending order
__device__ __forceinline__ void mma4(f32x16& acc, const float4& w, const float4& x) {
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(w.x, x.x, acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(w.y, x.y, acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(w.z, x.z, acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(w.w, x.w, acc, 0, 0, 0);
}

__device__ __forceinline__ float4 zero4() { return make_float4(0.f, 0.f, 0.f, 0.f); }

// rows [0, B) x columns [0, cols) of a row-major matrix into LDS rows of pitch XS; the rest of the 32 x cols8 block
// (cols8 = cols rounded up to 8) is zero
__device__ __forceinline__ void stage_rows(float* xs, const float* src, int ld, int B, int cols, int tid, int nt) {
  const int c4n = (cols + 7) / 8 * 2;  // float4 groups per row
  for (int i = tid; i < 32 * c4n; i += nt) {
    const int m = i / c4n, c = (i % c4n) * 4;
    float4 v = zero4();
    if (m < B) {
      const float* r = src + (size_t)m * ld + c;
      if (c + 4 <= cols) v = *reinterpret_cast<const float4*>(r);
      else {
        if (c < cols) v.x = r[0];
        if (c + 1 < cols) v.y = r[1];
        if (c + 2 < cols) v.z = r[2];
      }
    }
    *reinterpret_cast<float4*>(&xs[m * XS + c]) = v;
  }
}

// ---- forward: units [u0, u1) of one model per workgroup (8 waves; wave w owns output columns [32w, 32w+32)) ------
__global__ __launch_bounds__(512) void mlp_fwd_fused_kernel(const MlpFusedArgs a) {
  __shared__ float xs[32 * XS];
  __shared__ float rl[32];
  const int g = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lrow = lane & 31, lgrp = lane >> 5;
  const MlpTab* tb = a.tab[g];
  const float* P = a.p[g];
  const int n0 = wave * 32, n = n0 + lrow;
  // this lane's chunks of row n of W_u: all K/8 requests of a layer in flight together
  float4 wf[MAXK8];
  auto load_w = [&](int u) {
    const int K = u == 0 ? a.d_in : a.d, N = u < a.L ? a.d : a.n_out;
    const float* W = P + a.w_off[u];
#pragma unroll
    for (int s = 0; s < MAXK8; ++s)
      wf[s] = (8 * s < K && n < N) ? *reinterpret_cast<const float4*>(W + (size_t)n * K + 8 * s + 4 * lgrp) : zero4();
  };
  load_w(a.u0);  // in flight while the input rows are staged
  stage_rows(xs, a.u0 == 0 ? a.x[g] : tb->h[a.u0 - 1], a.u0 == 0 ? a.ld_in : a.ldd, a.B, a.u0 == 0 ? a.d_in : a.d, tid, 512);
  __syncthreads();
  for (int u = a.u0; u < a.u1; ++u) {
    const int K = u == 0 ? a.d_in : a.d, N = u < a.L ? a.d : a.n_out;
    const float* bias = P + a.b_off[u];
    const bool active = n0 < N;  // uniform over the wave
    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    float bv[4][4];
    if (active) {
#pragma unroll
      for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int nn = n0 + 8 * q + 4 * lgrp + e;
          bv[q][e] = nn < N ? bias[nn] : 0.f;
        }
#pragma unroll
      for (int s = 0; s < MAXK8; ++s)
        if (8 * s < K) mma4(acc, wf[s], *reinterpret_cast<const float4*>(&xs[lrow * XS + 8 * s + 4 * lgrp]));
    }
    if (u + 1 < a.u1) load_w(u + 1);  // the next layer's weights travel while this layer's outputs are finished
    // a lane holds, for row m = lrow, columns n0 + 8q + 4 lgrp + (0..3), q = 0..3
    float v[4][4];
    if (active) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int nq = n0 + 8 * q + 4 * lgrp;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          v[q][e] = acc[4 * q + e];
          if (nq + e < N) v[q][e] += bv[q][e];
        }
      }
    }
    __syncthreads();  // every wave has read this layer's input from LDS
    if (active) {
      const int m = lrow;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int nq = n0 + 8 * q + 4 * lgrp;
        if (nq >= N) continue;
        if (u < a.L) {
          float h[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) h[e] = act_fwd(v[q][e], a.act);
          if (m < a.B) {  // N = d is a multiple of 8: whole vectors
            *reinterpret_cast<float4*>(tb->z[u] + (size_t)m * a.ldd + nq) = make_float4(v[q][0], v[q][1], v[q][2], v[q][3]);
            *reinterpret_cast<float4*>(tb->h[u] + (size_t)m * a.ldd + nq) = make_float4(h[0], h[1], h[2], h[3]);
          }
          *reinterpret_cast<float4*>(&xs[m * XS + nq]) = make_float4(h[0], h[1], h[2], h[3]);
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (nq + e < N) {
              if (m < a.B) tb->logits[(size_t)m * a.ldv + nq + e] = v[q][e];
              xs[m * XS + nq + e] = v[q][e];
            }
        }
      }
    }
    __syncthreads();
    if (u == a.L) {
      // softmax cross-entropy of the 32 rows: lane m of the first wave walks its row in ascending class order
      const int C = a.n_out;
      if (wave == 0 && lane < 32) {
        const int m = lane;
        float rowloss = 0.f;
        if (m < a.B) {
          const float* z = &xs[m * XS];
          const int y = a.labels[m];
          float mx = -INFINITY;
          for (int c = 0; c < C; ++c) mx = fmaxf(mx, z[c]);
          float sum = 0.f;
          for (int c = 0; c < C; ++c) sum += expf(z[c] - mx);
          const float lse = logf(sum) + mx, inv_sum = 1.f / sum;
          float* dz = tb->dlogits + (size_t)m * a.ldv;
          for (int c = 0; c < a.ldv; ++c) dz[c] = c < C ? (expf(z[c] - mx) * inv_sum - (c == y ? 1.f : 0.f)) * a.inv_n : 0.f;
          rowloss = lse - z[y];
          tb->rowloss[m] = rowloss;
        }
        rl[m] = rowloss;
      }
      __syncthreads();
      if (tid == 0) {
        float t = 0.f;
        for (int m = 0; m < a.B; ++m) t += rl[m];  // ascending rows
        *a.loss[g] = t * a.inv_n;
      }
    }
  }
}

// ---- backward, part 1: dz_{u-1} = (dz_u W_u) * act'(z_{u-1}) for u = u1-1 ... max(u0, 1), one model per workgroup ----
__global__ __launch_bounds__(512) void mlp_dgrad_chain_kernel(const MlpFusedArgs a) {
  __shared__ float ds[32 * XS];
  const int g = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lrow = lane & 31, lgrp = lane >> 5;
  const MlpTab* tb = a.tab[g];
  const float* P = a.p[g];
  const int u_hi = a.u1 - 1, u_lo = a.u0 > 1 ? a.u0 : 1;
  if (u_hi < u_lo) return;
  const int n0 = wave * 32, n = n0 + lrow;
  const int Kin = a.d;                      // width of dz_{u-1} (u >= 1)
  const bool active = n0 < Kin;
  // W_u[k][n] for this lane's column n and the four rows k = 8s + 4 lgrp + (0..3) of every group s: buffer loads
  // with the row offset as the uniform part of the address; rows at or past K and columns at or past Kin lie
  // outside the descriptor and read as zero.  gate = z_{u-1} at the outputs this lane will hold.
  float4 wf[MAXK8], gate[4];
  auto load_w = [&](int u) {
    const int K = u < a.L ? a.d : a.n_out;  // width of dz_u: the sum runs over it
    const __amdgpu_buffer_rsrc_t rs =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(P + a.w_off[u]), 0, K * Kin * 4, 0x00020000);
    const int voff = n < Kin ? (4 * lgrp * Kin + n) * 4 : 0x7ffffff0;
#pragma unroll
    for (int s = 0; s < MAXK8; ++s) {
      wf[s] = zero4();
      if (8 * s < K) {
        const int so = 8 * s * Kin * 4, row = Kin * 4;
        wf[s].x = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, voff, so, 0));
        wf[s].y = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, voff, so + row, 0));
        wf[s].z = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, voff, so + 2 * row, 0));
        wf[s].w = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, voff, so + 3 * row, 0));
      }
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int nq = n0 + 8 * q + 4 * lgrp;
      gate[q] = (lrow < a.B && nq < Kin) ? *reinterpret_cast<const float4*>(tb->z[u - 1] + (size_t)lrow * a.ldd + nq) : zero4();
    }
  };
  if (active) load_w(u_hi);
  stage_rows(ds, u_hi < a.L ? tb->dz[u_hi] : tb->dlogits, u_hi < a.L ? a.ldd : a.ldv, a.B, u_hi < a.L ? a.d : a.n_out, tid, 512);
  __syncthreads();
  for (int u = u_hi; u >= u_lo; --u) {
    const int K = u < a.L ? a.d : a.n_out;
    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    float4 gz4[4];
    if (active) {
#pragma unroll
      for (int s = 0; s < MAXK8; ++s)
        if (8 * s < K) mma4(acc, wf[s], *reinterpret_cast<const float4*>(&ds[lrow * XS + 8 * s + 4 * lgrp]));
#pragma unroll
      for (int q = 0; q < 4; ++q) gz4[q] = gate[q];
      if (u - 1 >= u_lo) load_w(u - 1);  // the next unit's weights travel while this unit's outputs are finished
    }
    __syncthreads();  // every wave has read dz_u from LDS
    if (active) {
      const int m = lrow;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int nq = n0 + 8 * q + 4 * lgrp;
        if (nq >= Kin) continue;
        const float gz[4] = {gz4[q].x, gz4[q].y, gz4[q].z, gz4[q].w};
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = acc[4 * q + e] * act_grad(gz[e], a.act);
        const float4 o = make_float4(v[0], v[1], v[2], v[3]);
        if (m < a.B) *reinterpret_cast<float4*>(tb->dz[u - 1] + (size_t)m * a.ldd + nq) = o;
        *reinterpret_cast<float4*>(&ds[m * XS + nq]) = m < a.B ? o : zero4();
      }
    }
    __syncthreads();
  }
}

// ---- backward, part 2: dW_u = dz_u^T x_u with the update of W_u and b_u, for every unit of the shard -----------------
// grid (strip of 32 output rows, unit, model); wave w takes the 32-column tiles w, w+4 of the strip
template <int OPT>
__global__ __launch_bounds__(256) void mlp_wgrad_update_kernel(const MlpFusedArgs a) {
  const int strip = blockIdx.x, u = a.u0 + blockIdx.y, g = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lrow = lane & 31, lgrp = lane >> 5;
  const int N = u < a.L ? a.d : a.n_out, Kin = u == 0 ? a.d_in : a.d;
  if (strip * 32 >= N) return;
  const MlpTab* tb = a.tab[g];
  const float* dz = u < a.L ? tb->dz[u] : tb->dlogits;
  const int lddz = u < a.L ? a.ldd : a.ldv;
  const float* xin = u == 0 ? a.x[g] : tb->h[u - 1];
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

hipError_t launch_mlp_fwd_fused(const MlpFusedArgs& a, hipStream_t s) {
  hipError_t e = check(a);
  if (e != hipSuccess) return e;
  if (a.u1 == a.L + 1)
    for (int g = 0; g < a.G; ++g)
      if (!a.loss[g] || !a.labels) return hipErrorInvalidValue;
  hipLaunchKernelGGL(mlp_fwd_fused_kernel, dim3(a.G), dim3(512), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_mlp_dgrad_chain(const MlpFusedArgs& a, hipStream_t s) {
  hipError_t e = check(a);
  if (e != hipSuccess) return e;
  if (a.u1 - 1 < (a.u0 > 1 ? a.u0 : 1)) return hipSuccess;  // no unit of the shard has an input gradient to produce
  hipLaunchKernelGGL(mlp_dgrad_chain_kernel, dim3(a.G), dim3(512), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_mlp_wgrad_update(const MlpFusedArgs& a, hipStream_t s) {
  hipError_t e = check(a);
  if (e != hipSuccess) return e;
  for (int g = 0; g < a.G; ++g) {
    if (a.keep_grads ? !a.g[g] : (a.opt == 1 && (!a.m[g] || !a.v[g]))) return hipErrorInvalidValue;
  }
  const int widest = a.d > a.n_out ? a.d : a.n_out;
  const dim3 grid((widest + 31) / 32, a.u1 - a.u0, a.G);
  if (a.opt == 1) hipLaunchKernelGGL(mlp_wgrad_update_kernel<1>, grid, dim3(256), 0, s, a);
  else hipLaunchKernelGGL(mlp_wgrad_update_kernel<0>, grid, dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace hydra
