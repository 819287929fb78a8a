// Shard executor for MLP models: forward, backward and update of layer units [u0,u1) for a launch
// group of same-shaped shards of different models (paper, Introduction, "Motivation": features are
// sent layer to layer in the forward pass, gradients in the backward pass).
//
// unit l < L:  z_l = x_l W_l^T + b_l,  h_l = act(z_l),  x_{l+1} = h_l          (x_0 = the batch)
// unit L:      logits = x_L W_out^T + b_out, softmax cross-entropy
// backward of unit l given dz_l:  dW_l = dz_l^T x_l;  db_l = column sums of dz_l (same launch);
//                                 dz_{l-1} = (dz_l W_l) * act'(z_{l-1})         (l > 0)
#include <algorithm>
#include <cmath>

#include "hydra_internal.h"

namespace hydra {

static int rup8(int v) { return (v + 7) / 8 * 8; }

static const Tensor& W_of(const Model& m, int u) { return m.tensors[2 * u]; }
static const Tensor& b_of(const Model& m, int u) { return m.tensors[2 * u + 1]; }

// pointer to tensor `t` inside the shard's state block `base` (same offsets for p, g and w16)
template <typename T>
static T* at(T* base, const Shard& sh, const Tensor& t) { return base + (t.off - sh.off); }

// Small fp32 models (at most 32 rows per step, layers at most 256 wide) run whole shard phases in one launch each
// (mlp_fused.hip); the choice depends on the architecture and the batch alone, never on cuts, groups or policy.
bool mlp_runs_fused(const hydra_ctx* c, const Model& m) {
  const hydra_arch& a = m.arch;
  return a.kind == HYDRA_KIND_MLP && a.dtype == HYDRA_DTYPE_F32 && !c->spill &&
         mlp_fused_shape_ok(c->B, a.d_in, a.d_model, a.n_out, a.n_layers + 1);
}

static void fill_fused(hydra_ctx* c, const Bucket& b, int batch, int step, MlpFusedArgs& f) {
  const Model& m0 = c->models[b.members[0].first];
  const Shard& sh0 = m0.shards[b.members[0].second];
  const hydra_arch& a = m0.arch;
  f = MlpFusedArgs{};
  f.G = (int)b.members.size();
  f.B = c->B;
  f.d_in = a.d_in;
  f.d = a.d_model;
  f.n_out = a.n_out;
  f.L = a.n_layers;
  // the units of all the shards the group covers (a backward group lists its highest shard)
  const Shard& sh_lo = m0.shards[b.ph == HYDRA_PHASE_B ? b.shard_at(0, b.span - 1) : b.members[0].second];
  const Shard& sh_hi = m0.shards[b.ph == HYDRA_PHASE_B ? b.members[0].second : b.shard_at(0, b.span - 1)];
  f.u0 = sh_lo.u0;
  f.u1 = sh_hi.u1;
  f.act = a.act == HYDRA_ACT_RELU ? EPI_ACT_RELU : EPI_ACT_GELU;
  f.opt = m0.hp.opt == HYDRA_OPT_ADAM ? 1 : 0;
  f.keep_grads = c->fuse ? 0 : 1;
  f.ld_in = c->ld_in;
  f.ldd = rup8(a.d_model);
  f.ldv = rup8(a.n_out);
  for (int u = 0; u <= a.n_layers; ++u) {
    f.w_off[u] = (unsigned)W_of(m0, u).off;
    f.b_off[u] = (unsigned)b_of(m0, u).off;
  }
  f.inv_n = 1.0f / (float)c->B;
  f.labels = c->targets + (size_t)batch * c->B;
  for (int i = 0; i < f.G; ++i) {
    const Model& m = c->models[b.members[i].first];
    f.p[i] = m.p;
    f.g[i] = m.g;
    f.m[i] = m.m;
    f.v[i] = m.v;
    f.tab[i] = m.mlp.tab;
    f.x[i] = static_cast<const float*>(c->x_staged) + (size_t)batch * c->B * c->ld_in;
    f.loss[i] = m.loss_dev + step;
    f.hp[i] = step_hparams(m, step);
  }
}

// algorithmic flops of the products of units [u_lo, u_hi) for one model: 2 * rows * in * out each
static double unit_flops(const hydra_ctx* c, const hydra_arch& a, int u_lo, int u_hi) {
  double f = 0;
  for (int u = u_lo; u < u_hi; ++u)
    f += 2.0 * c->B * (u == 0 ? a.d_in : a.d_model) * (u < a.n_layers ? a.d_model : a.n_out);
  return f;
}

// the second launch of a small MLP's backward tasks: every weight gradient of units [f.u0, f.u1) with the update
static hydra_status mlp_fused_gradients(hydra_ctx* c, const Bucket& b, const MlpFusedArgs& f, hipStream_t s) {
  const hydra_arch& a0 = c->models[b.members[0].first].arch;
  double bytes = 0;
  for (int u = f.u0; u < f.u1; ++u) {
    const double in = u == 0 ? a0.d_in : a0.d_model, out = u < a0.n_layers ? a0.d_model : a0.n_out;
    bytes += fused_update_bytes(f.opt, false) * in * out + 4.0 * c->B * (in + out);
  }
  HYDRA_LAUNCH(c, c->fuse ? HYDRA_K_WGRAD_UPDATE : HYDRA_K_GEMM_WGRAD, s, unit_flops(c, a0, f.u0, f.u1) * f.G,
               c->fuse ? bytes * f.G : 0.0, launch_mlp_wgrad_update(f, s));
  return HYDRA_OK;
}

static hydra_status mlp_forward(hydra_ctx* c, const Bucket& b, int batch, int step, hipStream_t s) {
  const Model& m0 = c->models[b.members[0].first];
  if (mlp_runs_fused(c, m0)) {
    MlpFusedArgs f;
    fill_fused(c, b, batch, step, f);
    if (b.bspan > 0) {
      // the group also covers the backward tasks: forward and the chain of input gradients in one launch, then the
      // gradients with the update
      const hydra_arch& a0 = m0.arch;
      HYDRA_LAUNCH2(c, HYDRA_K_GEMM_FWD, HYDRA_K_GEMM_DGRAD, s, unit_flops(c, a0, f.u0, f.u1) * f.G,
                    unit_flops(c, a0, 1, f.u1) * f.G, 0.0, launch_mlp_fwd_chain(f, s));
      return mlp_fused_gradients(c, b, f, s);
    }
    HYDRA_LAUNCH(c, HYDRA_K_GEMM_FWD, s, unit_flops(c, m0.arch, f.u0, f.u1) * f.G, 0.0, launch_mlp_fwd_fused(f, s));
    return HYDRA_OK;
  }
  const Shard& sh0 = m0.shards[b.members[0].second];
  const hydra_arch& a = m0.arch;
  const bool bf = a.dtype == HYDRA_DTYPE_BF16;
  const size_t es = bf ? 2 : 4;
  const int L = a.n_layers, G = (int)b.members.size();
  const int ldd = rup8(a.d_model), ldv = rup8(a.n_out);
  for (int u = sh0.u0; u < sh0.u1; ++u) {
    GemmArgs g{};
    g.dtype = bf ? GEMM_BF16 : GEMM_F32;
    g.M = c->B;
    g.N = u < L ? a.d_model : a.n_out;
    g.K = u == 0 ? a.d_in : a.d_model;
    g.x_kmajor = g.w_kmajor = 1;
    g.ldx = u == 0 ? c->ld_in : ldd;
    g.ldw = W_of(m0, u).cols;
    g.G = G;
    g.ldo = u < L ? ldd : ldv;
    g.act = u < L ? (a.act == HYDRA_ACT_RELU ? EPI_ACT_RELU : EPI_ACT_GELU) : EPI_ACT_NONE;
    g.out_f32 = u < L ? 0 : 1;
    for (int i = 0; i < G; ++i) {
      const Model& m = c->models[b.members[i].first];
      const Shard& sh = m.shards[b.members[i].second];
      g.X[i] = u == 0 ? static_cast<const char*>(c->x_staged) + (size_t)batch * c->B * c->ld_in * es : m.mlp.h[u - 1];
      g.W[i] = bf ? (const void*)at(sh.w16, sh, W_of(m, u)) : (const void*)at(sh.p, sh, W_of(m, u));
      g.bias[i] = c->spill ? m.pv + m.voff[2 * u + 1] : at(sh.p, sh, b_of(m, u));
      if (u < L) {
        g.out[i] = m.mlp.h[u];
        g.pre[i] = m.mlp.z[u];
      } else {
        g.out[i] = m.mlp.logits;
      }
    }
    HYDRA_LAUNCH(c, HYDRA_K_GEMM_FWD, s, 2.0 * g.M * g.N * g.K * G, 0.0, launch_gemm(g, s));
    if (u == L) {
      SoftmaxCeArgs ce{};
      ce.dtype = g.dtype;
      ce.M = c->B;
      ce.C = a.n_out;
      ce.ldz = ce.lddz = ldv;
      ce.G = G;
      ce.inv_n = 1.0f / (float)c->B;
      ce.labels = c->targets + (size_t)batch * c->B;
      for (int i = 0; i < G; ++i) {
        const Model& m = c->models[b.members[i].first];
        ce.logits[i] = m.mlp.logits;
        ce.dz[i] = m.mlp.dlogits;
        ce.rowloss[i] = m.mlp.rowloss;
        ce.loss_out[i] = m.loss_dev + step;
      }
      ++c->launches;  // the row kernel and the reduction are two launches
      HYDRA_LAUNCH(c, HYDRA_K_SOFTMAX_CE, s, 0.0, (double)G * ce.M * ce.C * (4 + 4 + (bf ? 2 : 4)), launch_softmax_ce(ce, s));
    }
  }
  return HYDRA_OK;
}

static hydra_status mlp_backward(hydra_ctx* c, const Bucket& b, int batch, int step, hipStream_t s) {
  const Model& m0 = c->models[b.members[0].first];
  const Shard& sh0 = m0.shards[b.members[0].second];
  if (mlp_runs_fused(c, m0)) {
    const hydra_arch& a0 = m0.arch;
    MlpFusedArgs f;
    fill_fused(c, b, batch, step, f);
    // input gradients through units u1-1 ... max(u0, 1), before any weight of the shard changes
    const int u_lo = std::max(f.u0, 1);
    if (f.u1 - 1 >= u_lo)
      HYDRA_LAUNCH(c, HYDRA_K_GEMM_DGRAD, s, unit_flops(c, a0, u_lo, f.u1) * f.G, 0.0, launch_mlp_dgrad_chain(f, s));
    return mlp_fused_gradients(c, b, f, s);
  }
  const hydra_arch& a = m0.arch;
  const bool bf = a.dtype == HYDRA_DTYPE_BF16;
  const size_t es = bf ? 2 : 4;
  const int L = a.n_layers, G = (int)b.members.size();
  const int ldd = rup8(a.d_model), ldv = rup8(a.n_out);
  const int act = a.act == HYDRA_ACT_RELU ? EPI_ACT_RELU : EPI_ACT_GELU;
  for (int u = sh0.u1 - 1; u >= sh0.u0; --u) {
    const int N = u < L ? a.d_model : a.n_out;     // width of dz_u
    const int Kin = u == 0 ? a.d_in : a.d_model;   // width of x_u
    const int lddz = u < L ? ldd : ldv;
    // input gradient through the previous activation, before the weights of this unit change:
    // dz_{u-1}[B, Kin] = (dz_u W_u) * act'(z_{u-1})
    if (u > 0) {
      GemmArgs d{};
      d.dtype = bf ? GEMM_BF16 : GEMM_F32;
      d.M = c->B;
      d.N = Kin;
      d.K = N;
      d.x_kmajor = 1;
      d.w_kmajor = 0;
      d.ldx = lddz;
      d.ldw = W_of(m0, u).cols;
      d.G = G;
      d.ldo = d.ldg = ldd;
      d.act = act;
      for (int i = 0; i < G; ++i) {
        const Model& m = c->models[b.members[i].first];
        const Shard& sh = m.shards[b.members[i].second];
        d.X[i] = u < L ? m.mlp.dz[u] : m.mlp.dlogits;
        d.W[i] = bf ? (const void*)at(sh.w16, sh, W_of(m, u)) : (const void*)at(sh.p, sh, W_of(m, u));
        d.out[i] = m.mlp.dz[u - 1];
        d.gate[i] = m.mlp.z[u - 1];
      }
      HYDRA_LAUNCH(c, HYDRA_K_GEMM_DGRAD, s, 2.0 * d.M * d.N * d.K * G, 0.0, launch_gemm(d, s));
    }
    // weight gradient: dW[N, Kin] = sum_m dz[m, N] x[m, Kin]
    GemmArgs w{};
    w.dtype = bf ? GEMM_BF16 : GEMM_F32;
    w.M = N;
    w.N = Kin;
    w.K = c->B;
    w.x_kmajor = w.w_kmajor = 0;
    w.ldx = lddz;
    w.ldw = u == 0 ? c->ld_in : ldd;
    w.G = G;
    w.ldo = W_of(m0, u).cols;
    w.act = EPI_ACT_NONE;
    w.out_f32 = 1;
    for (int i = 0; i < G; ++i) {
      const Model& m = c->models[b.members[i].first];
      const Shard& sh = m.shards[b.members[i].second];
      const void* dz = u < L ? m.mlp.dz[u] : m.mlp.dlogits;
      w.X[i] = dz;
      w.W[i] = u == 0 ? static_cast<const char*>(c->x_staged) + (size_t)batch * c->B * c->ld_in * es : m.mlp.h[u - 1];
      w.out[i] = at(sh.g, sh, W_of(m, u));
      w.rowsum[i] = at(sh.g, sh, b_of(m, u));  // db = column sums of dz, from the GEMM's own dz fragments
    }
    if (c->fuse) {
      // the update of W_u runs in the epilogue of its gradient GEMM; the gradient is never stored
      GemmUpdate up{};
      up.opt = m0.hp.opt == HYDRA_OPT_ADAM ? 1 : 0;
      for (int i = 0; i < G; ++i) {
        const Model& m = c->models[b.members[i].first];
        const Shard& sh = m.shards[b.members[i].second];
        w.out[i] = nullptr;
        up.p[i] = at(sh.p, sh, W_of(m, u));
        up.m[i] = sh.m ? at(sh.m, sh, W_of(m, u)) : nullptr;
        up.v[i] = sh.v ? at(sh.v, sh, W_of(m, u)) : nullptr;
        up.w16[i] = sh.w16 ? at(sh.w16, sh, W_of(m, u)) : nullptr;
        up.hp[i] = step_hparams(m, step);
      }
      HYDRA_LAUNCH(c, HYDRA_K_WGRAD_UPDATE, s, 2.0 * w.M * w.N * w.K * G,
                   (fused_update_bytes(up.opt, bf) * w.M * w.N + (double)es * w.K * (w.M + w.N)) * G, launch_gemm_update(w, up, s));
    } else {
      HYDRA_LAUNCH(c, HYDRA_K_GEMM_WGRAD, s, 2.0 * w.M * w.N * w.K * G, 0.0, launch_gemm(w, s));
    }
  }
  return HYDRA_OK;
}

OptimHp step_hparams(const Model& m, int step) {
  const long t = m.t + step + 1;
  const double lr = m.hp.warmup_steps > 0 ? m.hp.lr * std::min(1.0, (double)t / m.hp.warmup_steps) : m.hp.lr;
  OptimHp h;
  h.lr = (float)lr;
  h.b1 = (float)m.hp.beta1;
  h.b2 = (float)m.hp.beta2;
  h.c1 = (float)(1.0 - m.hp.beta1);
  h.c2 = (float)(1.0 - m.hp.beta2);
  h.eps = (float)m.hp.eps;
  h.bc1 = (float)(1.0 / (1.0 - std::pow(m.hp.beta1, (double)t)));
  h.bc2 = (float)(1.0 / (1.0 - std::pow(m.hp.beta2, (double)t)));
  return h;
}

hydra_status fill_optim(hydra_ctx* c, const Bucket& b, int step, OptimArgs& o) {
  o = OptimArgs{};
  o.G = (int)b.members.size();
  const Model& m0 = c->models[b.members[0].first];
  o.opt = m0.hp.opt == HYDRA_OPT_ADAM ? 1 : 0;
  o.n = m0.shards[b.members[0].second].n;
  for (int i = 0; i < o.G; ++i) {
    const Model& m = c->models[b.members[i].first];
    const Shard& sh = m.shards[b.members[i].second];
    if ((m.hp.opt == HYDRA_OPT_ADAM) != (o.opt == 1) || sh.n != o.n)
      return c->fail(HYDRA_ERR_BAD_STATE, "launch group mixes optimizers or shard sizes");
    o.p[i] = sh.p;
    o.g[i] = sh.g;
    o.m[i] = sh.m;
    o.v[i] = sh.v;
    o.w16[i] = sh.w16;
    o.hp[i] = step_hparams(m, step);
  }
  return HYDRA_OK;
}

hydra_status run_update(hydra_ctx* c, const Bucket& b, int step, hipStream_t s) {
  OptimArgs o;
  hydra_status st = fill_optim(c, b, step, o);
  if (st != HYDRA_OK) return st;
  size_t n = o.n;
  if (c->fuse) {
    const Shard& sh0 = c->models[b.members[0].first].shards[b.members[0].second];
    if (mlp_runs_fused(c, c->models[b.members[0].first])) return HYDRA_OK;  // weights and biases were updated by the backward task
    if (!sh0.n_tail_chunks) return HYDRA_OK;  // every tensor of the shard was updated by its gradient GEMM
    o.chunks = sh0.tail_chunks;
    o.n_chunks = sh0.n_tail_chunks;
    n = sh0.n_tail;
  }
  // algorithmic traffic per parameter: SGD reads p,g and writes p (12 B); Adam reads p,g,m,v and writes
  // p,m,v (28 B); the bf16 working copy adds 2 B
  const double per = (o.opt == 1 ? 28.0 : 12.0) + (o.w16[0] ? 2.0 : 0.0);
  HYDRA_LAUNCH(c, HYDRA_K_OPTIM, s, 0.0, per * (double)n * o.G, launch_optim(o, s));
  return HYDRA_OK;
}

hydra_status mlp_run(hydra_ctx* c, const Bucket& b, int batch, int step, hipStream_t s) {
  if (b.ph == HYDRA_PHASE_F) return mlp_forward(c, b, batch, step, s);
  if (b.ph == HYDRA_PHASE_B) return mlp_backward(c, b, batch, step, s);
  return run_update(c, b, step, s);
}

}  // namespace hydra
