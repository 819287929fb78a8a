// Shard executor for pre-LN Transformer models (bf16): forward, backward and update of blocks
// [u0,u1) for a launch group of same-shaped shards of different models.  Unit 0 also embeds the
// tokens; the last unit also applies the final LayerNorm, the output Linear on the target rows and
// the loss.  Features flow block to block forward and gradients backward (paper, Introduction,
// "Motivation"); the hand-off between shards of a model is the device buffer x[u] / dx[u].
//
// block l:  a = LN1(x);  qkv = a Wqkv^T + b;  o = attention(qkv);  x1 = x + o Wo^T + bo;
//           f = LN2(x1);  hmid = GeLU(f W1^T + b1)          (plain)
//                         hmid = GeLU(f Wg^T + bg) * (f W1^T + b1)   (gated)
//           x' = x1 + hmid W2^T + b2
#include <cmath>

#include "hydra_internal.h"

namespace hydra {

namespace {

int rup8(int v) { return (v + 7) / 8 * 8; }

// tensor indices inside a model (canonical order)
struct Idx {
  int per, L;
  explicit Idx(const hydra_arch& a) : per(a.ffn_gated ? 14 : 12), L(a.n_layers) {}
  int blk(int l, int j) const { return 2 + per * l + j; }
  int ln1g(int l) const { return blk(l, 0); }
  int ln1b(int l) const { return blk(l, 1); }
  int wqkv(int l) const { return blk(l, 2); }
  int bqkv(int l) const { return blk(l, 3); }
  int wo(int l) const { return blk(l, 4); }
  int bo(int l) const { return blk(l, 5); }
  int ln2g(int l) const { return blk(l, 6); }
  int ln2b(int l) const { return blk(l, 7); }
  int w1(int l) const { return blk(l, 8); }
  int b1(int l) const { return blk(l, 9); }
  int wg(int l) const { return blk(l, 10); }
  int bg(int l) const { return blk(l, 11); }
  int w2(int l) const { return blk(l, per - 2); }
  int b2(int l) const { return blk(l, per - 1); }
  int lnfg() const { return 2 + per * L; }
  int lnfb() const { return 3 + per * L; }
  int whead() const { return 4 + per * L; }
  int bhead() const { return 5 + per * L; }
};

struct Ctx {
  hydra_ctx* c;
  const Bucket& b;
  hipStream_t s;
  int G, Tk, NT, d, F, V, H, DH, ldv;
  const hydra_arch& a;
  Idx ix;
  Ctx(hydra_ctx* c_, const Bucket& b_, hipStream_t s_)
      : c(c_), b(b_), s(s_), a(c_->models[b_.members[0].first].arch), ix(a) {
    G = (int)b.members.size();
    Tk = c->B * c->S;
    NT = c->B * c->P;
    d = a.d_model;
    F = a.d_ffn;
    V = a.n_out;
    H = a.n_heads;
    DH = d / H;
    ldv = rup8(V);
  }
  const Model& model(int i) const { return c->models[b.members[i].first]; }
  const Shard& shard(int i) const { return model(i).shards[b.members[i].second]; }
  // Where member i keeps the activations of its shard.  Normally everything is the model's own; in recomputation
  // mode only the shard's input and output (and their gradients) are, and the rest is the workspace of
  // (stream, position in the group).
  const TrWorkspace* wsp(int i) const { return c->recompute ? &c->ws[(size_t)b.stream * c->ws_group + i] : nullptr; }
  void* xin(int i, int r) const {   // input of the shard's r-th block; r = number of blocks: the shard's output
    const Shard& sh = shard(i);
    if (!c->recompute || r == 0 || r == sh.u1 - sh.u0) return model(i).tr.x[sh.u0 + r];
    return wsp(i)->xi[r];
  }
  void* dxin(int i, int r) const {
    const Shard& sh = shard(i);
    if (!c->recompute || r == 0 || r == sh.u1 - sh.u0) return model(i).tr.dx[sh.u0 + r];
    return wsp(i)->dxi[r];
  }
  const TrBlockActs& blk(int i, int r) const { return c->recompute ? wsp(i)->blk[r] : model(i).tr.blk[shard(i).u0 + r]; }
  const TrActs& scratch(int i) const { return c->recompute ? wsp(i)->sc : model(i).tr; }
  // pointers into the shard's state blocks for tensor j of member i
  const bf16_t* w16(int i, int j) const { return shard(i).w16 + (model(i).tensors[j].off - shard(i).off); }
  // fp32 vector tensors (biases, LayerNorm gains): the resident copy when the state is spilled
  const float* p32(int i, int j) const {
    if (c->spill) return model(i).pv + model(i).voff[j];
    return shard(i).p + (model(i).tensors[j].off - shard(i).off);
  }
  float* g32(int i, int j) const { return shard(i).g + (model(i).tensors[j].off - shard(i).off); }
};

}  // namespace

#define FOR_G for (int i = 0; i < x.G; ++i)

static hydra_status tr_forward(Ctx& x, int batch, int step) {
  hydra_ctx* c = x.c;
  const int n_units = x.shard(0).u1 - x.shard(0).u0;
  const int Tk = x.Tk, d = x.d, F = x.F;
  const bool first = x.shard(0).u0 == 0, last = x.shard(0).u1 == x.a.n_layers;
  if (first) {
    EmbedArgs e{};
    e.dtype = GEMM_BF16; e.tokens = Tk; e.S = c->S; e.d = d; e.ld = d; e.G = x.G;
    e.ids = c->ids + (size_t)batch * Tk;
    FOR_G { e.tok[i] = x.w16(i, 0); e.pos[i] = x.w16(i, 1); e.x[i] = x.xin(i, 0); }
    HYDRA_LAUNCH(c, HYDRA_K_EMBED, x.s, 0.0, (double)x.G * Tk * d * 2 * 3, launch_embed_fwd(e, x.s));
  }
  for (int r = 0; r < n_units; ++r) {
    auto L = [&](int i) { return x.shard(i).u0 + r; };
    auto A = [&](int i) -> const TrBlockActs& { return x.blk(i, r); };
    // a = LN1(x)
    LnArgs ln{};
    ln.dtype = GEMM_BF16; ln.rows = Tk; ln.d = d; ln.ld = d; ln.G = x.G; ln.eps = 1e-5f;
    FOR_G {
      ln.x[i] = x.xin(i, r); ln.y[i] = A(i).a; ln.gamma[i] = x.p32(i, x.ix.ln1g(L(i)));
      ln.beta[i] = x.p32(i, x.ix.ln1b(L(i))); ln.mean[i] = A(i).mu1; ln.rstd[i] = A(i).rs1;
    }
    HYDRA_LAUNCH(c, HYDRA_K_LAYERNORM, x.s, 0.0, (double)x.G * Tk * d * 4, launch_ln_fwd(ln, x.s));
    // qkv = a Wqkv^T + bqkv
    GemmArgs q{};
    q.dtype = GEMM_BF16; q.M = Tk; q.N = 3 * d; q.K = d; q.x_kmajor = q.w_kmajor = 1; q.ldx = d; q.ldw = d; q.ldo = 3 * d; q.G = x.G;
    FOR_G { q.X[i] = A(i).a; q.W[i] = x.w16(i, x.ix.wqkv(L(i))); q.bias[i] = x.p32(i, x.ix.bqkv(L(i))); q.out[i] = A(i).qkv; }
    HYDRA_LAUNCH(c, HYDRA_K_GEMM_FWD, x.s, 2.0 * q.M * q.N * q.K * x.G, 0.0, launch_gemm(q, x.s));
    // o = attention(q, k, v)
    AttnArgs at{};
    at.B = c->B; at.S = c->S; at.H = x.H; at.DH = x.DH; at.ld_qkv = 3 * d; at.ld_o = d; at.causal = x.a.causal; at.G = x.G;
    at.scale = (float)(1.0 / std::sqrt((double)x.DH));
    FOR_G {
      at.qkv[i] = static_cast<const bf16_t*>(A(i).qkv); at.o[i] = static_cast<bf16_t*>(A(i).o); at.lse[i] = A(i).lse;
    }
    const double att_fl = 4.0 * c->B * x.H * (double)c->S * c->S * x.DH * (x.a.causal ? 0.5 : 1.0) * x.G;
    HYDRA_LAUNCH(c, HYDRA_K_ATTENTION, x.s, att_fl, 0.0, launch_attn_fwd(at, x.s));
    // x1 = x + o Wo^T + bo
    GemmArgs o{};
    o.dtype = GEMM_BF16; o.M = Tk; o.N = d; o.K = d; o.x_kmajor = o.w_kmajor = 1; o.ldx = d; o.ldw = d; o.ldo = d; o.ldr = d; o.G = x.G;
    FOR_G {
      o.X[i] = A(i).o; o.W[i] = x.w16(i, x.ix.wo(L(i))); o.bias[i] = x.p32(i, x.ix.bo(L(i)));
      o.resid[i] = x.xin(i, r); o.out[i] = A(i).x1;
    }
    HYDRA_LAUNCH(c, HYDRA_K_GEMM_FWD, x.s, 2.0 * o.M * o.N * o.K * x.G, 0.0, launch_gemm(o, x.s));
    // f = LN2(x1)
    FOR_G {
      ln.x[i] = A(i).x1; ln.y[i] = A(i).f; ln.gamma[i] = x.p32(i, x.ix.ln2g(L(i))); ln.beta[i] = x.p32(i, x.ix.ln2b(L(i)));
      ln.mean[i] = A(i).mu2; ln.rstd[i] = A(i).rs2;
    }
    HYDRA_LAUNCH(c, HYDRA_K_LAYERNORM, x.s, 0.0, (double)x.G * Tk * d * 4, launch_ln_fwd(ln, x.s));
    // feed-forward
    GemmArgs f1{};
    f1.dtype = GEMM_BF16; f1.M = Tk; f1.N = F; f1.K = d; f1.x_kmajor = f1.w_kmajor = 1; f1.ldx = d; f1.ldw = d; f1.ldo = F; f1.G = x.G;
    if (!x.a.ffn_gated) {
      f1.act = EPI_ACT_GELU;
      FOR_G {
        f1.X[i] = A(i).f; f1.W[i] = x.w16(i, x.ix.w1(L(i))); f1.bias[i] = x.p32(i, x.ix.b1(L(i)));
        f1.pre[i] = A(i).z1; f1.out[i] = A(i).hmid;
      }
      HYDRA_LAUNCH(c, HYDRA_K_GEMM_FWD, x.s, 2.0 * f1.M * f1.N * f1.K * x.G, 0.0, launch_gemm(f1, x.s));
    } else {
      FOR_G { f1.X[i] = A(i).f; f1.W[i] = x.w16(i, x.ix.w1(L(i))); f1.bias[i] = x.p32(i, x.ix.b1(L(i))); f1.out[i] = A(i).z1; }
      HYDRA_LAUNCH(c, HYDRA_K_GEMM_FWD, x.s, 2.0 * f1.M * f1.N * f1.K * x.G, 0.0, launch_gemm(f1, x.s));
      GemmArgs fg = f1;
      fg.act = EPI_ACT_GELU;
      FOR_G {
        fg.W[i] = x.w16(i, x.ix.wg(L(i))); fg.bias[i] = x.p32(i, x.ix.bg(L(i))); fg.pre[i] = A(i).zg;
        fg.mul[i] = A(i).z1; fg.out[i] = A(i).hmid;
      }
      HYDRA_LAUNCH(c, HYDRA_K_GEMM_FWD, x.s, 2.0 * fg.M * fg.N * fg.K * x.G, 0.0, launch_gemm(fg, x.s));
    }
    // x' = x1 + hmid W2^T + b2
    GemmArgs f2{};
    f2.dtype = GEMM_BF16; f2.M = Tk; f2.N = d; f2.K = F; f2.x_kmajor = f2.w_kmajor = 1; f2.ldx = F; f2.ldw = F; f2.ldo = d; f2.ldr = d; f2.G = x.G;
    FOR_G {
      f2.X[i] = A(i).hmid; f2.W[i] = x.w16(i, x.ix.w2(L(i))); f2.bias[i] = x.p32(i, x.ix.b2(L(i)));
      f2.resid[i] = A(i).x1; f2.out[i] = x.xin(i, r + 1);
    }
    HYDRA_LAUNCH(c, HYDRA_K_GEMM_FWD, x.s, 2.0 * f2.M * f2.N * f2.K * x.G, 0.0, launch_gemm(f2, x.s));
  }
  if (last) {
    const int NT = x.NT, V = x.V;
    LnArgs ln{};
    ln.dtype = GEMM_BF16; ln.rows = Tk; ln.d = d; ln.ld = d; ln.G = x.G; ln.eps = 1e-5f;
    FOR_G {
      const Model& m = x.model(i);
      const TrActs& sc = x.scratch(i);
      ln.x[i] = x.xin(i, n_units); ln.y[i] = sc.xf; ln.gamma[i] = x.p32(i, Idx(m.arch).lnfg());
      ln.beta[i] = x.p32(i, Idx(m.arch).lnfb()); ln.mean[i] = sc.muf; ln.rstd[i] = sc.rsf;
    }
    HYDRA_LAUNCH(c, HYDRA_K_LAYERNORM, x.s, 0.0, (double)x.G * Tk * d * 4, launch_ln_fwd(ln, x.s));
    RowsArgs ga{};
    ga.dtype = GEMM_BF16; ga.n = NT; ga.d = d; ga.ld_src = d; ga.ld_dst = d; ga.G = x.G;
    ga.rows = c->tgt_pos + (size_t)batch * NT;
    FOR_G { ga.src[i] = x.scratch(i).xf; ga.dst[i] = x.scratch(i).xt; }
    HYDRA_LAUNCH(c, HYDRA_K_ELEMENTWISE, x.s, 0.0, (double)x.G * NT * d * 4, launch_gather_rows(ga, x.s));
    GemmArgs hd{};
    hd.dtype = GEMM_BF16; hd.M = NT; hd.N = V; hd.K = d; hd.x_kmajor = hd.w_kmajor = 1; hd.ldx = d; hd.ldw = d; hd.ldo = x.ldv;
    hd.out_f32 = 1; hd.G = x.G;
    FOR_G {
      const Model& m = x.model(i);
      hd.X[i] = x.scratch(i).xt; hd.W[i] = x.w16(i, Idx(m.arch).whead()); hd.bias[i] = x.p32(i, Idx(m.arch).bhead());
      hd.out[i] = x.scratch(i).logits;
    }
    HYDRA_LAUNCH(c, HYDRA_K_GEMM_FWD, x.s, 2.0 * hd.M * hd.N * hd.K * x.G, 0.0, launch_gemm(hd, x.s));
    SoftmaxCeArgs ce{};
    ce.dtype = GEMM_BF16; ce.M = NT; ce.C = V; ce.ldz = ce.lddz = x.ldv; ce.G = x.G; ce.inv_n = 1.0f / (float)NT;
    ce.labels = c->targets + (size_t)batch * NT;
    FOR_G {
      const Model& m = x.model(i);
      const TrActs& sc = x.scratch(i);
      ce.logits[i] = sc.logits; ce.dz[i] = sc.dlogits; ce.rowloss[i] = sc.rowloss; ce.loss_out[i] = m.loss_dev + step;
    }
    ++c->launches;
    HYDRA_LAUNCH(c, HYDRA_K_SOFTMAX_CE, x.s, 0.0, (double)x.G * NT * V * 10, launch_softmax_ce(ce, x.s));
  }
  return HYDRA_OK;
}

// weight gradient dW[N_out, K_in] = dy[rows, N_out]^T x_in[rows, K_in] of tensor jw[i] of member i, plus the
// bias gradient = column sums of dy (computed by the same launch from the dy fragments it loads).  In fused-update mode the GEMM's epilogue applies the update of
// the weight, so every reader of the old weight (the matching dgrad) must have been issued before.
static hydra_status wgrad(Ctx& x, int step, int rows, int n_out, int k_in, int ld_dy, int ld_x, const void* const* dy,
                          const void* const* xin, const int* jw, float* const* db) {
  hydra_ctx* c = x.c;
  GemmArgs w{};
  w.dtype = GEMM_BF16; w.M = n_out; w.N = k_in; w.K = rows; w.x_kmajor = w.w_kmajor = 0; w.ldx = ld_dy; w.ldw = ld_x;
  w.ldo = k_in; w.out_f32 = 1; w.G = x.G;
  FOR_G { w.X[i] = dy[i]; w.W[i] = xin[i]; w.out[i] = x.g32(i, jw[i]); w.rowsum[i] = db[i]; w.ws[i] = x.scratch(i).splitk; }
  w.ws_bytes = x.scratch(0).splitk_bytes;
  if (c->fuse) {
    GemmUpdate up{};
    up.opt = x.model(0).hp.opt == HYDRA_OPT_ADAM ? 1 : 0;
    FOR_G {
      const Shard& sh = x.shard(i);
      const size_t o = x.model(i).tensors[jw[i]].off - sh.off;
      w.out[i] = nullptr;
      up.p[i] = sh.p + o;
      up.m[i] = sh.m ? sh.m + o : nullptr;
      up.v[i] = sh.v ? sh.v + o : nullptr;
      up.w16[i] = sh.w16 + o;
      up.hp[i] = step_hparams(x.model(i), step);
    }
    HYDRA_LAUNCH(c, HYDRA_K_WGRAD_UPDATE, x.s, 2.0 * w.M * w.N * w.K * x.G,
                 (fused_update_bytes(up.opt, true) * w.M * w.N + 2.0 * w.K * (w.M + w.N)) * x.G, launch_gemm_update(w, up, x.s));
  } else {
    HYDRA_LAUNCH(c, HYDRA_K_GEMM_WGRAD, x.s, 2.0 * w.M * w.N * w.K * x.G, 0.0, launch_gemm(w, x.s));
  }
  return HYDRA_OK;
}

// input gradient dx[rows, K_in] = dy[rows, N_out] W[N_out, K_in] (+ optional gate / residual in the epilogue)
static hydra_status dgrad(Ctx& x, int rows, int n_out, int k_in, int ld_dy, const void* const* dy, const void* const* W,
                          void* const* dx, const void* const* gate, const void* const* resid) {
  hydra_ctx* c = x.c;
  GemmArgs g{};
  g.dtype = GEMM_BF16; g.M = rows; g.N = k_in; g.K = n_out; g.x_kmajor = 1; g.w_kmajor = 0; g.ldx = ld_dy; g.ldw = k_in;
  g.ldo = g.ldg = g.ldr = k_in; g.act = gate ? EPI_ACT_GELU : EPI_ACT_NONE; g.G = x.G;
  FOR_G {
    g.X[i] = dy[i]; g.W[i] = W[i]; g.out[i] = dx[i];
    g.gate[i] = gate ? gate[i] : nullptr;
    g.resid[i] = resid ? resid[i] : nullptr;
  }
  HYDRA_LAUNCH(c, HYDRA_K_GEMM_DGRAD, x.s, 2.0 * g.M * g.N * g.K * x.G, 0.0, launch_gemm(g, x.s));
  return HYDRA_OK;
}

#define TRY(expr)                      \
  do {                                 \
    hydra_status st_ = (expr);         \
    if (st_ != HYDRA_OK) return st_;   \
  } while (0)

static hydra_status tr_backward(Ctx& x, int batch, int step) {
  hydra_ctx* c = x.c;
  const int n_units = x.shard(0).u1 - x.shard(0).u0;
  const int Tk = x.Tk, d = x.d, F = x.F, G = x.G;
  const bool first = x.shard(0).u0 == 0, last = x.shard(0).u1 == x.a.n_layers;
  const void* pa[MAXG];
  const void* pb[MAXG];
  const void* pc[MAXG];
  const void* pd[MAXG];
  void* po[MAXG];
  int jw[MAXG];
  float* pbias[MAXG];
  if (last) {
    const int NT = x.NT, V = x.V;
    // head: dWhead = dlogits^T xt, dbhead = colsum(dlogits), dxt = dlogits Whead
    FOR_G {
      const Model& m = x.model(i);
      Idx ix(m.arch);
      const TrActs& sc = x.scratch(i);
      pa[i] = sc.dlogits; pb[i] = sc.xt; jw[i] = ix.whead(); pbias[i] = x.g32(i, ix.bhead());
      pc[i] = x.w16(i, ix.whead()); po[i] = sc.dxt;
    }
    TRY(dgrad(x, NT, V, d, x.ldv, pa, pc, po, nullptr, nullptr));
    TRY(wgrad(x, step, NT, V, d, x.ldv, d, pa, pb, jw, pbias));
    // scatter the target rows into a zero [Tk, d] gradient of the final LayerNorm's output
    FOR_G HYDRA_LAUNCH(c, HYDRA_K_ELEMENTWISE, x.s, 0.0, (double)Tk * d * 2,
                       launch_fill_u32(static_cast<uint32_t*>(x.scratch(i).dxf), (size_t)Tk * d / 2, 0u, x.s));
    RowsArgs sc{};
    sc.dtype = GEMM_BF16; sc.n = NT; sc.d = d; sc.ld_src = d; sc.ld_dst = d; sc.G = G;
    sc.rows = c->tgt_pos + (size_t)batch * NT;
    FOR_G { sc.src[i] = x.scratch(i).dxt; sc.dst[i] = x.scratch(i).dxf; }
    HYDRA_LAUNCH(c, HYDRA_K_ELEMENTWISE, x.s, 0.0, (double)G * NT * d * 4, launch_scatter_rows(sc, x.s));
    LnBwdArgs lb{};
    lb.dtype = GEMM_BF16; lb.rows = Tk; lb.d = d; lb.ld = d; lb.G = G;
    FOR_G {
      const Model& m = x.model(i);
      Idx ix(m.arch);
      const TrActs& ws = x.scratch(i);
      lb.x[i] = x.xin(i, n_units); lb.dy[i] = ws.dxf; lb.add[i] = nullptr; lb.dx[i] = x.dxin(i, n_units);
      lb.gamma[i] = x.p32(i, ix.lnfg()); lb.mean[i] = ws.muf; lb.rstd[i] = ws.rsf; lb.part[i] = ws.lnpart;
      lb.dgamma[i] = x.g32(i, ix.lnfg()); lb.dbeta[i] = x.g32(i, ix.lnfb());
    }
    ++c->launches;
    HYDRA_LAUNCH(c, HYDRA_K_LAYERNORM, x.s, 0.0, (double)G * Tk * d * 6, launch_ln_bwd(lb, x.s));
  }
  for (int r = n_units - 1; r >= 0; --r) {
    auto L = [&](int i) { return x.shard(i).u0 + r; };
    auto A = [&](int i) -> const TrBlockActs& { return x.blk(i, r); };
    auto T = [&](int i) -> const TrActs& { return x.scratch(i); };
    // FFN2: dW2 = dx2^T hmid, db2; dh = dx2 W2 (gated by GeLU'(z1) when the block is not gated)
    FOR_G {
      pa[i] = x.dxin(i, r + 1); pb[i] = A(i).hmid; jw[i] = x.ix.w2(L(i)); pbias[i] = x.g32(i, x.ix.b2(L(i)));
      pc[i] = x.w16(i, x.ix.w2(L(i))); pd[i] = A(i).z1;
      po[i] = x.a.ffn_gated ? T(i).dhm : T(i).dz1;
    }
    TRY(dgrad(x, Tk, d, F, d, pa, pc, po, x.a.ffn_gated ? nullptr : pd, nullptr));
    TRY(wgrad(x, step, Tk, d, F, d, F, pa, pb, jw, pbias));
    if (x.a.ffn_gated) {
      GatedBwdArgs gb{};
      gb.dtype = GEMM_BF16; gb.rows = Tk; gb.ld = F; gb.G = G;
      FOR_G { gb.dh[i] = T(i).dhm; gb.z1[i] = A(i).z1; gb.zg[i] = A(i).zg; gb.dz1[i] = T(i).dz1; gb.dzg[i] = T(i).dzg; }
      HYDRA_LAUNCH(c, HYDRA_K_ELEMENTWISE, x.s, 0.0, (double)G * Tk * F * 10, launch_gated_bwd(gb, x.s));
    }
    // FFN1: dW1 = dz1^T f, db1; df = dz1 W1 (+ dzg Wg)
    FOR_G {
      pa[i] = T(i).dz1; pb[i] = A(i).f; jw[i] = x.ix.w1(L(i)); pbias[i] = x.g32(i, x.ix.b1(L(i)));
      pc[i] = x.w16(i, x.ix.w1(L(i))); po[i] = T(i).df;
    }
    TRY(dgrad(x, Tk, F, d, F, pa, pc, po, nullptr, nullptr));
    TRY(wgrad(x, step, Tk, F, d, F, d, pa, pb, jw, pbias));
    if (x.a.ffn_gated) {
      FOR_G {
        pa[i] = T(i).dzg; jw[i] = x.ix.wg(L(i)); pbias[i] = x.g32(i, x.ix.bg(L(i)));
        pc[i] = x.w16(i, x.ix.wg(L(i))); pd[i] = T(i).df;
      }
      TRY(dgrad(x, Tk, F, d, F, pa, pc, po, nullptr, pd));  // df += dzg Wg (read and written by the same lane)
      TRY(wgrad(x, step, Tk, F, d, F, d, pa, pb, jw, pbias));
    }
    // LN2: dx1 = LN2'(df) + dx2
    LnBwdArgs lb{};
    lb.dtype = GEMM_BF16; lb.rows = Tk; lb.d = d; lb.ld = d; lb.G = G;
    FOR_G {
      lb.x[i] = A(i).x1; lb.dy[i] = T(i).df; lb.add[i] = x.dxin(i, r + 1); lb.dx[i] = T(i).dx1;
      lb.gamma[i] = x.p32(i, x.ix.ln2g(L(i))); lb.mean[i] = A(i).mu2; lb.rstd[i] = A(i).rs2; lb.part[i] = T(i).lnpart;
      lb.dgamma[i] = x.g32(i, x.ix.ln2g(L(i))); lb.dbeta[i] = x.g32(i, x.ix.ln2b(L(i)));
    }
    ++c->launches;
    HYDRA_LAUNCH(c, HYDRA_K_LAYERNORM, x.s, 0.0, (double)G * Tk * d * 8, launch_ln_bwd(lb, x.s));
    // Wo: dWo = dx1^T o, dbo; do = dx1 Wo
    FOR_G {
      pa[i] = T(i).dx1; pb[i] = A(i).o; jw[i] = x.ix.wo(L(i)); pbias[i] = x.g32(i, x.ix.bo(L(i)));
      pc[i] = x.w16(i, x.ix.wo(L(i))); po[i] = T(i).dob;
    }
    TRY(dgrad(x, Tk, d, d, d, pa, pc, po, nullptr, nullptr));
    TRY(wgrad(x, step, Tk, d, d, d, d, pa, pb, jw, pbias));
    // attention backward
    AttnBwdArgs ab{};
    ab.B = c->B; ab.S = c->S; ab.H = x.H; ab.DH = x.DH; ab.ld_qkv = 3 * d; ab.ld_o = d; ab.causal = x.a.causal; ab.G = G;
    ab.scale = (float)(1.0 / std::sqrt((double)x.DH));
    FOR_G {
      ab.qkv[i] = static_cast<const bf16_t*>(A(i).qkv); ab.o[i] = static_cast<const bf16_t*>(A(i).o);
      ab.dout[i] = static_cast<const bf16_t*>(T(i).dob); ab.lse[i] = A(i).lse; ab.delta[i] = T(i).delta;
      ab.dqkv[i] = static_cast<bf16_t*>(T(i).dqkv);
    }
    const double att_fl = 10.0 * c->B * x.H * (double)c->S * c->S * x.DH * (x.a.causal ? 0.5 : 1.0) * G;
    ++c->launches;
    HYDRA_LAUNCH(c, HYDRA_K_ATTENTION, x.s, att_fl, 0.0, launch_attn_bwd(ab, x.s));
    // Wqkv: dWqkv = dqkv^T a, dbqkv; da = dqkv Wqkv
    FOR_G {
      pa[i] = T(i).dqkv; pb[i] = A(i).a; jw[i] = x.ix.wqkv(L(i)); pbias[i] = x.g32(i, x.ix.bqkv(L(i)));
      pc[i] = x.w16(i, x.ix.wqkv(L(i))); po[i] = T(i).da;
    }
    TRY(dgrad(x, Tk, 3 * d, d, 3 * d, pa, pc, po, nullptr, nullptr));
    TRY(wgrad(x, step, Tk, 3 * d, d, 3 * d, d, pa, pb, jw, pbias));
    // LN1: dx = LN1'(da) + dx1
    FOR_G {
      lb.x[i] = x.xin(i, r); lb.dy[i] = T(i).da; lb.add[i] = T(i).dx1; lb.dx[i] = x.dxin(i, r);
      lb.gamma[i] = x.p32(i, x.ix.ln1g(L(i))); lb.mean[i] = A(i).mu1; lb.rstd[i] = A(i).rs1;
      lb.dgamma[i] = x.g32(i, x.ix.ln1g(L(i))); lb.dbeta[i] = x.g32(i, x.ix.ln1b(L(i)));
    }
    ++c->launches;
    HYDRA_LAUNCH(c, HYDRA_K_LAYERNORM, x.s, 0.0, (double)G * Tk * d * 8, launch_ln_bwd(lb, x.s));
  }
  if (first) {
    EmbedBwdArgs e{};
    e.dtype = GEMM_BF16; e.V = x.V; e.S = c->S; e.S_table = x.a.max_seq; e.B = c->B; e.d = d; e.ld = d; e.G = G;
    e.row_ptr = c->csr_ptr + (size_t)batch * (x.V + 1);
    e.positions = c->csr_pos + (size_t)batch * Tk;
    FOR_G { e.dx[i] = x.dxin(i, 0); e.dtok[i] = x.g32(i, 0); e.dpos[i] = x.g32(i, 1); }
    ++c->launches;
    HYDRA_LAUNCH(c, HYDRA_K_EMBED, x.s, 0.0, (double)G * ((double)Tk * d * 2 + ((double)x.V + x.a.max_seq) * d * 4),
                 launch_embed_bwd(e, x.s));
  }
  return HYDRA_OK;
}

hydra_status tr_run(hydra_ctx* c, const Bucket& b, int batch, int step, hipStream_t s) {
  Ctx x(c, b, s);
  if (c->recompute) {
    // A shard's block activations live in a workspace only while one of its tasks runs.  The forward task of every
    // shard but the last leaves the shard's output for the next shard; the backward task runs the forward again
    // (same kernels, same inputs, same bits) and then the backward.  The last shard's forward would be repeated
    // at once by its backward, so it is left to that task: the loss of the step is then written there.
    const bool last = x.shard(0).u1 == x.a.n_layers;
    if (b.ph == HYDRA_PHASE_F) return last ? HYDRA_OK : tr_forward(x, batch, step);
    if (b.ph == HYDRA_PHASE_B) {
      hydra_status st = tr_forward(x, batch, step);
      return st != HYDRA_OK ? st : tr_backward(x, batch, step);
    }
    return run_update(c, b, step, s);
  }
  if (b.ph == HYDRA_PHASE_F) return tr_forward(x, batch, step);
  if (b.ph == HYDRA_PHASE_B) return tr_backward(x, batch, step);
  return run_update(c, b, step, s);
}

}  // namespace hydra
