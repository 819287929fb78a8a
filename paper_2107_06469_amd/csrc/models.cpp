// Model registry: canonical tensor lists, shard cutting, device state and seeded initialisation.
#include <algorithm>
#include <cmath>
#include <cstring>

#include "hydra_internal.h"

namespace hydra {

static size_t rup(size_t v, size_t a) { return (v + a - 1) / a * a; }

static void add_tensor(Model& m, const std::string& name, int rows, int cols, int init, float a, int unit) {
  Tensor t;
  t.name = name;
  t.rows = rows;
  t.cols = cols;
  t.n = (size_t)rows * cols;
  t.init = init;
  t.a = a;
  t.unit = unit;
  t.fused = rows > 1 && name != "tok_emb" && name != "pos_emb";  // embedding gradients come from a scatter, not a GEMM
  t.off = m.n_block;
  m.n_block += rup(t.n, 64);
  m.tensors.push_back(t);
}

hydra_status build_tensors(hydra_ctx* c, Model& m) {
  const hydra_arch& a = m.arch;
  m.tensors.clear();
  m.n_block = 0;
  if (a.kind == HYDRA_KIND_MLP) {
    int prev = a.d_in;
    for (int l = 0; l < a.n_layers; ++l) {
      add_tensor(m, "W" + std::to_string(l), a.d_model, prev, INIT_UNIFORM, (float)std::sqrt(6.0 / prev), l);
      add_tensor(m, "b" + std::to_string(l), 1, a.d_model, INIT_ZERO, 0.f, l);
      prev = a.d_model;
    }
    add_tensor(m, "Wout", a.n_out, prev, INIT_UNIFORM, (float)std::sqrt(6.0 / prev), a.n_layers);
    add_tensor(m, "bout", 1, a.n_out, INIT_ZERO, 0.f, a.n_layers);
    m.n_units = a.n_layers + 1;
    return HYDRA_OK;
  }
  const int d = a.d_model, F = a.d_ffn, V = a.n_out, S = a.max_seq, L = a.n_layers;
  const float s02 = (float)(0.02 * std::sqrt(3.0));
  add_tensor(m, "tok_emb", V, d, INIT_UNIFORM, s02, 0);
  add_tensor(m, "pos_emb", S, d, INIT_UNIFORM, s02, 0);
  for (int l = 0; l < L; ++l) {
    std::string p = "L" + std::to_string(l) + ".";
    add_tensor(m, p + "ln1.g", 1, d, INIT_ONE, 0.f, l);
    add_tensor(m, p + "ln1.b", 1, d, INIT_ZERO, 0.f, l);
    add_tensor(m, p + "Wqkv", 3 * d, d, INIT_UNIFORM, s02, l);
    add_tensor(m, p + "bqkv", 1, 3 * d, INIT_ZERO, 0.f, l);
    add_tensor(m, p + "Wo", d, d, INIT_UNIFORM, s02, l);
    add_tensor(m, p + "bo", 1, d, INIT_ZERO, 0.f, l);
    add_tensor(m, p + "ln2.g", 1, d, INIT_ONE, 0.f, l);
    add_tensor(m, p + "ln2.b", 1, d, INIT_ZERO, 0.f, l);
    add_tensor(m, p + "W1", F, d, INIT_UNIFORM, s02, l);
    add_tensor(m, p + "b1", 1, F, INIT_ZERO, 0.f, l);
    if (a.ffn_gated) {
      add_tensor(m, p + "Wg", F, d, INIT_UNIFORM, s02, l);
      add_tensor(m, p + "bg", 1, F, INIT_ZERO, 0.f, l);
    }
    add_tensor(m, p + "W2", d, F, INIT_UNIFORM, s02, l);
    add_tensor(m, p + "b2", 1, d, INIT_ZERO, 0.f, l);
  }
  add_tensor(m, "lnf.g", 1, d, INIT_ONE, 0.f, L - 1);
  add_tensor(m, "lnf.b", 1, d, INIT_ZERO, 0.f, L - 1);
  add_tensor(m, "Whead", V, d, INIT_UNIFORM, s02, L - 1);
  add_tensor(m, "bhead", 1, V, INIT_ZERO, 0.f, L - 1);
  m.n_units = L;
  (void)c;
  return HYDRA_OK;
}

static uint64_t mix_sig(uint64_t h, uint64_t v) {
  h ^= v + 0x9E3779B97F4A7C15ull + (h << 6) + (h >> 2);
  return h;
}

static void point_shard(Model& m, Shard& sh) {
  sh.p = m.p ? m.p + sh.off : nullptr;
  sh.m = m.m ? m.m + sh.off : nullptr;
  sh.v = m.v ? m.v + sh.off : nullptr;
  sh.g = m.g ? m.g + sh.off : nullptr;
  sh.w16 = m.w16 ? m.w16 + sh.off : nullptr;
}

hydra_status cut_model(hydra_ctx* c, Model& m, const int32_t* cuts, int n_cuts) {
  const int U = m.n_units;
  std::vector<int> b{0};
  for (int i = 0; i < n_cuts; ++i) {
    if (cuts[i] <= b.back() || cuts[i] >= U)
      return c->fail(HYDRA_ERR_INVALID_ARG, "cut %d (= %d) must be strictly increasing and inside (0, %d)", i, cuts[i], U);
    b.push_back(cuts[i]);
  }
  b.push_back(U);
  for (Shard& old : m.shards) {
    if (old.loaded_ev) (void)hipEventDestroy(old.loaded_ev);
    if (old.updated_ev) (void)hipEventDestroy(old.updated_ev);
    if (old.stored_ev) (void)hipEventDestroy(old.stored_ev);
    if (old.tail_chunks || (c->dry && old.n_tail_chunks)) ctx_free(c, old.tail_chunks, (size_t)old.n_tail_chunks * sizeof(uint2));
  }
  m.shards.clear();
  const int nt = (int)m.tensors.size();
  for (size_t s = 0; s + 1 < b.size(); ++s) {
    Shard sh;
    sh.u0 = b[s];
    sh.u1 = b[s + 1];
    // tensors of units [u0,u1) form a contiguous range of the canonical order
    sh.t0 = nt;
    sh.t1 = 0;
    for (int j = 0; j < nt; ++j)
      if (m.tensors[j].unit >= sh.u0 && m.tensors[j].unit < sh.u1) {
        if (j < sh.t0) sh.t0 = j;
        if (j + 1 > sh.t1) sh.t1 = j + 1;
      }
    sh.off = m.tensors[sh.t0].off;
    sh.n = (sh.t1 < nt ? m.tensors[sh.t1].off : m.n_block) - sh.off;
    const hydra_arch& a = m.arch;
    uint64_t h = 0x1234;
    for (uint64_t v : {(uint64_t)a.kind, (uint64_t)a.dtype, (uint64_t)a.d_model, (uint64_t)a.n_heads, (uint64_t)a.d_ffn,
                       (uint64_t)a.n_out, (uint64_t)a.ffn_gated, (uint64_t)a.causal, (uint64_t)a.act, (uint64_t)a.max_seq,
                       (uint64_t)(sh.u1 - sh.u0), (uint64_t)(sh.u0 == 0), (uint64_t)(sh.u1 == U),
                       (uint64_t)(sh.u0 == 0 ? a.d_in : 0),
                       (uint64_t)m.hp.opt})  // a launch group applies one optimizer to all its members
      h = mix_sig(h, v);
    sh.sig = h;
    point_shard(m, sh);
    m.shards.push_back(sh);
  }
  return HYDRA_OK;
}

void* ctx_alloc(hydra_ctx* c, size_t bytes) {
  bytes = rup(bytes ? bytes : 1, 256);
  c->dev_bytes += bytes;
  if (c->dev_bytes > c->peak_dev_bytes) c->peak_dev_bytes = c->dev_bytes;
  if (c->dry) return nullptr;
  void* p = nullptr;
  if (c->opt.dev_alloc) p = c->opt.dev_alloc(bytes, c->opt.user);
  else if (hipMalloc(&p, bytes) != hipSuccess) p = nullptr;
  if (p) c->dev_allocs.push_back(p);
  return p;
}

void ctx_free(hydra_ctx* c, void* p, size_t bytes) {
  if (!p) {
    if (c->dry) c->dev_bytes -= rup(bytes ? bytes : 1, 256);
    return;
  }
  for (size_t i = 0; i < c->dev_allocs.size(); ++i)
    if (c->dev_allocs[i] == p) {
      c->dev_allocs.erase(c->dev_allocs.begin() + i);
      if (c->opt.dev_free) c->opt.dev_free(p, c->opt.user);
      else if (!c->opt.dev_alloc) (void)hipFree(p);
      c->dev_bytes -= rup(bytes ? bytes : 1, 256);
      return;
    }
}

void ctx_free_all(hydra_ctx* c) {
  for (void* p : c->dev_allocs) {
    if (c->opt.dev_free) c->opt.dev_free(p, c->opt.user);
    else if (!c->opt.dev_alloc) (void)hipFree(p);
  }
  c->dev_allocs.clear();
  c->dev_bytes = 0;
}

// SplitMix64 (Steele, Lea, Flood 2014): n-th output from state s
static uint64_t splitmix_at(uint64_t s, uint64_t n) {
  uint64_t z = s + (n + 1) * 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

uint64_t tensor_key(uint64_t seed, int model, int tensor) {
  const uint64_t stream_id = ((uint64_t)model << 20) | (uint64_t)tensor;
  return splitmix_at(splitmix_at(seed, 0) ^ stream_id, 0);
}

#define ALLOC_OR_FAIL(c, ptr, type, bytes)                                                       \
  do {                                                                                           \
    ptr = static_cast<type>(ctx_alloc(c, bytes));                                                \
    if (!ptr && !(c)->dry) return (c)->fail(HYDRA_ERR_OOM_DEVICE, "device allocation of %zu bytes failed", (size_t)(bytes)); \
  } while (0)

hydra_status alloc_models(hydra_ctx* c) {
  hipStream_t s = c->dry ? nullptr : c->streams[0];
  for (int k = 0; k < c->K; ++k) {
    Model& m = c->models[k];
    const size_t n = m.n_block;
    ALLOC_OR_FAIL(c, m.p, float*, n * 4);
    ALLOC_OR_FAIL(c, m.g, float*, n * 4);
    if (m.hp.opt == HYDRA_OPT_ADAM) {
      ALLOC_OR_FAIL(c, m.m, float*, n * 4);
      ALLOC_OR_FAIL(c, m.v, float*, n * 4);
    }
    if (m.arch.dtype == HYDRA_DTYPE_BF16) ALLOC_OR_FAIL(c, m.w16, bf16_t*, n * 2);
    if (c->dry) continue;
    HYDRA_HIP(c, launch_fill_f32(m.p, n, 0.f, s));
    HYDRA_HIP(c, launch_fill_f32(m.g, n, 0.f, s));
    if (m.m) HYDRA_HIP(c, launch_fill_f32(m.m, n, 0.f, s));
    if (m.v) HYDRA_HIP(c, launch_fill_f32(m.v, n, 0.f, s));
    for (size_t j = 0; j < m.tensors.size(); ++j) {
      const Tensor& t = m.tensors[j];
      if (t.init == INIT_ONE) HYDRA_HIP(c, launch_fill_f32(m.p + t.off, t.n, 1.f, s));
      else if (t.init == INIT_UNIFORM) {
        HYDRA_HIP(c, launch_init_uniform(m.p + t.off, t.n, tensor_key(c->seed, k, (int)j), t.a, s));
      }
    }
    if (m.w16) HYDRA_HIP(c, launch_cast_bf16(m.p, m.w16, n, s));
  }
  if (!c->dry) HYDRA_HIP(c, hipStreamSynchronize(s));
  return HYDRA_OK;
}

hydra_status build_update_chunks(hydra_ctx* c) {
  for (Model& m : c->models)
    for (Shard& sh : m.shards) {
      if (sh.n_tail_chunks) continue;
      std::vector<uint2> tab;
      sh.n_tail = 0;
      for (int j = sh.t0; j < sh.t1; ++j) {
        const Tensor& t = m.tensors[j];
        if (t.fused) continue;
        const size_t first = (t.off - sh.off) / 4, nv = rup(t.n, 64) / 4;  // the padding is updated too (it stays zero)
        for (size_t v = 0; v < nv; v += 256) tab.push_back(make_uint2((unsigned)(first + v), (unsigned)std::min<size_t>(256, nv - v)));
        sh.n_tail += nv * 4;
      }
      if (tab.empty()) continue;
      ALLOC_OR_FAIL(c, sh.tail_chunks, uint2*, tab.size() * sizeof(uint2));
      sh.n_tail_chunks = (int)tab.size();
      if (!c->dry) HYDRA_HIP(c, hipMemcpy(sh.tail_chunks, tab.data(), tab.size() * sizeof(uint2), hipMemcpyHostToDevice));
    }
  return HYDRA_OK;
}

// ---- Transformer activations --------------------------------------------------------------------------------
struct TrDims {
  size_t Tk, NT, d, F, V, ldv, bhs, H;
  bool gated;
};

static hydra_status alloc_block_acts(hydra_ctx* c, TrBlockActs& b, const TrDims& q) {
  ALLOC_OR_FAIL(c, b.a, void*, q.Tk * q.d * 2);
  ALLOC_OR_FAIL(c, b.qkv, void*, q.Tk * 3 * q.d * 2);
  ALLOC_OR_FAIL(c, b.o, void*, q.Tk * q.d * 2);
  ALLOC_OR_FAIL(c, b.x1, void*, q.Tk * q.d * 2);
  ALLOC_OR_FAIL(c, b.f, void*, q.Tk * q.d * 2);
  ALLOC_OR_FAIL(c, b.z1, void*, q.Tk * q.F * 2);
  if (q.gated) ALLOC_OR_FAIL(c, b.zg, void*, q.Tk * q.F * 2);
  ALLOC_OR_FAIL(c, b.hmid, void*, q.Tk * q.F * 2);
  ALLOC_OR_FAIL(c, b.mu1, float*, q.Tk * 4);
  ALLOC_OR_FAIL(c, b.rs1, float*, q.Tk * 4);
  ALLOC_OR_FAIL(c, b.mu2, float*, q.Tk * 4);
  ALLOC_OR_FAIL(c, b.rs2, float*, q.Tk * 4);
  ALLOC_OR_FAIL(c, b.lse, float*, q.bhs * 4);
  return HYDRA_OK;
}

// head buffers and backward scratch of one model (or one workspace)
// scratch of the largest split weight gradient of a block or of the head
static size_t splitk_bytes(const TrDims& q) {
  const int d = (int)q.d, F = (int)q.F, Tk = (int)q.Tk;
  size_t b = gemm_split_ws_bytes(3 * d, d, Tk, d);
  b = std::max(b, gemm_split_ws_bytes(d, d, Tk, d));
  b = std::max(b, gemm_split_ws_bytes(F, d, Tk, d));
  b = std::max(b, gemm_split_ws_bytes(d, F, Tk, F));
  return std::max(b, gemm_split_ws_bytes((int)q.V, d, (int)q.NT, d));
}

static hydra_status alloc_scratch(hydra_ctx* c, TrActs& t, const TrDims& q) {
  t.splitk_bytes = splitk_bytes(q);
  if (t.splitk_bytes) ALLOC_OR_FAIL(c, t.splitk, void*, t.splitk_bytes);
  ALLOC_OR_FAIL(c, t.xf, void*, q.Tk * q.d * 2);
  ALLOC_OR_FAIL(c, t.dxf, void*, q.Tk * q.d * 2);
  ALLOC_OR_FAIL(c, t.xt, void*, q.NT * q.d * 2);
  ALLOC_OR_FAIL(c, t.dxt, void*, q.NT * q.d * 2);
  ALLOC_OR_FAIL(c, t.logits, float*, q.NT * q.ldv * 4);
  ALLOC_OR_FAIL(c, t.dlogits, void*, q.NT * q.ldv * 2);
  ALLOC_OR_FAIL(c, t.rowloss, float*, q.NT * 4);
  ALLOC_OR_FAIL(c, t.muf, float*, q.Tk * 4);
  ALLOC_OR_FAIL(c, t.rsf, float*, q.Tk * 4);
  if (q.gated) {
    ALLOC_OR_FAIL(c, t.dhm, void*, q.Tk * q.F * 2);
    ALLOC_OR_FAIL(c, t.dzg, void*, q.Tk * q.F * 2);
  }
  ALLOC_OR_FAIL(c, t.dz1, void*, q.Tk * q.F * 2);
  ALLOC_OR_FAIL(c, t.df, void*, q.Tk * q.d * 2);
  ALLOC_OR_FAIL(c, t.dx1, void*, q.Tk * q.d * 2);
  ALLOC_OR_FAIL(c, t.dob, void*, q.Tk * q.d * 2);
  ALLOC_OR_FAIL(c, t.dqkv, void*, q.Tk * 3 * q.d * 2);
  ALLOC_OR_FAIL(c, t.da, void*, q.Tk * q.d * 2);
  ALLOC_OR_FAIL(c, t.delta, float*, q.bhs * 4);
  ALLOC_OR_FAIL(c, t.lnpart, float*, (size_t)ln_bwd_blocks((int)q.Tk, (int)q.d) * 2 * q.d * 4);
  return HYDRA_OK;
}

static TrDims dims_of(const hydra_ctx* c, const hydra_arch& a) {
  TrDims q{};
  q.Tk = (size_t)c->B * c->S;
  q.NT = (size_t)c->B * c->P;
  q.d = a.d_model;
  q.F = a.d_ffn;
  q.V = a.n_out;
  q.ldv = rup(a.n_out, 8);
  q.H = a.n_heads;
  q.bhs = (size_t)c->B * a.n_heads * c->S;
  q.gated = a.ffn_gated != 0;
  return q;
}

static size_t block_bytes(const TrDims& q) {
  return q.Tk * q.d * 2 * 7 + q.Tk * q.F * 2 * (q.gated ? 3 : 2) + q.Tk * 16 + q.bhs * 4;  // a, qkv (3), o, x1, f; z1, (zg,) hmid
}
static size_t scratch_bytes(const TrDims& q) {
  return q.Tk * q.d * 2 * 6 + q.Tk * 3 * q.d * 2 + q.NT * q.d * 4 + q.NT * q.ldv * 6 + q.NT * 4 + q.Tk * 8 +
         q.Tk * q.F * 2 * (q.gated ? 3 : 1) + q.bhs * 4 + (size_t)ln_bwd_blocks((int)q.Tk, (int)q.d) * 2 * q.d * 4 + splitk_bytes(q);
}

// Keeps every block's activations per model, or, when that exceeds activation_budget_bytes, only the hand-off
// buffers between shards per model plus a pool of shard-sized workspaces (the backward task of a shard then runs
// its forward again: same kernels on the same inputs, hence the same bits).
static hydra_status alloc_transformer_activations(hydra_ctx* c) {
  size_t keep_all = 0;
  for (const Model& m : c->models) {
    const TrDims q = dims_of(c, m.arch);
    keep_all += (size_t)m.arch.n_layers * block_bytes(q) + scratch_bytes(q);
  }
  if (c->opt.auto_budget && !c->opt.activation_budget_bytes) {
    // what the device has left once the state (or, when spilled, the state budget with its slots) is taken
    const size_t held = c->spill ? std::max(c->dev_bytes, c->opt.device_budget_bytes) : c->dev_bytes;
    const size_t left = c->capacity > held ? (size_t)(0.9 * (double)(c->capacity - held)) : 0;
    if (keep_all > left) c->opt.activation_budget_bytes = std::max<size_t>(left, 1);
  }
  c->recompute = c->opt.activation_budget_bytes > 0 && keep_all > c->opt.activation_budget_bytes;
  for (int k = 0; k < c->K; ++k) {
    Model& m = c->models[k];
    const hydra_arch& a = m.arch;
    const TrDims q = dims_of(c, a);
    TrActs& t = m.tr;
    t.x.assign(a.n_layers + 1, nullptr);
    t.dx.assign(a.n_layers + 1, nullptr);
    t.blk.assign(a.n_layers, TrBlockActs());
    std::vector<char> boundary(a.n_layers + 1, c->recompute ? 0 : 1);
    for (const Shard& sh : m.shards) boundary[sh.u0] = boundary[sh.u1] = 1;
    for (int l = 0; l <= a.n_layers; ++l) {
      if (!boundary[l]) continue;  // inside a shard: lives in the workspace of the running task
      ALLOC_OR_FAIL(c, t.x[l], void*, q.Tk * q.d * 2);
      ALLOC_OR_FAIL(c, t.dx[l], void*, q.Tk * q.d * 2);
    }
    if (c->recompute) continue;
    for (int l = 0; l < a.n_layers; ++l) {
      hydra_status st = alloc_block_acts(c, t.blk[l], q);
      if (st != HYDRA_OK) return st;
    }
    hydra_status st = alloc_scratch(c, t, q);
    if (st != HYDRA_OK) return st;
  }
  if (!c->recompute) return HYDRA_OK;
  // one workspace serves the largest shard of the widest model
  TrDims q = dims_of(c, c->models[0].arch);
  int max_units = 1;
  for (const Model& m : c->models) {
    const TrDims r = dims_of(c, m.arch);
    q.d = std::max(q.d, r.d);
    q.F = std::max(q.F, r.F);
    q.ldv = std::max(q.ldv, r.ldv);
    q.V = std::max(q.V, r.V);
    q.bhs = std::max(q.bhs, r.bhs);
    q.H = std::max(q.H, r.H);
    q.gated = q.gated || r.gated;
    for (const Shard& sh : m.shards) max_units = std::max(max_units, sh.u1 - sh.u0);
  }
  const size_t one = (size_t)max_units * block_bytes(q) + (size_t)(max_units - 1) * q.Tk * q.d * 4 + scratch_bytes(q);
  const int ns = c->dry ? std::max(1, c->opt.n_streams) : (int)c->streams.size();
  const int nc = ns >= 2 ? std::max(1, ns / 2) : 1;  // compute streams of the shard-parallel policy
  size_t n_ws = c->opt.activation_budget_bytes / one;
  if (n_ws < 1)
    return c->fail(HYDRA_ERR_OOM_DEVICE, "activation budget of %zu bytes is smaller than one shard's workspace (%zu bytes)",
                   c->opt.activation_budget_bytes, one);
  n_ws = std::min<size_t>(n_ws, (size_t)nc * MAXG);
  c->ws_streams = (int)std::min<size_t>(nc, n_ws);
  c->ws_group = (int)(n_ws / c->ws_streams);
  c->ws.assign((size_t)c->ws_streams * c->ws_group, TrWorkspace());
  for (TrWorkspace& w : c->ws) {
    w.blk.assign(max_units, TrBlockActs());
    w.xi.assign(max_units, nullptr);
    w.dxi.assign(max_units, nullptr);
    for (int u = 0; u < max_units; ++u) {
      hydra_status st = alloc_block_acts(c, w.blk[u], q);
      if (st != HYDRA_OK) return st;
      if (u == 0) continue;
      ALLOC_OR_FAIL(c, w.xi[u], void*, q.Tk * q.d * 2);
      ALLOC_OR_FAIL(c, w.dxi[u], void*, q.Tk * q.d * 2);
    }
    hydra_status st = alloc_scratch(c, w.sc, q);
    if (st != HYDRA_OK) return st;
  }
  return HYDRA_OK;
}

hydra_status alloc_activations(hydra_ctx* c) {
  for (int k = 0; k < c->K; ++k) {  // the loss buffer holds one float per step of an epoch
    Model& m = c->models[k];
    if (m.loss_cap >= c->n_batches) continue;
    if (m.loss_cap) ctx_free(c, m.loss_dev, (size_t)m.loss_cap * 4);
    ALLOC_OR_FAIL(c, m.loss_dev, float*, (size_t)c->n_batches * 4);
    m.loss_cap = c->n_batches;
  }
  if (c->acts_ready) return HYDRA_OK;
  for (int k = 0; k < c->K; ++k) {
    Model& m = c->models[k];
    const hydra_arch& a = m.arch;
    const size_t es = a.dtype == HYDRA_DTYPE_BF16 ? 2 : 4;
    if (a.kind == HYDRA_KIND_MLP) {
      const size_t ldd = rup(a.d_model, 8), ldv = rup(a.n_out, 8);
      MlpActs& t = m.mlp;
      t.z.assign(a.n_layers, nullptr);
      t.h.assign(a.n_layers, nullptr);
      t.dz.assign(a.n_layers, nullptr);
      for (int l = 0; l < a.n_layers; ++l) {
        ALLOC_OR_FAIL(c, t.z[l], void*, (size_t)c->B * ldd * es);
        ALLOC_OR_FAIL(c, t.h[l], void*, (size_t)c->B * ldd * es);
        ALLOC_OR_FAIL(c, t.dz[l], void*, (size_t)c->B * ldd * es);
      }
      ALLOC_OR_FAIL(c, t.logits, float*, (size_t)c->B * ldv * 4);
      ALLOC_OR_FAIL(c, t.dlogits, void*, (size_t)c->B * ldv * es);
      ALLOC_OR_FAIL(c, t.rowloss, float*, (size_t)c->B * 4);
      if (a.dtype == HYDRA_DTYPE_F32 && mlp_fused_shape_ok(c->B, a.d_in, a.d_model, a.n_out, a.n_layers + 1)) {
        ALLOC_OR_FAIL(c, t.tab, MlpTab*, sizeof(MlpTab));
        if (!c->dry) {
          MlpTab h{};
          for (int l = 0; l < a.n_layers; ++l) {
            h.z[l] = static_cast<float*>(t.z[l]);
            h.h[l] = static_cast<float*>(t.h[l]);
            h.dz[l] = static_cast<float*>(t.dz[l]);
          }
          h.logits = t.logits;
          h.dlogits = static_cast<float*>(t.dlogits);
          h.rowloss = t.rowloss;
          HYDRA_HIP(c, hipMemcpy(t.tab, &h, sizeof(MlpTab), hipMemcpyHostToDevice));
        }
      }
    }
  }
  if (c->models[0].arch.kind != HYDRA_KIND_MLP) {
    hydra_status st = alloc_transformer_activations(c);
    if (st != HYDRA_OK) return st;
  }
  c->acts_ready = true;
  return HYDRA_OK;
}

}  // namespace hydra
