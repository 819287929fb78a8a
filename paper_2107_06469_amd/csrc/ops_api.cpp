// C entry points of the individual device operations (include/hydra_ops.h).
#include <mutex>
#include <string>

#include "../../include/hydra.h"
#include "../../include/hydra_ops.h"
#include "kernels.h"

using namespace hydra;

static thread_local std::string g_ops_err;
static std::once_flag g_gemm_once;
static hipError_t g_gemm_init = hipSuccess;

static int done(hipError_t e, const char* what) {
  if (e == hipSuccess) return HYDRA_OK;
  g_ops_err = std::string(what) + ": " + hipGetErrorString(e);
  return e == hipErrorInvalidValue ? HYDRA_ERR_INVALID_ARG : HYDRA_ERR_DEVICE;
}

static int bad(const char* what) {
  g_ops_err = what;
  return HYDRA_ERR_INVALID_ARG;
}

int hydra::ops_fail(int status, const char* what, const char* detail) {
  g_ops_err = detail ? std::string(what) + ": " + detail : std::string(what);
  return status;
}

static int ensure_init() {
  std::call_once(g_gemm_once, [] { g_gemm_init = kernels_init(); });
  return g_gemm_init == hipSuccess ? 0 : done(g_gemm_init, "kernel set-up");
}

// splitmix64, n-th output from state s (twin of the device generator's keying step)
static uint64_t sm_at(uint64_t s, uint64_t n) {
  uint64_t z = s + (n + 1) * 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

// {lr, b1, b2, eps, bc1, bc2} in double -> the kernels' fp32 hyper-parameters (1 - b rounded once from double)
static OptimHp hp_row(const double* r) {
  OptimHp h;
  h.lr = (float)r[0]; h.b1 = (float)r[1]; h.b2 = (float)r[2];
  h.c1 = (float)(1.0 - r[1]); h.c2 = (float)(1.0 - r[2]);
  h.eps = (float)r[3]; h.bc1 = (float)r[4]; h.bc2 = (float)r[5];
  return h;
}

static void fill_gemm(const hydra_gemm_desc* d, GemmArgs& a) {
  a.dtype = d->dtype == HYDRA_OPS_F32 ? GEMM_F32 : GEMM_BF16;
  a.M = d->M; a.N = d->N; a.K = d->K;
  a.x_kmajor = d->x_kmajor; a.w_kmajor = d->w_kmajor;
  a.ldx = d->ldx; a.ldw = d->ldw; a.ldo = d->ldo; a.ldg = d->ldg; a.ldr = d->ldr;
  a.act = d->act; a.out_f32 = d->out_f32; a.tile = d->tile; a.G = d->G;
  for (int g = 0; g < d->G; ++g) {
    a.X[g] = d->X[g];
    a.W[g] = d->W[g];
    a.out[g] = d->out ? d->out[g] : nullptr;
    a.bias[g] = d->bias ? d->bias[g] : nullptr;
    a.pre[g] = d->pre ? d->pre[g] : nullptr;
    a.gate[g] = d->gate ? d->gate[g] : nullptr;
    a.resid[g] = d->resid ? d->resid[g] : nullptr;
    a.rowsum[g] = d->rowsum ? d->rowsum[g] : nullptr;
    a.ws[g] = d->ws ? d->ws[g] : nullptr;
  }
  a.ws_bytes = d->ws ? d->ws_bytes : 0;
}

extern "C" {

const char* hydra_ops_last_error(void) { return g_ops_err.c_str(); }

int hydra_op_gemm_split_k(int M, int N, int K) { return gemm_split_k(M, N, K); }
size_t hydra_op_gemm_split_ws_bytes(int M, int N, int K, int ldo) { return gemm_split_ws_bytes(M, N, K, ldo); }

int hydra_op_gemm(const hydra_gemm_desc* d, void* stream) {
  if (!d || !d->X || !d->W || !d->out || d->G < 1 || d->G > MAXG) return bad("hydra_op_gemm: NULL table or G out of range");
  if (int st = ensure_init()) return st;
  GemmArgs a{};
  fill_gemm(d, a);
  return done(launch_gemm(a, static_cast<hipStream_t>(stream)), "hydra_op_gemm");
}

int hydra_op_gemm_update(const hydra_gemm_desc* d, int opt, float* const* p, float* const* m, float* const* v,
                         void* const* w16, const double* hp, void* stream) {
  if (!d || !d->X || !d->W || !p || !hp || d->G < 1 || d->G > MAXG || (opt != 0 && opt != 1))
    return bad("hydra_op_gemm_update: NULL table, bad opt or G out of range");
  if (opt == 1 && (!m || !v)) return bad("hydra_op_gemm_update: Adam needs m and v");
  if (int st = ensure_init()) return st;
  GemmArgs a{};
  fill_gemm(d, a);
  GemmUpdate u{};
  u.opt = opt;
  for (int i = 0; i < d->G; ++i) {
    u.p[i] = p[i];
    u.m[i] = m ? m[i] : nullptr;
    u.v[i] = v ? v[i] : nullptr;
    u.w16[i] = w16 ? static_cast<bf16_t*>(w16[i]) : nullptr;
    u.hp[i] = hp_row(hp + 6 * i);
  }
  return done(launch_gemm_update(a, u, static_cast<hipStream_t>(stream)), "hydra_op_gemm_update");
}

size_t hydra_op_colsum_part_floats(int M, int N) { return colsum_part_floats(M, N); }

int hydra_op_colsum(int dtype, int M, int N, int ld, int G, const void* const* src, float* const* out,
                    float* const* part, void* stream) {
  if (!src || !out || G < 1 || G > MAXG) return bad("hydra_op_colsum: NULL table or G out of range");
  ColsumArgs a{};
  a.dtype = dtype == HYDRA_OPS_F32 ? GEMM_F32 : GEMM_BF16;
  a.M = M; a.N = N; a.ld = ld; a.G = G;
  for (int g = 0; g < G; ++g) {
    if (!src[g] || !out[g]) return bad("hydra_op_colsum: NULL entry");
    a.src[g] = src[g];
    a.out[g] = out[g];
    a.part[g] = part ? part[g] : nullptr;
  }
  return done(launch_colsum(a, static_cast<hipStream_t>(stream)), "hydra_op_colsum");
}

int hydra_op_softmax_ce(int dtype, int M, int C, int ldz, int lddz, float inv_n, int G, const float* const* logits,
                        const int32_t* labels, void* const* dz, float* const* rowloss, float* const* loss, void* stream) {
  if (!logits || !labels || !dz || !rowloss || !loss || G < 1 || G > MAXG) return bad("hydra_op_softmax_ce: NULL table or G out of range");
  SoftmaxCeArgs a{};
  a.dtype = dtype == HYDRA_OPS_F32 ? GEMM_F32 : GEMM_BF16;
  a.M = M; a.C = C; a.ldz = ldz; a.lddz = lddz; a.G = G; a.inv_n = inv_n;
  a.labels = labels;
  for (int g = 0; g < G; ++g) {
    if (!logits[g] || !dz[g] || !rowloss[g] || !loss[g]) return bad("hydra_op_softmax_ce: NULL entry");
    a.logits[g] = logits[g];
    a.dz[g] = dz[g];
    a.rowloss[g] = rowloss[g];
    a.loss_out[g] = loss[g];
  }
  return done(launch_softmax_ce(a, static_cast<hipStream_t>(stream)), "hydra_op_softmax_ce");
}

int hydra_op_optim(int opt, size_t n, int G, float* const* p, const float* const* g, float* const* m, float* const* v,
                   void* const* w16, const double* hp, void* stream) {
  if (!p || !g || !hp || G < 1 || G > MAXG || (opt != 0 && opt != 1)) return bad("hydra_op_optim: NULL table, bad opt or G out of range");
  if (opt == 1 && (!m || !v)) return bad("hydra_op_optim: Adam needs m and v");
  OptimArgs a{};
  a.opt = opt; a.G = G; a.n = n;
  for (int i = 0; i < G; ++i) {
    a.p[i] = p[i];
    a.g[i] = g[i];
    a.m[i] = m ? m[i] : nullptr;
    a.v[i] = v ? v[i] : nullptr;
    a.w16[i] = w16 ? static_cast<bf16_t*>(w16[i]) : nullptr;
    a.hp[i] = hp_row(hp + 6 * i);
  }
  return done(launch_optim(a, static_cast<hipStream_t>(stream)), "hydra_op_optim");
}

int hydra_op_init_uniform(float* dst, size_t n, uint64_t seed, uint64_t stream_id, float a, void* stream) {
  if (!dst) return bad("hydra_op_init_uniform: dst is NULL");
  const uint64_t key = sm_at(sm_at(seed, 0) ^ stream_id, 0);
  return done(launch_init_uniform(dst, n, key, a, static_cast<hipStream_t>(stream)), "hydra_op_init_uniform");
}

int hydra_op_layernorm_fwd(int dtype, int rows, int d, int ld, float eps, int G, const void* const* x, void* const* y,
                           const float* const* gamma, const float* const* beta, float* const* mean,
                           float* const* rstd, void* stream) {
  if (!x || !y || !gamma || !beta || !mean || !rstd || G < 1 || G > MAXG) return bad("hydra_op_layernorm_fwd: NULL table or G out of range");
  LnArgs a{};
  a.dtype = dtype == HYDRA_OPS_F32 ? GEMM_F32 : GEMM_BF16;
  a.rows = rows; a.d = d; a.ld = ld; a.G = G; a.eps = eps;
  for (int g = 0; g < G; ++g) {
    a.x[g] = x[g]; a.y[g] = y[g]; a.gamma[g] = gamma[g]; a.beta[g] = beta[g]; a.mean[g] = mean[g]; a.rstd[g] = rstd[g];
  }
  return done(launch_ln_fwd(a, static_cast<hipStream_t>(stream)), "hydra_op_layernorm_fwd");
}

size_t hydra_op_layernorm_part_floats(int rows, int d) { return (size_t)ln_bwd_blocks(rows, d) * 2 * d; }

int hydra_op_layernorm_bwd(int dtype, int rows, int d, int ld, int G, const void* const* x, const void* const* dy,
                           const void* const* add, void* const* dx, const float* const* gamma,
                           const float* const* mean, const float* const* rstd, float* const* part,
                           float* const* dgamma, float* const* dbeta, void* stream) {
  if (!x || !dy || !dx || !gamma || !mean || !rstd || !part || !dgamma || !dbeta || G < 1 || G > MAXG)
    return bad("hydra_op_layernorm_bwd: NULL table or G out of range");
  if (int st = ensure_init()) return st;
  LnBwdArgs a{};
  a.dtype = dtype == HYDRA_OPS_F32 ? GEMM_F32 : GEMM_BF16;
  a.rows = rows; a.d = d; a.ld = ld; a.G = G;
  for (int g = 0; g < G; ++g) {
    a.x[g] = x[g]; a.dy[g] = dy[g]; a.add[g] = add ? add[g] : nullptr; a.dx[g] = dx[g]; a.gamma[g] = gamma[g];
    a.mean[g] = mean[g]; a.rstd[g] = rstd[g]; a.part[g] = part[g]; a.dgamma[g] = dgamma[g]; a.dbeta[g] = dbeta[g];
  }
  return done(launch_ln_bwd(a, static_cast<hipStream_t>(stream)), "hydra_op_layernorm_bwd");
}


int hydra_op_attention_fwd(int B, int S, int H, int DH, int ld_qkv, int ld_o, int causal, float scale, int G,
                           const void* const* qkv, void* const* o, float* const* lse, void* stream) {
  if (!qkv || !o || !lse || G < 1 || G > MAXG) return bad("hydra_op_attention_fwd: NULL table or G out of range");
  if (int st = ensure_init()) return st;
  AttnArgs a{};
  a.B = B; a.S = S; a.H = H; a.DH = DH; a.ld_qkv = ld_qkv; a.ld_o = ld_o; a.causal = causal; a.G = G; a.scale = scale;
  for (int g = 0; g < G; ++g) {
    a.qkv[g] = static_cast<const bf16_t*>(qkv[g]); a.o[g] = static_cast<bf16_t*>(o[g]); a.lse[g] = lse[g];
   
  }
  return done(launch_attn_fwd(a, static_cast<hipStream_t>(stream)), "hydra_op_attention_fwd");
}

int hydra_op_attention_bwd(int B, int S, int H, int DH, int ld_qkv, int ld_o, int causal, float scale, int G,
                           const void* const* qkv, const void* const* o, const void* const* dout,
                           const float* const* lse, float* const* delta, void* const* dqkv,
                           void* stream) {
  if (!qkv || !o || !dout || !lse || !delta || !dqkv || G < 1 || G > MAXG)
    return bad("hydra_op_attention_bwd: NULL table or G out of range");
  if (int st = ensure_init()) return st;
  AttnBwdArgs a{};
  a.B = B; a.S = S; a.H = H; a.DH = DH; a.ld_qkv = ld_qkv; a.ld_o = ld_o; a.causal = causal; a.G = G; a.scale = scale;
  for (int g = 0; g < G; ++g) {
    a.qkv[g] = static_cast<const bf16_t*>(qkv[g]); a.o[g] = static_cast<const bf16_t*>(o[g]);
    a.dout[g] = static_cast<const bf16_t*>(dout[g]); a.lse[g] = lse[g]; a.delta[g] = delta[g];
    a.dqkv[g] = static_cast<bf16_t*>(dqkv[g]);
  }
  return done(launch_attn_bwd(a, static_cast<hipStream_t>(stream)), "hydra_op_attention_bwd");
}

int hydra_op_embed_fwd(int dtype, int tokens, int S, int d, int ld, int G, const int32_t* ids, const void* const* tok,
                       const void* const* pos, void* const* x, void* stream) {
  if (!ids || !tok || !pos || !x || G < 1 || G > MAXG) return bad("hydra_op_embed_fwd: NULL table or G out of range");
  EmbedArgs a{};
  a.dtype = dtype == HYDRA_OPS_F32 ? GEMM_F32 : GEMM_BF16;
  a.tokens = tokens; a.S = S; a.d = d; a.ld = ld; a.G = G; a.ids = ids;
  for (int g = 0; g < G; ++g) { a.tok[g] = tok[g]; a.pos[g] = pos[g]; a.x[g] = x[g]; }
  return done(launch_embed_fwd(a, static_cast<hipStream_t>(stream)), "hydra_op_embed_fwd");
}

int hydra_op_embed_bwd(int dtype, int V, int S, int S_table, int B, int d, int ld, int G, const int32_t* row_ptr,
                       const int32_t* positions, const void* const* dx, float* const* dtok, float* const* dpos,
                       void* stream) {
  if (!row_ptr || !positions || !dx || !dtok || !dpos || G < 1 || G > MAXG) return bad("hydra_op_embed_bwd: NULL table or G out of range");
  EmbedBwdArgs a{};
  a.dtype = dtype == HYDRA_OPS_F32 ? GEMM_F32 : GEMM_BF16;
  a.V = V; a.S = S; a.S_table = S_table; a.B = B; a.d = d; a.ld = ld; a.G = G; a.row_ptr = row_ptr; a.positions = positions;
  for (int g = 0; g < G; ++g) { a.dx[g] = dx[g]; a.dtok[g] = dtok[g]; a.dpos[g] = dpos[g]; }
  return done(launch_embed_bwd(a, static_cast<hipStream_t>(stream)), "hydra_op_embed_bwd");
}

int hydra_op_cast_bf16(const float* src, void* dst, size_t n, void* stream) {
  if (!src || !dst) return bad("hydra_op_cast_bf16: NULL pointer");
  return done(launch_cast_bf16(src, static_cast<bf16_t*>(dst), n, static_cast<hipStream_t>(stream)), "hydra_op_cast_bf16");
}

}  // extern "C"
