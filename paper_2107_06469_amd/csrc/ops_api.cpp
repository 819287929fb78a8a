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

// splitmix64, n-th output from state s (twin of the device generator's keying step)
static uint64_t sm_at(uint64_t s, uint64_t n) {
  uint64_t z = s + (n + 1) * 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

extern "C" {

const char* hydra_ops_last_error(void) { return g_ops_err.c_str(); }

int hydra_op_gemm(const hydra_gemm_desc* d, void* stream) {
  if (!d || !d->X || !d->W || !d->out || d->G < 1 || d->G > MAXG) return bad("hydra_op_gemm: NULL table or G out of range");
  std::call_once(g_gemm_once, [] { g_gemm_init = gemm_init(); });
  if (g_gemm_init != hipSuccess) return done(g_gemm_init, "hydra_op_gemm: kernel set-up");
  GemmArgs a{};
  a.dtype = d->dtype == HYDRA_OPS_F32 ? GEMM_F32 : GEMM_BF16;
  a.M = d->M; a.N = d->N; a.K = d->K;
  a.x_kmajor = d->x_kmajor; a.w_kmajor = d->w_kmajor;
  a.ldx = d->ldx; a.ldw = d->ldw; a.ldo = d->ldo; a.ldg = d->ldg; a.ldr = d->ldr;
  a.act = d->act; a.out_f32 = d->out_f32; a.tile = d->tile; a.G = d->G;
  for (int g = 0; g < d->G; ++g) {
    a.X[g] = d->X[g];
    a.W[g] = d->W[g];
    a.out[g] = d->out[g];
    a.bias[g] = d->bias ? d->bias[g] : nullptr;
    a.pre[g] = d->pre ? d->pre[g] : nullptr;
    a.gate[g] = d->gate ? d->gate[g] : nullptr;
    a.resid[g] = d->resid ? d->resid[g] : nullptr;
  }
  return done(launch_gemm(a, static_cast<hipStream_t>(stream)), "hydra_op_gemm");
}

int hydra_op_colsum(int dtype, int M, int N, int ld, int G, const void* const* src, float* const* out, void* stream) {
  if (!src || !out || G < 1 || G > MAXG) return bad("hydra_op_colsum: NULL table or G out of range");
  ColsumArgs a{};
  a.dtype = dtype == HYDRA_OPS_F32 ? GEMM_F32 : GEMM_BF16;
  a.M = M; a.N = N; a.ld = ld; a.G = G;
  for (int g = 0; g < G; ++g) {
    if (!src[g] || !out[g]) return bad("hydra_op_colsum: NULL entry");
    a.src[g] = src[g];
    a.out[g] = out[g];
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
    a.lr[i] = (float)hp[6 * i]; a.b1[i] = (float)hp[6 * i + 1]; a.b2[i] = (float)hp[6 * i + 2];
    a.c1[i] = (float)(1.0 - hp[6 * i + 1]); a.c2[i] = (float)(1.0 - hp[6 * i + 2]);
    a.eps[i] = (float)hp[6 * i + 3]; a.bc1[i] = (float)hp[6 * i + 4]; a.bc2[i] = (float)hp[6 * i + 5];
  }
  return done(launch_optim(a, static_cast<hipStream_t>(stream)), "hydra_op_optim");
}

int hydra_op_init_uniform(float* dst, size_t n, uint64_t seed, uint64_t stream_id, float a, void* stream) {
  if (!dst) return bad("hydra_op_init_uniform: dst is NULL");
  const uint64_t key = sm_at(sm_at(seed, 0) ^ stream_id, 0);
  return done(launch_init_uniform(dst, n, key, a, static_cast<hipStream_t>(stream)), "hydra_op_init_uniform");
}

int hydra_op_cast_bf16(const float* src, void* dst, size_t n, void* stream) {
  if (!src || !dst) return bad("hydra_op_cast_bf16: NULL pointer");
  return done(launch_cast_bf16(src, static_cast<bf16_t*>(dst), n, static_cast<hipStream_t>(stream)), "hydra_op_cast_bf16");
}

}  // extern "C"
