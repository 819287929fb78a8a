// Per-launch timing with HIP event pairs on the launching stream (measurement aid).
#include "hydra_internal.h"

namespace hydra {

static hipError_t next_event(hydra_ctx* c, hipEvent_t* e) {
  if (c->prof_used == c->prof_pool.size()) {
    hipEvent_t n;
    hipError_t r = hipEventCreate(&n);
    if (r != hipSuccess) return r;
    c->prof_pool.push_back(n);
  }
  *e = c->prof_pool[c->prof_used++];
  return hipSuccess;
}

hipError_t prof_begin(hydra_ctx* c, hipStream_t s, hipEvent_t* a) {
  hipError_t r = next_event(c, a);
  return r != hipSuccess ? r : hipEventRecord(*a, s);
}

hipError_t prof_end(hydra_ctx* c, hipStream_t s, hipEvent_t a, int cls, double flops, double bytes) {
  hipEvent_t b;
  hipError_t r = next_event(c, &b);
  if (r != hipSuccess) return r;
  r = hipEventRecord(b, s);
  if (r != hipSuccess) return r;
  c->prof_recs.push_back({cls, a, b, flops, bytes});
  return hipSuccess;
}

hydra_status prof_collect(hydra_ctx* c) {
  for (const auto& r : c->prof_recs) {
    float ms = 0.f;
    HYDRA_HIP(c, hipEventElapsedTime(&ms, r.a, r.b));
    auto& s = c->prof_sum[r.cls];
    ++s.launches;
    s.ms += ms;
    s.flops += r.flops;
    s.bytes += r.bytes;
  }
  c->prof_recs.clear();
  c->prof_used = 0;
  return HYDRA_OK;
}

}  // namespace hydra

extern "C" {

hydra_status hydra_profile_enable(hydra_ctx* c, int on) {
  if (!c) return HYDRA_ERR_INVALID_ARG;
  c->profiling = on != 0 && !c->dry;
  return HYDRA_OK;
}

hydra_status hydra_profile_read(hydra_ctx* c, int cls, int reset, hydra_kernel_profile* out) {
  if (!c) return HYDRA_ERR_INVALID_ARG;
  if (cls < 0 || cls >= HYDRA_K_COUNT || !out) return c->fail(HYDRA_ERR_INVALID_ARG, "bad kernel class or NULL output");
  const auto& s = c->prof_sum[cls];
  out->launches = s.launches;
  out->total_ms = s.ms;
  out->flops = s.flops;
  out->bytes = s.bytes;
  if (reset) c->prof_sum[cls] = hydra_ctx::ProfSum();
  return HYDRA_OK;
}

}  // extern "C"
