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

hipError_t prof_epoch_begin(hydra_ctx* c) {
  if (!c->prof_origin) {
    hipError_t r = hipEventCreate(&c->prof_origin);
    if (r != hipSuccess) return r;
  }
  return hipEventRecord(c->prof_origin, c->streams[0]);
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
  std::vector<std::pair<double, double>> iv;  // [start, end] of every launch, ms since the epoch's origin
  iv.reserve(c->prof_recs.size());
  for (const auto& r : c->prof_recs) {
    float ms = 0.f, at = 0.f;
    HYDRA_HIP(c, hipEventElapsedTime(&ms, r.a, r.b));
    if (c->prof_origin) {
      HYDRA_HIP(c, hipEventElapsedTime(&at, c->prof_origin, r.a));
      iv.push_back({(double)at, (double)at + ms});
    }
    auto& s = c->prof_sum[r.cls];
    ++s.launches;
    s.ms += ms;
    s.flops += r.flops;
    s.bytes += r.bytes;
  }
  // time during which at least one kernel was running: launches on different streams overlap, so the sum of their
  // durations can exceed the wall time; the union of the intervals cannot
  if (!iv.empty()) {
    std::sort(iv.begin(), iv.end());
    double busy = 0, lo = iv[0].first, hi = iv[0].second, first = iv[0].first, last = iv[0].second;
    for (size_t i = 1; i < iv.size(); ++i) {
      if (iv[i].first > hi) {
        busy += hi - lo;
        lo = iv[i].first;
        hi = iv[i].second;
      } else {
        hi = std::max(hi, iv[i].second);
      }
      last = std::max(last, iv[i].second);
    }
    busy += hi - lo;
    c->prof_busy_ms += busy;
    c->prof_span_ms += last - first;
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

hydra_status hydra_profile_busy(hydra_ctx* c, int reset, double* busy_ms, double* span_ms) {
  if (!c) return HYDRA_ERR_INVALID_ARG;
  if (!busy_ms || !span_ms) return c->fail(HYDRA_ERR_INVALID_ARG, "NULL output");
  *busy_ms = c->prof_busy_ms;
  *span_ms = c->prof_span_ms;
  if (reset) c->prof_busy_ms = c->prof_span_ms = 0;
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
