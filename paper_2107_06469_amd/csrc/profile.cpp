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

hipError_t prof_end(hydra_ctx* c, hipStream_t s, hipEvent_t a, int cls, double flops, double bytes, int cls2, double flops2) {
  hipEvent_t b;
  hipError_t r = next_event(c, &b);
  if (r != hipSuccess) return r;
  r = hipEventRecord(b, s);
  if (r != hipSuccess) return r;
  c->prof_recs.push_back({cls, a, b, flops, bytes, cls2, flops2});
  return hipSuccess;
}

// merges intervals into a sorted list of disjoint ones
static std::vector<std::pair<double, double>> union_of(std::vector<std::pair<double, double>> iv) {
  std::vector<std::pair<double, double>> u;
  std::sort(iv.begin(), iv.end());
  for (const auto& x : iv) {
    if (!u.empty() && x.first <= u.back().second) u.back().second = std::max(u.back().second, x.second);
    else u.push_back(x);
  }
  return u;
}

static double length_of(const std::vector<std::pair<double, double>>& u) {
  double t = 0;
  for (const auto& x : u) t += x.second - x.first;
  return t;
}

hydra_status prof_collect(hydra_ctx* c) {
  // [start, end] of every launch and of every spill copy, ms since the epoch's origin
  std::vector<std::pair<double, double>> kern, copy;
  for (const auto& r : c->prof_recs) {
    float ms = 0.f, at = 0.f;
    HYDRA_HIP(c, hipEventElapsedTime(&ms, r.a, r.b));
    if (c->prof_origin) {
      HYDRA_HIP(c, hipEventElapsedTime(&at, c->prof_origin, r.a));
      const bool is_copy = r.cls == HYDRA_K_COPY_H2D || r.cls == HYDRA_K_COPY_D2H;
      (is_copy ? copy : kern).push_back({(double)at, (double)at + ms});
    }
    // a launch of two classes counts in both, its time split in proportion to their flops
    const double share2 = r.cls2 >= 0 && r.flops + r.flops2 > 0 ? r.flops2 / (r.flops + r.flops2) : 0.0;
    auto& s = c->prof_sum[r.cls];
    ++s.launches;
    s.ms += ms * (1.0 - share2);
    s.flops += r.flops;
    s.bytes += r.bytes;
    if (r.cls2 >= 0) {
      auto& s2 = c->prof_sum[r.cls2];
      ++s2.launches;
      s2.ms += ms * share2;
      s2.flops += r.flops2;
    }
  }
  // time during which at least one kernel was running: launches on different streams overlap, so the sum of their
  // durations can exceed the wall time; the union of the intervals cannot
  const auto ku = union_of(kern), cu = union_of(copy);
  if (!ku.empty()) {
    double last = 0;
    for (const auto& x : ku) last = std::max(last, x.second);
    c->prof_busy_ms += length_of(ku);
    c->prof_span_ms += last - ku[0].first;
  }
  if (!cu.empty()) {
    double both = 0;  // two sorted lists of disjoint intervals: length of their intersection
    size_t i = 0, j = 0;
    while (i < ku.size() && j < cu.size()) {
      const double lo = std::max(ku[i].first, cu[j].first), hi = std::min(ku[i].second, cu[j].second);
      if (hi > lo) both += hi - lo;
      if (ku[i].second < cu[j].second) ++i;
      else ++j;
    }
    c->prof_copy_ms += length_of(cu);
    c->prof_copy_overlapped_ms += both;
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

hydra_status hydra_profile_copy_overlap(hydra_ctx* c, int reset, double* copy_ms, double* overlapped_ms) {
  if (!c) return HYDRA_ERR_INVALID_ARG;
  if (!copy_ms || !overlapped_ms) return c->fail(HYDRA_ERR_INVALID_ARG, "NULL output");
  *copy_ms = c->prof_copy_ms;
  *overlapped_ms = c->prof_copy_overlapped_ms;
  if (reset) c->prof_copy_ms = c->prof_copy_overlapped_ms = 0;
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
