// Shard scheduler: turns a scheduling policy into an ordered list of launch groups for one step
// and replays it for every step of an epoch on the context's streams.
//
// Tasks are F(k,s), B(k,s), U(k,s): forward, backward and update of shard s of model k.  Within a
// step F(k,s) needs F(k,s-1); B(k,s) needs B(k,s+1), or F(k,S-1) for the last shard; U(k,s) needs
// B(k,s).  Across steps F(k,s) needs the previous U(k,s).  Models never depend on each other, which
// is what lets a shard of one model run while another model's next shard waits on its dependency
// (paper, Introduction, "Model Selection Integration").  The order of a model's own tasks, and
// hence every value it computes, is the same under every policy.
#include <algorithm>
#include <chrono>
#include <set>

#include "hydra_internal.h"

namespace hydra {

static std::vector<Task> preds_of(const hydra_ctx* c, const Task& t) {
  const int S = (int)c->models[t.k].shards.size();
  std::vector<Task> p;
  if (t.ph == HYDRA_PHASE_F) {
    if (t.s > 0) p.push_back({t.k, t.s - 1, HYDRA_PHASE_F});
  } else if (t.ph == HYDRA_PHASE_B) {
    if (t.s < S - 1) p.push_back({t.k, t.s + 1, HYDRA_PHASE_B});
    else p.push_back({t.k, t.s, HYDRA_PHASE_F});
  } else {
    p.push_back({t.k, t.s, HYDRA_PHASE_B});
  }
  return p;
}

// 256 x 256 output tiles of the smallest matrix product of a forward or backward task of shard s of model m
// (rows = the step's tokens, columns = the hidden width): what one member adds to a grouped launch
static long min_tiles_of(const hydra_ctx* c, const Model& m) {
  const long rows = m.arch.kind == HYDRA_KIND_MLP ? c->B : (long)c->B * c->S;
  return ((rows + 255) / 256) * ((m.arch.d_model + 255) / 256);
}

// Launch-group size for n ready same-shaped tasks (automatic mode): as many groups as there are compute streams,
// as long as every group still brings at least 384 tiles (1.5 passes over 256 compute units) to its smallest launch.
static int auto_group_size(const hydra_ctx* c, const Model& m, int n, int n_compute_streams, int maxg) {
  const long per = min_tiles_of(c, m);
  long groups = std::max<long>(1, (long)n * per / 384);
  groups = std::min<long>(groups, std::max(1, n_compute_streams));
  const int g = (int)((n + groups - 1) / groups);
  return std::max(1, std::min(g, maxg));
}

// Small fp32 MLPs run a whole shard phase in one launch, and that launch can as well take the next shard's phase when
// the plan runs it next for these models, on the same stream: forward of shards s, s+1, ... or backward of shards
// s, s-1, ...  Such groups become one launch group that spans the shards (update groups of these models launch
// nothing when the update runs in the gradient kernel, and are stepped over, as are groups of other models).  Same kernels over the same
// units in the same order: the values do not change, only the number of launches.
static void merge_shard_spans(const hydra_ctx* c, std::vector<Bucket>& plan) {
  if (c->spill) return;
  auto fused = [&](const Bucket& b) {
    for (const auto& mem : b.members)
      if (!mlp_runs_fused(c, c->models[mem.first])) return false;
    return true;
  };
  for (size_t i = 0; i < plan.size(); ++i) {
    Bucket& a = plan[i];
    if (a.ph == HYDRA_PHASE_U || c->models[0].arch.kind != HYDRA_KIND_MLP || !fused(a)) continue;
    for (;;) {
      // the next group of these models: groups of other models in between neither feed it nor need it first
      auto shares_model = [&](const Bucket& x) {
        for (const auto& xm : x.members)
          for (const auto& am : a.members)
            if (xm.first == am.first) return true;
        return false;
      };
      size_t j = i + 1;
      while (j < plan.size() && ((plan[j].ph == HYDRA_PHASE_U && c->fuse && fused(plan[j])) || !shares_model(plan[j]))) ++j;
      if (j >= plan.size()) break;
      const Bucket& b = plan[j];
      bool ok = b.ph == a.ph && b.stream == a.stream && b.span == 1 && b.members.size() == a.members.size();
      for (size_t m = 0; ok && m < a.members.size(); ++m)
        ok = b.members[m].first == a.members[m].first && b.members[m].second == a.shard_at(m, a.span);
      if (!ok) break;
      ++a.span;
      plan.erase(plan.begin() + (long)j);
    }
  }
  // a forward group over all shards, and right behind it (for these models) the backward group over all shards: one
  // group; the gradient kernel that follows the fused launch is the backward tasks' second half
  for (size_t i = 0; i < plan.size(); ++i) {
    Bucket& a = plan[i];
    if (a.ph != HYDRA_PHASE_F || !fused(a)) continue;
    bool whole = true;
    for (const auto& mem : a.members)
      whole = whole && mem.second == 0 && a.span == (int)c->models[mem.first].shards.size();
    if (!whole) continue;
    auto shares_model = [&](const Bucket& x) {
      for (const auto& xm : x.members)
        for (const auto& am : a.members)
          if (xm.first == am.first) return true;
      return false;
    };
    size_t j = i + 1;
    while (j < plan.size() && !shares_model(plan[j])) ++j;
    if (j >= plan.size()) continue;
    const Bucket& b = plan[j];
    bool ok = b.ph == HYDRA_PHASE_B && b.stream == a.stream && b.span == a.span && b.bspan == 0 && b.members.size() == a.members.size();
    for (size_t m = 0; ok && m < a.members.size(); ++m)
      ok = b.members[m].first == a.members[m].first && b.members[m].second == a.span - 1;
    if (!ok) continue;
    a.bspan = b.span;
    plan.erase(plan.begin() + (long)j);
  }
}

static const char* ph_name(int ph) { return ph == 0 ? "F" : (ph == 1 ? "B" : "U"); }

hydra_status build_plan(hydra_ctx* c, const hydra_schedule* sch, std::vector<Bucket>& plan) {
  plan.clear();
  const int K = c->K;
  int maxg = c->spill ? std::min(MAXG, spill_max_group(c)) : MAXG;  // a group holds one slot per member
  if (c->recompute) maxg = std::min(maxg, c->ws_group);                  // ... and one activation workspace
  if (c->opt.max_group > 0) maxg = std::min(maxg, c->opt.max_group);
  const int ns = c->dry ? std::max(1, c->opt.n_streams) : (int)c->streams.size();
  size_t total = 0;
  for (int k = 0; k < K; ++k)
    if (c->models[k].active) total += 3 * c->models[k].shards.size();
  if (total == 0) return c->fail(HYDRA_ERR_BAD_STATE, "no model is active");

  if (sch->policy == HYDRA_SCHED_SEQUENTIAL) {
    for (int k = 0; k < K; ++k) {
      if (!c->models[k].active) continue;
      const int S = (int)c->models[k].shards.size();
      for (int s = 0; s < S; ++s) plan.push_back({HYDRA_PHASE_F, {{k, s}}, 0});
      for (int s = S - 1; s >= 0; --s) {
        plan.push_back({HYDRA_PHASE_B, {{k, s}}, 0});
        plan.push_back({HYDRA_PHASE_U, {{k, s}}, 0});
      }
    }
    return HYDRA_OK;
  }

  if (sch->policy == HYDRA_SCHED_TASK_PARALLEL) {
    // one task list per model (forward through its shards, then backward and update shard by shard), each on the
    // model's own stream; the lists are interleaved position by position so the host feeds all streams evenly
    int nstr = std::max(1, ns);
    if (c->recompute) nstr = std::min(nstr, c->ws_streams);  // a stream's tasks share its activation workspace
    std::vector<std::vector<Bucket>> lists;
    size_t longest = 0;
    for (int k = 0; k < K; ++k) {
      if (!c->models[k].active) continue;
      const int S = (int)c->models[k].shards.size(), str = (int)(lists.size() % nstr);
      std::vector<Bucket> l;
      for (int s = 0; s < S; ++s) l.push_back({HYDRA_PHASE_F, {{k, s}}, str});
      for (int s = S - 1; s >= 0; --s) {
        l.push_back({HYDRA_PHASE_B, {{k, s}}, str});
        l.push_back({HYDRA_PHASE_U, {{k, s}}, str});
      }
      longest = std::max(longest, l.size());
      lists.push_back(l);
    }
    // Spilled state: a model holds one state slot from each backward to the update behind it, so only as many
    // models as there are slots may be in flight at once; the lists are issued in waves of that many models.
    size_t wave = lists.size();
    if (c->spill) {
      wave = std::max<size_t>(1, std::min(wave, c->slots.size()));
      nstr = (int)std::min<size_t>(nstr, wave);
    }
    for (size_t w0 = 0; w0 < lists.size(); w0 += wave) {
      const size_t w1 = std::min(lists.size(), w0 + wave);
      for (size_t i = w0; i < w1; ++i)
        for (Bucket& b : lists[i]) b.stream = (int)((i - w0) % nstr);
      for (size_t pos = 0; pos < longest; ++pos)
        for (size_t i = w0; i < w1; ++i)
          if (pos < lists[i].size()) plan.push_back(lists[i][pos]);
    }
    return HYDRA_OK;
  }

  if (sch->policy == HYDRA_SCHED_EXPLICIT) {
    if (!sch->tasks || sch->n_tasks <= 0) return c->fail(HYDRA_ERR_INVALID_ARG, "explicit schedule without tasks");
    std::set<Task> done;
    for (int i = 0; i < sch->n_tasks; ++i) {
      Task t{sch->tasks[3 * i], sch->tasks[3 * i + 1], sch->tasks[3 * i + 2]};
      if (t.k < 0 || t.k >= K || t.s < 0 || t.s >= (int)c->models[t.k].shards.size() || t.ph < 0 || t.ph > 2)
        return c->fail(HYDRA_ERR_BAD_SCHEDULE, "task %d = (%d,%d,%d) does not exist", i, t.k, t.s, t.ph);
      if (!c->models[t.k].active) return c->fail(HYDRA_ERR_BAD_SCHEDULE, "task %d belongs to model %d, which is inactive", i, t.k);
      if (done.count(t))
        return c->fail(HYDRA_ERR_BAD_SCHEDULE, "task %d: %s(%d,%d) listed twice", i, ph_name(t.ph), t.k, t.s);
      for (const Task& p : preds_of(c, t))
        if (!done.count(p))
          return c->fail(HYDRA_ERR_BAD_SCHEDULE, "task %d: %s(%d,%d) is scheduled before %s(%d,%d)", i, ph_name(t.ph), t.k,
                         t.s, ph_name(p.ph), p.k, p.s);
      done.insert(t);
      // neighbours in the list with the same phase and shape share a launch group
      const uint64_t sig = c->models[t.k].shards[t.s].sig;
      bool joined = false;
      if (!plan.empty() && plan.back().ph == t.ph && (int)plan.back().members.size() < maxg) {
        const auto& mb = plan.back().members;
        bool same = c->models[mb[0].first].shards[mb[0].second].sig == sig;
        for (const auto& q : mb) same = same && q.first != t.k;
        if (same) {
          plan.back().members.push_back({t.k, t.s});
          joined = true;
        }
      }
      if (!joined) plan.push_back({t.ph, {{t.k, t.s}}, 0});
    }
    if (done.size() != total)
      return c->fail(HYDRA_ERR_BAD_SCHEDULE, "schedule lists %zu of the %zu (model, shard, phase) tasks", done.size(), total);
    return HYDRA_OK;
  }

  if (sch->policy != HYDRA_SCHED_SHARD_PARALLEL) return c->fail(HYDRA_ERR_INVALID_ARG, "unknown policy %d", sch->policy);

  // wavefronts of ready tasks; inside a wavefront tasks are bucketed by (phase, signature)
  int nc = ns >= 2 ? std::max(1, ns / 2) : 1;  // streams [0,nc): F and B; [nc,ns): U
  if (c->recompute) nc = std::min(nc, c->ws_streams);  // every compute stream needs its own activation workspaces
  int nu = ns - nc;
  if (c->opt.max_group == 0) {
    // launch-bound models (all of them together fill less than a quarter of the compute units with 256 x 256 tiles):
    // their kernels take microseconds, less than a dependency that crosses streams costs, so everything stays on
    // one stream and the launches simply queue
    long all_tiles = 0;
    for (int k = 0; k < K; ++k)
      if (c->models[k].active) all_tiles += min_tiles_of(c, c->models[k]);
    if (all_tiles < 64) {
      nc = 1;
      nu = 0;
    }
  }
  int next_u = 0;
  std::set<Task> issued;
  while (issued.size() < total) {
    std::vector<Task> ready, also_issued;
    for (int k = 0; k < K; ++k)
      for (int s = 0; c->models[k].active && s < (int)c->models[k].shards.size(); ++s)
        for (int ph = 0; ph < 3; ++ph) {
          Task t{k, s, ph};
          if (issued.count(t)) continue;
          bool ok = true;
          for (const Task& p : preds_of(c, t)) ok = ok && issued.count(p);
          if (ok) ready.push_back(t);
        }
    // deterministic bucket order: backward first (it is on the critical path), then forward, then update
    auto rank = [](int ph) { return ph == HYDRA_PHASE_B ? 0 : (ph == HYDRA_PHASE_F ? 1 : 2); };
    std::map<std::pair<int, uint64_t>, std::vector<Task>> groups;
    std::vector<std::pair<int, uint64_t>> order;
    for (const Task& t : ready) {
      auto key = std::make_pair(rank(t.ph), c->models[t.k].shards[t.s].sig);
      if (!groups.count(key)) order.push_back(key);
      groups[key].push_back(t);
    }
    std::stable_sort(order.begin(), order.end(), [](const auto& x, const auto& y) { return x.first < y.first; });
    int next_c = 0;
    for (const auto& key : order) {
      const std::vector<Task>& ts = groups[key];
      // update tasks stream their shard's state once: one launch for all of them; forward and backward groups are
      // sized by the tile count of their products unless the caller fixed the size
      const int gs = (c->opt.max_group > 0 || ts[0].ph == HYDRA_PHASE_U)
                         ? maxg : auto_group_size(c, c->models[ts[0].k], (int)ts.size(), nc, maxg);
      for (size_t i = 0; i < ts.size(); i += gs) {
        Bucket b;
        b.ph = ts[i].ph;
        for (size_t j = i; j < std::min(ts.size(), i + (size_t)gs); ++j) b.members.push_back({ts[j].k, ts[j].s});
        if (b.ph == HYDRA_PHASE_U && nu > 0) b.stream = nc + (next_u++ % nu);
        else b.stream = next_c++ % nc;
        plan.push_back(b);
        if (c->spill && b.ph == HYDRA_PHASE_B) {
          // a backward holds a state slot until its update has run: schedule the update right behind it
          Bucket u = b;
          u.ph = HYDRA_PHASE_U;
          u.stream = nu > 0 ? nc + (next_u++ % nu) : b.stream;
          plan.push_back(u);
          for (const auto& mem : u.members) also_issued.push_back({mem.first, mem.second, HYDRA_PHASE_U});
        }
      }
    }
    for (const Task& t : ready) issued.insert(t);
    for (const Task& t : also_issued) issued.insert(t);
  }
  merge_shard_spans(c, plan);
  return HYDRA_OK;
}

hydra_status run_epoch(hydra_ctx* c, const std::vector<Bucket>& plan, hydra_epoch_stats* stats) {
  const size_t nb = plan.size();
  c->launches = 0;
  c->grouped_tasks = 0;
  c->h2d_bytes = c->d2h_bytes = 0;
  if (!c->dry) {
    while (c->events.size() < 2 * nb) {
      hipEvent_t e;
      HYDRA_HIP(c, hipEventCreateWithFlags(&e, hipEventDisableTiming));
      c->events.push_back(e);
    }
    for (hipStream_t s : c->streams) HYDRA_HIP(c, hipStreamSynchronize(s));
    if (c->profiling) HYDRA_HIP(c, prof_epoch_begin(c));
  }
  struct Done { hipEvent_t ev; int stream; };
  std::map<Task, Done> last;  // most recent completion event of every task
  const auto t0 = std::chrono::steady_clock::now();
  for (int step = 0; step < c->n_batches; ++step) {
    for (size_t i = 0; i < nb; ++i) {
      const Bucket& b = plan[i];
      if (b.members.size() > 1) c->grouped_tasks += b.members.size() * (b.span + b.bspan);
      if (c->dry) {
        hydra_status st = HYDRA_OK;
        if (c->spill && b.ph == HYDRA_PHASE_B)
          for (const auto& mem : b.members)
            if ((st = spill_acquire(c, mem.first, mem.second, nullptr, true)) != HYDRA_OK) return st;
        st = run_bucket(c, b, step, step, nullptr);
        if (st != HYDRA_OK) return st;
        if (c->spill && b.ph == HYDRA_PHASE_U)
          for (const auto& mem : b.members)
            if ((st = spill_after_update(c, mem.first, mem.second, nullptr, true)) != HYDRA_OK) return st;
        continue;
      }
      hipStream_t s = c->streams[b.stream];
      std::vector<hipEvent_t> waited;
      hipError_t werr = hipSuccess;
      b.for_each_task([&](int k, int sh, int ph) {  // every task the group covers
        Task t{k, sh, ph};
        std::vector<Task> deps = preds_of(c, t);
        if (ph == HYDRA_PHASE_F) deps.push_back({t.k, t.s, HYDRA_PHASE_U});  // previous step's update
        for (const Task& d : deps) {
          auto it = last.find(d);
          if (it == last.end() || it->second.stream == b.stream) continue;
          if (std::find(waited.begin(), waited.end(), it->second.ev) != waited.end()) continue;
          if (werr == hipSuccess) werr = hipStreamWaitEvent(s, it->second.ev, 0);
          waited.push_back(it->second.ev);
        }
      });
      HYDRA_HIP(c, werr);
      hydra_status st = HYDRA_OK;
      if (c->spill && b.ph == HYDRA_PHASE_B)
        for (const auto& mem : b.members)
          if ((st = spill_acquire(c, mem.first, mem.second, s, c->sync_spill)) != HYDRA_OK) return st;
      if (c->spill && b.ph == HYDRA_PHASE_U)
        for (const auto& mem : b.members)
          if ((st = spill_before_update(c, mem.first, mem.second, s)) != HYDRA_OK) return st;
      st = run_bucket(c, b, step, step, s);
      if (st != HYDRA_OK) return st;
      if (c->spill && b.ph == HYDRA_PHASE_U)
        for (const auto& mem : b.members)
          if ((st = spill_after_update(c, mem.first, mem.second, s, c->sync_spill)) != HYDRA_OK) return st;
      hipEvent_t ev = c->events[(step & 1) * nb + i];
      HYDRA_HIP(c, hipEventRecord(ev, s));
      b.for_each_task([&](int k, int sh, int ph) { last[{k, sh, ph}] = {ev, b.stream}; });
    }
  }
  if (!c->dry) {
    for (hipStream_t s : c->streams) HYDRA_HIP(c, hipStreamSynchronize(s));
    if (c->copy_in) HYDRA_HIP(c, hipStreamSynchronize(c->copy_in));
    if (c->copy_out) HYDRA_HIP(c, hipStreamSynchronize(c->copy_out));
  }
  const auto t1 = std::chrono::steady_clock::now();
  if (!c->dry && c->profiling) {
    hydra_status ps = prof_collect(c);
    if (ps != HYDRA_OK) return ps;
  }
  // losses of this epoch
  for (int k = 0; k < c->K; ++k) {
    Model& m = c->models[k];
    if (!m.active) continue;
    std::vector<float> l(c->n_batches, 0.f);
    if (!c->dry) HYDRA_HIP(c, hipMemcpy(l.data(), m.loss_dev, l.size() * 4, hipMemcpyDeviceToHost));
    m.losses.insert(m.losses.end(), l.begin(), l.end());
  }
  if (stats) {
    stats->wall_ms = std::chrono::duration<double, std::milli>(t1 - t0).count();
    stats->h2d_bytes = c->h2d_bytes;
    stats->d2h_bytes = c->d2h_bytes;
    stats->launches = c->launches;
    stats->grouped_tasks = c->grouped_tasks;
    stats->peak_dev_bytes = c->peak_dev_bytes;
    stats->peak_host_bytes = c->peak_host_bytes;
    stats->steps = c->n_batches;
  }
  return HYDRA_OK;
}

}  // namespace hydra
