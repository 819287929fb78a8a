// The C boundary declared in include/hydra.h: argument checking, call-order checking and copies
// between caller memory and the device.  No exception leaves these functions.
#include <algorithm>
#include <cstring>
#include <new>
#include <vector>

#include "hydra_internal.h"

using namespace hydra;

static std::string g_create_error;

#define HYDRA_TRY try {
#define HYDRA_CATCH(c)                                                          \
  }                                                                             \
  catch (const std::bad_alloc&) { return (c)->fail(HYDRA_ERR_OOM_HOST, "host allocation failed"); } \
  catch (const std::exception& e) { return (c)->fail(HYDRA_ERR_DEVICE, "internal error: %s", e.what()); }

extern "C" {

hydra_status hydra_create(const hydra_options* opts, hydra_ctx** out) {
  if (!out) {
    g_create_error = "hydra_create: out is NULL";
    return HYDRA_ERR_INVALID_ARG;
  }
  hydra_ctx* c = nullptr;
  try {
    c = new hydra_ctx();
  } catch (...) {
    g_create_error = "hydra_create: host allocation failed";
    return HYDRA_ERR_OOM_HOST;
  }
  if (opts) c->opt = *opts;
  c->dry = c->opt.dry_run != 0;
  if (c->opt.max_group < 0 || c->opt.max_group > hydra::MAXG) {
    g_create_error = "hydra_create: max_group must be 0 (automatic) or 1..16";
    delete c;
    return HYDRA_ERR_INVALID_ARG;
  }
  if (c->opt.n_streams < 0 || (c->opt.n_streams > 0 && !c->opt.streams && !c->dry) ||
      ((c->opt.dev_alloc == nullptr) != (c->opt.dev_free == nullptr))) {
    g_create_error = "hydra_create: inconsistent options (streams / allocator callbacks)";
    delete c;
    return HYDRA_ERR_INVALID_ARG;
  }
  if (!c->dry) {
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) {
      g_create_error = "hydra_create: no HIP device is available (use dry_run for planning without a device)";
      delete c;
      return HYDRA_ERR_DEVICE;
    }
    hipError_t e = kernels_init();
    if (e == hipSuccess) e = mlp_fused_init();
    if (e != hipSuccess) {
      g_create_error = std::string("hydra_create: kernel set-up failed: ") + hipGetErrorString(e);
      delete c;
      return HYDRA_ERR_DEVICE;
    }
    if (c->opt.n_streams > 0) {
      for (int i = 0; i < c->opt.n_streams; ++i) c->streams.push_back(static_cast<hipStream_t>(c->opt.streams[i]));
    } else {
      c->own_streams = true;
      for (int i = 0; i < 4; ++i) {
        hipStream_t s;
        if (hipStreamCreateWithFlags(&s, hipStreamNonBlocking) != hipSuccess) {
          g_create_error = "hydra_create: stream creation failed";
          delete c;
          return HYDRA_ERR_DEVICE;
        }
        c->streams.push_back(s);
      }
    }
  }
  *out = c;
  return HYDRA_OK;
}

hydra_status hydra_destroy(hydra_ctx* c) {
  if (!c) return HYDRA_ERR_INVALID_ARG;
  if (!c->dry) {
    for (hipStream_t s : c->streams) (void)hipStreamSynchronize(s);
    for (hipEvent_t e : c->events) (void)hipEventDestroy(e);
    for (hipEvent_t e : c->prof_pool) (void)hipEventDestroy(e);
    if (c->prof_origin) (void)hipEventDestroy(c->prof_origin);
    spill_release_all(c);
    ctx_free_all(c);
    if (c->own_streams)
      for (hipStream_t s : c->streams) (void)hipStreamDestroy(s);
  }
  delete c;
  return HYDRA_OK;
}

const char* hydra_last_error(const hydra_ctx* c) { return c ? c->err.c_str() : g_create_error.c_str(); }

static hydra_status check_arch(hydra_ctx* c, const hydra_arch& a, int i) {
  if (a.kind < 0 || a.kind > 2) return c->fail(HYDRA_ERR_INVALID_ARG, "arch %d: unknown kind %d", i, a.kind);
  if (a.dtype != HYDRA_DTYPE_F32 && a.dtype != HYDRA_DTYPE_BF16) return c->fail(HYDRA_ERR_INVALID_ARG, "arch %d: unknown dtype", i);
  if (a.n_layers < (a.kind == HYDRA_KIND_MLP ? 0 : 1) || a.d_model < 1 || a.n_out < 1)
    return c->fail(HYDRA_ERR_INVALID_ARG, "arch %d: n_layers, d_model and n_out must be positive", i);
  if (a.d_model % 8) return c->fail(HYDRA_ERR_UNSUPPORTED, "arch %d: d_model must be a multiple of 8", i);
  if (a.kind == HYDRA_KIND_MLP) {
    if (a.d_in < 1 || a.d_in % 8) return c->fail(HYDRA_ERR_UNSUPPORTED, "arch %d: d_in must be a positive multiple of 8", i);
    if (a.act != HYDRA_ACT_RELU && a.act != HYDRA_ACT_GELU) return c->fail(HYDRA_ERR_INVALID_ARG, "arch %d: unknown activation", i);
  } else {
    if (a.n_heads < 1 || a.d_model % a.n_heads) return c->fail(HYDRA_ERR_INVALID_ARG, "arch %d: n_heads must divide d_model", i);
    if (a.d_ffn < 1 || a.d_ffn % 8) return c->fail(HYDRA_ERR_UNSUPPORTED, "arch %d: d_ffn must be a positive multiple of 8", i);
    if (a.max_seq < 1) return c->fail(HYDRA_ERR_INVALID_ARG, "arch %d: max_seq must be positive", i);
    if ((a.kind == HYDRA_KIND_DECODER) != (a.causal != 0))
      return c->fail(HYDRA_ERR_INVALID_ARG, "arch %d: decoders are causal, encoders are not", i);
  }
  return HYDRA_OK;
}

hydra_status hydra_define_models(hydra_ctx* c, int K, const hydra_arch* archs, int n_archs, const hydra_hparams* grid,
                                 uint64_t seed) {
  if (!c) return HYDRA_ERR_INVALID_ARG;
  HYDRA_TRY
  if (c->state != ST_CREATED) return c->fail(HYDRA_ERR_BAD_STATE, "models are already defined");
  if (K < 1 || !archs || !grid || (n_archs != 1 && n_archs != K))
    return c->fail(HYDRA_ERR_INVALID_ARG, "need K >= 1, archs with 1 or K entries and a grid with K entries");
  for (int i = 0; i < n_archs; ++i) {
    hydra_status st = check_arch(c, archs[i], i);
    if (st != HYDRA_OK) return st;
    if (archs[i].kind != archs[0].kind || archs[i].dtype != archs[0].dtype)
      return c->fail(HYDRA_ERR_UNSUPPORTED, "all models of a context must share kind and dtype");
  }
  for (int k = 0; k < K; ++k) {
    const hydra_hparams& h = grid[k];
    if (h.opt != HYDRA_OPT_SGD && h.opt != HYDRA_OPT_ADAM) return c->fail(HYDRA_ERR_INVALID_ARG, "grid %d: unknown optimizer", k);
    if (!(h.lr >= 0.0) || h.warmup_steps < 0) return c->fail(HYDRA_ERR_INVALID_ARG, "grid %d: lr and warmup must be >= 0", k);
    if (h.opt == HYDRA_OPT_ADAM && !(h.beta1 >= 0 && h.beta1 < 1 && h.beta2 >= 0 && h.beta2 < 1 && h.eps >= 0))
      return c->fail(HYDRA_ERR_INVALID_ARG, "grid %d: Adam needs 0 <= beta < 1 and eps >= 0", k);
  }
  c->K = K;
  c->seed = seed;
  c->models.assign(K, Model());
  for (int k = 0; k < K; ++k) {
    Model& m = c->models[k];
    m.arch = archs[n_archs == 1 ? 0 : k];
    m.hp = grid[k];
    hydra_status st = build_tensors(c, m);
    if (st == HYDRA_OK) st = cut_model(c, m, nullptr, 0);
    if (st != HYDRA_OK) {
      c->models.clear();
      return st;
    }
  }
  if (c->opt.auto_budget) {
    // memory-aware default: keep state resident while it leaves room for activations, otherwise spill it
    c->capacity = c->opt.device_capacity_bytes;
    if (!c->capacity && !c->dry) {
      size_t fr = 0, tot = 0;
      HYDRA_HIP(c, hipMemGetInfo(&fr, &tot));
      c->capacity = fr;
    }
    if (!c->capacity) {
      c->models.clear();
      return c->fail(HYDRA_ERR_INVALID_ARG, "auto_budget in a dry run needs device_capacity_bytes");
    }
    bool can_spill = true;
    for (const Model& m : c->models) can_spill = can_spill && m.arch.dtype == HYDRA_DTYPE_BF16 && m.hp.opt == HYDRA_OPT_ADAM;
    if (!c->opt.device_budget_bytes && can_spill && (double)resident_state_bytes(c) > 0.85 * (double)c->capacity)
      c->opt.device_budget_bytes = (size_t)(0.55 * (double)c->capacity);
  }
  c->spill = c->opt.device_budget_bytes > 0 && resident_state_bytes(c) > c->opt.device_budget_bytes;
  c->fuse = !c->spill && !c->opt.keep_grads;
  hydra_status st = c->spill ? spill_alloc_models(c) : alloc_models(c);
  if (st != HYDRA_OK) {
    if (!c->dry) spill_release_all(c);
    ctx_free_all(c);
    c->models.clear();
    return st;
  }
  for (Model& m : c->models)
    for (Shard& sh : m.shards) {  // re-point after allocation
      sh.p = m.p ? m.p + sh.off : nullptr;
      sh.m = m.m ? m.m + sh.off : nullptr;
      sh.v = m.v ? m.v + sh.off : nullptr;
      sh.g = m.g ? m.g + sh.off : nullptr;
      sh.w16 = m.w16 ? m.w16 + sh.off : nullptr;
    }
  c->state = ST_DEFINED;
  return HYDRA_OK;
  HYDRA_CATCH(c)
}

hydra_status hydra_shard(hydra_ctx* c, int model, const int32_t* cuts, int n_cuts) {
  if (!c) return HYDRA_ERR_INVALID_ARG;
  HYDRA_TRY
  if (c->state < ST_DEFINED) return c->fail(HYDRA_ERR_BAD_STATE, "define models before sharding them");
  if (model < -1 || model >= c->K) return c->fail(HYDRA_ERR_INVALID_ARG, "model %d does not exist", model);
  if (n_cuts < 0 || (n_cuts > 0 && !cuts)) return c->fail(HYDRA_ERR_INVALID_ARG, "n_cuts < 0 or cuts is NULL");
  if (c->state == ST_DATA && c->opt.activation_budget_bytes > 0 && c->models[0].arch.kind != HYDRA_KIND_MLP)
    return c->fail(HYDRA_ERR_BAD_STATE, "with an activation budget the hand-off buffers follow the cuts: shard before hydra_set_data");
  // validate every affected model before changing any
  for (int k = 0; k < c->K; ++k) {
    if (model != -1 && model != k) continue;
    Model tmp = c->models[k];
    tmp.shards.clear();  // the copy must not release the events and tables the real shards own
    hydra_status st = cut_model(c, tmp, cuts, n_cuts);
    if (st != HYDRA_OK) return st;
  }
  for (int k = 0; k < c->K; ++k)
    if (model == -1 || model == k) cut_model(c, c->models[k], cuts, n_cuts);
  if (c->state < ST_SHARDED) c->state = ST_SHARDED;
  return HYDRA_OK;
  HYDRA_CATCH(c)
}

// Smallest possible largest-shard cost of a contiguous partition of cost[0..U) into exactly S parts, and its cuts.
static size_t balanced_partition(const std::vector<size_t>& cost, int S, std::vector<int32_t>& cuts) {
  const int U = (int)cost.size();
  std::vector<size_t> pre(U + 1, 0);
  for (int i = 0; i < U; ++i) pre[i + 1] = pre[i] + cost[i];
  const size_t INF = ~(size_t)0;
  // best[s][i]: minimal largest part when the first i units form s parts
  std::vector<std::vector<size_t>> best(S + 1, std::vector<size_t>(U + 1, INF));
  std::vector<std::vector<int>> from(S + 1, std::vector<int>(U + 1, 0));
  best[0][0] = 0;
  for (int s = 1; s <= S; ++s)
    for (int i = s; i <= U; ++i)
      for (int j = s - 1; j < i; ++j) {
        if (best[s - 1][j] == INF) continue;
        const size_t v = std::max(best[s - 1][j], pre[i] - pre[j]);
        if (v < best[s][i]) {  // strict: ties keep the earliest cut, which makes the result unique
          best[s][i] = v;
          from[s][i] = j;
        }
      }
  cuts.clear();
  for (int s = S, i = U; s > 1; --s) {
    i = from[s][i];
    cuts.insert(cuts.begin(), i);
  }
  return best[S][U];
}

hydra_status hydra_auto_shard(hydra_ctx* c, int model, size_t max_shard_bytes, int n_shards, int32_t* cuts_out, int cap,
                              int* n_cuts) {
  if (!c) return HYDRA_ERR_INVALID_ARG;
  HYDRA_TRY
  if (c->state < ST_DEFINED) return c->fail(HYDRA_ERR_BAD_STATE, "define models before sharding them");
  if (model < -1 || model >= c->K) return c->fail(HYDRA_ERR_INVALID_ARG, "model %d does not exist", model);
  if (n_shards < 0 || (max_shard_bytes == 0 && n_shards < 1))
    return c->fail(HYDRA_ERR_INVALID_ARG, "give a byte bound, a shard count, or both");
  std::vector<std::vector<int32_t>> chosen(c->K);
  for (int k = 0; k < c->K; ++k) {
    if (model != -1 && model != k) continue;
    const Model& m = c->models[k];
    // bytes a shard holds per parameter: master, gradient, (Adam moments,) (bf16 working copy)
    const size_t per = 8 + (m.hp.opt == HYDRA_OPT_ADAM ? 8 : 0) + (m.arch.dtype == HYDRA_DTYPE_BF16 ? 2 : 0);
    std::vector<size_t> cost(m.n_units, 0);
    for (const Tensor& t : m.tensors) cost[t.unit] += (t.n + 63) / 64 * 64 * per;
    if (n_shards > m.n_units) return c->fail(HYDRA_ERR_INVALID_ARG, "model %d has %d layer units, fewer than %d shards", k, m.n_units, n_shards);
    int S = std::max(1, n_shards);
    std::vector<int32_t> cuts;
    size_t worst = balanced_partition(cost, S, cuts);
    while (max_shard_bytes && worst > max_shard_bytes) {
      if (S == m.n_units)
        return c->fail(HYDRA_ERR_INVALID_ARG, "model %d: one layer unit alone holds %zu bytes, more than the bound of %zu", k, worst,
                       max_shard_bytes);
      worst = balanced_partition(cost, ++S, cuts);
    }
    chosen[k] = cuts;
  }
  if (model >= 0) {
    if (n_cuts) *n_cuts = (int)chosen[model].size();
    if (cuts_out) {
      if (cap < (int)chosen[model].size())
        return c->fail(HYDRA_ERR_BUFFER_TOO_SMALL, "need room for %zu cuts, got %d", chosen[model].size(), cap);
      std::copy(chosen[model].begin(), chosen[model].end(), cuts_out);
    }
  }
  for (int k = 0; k < c->K; ++k) {
    if (model != -1 && model != k) continue;
    hydra_status st = hydra_shard(c, k, chosen[k].data(), (int)chosen[k].size());
    if (st != HYDRA_OK) return st;
  }
  return HYDRA_OK;
  HYDRA_CATCH(c)
}

hydra_status hydra_set_active(hydra_ctx* c, int model, int active) {
  if (!c) return HYDRA_ERR_INVALID_ARG;
  if (c->state < ST_DEFINED) return c->fail(HYDRA_ERR_BAD_STATE, "no models are defined");
  if (model < 0 || model >= c->K) return c->fail(HYDRA_ERR_INVALID_ARG, "model %d does not exist", model);
  c->models[model].active = active != 0;
  return HYDRA_OK;
}

hydra_status hydra_set_data(hydra_ctx* c, const void* inputs, const int32_t* tgt_pos, const int32_t* targets, int n_batches,
                            int B, int S_or_d, int P) {
  if (!c) return HYDRA_ERR_INVALID_ARG;
  HYDRA_TRY
  if (c->state < ST_SHARDED) return c->fail(HYDRA_ERR_BAD_STATE, "shard the models before setting data");
  if (!inputs || !targets || n_batches < 1 || B < 1) return c->fail(HYDRA_ERR_INVALID_ARG, "inputs/targets NULL or empty");
  const hydra_arch& a = c->models[0].arch;
  if (c->state == ST_DATA) {  // replacing the data set: batch geometry must stay (activations are sized by it)
    if (B != c->B || (a.kind != HYDRA_KIND_MLP && (S_or_d != c->S || P != c->P)))
      return c->fail(HYDRA_ERR_INVALID_ARG, "new data must keep the batch size (and sequence / target counts)");
    for (hipStream_t st : c->streams) HYDRA_HIP(c, hipStreamSynchronize(st));
    ctx_free(c, c->x_staged, c->x_bytes);
    ctx_free(c, c->ids, c->ids_bytes);
    ctx_free(c, c->tgt_pos, c->tp_bytes);
    ctx_free(c, c->targets, c->tg_bytes);
    ctx_free(c, c->csr_ptr, c->csr_ptr_bytes);
    ctx_free(c, c->csr_pos, c->csr_pos_bytes);
    c->x_staged = nullptr;
    c->ids = c->tgt_pos = c->targets = c->csr_ptr = c->csr_pos = nullptr;
  }
  c->n_batches = n_batches;
  c->B = B;
  hipStream_t s = c->dry ? nullptr : c->streams[0];
  if (a.kind == HYDRA_KIND_MLP) {
    if (S_or_d != a.d_in || P != 0 || tgt_pos) return c->fail(HYDRA_ERR_INVALID_ARG, "MLP data: S_or_d must equal d_in, P = 0, target_pos NULL");
    const size_t rows = (size_t)n_batches * B;
    for (size_t i = 0; i < rows; ++i)
      if (targets[i] < 0 || targets[i] >= a.n_out) return c->fail(HYDRA_ERR_INVALID_ARG, "target %zu out of range", i);
    const bool bf = a.dtype == HYDRA_DTYPE_BF16;
    c->ld_in = a.d_in;
    c->x_bytes = rows * c->ld_in * (bf ? 2 : 4);
    c->tg_bytes = rows * 4;
    c->x_staged = ctx_alloc(c, c->x_bytes);
    c->targets = static_cast<int32_t*>(ctx_alloc(c, c->tg_bytes));
    if (!c->dry) {
      if (!c->x_staged || !c->targets) return c->fail(HYDRA_ERR_OOM_DEVICE, "device allocation for the data failed");
      float* tmp = static_cast<float*>(ctx_alloc(c, rows * a.d_in * 4));
      if (!tmp) return c->fail(HYDRA_ERR_OOM_DEVICE, "device allocation for the data failed");
      HYDRA_HIP(c, hipMemcpyAsync(tmp, inputs, rows * a.d_in * 4, hipMemcpyHostToDevice, s));
      HYDRA_HIP(c, hipMemcpyAsync(c->targets, targets, rows * 4, hipMemcpyHostToDevice, s));
      HYDRA_HIP(c, launch_stage_rows(tmp, c->x_staged, (int)rows, a.d_in, c->ld_in, bf ? 1 : 0, s));
      HYDRA_HIP(c, hipStreamSynchronize(s));
      ctx_free(c, tmp, rows * a.d_in * 4);
    }
  } else {
    const int S = S_or_d, V = a.n_out;
    if (!tgt_pos || P < 1 || S < 1) return c->fail(HYDRA_ERR_INVALID_ARG, "Transformer data needs target_pos, P >= 1 and S >= 1");
    for (const Model& m : c->models) {
      if (S > m.arch.max_seq) return c->fail(HYDRA_ERR_INVALID_ARG, "S = %d exceeds max_seq = %d", S, m.arch.max_seq);
      if (m.arch.dtype != HYDRA_DTYPE_BF16) return c->fail(HYDRA_ERR_UNSUPPORTED, "Transformer models run in bf16 only");
      const int dh = m.arch.d_model / m.arch.n_heads;
      if (dh != 64 && dh != 128) return c->fail(HYDRA_ERR_UNSUPPORTED, "head width %d: the attention kernels take 64 or 128", dh);
    }
    if (P > S) return c->fail(HYDRA_ERR_INVALID_ARG, "P = %d target positions exceed S = %d", P, S);
    const int32_t* ids = static_cast<const int32_t*>(inputs);
    const size_t Tk = (size_t)B * S, NT = (size_t)B * P;
    std::vector<int32_t> rows((size_t)n_batches * NT), ptr((size_t)n_batches * (V + 1)), pos((size_t)n_batches * Tk);
    for (int nb = 0; nb < n_batches; ++nb) {
      const int32_t* id = ids + (size_t)nb * Tk;
      int32_t* rp = ptr.data() + (size_t)nb * (V + 1);
      std::fill(rp, rp + V + 1, 0);
      for (size_t t = 0; t < Tk; ++t) {
        if (id[t] < 0 || id[t] >= V) return c->fail(HYDRA_ERR_INVALID_ARG, "token id %d at batch %d is outside [0,%d)", id[t], nb, V);
        ++rp[id[t] + 1];
      }
      for (int v = 0; v < V; ++v) rp[v + 1] += rp[v];
      std::vector<int32_t> fill(rp, rp + V);
      int32_t* ps = pos.data() + (size_t)nb * Tk;
      for (size_t t = 0; t < Tk; ++t) ps[fill[id[t]]++] = (int32_t)t;   // ascending token index inside every id
      for (int b = 0; b < B; ++b)
        for (int p = 0; p < P; ++p) {
          const size_t i = ((size_t)nb * B + b) * P + p;
          if (tgt_pos[i] < 0 || tgt_pos[i] >= S || (p > 0 && tgt_pos[i] <= tgt_pos[i - 1]))
            return c->fail(HYDRA_ERR_INVALID_ARG, "target positions of sequence %d in batch %d must be ascending and inside [0,%d)", b, nb, S);
          if (targets[i] < 0 || targets[i] >= V) return c->fail(HYDRA_ERR_INVALID_ARG, "target %zu out of range", i);
          rows[i] = b * S + tgt_pos[i];
        }
    }
    c->S = S;
    c->P = P;
    c->ids_bytes = (size_t)n_batches * Tk * 4;
    c->tp_bytes = c->tg_bytes = (size_t)n_batches * NT * 4;
    c->csr_ptr_bytes = ptr.size() * 4;
    c->csr_pos_bytes = pos.size() * 4;
    c->ids = static_cast<int32_t*>(ctx_alloc(c, c->ids_bytes));
    c->tgt_pos = static_cast<int32_t*>(ctx_alloc(c, c->tp_bytes));
    c->targets = static_cast<int32_t*>(ctx_alloc(c, c->tg_bytes));
    c->csr_ptr = static_cast<int32_t*>(ctx_alloc(c, c->csr_ptr_bytes));
    c->csr_pos = static_cast<int32_t*>(ctx_alloc(c, c->csr_pos_bytes));
    if (!c->dry) {
      if (!c->ids || !c->tgt_pos || !c->targets || !c->csr_ptr || !c->csr_pos)
        return c->fail(HYDRA_ERR_OOM_DEVICE, "device allocation for the data failed");
      HYDRA_HIP(c, hipMemcpy(c->ids, ids, c->ids_bytes, hipMemcpyHostToDevice));
      HYDRA_HIP(c, hipMemcpy(c->tgt_pos, rows.data(), c->tp_bytes, hipMemcpyHostToDevice));
      HYDRA_HIP(c, hipMemcpy(c->targets, targets, c->tg_bytes, hipMemcpyHostToDevice));
      HYDRA_HIP(c, hipMemcpy(c->csr_ptr, ptr.data(), c->csr_ptr_bytes, hipMemcpyHostToDevice));
      HYDRA_HIP(c, hipMemcpy(c->csr_pos, pos.data(), c->csr_pos_bytes, hipMemcpyHostToDevice));
    }
  }
  hydra_status st = alloc_activations(c);
  if (st != HYDRA_OK) return st;
  c->state = ST_DATA;
  return HYDRA_OK;
  HYDRA_CATCH(c)
}

hydra_status hydra_train_epoch(hydra_ctx* c, const hydra_schedule* sch, hydra_epoch_stats* stats) {
  if (!c) return HYDRA_ERR_INVALID_ARG;
  HYDRA_TRY
  if (c->state != ST_DATA) return c->fail(HYDRA_ERR_BAD_STATE, "set the data before training");
  if (!sch) return c->fail(HYDRA_ERR_INVALID_ARG, "schedule is NULL");
  std::vector<Bucket> plan;
  hydra_status st = HYDRA_OK;
  if (c->spill) {
    if ((st = spill_prepare(c)) != HYDRA_OK) return st;
    c->sync_spill = sch->policy == HYDRA_SCHED_SEQUENTIAL;
  }
  if (c->fuse && (st = build_update_chunks(c)) != HYDRA_OK) return st;
  st = build_plan(c, sch, plan);
  if (st != HYDRA_OK) return st;
  hydra_epoch_stats local{};
  st = run_epoch(c, plan, &local);
  if (st != HYDRA_OK) return st;
  for (Model& m : c->models)
    if (m.active) m.t += c->n_batches;
  if (stats) *stats = local;
  return HYDRA_OK;
  HYDRA_CATCH(c)
}

static hydra_status copy_out(hydra_ctx* c, int model, int tensor, float* dst, size_t cap, size_t* n_written, bool grads) {
  if (c->state < ST_DEFINED) return c->fail(HYDRA_ERR_BAD_STATE, "no models are defined");
  if (model < 0 || model >= c->K) return c->fail(HYDRA_ERR_INVALID_ARG, "model %d does not exist", model);
  Model& m = c->models[model];
  const int nt = (int)m.tensors.size();
  if (tensor < -1 || tensor >= nt) return c->fail(HYDRA_ERR_INVALID_ARG, "tensor %d does not exist", tensor);
  size_t need = 0;
  for (int j = 0; j < nt; ++j)
    if (tensor == -1 || tensor == j) need += m.tensors[j].n;
  if (!n_written) return c->fail(HYDRA_ERR_INVALID_ARG, "n_written is NULL");
  if (cap < need || !dst) {
    *n_written = need;
    return c->fail(HYDRA_ERR_BUFFER_TOO_SMALL, "need room for %zu floats, got %zu", need, cap);
  }
  if (c->dry) return c->fail(HYDRA_ERR_BAD_STATE, "a dry-run context holds no values");
  for (hipStream_t s : c->streams) HYDRA_HIP(c, hipStreamSynchronize(s));
  if (c->spill && grads) return c->fail(HYDRA_ERR_UNSUPPORTED, "gradients are transient while state is spilled to host memory");
  if (c->fuse && grads)
    return c->fail(HYDRA_ERR_UNSUPPORTED, "weight gradients are not stored when updates run inside the gradient kernels; create the context with keep_grads = 1");
  if (c->spill) {
    if (c->copy_out) HYDRA_HIP(c, hipStreamSynchronize(c->copy_out));
    size_t o2 = 0;
    for (int j = 0; j < nt; ++j) {
      if (tensor != -1 && tensor != j) continue;
      m.host_p.pieces(m.tensors[j].off, m.tensors[j].n, [&](float* h, size_t at, size_t take) { memcpy(dst + o2 + at, h, take * 4); });
      o2 += m.tensors[j].n;
    }
    *n_written = need;
    return HYDRA_OK;
  }
  const float* src = grads ? m.g : m.p;
  size_t o = 0;
  for (int j = 0; j < nt; ++j) {
    if (tensor != -1 && tensor != j) continue;
    HYDRA_HIP(c, hipMemcpy(dst + o, src + m.tensors[j].off, m.tensors[j].n * 4, hipMemcpyDeviceToHost));
    o += m.tensors[j].n;
  }
  *n_written = need;
  return HYDRA_OK;
}

hydra_status hydra_read_params(hydra_ctx* c, int model, int tensor, float* dst, size_t cap, size_t* n_written) {
  if (!c) return HYDRA_ERR_INVALID_ARG;
  HYDRA_TRY
  return copy_out(c, model, tensor, dst, cap, n_written, false);
  HYDRA_CATCH(c)
}

hydra_status hydra_read_grads(hydra_ctx* c, int model, int tensor, float* dst, size_t cap, size_t* n_written) {
  if (!c) return HYDRA_ERR_INVALID_ARG;
  HYDRA_TRY
  return copy_out(c, model, tensor, dst, cap, n_written, true);
  HYDRA_CATCH(c)
}

hydra_status hydra_write_params(hydra_ctx* c, int model, int tensor, const float* src, size_t n) {
  if (!c) return HYDRA_ERR_INVALID_ARG;
  HYDRA_TRY
  if (c->state < ST_DEFINED) return c->fail(HYDRA_ERR_BAD_STATE, "no models are defined");
  if (model < 0 || model >= c->K) return c->fail(HYDRA_ERR_INVALID_ARG, "model %d does not exist", model);
  Model& m = c->models[model];
  const int nt = (int)m.tensors.size();
  if (tensor < -1 || tensor >= nt || !src) return c->fail(HYDRA_ERR_INVALID_ARG, "tensor %d does not exist or src is NULL", tensor);
  size_t need = 0;
  for (int j = 0; j < nt; ++j)
    if (tensor == -1 || tensor == j) need += m.tensors[j].n;
  if (n != need) return c->fail(HYDRA_ERR_INVALID_ARG, "expected %zu floats, got %zu", need, n);
  if (c->dry) return HYDRA_OK;
  for (hipStream_t s : c->streams) HYDRA_HIP(c, hipStreamSynchronize(s));
  size_t o = 0;
  for (int j = 0; j < nt; ++j) {
    if (tensor != -1 && tensor != j) continue;
    const Tensor& t = m.tensors[j];
    if (c->spill) {
      m.host_p.pieces(t.off, t.n, [&](float* h, size_t at, size_t take) { memcpy(h, src + o + at, take * 4); });
      float* tmp = static_cast<float*>(ctx_alloc(c, t.n * 4));
      if (!tmp) return c->fail(HYDRA_ERR_OOM_DEVICE, "device allocation failed");
      HYDRA_HIP(c, hipMemcpy(tmp, src + o, t.n * 4, hipMemcpyHostToDevice));
      HYDRA_HIP(c, launch_cast_bf16(tmp, m.w16 + t.off, t.n, c->streams[0]));
      if (m.voff[j] >= 0) HYDRA_HIP(c, hipMemcpyAsync(m.pv + m.voff[j], tmp, t.n * 4, hipMemcpyDeviceToDevice, c->streams[0]));
      HYDRA_HIP(c, hipStreamSynchronize(c->streams[0]));
      ctx_free(c, tmp, t.n * 4);
      o += t.n;
      continue;
    }
    HYDRA_HIP(c, hipMemcpy(m.p + t.off, src + o, t.n * 4, hipMemcpyHostToDevice));
    if (m.w16) HYDRA_HIP(c, launch_cast_bf16(m.p + t.off, m.w16 + t.off, t.n, c->streams[0]));
    o += t.n;
  }
  HYDRA_HIP(c, hipStreamSynchronize(c->streams[0]));
  return HYDRA_OK;
  HYDRA_CATCH(c)
}

hydra_status hydra_read_optimizer_state(hydra_ctx* c, int model, float* m_dst, float* v_dst, size_t cap, size_t* n_written,
                                        int64_t* steps) {
  if (!c) return HYDRA_ERR_INVALID_ARG;
  HYDRA_TRY
  if (c->state < ST_DEFINED) return c->fail(HYDRA_ERR_BAD_STATE, "no models are defined");
  if (model < 0 || model >= c->K) return c->fail(HYDRA_ERR_INVALID_ARG, "model %d does not exist", model);
  if (!n_written || !steps) return c->fail(HYDRA_ERR_INVALID_ARG, "n_written or steps is NULL");
  Model& m = c->models[model];
  size_t need = 0;
  if (m.hp.opt == HYDRA_OPT_ADAM)
    for (const Tensor& t : m.tensors) need += t.n;
  if (need && (cap < need || !m_dst || !v_dst)) {
    *n_written = need;
    return c->fail(HYDRA_ERR_BUFFER_TOO_SMALL, "need room for %zu floats per array, got %zu", need, cap);
  }
  if (c->dry) return c->fail(HYDRA_ERR_BAD_STATE, "a dry-run context holds no values");
  for (hipStream_t s : c->streams) HYDRA_HIP(c, hipStreamSynchronize(s));
  if (c->copy_out) HYDRA_HIP(c, hipStreamSynchronize(c->copy_out));
  size_t o = 0;
  if (need)
    for (const Tensor& t : m.tensors) {
      if (c->spill) {
        m.host_m.pieces(t.off, t.n, [&](float* h, size_t at, size_t take) { memcpy(m_dst + o + at, h, take * 4); });
        m.host_v.pieces(t.off, t.n, [&](float* h, size_t at, size_t take) { memcpy(v_dst + o + at, h, take * 4); });
      } else {
        HYDRA_HIP(c, hipMemcpy(m_dst + o, m.m + t.off, t.n * 4, hipMemcpyDeviceToHost));
        HYDRA_HIP(c, hipMemcpy(v_dst + o, m.v + t.off, t.n * 4, hipMemcpyDeviceToHost));
      }
      o += t.n;
    }
  *n_written = need;
  *steps = (int64_t)m.t;
  return HYDRA_OK;
  HYDRA_CATCH(c)
}

hydra_status hydra_write_optimizer_state(hydra_ctx* c, int model, const float* m_src, const float* v_src, size_t n,
                                         int64_t steps) {
  if (!c) return HYDRA_ERR_INVALID_ARG;
  HYDRA_TRY
  if (c->state < ST_DEFINED) return c->fail(HYDRA_ERR_BAD_STATE, "no models are defined");
  if (model < 0 || model >= c->K) return c->fail(HYDRA_ERR_INVALID_ARG, "model %d does not exist", model);
  if (steps < 0) return c->fail(HYDRA_ERR_INVALID_ARG, "steps must be >= 0");
  Model& m = c->models[model];
  size_t need = 0;
  if (m.hp.opt == HYDRA_OPT_ADAM)
    for (const Tensor& t : m.tensors) need += t.n;
  if (n != need || (need && (!m_src || !v_src))) return c->fail(HYDRA_ERR_INVALID_ARG, "expected %zu floats per array, got %zu", need, n);
  m.t = (long)steps;
  if (c->dry || !need) return HYDRA_OK;
  for (hipStream_t s : c->streams) HYDRA_HIP(c, hipStreamSynchronize(s));
  if (c->copy_out) HYDRA_HIP(c, hipStreamSynchronize(c->copy_out));
  size_t o = 0;
  for (const Tensor& t : m.tensors) {
    if (c->spill) {
      m.host_m.pieces(t.off, t.n, [&](float* h, size_t at, size_t take) { memcpy(h, m_src + o + at, take * 4); });
      m.host_v.pieces(t.off, t.n, [&](float* h, size_t at, size_t take) { memcpy(h, v_src + o + at, take * 4); });
    } else {
      HYDRA_HIP(c, hipMemcpy(m.m + t.off, m_src + o, t.n * 4, hipMemcpyHostToDevice));
      HYDRA_HIP(c, hipMemcpy(m.v + t.off, v_src + o, t.n * 4, hipMemcpyHostToDevice));
    }
    o += t.n;
  }
  return HYDRA_OK;
  HYDRA_CATCH(c)
}

hydra_status hydra_read_loss(hydra_ctx* c, int model, float* dst, size_t cap, size_t* n_written) {
  if (!c) return HYDRA_ERR_INVALID_ARG;
  HYDRA_TRY
  if (c->state < ST_DEFINED) return c->fail(HYDRA_ERR_BAD_STATE, "no models are defined");
  if (model < 0 || model >= c->K) return c->fail(HYDRA_ERR_INVALID_ARG, "model %d does not exist", model);
  if (!n_written) return c->fail(HYDRA_ERR_INVALID_ARG, "n_written is NULL");
  const std::vector<float>& l = c->models[model].losses;
  if (cap < l.size() || (!dst && !l.empty())) {
    *n_written = l.size();
    return c->fail(HYDRA_ERR_BUFFER_TOO_SMALL, "need room for %zu floats, got %zu", l.size(), cap);
  }
  if (!l.empty()) memcpy(dst, l.data(), l.size() * 4);
  *n_written = l.size();
  return HYDRA_OK;
  HYDRA_CATCH(c)
}

hydra_status hydra_tensor_count(hydra_ctx* c, int model, int* n_tensors) {
  if (!c) return HYDRA_ERR_INVALID_ARG;
  if (c->state < ST_DEFINED) return c->fail(HYDRA_ERR_BAD_STATE, "no models are defined");
  if (model < 0 || model >= c->K || !n_tensors) return c->fail(HYDRA_ERR_INVALID_ARG, "bad model or NULL output");
  *n_tensors = (int)c->models[model].tensors.size();
  return HYDRA_OK;
}

hydra_status hydra_tensor_shape(hydra_ctx* c, int model, int tensor, int* rows, int* cols) {
  if (!c) return HYDRA_ERR_INVALID_ARG;
  if (c->state < ST_DEFINED) return c->fail(HYDRA_ERR_BAD_STATE, "no models are defined");
  if (model < 0 || model >= c->K || !rows || !cols) return c->fail(HYDRA_ERR_INVALID_ARG, "bad model or NULL output");
  const Model& m = c->models[model];
  if (tensor < 0 || tensor >= (int)m.tensors.size()) return c->fail(HYDRA_ERR_INVALID_ARG, "tensor %d does not exist", tensor);
  *rows = m.tensors[tensor].rows;
  *cols = m.tensors[tensor].cols;
  return HYDRA_OK;
}

hydra_status hydra_shard_count(hydra_ctx* c, int model, int* n_shards) {
  if (!c) return HYDRA_ERR_INVALID_ARG;
  if (c->state < ST_DEFINED) return c->fail(HYDRA_ERR_BAD_STATE, "no models are defined");
  if (model < 0 || model >= c->K || !n_shards) return c->fail(HYDRA_ERR_INVALID_ARG, "bad model or NULL output");
  *n_shards = (int)c->models[model].shards.size();
  return HYDRA_OK;
}

}  // extern "C"
