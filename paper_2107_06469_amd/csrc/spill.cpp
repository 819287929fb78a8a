// Residency manager: when the parameters and optimizer state of all models do not fit the device
// budget, the fp32 master weights and the Adam moments of every shard live in pinned host memory and
// visit the device only around their update (paper, Approach: shard-level work "extends the capacity
// of model-selection systems to larger-than-memory models"; here the extra capacity is host DRAM).
//
// Always resident: the bf16 working weights (forward and backward read only those) and a small fp32
// copy of every vector tensor (biases, LayerNorm gains), which kernels read in fp32.
// Slots: device buffers of 4 x max-shard-elements floats (master, m, v, gradient).  A shard takes a
// slot when its backward is issued (the gradient is written there), its state is copied in on the
// copy-in stream while the backward runs, the update waits for that copy, and the state is copied back
// on the copy-out stream, after which the slot is free again.  All ordering is by HIP events; the host
// never waits.  Values are bit-identical to the resident path: the same kernels see the same numbers.
#include <algorithm>
#include <cstring>

#include "hydra_internal.h"

namespace hydra {

static size_t rup(size_t v, size_t a) { return (v + a - 1) / a * a; }

// n zero-filled floats of pinned host memory
static hydra_status host_alloc(hydra_ctx* c, HostBlock* out, size_t n) {
  const size_t bytes = n * 4;
  c->host_bytes += bytes;
  c->peak_host_bytes = std::max(c->peak_host_bytes, c->host_bytes);
  if (c->opt.host_budget_bytes && c->host_bytes > c->opt.host_budget_bytes)
    return c->fail(HYDRA_ERR_OOM_HOST, "pinned host memory for spilled state (%zu bytes) exceeds the host budget", c->host_bytes);
  out->chunk.clear();
  out->n = n;
  if (c->dry) return HYDRA_OK;
  for (size_t at = 0; at < n; at += HostBlock::CHUNK) {
    const size_t take = std::min(HostBlock::CHUNK, n - at);
    void* p = nullptr;
    if (hipHostMalloc(&p, take * 4, hipHostMallocDefault) != hipSuccess)
      return c->fail(HYDRA_ERR_OOM_HOST, "hipHostMalloc of %zu bytes failed (%zu bytes of pinned memory held)", take * 4, c->host_bytes);
    c->host_allocs.push_back(p);
    out->chunk.push_back(static_cast<float*>(p));
    memset(p, 0, take * 4);
  }
  return HYDRA_OK;
}

// copies elements [off, off+cnt) between a host block and device memory, piece by piece, on stream s
static hipError_t copy_in_pieces(const HostBlock& hb, size_t off, size_t cnt, float* dev, hipStream_t s) {
  hipError_t e = hipSuccess;
  hb.pieces(off, cnt, [&](float* h, size_t at, size_t take) {
    if (e == hipSuccess) e = hipMemcpyAsync(dev + at, h, take * 4, hipMemcpyHostToDevice, s);
  });
  return e;
}
static hipError_t copy_out_pieces(const HostBlock& hb, size_t off, size_t cnt, const float* dev, hipStream_t s) {
  hipError_t e = hipSuccess;
  hb.pieces(off, cnt, [&](float* h, size_t at, size_t take) {
    if (e == hipSuccess) e = hipMemcpyAsync(h, dev + at, take * 4, hipMemcpyDeviceToHost, s);
  });
  return e;
}

// bytes the resident path would hold for parameters, gradients, optimizer state and working copies
size_t resident_state_bytes(const hydra_ctx* c) {
  size_t total = 0;
  for (const Model& m : c->models)
    total += m.n_block * (4 + 4 + (m.hp.opt == HYDRA_OPT_ADAM ? 8 : 0) + (m.arch.dtype == HYDRA_DTYPE_BF16 ? 2 : 0));
  return total;
}

// define_models in spill mode: working weights and vectors on the device, master/m/v in pinned host memory
hydra_status spill_alloc_models(hydra_ctx* c) {
  hipStream_t s = c->dry ? nullptr : c->streams[0];
  size_t max_tensor = 0;
  for (Model& m : c->models) {
    if (m.arch.dtype != HYDRA_DTYPE_BF16 || m.hp.opt != HYDRA_OPT_ADAM)
      return c->fail(HYDRA_ERR_UNSUPPORTED, "spilling to host memory is implemented for bf16 models trained with Adam");
    m.voff.assign(m.tensors.size(), -1);
    m.n_vec = 0;
    for (size_t j = 0; j < m.tensors.size(); ++j) {
      max_tensor = std::max(max_tensor, m.tensors[j].n);
      if (m.tensors[j].rows == 1) {
        m.voff[j] = (long)m.n_vec;
        m.n_vec += rup(m.tensors[j].n, 64);
      }
    }
  }
  float* tmp = static_cast<float*>(ctx_alloc(c, rup(max_tensor, 64) * 4));
  if (!tmp && !c->dry) return c->fail(HYDRA_ERR_OOM_DEVICE, "device allocation failed");
  for (int k = 0; k < c->K; ++k) {
    Model& m = c->models[k];
    m.w16 = static_cast<bf16_t*>(ctx_alloc(c, m.n_block * 2));
    m.pv = static_cast<float*>(ctx_alloc(c, std::max<size_t>(m.n_vec, 64) * 4));
    if (!c->dry && (!m.w16 || !m.pv)) return c->fail(HYDRA_ERR_OOM_DEVICE, "device allocation failed");
    c->state_bytes += m.n_block * 2 + std::max<size_t>(m.n_vec, 64) * 4;
    hydra_status st;
    if ((st = host_alloc(c, &m.host_p, m.n_block)) != HYDRA_OK) return st;
    if ((st = host_alloc(c, &m.host_m, m.n_block)) != HYDRA_OK) return st;
    if ((st = host_alloc(c, &m.host_v, m.n_block)) != HYDRA_OK) return st;
    if (c->dry) continue;
    HYDRA_HIP(c, launch_fill_u32(reinterpret_cast<uint32_t*>(m.w16), m.n_block / 2, 0u, s));
    HYDRA_HIP(c, launch_fill_f32(m.pv, std::max<size_t>(m.n_vec, 64), 0.f, s));
    for (size_t j = 0; j < m.tensors.size(); ++j) {
      const Tensor& t = m.tensors[j];
      if (t.init == INIT_ZERO) continue;
      if (t.init == INIT_ONE) HYDRA_HIP(c, launch_fill_f32(tmp, t.n, 1.f, s));
      else HYDRA_HIP(c, launch_init_uniform(tmp, t.n, tensor_key(c->seed, k, (int)j), t.a, s));
      HYDRA_HIP(c, launch_cast_bf16(tmp, m.w16 + t.off, t.n, s));
      if (m.voff[j] >= 0) HYDRA_HIP(c, hipMemcpyAsync(m.pv + m.voff[j], tmp, t.n * 4, hipMemcpyDeviceToDevice, s));
      HYDRA_HIP(c, copy_out_pieces(m.host_p, t.off, t.n, tmp, s));
      HYDRA_HIP(c, hipStreamSynchronize(s));
    }
  }
  if (!c->dry) {
    ctx_free(c, tmp, rup(max_tensor, 64) * 4);
    hipStream_t cs[2];
    for (int i = 0; i < 2; ++i) HYDRA_HIP(c, hipStreamCreateWithFlags(&cs[i], hipStreamNonBlocking));
    c->copy_in = cs[0];
    c->copy_out = cs[1];
  } else {
    c->dev_bytes -= rup(rup(max_tensor, 64) * 4, 256);
  }
  return HYDRA_OK;
}

// slots for the coming epoch (shard sizes are known now)
hydra_status spill_prepare(hydra_ctx* c) {
  size_t max_n = 0, n_shards = 0;
  for (const Model& m : c->models)
    for (const Shard& sh : m.shards) {
      max_n = std::max(max_n, sh.n);
      ++n_shards;
    }
  for (auto& sl : c->slots) sl.held = false;
  for (Model& m : c->models)
    for (Shard& sh : m.shards) sh.slot = -1;
  if (max_n == c->slot_elems && !c->slots.empty()) return HYDRA_OK;
  for (auto& sl : c->slots) ctx_free(c, sl.base, c->slot_elems * 16);
  c->slots.clear();
  c->slot_elems = max_n;
  const size_t slot_bytes = max_n * 16;
  // the budget bounds parameter and optimizer-state bytes: what the resident working weights and vectors leave
  const size_t left = c->opt.device_budget_bytes > c->state_bytes ? c->opt.device_budget_bytes - c->state_bytes : 0;
  size_t n = std::min(left / std::max<size_t>(slot_bytes, 1), n_shards);
  if (n < 1) return c->fail(HYDRA_ERR_OOM_DEVICE, "device budget leaves no room for one shard's state (%zu bytes needed, %zu left)", slot_bytes, left);
  for (size_t i = 0; i < n; ++i) {
    hydra_ctx::Slot sl;
    sl.base = static_cast<float*>(ctx_alloc(c, slot_bytes));
    if (!sl.base && !c->dry) return c->fail(HYDRA_ERR_OOM_DEVICE, "device allocation of a %zu-byte slot failed", slot_bytes);
    if (!c->dry) {
      HYDRA_HIP(c, hipEventCreateWithFlags(&sl.free_ev, hipEventDisableTiming));
      HYDRA_HIP(c, launch_fill_f32(sl.base, max_n * 4, 0.f, c->streams[0]));
      HYDRA_HIP(c, hipStreamSynchronize(c->streams[0]));
    }
    c->slots.push_back(sl);
  }
  c->next_slot = 0;
  return HYDRA_OK;
}

int spill_max_group(const hydra_ctx* c) { return std::max<int>(1, (int)c->slots.size() / 2); }

// before the backward of (k,s) is issued on `compute`: give the shard a slot and start copying its state in
hydra_status spill_acquire(hydra_ctx* c, int k, int s, hipStream_t compute, bool synchronous) {
  Model& m = c->models[k];
  Shard& sh = m.shards[s];
  // first slot, in ring order from the one after the last grant, whose tenant's update has been scheduled
  size_t at = c->next_slot, tried = 0;
  while (tried < c->slots.size() && c->slots[at].held) {
    at = (at + 1) % c->slots.size();
    ++tried;
  }
  if (tried == c->slots.size())
    return c->fail(HYDRA_ERR_BAD_SCHEDULE, "backward of (%d,%d): the %zu state slots the device budget allows are all held "
                   "by shards whose update has not been scheduled yet", k, s, c->slots.size());
  hydra_ctx::Slot& sl = c->slots[at];
  sl.held = true;
  c->next_slot = (at + 1) % c->slots.size();
  sh.p = sl.base;
  sh.m = sl.base + c->slot_elems;
  sh.v = sl.base + 2 * c->slot_elems;
  sh.g = sl.base + 3 * c->slot_elems;
  sh.slot = (int)(&sl - c->slots.data());
  const size_t bytes = sh.n * 4;
  c->h2d_bytes += 3 * bytes;
  if (c->dry) return HYDRA_OK;
  hipStream_t in = synchronous ? compute : c->copy_in;
  if (sl.used) {  // the previous tenant's state must have left
    HYDRA_HIP(c, hipStreamWaitEvent(in, sl.free_ev, 0));
    if (in != compute) HYDRA_HIP(c, hipStreamWaitEvent(compute, sl.free_ev, 0));
  }
  sl.used = true;
  // the shard's own state must have reached host memory: its copy-out of the previous step runs on another stream
  // and nothing else orders it before this copy-in (the slot's event belongs to whichever shard held the slot last)
  if (sh.stored_ev) HYDRA_HIP(c, hipStreamWaitEvent(in, sh.stored_ev, 0));
  hipEvent_t pa = nullptr;
  if (c->profiling) HYDRA_HIP(c, prof_begin(c, in, &pa));
  HYDRA_HIP(c, copy_in_pieces(m.host_p, sh.off, sh.n, sh.p, in));
  HYDRA_HIP(c, copy_in_pieces(m.host_m, sh.off, sh.n, sh.m, in));
  HYDRA_HIP(c, copy_in_pieces(m.host_v, sh.off, sh.n, sh.v, in));
  if (c->profiling) HYDRA_HIP(c, prof_end(c, in, pa, HYDRA_K_COPY_H2D, 0.0, 3.0 * bytes));
  if (!sh.loaded_ev) HYDRA_HIP(c, hipEventCreateWithFlags(&sh.loaded_ev, hipEventDisableTiming));
  HYDRA_HIP(c, hipEventRecord(sh.loaded_ev, in));
  return HYDRA_OK;
}

// before the update of (k,s) is issued on `compute`
hydra_status spill_before_update(hydra_ctx* c, int k, int s, hipStream_t compute) {
  Shard& sh = c->models[k].shards[s];
  if (c->dry) return HYDRA_OK;
  if (sh.slot < 0 || !sh.loaded_ev) return c->fail(HYDRA_ERR_BAD_STATE, "update of a shard that holds no slot");
  HYDRA_HIP(c, hipStreamWaitEvent(compute, sh.loaded_ev, 0));
  return HYDRA_OK;
}

// after the update of (k,s) has been issued on `compute`: refresh the resident vectors, copy the state out
hydra_status spill_after_update(hydra_ctx* c, int k, int s, hipStream_t compute, bool synchronous) {
  Model& m = c->models[k];
  Shard& sh = m.shards[s];
  const size_t bytes = sh.n * 4;
  c->d2h_bytes += 3 * bytes;
  if (sh.slot >= 0) c->slots[sh.slot].held = false;
  if (c->dry) {
    sh.slot = -1;
    return HYDRA_OK;
  }
  for (int j = sh.t0; j < sh.t1; ++j)
    if (m.voff[j] >= 0)
      HYDRA_HIP(c, hipMemcpyAsync(m.pv + m.voff[j], sh.p + (m.tensors[j].off - sh.off), m.tensors[j].n * 4,
                                  hipMemcpyDeviceToDevice, compute));
  hydra_ctx::Slot& sl = c->slots[sh.slot];
  hipStream_t out = synchronous ? compute : c->copy_out;
  if (out != compute) {
    if (!sh.updated_ev) HYDRA_HIP(c, hipEventCreateWithFlags(&sh.updated_ev, hipEventDisableTiming));
    HYDRA_HIP(c, hipEventRecord(sh.updated_ev, compute));
    HYDRA_HIP(c, hipStreamWaitEvent(out, sh.updated_ev, 0));
  }
  hipEvent_t pa = nullptr;
  if (c->profiling) HYDRA_HIP(c, prof_begin(c, out, &pa));
  HYDRA_HIP(c, copy_out_pieces(m.host_p, sh.off, sh.n, sh.p, out));
  HYDRA_HIP(c, copy_out_pieces(m.host_m, sh.off, sh.n, sh.m, out));
  HYDRA_HIP(c, copy_out_pieces(m.host_v, sh.off, sh.n, sh.v, out));
  if (c->profiling) HYDRA_HIP(c, prof_end(c, out, pa, HYDRA_K_COPY_D2H, 0.0, 3.0 * bytes));
  HYDRA_HIP(c, hipEventRecord(sl.free_ev, out));
  if (!sh.stored_ev) HYDRA_HIP(c, hipEventCreateWithFlags(&sh.stored_ev, hipEventDisableTiming));
  HYDRA_HIP(c, hipEventRecord(sh.stored_ev, out));
  sh.p = sh.m = sh.v = sh.g = nullptr;
  sh.slot = -1;
  return HYDRA_OK;
}

void spill_release_all(hydra_ctx* c) {
  if (c->copy_in) {
    (void)hipStreamSynchronize(c->copy_in);
    (void)hipStreamDestroy(c->copy_in);
  }
  if (c->copy_out) {
    (void)hipStreamSynchronize(c->copy_out);
    (void)hipStreamDestroy(c->copy_out);
  }
  for (auto& sl : c->slots)
    if (sl.free_ev) (void)hipEventDestroy(sl.free_ev);
  for (Model& m : c->models)
    for (Shard& sh : m.shards) {
      if (sh.loaded_ev) (void)hipEventDestroy(sh.loaded_ev);
      if (sh.updated_ev) (void)hipEventDestroy(sh.updated_ev);
      if (sh.stored_ev) (void)hipEventDestroy(sh.stored_ev);
    }
  for (void* p : c->host_allocs) (void)hipHostFree(p);
  c->host_allocs.clear();
}

}  // namespace hydra
