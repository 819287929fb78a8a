// Host-side structures of the shard-parallel trainer (not part of the C boundary).
#pragma once
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <map>
#include <string>
#include <utility>
#include <vector>

#include "../../include/hydra.h"
#include "kernels.h"

namespace hydra {

enum { INIT_ZERO = 0, INIT_ONE = 1, INIT_UNIFORM = 2 };

struct Tensor {
  std::string name;
  int rows = 0, cols = 0;  // vectors: rows = 1
  size_t n = 0;            // rows * cols
  int init = INIT_ZERO;
  float a = 0.f;           // bound of the uniform init
  int unit = 0;            // layer unit that owns it
  size_t off = 0;          // element offset inside the model's parameter block (64-element aligned)
  bool fused = false;      // a matrix whose gradient one GEMM produces: its update can run in that GEMM's epilogue
};

// A shard: layer units [u0, u1) of one model (paper, Introduction: a contiguous piece of the model)
// with the parameters, gradients and optimizer state of those units.  Tensors of a shard are a
// contiguous range of the model's canonical order, so its state is one contiguous block.
struct Shard {
  int u0 = 0, u1 = 0;
  int t0 = 0, t1 = 0;      // tensor range [t0, t1)
  size_t off = 0, n = 0;   // element range inside the model block (n is a multiple of 64)
  uint64_t sig = 0;        // shape signature: shards with equal signatures can share a grouped launch
  // device pointers of the shard's state (null while spilled)
  float *p = nullptr, *m = nullptr, *v = nullptr, *g = nullptr;
  bf16_t* w16 = nullptr;
  // spill mode: slot held between the shard's backward and the end of its update, and the events that order it
  int slot = -1;
  hipEvent_t loaded_ev = nullptr, updated_ev = nullptr;
  hipEvent_t stored_ev = nullptr;  // the shard's state has been copied back to host memory after its last update
  // fused-update mode: the pieces of the block that the update task still owns (tensors that are not `fused`),
  // as a device table of (first 16-byte vector, vectors <= 256) pairs relative to the shard's block
  uint2* tail_chunks = nullptr;
  int n_tail_chunks = 0;
  size_t n_tail = 0;  // elements covered by the table
};

struct MlpActs {                // per model, allocated by set_data
  std::vector<void*> z, h, dz;  // per hidden unit: pre-activation, activation, gradient w.r.t. z  [B, ldd]
  float* logits = nullptr;      // [B, ldv] fp32
  void* dlogits = nullptr;      // [B, ldv] operand dtype
  float* rowloss = nullptr;     // [B]
  MlpTab* tab = nullptr;        // device copy of the pointers above for the kernels that run whole shard phases
};

// Transformer activations of one model (bf16), allocated by set_data.  Tk = B*S tokens, NT = B*P targets.
struct TrBlockActs {
  void *a = nullptr, *qkv = nullptr, *o = nullptr, *x1 = nullptr, *f = nullptr;  // [Tk,d], [Tk,3d], [Tk,d] x3
  void *z1 = nullptr, *zg = nullptr, *hmid = nullptr;                            // [Tk,F]
  float *mu1 = nullptr, *rs1 = nullptr, *mu2 = nullptr, *rs2 = nullptr;          // [Tk]
  float* lse = nullptr;                                                          // [B*H*S]
};
struct TrActs {
  std::vector<void*> x;    // [L+1]: x[l] = input of block l, x[L] = output of the last block; [Tk,d]
  std::vector<void*> dx;   // [L+1]: gradient w.r.t. x[l]
  std::vector<TrBlockActs> blk;
  void *xf = nullptr, *xt = nullptr, *dlogits = nullptr, *dxt = nullptr, *dxf = nullptr;
  float *logits = nullptr, *rowloss = nullptr, *muf = nullptr, *rsf = nullptr;
  // backward scratch shared by the blocks of the model
  void *dhm = nullptr, *dz1 = nullptr, *dzg = nullptr, *df = nullptr, *dx1 = nullptr, *dob = nullptr,
       *dqkv = nullptr, *da = nullptr;
  float *delta = nullptr, *lnpart = nullptr;
  void* splitk = nullptr;   // partial sums of weight gradients whose sum over the tokens is split (gemm_split_k)
  size_t splitk_bytes = 0;
};

// Recomputation mode: the per-block activations and the backward scratch of one shard task.  A pool of these
// replaces the per-model buffers; a task uses the workspace of (its stream, its position in the launch group).
struct TrWorkspace {
  std::vector<TrBlockActs> blk;  // one per unit of the largest shard
  std::vector<void*> xi, dxi;    // block inputs / their gradients strictly inside a shard
  TrActs sc;                     // head buffers and backward scratch (x, dx, blk unused)
};

// A model-sized fp32 array in pinned host memory, held as chunks of at most CHUNK elements (one pinned allocation
// each: very large single pinned allocations are refused by the runtime).
struct HostBlock {
  static constexpr size_t CHUNK = (size_t)512 << 20;  // elements per chunk (2 GiB)
  std::vector<float*> chunk;
  size_t n = 0;
  // calls f(host pointer, offset into the range, elements) for every piece of elements [off, off+cnt)
  template <class F>
  void pieces(size_t off, size_t cnt, F f) const {
    size_t done = 0;
    while (done < cnt) {
      const size_t at = off + done, ci = at / CHUNK, in = at % CHUNK, take = std::min(cnt - done, CHUNK - in);
      f(chunk[ci] + in, done, take);
      done += take;
    }
  }
};

struct Model {
  hydra_arch arch{};
  hydra_hparams hp{};
  std::vector<Tensor> tensors;
  size_t n_block = 0;           // padded elements of the whole parameter block
  std::vector<Shard> shards;
  int n_units = 0;
  // whole-model state blocks (resident mode): shards point into these
  float *p = nullptr, *m = nullptr, *v = nullptr, *g = nullptr;
  bf16_t* w16 = nullptr;
  MlpActs mlp;
  TrActs tr;
  // spill mode: resident fp32 copy of the vector tensors (offset per tensor, -1 for matrices) and the pinned
  // host home of master weights and Adam moments
  float* pv = nullptr;
  std::vector<long> voff;
  size_t n_vec = 0;
  HostBlock host_p, host_m, host_v;
  float* loss_dev = nullptr;    // one float per step of the current epoch
  int loss_cap = 0;
  std::vector<float> losses;    // all steps so far (host)
  long t = 0;                   // optimizer steps taken
  bool active = true;           // inactive models are left out of the epochs that follow (model selection)
};

struct Task {
  int k, s, ph;
  bool operator<(const Task& o) const { return k != o.k ? k < o.k : (s != o.s ? s < o.s : ph < o.ph); }
  bool operator==(const Task& o) const { return k == o.k && s == o.s && ph == o.ph; }
};

// A launch group: same phase, same shard signature, different models.
struct Bucket {
  int ph = 0;
  std::vector<std::pair<int, int>> members;  // (model, shard)
  int stream = 0;
  // A launch group may cover `span` consecutive shard tasks of each member: shards second, second+1, ... for a forward
  // group, second, second-1, ... for a backward group (the order the tasks run in).  Only where one launch can take
  // several shards (the small-MLP kernels): the tasks' dependencies and completion are those of all of them together.
  int span = 1;
  int shard_at(size_t member, int j) const { return ph == 1 ? members[member].second - j : members[member].second + j; }
  // A forward group that spans all of its members' shards may also take the backward tasks that the plan runs right
  // behind it (shards second + span - 1, second + span - 2, ...: `bspan` of them, all or none): the small-MLP kernels
  // go from the loss straight into the chain of input gradients.
  int bspan = 0;
  int back_shard_at(size_t member, int j) const { return members[member].second + span - 1 - j; }
  // every (model, shard, phase) task the group covers, in the order they run
  template <typename F>
  void for_each_task(F&& f) const {
    for (size_t mi = 0; mi < members.size(); ++mi) {
      for (int j = 0; j < span; ++j) f(members[mi].first, shard_at(mi, j), ph);
      for (int j = 0; j < bspan; ++j) f(members[mi].first, back_shard_at(mi, j), 1);
    }
  }
};

enum State { ST_CREATED = 0, ST_DEFINED = 1, ST_SHARDED = 2, ST_DATA = 3 };

}  // namespace hydra

struct hydra_ctx {
  hydra_options opt{};
  bool dry = false;
  int state = hydra::ST_CREATED;
  std::string err;
  int K = 0;
  uint64_t seed = 0;
  std::vector<hydra::Model> models;
  // data (device)
  int n_batches = 0, B = 0, S = 0, P = 0, ld_in = 0;
  size_t x_bytes = 0, ids_bytes = 0, tp_bytes = 0, tg_bytes = 0;
  void* x_staged = nullptr;      // MLP: [n_batches, B, ld_in] operand dtype
  int32_t* ids = nullptr;        // Transformer: [n_batches, B, S]
  int32_t* tgt_pos = nullptr;    // Transformer: [n_batches, B*P] row index (b*S + position) of every target
  int32_t* csr_ptr = nullptr;    // Transformer: [n_batches, V+1] CSR over token ids of each batch
  int32_t* csr_pos = nullptr;    // Transformer: [n_batches, B*S] token indices grouped by id
  size_t csr_ptr_bytes = 0, csr_pos_bytes = 0;
  int32_t* targets = nullptr;    // [n_batches, B] or [n_batches, B, P]
  bool acts_ready = false;
  // activation_budget_bytes forces recomputation: workspaces [stream][member], ws_streams * ws_group of them
  bool recompute = false;
  std::vector<hydra::TrWorkspace> ws;
  int ws_streams = 0, ws_group = 0;
  // streams / events
  std::vector<hipStream_t> streams;
  bool own_streams = false;
  std::vector<hipEvent_t> events;
  // allocations
  std::vector<void*> dev_allocs;
  size_t dev_bytes = 0, peak_dev_bytes = 0;
  size_t capacity = 0;  // auto_budget: the device memory the budgets are planned for
  // spill mode (state does not fit device_budget_bytes)
  // weight updates run in the epilogue of the weight-gradient GEMM (resident state, gradients not kept)
  bool fuse = false;
  bool spill = false, sync_spill = false;
  struct Slot { float* base = nullptr; hipEvent_t free_ev = nullptr; bool used = false, held = false; };
  std::vector<Slot> slots;
  size_t slot_elems = 0, next_slot = 0;
  size_t state_bytes = 0;  // resident parameter bytes (working weights, vectors) counted against the budget
  hipStream_t copy_in = nullptr, copy_out = nullptr;
  std::vector<void*> host_allocs;
  size_t host_bytes = 0, peak_host_bytes = 0;
  // accounting of the running epoch
  uint64_t launches = 0, grouped_tasks = 0, h2d_bytes = 0, d2h_bytes = 0;
  // optional per-launch timing (hydra_profile_enable): event pairs on the launching stream
  bool profiling = false;
  // cls2 >= 0: the launch also does flops2 of work of a second class; its time is split in proportion to the flops
  struct ProfRec { int cls; hipEvent_t a, b; double flops, bytes; int cls2; double flops2; };
  std::vector<ProfRec> prof_recs;
  std::vector<hipEvent_t> prof_pool;
  size_t prof_used = 0;
  struct ProfSum { uint64_t launches = 0; double ms = 0, flops = 0, bytes = 0; };
  ProfSum prof_sum[HYDRA_K_COUNT];
  hipEvent_t prof_origin = nullptr;   // recorded when a profiled epoch starts, after the streams have drained
  double prof_busy_ms = 0, prof_span_ms = 0;
  double prof_copy_ms = 0, prof_copy_overlapped_ms = 0;  // union of the spill copies' intervals / its part under kernels  // union of the launches' [start, end] intervals / first start to last end

  hydra_status fail(hydra_status st, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    err = buf;
    return st;
  }
};

namespace hydra {

// models.cpp
hydra_status build_tensors(hydra_ctx* c, Model& m);
hydra_status cut_model(hydra_ctx* c, Model& m, const int32_t* cuts, int n_cuts);
hydra_status alloc_models(hydra_ctx* c);
hydra_status alloc_activations(hydra_ctx* c);
hydra_status build_update_chunks(hydra_ctx* c);  // fused-update mode: the per-shard tables of what the update task owns
void* ctx_alloc(hydra_ctx* c, size_t bytes);  // nullptr on failure (or in dry-run, where only bytes are counted)
void ctx_free(hydra_ctx* c, void* p, size_t bytes);
void ctx_free_all(hydra_ctx* c);

// spill.cpp
size_t resident_state_bytes(const hydra_ctx* c);
hydra_status spill_alloc_models(hydra_ctx* c);
hydra_status spill_prepare(hydra_ctx* c);
int spill_max_group(const hydra_ctx* c);
hydra_status spill_acquire(hydra_ctx* c, int k, int s, hipStream_t compute, bool synchronous);
hydra_status spill_before_update(hydra_ctx* c, int k, int s, hipStream_t compute);
hydra_status spill_after_update(hydra_ctx* c, int k, int s, hipStream_t compute, bool synchronous);
void spill_release_all(hydra_ctx* c);
uint64_t tensor_key(uint64_t seed, int model, int tensor);  // models.cpp: key of the init stream of a tensor

// scheduler.cpp
hydra_status build_plan(hydra_ctx* c, const hydra_schedule* sch, std::vector<Bucket>& plan);
hydra_status run_epoch(hydra_ctx* c, const std::vector<Bucket>& plan, hydra_epoch_stats* stats);

// exec_mlp.cpp / exec_transformer.cpp: run one launch group (forward, backward or update of its shards)
hydra_status mlp_run(hydra_ctx* c, const Bucket& b, int batch, int step_in_epoch, hipStream_t s);
hydra_status tr_run(hydra_ctx* c, const Bucket& b, int batch, int step_in_epoch, hipStream_t s);
hydra_status fill_optim(hydra_ctx* c, const Bucket& b, int step, OptimArgs& o);
OptimHp step_hparams(const Model& m, int step_in_epoch);  // fp32 hyper-parameters of optimizer step m.t + step_in_epoch + 1
bool mlp_runs_fused(const hydra_ctx* c, const Model& m);  // small fp32 MLP: whole shard phases in one launch each
// runs the update task of a launch group: the whole block, or only what the fused epilogues leave
hydra_status run_update(hydra_ctx* c, const Bucket& b, int step, hipStream_t s);
inline hydra_status run_bucket(hydra_ctx* c, const Bucket& b, int batch, int step, hipStream_t s) {
  return c->models[0].arch.kind == HYDRA_KIND_MLP ? mlp_run(c, b, batch, step, s) : tr_run(c, b, batch, step, s);
}

#define HYDRA_HIP(c, expr)                                                                              \
  do {                                                                                                  \
    hipError_t e_ = (expr);                                                                             \
    if (e_ != hipSuccess) return (c)->fail(HYDRA_ERR_DEVICE, "%s: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

// algorithmic HBM bytes per parameter of an update applied in a gradient GEMM's epilogue: the state is read and
// written once (p, and m, v for Adam), the working copy written, the gradient never stored
inline double fused_update_bytes(int opt, bool bf16) { return (opt == 1 ? 24.0 : 8.0) + (bf16 ? 2.0 : 0.0); }

// profile.cpp: event pair around one launch when profiling is on
hipError_t prof_epoch_begin(hydra_ctx* c);  // records the time origin of a profiled epoch on stream 0
hipError_t prof_begin(hydra_ctx* c, hipStream_t s, hipEvent_t* a);
hipError_t prof_end(hydra_ctx* c, hipStream_t s, hipEvent_t a, int cls, double flops, double bytes, int cls2 = -1,
                    double flops2 = 0.0);
hydra_status prof_collect(hydra_ctx* c);  // after the streams have drained

// a kernel launch of class `cls` on stream `s` doing `flops` / moving `bytes` of algorithmic work:
// counted always, executed unless the context is a dry run, timed when profiling is on
#define HYDRA_LAUNCH(c, cls, s, flops, bytes, expr) HYDRA_LAUNCH2(c, cls, -1, s, flops, 0.0, bytes, expr)
// ... of two classes (one kernel that does, say, a forward and an input-gradient pass)
#define HYDRA_LAUNCH2(c, cls, cls2, s, flops, flops2, bytes, expr)                                      \
  do {                                                                                                  \
    ++(c)->launches;                                                                                    \
    if (!(c)->dry) {                                                                                    \
      hipEvent_t pa_ = nullptr;                                                                         \
      hipError_t e_ = (c)->profiling ? prof_begin(c, s, &pa_) : hipSuccess;                             \
      if (e_ == hipSuccess) e_ = (expr);                                                                \
      if (e_ == hipSuccess && (c)->profiling) e_ = prof_end(c, s, pa_, cls, flops, bytes, cls2, flops2); \
      if (e_ != hipSuccess) return (c)->fail(HYDRA_ERR_DEVICE, "%s: %s", #expr, hipGetErrorString(e_)); \
    }                                                                                                   \
  } while (0)

}  // namespace hydra
