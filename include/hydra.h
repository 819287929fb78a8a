/*
 * hydra.h -- C boundary of the shard-parallel multi-model trainer.
 *
 * Problem statement (paper, Introduction, "Model Selection Integration"; Approach): a user has K
 * configurations of one model family for the same task and wants all of them trained.  Each model
 * is cut into shards (contiguous layer ranges; Introduction, second paragraph, and Figure 1), and
 * forward, backward and update work of shards belonging to different models is interleaved so the
 * device does not idle on one model's layer-to-layer dependency (Approach, first paragraph).  The
 * result must equal unsharded training of every model (Approach, "Desiderata", third item).
 *
 * General conventions
 *  - Every call returns a hydra_status; nothing throws or aborts across this boundary.  On error
 *    the out-parameters are left untouched and hydra_last_error() describes the failure.
 *  - All pointers in these signatures are HOST pointers unless a comment says "device".  The caller
 *    owns every buffer it passes in or receives into; the library copies in and out.
 *  - The context owns all device memory and pinned host memory it allocates and releases them in
 *    hydra_destroy().  A context is not thread-safe.
 *  - Call order: create -> define_models -> shard -> set_data -> train_epoch* -> read_*.
 *    A call made out of order returns HYDRA_ERR_BAD_STATE.
 *  - Layer units.  MLP with L hidden layers: units 0..L-1 are Linear+activation, unit L is the
 *    output Linear with the softmax cross-entropy loss (L+1 units).  Transformer with L blocks:
 *    unit i is block i; unit 0 also embeds the tokens; unit L-1 also holds the final LayerNorm,
 *    the output Linear (applied to target rows only) and the loss (L units).
 *  - Canonical tensor order of one model (all stored row-major, matrices as [out, in]):
 *      MLP:         W_0, b_0, ..., W_{L-1}, b_{L-1}, W_out, b_out
 *      Transformer: tok_emb[V,d], pos_emb[S,d],
 *                   per block: ln1.g, ln1.b, Wqkv[3d,d], bqkv, Wo[d,d], bo, ln2.g, ln2.b,
 *                              W1[F,d], b1, (Wg[F,d], bg if gated,) W2[d,F], b2,
 *                   lnf.g, lnf.b, Whead[V,d], bhead
 *    Rows [0,d) of Wqkv produce queries, [d,2d) keys, [2d,3d) values; head h owns columns
 *    [h*dh,(h+1)*dh) of each.
 */
#ifndef HYDRA_H
#define HYDRA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct hydra_ctx hydra_ctx; /* opaque, owned by the library */

typedef enum {
  HYDRA_OK = 0,
  HYDRA_ERR_INVALID_ARG = 1,
  HYDRA_ERR_BAD_STATE = 2,
  HYDRA_ERR_BAD_SCHEDULE = 3,
  HYDRA_ERR_OOM_DEVICE = 4,
  HYDRA_ERR_OOM_HOST = 5,
  HYDRA_ERR_DEVICE = 6,
  HYDRA_ERR_UNSUPPORTED = 7,
  HYDRA_ERR_BUFFER_TOO_SMALL = 8
} hydra_status;

enum { HYDRA_KIND_MLP = 0, HYDRA_KIND_ENCODER = 1, HYDRA_KIND_DECODER = 2 };
enum { HYDRA_ACT_RELU = 0, HYDRA_ACT_GELU = 1 };
enum { HYDRA_DTYPE_F32 = 0,          /* fp32 weights, activations and arithmetic                    */
       HYDRA_DTYPE_BF16 = 1 };       /* bf16 working weights/activations, fp32 master + optimizer   */
enum { HYDRA_OPT_SGD = 0, HYDRA_OPT_ADAM = 1 };
enum { HYDRA_PHASE_F = 0, HYDRA_PHASE_B = 1, HYDRA_PHASE_U = 2 };
enum { HYDRA_SCHED_SEQUENTIAL = 0,   /* model-major, one shard task at a time, one stream, ungrouped
                                        launches: traditional model parallelism, the paper's
                                        comparison point (Introduction, "Motivation")                */
       HYDRA_SCHED_SHARD_PARALLEL = 1,/* every ready shard task is issued; same-shaped tasks of
                                        different models share one grouped launch, the rest spread
                                        over streams (Approach, first paragraph)                     */
       HYDRA_SCHED_EXPLICIT = 2,     /* caller-given order for one step, replayed every step        */
       HYDRA_SCHED_TASK_PARALLEL = 3 };/* every model is one task of its own (paper, Introduction,
                                        "Motivation": task parallelism): its shard tasks run in model
                                        order on the model's stream (model k on stream k mod n_streams),
                                        nothing is grouped across models                             */

/* Memory and streams come from the caller (PyTorch in the Python binding).  Every field may be
 * zero/NULL: the library then uses hipMalloc/hipFree and creates its own streams. */
typedef struct {
  void* (*dev_alloc)(size_t bytes, void* user); /* returns a DEVICE pointer, 256-byte aligned, or NULL */
  void (*dev_free)(void* dev_ptr, void* user);
  void* user;
  void* const* streams;        /* n_streams hipStream_t handles, default priority, owned by caller   */
  int n_streams;
  size_t device_budget_bytes;  /* 0 = unlimited.  Upper bound on device bytes held by parameters and
                                  optimizer state; smaller than the total forces inactive shards to
                                  be spilled to pinned host memory                                   */
  size_t host_budget_bytes;    /* 0 = unlimited.  Upper bound on pinned host bytes used for spill    */
  int dry_run;                 /* 1: plan only.  No device is touched; define/shard/set_data record
                                  shapes, train_epoch validates the schedule and fills the stats     */
  int keep_grads;              /* 0: the update of a weight matrix runs inside the kernel that produces
                                  its gradient and that gradient is never stored (hydra_read_grads
                                  is then refused); 1: every gradient is stored and the update task
                                  applies all of them.  Both give the same parameters bit for bit.
                                  Spilled state always keeps gradients                               */
  size_t activation_budget_bytes; /* 0 = every activation a backward pass needs is kept from the forward
                                  pass.  Otherwise an upper bound on the device bytes of per-block
                                  activations and backward scratch (Transformer models): when keeping
                                  everything would exceed it, a forward task keeps only the shard's
                                  input and output, the per-block buffers come from a pool of shard-sized
                                  workspaces that fit the bound, and a backward task first runs the
                                  shard's forward again.  The arithmetic, and hence every bit of the
                                  result, is unchanged.  With a bound set, shard before hydra_set_data  */
  int max_group;               /* largest number of same-shaped shard tasks of different models that share one
                                  grouped launch under the shard-parallel and explicit schedules: 0 = as many
                                  as are ready (at most 16), 1..16 = that many; the ready tasks beyond a group
                                  go to the next compute stream.  Results do not depend on it.  Automatic:
                                  the ready tasks of one shape are split into as many groups as there are
                                  compute streams while every group still holds at least 384 tiles of 256 x 256
                                  outputs of the shard's smallest matrix product (one and a half passes over the
                                  256 compute units): below that a launch would leave units idle, which is what
                                  grouping across models is for; above it, groups side by side on two streams let
                                  one group's output stores overlap the other's products                  */
  int auto_budget;             /* 1: the library chooses the two budgets above itself, from the memory the device
                                  has (the scheduler the paper leaves as its next step is to automate sharding and
                                  training; Evaluation, "Execution Plan").  State stays resident while parameters,
                                  gradients and optimizer state of all models take at most 85 % of the capacity;
                                  otherwise device_budget_bytes = 55 % of it (bf16 models trained with Adam).
                                  Activations are kept while they fit 90 % of what is then left, otherwise
                                  activation_budget_bytes = that amount and backward tasks recompute.  A budget
                                  the caller gives (non-zero) is kept.  Results do not depend on any of this  */
  size_t device_capacity_bytes;/* with auto_budget: the memory to plan for; 0 = the free device memory reported by
                                  the runtime when the models are defined (a dry run needs a value)          */
} hydra_options;

typedef struct {
  int kind;      /* HYDRA_KIND_*                                                                    */
  int n_layers;  /* hidden Linear layers (MLP) or blocks (Transformer)                              */
  int d_in;      /* MLP input width (ignored for Transformers)                                      */
  int d_model;   /* hidden width                                                                    */
  int n_heads;   /* Transformer only; must divide d_model                                           */
  int d_ffn;     /* Transformer only                                                                */
  int n_out;     /* classes (MLP) or vocabulary size (Transformer)                                  */
  int max_seq;   /* Transformer only: rows of the position table                                    */
  int act;       /* HYDRA_ACT_* of the MLP hidden layers (Transformers always use GeLU)             */
  int ffn_gated; /* Transformer: 1 = W2( GeLU(Wg f + bg) * (W1 f + b1) ), 0 = W2 GeLU(W1 f + b1)    */
  int causal;    /* Transformer: 1 = scores above the diagonal are masked out                       */
  int dtype;     /* HYDRA_DTYPE_*                                                                   */
} hydra_arch;

typedef struct {
  int opt;                        /* HYDRA_OPT_*                                                    */
  double lr, beta1, beta2, eps;   /* Adam: bias-corrected, eps added outside the square root        */
  int warmup_steps;               /* lr_t = lr*min(1, t/warmup) for t = 1,2,... when > 0            */
} hydra_hparams;

typedef struct {
  int policy;                     /* HYDRA_SCHED_*                                                  */
  const int32_t* tasks;           /* EXPLICIT: n_tasks (model, shard, phase) triples for one step   */
  int n_tasks;
} hydra_schedule;

typedef struct {
  double wall_ms;                 /* host clock around the epoch, device drained at both ends       */
  uint64_t h2d_bytes, d2h_bytes;  /* spill traffic of the epoch                                     */
  uint64_t launches;              /* kernel launches issued                                         */
  uint64_t grouped_tasks;         /* shard tasks that ran inside a launch group of size > 1         */
  uint64_t peak_dev_bytes, peak_host_bytes;
  int32_t steps;                  /* steps run by this epoch                                        */
} hydra_epoch_stats;

hydra_status hydra_create(const hydra_options* opts /* nullable */, hydra_ctx** out);
hydra_status hydra_destroy(hydra_ctx* ctx);

/* Registers K models (paper, "Model Selection Integration": many hyper-parameter configurations of
 * one task).  archs has 1 entry (shared by all K) or K entries (same family, e.g. differing depth);
 * grid has K entries.  Parameters are initialised on the device from `seed` with a counter-based
 * generator keyed by (seed, model, tensor): MLP matrices U(-a,a) with a = sqrt(6/fan_in),
 * Transformer matrices and embeddings U(-a,a) with a = 0.02*sqrt(3), biases 0, LayerNorm gain 1. */
hydra_status hydra_define_models(hydra_ctx* ctx, int K, const hydra_arch* archs, int n_archs,
                                 const hydra_hparams* grid, uint64_t seed);

/* Cuts model `model` (or every model when model = -1) into n_cuts+1 shards: cuts are strictly
 * increasing interior layer-unit indices (paper, Introduction: a shard is a contiguous piece of the
 * model; Figure 1).  n_cuts = 0 keeps the model whole.  Calling it again re-cuts. */
hydra_status hydra_shard(hydra_ctx* ctx, int model, const int32_t* cuts, int n_cuts);

/* Automatic sharder (the step the paper names as next, Evaluation, "Execution Plan": choosing the partition instead of taking it
 * from the caller).  Cuts model `model` (-1: every model) into the fewest shards whose parameter, gradient and
 * optimizer-state bytes each stay within max_shard_bytes and, among the partitions with that many shards, one
 * that minimises the largest shard (contiguous partition of the layer units by dynamic programming).  With
 * max_shard_bytes = 0 the model is cut into exactly n_shards balanced shards (n_shards >= 1, at most the number
 * of layer units); otherwise n_shards is a lower bound (0 = none).  The cuts are applied as by hydra_shard and,
 * for model >= 0, written to cuts_out (cap entries; n_cuts receives the count; both may be NULL).
 * HYDRA_ERR_INVALID_ARG when one layer unit alone exceeds max_shard_bytes. */
hydra_status hydra_auto_shard(hydra_ctx* ctx, int model, size_t max_shard_bytes, int n_shards, int32_t* cuts_out,
                              int cap, int* n_cuts);

/* Model selection (paper, Introduction, "Model Selection Integration"): a model marked inactive is left out of
 * the following epochs (its tasks are not scheduled, its state stays where it is and can still be read); the
 * other models' results do not change by a bit.  Every model starts active.  An EXPLICIT schedule lists the
 * tasks of the active models only. */
hydra_status hydra_set_active(hydra_ctx* ctx, int model, int active);

/* The training data, shared by all models, copied to the device.
 *  MLP:         inputs fp32 [n_batches, B, d_in]; targets int32 [n_batches, B]; target_pos NULL;
 *               S_or_d = d_in; P = 0.
 *  Transformer: inputs int32 [n_batches, B, S] token ids; target_pos int32 [n_batches, B, P]
 *               ascending positions per sequence; targets int32 [n_batches, B, P]; S_or_d = S. */
hydra_status hydra_set_data(hydra_ctx* ctx, const void* inputs, const int32_t* target_pos,
                            const int32_t* targets, int n_batches, int B, int S_or_d, int P);

/* One pass over the n_batches batches: step t uses batch (t-1) mod n_batches, every model runs
 * forward, backward and update on it, in the order the schedule allows (dependencies: a shard's
 * forward needs the previous shard's forward and its own previous update; its backward needs the
 * next shard's backward, the last shard's its own forward; its update needs its backward).
 * An EXPLICIT order that violates them returns HYDRA_ERR_BAD_SCHEDULE before anything runs.
 * Returns after the device has drained.  stats may be NULL. */
hydra_status hydra_train_epoch(hydra_ctx* ctx, const hydra_schedule* schedule, hydra_epoch_stats* stats);

/* Copies fp32 master parameters of one model to dst.  tensor = -1: all tensors concatenated in
 * canonical order; otherwise that tensor.  cap and *n_written count floats; if cap is too small
 * returns HYDRA_ERR_BUFFER_TOO_SMALL with *n_written = required count. */
hydra_status hydra_read_params(hydra_ctx* ctx, int model, int tensor, float* dst, size_t cap, size_t* n_written);

/* Per-step losses of one model so far (the loss before that step's update), oldest first. */
hydra_status hydra_read_loss(hydra_ctx* ctx, int model, float* dst, size_t cap, size_t* n_written);

/* Test/debug helpers under the same conventions.  read_grads returns the gradients of the most
 * recent backward pass; write_params overwrites master (and working) weights of one tensor or all. */
hydra_status hydra_read_grads(hydra_ctx* ctx, int model, int tensor, float* dst, size_t cap, size_t* n_written);
hydra_status hydra_write_params(hydra_ctx* ctx, int model, int tensor, const float* src, size_t n);

/* Checkpoint and resume.  A model's training state is its parameters (hydra_read_params / hydra_write_params), the
 * optimizer's moments and the number of steps taken (which sets Adam's bias corrections and the warm-up).  read copies
 * the first moments of all tensors in canonical order to m_dst and the second moments to v_dst (cap floats each;
 * too small: HYDRA_ERR_BUFFER_TOO_SMALL with *n_written = the count per array; SGD models have no moments and report
 * 0) and the step count to *steps.  write restores them (n floats each, the count read reports) into a context whose
 * models were defined with the same architectures.  Training on from restored state gives the bits uninterrupted
 * training gives (paper, Approach, "Desiderata", third item, extended over a restart). */
hydra_status hydra_read_optimizer_state(hydra_ctx* ctx, int model, float* m_dst, float* v_dst, size_t cap, size_t* n_written,
                                        int64_t* steps);
hydra_status hydra_write_optimizer_state(hydra_ctx* ctx, int model, const float* m_src, const float* v_src, size_t n,
                                         int64_t steps);

/* Shape queries: number of tensors of a model; elements, rows and columns of one tensor;
 * number of shards of a model. */
hydra_status hydra_tensor_count(hydra_ctx* ctx, int model, int* n_tensors);
hydra_status hydra_tensor_shape(hydra_ctx* ctx, int model, int tensor, int* rows, int* cols);
hydra_status hydra_shard_count(hydra_ctx* ctx, int model, int* n_shards);

/* Measurement aid.  While enabled, every kernel launch of hydra_train_epoch is bracketed by a pair of
 * HIP events recorded on the stream the kernel is launched on; after the epoch the elapsed times are
 * summed per kernel class together with the algorithmic work of those launches (GEMMs: 2*M*N*K flops
 * per problem; optimizer: bytes read + written per parameter).  Sums accumulate until read with
 * reset = 1.  Disabled by default. */
enum { HYDRA_K_GEMM_FWD = 0, HYDRA_K_GEMM_DGRAD = 1, HYDRA_K_GEMM_WGRAD = 2, HYDRA_K_OPTIM = 3,
       HYDRA_K_SOFTMAX_CE = 4, HYDRA_K_COLSUM = 5, HYDRA_K_LAYERNORM = 6, HYDRA_K_ATTENTION = 7,
       HYDRA_K_EMBED = 8, HYDRA_K_ELEMENTWISE = 9,
       HYDRA_K_WGRAD_UPDATE = 10, /* weight-gradient GEMM with the parameter update in its epilogue */
       HYDRA_K_COPY_H2D = 11,     /* spilled state copied in from pinned host memory (not a kernel: bytes only) */
       HYDRA_K_COPY_D2H = 12,     /* ... and copied back out after the update                                   */
       HYDRA_K_COUNT = 13 };
typedef struct {
  uint64_t launches;
  double total_ms;   /* sum of event-pair times                                                     */
  double flops;      /* algorithmic floating-point operations of those launches                     */
  double bytes;      /* algorithmic bytes of those launches                                         */
} hydra_kernel_profile;
hydra_status hydra_profile_enable(hydra_ctx* ctx, int on);
hydra_status hydra_profile_read(hydra_ctx* ctx, int kernel_class, int reset, hydra_kernel_profile* out);
/* Device-busy time of the profiled epochs (paper, Approach, "Desiderata", first item: the device is to be kept
 * utilised throughout): busy_ms = length of the union of all launches' [start, end] intervals (launches on different
 * streams overlap, so this is at most the wall time, unlike the sum of the durations), span_ms = first start to last
 * end, summed over the epochs.  Accumulates until read with reset = 1. */
hydra_status hydra_profile_busy(hydra_ctx* ctx, int reset, double* busy_ms, double* span_ms);
/* Spill copies of the profiled epochs against the kernels (paper, Approach: work of other shards hides the wait for
 * one shard's data): copy_ms = length of the union of the copy intervals of both directions, overlapped_ms = the part
 * of it during which at least one kernel was running.  Both 0 when nothing is spilled.  Accumulates until read with
 * reset = 1. */
hydra_status hydra_profile_copy_overlap(hydra_ctx* ctx, int reset, double* copy_ms, double* overlapped_ms);

/* Library-owned string, valid until the next call on ctx (ctx may be NULL: last create error). */
const char* hydra_last_error(const hydra_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* HYDRA_H */
