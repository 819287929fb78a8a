// Launchers of the device kernels.  Every launcher enqueues on the given stream and returns the
// HIP status of the launch; none allocates or synchronises.  Pointers are device pointers.
//
// "Grouped" launches run the same operation for G independent problems of identical shape, one
// per model, in a single grid: this is how ready shards of different models that share a shape
// fill the device together (paper, Approach: the unit of parallel work is the shard, and shards
// of different models are independent).  Results of a problem never depend on G or on its
// position in the group.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hydra {

constexpr int MAXG = 16;  // problems per grouped launch

typedef uint16_t bf16_t;  // storage type of bf16 values (top half of an fp32, round-to-nearest-even)

enum { EPI_ACT_NONE = 0, EPI_ACT_RELU = 1, EPI_ACT_GELU = 2 };
enum { GEMM_F32 = 0, GEMM_BF16 = 1 };

// C[M,N] = sum_k X(m,k) * W(n,k) followed by the epilogue
//   v = acc (+ bias[n]);  pre[m,n] = v (optional);
//   v = gate ? v * act'(gate[m,n]) : act(v);  v *= mul[m,n] (optional);  v += resid[m,n] (optional);
//   out[m,n] = v.
// x_kmajor: X stored [M, ldx] with k contiguous, else stored [K, ldx] with m contiguous.
// w_kmajor: W stored [N, ldw] with k contiguous, else stored [K, ldw] with n contiguous.
// Leading dimensions are in elements and must be multiples of 16 bytes worth of elements, and at
// least the contiguous extent rounded up to that; base pointers 16-byte aligned.
struct GemmArgs {
  int dtype;  // GEMM_F32: operands fp32; GEMM_BF16: operands bf16.  Accumulation is fp32.
  int M, N, K;
  int x_kmajor, w_kmajor;
  int ldx, ldw;
  int G;
  const void* X[MAXG];
  const void* W[MAXG];
  const float* bias[MAXG];  // fp32 [N] or null (all-or-none across the group)
  void* out[MAXG];          // [M, ldo], operand dtype, or fp32 when out_f32
  void* pre[MAXG];          // nullable, [M, ldo], operand dtype
  const void* gate[MAXG];   // nullable, [M, ldg], operand dtype
  const void* resid[MAXG];  // nullable, [M, ldr], operand dtype
  const void* mul[MAXG];    // nullable, [M, ldo], operand dtype: v *= mul[m,n] after the activation
  float* rowsum[MAXG];      // nullable, fp32 [M]: receives sum_k X(m,k) (x_kmajor = w_kmajor = 0 only): with X = dY
                            // of a Linear layer this is its bias gradient
  int ldo, ldg, ldr;
  int act;
  int out_f32;
  // Optional scratch for weight-gradient problems (x_kmajor = w_kmajor = 0, bf16) whose output has too few tiles to
  // fill the device: with ws non-null (all-or-none, 32-byte aligned, ws_bytes each) and gemm_split_k(M, N, K) = S > 1
  // the sum over k is cut into S contiguous ranges whose partial sums go to ws and are added in ascending order by a
  // second launch, which also applies the epilogue (plain store or update).  S depends on the shape alone, so a
  // result depends on neither the group nor the tile code; gemm_split_ws_bytes gives the bytes S needs.
  void* ws[MAXG];
  size_t ws_bytes;
  int split_k;  // set by the launcher
  int tile;  // 0 = choose by problem size; 1 = 256x256, 2 = 128x128, 3 = 32x128, 4 = 256x256 with operands staged
             // through registers even where the direct-to-LDS kernel applies (tests, tuning)
};
hipError_t launch_gemm(const GemmArgs& a, hipStream_t s);
int gemm_split_k(int M, int N, int K);              // 1 = no split
size_t gemm_split_ws_bytes(int M, int N, int K, int ldo);  // 0 when gemm_split_k is 1
// Must be called once per process before the first launch_gemm (sets the kernels' LDS limits).
hipError_t gemm_init();

// ---- elementwise / reductions (see each .hip file for definitions) ---------------------------------

struct PtrGroup {
  int G;
  void* p[MAXG];
};

// dst[i] = uniform on [-a, a): counter RNG keyed by key, index i.  a2 = 2a.
hipError_t launch_init_uniform(float* dst, size_t n, uint64_t key, float a, hipStream_t s);
hipError_t launch_fill_f32(float* dst, size_t n, float v, hipStream_t s);
hipError_t launch_fill_u32(uint32_t* dst, size_t n, uint32_t v, hipStream_t s);
// dst[i] = bf16(src[i]) for i < n
hipError_t launch_cast_bf16(const float* src, bf16_t* dst, size_t n, hipStream_t s);
// rows x cols (fp32, contiguous) -> rows x ld (fp32 or bf16), padding columns untouched
hipError_t launch_stage_rows(const float* src, void* dst, int rows, int cols, int ld, int to_bf16, hipStream_t s);

// Column sums: out_g[n] = sum_m src_g[m,n] for m < M (fp32 accumulation in a fixed order).
// part: scratch of colsum_part_floats(M, N) floats per problem (none needed for M <= 256).
struct ColsumArgs {
  int dtype, M, N, ld, G;
  const void* src[MAXG];
  float* out[MAXG];
  float* part[MAXG];
};
size_t colsum_part_floats(int M, int N);
hipError_t launch_colsum(const ColsumArgs& a, hipStream_t s);
// records the text hydra_ops_last_error() returns ("what" or "what: detail") and returns `status`
int ops_fail(int status, const char* what, const char* detail = nullptr);

// Softmax cross-entropy over rows of fp32 logits [M, ldz] with C classes:
//   rowloss[m] = logsumexp(z_m) - z_m[y_m];  dz[m,c] = (softmax(z_m)[c] - [c == y_m]) * inv_n
// then loss_out_g[0] = inv_n * sum_m rowloss[m] (fixed order).  dz has dtype `dtype`, leading dim lddz;
// padding columns [C, lddz) are written as zero.
struct SoftmaxCeArgs {
  int dtype, M, C, ldz, lddz, G;
  float inv_n;
  const float* logits[MAXG];
  const int32_t* labels;  // shared by the group, [M]
  void* dz[MAXG];
  float* rowloss[MAXG];   // scratch [M]
  float* loss_out[MAXG];  // one float each
};
hipError_t launch_softmax_ce(const SoftmaxCeArgs& a, hipStream_t s);

// Optimizer over flat fp32 blocks of n elements (n multiple of 4).
//   SGD:  p -= lr * g
//   Adam: m = b1 m + c1 g; v = b2 v + c2 g^2; p -= lr * (m*bc1) / (sqrt(v*bc2) + eps)
// with c = 1 - b and bc1 = 1/(1-b1^t), bc2 = 1/(1-b2^t) rounded from double by the host.  When w16 is
// non-null the bf16 working copy is refreshed: w16 = bf16(p).
// With chunks non-null only the listed pieces of the block are updated: chunk i covers elements
// [4*chunks[i].x, 4*(chunks[i].x + chunks[i].y)) with chunks[i].y <= 256 (a device array shared by the group).
struct OptimHp {
  float lr, b1, b2, c1, c2, eps, bc1, bc2;
};
struct OptimArgs {
  int opt, G;
  size_t n;
  float* p[MAXG];
  const float* g[MAXG];
  float* m[MAXG];
  float* v[MAXG];
  bf16_t* w16[MAXG];
  OptimHp hp[MAXG];
  const uint2* chunks;
  int n_chunks;
};
hipError_t launch_optim(const OptimArgs& a, hipStream_t s);

// Weight gradient with the update in its epilogue: acc = sum_k X(m,k) W(n,k) is the gradient of
// parameter element [m, n] (row pitch ldo), which the lane that holds it applies at once to p (and
// m, v, w16) exactly as launch_optim would; the gradient itself is stored only when a.out is non-null.
// Requires x_kmajor = w_kmajor = 0, out_f32, and no bias/pre/gate/resid/mul/activation.
struct GemmUpdate {
  int opt;
  float* p[MAXG];
  float* m[MAXG];
  float* v[MAXG];
  bf16_t* w16[MAXG];  // all-or-none across the group
  OptimHp hp[MAXG];
};
hipError_t launch_gemm_update(const GemmArgs& a, const GemmUpdate& u, hipStream_t s);

// ---- whole shard phases of small fp32 MLPs in one launch (mlp_fused.hip) --------------------------------------
// For models with at most 32 rows per step and layers at most 256 wide: the forward pass of a shard's units [u0, u1)
// is one launch (with the softmax cross-entropy when the shard ends the model), the backward pass two (the chain of
// input gradients, then every weight gradient of the shard together with the update of its weights and biases, or
// with keep_grads the stored gradients instead).  Unit u < L is Linear + activation, unit L the output Linear + loss.
constexpr int MLP_FUSED_MAX_UNITS = 16;
struct MlpTab {                      // device-resident table of one model's activation buffers (fp32)
  float* z[MLP_FUSED_MAX_UNITS];     // [B, ldd] pre-activations of the hidden units
  float* h[MLP_FUSED_MAX_UNITS];     // [B, ldd] activations
  float* dz[MLP_FUSED_MAX_UNITS];    // [B, ldd] gradients w.r.t. the pre-activations
  float* logits;                     // [B, ldv]
  float* dlogits;                    // [B, ldv]
  float* rowloss;                    // [B]
};
struct MlpFusedArgs {
  int G, B, d_in, d, n_out, L, u0, u1, act, opt, keep_grads;
  int ld_in, ldd, ldv;                          // row pitches of the batch, of z/h/dz, of logits/dlogits
  unsigned w_off[MLP_FUSED_MAX_UNITS];          // element offsets of W_u [out, in] and b_u in a model's parameter block
  unsigned b_off[MLP_FUSED_MAX_UNITS];
  float inv_n;                                  // 1 / B
  const int32_t* labels;                        // [B], shared by the group
  float* p[MAXG];                               // parameter blocks (and gradient / moment blocks laid out alike)
  float* g[MAXG];
  float* m[MAXG];
  float* v[MAXG];
  const MlpTab* tab[MAXG];                      // device pointers
  const float* x[MAXG];                         // [B, ld_in] rows of the step's batch
  float* loss[MAXG];                            // one float each: the step's loss
  OptimHp hp[MAXG];
};
bool mlp_fused_shape_ok(int B, int d_in, int d, int n_out, int n_units);
hipError_t mlp_fused_init();  // once per device before the first launch (raises the forward kernel's LDS limit)
hipError_t launch_mlp_fwd_fused(const MlpFusedArgs& a, hipStream_t s);
hipError_t launch_mlp_dgrad_chain(const MlpFusedArgs& a, hipStream_t s);   // no launch when the shard has no unit > 0
hipError_t launch_mlp_fwd_chain(const MlpFusedArgs& a, hipStream_t s);     // both of the above in one launch; units [0, L+1) only
hipError_t launch_mlp_wgrad_update(const MlpFusedArgs& a, hipStream_t s);

// ---- LayerNorm (layernorm.hip) --------------------------------------------------------------------------
// y = (x-mean)*rstd*gamma + beta over rows of width d (d % 8 == 0, d <= 4096); mean/rstd fp32 per row.
struct LnArgs {
  int dtype, rows, d, ld, G;
  float eps;
  const void* x[MAXG];
  void* y[MAXG];
  const float* gamma[MAXG];
  const float* beta[MAXG];
  float* mean[MAXG];
  float* rstd[MAXG];
};
hipError_t launch_ln_fwd(const LnArgs& a, hipStream_t s);
// dx = rstd*(g - mean(g) - xhat*mean(g*xhat)) + add (add optional), g = dy*gamma;
// dgamma = sum_rows dy*xhat, dbeta = sum_rows dy.  part: scratch of ln_bwd_blocks(rows, d)*2*d floats.
struct LnBwdArgs {
  int dtype, rows, d, ld, G;
  const void* x[MAXG];
  const void* dy[MAXG];
  const void* add[MAXG];
  void* dx[MAXG];
  const float* gamma[MAXG];
  const float* mean[MAXG];
  const float* rstd[MAXG];
  float* part[MAXG];
  float* dgamma[MAXG];
  float* dbeta[MAXG];
};
int ln_bwd_blocks(int rows, int d);
hipError_t launch_ln_bwd(const LnBwdArgs& a, hipStream_t s);
hipError_t ln_init();

// ---- embedding, row gather/scatter, gated feed-forward pieces (embedding.hip) -------------------------------
struct EmbedArgs {
  int dtype, tokens, S, d, ld, G;
  const int32_t* ids;  // [tokens], shared by the group
  const void* tok[MAXG];
  const void* pos[MAXG];
  void* x[MAXG];
};
hipError_t launch_embed_fwd(const EmbedArgs& a, hipStream_t s);
struct EmbedBwdArgs {
  int dtype, V, S, S_table, B, d, ld, G;
  const int32_t* row_ptr;    // [V+1] CSR over token ids of this batch
  const int32_t* positions;  // [B*S] token indices grouped by id, ascending inside a group
  const void* dx[MAXG];
  float* dtok[MAXG];  // [V, d]
  float* dpos[MAXG];  // [S_table, d]
};
hipError_t launch_embed_bwd(const EmbedBwdArgs& a, hipStream_t s);
struct RowsArgs {
  int dtype, n, d, ld_src, ld_dst, G;
  const int32_t* rows;  // [n], shared by the group
  const void* src[MAXG];
  void* dst[MAXG];
};
hipError_t launch_gather_rows(const RowsArgs& a, hipStream_t s);   // dst[r] = src[rows[r]]
hipError_t launch_scatter_rows(const RowsArgs& a, hipStream_t s);  // dst[rows[r]] = src[r]
struct GatedBwdArgs {
  int dtype, rows, ld, G;
  const void* dh[MAXG];
  const void* z1[MAXG];
  const void* zg[MAXG];
  void* dz1[MAXG];
  void* dzg[MAXG];
};
hipError_t launch_gated_bwd(const GatedBwdArgs& a, hipStream_t s);

// ---- attention (attention.hip), bf16 only, head width 64 or 128 ------------------------------------------
struct AttnArgs {
  int B, S, H, DH, ld_qkv, ld_o, causal, G;
  float scale;
  const bf16_t* qkv[MAXG];
  bf16_t* o[MAXG];
  float* lse[MAXG];  // [B*H*S]
};
hipError_t launch_attn_fwd(const AttnArgs& a, hipStream_t s);
struct AttnBwdArgs {
  int B, S, H, DH, ld_qkv, ld_o, causal, G;
  float scale;
  const bf16_t* qkv[MAXG];
  const bf16_t* o[MAXG];
  const bf16_t* dout[MAXG];
  const float* lse[MAXG];
  float* delta[MAXG];  // [B*H*S] scratch, written by the dq kernel and read by the dk/dv kernel
  bf16_t* dqkv[MAXG];
};
hipError_t launch_attn_bwd(const AttnBwdArgs& a, hipStream_t s);
hipError_t attn_init();

// all per-process kernel set-up (LDS limits); call once before the first launch
hipError_t kernels_init();

}  // namespace hydra
