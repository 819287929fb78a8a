/*
 * hydra_ops.h -- C entry points of the individual device operations the trainer is built from.
 *
 * They exist so that every kernel can be checked and timed on its own.  All data pointers are
 * DEVICE pointers owned by the caller; the pointer tables themselves (X, W, ...) are HOST arrays of
 * G entries.  `stream` is a hipStream_t (NULL = the default stream).  Calls enqueue work and return;
 * they neither allocate nor synchronise.  Return value: 0 on success, otherwise a hydra_status
 * (HYDRA_ERR_INVALID_ARG for shapes/alignments the kernel does not accept, HYDRA_ERR_DEVICE for a
 * launch failure); hydra_ops_last_error() gives the text.
 *
 * The operations are the ones a forward pass, a backward pass and a gradient update of a shard
 * consist of (paper, Introduction, "Motivation": features flow layer to layer forward, gradients
 * backward; Approach, "Desiderata": gradient updates must be exactly those of unsharded training),
 * written for G same-shaped problems of different models at once (Approach: shards of different
 * models are independent units of parallel work).
 */
#ifndef HYDRA_OPS_H
#define HYDRA_OPS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { HYDRA_OPS_F32 = 0, HYDRA_OPS_BF16 = 1 };                  /* operand dtype                    */
enum { HYDRA_EPI_NONE = 0, HYDRA_EPI_RELU = 1, HYDRA_EPI_GELU = 2 };

/* out_g[M,N] = epilogue( sum_k X_g(m,k) * W_g(n,k) ), fp32 accumulation.
 *   epilogue: v = acc + bias[n] (if bias); pre[m,n] = v (if pre);
 *             v = gate ? v * act'(gate[m,n]) : act(v);  v += resid[m,n] (if resid); out[m,n] = v.
 * x_kmajor = 1: X_g stored [M, ldx], k contiguous; 0: stored [K, ldx], m contiguous.
 * w_kmajor = 1: W_g stored [N, ldw], k contiguous; 0: stored [K, ldw], n contiguous.
 * Forward Linear: X = input, W = weight[out,in], both k-major.  Input gradient: X = dY (k-major),
 * W = weight (k is its slow index).  Weight gradient: X = dY, W = input, both with k slow.
 * Leading dimensions count elements; ldx, ldw multiples of 16 bytes and >= the contiguous extent
 * rounded up to 16 bytes; ldo, ldg, ldr multiples of 8 and >= N.  bias is fp32 [N].  out is fp32
 * when out_f32, else the operand dtype; pre, gate, resid have the operand dtype.  Optional tables
 * may be NULL.  tile: 0 = automatic, 1 = 256x256, 2 = 128x128, 3 = 32x128 workgroup tiles, 4 = 256x256 with
 * operands staged through registers (1 loads bf16 k-contiguous operands straight into LDS).  All give the
 * same bits. */
typedef struct {
  int dtype, M, N, K, x_kmajor, w_kmajor, ldx, ldw, ldo, ldg, ldr, act, out_f32, tile, G;
  const void* const* X;
  const void* const* W;
  const float* const* bias;
  void* const* out;
  void* const* pre;
  const void* const* gate;
  const void* const* resid;
  float* const* rowsum; /* optional, weight-gradient layout (x_kmajor = w_kmajor = 0) only: rowsum_g[m] =
                           sum_k X_g(m,k) in fp32, M floats each; with X = dY this is the bias gradient */
  void* const* ws;      /* optional device scratch, 32-byte aligned, ws_bytes each: a bf16 weight-gradient problem
                           (x_kmajor = w_kmajor = 0, out_f32, no bias/pre/gate/resid, no activation) with
                           hydra_op_gemm_split_k(M, N, K) = S > 1 then sums S contiguous ranges of k separately and
                           adds the partial sums in ascending order in a second launch.  S depends on the shape
                           alone.  Without scratch (or with too little) the sum runs in one chain */
  size_t ws_bytes;
} hydra_gemm_desc;
int hydra_op_gemm_split_k(int M, int N, int K);                   /* 1 = this shape is never split   */
size_t hydra_op_gemm_split_ws_bytes(int M, int N, int K, int ldo);  /* scratch bytes per problem, 0 if S = 1 */
int hydra_op_gemm(const hydra_gemm_desc* d, void* stream);

/* out_g[n] = sum_{m<M} src_g[m,n]; src has the operand dtype and leading dimension ld, out is fp32.
 * part_g: scratch of hydra_op_colsum_part_floats(M, N) floats (0 for M <= 256: the table may then be NULL). */
int hydra_op_colsum(int dtype, int M, int N, int ld, int G, const void* const* src, float* const* out,
                    float* const* part, void* stream);
size_t hydra_op_colsum_part_floats(int M, int N);

/* hydra_op_colsum for callers that cannot allocate device memory or hand over scratch: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same kernels, same order of additions and therefore the same
 * bits as hydra_op_colsum; the partial sums live in an array built into the library (one copy per GPU, held until the
 * process ends) of hydra_op_colsum_noalloc_max_floats() = 1048576 floats (4 MiB).  A call needs
 * G * hydra_op_colsum_part_floats(M, N) of them; more returns HYDRA_ERR_INVALID_ARG and nothing is launched.  The
 * call allocates and frees nothing and does not synchronise.  Every call on a GPU uses that GPU's one array: calls
 * whose kernels may overlap on one GPU (different streams, or different threads) race; calls on one stream do not. */
int hydra_op_colsum_noalloc(int dtype, int M, int N, int ld, int G, const void* const* src, float* const* out,
                            void* stream);
size_t hydra_op_colsum_noalloc_max_floats(void);

/* Softmax cross-entropy over fp32 logits [M, ldz] with C classes and int32 labels [M] (shared by the
 * group): rowloss_g[m] = logsumexp(z_m) - z_m[y_m]; dz_g[m,c] = (softmax(z_m)[c] - [c==y_m]) * inv_n
 * in the operand dtype with leading dimension lddz (columns [C,lddz) are zeroed);
 * loss_g[0] = inv_n * sum_m rowloss_g[m]. */
int hydra_op_softmax_ce(int dtype, int M, int C, int ldz, int lddz, float inv_n, int G, const float* const* logits,
                        const int32_t* labels, void* const* dz, float* const* rowloss, float* const* loss, void* stream);

/* Optimizer step over flat fp32 blocks of n elements (n % 4 == 0).  opt 0 = SGD (m, v ignored),
 * 1 = Adam with bias-correction factors bc1 = 1/(1-b1^t), bc2 = 1/(1-b2^t) given per problem.
 * w16 (optional) receives the bf16 rounding of the updated parameters.  hp: G rows of
 * {lr, b1, b2, eps, bc1, bc2} in double (host); they are rounded to fp32 once, as is 1-b. */
int hydra_op_optim(int opt, size_t n, int G, float* const* p, const float* const* g, float* const* m, float* const* v,
                   void* const* w16, const double* hp, void* stream);

/* Weight gradient with the optimizer step in its epilogue (paper, Approach, "Desiderata": the update
 * is the one a separate optimizer pass would apply, bit for bit).  d describes the gradient GEMM
 * dW_g[M,N] = sum_k X_g(m,k) W_g(n,k) with x_kmajor = w_kmajor = 0, out_f32 = 1, no bias/pre/gate/resid
 * and act = HYDRA_EPI_NONE; element [m,n] of the gradient updates p_g[m*ldo + n] (and m_g, v_g, w16_g
 * at the same index) as hydra_op_optim would.  d->out may be NULL (the gradient is then never
 * stored) or a table of fp32 [M, ldo] buffers that also receive it.  p, m, v 32-byte aligned, w16 16-byte;
 * hp as for hydra_op_optim.  Errors: HYDRA_ERR_INVALID_ARG for shapes or tables the kernel cannot take. */
int hydra_op_gemm_update(const hydra_gemm_desc* d, int opt, float* const* p, float* const* m, float* const* v,
                         void* const* w16, const double* hp, void* stream);

/* dst[i] = u_i * 2a - a with u_i the 24-bit uniform of the counter generator (SplitMix64 keyed by
 * (seed, stream_id)); the values a model's tensor `stream_id = (model << 20) | tensor` is initialised with. */
int hydra_op_init_uniform(float* dst, size_t n, uint64_t seed, uint64_t stream_id, float a, void* stream);

/* dst[i] = bf16(src[i]) (round to nearest even), i < n. */
int hydra_op_cast_bf16(const float* src, void* dst, size_t n, void* stream);

/* LayerNorm over rows of width d (d % 8 == 0, d <= 4096, ld % 8 == 0): per row mu = mean, var = biased
 * variance, y = (x-mu)/sqrt(var+eps)*gamma + beta.  x, y have the operand dtype; gamma, beta, mean, rstd fp32. */
int hydra_op_layernorm_fwd(int dtype, int rows, int d, int ld, float eps, int G, const void* const* x, void* const* y,
                           const float* const* gamma, const float* const* beta, float* const* mean,
                           float* const* rstd, void* stream);
/* Adjoint: dx = rstd*(g - mean(g) - xhat*mean(g*xhat)) + add, g = dy*gamma (add optional: NULL table);
 * dgamma = sum_rows dy*xhat; dbeta = sum_rows dy.  part_g: scratch of hydra_op_layernorm_part_floats(rows, d) floats. */
int hydra_op_layernorm_bwd(int dtype, int rows, int d, int ld, int G, const void* const* x, const void* const* dy,
                           const void* const* add, void* const* dx, const float* const* gamma,
                           const float* const* mean, const float* const* rstd, float* const* part,
                           float* const* dgamma, float* const* dbeta, void* stream);
size_t hydra_op_layernorm_part_floats(int rows, int d);

/* Attention, bf16, head width DH in {64,128}.  qkv_g [B*S, ld_qkv]: q of head h at columns [h*DH,(h+1)*DH),
 * k at H*DH + the same, v at 2*H*DH + the same.  o_g [B*S, ld_o].  P = softmax(q k^T * scale (+ causal mask)),
 * o = P v, lse_g [B*H*S] = log-sum-exp of the scaled scores. */
int hydra_op_attention_fwd(int B, int S, int H, int DH, int ld_qkv, int ld_o, int causal, float scale, int G,
                           const void* const* qkv, void* const* o, float* const* lse, void* stream);
/* Adjoint given dout_g [B*S, ld_o] (gradient w.r.t. o): dqkv_g in the layout of qkv; delta_g [B*H*S] scratch. */
int hydra_op_attention_bwd(int B, int S, int H, int DH, int ld_qkv, int ld_o, int causal, float scale, int G,
                           const void* const* qkv, const void* const* o, const void* const* dout,
                           const float* const* lse, float* const* delta, void* const* dqkv, void* stream);

/* x_g[t,:] = tok_g[ids[t],:] + pos_g[t mod S,:]; ids int32 [tokens] shared by the group; tables in the operand dtype. */
int hydra_op_embed_fwd(int dtype, int tokens, int S, int d, int ld, int G, const int32_t* ids, const void* const* tok,
                       const void* const* pos, void* const* x, void* stream);
/* dtok_g[v,:] = sum of dx_g[t,:] over tokens with id v, listed by the CSR (row_ptr [V+1], positions [B*S], both
 * int32 device arrays); dpos_g[s,:] = sum_b dx_g[b*S+s,:] for s < S, zero for S <= s < S_table.  Outputs fp32. */
int hydra_op_embed_bwd(int dtype, int V, int S, int S_table, int B, int d, int ld, int G, const int32_t* row_ptr,
                       const int32_t* positions, const void* const* dx, float* const* dtok, float* const* dpos,
                       void* stream);

/* Measurement aid: enqueues n launches of a kernel that does nothing (one wave) on `stream`.  The time per launch of
 * a long run of them is the floor under any step that is a chain of dependent launches, which is what bounds the
 * smallest workload (its whole step is microseconds of arithmetic). */
int hydra_op_empty_launches(int n, void* stream);

const char* hydra_ops_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* HYDRA_OPS_H */
