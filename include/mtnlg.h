/*
 * mtnlg.h -- C ABI of the MI355X (gfx950) transformer-layer-slice library.
 *
 * The library computes the forward and backward pass of ONE GPU's share of a
 * GPT-2 style pre-LayerNorm decoder layer stack under Megatron tensor slicing,
 * as used for MT-NLG 530B (paper: Section 3.2 "Model and Training Process" for
 * the model: 105 layers, hidden 20480, 128 heads, sequence 2048, 8-way tensor
 * and 35-way pipeline parallelism; Section 2.1 "Tensor Model Parallelism" for
 * the slicing; Section 2.3 for bf16 mixed precision; Section 2.1 "Memory
 * Efficiency" for activation recomputation and gradient accumulation).
 *
 * One layer on tensor-parallel rank r (T = micro_batch*seq tokens, p =
 * heads_local*head_dim, F = ffn_local):
 *
 *   u1  = LN(x; ln1_g, ln1_b)                      [T,h]
 *   qkv = u1 w_qkv^T + b_qkv                       [T,3p]  column-parallel
 *   a   = causal softmax attention per local head  [T,p]
 *   A_r = a w_o^T                                  [T,h]   row-parallel PARTIAL
 *   x1  = x + reduce(A_r) + b_o
 *   u2  = LN(x1; ln2_g, ln2_b)
 *   z   = u2 w_fc1^T + b_fc1 ; g = GeLU(z)         [T,F]   column-parallel
 *   M_r = g w_fc2^T                                [T,h]   row-parallel PARTIAL
 *   y   = x1 + reduce(M_r) + b_fc2
 *
 * reduce() is the sum over the tensor-parallel group.  The library never talks
 * to another GPU: with a NULL hook the partial is used as if it were the sum
 * (a group of one); a non-NULL hook is called on the partial buffer at each of
 * the four reduce points (two forward, two backward) and must leave the sum in
 * place, enqueued on the given stream.
 *
 * ALL data pointers are DEVICE pointers (HIP global memory) unless stated.
 * Descriptor / weight-table / grad-table structs themselves live in HOST memory.
 * The library allocates no device memory, launches only on the stream it is
 * given and never synchronises the host.  Its only process-wide state: per-device
 * marks that a kernel's attributes have been set, the address of the static
 * array of mtnlg_colsum_static, and the optional timing record.
 *
 * Layouts (row-major everywhere):
 *   activations  [micro_batch, seq, hidden], hidden contiguous
 *   linear weights [out_features, in_features]  (y = x W^T)
 *   w_qkv rows (and qkv columns) ordered [head][q|k|v][head_dim], so a rank's
 *   slice of the unsliced matrix is one contiguous row block.
 *   The caller passes dense local copies of its slice.
 * Element type: float when desc.dtype == MTNLG_F32, bfloat16 (round to nearest
 * even on every store) when MTNLG_BF16; all accumulation, softmax, LayerNorm and
 * GeLU arithmetic is fp32 in both cases.  All pointers 16-byte aligned.
 *
 * Every entry point returns an int status: 0 on success, a negative
 * mtnlg_status otherwise.  Outputs are unspecified after an error.  Nothing
 * throws or aborts across this boundary.
 */
#ifndef MTNLG_H_
#define MTNLG_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Every int-returning entry point returns one of these.  Arguments are checked before any
 * launch: a size or count <= 0 (an empty problem), an unknown enum value, a non-finite scale or
 * aliasing the call forbids is MTNLG_INVALID_ARG; a missing required pointer MTNLG_NULL_POINTER;
 * a shape the kernels do not cover (e.g. widths that are not multiples of 8 on the bf16 path)
 * MTNLG_UNSUPPORTED_SHAPE; after an error the outputs are unspecified.  Size queries return 0
 * for descriptors that would be rejected. */
enum mtnlg_status {
  MTNLG_OK = 0,
  MTNLG_INVALID_ARG = -1,
  MTNLG_NULL_POINTER = -2,
  MTNLG_UNSUPPORTED_SHAPE = -3,
  MTNLG_WORKSPACE_TOO_SMALL = -4,
  MTNLG_HIP_ERROR = -5,      /* a launch was refused (hipGetLastError after it; no synchronisation) */
  MTNLG_REDUCE_FAILED = -6   /* the caller's reduce hook returned non-zero */
};

enum mtnlg_dtype { MTNLG_F32 = 0, MTNLG_BF16 = 1 };
enum mtnlg_gelu { MTNLG_GELU_TANH = 0, MTNLG_GELU_ERF = 1 };

/* desc.flags */
#define MTNLG_RECOMPUTE 1u        /* stage_step keeps only layer inputs and reruns each
                                     layer's forward just before its backward            */
#define MTNLG_ACCUMULATE_WGRAD 2u /* parameter grads are added into the grad buffers
                                     (gradient accumulation over micro-batches)          */
#define MTNLG_WGRAD_FP32 4u       /* parameter grad buffers are float even on the bf16 path */

typedef struct {
  int32_t hidden;       /* h                                                     */
  int32_t heads_local;  /* n: attention heads of this slice                      */
  int32_t head_dim;     /* d                                                     */
  int32_t ffn_local;    /* F: FFN columns of this slice                          */
  int32_t seq;          /* s                                                     */
  int32_t micro_batch;  /* b                                                     */
  int32_t tp_size;      /* R >= 1 (metadata handed to the reduce hook's owner)   */
  int32_t tp_rank;      /* 0 <= r < R                                            */
  int32_t dtype;        /* mtnlg_dtype                                           */
  int32_t gelu;         /* mtnlg_gelu                                            */
  float ln_eps;         /* 0 => 1e-5                                             */
  float softmax_scale;  /* 0 => 1/sqrt(head_dim)                                 */
  uint32_t flags;
} mtnlg_layer_desc;

/* Parameter tables (host structs of device pointers).  Shapes:
 *   ln1_g, ln1_b, ln2_g, ln2_b, b_o, b_fc2 : [h]
 *   w_qkv [3p,h]  b_qkv [3p]  w_o [h,p]  w_fc1 [F,h]  b_fc1 [F]  w_fc2 [h,F]   */
typedef struct {
  const void *ln1_g, *ln1_b, *w_qkv, *b_qkv, *w_o, *b_o;
  const void *ln2_g, *ln2_b, *w_fc1, *b_fc1, *w_fc2, *b_fc2;
} mtnlg_layer_weights;

/* Same shapes; element type is desc.dtype's, or float under MTNLG_WGRAD_FP32. */
typedef struct {
  void *ln1_g, *ln1_b, *w_qkv, *b_qkv, *w_o, *b_o;
  void *ln2_g, *ln2_b, *w_fc1, *b_fc1, *w_fc2, *b_fc2;
} mtnlg_layer_grads;

/* Sum `count` elements of type `dtype` at device pointer `buf` over the tensor-
 * parallel group, in place, enqueued on `stream` (a hipStream_t).  Return 0 on
 * success.  Called from the host thread that called the library. */
typedef int (*mtnlg_reduce_fn)(void *buf, size_t count, int dtype, void *stream, void *user);

/* Byte offsets, inside one layer's `saved` block, of what forward keeps for
 * backward.  u1,x1,u2 [T,h]; qkv [T,3p]; a [T,p]; z,g [T,F] in the storage
 * dtype; mu*, rs* [T] and lse [b,n,s] (log-sum-exp of the scaled, masked
 * scores) in float. */
typedef struct {
  size_t u1, qkv, a, x1, u2, z, g, mu1, rs1, mu2, rs2, lse, total;
} mtnlg_saved_layout;

/* --- queries (host only, no GPU work) --------------------------------------- */
int mtnlg_version(void);
const char *mtnlg_status_string(int status);
/* 0 if the shape is supported, else a negative status.
 * Requirements: all sizes > 0; hidden, ffn_local, head_dim multiples of 8;
 * hidden <= 32768; head_dim <= 256; 0 <= tp_rank < tp_size. */
int mtnlg_layer_desc_check(const mtnlg_layer_desc *desc);
int mtnlg_saved_layout_get(const mtnlg_layer_desc *desc, mtnlg_saved_layout *out);
/* Bytes of one layer's `saved` block (0 on a bad descriptor). */
size_t mtnlg_saved_bytes(const mtnlg_layer_desc *desc);
/* Bytes of the `saved` area mtnlg_stage_step needs for n_layers: per layer the
 * layer input [T,h] plus either a full saved block, or (MTNLG_RECOMPUTE) one
 * shared saved block for the layer being recomputed. */
size_t mtnlg_stage_saved_bytes(const mtnlg_layer_desc *desc, int n_layers);
/* Bytes of scratch any of the three calls below needs (max over them). */
size_t mtnlg_workspace_bytes(const mtnlg_layer_desc *desc);

/* --- the hot path ------------------------------------------------------------ */

/* Forward of one layer slice: the decoder layer of the paper's Section 3.2 ("Model and Training Process") under the
 * tensor slicing of Section 2.1 ("Tensor Model Parallelism"): column-parallel QKV and FC1, row-parallel projection
 * and FC2 whose outputs are partial sums; storage in bf16 with fp32 arithmetic as in Section 2.3 (equations at the
 * top of this file).
 *   x [T,h] in, y [T,h] out (y must not alias x); saved: this layer's block of
 *   mtnlg_saved_bytes() bytes, written; workspace: scratch, contents destroyed.
 *   reduce/user: tensor-parallel sum hook or NULL.  stream: hipStream_t (NULL =
 *   the null stream). */
int mtnlg_layer_fwd(const mtnlg_layer_desc *desc, const mtnlg_layer_weights *w, const void *x,
                    void *y, void *saved, void *workspace, size_t workspace_bytes,
                    mtnlg_reduce_fn reduce, void *user, void *stream);

/* Backward of one layer slice: the adjoint of mtnlg_layer_fwd, i.e. the other half of the per-GPU work that the
 * paper's Section 2.4 throughput figures count; the two backward sums over the tensor-parallel group of Section 2.1
 * sit at the hook.  Parameter gradients in the storage type ("2 bytes" per gradient, Section 2.1 "Memory
 * Efficiency") or in float under MTNLG_WGRAD_FP32 (the fp32 gradient copy of the same passage).
 *   x: the layer input given to forward; saved: the block forward wrote;
 *   dy [T,h]: gradient of y; dx [T,h] out: gradient of x (may not alias dy);
 *   grads: all 12 parameter gradients, overwritten, or added to under
 *   MTNLG_ACCUMULATE_WGRAD. */
int mtnlg_layer_bwd(const mtnlg_layer_desc *desc, const mtnlg_layer_weights *w, const void *x,
                    const void *saved, const void *dy, void *dx, const mtnlg_layer_grads *grads,
                    void *workspace, size_t workspace_bytes, mtnlg_reduce_fn reduce, void *user,
                    void *stream);

/* One pipeline-stage step -- what one GPU of a pipeline stage does for one micro-batch (Section 2.1, paragraph
 * "Pipeline Model Parallelism"; Section 3.2: 105 layers under 35-way pipeline parallelism = 3 layers per GPU;
 * Section 2.1, paragraph "Memory Efficiency", for the activation recomputation that MTNLG_RECOMPUTE selects):
 * forward through n_layers stacked slices (layer l's y
 * is layer l+1's x), then backward through them in reverse, all on `stream`
 * with no host synchronisation.  w and grads are host arrays of n_layers tables.
 *   x_in [T,h], dy_out [T,h] in; y_out [T,h], dx_in [T,h] out.
 *   saved: mtnlg_stage_saved_bytes() bytes.  Under MTNLG_RECOMPUTE only each
 *   layer's input is kept and the layer's forward is rerun inside backward
 *   (same function, same results). */
int mtnlg_stage_step(const mtnlg_layer_desc *desc, int n_layers, const mtnlg_layer_weights *w,
                     const void *x_in, const void *dy_out, void *y_out, void *dx_in,
                     const mtnlg_layer_grads *grads, void *saved, size_t saved_bytes,
                     void *workspace, size_t workspace_bytes, mtnlg_reduce_fn reduce, void *user,
                     void *stream);

/* The same step over n_micro micro-batches with the parameter gradients summed over them -- the
 * gradient accumulation of Section 2.1 (paragraph "Memory Efficiency") as one pipeline rank sees it in the
 * steady state of the 1F1B schedule (Section 2.1, paragraph "Pipeline Model Parallelism"): micro-batch 0 overwrites
 * the gradient buffers
 * (adds to them if desc carries MTNLG_ACCUMULATE_WGRAD), the following ones add.  With bf16 gradient
 * buffers every addition rounds; MTNLG_WGRAD_FP32 gives the fp32 buffers the paper accumulates in.
 *   x_in, dy_out in, y_out, dx_in out: [n_micro][T,h], micro-batches contiguous one after the other.
 *   saved and workspace are those of one micro-batch and are reused by each (the activations of a
 *   micro-batch are dead once its backward has run).  Other arguments, ownership and errors as
 *   mtnlg_stage_step; n_micro <= 0 is MTNLG_INVALID_ARG. */
int mtnlg_stage_step_accumulate(const mtnlg_layer_desc *desc, int n_layers, const mtnlg_layer_weights *w,
                                int n_micro, const void *x_in, const void *dy_out, void *y_out, void *dx_in,
                                const mtnlg_layer_grads *grads, void *saved, size_t saved_bytes,
                                void *workspace, size_t workspace_bytes, mtnlg_reduce_fn reduce, void *user,
                                void *stream);

/* --- single operations of the path (used by stage/layer calls; exported so each
 *     kernel can be checked and timed alone) ----------------------------------- */

enum mtnlg_gemm_layout {
  MTNLG_GEMM_NT = 0, /* C[M,N] = A[M,K] * B[N,K]^T   forward linears (x W^T)         */
  MTNLG_GEMM_NN = 1, /* C[M,N] = A[M,K] * B[K,N]     data gradients (dY W)           */
  MTNLG_GEMM_TN = 2  /* C[M,N] = A[K,M]^T * B[K,N]   weight gradients (dY^T X)       */
};

/* gemm epilogue flags */
#define MTNLG_EPI_BIAS 1u       /* + bias[n] (float-typed storage dtype vector of N)   */
#define MTNLG_EPI_GELU 2u       /* C = GeLU(acc+bias), and pre-activation to `aux`      */
#define MTNLG_EPI_RESIDUAL 4u   /* + aux[m,n] (same shape/ld as C) read                 */
#define MTNLG_EPI_ACCUMULATE 8u /* C += result                                          */
#define MTNLG_EPI_OUT_F32 16u   /* C is float even when inputs are bf16                 */
#define MTNLG_EPI_GELU_ERF 32u  /* with MTNLG_EPI_GELU / _GELU_GRAD: erf form, not tanh   */
#define MTNLG_EPI_GELU_GRAD 64u /* C = acc * GeLU'(aux[m,n]): the activation's backward
                                   fused into the product that yields dg (aux = z, read)  */

/* General matrix product with fp32 accumulation, dense row-major operands
 * (leading dimension = row length).  dtype selects float or bf16 inputs.
 * aux: pre-activation output under EPI_GELU, residual input under EPI_RESIDUAL, pre-activation input under
 * EPI_GELU_GRAD (at most one of the three; EPI_GELU_GRAD goes with neither bias nor accumulate).
 * workspace (nullable): mtnlg_gemm_workspace() bytes of scratch that lets a problem
 * whose last round of output tiles would leave most compute units idle split those
 * tiles along K; without it the same result is computed by whole tiles only. */
size_t mtnlg_gemm_workspace(int dtype, int layout, int64_t M, int64_t N, int64_t K);
int mtnlg_gemm(int dtype, int layout, int64_t M, int64_t N, int64_t K, const void *A, const void *B,
               void *C, const void *bias, void *aux, uint32_t epilogue, void *workspace,
               size_t workspace_bytes, void *stream);

/* out = LN(x [+ partial + bias]) per token row; if partial != NULL also writes
 * xsum = x + partial + bias (bias may be NULL).  mean/rstd [T] float out. */
int mtnlg_layernorm_fwd(int dtype, int64_t T, int64_t h, const void *x, const void *partial,
                        const void *bias, const void *gamma, const void *beta, float eps,
                        void *xsum, void *out, float *mean, float *rstd, void *stream);

/* dx = dres + LN^T(dout) ; dgamma, dbeta (float or storage dtype per grad_f32),
 * overwritten or accumulated.  x is the LayerNorm's input.  dres may be NULL.
 * colsum_dx (nullable, [h]): also receives sum over tokens of dx (a bias grad).
 * workspace: >= mtnlg_layernorm_bwd_workspace(T,h) bytes. */
size_t mtnlg_layernorm_bwd_workspace(int64_t T, int64_t h);
int mtnlg_layernorm_bwd(int dtype, int64_t T, int64_t h, const void *x, const void *gamma,
                        const float *mean, const float *rstd, const void *dout, const void *dres,
                        void *dx, void *dgamma, void *dbeta, void *colsum_dx, int grad_f32,
                        int accumulate, void *workspace, void *stream);

/* Causal softmax attention over local heads.  qkv [b*s, n*3*d] (columns
 * [head][q|k|v][d]) -> a [b*s, n*d], lse [b,n,s] float. */
int mtnlg_attention_fwd(int dtype, int32_t b, int32_t s, int32_t n, int32_t d, float scale,
                        const void *qkv, void *a, float *lse, void *stream);
/* Adjoint: da [b*s, n*d] -> dqkv [b*s, n*3*d].  workspace >= mtnlg_attention_bwd_workspace(). */
size_t mtnlg_attention_bwd_workspace(int32_t b, int32_t s, int32_t n, int32_t d);
int mtnlg_attention_bwd(int dtype, int32_t b, int32_t s, int32_t n, int32_t d, float scale,
                        const void *qkv, const void *a, const float *lse, const void *da,
                        void *dqkv, void *workspace, void *stream);

/* g = GeLU(z) elementwise over count elements. */
int mtnlg_gelu_fwd(int dtype, int gelu, int64_t count, const void *z, void *g, void *stream);
/* dz = dg * GeLU'(z) (dz may alias dg). */
int mtnlg_gelu_bwd(int dtype, int gelu, int64_t count, const void *z, const void *dg, void *dz,
                   void *stream);
/* out[c] = sum_t in[t,c] over a [T,C] matrix (a bias gradient); out float or storage dtype.
 * workspace >= mtnlg_colsum_workspace(T,C) bytes. */
size_t mtnlg_colsum_workspace(int64_t T, int64_t C);
int mtnlg_colsum(int dtype, int64_t T, int64_t C, const void *in, void *out, int out_f32,
                 int accumulate, void *workspace, void *stream);
/* mtnlg_colsum for callers that cannot allocate device memory or hand over a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): same arguments without the workspace, same
 * kernels, same result bit for bit.  The partial sums go through a 4 MiB array that the library holds on every
 * GPU it has run this call on until the process ends; the call allocates and frees nothing.
 * Limit: C <= mtnlg_colsum_static_max_columns() (32768), beyond that MTNLG_WORKSPACE_TOO_SMALL.  Every call on a
 * GPU shares that GPU's array: calls that overlap on one GPU (different streams or threads) race; calls on one
 * stream are ordered.  Other errors as mtnlg_colsum; MTNLG_HIP_ERROR also if the array's address cannot be had. */
int64_t mtnlg_colsum_static_max_columns(void);
int mtnlg_colsum_static(int dtype, int64_t T, int64_t C, const void *in, void *out, int out_f32, int accumulate,
                        void *stream);
/* out = res + partial + bias[col] over [T,h] (bias nullable). */
int mtnlg_bias_residual(int dtype, int64_t T, int64_t h, const void *res, const void *partial,
                        const void *bias, void *out, void *stream);

/* --- first and last pipeline stage's extras (the paper names the GPT-2 decoder, Section 3.2, and
 *     prints none of this: token embedding E [V,h] with learned positions P [s,h], final LayerNorm,
 *     output projection tied to E, next-token cross-entropy).  Under the tensor slicing of
 *     Section 2.1 a rank owns the contiguous rows [vocab_start, vocab_start + vocab_local) of E. --- */

typedef struct {
  int32_t hidden;       /* h                                                                     */
  int32_t vocab_local;  /* rows of E on this rank (bf16 path: a multiple of 8)                   */
  int32_t vocab_start;  /* global id of this rank's first row                                    */
  int32_t seq, micro_batch; /* s, b; T = b * s tokens, token-major like the layer activations     */
  int32_t dtype;        /* MTNLG_F32 or MTNLG_BF16 (storage; statistics and logits are fp32)     */
  float ln_eps;
} mtnlg_head_desc;

enum mtnlg_reduce_op { MTNLG_REDUCE_SUM = 0, MTNLG_REDUCE_MAX = 1 };
/* Exchange hook of a vocabulary-sliced group: replace buf[0..count) (device, element type `dtype`)
 * by its elementwise sum or maximum over the ranks, enqueued on `stream`; return 0.  NULL = a group
 * of one (the local values are the group's). */
typedef int (*mtnlg_reduce_op_fn)(void *buf, size_t count, int dtype, int op, void *stream, void *user);

/* x [T,h] = sum over ranks of (E[tokens[t] - vocab_start] if the id is this rank's, else 0), hook
 * (SUM), then + P[t mod s].  tokens: device int32 [T], global ids.  emb [vocab_local,h], pos [s,h]. */
int mtnlg_embedding_fwd(const mtnlg_head_desc *desc, const int32_t *tokens, const void *emb, const void *pos,
                        void *x, mtnlg_reduce_op_fn reduce, void *user, void *stream);
/* demb [vocab_local,h] = per token id of this rank, the sum (in token order: deterministic) of the
 * rows of dx [T,h]; dpos [s,h] = dx summed over the batch.  Both overwritten, storage dtype. */
int mtnlg_embedding_bwd(const mtnlg_head_desc *desc, const int32_t *tokens, const void *dx, void *demb,
                        void *dpos, void *stream);
/* Last stage, forward and backward in one call: u = LN(x); logits = u E^T (this rank's block, fp32);
 * loss[t] = log sum_v exp(logits[t,v]) - logits[t, targets[t]] with the maximum, the sum of
 * exponentials and the target's logit exchanged through the hook (MAX, SUM, SUM);
 * dlogits = dloss[t] * (softmax - onehot) (dloss NULL: 1/T each, the mean loss);
 * du = dlogits E, hook (SUM); demb = dlogits^T u; dx, d_ln_g, d_ln_b = LN backward.
 *   x [T,h] in; targets: device int32 [T] global ids; loss: device float [T] out; dx [T,h],
 *   d_ln_g, d_ln_b [h], demb [vocab_local,h] out (storage dtype, overwritten).
 *   workspace >= mtnlg_lm_head_workspace(desc) bytes.  Errors as for the layer calls. */
size_t mtnlg_lm_head_workspace(const mtnlg_head_desc *desc);
int mtnlg_lm_head_step(const mtnlg_head_desc *desc, const void *x, const void *ln_g, const void *ln_b,
                       const void *emb, const int32_t *targets, const float *dloss, float *loss, void *dx,
                       void *d_ln_g, void *d_ln_b, void *demb, void *workspace, size_t workspace_bytes,
                       mtnlg_reduce_op_fn reduce, void *user, void *stream);

/* --- optimizer step on the slice (Section 3.2: Adam, beta1 0.9, beta2 0.95, epsilon 1e-8, gradient
 *     norm clipped at 1.0, weight decay 0.1; Section 2.1: fp32 copies of weights and gradients and the
 *     two Adam states, 20 bytes per parameter).  Works on the fp32 gradient buffers that
 *     MTNLG_WGRAD_FP32 makes the backward pass accumulate into. ------------------------------------- */

typedef struct {
  float lr;            /* learning rate of this step (warm-up and decay are the caller's)            */
  float beta1, beta2;  /* decay rates of the two moments, in [0,1)                                   */
  float eps;           /* added to the root of the second moment, > 0                                */
  float weight_decay;  /* decoupled: lr * weight_decay * weight is subtracted; 0 for tensors that    */
                       /* do not decay                                                               */
  float max_grad_norm; /* clip the global gradient norm at this value; <= 0: no clipping             */
  int32_t step;        /* update count t, from 1, for the bias corrections 1 - beta^t                */
} mtnlg_adam_desc;

/* sqnorm[0] (device float) = sum of squares of grad[0..count), or that added to sqnorm[0] when
 * accumulate != 0 (one scalar over several tensors).  Deterministic: fixed ranges, fixed summation
 * tree, fp64 partial sums.  Across ranks the scalars are summed by the caller before mtnlg_adam_step.
 * grad 16-byte aligned; workspace >= mtnlg_grad_sqnorm_workspace() bytes, 8-byte aligned. */
size_t mtnlg_grad_sqnorm_workspace(void);
int mtnlg_grad_sqnorm(int64_t count, const float *grad, void *workspace, float *sqnorm, int accumulate,
                      void *stream);
/* One Adam update of `count` parameters, in place on the fp32 weight `master` and the moments m, v:
 *   g' = grad * min(1, max_grad_norm / (sqrt(sqnorm[0]) + 1e-6));  m = beta1 m + (1-beta1) g';
 *   v = beta2 v + (1-beta2) g'^2;  master -= lr * ((m / (1-beta1^t)) / (sqrt(v / (1-beta2^t)) + eps)
 *   + weight_decay * master);  weight_bf16 (nullable) = master rounded to nearest even.
 * sqnorm: device scalar holding the squared global gradient norm (NULL: no clipping); it is read on the
 * device, nothing synchronises with the host.  All fp32 pointers 16-byte aligned, weight_bf16 8-byte.
 * grad is not modified.  Errors: MTNLG_NULL_POINTER, MTNLG_INVALID_ARG (count <= 0, step < 1, rates
 * out of range, alignment), MTNLG_HIP_ERROR. */
int mtnlg_adam_step(const mtnlg_adam_desc *desc, int64_t count, float *master, float *m, float *v,
                    const float *grad, void *weight_bf16, const float *sqnorm, void *stream);

/* --- per-kernel-class timing (optional) --------------------------------------
 * While enabled, the library records a HIP event on the launch stream after each
 * of its launches (and one before the first of a run); a launch is timed from the
 * event that closed the previous launch on the same stream, so work that the
 * caller enqueues between two library launches counts for the second.
 * mtnlg_profile_read synchronises those events and returns, per class, the number
 * of launches and their summed duration in milliseconds, then clears the record.
 * Event objects are host-side resources created on demand and destroyed by
 * mtnlg_profile_enable(0).  Not thread-safe. */
enum mtnlg_kernel_class {
  MTNLG_K_GEMM_NT = 0, MTNLG_K_GEMM_NN, MTNLG_K_GEMM_TN, MTNLG_K_ATTN_FWD, MTNLG_K_ATTN_BWD,
  MTNLG_K_LN_FWD, MTNLG_K_LN_BWD, MTNLG_K_GELU, MTNLG_K_COLSUM, MTNLG_K_ELEMENTWISE,
  MTNLG_K_CLASSES
};
int mtnlg_profile_enable(int on);
/* paused != 0: stop recording, keep what is recorded; 0: record again (timing must have been enabled). */
int mtnlg_profile_pause(int paused);
int mtnlg_profile_read(int32_t *launches /*[MTNLG_K_CLASSES]*/, float *ms /*[MTNLG_K_CLASSES]*/);

/* --- measurement aids: what the chip sustains, with the benchmark's data, on the two resources that
 *     bound the layer's kernels (the throughput figures of the paper's Section 2.4 are fractions of a peak;
 *     these give the peak as measured next to the nominal one) ----------------------------------------------
 * mtnlg_calibrate_mfma: `workgroups` workgroups of 8 waves run `iters` rounds of 16 bf16 matrix-core
 * instructions (16x16x32, fp32 accumulate; issued in the order the GEMM kernel uses) each on fragments taken from `operands` (device, bf16,
 * mtnlg_calibrate_mfma_operand_bytes(workgroups) bytes, any finite values: the clock the power limit allows
 * depends on the data); nothing else runs in the loop.  out: device float[workgroups * 512], written.  The
 * work is mtnlg_calibrate_mfma_flops(workgroups, iters) FLOP; the caller times the launch.
 * mtnlg_calibrate_copy: dst[0..bytes) = src[0..bytes) (device, 16-byte aligned, bytes a multiple of 16, no
 * overlap) by a plain streaming kernel: 2 * bytes of HBM traffic. */
size_t mtnlg_calibrate_mfma_operand_bytes(int workgroups);
int64_t mtnlg_calibrate_mfma_flops(int workgroups, int iters);
int mtnlg_calibrate_mfma(int workgroups, int iters, const void *operands, float *out, void *stream);
int mtnlg_calibrate_copy(void *dst, const void *src, int64_t bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* MTNLG_H_ */
