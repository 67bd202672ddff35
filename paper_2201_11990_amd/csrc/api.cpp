// Host orchestration behind the C ABI: descriptor checks, buffer carving, and the
// sequence of kernel launches that make one layer's forward, its backward, and a
// pipeline-stage step.  Equations: see include/mtnlg.h.
#include <math.h>
#include <string.h>

#include "common.h"

using namespace mtnlg;

namespace {

struct Shape {
  int64_t T, h, p, F;
  int b, s, n, d;
  size_t es;  // bytes per stored element
  int dtype, gelu_erf;
  float eps, scale;
  bool acc, g32;
};

int make_shape(const mtnlg_layer_desc *D, Shape *S) {
  if (!D) return MTNLG_NULL_POINTER;
  if (D->hidden <= 0 || D->heads_local <= 0 || D->head_dim <= 0 || D->ffn_local <= 0 || D->seq <= 0 ||
      D->micro_batch <= 0 || D->tp_size <= 0 || D->tp_rank < 0 || D->tp_rank >= D->tp_size)
    return MTNLG_INVALID_ARG;
  if (D->dtype != MTNLG_F32 && D->dtype != MTNLG_BF16) return MTNLG_INVALID_ARG;
  if (D->gelu != MTNLG_GELU_TANH && D->gelu != MTNLG_GELU_ERF) return MTNLG_INVALID_ARG;
  if (D->ln_eps < 0.0f || D->softmax_scale < 0.0f || !isfinite(D->ln_eps) || !isfinite(D->softmax_scale))
    return MTNLG_INVALID_ARG;
  if (D->flags & ~(MTNLG_RECOMPUTE | MTNLG_ACCUMULATE_WGRAD | MTNLG_WGRAD_FP32)) return MTNLG_INVALID_ARG;
  if (D->hidden % 8 || D->ffn_local % 8 || D->head_dim % 8) return MTNLG_UNSUPPORTED_SHAPE;
  if (D->hidden > 32768 || D->head_dim > 256) return MTNLG_UNSUPPORTED_SHAPE;
  if ((int64_t)D->seq * D->micro_batch > (int64_t)1 << 30) return MTNLG_UNSUPPORTED_SHAPE;
  if ((int64_t)D->heads_local * D->head_dim > (int64_t)1 << 24 || D->ffn_local > 1 << 24)
    return MTNLG_UNSUPPORTED_SHAPE;
  // attention: the MFMA kernels within their limits, otherwise the vector-ALU kernels up to their sequence limit,
  // decided here so that a layer call fails before its first launch
  if (!attention_mfma_takes(D->dtype, D->micro_batch, D->seq, D->heads_local, D->head_dim) &&
      (D->seq > ATTENTION_SIMPLE_MAX_SEQ || D->heads_local > 65535 || D->micro_batch > 65535))
    return MTNLG_UNSUPPORTED_SHAPE;
  S->b = D->micro_batch; S->s = D->seq; S->n = D->heads_local; S->d = D->head_dim;
  S->T = (int64_t)S->b * S->s; S->h = D->hidden; S->p = (int64_t)S->n * S->d; S->F = D->ffn_local;
  S->dtype = D->dtype;
  S->es = D->dtype == MTNLG_BF16 ? 2 : 4;
  S->gelu_erf = D->gelu == MTNLG_GELU_ERF;
  S->eps = D->ln_eps > 0.0f ? D->ln_eps : 1e-5f;
  S->scale = D->softmax_scale > 0.0f ? D->softmax_scale : 1.0f / sqrtf((float)S->d);
  S->acc = (D->flags & MTNLG_ACCUMULATE_WGRAD) != 0;
  S->g32 = (D->flags & MTNLG_WGRAD_FP32) != 0 || D->dtype == MTNLG_F32;
  return MTNLG_OK;
}

struct Carver {
  size_t off = 0;
  size_t take(size_t bytes) {
    size_t at = off;
    off = align_up(off + bytes, 256);
    return at;
  }
};

void saved_layout(const Shape &S, mtnlg_saved_layout *L) {
  Carver c;
  L->u1 = c.take(S.T * S.h * S.es);
  L->qkv = c.take(S.T * 3 * S.p * S.es);
  L->a = c.take(S.T * S.p * S.es);
  L->x1 = c.take(S.T * S.h * S.es);
  L->u2 = c.take(S.T * S.h * S.es);
  L->z = c.take(S.T * S.F * S.es);
  L->g = c.take(S.T * S.F * S.es);
  L->mu1 = c.take(S.T * 4);
  L->rs1 = c.take(S.T * 4);
  L->mu2 = c.take(S.T * 4);
  L->rs2 = c.take(S.T * 4);
  L->lse = c.take((size_t)S.b * S.n * S.s * 4);
  L->total = c.off;
}

// Scratch carved from the caller's workspace.
struct Work {
  size_t dgz, du, dx1, da, dqkv, red, attn, ping, pong, gemm, gemm_bytes, total;
};

void work_layout(const Shape &S, Work *W) {
  Carver c;
  W->du = c.take(S.T * S.h * S.es);   // forward: row-parallel partial; backward: du partial
  W->dgz = c.take(S.T * S.F * S.es);
  W->dx1 = c.take(S.T * S.h * S.es);
  W->da = c.take(S.T * S.p * S.es);
  W->dqkv = c.take(S.T * 3 * S.p * S.es);
  size_t red = mtnlg_layernorm_bwd_workspace(S.T, S.h);
  size_t c1 = mtnlg_colsum_workspace(S.T, S.F), c2 = mtnlg_colsum_workspace(S.T, 3 * S.p);
  if (c1 > red) red = c1;
  if (c2 > red) red = c2;
  W->red = c.take(red);
  W->attn = c.take(mtnlg_attention_bwd_workspace(S.b, S.s, S.n, S.d));
  W->ping = c.take(S.T * S.h * S.es);  // stage step: gradient hand-over between layers
  W->pong = c.take(S.T * S.h * S.es);
  // split-K scratch: the largest need over the layer's twelve GEMMs
  size_t gw = 0;
  const int64_t shapes[12][3] = {{S.T, 3 * S.p, S.h}, {S.T, S.h, S.p}, {S.T, S.F, S.h}, {S.T, S.h, S.F},   // forward
                                 {S.T, S.F, S.h}, {S.T, S.h, S.F}, {S.T, S.p, S.h}, {S.T, S.h, 3 * S.p},   // input gradients
                                 {S.h, S.F, S.T}, {S.F, S.h, S.T}, {S.h, S.p, S.T}, {3 * S.p, S.h, S.T}};  // weight gradients
  for (int i = 0; i < 12; ++i) {
    const int layout = i < 4 ? MTNLG_GEMM_NT : i < 8 ? MTNLG_GEMM_NN : MTNLG_GEMM_TN;
    size_t b = mtnlg_gemm_workspace(S.dtype, layout, shapes[i][0], shapes[i][1], shapes[i][2]);
    if (b > gw) gw = b;
  }
  W->gemm_bytes = gw;
  W->gemm = c.take(gw);
  W->total = c.off;
}

inline char *at(void *base, size_t off) { return static_cast<char *>(base) + off; }
inline const char *at(const void *base, size_t off) { return static_cast<const char *>(base) + off; }

bool weights_ok(const mtnlg_layer_weights *w) {
  return w && w->ln1_g && w->ln1_b && w->w_qkv && w->b_qkv && w->w_o && w->b_o && w->ln2_g && w->ln2_b &&
         w->w_fc1 && w->b_fc1 && w->w_fc2 && w->b_fc2;
}
bool grads_ok(const mtnlg_layer_grads *g) {
  return g && g->ln1_g && g->ln1_b && g->w_qkv && g->b_qkv && g->w_o && g->b_o && g->ln2_g && g->ln2_b &&
         g->w_fc1 && g->b_fc1 && g->w_fc2 && g->b_fc2;
}

int call_reduce(mtnlg_reduce_fn reduce, void *user, void *buf, size_t count, int dtype, hipStream_t st) {
  if (!reduce) return MTNLG_OK;
  return reduce(buf, count, dtype, (void *)st, user) == 0 ? MTNLG_OK : MTNLG_REDUCE_FAILED;
}

// Forward of one layer.  with_output = false stops after GeLU (everything backward
// needs is then in `saved`; y is not produced) -- used when a forward is rerun
// only to rebuild activations.
int layer_fwd_impl(const Shape &S, const mtnlg_layer_weights *w, const void *x, void *y, void *saved,
                   void *ws, mtnlg_reduce_fn reduce, void *user, hipStream_t st, bool with_output) {
  mtnlg_saved_layout L;
  saved_layout(S, &L);
  Work W;
  work_layout(S, &W);
  float *mu1 = (float *)at(saved, L.mu1), *rs1 = (float *)at(saved, L.rs1);
  float *mu2 = (float *)at(saved, L.mu2), *rs2 = (float *)at(saved, L.rs2);
  void *u1 = at(saved, L.u1), *qkv = at(saved, L.qkv), *a = at(saved, L.a), *x1 = at(saved, L.x1);
  void *u2 = at(saved, L.u2), *z = at(saved, L.z), *g = at(saved, L.g);
  void *partial = at(ws, W.du), *gws = at(ws, W.gemm);
  const uint32_t gelu_flags = MTNLG_EPI_BIAS | MTNLG_EPI_GELU | (S.gelu_erf ? MTNLG_EPI_GELU_ERF : 0u);

  // u1 = LN1(x)
  MTNLG_TRY(mtnlg_layernorm_fwd(S.dtype, S.T, S.h, x, nullptr, nullptr, w->ln1_g, w->ln1_b, S.eps, nullptr,
                                u1, mu1, rs1, st));
  // qkv = u1 Wqkv^T + bqkv
  MTNLG_TRY(mtnlg_gemm(S.dtype, MTNLG_GEMM_NT, S.T, 3 * S.p, S.h, u1, w->w_qkv, qkv, w->b_qkv, nullptr,
                       MTNLG_EPI_BIAS, gws, W.gemm_bytes, st));
  // a = causal attention
  MTNLG_TRY(mtnlg_attention_fwd(S.dtype, S.b, S.s, S.n, S.d, S.scale, qkv, a, (float *)at(saved, L.lse), st));
  if (reduce) {
    // A_r = a Wo^T ; sum over the group ; x1 = x + A + bo ; u2 = LN2(x1)
    MTNLG_TRY(mtnlg_gemm(S.dtype, MTNLG_GEMM_NT, S.T, S.h, S.p, a, w->w_o, partial, nullptr, nullptr, 0, gws, W.gemm_bytes, st));
    MTNLG_TRY(call_reduce(reduce, user, partial, (size_t)(S.T * S.h), S.dtype, st));
    MTNLG_TRY(mtnlg_layernorm_fwd(S.dtype, S.T, S.h, x, partial, w->b_o, w->ln2_g, w->ln2_b, S.eps, x1, u2,
                                  mu2, rs2, st));
  } else {
    // group of one: the residual and bias ride in the projection's epilogue
    MTNLG_TRY(mtnlg_gemm(S.dtype, MTNLG_GEMM_NT, S.T, S.h, S.p, a, w->w_o, x1, w->b_o, const_cast<void *>(x),
                         MTNLG_EPI_BIAS | MTNLG_EPI_RESIDUAL, gws, W.gemm_bytes, st));
    MTNLG_TRY(mtnlg_layernorm_fwd(S.dtype, S.T, S.h, x1, nullptr, nullptr, w->ln2_g, w->ln2_b, S.eps, nullptr,
                                  u2, mu2, rs2, st));
  }
  // z = u2 W1^T + b1 ; g = GeLU(z)
  MTNLG_TRY(mtnlg_gemm(S.dtype, MTNLG_GEMM_NT, S.T, S.F, S.h, u2, w->w_fc1, g, w->b_fc1, z, gelu_flags, gws, W.gemm_bytes, st));
  if (!with_output) return MTNLG_OK;
  if (reduce) {
    MTNLG_TRY(mtnlg_gemm(S.dtype, MTNLG_GEMM_NT, S.T, S.h, S.F, g, w->w_fc2, partial, nullptr, nullptr, 0, gws, W.gemm_bytes, st));
    MTNLG_TRY(call_reduce(reduce, user, partial, (size_t)(S.T * S.h), S.dtype, st));
    MTNLG_TRY(mtnlg_bias_residual(S.dtype, S.T, S.h, x1, partial, w->b_fc2, y, st));
  } else {
    MTNLG_TRY(mtnlg_gemm(S.dtype, MTNLG_GEMM_NT, S.T, S.h, S.F, g, w->w_fc2, y, w->b_fc2, x1,
                         MTNLG_EPI_BIAS | MTNLG_EPI_RESIDUAL, gws, W.gemm_bytes, st));
  }
  return MTNLG_OK;
}

int layer_bwd_impl(const Shape &S, const mtnlg_layer_weights *w, const void *x, const void *saved,
                   const void *dy, void *dx, const mtnlg_layer_grads *G, void *ws, mtnlg_reduce_fn reduce,
                   void *user, hipStream_t st) {
  mtnlg_saved_layout L;
  saved_layout(S, &L);
  Work W;
  work_layout(S, &W);
  const float *mu1 = (const float *)at(saved, L.mu1), *rs1 = (const float *)at(saved, L.rs1);
  const float *mu2 = (const float *)at(saved, L.mu2), *rs2 = (const float *)at(saved, L.rs2);
  const void *u1 = at(saved, L.u1), *qkv = at(saved, L.qkv), *a = at(saved, L.a), *x1 = at(saved, L.x1);
  const void *u2 = at(saved, L.u2), *z = at(saved, L.z), *g = at(saved, L.g);
  const float *lse = (const float *)at(saved, L.lse);
  void *dgz = at(ws, W.dgz), *du = at(ws, W.du), *dx1 = at(ws, W.dx1), *da = at(ws, W.da);
  void *dqkv = at(ws, W.dqkv), *red = at(ws, W.red), *attn_ws = at(ws, W.attn), *gws = at(ws, W.gemm);
  const int g32 = S.g32 ? 1 : 0, acc = S.acc ? 1 : 0;
  const uint32_t wg_epi = (S.acc ? MTNLG_EPI_ACCUMULATE : 0u) | ((S.g32 && S.dtype == MTNLG_BF16) ? MTNLG_EPI_OUT_F32 : 0u);

  // y = x1 + M + b2:  db2 = sum_t dy ; dW2 = dy^T g ; dz = (dy W2) o GeLU'(z), the activation's backward in the
  // epilogue of the product (dg itself is never stored) ; db1 = sum_t dz
  MTNLG_TRY(mtnlg_colsum(S.dtype, S.T, S.h, dy, G->b_fc2, g32, acc, red, st));
  MTNLG_TRY(mtnlg_gemm(S.dtype, MTNLG_GEMM_TN, S.h, S.F, S.T, dy, g, G->w_fc2, nullptr, nullptr, wg_epi, gws, W.gemm_bytes, st));
  MTNLG_TRY(mtnlg_gemm(S.dtype, MTNLG_GEMM_NN, S.T, S.F, S.h, dy, w->w_fc2, dgz, nullptr, const_cast<void *>(z),
                       MTNLG_EPI_GELU_GRAD | (S.gelu_erf ? MTNLG_EPI_GELU_ERF : 0u), gws, W.gemm_bytes, st));
  MTNLG_TRY(mtnlg_colsum(S.dtype, S.T, S.F, dgz, G->b_fc1, g32, acc, red, st));
  // du2_r = dz W1 ; dW1 = dz^T u2
  MTNLG_TRY(mtnlg_gemm(S.dtype, MTNLG_GEMM_NN, S.T, S.h, S.F, dgz, w->w_fc1, du, nullptr, nullptr, 0, gws, W.gemm_bytes, st));
  MTNLG_TRY(mtnlg_gemm(S.dtype, MTNLG_GEMM_TN, S.F, S.h, S.T, dgz, u2, G->w_fc1, nullptr, nullptr, wg_epi, gws, W.gemm_bytes, st));
  MTNLG_TRY(call_reduce(reduce, user, du, (size_t)(S.T * S.h), S.dtype, st));
  // dx1 = dy + LN2^T(du2) ; dgamma2, dbeta2 ; dbo = sum_t dx1
  MTNLG_TRY(mtnlg_layernorm_bwd(S.dtype, S.T, S.h, x1, w->ln2_g, mu2, rs2, du, dy, dx1, G->ln2_g, G->ln2_b,
                                G->b_o, g32, acc, red, st));
  // da = dx1 Wo ; dWo = dx1^T a
  MTNLG_TRY(mtnlg_gemm(S.dtype, MTNLG_GEMM_NN, S.T, S.p, S.h, dx1, w->w_o, da, nullptr, nullptr, 0, gws, W.gemm_bytes, st));
  MTNLG_TRY(mtnlg_gemm(S.dtype, MTNLG_GEMM_TN, S.h, S.p, S.T, dx1, a, G->w_o, nullptr, nullptr, wg_epi, gws, W.gemm_bytes, st));
  // attention backward
  MTNLG_TRY(mtnlg_attention_bwd(S.dtype, S.b, S.s, S.n, S.d, S.scale, qkv, a, lse, da, dqkv, attn_ws, st));
  // dbqkv = sum_t dqkv ; du1_r = dqkv Wqkv ; dWqkv = dqkv^T u1
  MTNLG_TRY(mtnlg_colsum(S.dtype, S.T, 3 * S.p, dqkv, G->b_qkv, g32, acc, red, st));
  MTNLG_TRY(mtnlg_gemm(S.dtype, MTNLG_GEMM_NN, S.T, S.h, 3 * S.p, dqkv, w->w_qkv, du, nullptr, nullptr, 0, gws, W.gemm_bytes, st));
  MTNLG_TRY(mtnlg_gemm(S.dtype, MTNLG_GEMM_TN, 3 * S.p, S.h, S.T, dqkv, u1, G->w_qkv, nullptr, nullptr, wg_epi, gws, W.gemm_bytes, st));
  MTNLG_TRY(call_reduce(reduce, user, du, (size_t)(S.T * S.h), S.dtype, st));
  // dx = dx1 + LN1^T(du1) ; dgamma1, dbeta1
  MTNLG_TRY(mtnlg_layernorm_bwd(S.dtype, S.T, S.h, x, w->ln1_g, mu1, rs1, du, dx1, dx, G->ln1_g, G->ln1_b,
                                nullptr, g32, acc, red, st));
  return MTNLG_OK;
}

}  // namespace

extern "C" {

int mtnlg_version(void) { return 1; }

const char *mtnlg_status_string(int status) {
  switch (status) {
    case MTNLG_OK: return "ok";
    case MTNLG_INVALID_ARG: return "invalid argument";
    case MTNLG_NULL_POINTER: return "null pointer";
    case MTNLG_UNSUPPORTED_SHAPE: return "unsupported shape";
    case MTNLG_WORKSPACE_TOO_SMALL: return "workspace too small";
    case MTNLG_HIP_ERROR: return "HIP error";
    case MTNLG_REDUCE_FAILED: return "reduce hook failed";
    default: return "unknown status";
  }
}

int mtnlg_layer_desc_check(const mtnlg_layer_desc *desc) {
  Shape S;
  return make_shape(desc, &S);
}

int mtnlg_saved_layout_get(const mtnlg_layer_desc *desc, mtnlg_saved_layout *out) {
  if (!out) return MTNLG_NULL_POINTER;
  Shape S;
  MTNLG_TRY(make_shape(desc, &S));
  saved_layout(S, out);
  return MTNLG_OK;
}

size_t mtnlg_saved_bytes(const mtnlg_layer_desc *desc) {
  mtnlg_saved_layout L;
  return mtnlg_saved_layout_get(desc, &L) == MTNLG_OK ? L.total : 0;
}

size_t mtnlg_stage_saved_bytes(const mtnlg_layer_desc *desc, int n_layers) {
  Shape S;
  if (n_layers <= 0 || make_shape(desc, &S) != MTNLG_OK) return 0;
  mtnlg_saved_layout L;
  saved_layout(S, &L);
  size_t slot = align_up(S.T * S.h * S.es, 256);
  size_t blocks = (desc->flags & MTNLG_RECOMPUTE) ? 1 : (size_t)n_layers;
  return (size_t)n_layers * slot + blocks * L.total;
}

size_t mtnlg_workspace_bytes(const mtnlg_layer_desc *desc) {
  Shape S;
  if (make_shape(desc, &S) != MTNLG_OK) return 0;
  Work W;
  work_layout(S, &W);
  return W.total;
}

int mtnlg_layer_fwd(const mtnlg_layer_desc *desc, const mtnlg_layer_weights *w, const void *x, void *y,
                    void *saved, void *workspace, size_t workspace_bytes, mtnlg_reduce_fn reduce,
                    void *user, void *stream) {
  Shape S;
  MTNLG_TRY(make_shape(desc, &S));
  if (!weights_ok(w) || !x || !y || !saved || !workspace) return MTNLG_NULL_POINTER;
  if (x == y) return MTNLG_INVALID_ARG;
  if (workspace_bytes < mtnlg_workspace_bytes(desc)) return MTNLG_WORKSPACE_TOO_SMALL;
  return layer_fwd_impl(S, w, x, y, saved, workspace, reduce, user, (hipStream_t)stream, true);
}

int mtnlg_layer_bwd(const mtnlg_layer_desc *desc, const mtnlg_layer_weights *w, const void *x,
                    const void *saved, const void *dy, void *dx, const mtnlg_layer_grads *grads,
                    void *workspace, size_t workspace_bytes, mtnlg_reduce_fn reduce, void *user,
                    void *stream) {
  Shape S;
  MTNLG_TRY(make_shape(desc, &S));
  if (!weights_ok(w) || !grads_ok(grads) || !x || !saved || !dy || !dx || !workspace) return MTNLG_NULL_POINTER;
  if (dx == dy) return MTNLG_INVALID_ARG;
  if (workspace_bytes < mtnlg_workspace_bytes(desc)) return MTNLG_WORKSPACE_TOO_SMALL;
  return layer_bwd_impl(S, w, x, saved, dy, dx, grads, workspace, reduce, user, (hipStream_t)stream);
}

int mtnlg_stage_step(const mtnlg_layer_desc *desc, int n_layers, const mtnlg_layer_weights *w,
                     const void *x_in, const void *dy_out, void *y_out, void *dx_in,
                     const mtnlg_layer_grads *grads, void *saved, size_t saved_bytes, void *workspace,
                     size_t workspace_bytes, mtnlg_reduce_fn reduce, void *user, void *stream) {
  Shape S;
  MTNLG_TRY(make_shape(desc, &S));
  if (n_layers <= 0) return MTNLG_INVALID_ARG;
  if (!w || !grads || !x_in || !dy_out || !y_out || !dx_in || !saved || !workspace) return MTNLG_NULL_POINTER;
  for (int l = 0; l < n_layers; ++l)
    if (!weights_ok(&w[l]) || !grads_ok(&grads[l])) return MTNLG_NULL_POINTER;
  if (x_in == y_out || dy_out == dx_in) return MTNLG_INVALID_ARG;
  if (workspace_bytes < mtnlg_workspace_bytes(desc)) return MTNLG_WORKSPACE_TOO_SMALL;
  if (saved_bytes < mtnlg_stage_saved_bytes(desc, n_layers)) return MTNLG_WORKSPACE_TOO_SMALL;
  hipStream_t st = (hipStream_t)stream;
  const bool recompute = (desc->flags & MTNLG_RECOMPUTE) != 0;
  mtnlg_saved_layout L;
  saved_layout(S, &L);
  Work W;
  work_layout(S, &W);
  const size_t slot = align_up(S.T * S.h * S.es, 256);
  char *blocks = at(saved, (size_t)n_layers * slot);
  auto layer_in = [&](int l) -> const void * { return l == 0 ? x_in : at(saved, (size_t)(l - 1) * slot); };
  auto layer_block = [&](int l) -> void * { return blocks + (recompute ? 0 : (size_t)l * L.total); };

  for (int l = 0; l < n_layers; ++l) {
    void *out = l == n_layers - 1 ? y_out : at(saved, (size_t)l * slot);
    MTNLG_TRY(layer_fwd_impl(S, &w[l], layer_in(l), out, layer_block(l), workspace, reduce, user, st, true));
  }
  const void *gin = dy_out;
  for (int l = n_layers - 1; l >= 0; --l) {
    // the last layer's activations are still in the shared block after the forward sweep
    if (recompute && l != n_layers - 1)
      MTNLG_TRY(layer_fwd_impl(S, &w[l], layer_in(l), nullptr, layer_block(l), workspace, reduce, user, st, false));
    void *gout = l == 0 ? dx_in : at(workspace, ((n_layers - 1 - l) & 1) ? W.pong : W.ping);
    MTNLG_TRY(layer_bwd_impl(S, &w[l], layer_in(l), layer_block(l), gin, gout, &grads[l], workspace, reduce,
                             user, st));
    gin = gout;
  }
  return MTNLG_OK;
}

int mtnlg_stage_step_accumulate(const mtnlg_layer_desc *desc, int n_layers, const mtnlg_layer_weights *w,
                                int n_micro, const void *x_in, const void *dy_out, void *y_out, void *dx_in,
                                const mtnlg_layer_grads *grads, void *saved, size_t saved_bytes, void *workspace,
                                size_t workspace_bytes, mtnlg_reduce_fn reduce, void *user, void *stream) {
  Shape S;
  MTNLG_TRY(make_shape(desc, &S));
  if (n_micro <= 0) return MTNLG_INVALID_ARG;
  if (!x_in || !dy_out || !y_out || !dx_in) return MTNLG_NULL_POINTER;
  const size_t stride = (size_t)(S.T * S.h * S.es);   // one micro-batch of [T,h]
  mtnlg_layer_desc d = *desc;
  for (int m = 0; m < n_micro; ++m) {
    if (m == 1) d.flags |= MTNLG_ACCUMULATE_WGRAD;
    MTNLG_TRY(mtnlg_stage_step(&d, n_layers, w, at(x_in, m * stride), at(dy_out, m * stride), at(y_out, m * stride),
                               at(dx_in, m * stride), grads, saved, saved_bytes, workspace, workspace_bytes, reduce,
                               user, stream));
  }
  return MTNLG_OK;
}

size_t mtnlg_gemm_workspace(int dtype, int layout, int64_t M, int64_t N, int64_t K) {
  if (layout < 0 || layout > 2) return 0;
  return dtype == MTNLG_BF16 ? gemm_mfma_workspace_bytes(layout, M, N, K) : 0;
}

int mtnlg_gemm(int dtype, int layout, int64_t M, int64_t N, int64_t K, const void *A, const void *B, void *C,
               const void *bias, void *aux, uint32_t epilogue, void *workspace, size_t workspace_bytes,
               void *stream) {
  if (!A || !B || !C) return MTNLG_NULL_POINTER;
  if (M <= 0 || N <= 0 || K <= 0 || layout < 0 || layout > 2) return MTNLG_INVALID_ARG;
  if (dtype != MTNLG_F32 && dtype != MTNLG_BF16) return MTNLG_INVALID_ARG;
  if ((epilogue & MTNLG_EPI_BIAS) && !bias) return MTNLG_NULL_POINTER;
  if (epilogue & ~(MTNLG_EPI_BIAS | MTNLG_EPI_GELU | MTNLG_EPI_RESIDUAL | MTNLG_EPI_ACCUMULATE | MTNLG_EPI_OUT_F32 |
                   MTNLG_EPI_GELU_ERF | MTNLG_EPI_GELU_GRAD))
    return MTNLG_INVALID_ARG;
  if ((epilogue & (MTNLG_EPI_GELU | MTNLG_EPI_RESIDUAL | MTNLG_EPI_GELU_GRAD)) && !aux) return MTNLG_NULL_POINTER;
  if ((epilogue & MTNLG_EPI_GELU) && (epilogue & (MTNLG_EPI_RESIDUAL | MTNLG_EPI_ACCUMULATE | MTNLG_EPI_OUT_F32)))
    return MTNLG_INVALID_ARG;
  if ((epilogue & MTNLG_EPI_GELU_GRAD) &&
      (epilogue & (MTNLG_EPI_GELU | MTNLG_EPI_RESIDUAL | MTNLG_EPI_ACCUMULATE | MTNLG_EPI_BIAS)))
    return MTNLG_INVALID_ARG;
  if (dtype == MTNLG_F32) epilogue &= ~MTNLG_EPI_OUT_F32;
  hipStream_t st = (hipStream_t)stream;
  if (dtype == MTNLG_BF16) {
    int r = gemm_mfma_bf16(layout, M, N, K, A, B, C, bias, aux, epilogue, workspace, workspace_bytes, st);
    if (r != MTNLG_UNSUPPORTED_SHAPE) return r;
  }
  return gemm_generic(dtype, layout, M, N, K, A, B, C, bias, aux, epilogue, st);
}

int mtnlg_attention_fwd(int dtype, int32_t b, int32_t s, int32_t n, int32_t d, float scale, const void *qkv,
                        void *a, float *lse, void *stream) {
  if (!qkv || !a || !lse) return MTNLG_NULL_POINTER;
  if (b <= 0 || s <= 0 || n <= 0 || d <= 0 || !(scale > 0.0f)) return MTNLG_INVALID_ARG;
  if (attention_mfma_takes(dtype, b, s, n, d))
    return attention_fwd_mfma(b, s, n, d, scale, qkv, a, lse, (hipStream_t)stream);
  return attention_fwd_simple(dtype, b, s, n, d, scale, qkv, a, lse, (hipStream_t)stream);
}

size_t mtnlg_attention_bwd_workspace(int32_t b, int32_t s, int32_t n, int32_t d) {
  if (b <= 0 || s <= 0 || n <= 0 || d <= 0) return 0;
  return attention_bwd_workspace_bytes(b, s, n, d);
}

int mtnlg_attention_bwd(int dtype, int32_t b, int32_t s, int32_t n, int32_t d, float scale, const void *qkv,
                        const void *a, const float *lse, const void *da, void *dqkv, void *workspace,
                        void *stream) {
  if (!qkv || !a || !lse || !da || !dqkv || !workspace) return MTNLG_NULL_POINTER;
  if (b <= 0 || s <= 0 || n <= 0 || d <= 0 || !(scale > 0.0f)) return MTNLG_INVALID_ARG;
  if (attention_mfma_takes(dtype, b, s, n, d))
    return attention_bwd_mfma(b, s, n, d, scale, qkv, a, lse, da, dqkv, workspace, (hipStream_t)stream);
  return attention_bwd_simple(dtype, b, s, n, d, scale, qkv, a, lse, da, dqkv, workspace, (hipStream_t)stream);
}

}  // extern "C"
