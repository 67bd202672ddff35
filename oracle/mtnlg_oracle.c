/*
 * mtnlg_oracle.c -- TEST INFRASTRUCTURE, not product code.
 *
 * Plain, slow, fp64 CPU definition of what one tensor-parallel slice of a
 * pre-LayerNorm GPT decoder layer computes, forward and backward.  Only the
 * test-suite, the smoke check and the cpu_baseline leg of the benchmark may
 * call into this file; the GPU library shares no code with it.
 *
 * What the paper fixes (Section 3.2, "Model and Training Process"): a GPT-2
 * style left-to-right transformer decoder; 105 layers, hidden 20480, 128
 * heads, sequence 2048, 8-way tensor slicing.  Section 2.1 ("Tensor Model
 * Parallelism") fixes the slicing: each layer is partitioned across the
 * workers and activations are exchanged (summed) once per block per pass.
 * The paper prints no layer equations; the block below is the GPT-2 decoder
 * layer under the readings listed in the design notes of this repository
 * (pre-LN, biased variance, eps inside the square root, tanh-GeLU unless
 * gelu_exact, softmax scale 1/sqrt(d), causal mask with the diagonal kept,
 * all four linears biased, no dropout).
 *
 *   u1  = LN(x; g1, b1)
 *   qkv = u1 Wqkv^T + bqkv          columns ordered [head][q|k|v][d]
 *   P_j = rowsoftmax(mask(q_j k_j^T * scale)),  a_j = P_j v_j
 *   A_r = concat_j(a_j) Wo^T        (partial sum of the row-parallel linear)
 *   x1  = x + reduce(A_r) + bo
 *   u2  = LN(x1; g2, b2);  z = u2 W1^T + bfc1;  g = GeLU(z)
 *   M_r = g W2^T;          y = x1 + reduce(M_r) + bfc2
 *
 * Backward is the analytic adjoint, written step by step below.  Every loop
 * is the definition itself: no tiling, no fusion, no reassociation other than
 * what "#pragma omp simd reduction" allows inside a single dot product.
 *
 * Pins (tests/test_oracle_*.py): central finite differences of every gradient,
 * agreement with an independent autograd composition of library ops, softmax /
 * LayerNorm / causal invariants, textbook special cases, the TP-sum identity,
 * and the paper's closed forms (parameter count, activation bytes, init std).
 */
#include <math.h>
#include <omp.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
  int32_t hidden;      /* h */
  int32_t heads;       /* n  (local heads of this slice) */
  int32_t head_dim;    /* d */
  int32_t ffn;         /* F  (local FFN width of this slice) */
  int32_t seq;         /* s */
  int32_t batch;       /* b */
  int32_t gelu_exact;  /* 0: tanh form, 1: erf form */
  int32_t pad_;
  double ln_eps;
  double softmax_scale; /* <= 0 means 1/sqrt(d) */
} orc_dims;

typedef struct {
  const double *ln1_g, *ln1_b, *w_qkv, *b_qkv, *w_o, *b_o;
  const double *ln2_g, *ln2_b, *w_fc1, *b_fc1, *w_fc2, *b_fc2;
} orc_weights;

typedef struct {
  double *ln1_g, *ln1_b, *w_qkv, *b_qkv, *w_o, *b_o;
  double *ln2_g, *ln2_b, *w_fc1, *b_fc1, *w_fc2, *b_fc2;
} orc_grads;

/* Everything the forward pass produces on the way; caller allocates.
 *   u1,x1,u2 : [T,h]   mu1,rs1,mu2,rs2 : [T]   qkv : [T,3p]   a : [T,p]
 *   z,g : [T,F]        A_r, M_r : [T,h] (partials before the reduce point)  */
typedef struct {
  double *u1, *mu1, *rs1, *qkv, *a, *A_r, *x1, *u2, *mu2, *rs2, *z, *g, *M_r;
} orc_saved;

/* Sum across tensor-parallel ranks at a reduce point; NULL means a group of one. */
typedef void (*orc_reduce_fn)(double *buf, size_t count, void *user);

/* ------------------------------------------------------------------ */
/* GeLU (reading: GPT-2's tanh form by default, erf form on request)   */
/* ------------------------------------------------------------------ */
static const double kSqrt2OverPi = 0.79788456080286535587989211986876;
static const double kGeluC = 0.044715;

double orc_gelu(double z, int exact) {
  if (exact) return 0.5 * z * (1.0 + erf(z * 0.70710678118654752440));
  return 0.5 * z * (1.0 + tanh(kSqrt2OverPi * (z + kGeluC * z * z * z)));
}

double orc_gelu_grad(double z, int exact) {
  if (exact) {
    double cdf = 0.5 * (1.0 + erf(z * 0.70710678118654752440));
    double pdf = exp(-0.5 * z * z) * 0.39894228040143267793994605993438;
    return cdf + z * pdf;
  }
  double inner = kSqrt2OverPi * (z + kGeluC * z * z * z);
  double th = tanh(inner);
  double dinner = kSqrt2OverPi * (1.0 + 3.0 * kGeluC * z * z);
  return 0.5 * (1.0 + th) + 0.5 * z * (1.0 - th * th) * dinner;
}

/* ------------------------------------------------------------------ */
/* LayerNorm over the last axis, per token row                         */
/* ------------------------------------------------------------------ */
void orc_layernorm_fwd(const double *x, const double *gamma, const double *beta,
                       int64_t T, int64_t h, double eps, double *out,
                       double *mean, double *rstd) {
#pragma omp parallel for schedule(static)
  for (int64_t t = 0; t < T; ++t) {
    const double *row = x + t * h;
    double mu = 0.0;
    for (int64_t i = 0; i < h; ++i) mu += row[i];
    mu /= (double)h;
    double var = 0.0;
    for (int64_t i = 0; i < h; ++i) var += (row[i] - mu) * (row[i] - mu);
    var /= (double)h; /* biased variance */
    double rs = 1.0 / sqrt(var + eps);
    for (int64_t i = 0; i < h; ++i)
      out[t * h + i] = gamma[i] * (row[i] - mu) * rs + beta[i];
    if (mean) mean[t] = mu;
    if (rstd) rstd[t] = rs;
  }
}

/* Adjoint of LayerNorm.  With xhat = (x-mu)*rs and dxhat = dout*gamma:
 *   dx = rs * (dxhat - mean(dxhat) - xhat * mean(dxhat*xhat))
 *   dgamma = sum_t dout*xhat,  dbeta = sum_t dout                        */
void orc_layernorm_bwd(const double *x, const double *gamma, const double *mean,
                       const double *rstd, const double *dout, int64_t T,
                       int64_t h, double *dx, double *dgamma, double *dbeta) {
#pragma omp parallel for schedule(static)
  for (int64_t t = 0; t < T; ++t) {
    const double *row = x + t * h;
    const double *dr = dout + t * h;
    double mu = mean[t], rs = rstd[t];
    double m1 = 0.0, m2 = 0.0;
    for (int64_t i = 0; i < h; ++i) {
      double xhat = (row[i] - mu) * rs;
      double dxh = dr[i] * gamma[i];
      m1 += dxh;
      m2 += dxh * xhat;
    }
    m1 /= (double)h;
    m2 /= (double)h;
    for (int64_t i = 0; i < h; ++i) {
      double xhat = (row[i] - mu) * rs;
      double dxh = dr[i] * gamma[i];
      dx[t * h + i] = rs * (dxh - m1 - xhat * m2);
    }
  }
  if (dgamma || dbeta) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < h; ++i) {
      double sg = 0.0, sb = 0.0;
      for (int64_t t = 0; t < T; ++t) {
        double xhat = (x[t * h + i] - mean[t]) * rstd[t];
        sg += dout[t * h + i] * xhat;
        sb += dout[t * h + i];
      }
      if (dgamma) dgamma[i] = sg;
      if (dbeta) dbeta[i] = sb;
    }
  }
}

/* ------------------------------------------------------------------ */
/* Linear layers: out[t,n] = sum_k x[t,k] W[n,k] (+ bias[n])           */
/* ------------------------------------------------------------------ */
void orc_linear_fwd(const double *x, const double *W, const double *bias,
                    int64_t T, int64_t N, int64_t K, double *out) {
#pragma omp parallel for schedule(static)
  for (int64_t t = 0; t < T; ++t) {
    for (int64_t n = 0; n < N; ++n) {
      const double *xr = x + t * K, *wr = W + n * K;
      double acc = 0.0;
#pragma omp simd reduction(+ : acc)
      for (int64_t k = 0; k < K; ++k) acc += xr[k] * wr[k];
      out[t * N + n] = acc + (bias ? bias[n] : 0.0);
    }
  }
}

/* dx[t,k] = sum_n dout[t,n] W[n,k] */
void orc_linear_dgrad(const double *dout, const double *W, int64_t T, int64_t N,
                      int64_t K, double *dx) {
#pragma omp parallel for schedule(static)
  for (int64_t t = 0; t < T; ++t) {
    double *dr = dx + t * K;
    for (int64_t k = 0; k < K; ++k) dr[k] = 0.0;
    for (int64_t n = 0; n < N; ++n) {
      double go = dout[t * N + n];
      const double *wr = W + n * K;
#pragma omp simd
      for (int64_t k = 0; k < K; ++k) dr[k] += go * wr[k];
    }
  }
}

/* dW[n,k] = sum_t dout[t,n] x[t,k];  db[n] = sum_t dout[t,n] */
void orc_linear_wgrad(const double *dout, const double *x, int64_t T, int64_t N,
                      int64_t K, double *dW, double *db) {
#pragma omp parallel for schedule(static)
  for (int64_t n = 0; n < N; ++n) {
    double *wr = dW + n * K;
    for (int64_t k = 0; k < K; ++k) wr[k] = 0.0;
    double sb = 0.0;
    for (int64_t t = 0; t < T; ++t) {
      double go = dout[t * N + n];
      const double *xr = x + t * K;
      sb += go;
#pragma omp simd
      for (int64_t k = 0; k < K; ++k) wr[k] += go * xr[k];
    }
    if (db) db[n] = sb;
  }
}

/* ------------------------------------------------------------------ */
/* Causal softmax attention over the local heads                       */
/* qkv: [b*s, n*3*d], column (j, c, e) at j*3d + c*d + e, c in {q,k,v}  */
/* ------------------------------------------------------------------ */
static double eff_scale(const orc_dims *D) {
  return D->softmax_scale > 0.0 ? D->softmax_scale : 1.0 / sqrt((double)D->head_dim);
}

/* One row of P for query t of (batch bi, head j): P[0..t], entries above the
 * diagonal are zero by the mask and are not stored. */
static void softmax_row(const orc_dims *D, const double *qkv, int64_t bi, int64_t j,
                        int64_t t, double *P) {
  const int64_t d = D->head_dim, s = D->seq, ld = (int64_t)D->heads * 3 * d;
  const double sc = eff_scale(D);
  const double *q = qkv + (bi * s + t) * ld + j * 3 * d;
  double mx = -INFINITY;
  for (int64_t u = 0; u <= t; ++u) {
    const double *k = qkv + (bi * s + u) * ld + j * 3 * d + d;
    double acc = 0.0;
    for (int64_t e = 0; e < d; ++e) acc += q[e] * k[e];
    P[u] = acc * sc;
    if (P[u] > mx) mx = P[u];
  }
  double den = 0.0;
  for (int64_t u = 0; u <= t; ++u) {
    P[u] = exp(P[u] - mx);
    den += P[u];
  }
  for (int64_t u = 0; u <= t; ++u) P[u] /= den;
}

/* a[t, j*d + e] = sum_{u<=t} P_j[t,u] v_j[u,e].  If P_out is non-NULL it
 * receives the dense [b, n, s, s] probabilities (zeros above the diagonal). */
void orc_attention_fwd(const orc_dims *D, const double *qkv, double *a, double *P_out) {
  const int64_t d = D->head_dim, s = D->seq, n = D->heads, b = D->batch;
  const int64_t ld = n * 3 * d, p = n * d;
#pragma omp parallel
  {
    double *P = (double *)malloc((size_t)s * sizeof(double));
#pragma omp for collapse(2) schedule(dynamic, 8)
    for (int64_t bj = 0; bj < b * n; ++bj) {
      for (int64_t t = 0; t < s; ++t) {
        int64_t bi = bj / n, j = bj % n;
        softmax_row(D, qkv, bi, j, t, P);
        double *ar = a + (bi * s + t) * p + j * d;
        for (int64_t e = 0; e < d; ++e) ar[e] = 0.0;
        for (int64_t u = 0; u <= t; ++u) {
          const double *v = qkv + (bi * s + u) * ld + j * 3 * d + 2 * d;
          for (int64_t e = 0; e < d; ++e) ar[e] += P[u] * v[e];
        }
        if (P_out) {
          double *po = P_out + ((bi * n + j) * s + t) * s;
          for (int64_t u = 0; u < s; ++u) po[u] = (u <= t) ? P[u] : 0.0;
        }
      }
    }
    free(P);
  }
}

/* Adjoint of attention for one (batch, head) at a time:
 *   dv = P^T da;  dP = da v^T;  dS = P o (dP - rowsum(dP o P));
 *   dq = scale * dS k;  dk = scale * dS^T q.                              */
void orc_attention_bwd(const orc_dims *D, const double *qkv, const double *da,
                       double *dqkv) {
  const int64_t d = D->head_dim, s = D->seq, n = D->heads, b = D->batch;
  const int64_t ld = n * 3 * d, p = n * d;
  const double sc = eff_scale(D);
  memset(dqkv, 0, (size_t)(b * s * ld) * sizeof(double));
#pragma omp parallel
  {
    double *P = (double *)malloc((size_t)s * sizeof(double));
    double *dP = (double *)malloc((size_t)s * sizeof(double));
    /* one (batch, head) per thread at a time: its dk/dv rows are touched by
     * every query row, so rows of one head are not split across threads */
#pragma omp for schedule(dynamic, 1)
    for (int64_t bj = 0; bj < b * n; ++bj) {
      int64_t bi = bj / n, j = bj % n;
      for (int64_t t = 0; t < s; ++t) {
        softmax_row(D, qkv, bi, j, t, P);
        const double *dar = da + (bi * s + t) * p + j * d;
        const double *q = qkv + (bi * s + t) * ld + j * 3 * d;
        double *dq = dqkv + (bi * s + t) * ld + j * 3 * d;
        double dot = 0.0;
        for (int64_t u = 0; u <= t; ++u) {
          const double *v = qkv + (bi * s + u) * ld + j * 3 * d + 2 * d;
          double acc = 0.0;
          for (int64_t e = 0; e < d; ++e) acc += dar[e] * v[e];
          dP[u] = acc;
          dot += acc * P[u];
        }
        for (int64_t u = 0; u <= t; ++u) {
          const double *k = qkv + (bi * s + u) * ld + j * 3 * d + d;
          double *dk = dqkv + (bi * s + u) * ld + j * 3 * d + d;
          double *dv = dqkv + (bi * s + u) * ld + j * 3 * d + 2 * d;
          double dS = P[u] * (dP[u] - dot);
          for (int64_t e = 0; e < d; ++e) {
            dv[e] += P[u] * dar[e];
            dq[e] += sc * dS * k[e];
            dk[e] += sc * dS * q[e];
          }
        }
      }
    }
    free(P);
    free(dP);
  }
}

/* ------------------------------------------------------------------ */
/* The two halves of the layer, each ending in a row-parallel partial  */
/* ------------------------------------------------------------------ */
static int64_t tokens(const orc_dims *D) { return (int64_t)D->batch * D->seq; }

/* LN1 -> QKV -> attention -> projection without bias: A_r */
void orc_attn_half_fwd(const orc_dims *D, const orc_weights *W, const double *x,
                       orc_saved *S) {
  const int64_t T = tokens(D), h = D->hidden, p = (int64_t)D->heads * D->head_dim;
  orc_layernorm_fwd(x, W->ln1_g, W->ln1_b, T, h, D->ln_eps, S->u1, S->mu1, S->rs1);
  orc_linear_fwd(S->u1, W->w_qkv, W->b_qkv, T, 3 * p, h, S->qkv);
  orc_attention_fwd(D, S->qkv, S->a, NULL);
  orc_linear_fwd(S->a, W->w_o, NULL, T, h, p, S->A_r);
}

/* LN2 -> FC1 + bias -> GeLU -> FC2 without bias: M_r */
void orc_mlp_half_fwd(const orc_dims *D, const orc_weights *W, orc_saved *S) {
  const int64_t T = tokens(D), h = D->hidden, F = D->ffn;
  orc_layernorm_fwd(S->x1, W->ln2_g, W->ln2_b, T, h, D->ln_eps, S->u2, S->mu2, S->rs2);
  orc_linear_fwd(S->u2, W->w_fc1, W->b_fc1, T, F, h, S->z);
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < T * F; ++i) S->g[i] = orc_gelu(S->z[i], D->gelu_exact);
  orc_linear_fwd(S->g, W->w_fc2, NULL, T, h, F, S->M_r);
}

void orc_layer_fwd(const orc_dims *D, const orc_weights *W, const double *x,
                   double *y, orc_saved *S, orc_reduce_fn reduce, void *user) {
  const int64_t T = tokens(D), h = D->hidden;
  orc_attn_half_fwd(D, W, x, S);
  if (reduce) reduce(S->A_r, (size_t)(T * h), user);
  for (int64_t t = 0; t < T; ++t)
    for (int64_t i = 0; i < h; ++i)
      S->x1[t * h + i] = x[t * h + i] + S->A_r[t * h + i] + W->b_o[i];
  orc_mlp_half_fwd(D, W, S);
  if (reduce) reduce(S->M_r, (size_t)(T * h), user);
  for (int64_t t = 0; t < T; ++t)
    for (int64_t i = 0; i < h; ++i)
      y[t * h + i] = S->x1[t * h + i] + S->M_r[t * h + i] + W->b_fc2[i];
}

/* MLP half backward: given dy (grad of y), produce the partial du2_r and the
 * grads of W2, W1, b1.  (b2's grad and the residual path are the caller's.) */
void orc_mlp_half_bwd(const orc_dims *D, const orc_weights *W, const orc_saved *S,
                      const double *dy, double *du2_r, orc_grads *G) {
  const int64_t T = tokens(D), h = D->hidden, F = D->ffn;
  double *dg = (double *)malloc((size_t)(T * F) * sizeof(double));
  orc_linear_dgrad(dy, W->w_fc2, T, h, F, dg);             /* dg = dy W2      */
  orc_linear_wgrad(dy, S->g, T, h, F, G->w_fc2, NULL);     /* dW2 = dy^T g    */
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < T * F; ++i)                      /* dz = dg o GeLU' */
    dg[i] *= orc_gelu_grad(S->z[i], D->gelu_exact);
  orc_linear_wgrad(dg, S->u2, T, F, h, G->w_fc1, G->b_fc1);/* dW1, db1        */
  orc_linear_dgrad(dg, W->w_fc1, T, F, h, du2_r);          /* du2_r = dz W1   */
  free(dg);
}

/* Attention half backward: given dx1 (grad of x1 through the A branch, i.e. the
 * grad of A), produce partial du1_r and grads of Wo, Wqkv, bqkv. */
void orc_attn_half_bwd(const orc_dims *D, const orc_weights *W, const orc_saved *S,
                       const double *dA, double *du1_r, orc_grads *G) {
  const int64_t T = tokens(D), h = D->hidden, p = (int64_t)D->heads * D->head_dim;
  double *da = (double *)malloc((size_t)(T * p) * sizeof(double));
  double *dqkv = (double *)malloc((size_t)(T * 3 * p) * sizeof(double));
  orc_linear_dgrad(dA, W->w_o, T, h, p, da);               /* da = dA Wo      */
  orc_linear_wgrad(dA, S->a, T, h, p, G->w_o, NULL);       /* dWo = dA^T a    */
  orc_attention_bwd(D, S->qkv, da, dqkv);
  orc_linear_wgrad(dqkv, S->u1, T, 3 * p, h, G->w_qkv, G->b_qkv);
  orc_linear_dgrad(dqkv, W->w_qkv, T, 3 * p, h, du1_r);    /* du1_r = dqkv Wqkv */
  free(da);
  free(dqkv);
}

void orc_layer_bwd(const orc_dims *D, const orc_weights *W, const double *x,
                   const orc_saved *S, const double *dy, double *dx, orc_grads *G,
                   orc_reduce_fn reduce, void *user) {
  const int64_t T = tokens(D), h = D->hidden;
  double *du = (double *)malloc((size_t)(T * h) * sizeof(double));
  double *dx1 = (double *)malloc((size_t)(T * h) * sizeof(double));
  double *tmp = (double *)malloc((size_t)(T * h) * sizeof(double));

  /* y = x1 + M + b2 */
  for (int64_t i = 0; i < h; ++i) {
    double sb = 0.0;
    for (int64_t t = 0; t < T; ++t) sb += dy[t * h + i];
    G->b_fc2[i] = sb;
  }
  orc_mlp_half_bwd(D, W, S, dy, du, G);
  if (reduce) reduce(du, (size_t)(T * h), user);
  orc_layernorm_bwd(S->x1, W->ln2_g, S->mu2, S->rs2, du, T, h, tmp, G->ln2_g, G->ln2_b);
  for (int64_t i = 0; i < T * h; ++i) dx1[i] = dy[i] + tmp[i];

  /* x1 = x + A + bo */
  for (int64_t i = 0; i < h; ++i) {
    double sb = 0.0;
    for (int64_t t = 0; t < T; ++t) sb += dx1[t * h + i];
    G->b_o[i] = sb;
  }
  orc_attn_half_bwd(D, W, S, dx1, du, G);
  if (reduce) reduce(du, (size_t)(T * h), user);
  orc_layernorm_bwd(x, W->ln1_g, S->mu1, S->rs1, du, T, h, tmp, G->ln1_g, G->ln1_b);
  for (int64_t i = 0; i < T * h; ++i) dx[i] = dx1[i] + tmp[i];

  free(du);
  free(dx1);
  free(tmp);
}

int orc_abi_version(void) { return 1; }

/* Threads the parallel loops above will use (for reporting next to timings). */
int orc_num_threads(void) { return omp_get_max_threads(); }
