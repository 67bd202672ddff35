/*
 * sanitize_main.c -- TEST INFRASTRUCTURE: the fp64 oracle compiled together with this driver under
 * AddressSanitizer and UndefinedBehaviorSanitizer (tests/test_oracle_sanitizers.py builds and runs it).
 *
 * Every buffer is a heap block of exactly the size the oracle's interface states, so an index that leaves a
 * tensor is reported.  The run covers ragged shapes, both GeLU forms, the reduce hook, and re-checks a few
 * pins in C so that the instrumented code is known to compute the same function: softmax rows sum to one and
 * are zero above the diagonal, zero weights leave y = x + b_o + b_fc2, and central finite differences of the
 * scalar loss sum(y o dy) agree with the analytic dx and with entries of every parameter gradient.
 */
#include <stdio.h>

#include "mtnlg_oracle.c"

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static double rnd(void) { /* uniform in (-1, 1): splitmix64 */
  uint64_t z = (rng_state += 0x9E3779B97F4A7C15ull);
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  z ^= z >> 31;
  return (double)(z >> 11) / 4503599627370496.0 - 1.0;
}
static double *block(int64_t n, double scale, double shift) {
  double *p = (double *)malloc((size_t)n * sizeof(double));
  if (!p) { fprintf(stderr, "out of memory\n"); exit(2); }
  for (int64_t i = 0; i < n; ++i) p[i] = shift + scale * rnd();
  return p;
}
static int failures = 0;
#define CHECK(cond, ...) do { if (!(cond)) { fprintf(stderr, "FAIL: " __VA_ARGS__); fprintf(stderr, "\n"); ++failures; } } while (0)

typedef struct { double *p[12]; int64_t n[12]; } params;
static const char *NAMES[12] = {"ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o", "ln2_g", "ln2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2"};

static params make_params(const orc_dims *D, double wscale, int zero) {
  const int64_t h = D->hidden, p = (int64_t)D->heads * D->head_dim, F = D->ffn;
  const int64_t n[12] = {h, h, 3 * p * h, 3 * p, h * p, h, h, h, F * h, F, h * F, h};
  params P;
  for (int i = 0; i < 12; ++i) {
    P.n[i] = n[i];
    const int is_gain = (i == 0 || i == 6), is_matrix = (i == 2 || i == 4 || i == 8 || i == 10);
    P.p[i] = block(n[i], zero && is_matrix ? 0.0 : (is_matrix ? wscale : 0.3), is_gain ? 1.0 : 0.0);
  }
  return P;
}
static void free_params(params *P) { for (int i = 0; i < 12; ++i) free(P->p[i]); }
static orc_weights as_weights(const params *P) {
  orc_weights W = {P->p[0], P->p[1], P->p[2], P->p[3], P->p[4], P->p[5], P->p[6], P->p[7], P->p[8], P->p[9], P->p[10], P->p[11]};
  return W;
}
static orc_grads as_grads(params *P) {
  orc_grads G = {P->p[0], P->p[1], P->p[2], P->p[3], P->p[4], P->p[5], P->p[6], P->p[7], P->p[8], P->p[9], P->p[10], P->p[11]};
  return G;
}
static orc_saved make_saved(const orc_dims *D) {
  const int64_t T = (int64_t)D->batch * D->seq, h = D->hidden, p = (int64_t)D->heads * D->head_dim, F = D->ffn;
  orc_saved S = {block(T * h, 0, 0), block(T, 0, 0), block(T, 0, 0), block(T * 3 * p, 0, 0), block(T * p, 0, 0),
                 block(T * h, 0, 0), block(T * h, 0, 0), block(T * h, 0, 0), block(T, 0, 0), block(T, 0, 0),
                 block(T * F, 0, 0), block(T * F, 0, 0), block(T * h, 0, 0)};
  return S;
}
static void free_saved(orc_saved *S) {
  double *all[13] = {S->u1, S->mu1, S->rs1, S->qkv, S->a, S->A_r, S->x1, S->u2, S->mu2, S->rs2, S->z, S->g, S->M_r};
  for (int i = 0; i < 13; ++i) free(all[i]);
}

static int hook_calls = 0;
static void counting_hook(double *buf, size_t count, void *user) { (void)buf; (void)user; hook_calls += count > 0; }

static double loss(const orc_dims *D, const orc_weights *W, const double *x, const double *dy) {
  const int64_t T = (int64_t)D->batch * D->seq, h = D->hidden;
  orc_saved S = make_saved(D);
  double *y = block(T * h, 0, 0), l = 0.0;
  orc_layer_fwd(D, W, x, y, &S, NULL, NULL);
  for (int64_t i = 0; i < T * h; ++i) l += y[i] * dy[i];
  free(y);
  free_saved(&S);
  return l;
}

static void run_case(int h, int n, int d, int F, int s, int b, int gelu_exact) {
  orc_dims D = {h, n, d, F, s, b, gelu_exact, 0, 1e-5, 0.0};
  const int64_t T = (int64_t)b * s, p = (int64_t)n * d;
  params P = make_params(&D, 0.4, 0);
  orc_weights W = as_weights(&P);
  double *x = block(T * h, 1.0, 0.0), *dy = block(T * h, 1.0, 0.0), *y = block(T * h, 0, 0), *dx = block(T * h, 0, 0);
  orc_saved S = make_saved(&D);
  hook_calls = 0;
  orc_layer_fwd(&D, &W, x, y, &S, counting_hook, NULL);
  params GP = make_params(&D, 0.0, 0);
  orc_grads G = as_grads(&GP);
  orc_layer_bwd(&D, &W, x, &S, dy, dx, &G, counting_hook, NULL);
  CHECK(hook_calls == 4, "the reduce hook is called at four points, saw %d", hook_calls);

  /* softmax rows */
  double *Pm = block((int64_t)b * n * s * s, 0, 0), *a = block(T * p, 0, 0);
  orc_attention_fwd(&D, S.qkv, a, Pm);
  for (int64_t r = 0; r < (int64_t)b * n * s; ++r) {
    double sum = 0.0;
    const int64_t t = r % s;
    for (int64_t u = 0; u < s; ++u) {
      sum += Pm[r * s + u];
      if (u > t) CHECK(Pm[r * s + u] == 0.0, "probability above the diagonal (row %ld col %ld)", (long)r, (long)u);
    }
    CHECK(fabs(sum - 1.0) < 1e-13, "softmax row %ld sums to %.17g", (long)r, sum);
  }
  free(Pm);
  free(a);

  /* central finite differences of sum(y o dy): a few entries of x and of every parameter tensor */
  const double eps = 1e-5;
  for (int k = 0; k < 3; ++k) {
    const int64_t i = ((int64_t)(fabs(rnd()) * (double)(T * h))) % (T * h);
    const double keep = x[i];
    x[i] = keep + eps; const double lp = loss(&D, &W, x, dy);
    x[i] = keep - eps; const double lm = loss(&D, &W, x, dy);
    x[i] = keep;
    const double fd = (lp - lm) / (2 * eps);
    CHECK(fabs(fd - dx[i]) <= 1e-6 * (1.0 + fabs(fd)), "dx[%ld]: analytic %.12g, differences %.12g", (long)i, dx[i], fd);
  }
  for (int t = 0; t < 12; ++t) {
    const int64_t i = ((int64_t)(fabs(rnd()) * (double)P.n[t])) % P.n[t];
    const double keep = P.p[t][i];
    P.p[t][i] = keep + eps; const double lp = loss(&D, &W, x, dy);
    P.p[t][i] = keep - eps; const double lm = loss(&D, &W, x, dy);
    P.p[t][i] = keep;
    const double fd = (lp - lm) / (2 * eps);
    CHECK(fabs(fd - GP.p[t][i]) <= 1e-6 * (1.0 + fabs(fd)), "d%s[%ld]: analytic %.12g, differences %.12g", NAMES[t], (long)i, GP.p[t][i], fd);
  }

  /* zero matrices: y = x + b_o + b_fc2 */
  params Z = make_params(&D, 0.0, 1);
  orc_weights WZ = as_weights(&Z);
  orc_layer_fwd(&D, &WZ, x, y, &S, NULL, NULL);
  for (int64_t t = 0; t < T; ++t)
    for (int64_t i = 0; i < h; ++i)
      CHECK(fabs(y[t * h + i] - (x[t * h + i] + Z.p[5][i] + Z.p[11][i])) < 1e-14, "residual identity at (%ld, %ld)", (long)t, (long)i);
  free_params(&Z);
  free_params(&GP);
  free_params(&P);
  free_saved(&S);
  free(x); free(dy); free(y); free(dx);
}

int main(void) {
  run_case(24, 2, 8, 40, 7, 2, 0);    /* ragged everything */
  run_case(16, 1, 16, 16, 1, 3, 1);   /* sequences of one token, erf GeLU */
  run_case(40, 5, 8, 24, 13, 1, 0);   /* more heads than a vector is wide */
  if (failures) { fprintf(stderr, "%d check(s) failed\n", failures); return 1; }
  printf("oracle under sanitizers: ok\n");
  return 0;
}
