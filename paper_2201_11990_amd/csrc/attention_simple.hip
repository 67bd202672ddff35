// Causal softmax attention, forward and backward, on the vector ALUs with fp32
// arithmetic: one 256-thread workgroup per (batch, head, row).  This is the
// attention of the fp32 path and the fallback for head sizes the MFMA kernels do
// not take.  Sequence length up to 4096 (a row of scores is held in LDS).
//
//   S[t,u] = scale * q_t . k_u  (u <= t),  P = rowsoftmax(S),  a_t = sum_u P[t,u] v_u
//   lse[t] = log sum_u exp(S[t,u])
// backward, with D_t = da_t . a_t = sum_u P[t,u] dP[t,u]:
//   dP[t,u] = da_t . v_u,  dS = P o (dP - D),  dq_t = scale sum_u dS[t,u] k_u,
//   dk_u = scale sum_t dS[t,u] q_t,  dv_u = sum_t P[t,u] da_t
#include "common.h"

namespace mtnlg {

constexpr int ATT_MAX_D = 256;
constexpr int ATT_SIMPLE_MAX_S = ATTENTION_SIMPLE_MAX_SEQ;

template <typename E>
__device__ __forceinline__ float dot_row(const float *__restrict__ a_lds, const E *__restrict__ row, int d) {
  float acc = 0.0f;
  for (int e = 0; e < d; e += 8) {
    float v[8];
    load8(row + e, v);
#pragma unroll
    for (int i = 0; i < 8; ++i) acc = fmaf(a_lds[e + i], v[i], acc);
  }
  return acc;
}

__device__ __forceinline__ float block_reduce(float v, float *red, bool is_max) {
  v = is_max ? wave_max(v) : wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return is_max ? fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3])) : red[0] + red[1] + red[2] + red[3];
}

// Accumulate out[e] = mul * sum_{i<count} w[i] * rows[(first+i)*ld + e] over the workgroup.
// Waves split i, lanes split e; partials merged through `part` ([4][ATT_MAX_D]).
template <typename E>
__device__ __forceinline__ void weighted_row_sum(const float *w, int count, const E *rows, int64_t ld,
                                                 int d, float mul, float *part, E *out) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float acc[ATT_MAX_D / 64] = {};
  __syncthreads();  // w[] complete, part[] no longer read
  for (int i = wave; i < count; i += 4) {
    const float wi = w[i];
    const E *r = rows + (int64_t)i * ld;
#pragma unroll
    for (int c = 0; c < ATT_MAX_D / 64; ++c) {
      int e = lane + 64 * c;
      if (e < d) acc[c] = fmaf(wi, to_f32(r[e]), acc[c]);
    }
  }
#pragma unroll
  for (int c = 0; c < ATT_MAX_D / 64; ++c) part[wave * ATT_MAX_D + lane + 64 * c] = acc[c];
  __syncthreads();
  for (int e = threadIdx.x; e < d; e += 256)
    out[e] = from_f32<E>(mul * (part[e] + part[ATT_MAX_D + e] + part[2 * ATT_MAX_D + e] + part[3 * ATT_MAX_D + e]));
}

template <typename E>
__global__ __launch_bounds__(256) void attn_fwd_simple(int s, int n, int d, float scale,
                                                       const E *__restrict__ qkv, E *__restrict__ a,
                                                       float *__restrict__ lse) {
  extern __shared__ float smem[];
  float *qs = smem;                    // [ATT_MAX_D]
  float *part = qs + ATT_MAX_D;        // [4*ATT_MAX_D]
  float *red = part + 4 * ATT_MAX_D;   // [4]
  float *sc = red + 4;                 // [s]
  const int t = blockIdx.x, j = blockIdx.y, bi = blockIdx.z;
  const int64_t ld = (int64_t)n * 3 * d;
  const E *base = qkv + (int64_t)bi * s * ld + (int64_t)j * 3 * d;
  for (int e = threadIdx.x; e < d; e += 256) qs[e] = to_f32(base[(int64_t)t * ld + e]);
  __syncthreads();
  float mx = -INFINITY;
  for (int u = threadIdx.x; u <= t; u += 256) {
    float v = scale * dot_row(qs, base + (int64_t)u * ld + d, d);
    sc[u] = v;
    mx = fmaxf(mx, v);
  }
  mx = block_reduce(mx, red, true);
  float den = 0.0f;
  for (int u = threadIdx.x; u <= t; u += 256) {
    float p = expf(sc[u] - mx);
    sc[u] = p;
    den += p;
  }
  den = block_reduce(den, red, false);
  if (threadIdx.x == 0) lse[((int64_t)bi * n + j) * s + t] = mx + logf(den);
  weighted_row_sum<E>(sc, t + 1, base + 2 * d, ld, d, 1.0f / den, part,
                      a + ((int64_t)bi * s + t) * ((int64_t)n * d) + (int64_t)j * d);
}

// D[b,n,t] = da_t . a_t for head j
template <typename E>
__global__ __launch_bounds__(64) void attn_bwd_dot(int s, int n, int d, const E *__restrict__ a,
                                                   const E *__restrict__ da, float *__restrict__ D) {
  const int t = blockIdx.x, j = blockIdx.y, bi = blockIdx.z;
  const int64_t off = ((int64_t)bi * s + t) * ((int64_t)n * d) + (int64_t)j * d;
  float acc = 0.0f;
  for (int e = threadIdx.x; e < d; e += 64) acc += to_f32(a[off + e]) * to_f32(da[off + e]);
  acc = wave_sum(acc);
  if (threadIdx.x == 0) D[((int64_t)bi * n + j) * s + t] = acc;
}

template <typename E>
__global__ __launch_bounds__(256) void attn_bwd_dq_simple(int s, int n, int d, float scale,
                                                          const E *__restrict__ qkv,
                                                          const float *__restrict__ lse,
                                                          const float *__restrict__ D,
                                                          const E *__restrict__ da,
                                                          E *__restrict__ dqkv) {
  extern __shared__ float smem[];
  float *qs = smem;                    // [ATT_MAX_D]
  float *das = qs + ATT_MAX_D;         // [ATT_MAX_D]
  float *part = das + ATT_MAX_D;       // [4*ATT_MAX_D]
  float *ds = part + 4 * ATT_MAX_D;    // [s]
  const int t = blockIdx.x, j = blockIdx.y, bi = blockIdx.z;
  const int64_t ld = (int64_t)n * 3 * d;
  const E *base = qkv + (int64_t)bi * s * ld + (int64_t)j * 3 * d;
  const E *dar = da + ((int64_t)bi * s + t) * ((int64_t)n * d) + (int64_t)j * d;
  for (int e = threadIdx.x; e < d; e += 256) {
    qs[e] = to_f32(base[(int64_t)t * ld + e]);
    das[e] = to_f32(dar[e]);
  }
  __syncthreads();
  const float l = lse[((int64_t)bi * n + j) * s + t], Dt = D[((int64_t)bi * n + j) * s + t];
  for (int u = threadIdx.x; u <= t; u += 256) {
    float p = expf(scale * dot_row(qs, base + (int64_t)u * ld + d, d) - l);
    float dp = dot_row(das, base + (int64_t)u * ld + 2 * d, d);
    ds[u] = p * (dp - Dt);
  }
  weighted_row_sum<E>(ds, t + 1, base + d, ld, d, scale, part,
                      dqkv + ((int64_t)bi * s + t) * ld + (int64_t)j * 3 * d);
}

template <typename E>
__global__ __launch_bounds__(256) void attn_bwd_dkv_simple(int s, int n, int d, float scale,
                                                           const E *__restrict__ qkv,
                                                           const float *__restrict__ lse,
                                                           const float *__restrict__ D,
                                                           const E *__restrict__ da,
                                                           E *__restrict__ dqkv) {
  extern __shared__ float smem[];
  float *ks = smem;                    // [ATT_MAX_D]
  float *vs = ks + ATT_MAX_D;          // [ATT_MAX_D]
  float *part = vs + ATT_MAX_D;        // [4*ATT_MAX_D]
  float *ps = part + 4 * ATT_MAX_D;    // [s]
  float *ds = ps + s;                  // [s]
  const int u = blockIdx.x, j = blockIdx.y, bi = blockIdx.z;
  const int64_t ld = (int64_t)n * 3 * d, p_ld = (int64_t)n * d;
  const E *base = qkv + (int64_t)bi * s * ld + (int64_t)j * 3 * d;
  const E *dab = da + (int64_t)bi * s * p_ld + (int64_t)j * d;
  for (int e = threadIdx.x; e < d; e += 256) {
    ks[e] = to_f32(base[(int64_t)u * ld + d + e]);
    vs[e] = to_f32(base[(int64_t)u * ld + 2 * d + e]);
  }
  __syncthreads();
  const float *lrow = lse + ((int64_t)bi * n + j) * s, *Drow = D + ((int64_t)bi * n + j) * s;
  for (int t = u + threadIdx.x; t < s; t += 256) {
    float p = expf(scale * dot_row(ks, base + (int64_t)t * ld, d) - lrow[t]);
    float dp = dot_row(vs, dab + (int64_t)t * p_ld, d);
    ps[t - u] = p;
    ds[t - u] = p * (dp - Drow[t]);
  }
  E *out = dqkv + ((int64_t)bi * s + u) * ld + (int64_t)j * 3 * d;
  weighted_row_sum<E>(ps, s - u, dab + (int64_t)u * p_ld, p_ld, d, 1.0f, part, out + 2 * d);  // dv
  weighted_row_sum<E>(ds, s - u, base + (int64_t)u * ld, ld, d, scale, part, out + d);        // dk
}

template <typename E>
static int fwd_launch(int b, int s, int n, int d, float scale, const void *qkv, void *a, float *lse,
                      hipStream_t st) {
  size_t smem = (size_t)(5 * ATT_MAX_D + 4 + s) * sizeof(float);
  LaunchScope scope(MTNLG_K_ATTN_FWD, st);
  attn_fwd_simple<E><<<dim3(s, n, b), 256, smem, st>>>(s, n, d, scale, (const E *)qkv, (E *)a, lse);
  return check_launch();
}

template <typename E>
static int bwd_launch(int b, int s, int n, int d, float scale, const void *qkv, const void *a,
                      const float *lse, const void *da, void *dqkv, void *ws, hipStream_t st) {
  float *D = (float *)ws;
  LaunchScope scope(MTNLG_K_ATTN_BWD, st);
  attn_bwd_dot<E><<<dim3(s, n, b), 64, 0, st>>>(s, n, d, (const E *)a, (const E *)da, D);
  MTNLG_TRY(check_launch());
  size_t smem1 = (size_t)(6 * ATT_MAX_D + s) * sizeof(float);
  attn_bwd_dq_simple<E><<<dim3(s, n, b), 256, smem1, st>>>(s, n, d, scale, (const E *)qkv, lse, D,
                                                           (const E *)da, (E *)dqkv);
  MTNLG_TRY(check_launch());
  size_t smem2 = (size_t)(6 * ATT_MAX_D + 2 * s) * sizeof(float);
  attn_bwd_dkv_simple<E><<<dim3(s, n, b), 256, smem2, st>>>(s, n, d, scale, (const E *)qkv, lse, D,
                                                            (const E *)da, (E *)dqkv);
  return check_launch();
}

int attention_fwd_simple(int dtype, int b, int s, int n, int d, float scale, const void *qkv, void *a,
                         float *lse, hipStream_t stream) {
  if (d % 8 || d > ATT_MAX_D || s > ATT_SIMPLE_MAX_S || n > 65535 || b > 65535)
    return MTNLG_UNSUPPORTED_SHAPE;
  if (dtype == MTNLG_F32) return fwd_launch<float>(b, s, n, d, scale, qkv, a, lse, stream);
  if (dtype == MTNLG_BF16) return fwd_launch<bf16>(b, s, n, d, scale, qkv, a, lse, stream);
  return MTNLG_INVALID_ARG;
}

int attention_bwd_simple(int dtype, int b, int s, int n, int d, float scale, const void *qkv,
                         const void *a, const float *lse, const void *da, void *dqkv, void *ws,
                         hipStream_t stream) {
  if (d % 8 || d > ATT_MAX_D || s > ATT_SIMPLE_MAX_S || n > 65535 || b > 65535)
    return MTNLG_UNSUPPORTED_SHAPE;
  if (dtype == MTNLG_F32) return bwd_launch<float>(b, s, n, d, scale, qkv, a, lse, da, dqkv, ws, stream);
  if (dtype == MTNLG_BF16) return bwd_launch<bf16>(b, s, n, d, scale, qkv, a, lse, da, dqkv, ws, stream);
  return MTNLG_INVALID_ARG;
}

}  // namespace mtnlg
