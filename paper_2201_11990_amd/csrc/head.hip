// First and last pipeline stage's extras around the layer stack: the vocabulary-sliced token
// embedding with learned positions, and the final LayerNorm + tied output projection +
// next-token cross-entropy with their backward.  The paper (Section 3.2) names the GPT-2 decoder
// and prints none of this; the tensor slicing of Section 2.1 is applied to the vocabulary the way
// it is applied to the linears: contiguous row blocks of the embedding matrix per rank.
//
// The matrix products and the LayerNorm are the library's own (mtnlg_gemm, mtnlg_layernorm_*);
// this file adds the HBM-bound pieces:
//   embedding forward  : one workgroup per token, copies its row of E (or zeros when the token
//                        belongs to another rank) -- the position row is added after the hook;
//   embedding backward : one workgroup per (vocabulary row, 1024-column chunk) scans the token ids
//                        in order and sums the matching rows of dx: fixed order, no atomics;
//                        the position gradient is a sum over the batch;
//   cross-entropy      : three row kernels (maximum | sum of exponentials and the target's logit |
//                        loss and gradient), split where a tensor-parallel group exchanges values.
#include <math.h>

#include "common.h"

namespace mtnlg {

namespace {

template <typename E>
__global__ __launch_bounds__(256) void embedding_fwd_kernel(int64_t h, int vocab_local, int vocab_start,
                                                            const int32_t *__restrict__ tokens, const E *__restrict__ emb,
                                                            E *__restrict__ x) {
  const int64_t t = blockIdx.x;
  const int v = tokens[t] - vocab_start;
  const bool mine = v >= 0 && v < vocab_local;
  const E *src = emb + (int64_t)(mine ? v : 0) * h;
  E *dst = x + t * h;
  for (int64_t c = threadIdx.x * 8; c < h; c += 256 * 8) {
    float val[8];
    if (mine) load8(src + c, val);
    else
#pragma unroll
      for (int e = 0; e < 8; ++e) val[e] = 0.0f;
    store8(dst + c, val);
  }
}

// x[t] += P[t % seq]
template <typename E>
__global__ __launch_bounds__(256) void add_positions_kernel(int64_t h, int seq, const E *__restrict__ pos, E *__restrict__ x) {
  const int64_t t = blockIdx.x;
  const E *src = pos + (t % seq) * h;
  E *dst = x + t * h;
  for (int64_t c = threadIdx.x * 8; c < h; c += 256 * 8) {
    float a[8], b[8];
    load8(dst + c, a);
    load8(src + c, b);
#pragma unroll
    for (int e = 0; e < 8; ++e) a[e] += b[e];
    store8(dst + c, a);
  }
}

// dE[v, c0 .. c0+1023] = sum over tokens t (in order) with tokens[t] == vocab_start + v of dx[t, ...]
template <typename E>
__global__ __launch_bounds__(128) void embedding_bwd_kernel(int64_t T, int64_t h, int vocab_start,
                                                            const int32_t *__restrict__ tokens, const E *__restrict__ dx,
                                                            E *__restrict__ dE) {
  const int v = blockIdx.x, id = vocab_start + v;
  const int64_t c = (int64_t)blockIdx.y * 1024 + threadIdx.x * 8;
  float acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = 0.0f;
  for (int64_t t = 0; t < T; ++t) {
    if (tokens[t] == id && c < h) {   // workgroup-uniform test on the id, so every lane takes the same tokens
      float d[8];
      load8(dx + t * h + c, d);
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] += d[e];
    }
  }
  if (c < h) store8(dE + (int64_t)v * h + c, acc);
}

// dP[s] = sum over the batch of dx[b, s]
template <typename E>
__global__ __launch_bounds__(256) void position_bwd_kernel(int batch, int seq, int64_t h, const E *__restrict__ dx,
                                                           E *__restrict__ dP) {
  const int s = blockIdx.x;
  for (int64_t c = threadIdx.x * 8; c < h; c += 256 * 8) {
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.0f;
    for (int b = 0; b < batch; ++b) {
      float d[8];
      load8(dx + ((int64_t)b * seq + s) * h + c, d);
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] += d[e];
    }
    store8(dP + (int64_t)s * h + c, acc);
  }
}

__device__ __forceinline__ float block_reduce(float v, bool is_max, float *red) {
  v = is_max ? wave_max(v) : wave_sum(v);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  __syncthreads();
  if (lane == 0) red[wave] = v;
  __syncthreads();
  float r = red[0];
  for (int w = 1; w < (int)(blockDim.x >> 6); ++w) r = is_max ? fmaxf(r, red[w]) : r + red[w];
  return r;
}

// one workgroup per token row of the fp32 logits [T, Vl]
__global__ __launch_bounds__(256) void ce_max_kernel(int64_t Vl, const float *__restrict__ logits, float *__restrict__ m) {
  __shared__ float red[4];
  const float *row = logits + (int64_t)blockIdx.x * Vl;
  float mx = -INFINITY;
  for (int64_t c = threadIdx.x; c < Vl; c += 256) mx = fmaxf(mx, row[c]);
  mx = block_reduce(mx, true, red);
  if (threadIdx.x == 0) m[blockIdx.x] = mx;
}

__global__ __launch_bounds__(256) void ce_sum_kernel(int64_t Vl, int vocab_start, const float *__restrict__ logits,
                                                     const float *__restrict__ m, const int32_t *__restrict__ targets,
                                                     float *__restrict__ s, float *__restrict__ tl) {
  __shared__ float red[4];
  const float *row = logits + (int64_t)blockIdx.x * Vl;
  const float mx = m[blockIdx.x];
  float acc = 0.0f;
  for (int64_t c = threadIdx.x; c < Vl; c += 256) acc += __expf(row[c] - mx);
  acc = block_reduce(acc, false, red);
  if (threadIdx.x == 0) {
    s[blockIdx.x] = acc;
    const int v = targets[blockIdx.x] - vocab_start;
    tl[blockIdx.x] = (v >= 0 && v < Vl) ? row[v] : 0.0f;
  }
}

template <typename E>
__global__ __launch_bounds__(256) void ce_grad_kernel(int64_t T, int64_t Vl, int vocab_start, const float *__restrict__ logits,
                                                      const float *__restrict__ m, const float *__restrict__ s,
                                                      const float *__restrict__ tl, const int32_t *__restrict__ targets,
                                                      const float *__restrict__ dloss, float *__restrict__ loss,
                                                      E *__restrict__ dlogits) {
  const int64_t t = blockIdx.x;
  const float *row = logits + t * Vl;
  const float mx = m[t], sum = s[t];
  const float w = (dloss != nullptr ? dloss[t] : 1.0f / (float)T), scale = w / sum;
  const int v = targets[t] - vocab_start;
  if (threadIdx.x == 0) loss[t] = logf(sum) + mx - tl[t];
  E *out = dlogits + t * Vl;
  for (int64_t c = threadIdx.x; c < Vl; c += 256) {
    float d = __expf(row[c] - mx) * scale;
    if (c == v) d -= w;
    out[c] = from_f32<E>(d);
  }
}

struct HeadWork {
  size_t u, mean, rstd, logits, dlogits, m, s, tl, du, red, gemm, gemm_bytes, total;
};

void head_layout(const mtnlg_head_desc *d, HeadWork *W) {
  const size_t T = (size_t)d->micro_batch * d->seq, h = d->hidden, Vl = d->vocab_local;
  const size_t es = d->dtype == MTNLG_BF16 ? 2 : 4;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    const size_t o = off;
    off += align_up(bytes, 256);
    return o;
  };
  W->u = take(T * h * es);
  W->mean = take(T * 4);
  W->rstd = take(T * 4);
  W->logits = take(T * Vl * 4);
  W->dlogits = take(T * Vl * es);
  W->m = take(T * 4);
  W->s = take(T * 4);
  W->tl = take(T * 4);
  W->du = take(T * h * es);
  W->red = take(mtnlg_layernorm_bwd_workspace((int64_t)T, (int64_t)h));
  size_t gb = mtnlg_gemm_workspace(d->dtype, MTNLG_GEMM_NT, (int64_t)T, (int64_t)Vl, (int64_t)h);
  const size_t g2 = mtnlg_gemm_workspace(d->dtype, MTNLG_GEMM_NN, (int64_t)T, (int64_t)h, (int64_t)Vl);
  const size_t g3 = mtnlg_gemm_workspace(d->dtype, MTNLG_GEMM_TN, (int64_t)Vl, (int64_t)h, (int64_t)T);
  gb = gb > g2 ? gb : g2;
  gb = gb > g3 ? gb : g3;
  W->gemm_bytes = gb;
  W->gemm = take(gb);
  W->total = off;
}

int head_desc_check(const mtnlg_head_desc *d) {
  if (!d) return MTNLG_NULL_POINTER;
  if (d->dtype != MTNLG_F32 && d->dtype != MTNLG_BF16) return MTNLG_INVALID_ARG;
  if (d->hidden <= 0 || d->vocab_local <= 0 || d->vocab_start < 0 || d->seq <= 0 || d->micro_batch <= 0) return MTNLG_INVALID_ARG;
  if (!(d->ln_eps >= 0.0f) || !isfinite(d->ln_eps)) return MTNLG_INVALID_ARG;
  if (d->hidden % 8 != 0) return MTNLG_UNSUPPORTED_SHAPE;   // 16-byte row accesses
  if (d->dtype == MTNLG_BF16 && d->vocab_local % 8 != 0) return MTNLG_UNSUPPORTED_SHAPE;
  return MTNLG_OK;
}

inline char *at(void *base, size_t off) { return static_cast<char *>(base) + off; }

int call_hook(mtnlg_reduce_op_fn reduce, void *user, void *buf, size_t count, int dtype, int op, hipStream_t st) {
  if (!reduce) return MTNLG_OK;
  return reduce(buf, count, dtype, op, (void *)st, user) == 0 ? MTNLG_OK : MTNLG_REDUCE_FAILED;
}

}  // namespace

}  // namespace mtnlg

using namespace mtnlg;

extern "C" {

size_t mtnlg_lm_head_workspace(const mtnlg_head_desc *desc) {
  if (head_desc_check(desc) != MTNLG_OK) return 0;
  HeadWork W;
  head_layout(desc, &W);
  return W.total;
}

int mtnlg_embedding_fwd(const mtnlg_head_desc *desc, const int32_t *tokens, const void *emb, const void *pos, void *x,
                        mtnlg_reduce_op_fn reduce, void *user, void *stream) {
  MTNLG_TRY(head_desc_check(desc));
  if (!tokens || !emb || !pos || !x) return MTNLG_NULL_POINTER;
  const int64_t T = (int64_t)desc->micro_batch * desc->seq, h = desc->hidden;
  hipStream_t st = (hipStream_t)stream;
  {
    LaunchScope scope(MTNLG_K_ELEMENTWISE, st);
    if (desc->dtype == MTNLG_BF16)
      embedding_fwd_kernel<bf16><<<(unsigned)T, 256, 0, st>>>(h, desc->vocab_local, desc->vocab_start, tokens, (const bf16 *)emb, (bf16 *)x);
    else
      embedding_fwd_kernel<float><<<(unsigned)T, 256, 0, st>>>(h, desc->vocab_local, desc->vocab_start, tokens, (const float *)emb, (float *)x);
    MTNLG_TRY(check_launch());
  }
  MTNLG_TRY(call_hook(reduce, user, x, (size_t)(T * h), desc->dtype, MTNLG_REDUCE_SUM, st));
  LaunchScope scope(MTNLG_K_ELEMENTWISE, st);
  if (desc->dtype == MTNLG_BF16) add_positions_kernel<bf16><<<(unsigned)T, 256, 0, st>>>(h, desc->seq, (const bf16 *)pos, (bf16 *)x);
  else add_positions_kernel<float><<<(unsigned)T, 256, 0, st>>>(h, desc->seq, (const float *)pos, (float *)x);
  return check_launch();
}

int mtnlg_embedding_bwd(const mtnlg_head_desc *desc, const int32_t *tokens, const void *dx, void *demb, void *dpos,
                        void *stream) {
  MTNLG_TRY(head_desc_check(desc));
  if (!tokens || !dx || !demb || !dpos) return MTNLG_NULL_POINTER;
  if (desc->vocab_local > 65535 * 32) return MTNLG_UNSUPPORTED_SHAPE;
  const int64_t T = (int64_t)desc->micro_batch * desc->seq, h = desc->hidden;
  hipStream_t st = (hipStream_t)stream;
  const dim3 grid((unsigned)desc->vocab_local, (unsigned)((h + 1023) / 1024));
  LaunchScope scope(MTNLG_K_ELEMENTWISE, st);
  if (desc->dtype == MTNLG_BF16) {
    embedding_bwd_kernel<bf16><<<grid, 128, 0, st>>>(T, h, desc->vocab_start, tokens, (const bf16 *)dx, (bf16 *)demb);
    MTNLG_TRY(check_launch());
    position_bwd_kernel<bf16><<<(unsigned)desc->seq, 256, 0, st>>>(desc->micro_batch, desc->seq, h, (const bf16 *)dx, (bf16 *)dpos);
  } else {
    embedding_bwd_kernel<float><<<grid, 128, 0, st>>>(T, h, desc->vocab_start, tokens, (const float *)dx, (float *)demb);
    MTNLG_TRY(check_launch());
    position_bwd_kernel<float><<<(unsigned)desc->seq, 256, 0, st>>>(desc->micro_batch, desc->seq, h, (const float *)dx, (float *)dpos);
  }
  return check_launch();
}

int mtnlg_lm_head_step(const mtnlg_head_desc *desc, const void *x, const void *ln_g, const void *ln_b, const void *emb,
                       const int32_t *targets, const float *dloss, float *loss, void *dx, void *d_ln_g, void *d_ln_b,
                       void *demb, void *workspace, size_t workspace_bytes, mtnlg_reduce_op_fn reduce, void *user,
                       void *stream) {
  MTNLG_TRY(head_desc_check(desc));
  if (!x || !ln_g || !ln_b || !emb || !targets || !loss || !dx || !d_ln_g || !d_ln_b || !demb || !workspace)
    return MTNLG_NULL_POINTER;
  HeadWork W;
  head_layout(desc, &W);
  if (workspace_bytes < W.total) return MTNLG_WORKSPACE_TOO_SMALL;
  const int dt = desc->dtype;
  const float eps = desc->ln_eps > 0.0f ? desc->ln_eps : 1e-5f;   // 0 = the default, as in the layer descriptor
  const int64_t T = (int64_t)desc->micro_batch * desc->seq, h = desc->hidden, Vl = desc->vocab_local;
  hipStream_t st = (hipStream_t)stream;
  void *u = at(workspace, W.u), *dlogits = at(workspace, W.dlogits), *du = at(workspace, W.du);
  float *mean = (float *)at(workspace, W.mean), *rstd = (float *)at(workspace, W.rstd);
  float *logits = (float *)at(workspace, W.logits);
  float *m = (float *)at(workspace, W.m), *s = (float *)at(workspace, W.s), *tl = (float *)at(workspace, W.tl);
  void *gws = at(workspace, W.gemm);

  // u = LN(x) ; logits = u E^T in fp32
  MTNLG_TRY(mtnlg_layernorm_fwd(dt, T, h, x, nullptr, nullptr, ln_g, ln_b, eps, nullptr, u, mean, rstd, st));
  MTNLG_TRY(mtnlg_gemm(dt, MTNLG_GEMM_NT, T, Vl, h, u, emb, logits, nullptr, nullptr, MTNLG_EPI_OUT_F32, gws, W.gemm_bytes, st));
  // softmax statistics, with the three exchanges of a vocabulary-sliced group
  {
    LaunchScope scope(MTNLG_K_ELEMENTWISE, st);
    ce_max_kernel<<<(unsigned)T, 256, 0, st>>>(Vl, logits, m);
    MTNLG_TRY(check_launch());
  }
  MTNLG_TRY(call_hook(reduce, user, m, (size_t)T, MTNLG_F32, MTNLG_REDUCE_MAX, st));
  {
    LaunchScope scope(MTNLG_K_ELEMENTWISE, st);
    ce_sum_kernel<<<(unsigned)T, 256, 0, st>>>(Vl, desc->vocab_start, logits, m, targets, s, tl);
    MTNLG_TRY(check_launch());
  }
  MTNLG_TRY(call_hook(reduce, user, s, (size_t)T, MTNLG_F32, MTNLG_REDUCE_SUM, st));
  MTNLG_TRY(call_hook(reduce, user, tl, (size_t)T, MTNLG_F32, MTNLG_REDUCE_SUM, st));
  {
    LaunchScope scope(MTNLG_K_ELEMENTWISE, st);
    if (dt == MTNLG_BF16)
      ce_grad_kernel<bf16><<<(unsigned)T, 256, 0, st>>>(T, Vl, desc->vocab_start, logits, m, s, tl, targets, dloss, loss, (bf16 *)dlogits);
    else
      ce_grad_kernel<float><<<(unsigned)T, 256, 0, st>>>(T, Vl, desc->vocab_start, logits, m, s, tl, targets, dloss, loss, (float *)dlogits);
    MTNLG_TRY(check_launch());
  }
  // du = dlogits E (partial over the vocabulary slices) ; dE = dlogits^T u
  MTNLG_TRY(mtnlg_gemm(dt, MTNLG_GEMM_NN, T, h, Vl, dlogits, emb, du, nullptr, nullptr, 0, gws, W.gemm_bytes, st));
  MTNLG_TRY(mtnlg_gemm(dt, MTNLG_GEMM_TN, Vl, h, T, dlogits, u, demb, nullptr, nullptr, 0, gws, W.gemm_bytes, st));
  MTNLG_TRY(call_hook(reduce, user, du, (size_t)(T * h), dt, MTNLG_REDUCE_SUM, st));
  // dx = LN^T(du) ; dgamma, dbeta
  return mtnlg_layernorm_bwd(dt, T, h, x, ln_g, mean, rstd, du, nullptr, dx, d_ln_g, d_ln_b, nullptr, 0, 0,
                             at(workspace, W.red), st);
}

}  // extern "C"
