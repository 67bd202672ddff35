// HBM-bound kernels of the layer: LayerNorm forward (optionally fused with the
// bias + residual add that precedes it), LayerNorm backward, GeLU forward and
// backward, bias + residual, and the column reductions that produce bias and
// LayerNorm parameter gradients.  All arithmetic fp32; 16-byte (bf16) or
// 32-byte (float) accesses per lane, consecutive lanes on consecutive addresses.
#include <mutex>

#include "common.h"

namespace mtnlg {

// Sum over the NTHR threads of a workgroup; result valid in every thread.
template <int NTHR>
__device__ __forceinline__ float block_sum(float v, float *lds) {
  constexpr int NW = NTHR / 64;
  v = wave_sum(v);
  __syncthreads();  // protects lds against a previous use
  if ((threadIdx.x & 63) == 0) lds[threadIdx.x >> 6] = v;
  __syncthreads();
  float s = 0.0f;
#pragma unroll
  for (int w = 0; w < NW; ++w) s += lds[w];
  return s;
}

// ---------------------------------------------------------------- LayerNorm fwd
// One workgroup of NTHR threads per token row; the row lives in registers (NV groups
// of 8 per thread).  v = x (+ partial + bias); optional xsum = v; out = LN(v).
template <typename E, int NTHR, int NV>
__global__ __launch_bounds__(NTHR) void ln_fwd_kernel(int64_t h, const E *__restrict__ x,
                                                      const E *__restrict__ partial,
                                                      const E *__restrict__ bias,
                                                      const E *__restrict__ gamma,
                                                      const E *__restrict__ beta, float eps,
                                                      E *__restrict__ xsum, E *__restrict__ out,
                                                      float *__restrict__ mean,
                                                      float *__restrict__ rstd) {
  __shared__ float red[NTHR / 64];
  const int64_t row = blockIdx.x;
  const int nvec = (int)(h / 8);
  float v[NV][8];
  float s = 0.0f;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    int j = threadIdx.x + i * NTHR;
    if (j < nvec) {
      load8(x + row * h + (int64_t)j * 8, v[i]);
      if (partial) {
        float pa[8];
        load8(partial + row * h + (int64_t)j * 8, pa);
#pragma unroll
        for (int e = 0; e < 8; ++e) v[i][e] += pa[e];
        if (bias) {
          load8(bias + (int64_t)j * 8, pa);
#pragma unroll
          for (int e = 0; e < 8; ++e) v[i][e] += pa[e];
        }
        if constexpr (sizeof(E) == 2) {
          // the residual stream is stored in bf16: normalise the stored value
#pragma unroll
          for (int e = 0; e < 8; ++e) v[i][e] = to_f32(from_f32<E>(v[i][e]));
        }
        if (xsum) store8(xsum + row * h + (int64_t)j * 8, v[i]);
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) s += v[i][e];
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) v[i][e] = 0.0f;
    }
  }
  const float mu = block_sum<NTHR>(s, red) / (float)h;
  float q = 0.0f;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    int j = threadIdx.x + i * NTHR;
    if (j < nvec) {
#pragma unroll
      for (int e = 0; e < 8; ++e) q += (v[i][e] - mu) * (v[i][e] - mu);
    }
  }
  const float var = block_sum<NTHR>(q, red) / (float)h;
  const float rs = rsqrtf(var + eps);
  if (threadIdx.x == 0) {
    mean[row] = mu;
    rstd[row] = rs;
  }
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    int j = threadIdx.x + i * NTHR;
    if (j < nvec) {
      float g[8], b[8], o[8];
      load8(gamma + (int64_t)j * 8, g);
      load8(beta + (int64_t)j * 8, b);
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e] = g[e] * ((v[i][e] - mu) * rs) + b[e];
      store8(out + row * h + (int64_t)j * 8, o);
    }
  }
}

template <typename E>
static int ln_fwd_launch(int64_t T, int64_t h, const void *x, const void *partial, const void *bias,
                         const void *gamma, const void *beta, float eps, void *xsum, void *out,
                         float *mean, float *rstd, hipStream_t st) {
  const int nvec = (int)(h / 8);
#define LNF(NTHR, NV)                                                                             \
  ln_fwd_kernel<E, NTHR, NV><<<dim3((unsigned)T), NTHR, 0, st>>>(                                 \
      h, (const E *)x, (const E *)partial, (const E *)bias, (const E *)gamma, (const E *)beta, eps, \
      (E *)xsum, (E *)out, mean, rstd)
  LaunchScope scope(MTNLG_K_LN_FWD, st);
  if (nvec <= 256) LNF(256, 1);
  else if (nvec <= 512) LNF(256, 2);
  else if (nvec <= 1024) LNF(256, 4);
  else if (nvec <= 2048) LNF(1024, 2);
  else if (nvec <= 3072) LNF(1024, 3);
  else if (nvec <= 4096) LNF(1024, 4);
  else return MTNLG_UNSUPPORTED_SHAPE;
#undef LNF
  return check_launch();
}

// ---------------------------------------------------------------- LayerNorm bwd
// One 1024-thread workgroup walks `rows_per` consecutive token rows; a thread owns the
// same NV groups of 8 columns in every row, so the column sums
//   dgamma = sum_t dout*xhat,  dbeta = sum_t dout,  (CS) colsum = sum_t dx
// build up in its registers while the rows stream through once from HBM:
//   pass 1 over the row: xhat, dxh = dout*gamma -> row sums m1 = mean(dxh), m2 = mean(dxh*xhat)
//   pass 2 (row re-read, L2-resident): dx = dres + rs * (dxh - m1 - xhat*m2)
// Workgroup b leaves its column sums in ws[o][b][h]; a second kernel adds them in a
// fixed order.
constexpr int LNB_THREADS = 1024, LNB_MAX_WGS = 256;

template <typename E, int NV, bool CS>
__global__ __launch_bounds__(LNB_THREADS) void ln_bwd_fused_kernel(
    int64_t T, int64_t h, int rows_per, const E *__restrict__ x, const E *__restrict__ gamma,
    const float *__restrict__ mean, const float *__restrict__ rstd, const E *__restrict__ dout,
    const E *__restrict__ dres, E *__restrict__ dx, float *__restrict__ ws) {
  __shared__ float red[2][LNB_THREADS / 64];
  const int nvec = (int)(h / 8);
  const int64_t row0 = (int64_t)blockIdx.x * rows_per;
  const int64_t row1 = row0 + rows_per < T ? row0 + rows_per : T;
  float dg[NV][8] = {}, db[NV][8] = {}, cs[CS ? NV : 1][8] = {};
  for (int64_t row = row0; row < row1; ++row) {
    const float mu = mean[row], rs = rstd[row];
    float s1 = 0.0f, s2 = 0.0f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int j = threadIdx.x + i * LNB_THREADS;
      if (j < nvec) {
        float xv[8], dv[8], g[8];
        load8(x + row * h + (int64_t)j * 8, xv);
        load8(dout + row * h + (int64_t)j * 8, dv);
        load8(gamma + (int64_t)j * 8, g);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float xh = (xv[e] - mu) * rs, dh = dv[e] * g[e];
          s1 += dh;
          s2 += dh * xh;
          dg[i][e] += dv[e] * xh;
          db[i][e] += dv[e];
        }
      }
    }
    // both row sums through one pair of barriers
    s1 = wave_sum(s1);
    s2 = wave_sum(s2);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) {
      red[0][threadIdx.x >> 6] = s1;
      red[1][threadIdx.x >> 6] = s2;
    }
    __syncthreads();
    float m1 = 0.0f, m2 = 0.0f;
#pragma unroll
    for (int w = 0; w < LNB_THREADS / 64; ++w) {
      m1 += red[0][w];
      m2 += red[1][w];
    }
    m1 /= (float)h;
    m2 /= (float)h;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int j = threadIdx.x + i * LNB_THREADS;
      if (j < nvec) {
        float xv[8], dv[8], g[8], o[8];
        load8(x + row * h + (int64_t)j * 8, xv);
        load8(dout + row * h + (int64_t)j * 8, dv);
        load8(gamma + (int64_t)j * 8, g);
        if (dres) load8(dres + row * h + (int64_t)j * 8, o);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float xh = (xv[e] - mu) * rs, dh = dv[e] * g[e];
          o[e] = (dres ? o[e] : 0.0f) + rs * (dh - m1 - xh * m2);
          if constexpr (CS) cs[i][e] += to_f32(from_f32<E>(o[e]));  // the stored value
        }
        store8(dx + row * h + (int64_t)j * 8, o);
      }
    }
  }
  const int64_t stride = (int64_t)gridDim.x * h;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int j = threadIdx.x + i * LNB_THREADS;
    if (j < nvec) {
      float *o = ws + (int64_t)blockIdx.x * h + (int64_t)j * 8;
      store8(o, dg[i]);
      store8(o + stride, db[i]);
      if constexpr (CS) store8(o + 2 * stride, cs[i]);
    }
  }
}

// ---------------------------------------------------------------- column reductions
// Stage 1: workgroup (bx, by) owns 512 columns [bx*512, +512) and the rows
// t = by*4 + wave, stepping by 4*gridDim.y.  Lane l owns columns 8l..8l+7 of
// the strip.  MODE 0: sum of in.  MODE 1 (LayerNorm): out0 = sum dout*xhat,
// out1 = sum dout, and, if dx != NULL, out2 = sum dx.
// Partials land in ws as [nout][gridDim.y][C] floats; stage 2 adds them up in a
// fixed order, so results do not depend on scheduling.
constexpr int CR_COLS = 512;

template <typename E, int MODE>
__global__ __launch_bounds__(256) void colreduce_stage1(int64_t T, int64_t C,
                                                        const E *__restrict__ in,
                                                        const E *__restrict__ x,
                                                        const float *__restrict__ mean,
                                                        const float *__restrict__ rstd,
                                                        const E *__restrict__ dx,
                                                        float *__restrict__ ws) {
  constexpr int NOUT = MODE == 0 ? 1 : 3;
  __shared__ float red[4][NOUT][CR_COLS];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t c0 = (int64_t)blockIdx.x * CR_COLS + lane * 8;
  float acc[NOUT][8] = {};
  if (c0 < C) {
    for (int64_t t = (int64_t)blockIdx.y * 4 + wave; t < T; t += 4 * (int64_t)gridDim.y) {
      float a[8];
      load8(in + t * C + c0, a);
      if constexpr (MODE == 0) {
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[0][e] += a[e];
      } else {
        float xv[8];
        load8(x + t * C + c0, xv);
        const float mu = mean[t], rs = rstd[t];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          acc[0][e] += a[e] * ((xv[e] - mu) * rs);
          acc[1][e] += a[e];
        }
        if (dx) {
          load8(dx + t * C + c0, xv);
#pragma unroll
          for (int e = 0; e < 8; ++e) acc[2][e] += xv[e];
        }
      }
    }
  }
#pragma unroll
  for (int o = 0; o < NOUT; ++o)
#pragma unroll
    for (int e = 0; e < 8; ++e) red[wave][o][lane * 8 + e] = acc[o][e];
  __syncthreads();
  for (int i = threadIdx.x; i < NOUT * CR_COLS; i += 256) {
    int o = i / CR_COLS, c = i % CR_COLS;
    int64_t col = (int64_t)blockIdx.x * CR_COLS + c;
    if (col < C) {
      float s = red[0][o][c] + red[1][o][c] + red[2][o][c] + red[3][o][c];
      ws[((int64_t)o * gridDim.y + blockIdx.y) * C + col] = s;
    }
  }
}

// Stage 2: out_o[c] (+)= sum_r ws[o][r][c] for up to three outputs o = blockIdx.y.
// A workgroup owns 64 columns; wave w adds rows w, w+4, ... in order, the four wave
// sums are then added in order: a fixed summation tree, independent of scheduling.
struct Stage2Outs {
  void *out[3];
};
template <typename O>
__global__ __launch_bounds__(256) void colreduce_stage2(int64_t C, int nrb, const float *__restrict__ ws,
                                                        Stage2Outs outs, int accumulate) {
  __shared__ float part[4][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t c = (int64_t)blockIdx.x * 64 + lane;
  const float *src = ws + (int64_t)blockIdx.y * nrb * C;
  float s0 = 0.0f, s1 = 0.0f;
  if (c < C) {
    int r = wave;
    for (; r + 4 < nrb; r += 8) {
      s0 += src[(int64_t)r * C + c];
      s1 += src[(int64_t)(r + 4) * C + c];
    }
    if (r < nrb) s0 += src[(int64_t)r * C + c];
  }
  part[wave][lane] = s0 + s1;
  __syncthreads();
  if (wave == 0 && c < C) {
    float s = part[0][lane] + part[1][lane] + part[2][lane] + part[3][lane];
    O *out = static_cast<O *>(outs.out[blockIdx.y]);
    if (accumulate) s += to_f32(out[c]);
    out[c] = from_f32<O>(s);
  }
}

static int colreduce_rowblocks(int64_t T) {
  int64_t rb = (T + 63) / 64;  // at least 16 rows per wave
  if (rb < 1) rb = 1;
  if (rb > 32) rb = 32;
  return (int)rb;
}

// ws holds nout consecutive [nrb][C] partial blocks; outs their destinations.
template <typename E>
static void stage2_launch(int64_t C, int nrb, const float *ws, int nout, void *o0, void *o1, void *o2,
                          int out_f32, int accumulate, hipStream_t st) {
  dim3 grid((unsigned)((C + 63) / 64), (unsigned)nout);
  Stage2Outs outs{{o0, o1, o2}};
  if (out_f32)
    colreduce_stage2<float><<<grid, 256, 0, st>>>(C, nrb, ws, outs, accumulate);
  else
    colreduce_stage2<E><<<grid, 256, 0, st>>>(C, nrb, ws, outs, accumulate);
}

static int ln_bwd_workgroups(int64_t T) { return (int)(T < LNB_MAX_WGS ? T : LNB_MAX_WGS); }

template <typename E>
static int ln_bwd_launch(int64_t T, int64_t h, const void *x, const void *gamma, const float *mean,
                         const float *rstd, const void *dout, const void *dres, void *dx,
                         void *dgamma, void *dbeta, void *colsum_dx, int grad_f32, int accumulate,
                         void *workspace, hipStream_t st) {
  const int nvec = (int)(h / 8);
  const int rows_per = (int)((T + LNB_MAX_WGS - 1) / LNB_MAX_WGS);
  const int nwg = (int)((T + rows_per - 1) / rows_per);  // <= ln_bwd_workgroups(T)
  float *ws = (float *)workspace;
#define LNB(NV, CS)                                                                                  \
  ln_bwd_fused_kernel<E, NV, CS><<<dim3((unsigned)nwg), LNB_THREADS, 0, st>>>(                       \
      T, h, rows_per, (const E *)x, (const E *)gamma, mean, rstd, (const E *)dout, (const E *)dres, \
      (E *)dx, ws)
  LaunchScope scope(MTNLG_K_LN_BWD, st);
  if (colsum_dx) {
    if (nvec <= 1024) LNB(1, true);
    else if (nvec <= 2048) LNB(2, true);
    else if (nvec <= 3072) LNB(3, true);
    else if (nvec <= 4096) LNB(4, true);
    else return MTNLG_UNSUPPORTED_SHAPE;
  } else {
    if (nvec <= 1024) LNB(1, false);
    else if (nvec <= 2048) LNB(2, false);
    else if (nvec <= 3072) LNB(3, false);
    else if (nvec <= 4096) LNB(4, false);
    else return MTNLG_UNSUPPORTED_SHAPE;
  }
#undef LNB
  MTNLG_TRY(check_launch());
  stage2_launch<E>(h, nwg, ws, colsum_dx ? 3 : 2, dgamma, dbeta, colsum_dx, grad_f32, accumulate, st);
  return check_launch();
}

template <typename E>
static int colsum_launch(int64_t T, int64_t C, const void *in, void *out, int out_f32, int accumulate,
                         void *workspace, hipStream_t st) {
  const int nrb = colreduce_rowblocks(T);
  dim3 grid((unsigned)((C + CR_COLS - 1) / CR_COLS), (unsigned)nrb);
  LaunchScope scope(MTNLG_K_COLSUM, st);
  colreduce_stage1<E, 0><<<grid, 256, 0, st>>>(T, C, (const E *)in, nullptr, nullptr, nullptr, nullptr,
                                               (float *)workspace);
  MTNLG_TRY(check_launch());
  stage2_launch<E>(C, nrb, (const float *)workspace, 1, out, nullptr, nullptr, out_f32, accumulate, st);
  return check_launch();
}

// ---------------------------------------------------------------- GeLU / residual
template <typename E>
__global__ __launch_bounds__(256) void gelu_fwd_kernel(int64_t nvec, const E *__restrict__ z,
                                                       E *__restrict__ g, int erf_form) {
  for (int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x; j < nvec; j += (int64_t)gridDim.x * 256) {
    float v[8];
    load8(z + j * 8, v);
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = gelu_f(v[e], erf_form != 0);
    store8(g + j * 8, v);
  }
}

template <typename E>
__global__ __launch_bounds__(256) void gelu_bwd_kernel(int64_t nvec, const E *__restrict__ z,
                                                       const E *dg, E *dz, int erf_form) {
  for (int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x; j < nvec; j += (int64_t)gridDim.x * 256) {
    float v[8], d[8];
    load8(z + j * 8, v);
    load8(dg + j * 8, d);
#pragma unroll
    for (int e = 0; e < 8; ++e) d[e] *= gelu_grad_f(v[e], erf_form != 0);
    store8(dz + j * 8, d);
  }
}

template <typename E>
__global__ __launch_bounds__(256) void bias_residual_kernel(int64_t T, int64_t h,
                                                            const E *__restrict__ res,
                                                            const E *__restrict__ partial,
                                                            const E *__restrict__ bias,
                                                            E *__restrict__ out) {
  const int64_t hv = h / 8, nvec = T * hv;
  for (int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x; j < nvec; j += (int64_t)gridDim.x * 256) {
    float a[8], b[8];
    load8(res + j * 8, a);
    load8(partial + j * 8, b);
#pragma unroll
    for (int e = 0; e < 8; ++e) a[e] += b[e];
    if (bias) {
      load8(bias + (j % hv) * 8, b);
#pragma unroll
      for (int e = 0; e < 8; ++e) a[e] += b[e];
    }
    store8(out + j * 8, a);
  }
}

static unsigned ew_grid(int64_t nvec) {
  int64_t g = (nvec + 255) / 256;
  if (g > 256 * 16) g = 256 * 16;
  if (g < 1) g = 1;
  return (unsigned)g;
}

}  // namespace mtnlg

using namespace mtnlg;

extern "C" {

int mtnlg_layernorm_fwd(int dtype, int64_t T, int64_t h, const void *x, const void *partial,
                        const void *bias, const void *gamma, const void *beta, float eps, void *xsum,
                        void *out, float *mean, float *rstd, void *stream) {
  if (!x || !gamma || !beta || !out || !mean || !rstd) return MTNLG_NULL_POINTER;
  if (T <= 0 || h <= 0) return MTNLG_INVALID_ARG;
  if (h % 8 || h > 32768) return MTNLG_UNSUPPORTED_SHAPE;
  hipStream_t st = (hipStream_t)stream;
  if (dtype == MTNLG_F32)
    return ln_fwd_launch<float>(T, h, x, partial, bias, gamma, beta, eps, xsum, out, mean, rstd, st);
  if (dtype == MTNLG_BF16)
    return ln_fwd_launch<bf16>(T, h, x, partial, bias, gamma, beta, eps, xsum, out, mean, rstd, st);
  return MTNLG_INVALID_ARG;
}

size_t mtnlg_layernorm_bwd_workspace(int64_t T, int64_t h) {
  if (T <= 0 || h <= 0) return 0;
  return (size_t)3 * ln_bwd_workgroups(T) * (size_t)h * sizeof(float);
}

int mtnlg_layernorm_bwd(int dtype, int64_t T, int64_t h, const void *x, const void *gamma,
                        const float *mean, const float *rstd, const void *dout, const void *dres,
                        void *dx, void *dgamma, void *dbeta, void *colsum_dx, int grad_f32,
                        int accumulate, void *workspace, void *stream) {
  if (!x || !gamma || !mean || !rstd || !dout || !dx || !dgamma || !dbeta || !workspace)
    return MTNLG_NULL_POINTER;
  if (T <= 0 || h <= 0) return MTNLG_INVALID_ARG;
  if (h % 8 || h > 32768) return MTNLG_UNSUPPORTED_SHAPE;
  hipStream_t st = (hipStream_t)stream;
  if (dtype == MTNLG_F32)
    return ln_bwd_launch<float>(T, h, x, gamma, mean, rstd, dout, dres, dx, dgamma, dbeta, colsum_dx,
                                1, accumulate, workspace, st);
  if (dtype == MTNLG_BF16)
    return ln_bwd_launch<bf16>(T, h, x, gamma, mean, rstd, dout, dres, dx, dgamma, dbeta, colsum_dx,
                               grad_f32, accumulate, workspace, st);
  return MTNLG_INVALID_ARG;
}

int mtnlg_gelu_fwd(int dtype, int gelu, int64_t count, const void *z, void *g, void *stream) {
  if (!z || !g) return MTNLG_NULL_POINTER;
  if (count <= 0 || (gelu != 0 && gelu != 1)) return MTNLG_INVALID_ARG;
  if (count % 8) return MTNLG_UNSUPPORTED_SHAPE;
  hipStream_t st = (hipStream_t)stream;
  LaunchScope scope(MTNLG_K_GELU, st);
  if (dtype == MTNLG_F32)
    gelu_fwd_kernel<float><<<ew_grid(count / 8), 256, 0, st>>>(count / 8, (const float *)z, (float *)g, gelu);
  else if (dtype == MTNLG_BF16)
    gelu_fwd_kernel<bf16><<<ew_grid(count / 8), 256, 0, st>>>(count / 8, (const bf16 *)z, (bf16 *)g, gelu);
  else
    return MTNLG_INVALID_ARG;
  return check_launch();
}

int mtnlg_gelu_bwd(int dtype, int gelu, int64_t count, const void *z, const void *dg, void *dz,
                   void *stream) {
  if (!z || !dg || !dz) return MTNLG_NULL_POINTER;
  if (count <= 0 || (gelu != 0 && gelu != 1)) return MTNLG_INVALID_ARG;
  if (count % 8) return MTNLG_UNSUPPORTED_SHAPE;
  hipStream_t st = (hipStream_t)stream;
  LaunchScope scope(MTNLG_K_GELU, st);
  if (dtype == MTNLG_F32)
    gelu_bwd_kernel<float><<<ew_grid(count / 8), 256, 0, st>>>(count / 8, (const float *)z,
                                                               (const float *)dg, (float *)dz, gelu);
  else if (dtype == MTNLG_BF16)
    gelu_bwd_kernel<bf16><<<ew_grid(count / 8), 256, 0, st>>>(count / 8, (const bf16 *)z,
                                                              (const bf16 *)dg, (bf16 *)dz, gelu);
  else
    return MTNLG_INVALID_ARG;
  return check_launch();
}

size_t mtnlg_colsum_workspace(int64_t T, int64_t C) {
  if (T <= 0 || C <= 0) return 0;
  return (size_t)colreduce_rowblocks(T) * (size_t)C * sizeof(float);
}

int mtnlg_colsum(int dtype, int64_t T, int64_t C, const void *in, void *out, int out_f32,
                 int accumulate, void *workspace, void *stream) {
  if (!in || !out || !workspace) return MTNLG_NULL_POINTER;
  if (T <= 0 || C <= 0) return MTNLG_INVALID_ARG;
  if (C % 8) return MTNLG_UNSUPPORTED_SHAPE;
  hipStream_t st = (hipStream_t)stream;
  if (dtype == MTNLG_F32) return colsum_launch<float>(T, C, in, out, 1, accumulate, workspace, st);
  if (dtype == MTNLG_BF16) return colsum_launch<bf16>(T, C, in, out, out_f32, accumulate, workspace, st);
  return MTNLG_INVALID_ARG;
}

int mtnlg_bias_residual(int dtype, int64_t T, int64_t h, const void *res, const void *partial,
                        const void *bias, void *out, void *stream) {
  if (!res || !partial || !out) return MTNLG_NULL_POINTER;
  if (T <= 0 || h <= 0) return MTNLG_INVALID_ARG;
  if (h % 8) return MTNLG_UNSUPPORTED_SHAPE;
  hipStream_t st = (hipStream_t)stream;
  LaunchScope scope(MTNLG_K_ELEMENTWISE, st);
  if (dtype == MTNLG_F32)
    bias_residual_kernel<float><<<ew_grid(T * h / 8), 256, 0, st>>>(T, h, (const float *)res,
                                                                    (const float *)partial,
                                                                    (const float *)bias, (float *)out);
  else if (dtype == MTNLG_BF16)
    bias_residual_kernel<bf16><<<ew_grid(T * h / 8), 256, 0, st>>>(T, h, (const bf16 *)res,
                                                                   (const bf16 *)partial,
                                                                   (const bf16 *)bias, (bf16 *)out);
  else
    return MTNLG_INVALID_ARG;
  return check_launch();
}

// ---- column sum for callers that cannot allocate device memory -------------------------------------------
// Same kernels as mtnlg_colsum; the stage-1 partials ([row blocks <= 32][C] floats) live in a file-scope device
// array instead of a caller's workspace.  Every GPU the library runs on holds its own copy of the array (4 MiB)
// at its own address until the process ends; in host code the array's name is only a handle, so the address is
// asked for once per device (with that device current) and kept.
namespace mtnlg {
constexpr int64_t COLSUM_STATIC_MAX_COLS = 32768;
constexpr int COLSUM_STATIC_MAX_DEVICES = 64;
static __device__ __align__(256) float scratch[32 * COLSUM_STATIC_MAX_COLS];

static std::mutex g_scratch_mutex;
static float *g_scratch_ptr[COLSUM_STATIC_MAX_DEVICES] = {};

// Device address of `scratch` on the current device, nullptr on failure.
static float *scratch_on_current_device() {
  int device = -1;
  if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= COLSUM_STATIC_MAX_DEVICES) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[device]) {
    float *ptr = nullptr;
    if (hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
    g_scratch_ptr[device] = ptr;
  }
  return g_scratch_ptr[device];
}
}  // namespace mtnlg

int64_t mtnlg_colsum_static_max_columns(void) { return COLSUM_STATIC_MAX_COLS; }

int mtnlg_colsum_static(int dtype, int64_t T, int64_t C, const void *in, void *out, int out_f32, int accumulate,
                        void *stream) {
  if (!in || !out) return MTNLG_NULL_POINTER;
  if (T <= 0 || C <= 0) return MTNLG_INVALID_ARG;
  if (dtype != MTNLG_F32 && dtype != MTNLG_BF16) return MTNLG_INVALID_ARG;
  if (C % 8) return MTNLG_UNSUPPORTED_SHAPE;
  if (C > COLSUM_STATIC_MAX_COLS) return MTNLG_WORKSPACE_TOO_SMALL;   // the partials would not fit the static array
  float *ptr = scratch_on_current_device();
  if (!ptr) return MTNLG_HIP_ERROR;
  // Stage 1 writes every partial that stage 2 reads ([row blocks][C], all columns < C), so nothing in the array
  // has to start at zero and what an earlier, larger call left behind is never read.
  hipStream_t st = (hipStream_t)stream;
  if (dtype == MTNLG_F32) return colsum_launch<float>(T, C, in, out, 1, accumulate, ptr, st);
  return colsum_launch<bf16>(T, C, in, out, out_f32, accumulate, ptr, st);
}

}  // extern "C"
