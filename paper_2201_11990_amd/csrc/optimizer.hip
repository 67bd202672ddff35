// Optimizer step on one rank's parameter slice (Section 3.2 of the paper: Adam with
// beta1 = 0.9, beta2 = 0.95, epsilon = 1e-8, gradient-norm clipping at 1.0, weight decay 0.1;
// Section 2.1: fp32 copies of weights and gradients plus the two Adam states next to the
// half-precision weights, 20 bytes per parameter).  Two HBM-bound kernels:
//   squared gradient norm  : deterministic two-stage sum (fixed block ranges, fixed tree),
//                            fp64 accumulation, 4 bytes read per parameter;
//   fused Adam step        : per parameter reads gradient, weight and both moments (16 bytes),
//                            writes weight and moments back and the bf16 weight for the next
//                            forward pass (14 bytes); the clipping factor comes from a device
//                            scalar so that nothing synchronises with the host.
// Every lane moves 16 bytes per access, lanes on consecutive addresses.
#include <math.h>

#include "common.h"

namespace mtnlg {

namespace {

constexpr int kNormBlocks = 2048;   // stage-1 partial sums

__global__ __launch_bounds__(256) void sqnorm_stage1(int64_t count, const float *__restrict__ g, double *__restrict__ partial) {
  // block b owns the contiguous range [b * chunk, (b + 1) * chunk), chunk a multiple of 1024 elements
  const int64_t chunk = ((count + kNormBlocks - 1) / kNormBlocks + 1023) / 1024 * 1024;
  const int64_t lo = blockIdx.x * chunk, hi = lo + chunk < count ? lo + chunk : count;
  double s = 0.0;
  for (int64_t i = lo + threadIdx.x * 4; i < hi; i += 1024) {
    if (i + 4 <= hi) {
      const f32x4 v = *reinterpret_cast<const f32x4 *>(g + i);
      s += (double)v[0] * v[0] + (double)v[1] * v[1] + (double)v[2] * v[2] + (double)v[3] * v[3];
    } else {
      for (int64_t j = i; j < hi; ++j) s += (double)g[j] * g[j];
    }
  }
  __shared__ double red[256];
  red[threadIdx.x] = s;
  __syncthreads();
  for (int off = 128; off > 0; off >>= 1) {
    if ((int)threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
    __syncthreads();
  }
  if (threadIdx.x == 0) partial[blockIdx.x] = red[0];
}

__global__ __launch_bounds__(256) void sqnorm_stage2(const double *__restrict__ partial, float *__restrict__ out, int accumulate) {
  __shared__ double red[256];
  double s = 0.0;
  for (int i = threadIdx.x; i < kNormBlocks; i += 256) s += partial[i];
  red[threadIdx.x] = s;
  __syncthreads();
  for (int off = 128; off > 0; off >>= 1) {
    if ((int)threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
    __syncthreads();
  }
  if (threadIdx.x == 0) out[0] = (float)(accumulate ? (double)out[0] + red[0] : red[0]);
}

struct AdamArgs {
  float lr, beta1, beta2, eps, wd, max_norm;
  float inv_c1, inv_c2;   // 1 / (1 - beta1^t), 1 / (1 - beta2^t)
};

__device__ __forceinline__ void adam_one(const AdamArgs &a, float coef, float g, float &p, float &m, float &v) {
  g *= coef;
  m = a.beta1 * m + (1.0f - a.beta1) * g;
  v = a.beta2 * v + (1.0f - a.beta2) * g * g;
  const float mh = m * a.inv_c1, vh = v * a.inv_c2;
  p = p - a.lr * (mh / (sqrtf(vh) + a.eps) + a.wd * p);
}

__global__ __launch_bounds__(256) void adam_kernel(AdamArgs a, int64_t count, float *__restrict__ p, float *__restrict__ m,
                                                   float *__restrict__ v, const float *__restrict__ g,
                                                   bf16 *__restrict__ w16, const float *__restrict__ sqnorm) {
  float coef = 1.0f;
  if (sqnorm != nullptr && a.max_norm > 0.0f) coef = fminf(1.0f, a.max_norm / (sqrtf(sqnorm[0]) + 1e-6f));
  const int64_t stride = (int64_t)gridDim.x * 256 * 4;
  for (int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4; i < count; i += stride) {
    if (i + 4 <= count) {
      f32x4 pv = *reinterpret_cast<const f32x4 *>(p + i), mv = *reinterpret_cast<const f32x4 *>(m + i);
      f32x4 vv = *reinterpret_cast<const f32x4 *>(v + i);
      const f32x4 gv = *reinterpret_cast<const f32x4 *>(g + i);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        float pe = pv[e], me = mv[e], ve = vv[e];
        adam_one(a, coef, gv[e], pe, me, ve);
        pv[e] = pe;
        mv[e] = me;
        vv[e] = ve;
      }
      *reinterpret_cast<f32x4 *>(p + i) = pv;
      *reinterpret_cast<f32x4 *>(m + i) = mv;
      *reinterpret_cast<f32x4 *>(v + i) = vv;
      if (w16 != nullptr) {
        bf16x4 h;
#pragma unroll
        for (int e = 0; e < 4; ++e) h[e] = (bf16)pv[e];
        *reinterpret_cast<bf16x4 *>(w16 + i) = h;
      }
    } else {
      for (int64_t j = i; j < count; ++j) {
        float pj = p[j], mj = m[j], vj = v[j];
        adam_one(a, coef, g[j], pj, mj, vj);
        p[j] = pj;
        m[j] = mj;
        v[j] = vj;
        if (w16 != nullptr) w16[j] = (bf16)pj;
      }
    }
  }
}

}  // namespace

}  // namespace mtnlg

using namespace mtnlg;

extern "C" {

size_t mtnlg_grad_sqnorm_workspace(void) { return kNormBlocks * sizeof(double); }

int mtnlg_grad_sqnorm(int64_t count, const float *grad, void *workspace, float *sqnorm, int accumulate, void *stream) {
  if (!grad || !workspace || !sqnorm) return MTNLG_NULL_POINTER;
  if (count <= 0) return MTNLG_INVALID_ARG;
  if (((uintptr_t)grad & 15) || ((uintptr_t)workspace & 7)) return MTNLG_INVALID_ARG;
  hipStream_t st = (hipStream_t)stream;
  LaunchScope scope(MTNLG_K_ELEMENTWISE, st);
  sqnorm_stage1<<<kNormBlocks, 256, 0, st>>>(count, grad, (double *)workspace);
  MTNLG_TRY(check_launch());
  sqnorm_stage2<<<1, 256, 0, st>>>((const double *)workspace, sqnorm, accumulate ? 1 : 0);
  return check_launch();
}

int mtnlg_adam_step(const mtnlg_adam_desc *desc, int64_t count, float *master, float *m, float *v, const float *grad,
                    void *weight_bf16, const float *sqnorm, void *stream) {
  if (!desc || !master || !m || !v || !grad) return MTNLG_NULL_POINTER;
  if (count <= 0 || desc->step < 1) return MTNLG_INVALID_ARG;
  if (!(desc->beta1 >= 0.0f && desc->beta1 < 1.0f && desc->beta2 >= 0.0f && desc->beta2 < 1.0f && desc->eps > 0.0f))
    return MTNLG_INVALID_ARG;
  if (((uintptr_t)master | (uintptr_t)m | (uintptr_t)v | (uintptr_t)grad) & 15) return MTNLG_INVALID_ARG;
  if ((uintptr_t)weight_bf16 & 7) return MTNLG_INVALID_ARG;
  AdamArgs a;
  a.lr = desc->lr;
  a.beta1 = desc->beta1;
  a.beta2 = desc->beta2;
  a.eps = desc->eps;
  a.wd = desc->weight_decay;
  a.max_norm = desc->max_grad_norm;
  a.inv_c1 = (float)(1.0 / (1.0 - pow((double)desc->beta1, (double)desc->step)));
  a.inv_c2 = (float)(1.0 / (1.0 - pow((double)desc->beta2, (double)desc->step)));
  hipStream_t st = (hipStream_t)stream;
  int64_t blocks = (count + 1023) / 1024;
  if (blocks > 8192) blocks = 8192;   // grid-stride beyond: 32 workgroups per CU
  LaunchScope scope(MTNLG_K_ELEMENTWISE, st);
  adam_kernel<<<(unsigned)blocks, 256, 0, st>>>(a, count, master, m, v, grad, (bf16 *)weight_bf16, sqnorm);
  return check_launch();
}

}  // extern "C"
