// Measurement aids: what this chip sustains on the two resources the layer's kernels are bound by, measured
// with the same data and in the same process as the benchmark.
//
//  * mtnlg_calibrate_mfma: a loop of nothing but v_mfma_f32_16x16x32_bf16 (the instruction of the GEMM and
//    attention kernels) on the caller's operands, 8 waves per compute unit (two per SIMD, as in the GEMM), every
//    wave working on 4 x 2 accumulator blocks with two k-steps of operand fragments, in the order the GEMM kernel
//    issues them: both k-steps of a block back to back, neighbouring instructions sharing an operand (the order
//    matters: under the power limit this one sustains 8 % more than k-step after k-step).  No LDS, no memory
//    traffic inside the loop: its rate is the matrix pipes' rate at the clock the board's power limit allows for
//    this data.
//  * mtnlg_calibrate_copy: a plain streaming copy, 16 bytes per lane: the HBM rate a kernel of this library
//    can expect, and a kernel of known size to scale the profiler's byte counters by.
#include "common.h"

namespace mtnlg {

constexpr int CAL_WAVES = 8, CAL_NA = 4, CAL_NB = 2, CAL_KSTEPS = 2;

__global__ __launch_bounds__(64 * CAL_WAVES, 1) void calibrate_mfma_kernel(const bf16 *__restrict__ operands, int iters,
                                                                           float *__restrict__ out) {
  // every thread takes its own 12 fragments of 8 values from the operand buffer
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const bf16x8 *src = reinterpret_cast<const bf16x8 *>(operands) + t * (CAL_KSTEPS * (CAL_NA + CAL_NB));
  bf16x8 a[CAL_KSTEPS][CAL_NA], b[CAL_KSTEPS][CAL_NB];
#pragma unroll
  for (int k = 0; k < CAL_KSTEPS; ++k) {
#pragma unroll
    for (int i = 0; i < CAL_NA; ++i) a[k][i] = src[k * (CAL_NA + CAL_NB) + i];
#pragma unroll
    for (int j = 0; j < CAL_NB; ++j) b[k][j] = src[k * (CAL_NA + CAL_NB) + CAL_NA + j];
  }
  f32x4 acc[CAL_NA][CAL_NB];
#pragma unroll
  for (int i = 0; i < CAL_NA; ++i)
#pragma unroll
    for (int j = 0; j < CAL_NB; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.0f;
  for (int it = 0; it < iters; ++it) {
    // a snake through (i, j, k-step): every step keeps the accumulator or one operand
#pragma unroll
    for (int n = 0; n < CAL_NA * CAL_NB * CAL_KSTEPS; ++n) {
      const int i = n / (CAL_NB * CAL_KSTEPS);
      const int m = (i & 1) ? CAL_NB * CAL_KSTEPS - 1 - n % (CAL_NB * CAL_KSTEPS) : n % (CAL_NB * CAL_KSTEPS);
      const int j = m / CAL_KSTEPS, k = (m % CAL_KSTEPS) ^ (j & 1);
      acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[k][i], b[k][j], acc[i][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  float s = 0.0f;
#pragma unroll
  for (int i = 0; i < CAL_NA; ++i)
#pragma unroll
    for (int j = 0; j < CAL_NB; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) s += acc[i][j][e];
  out[t] = s;
}

__global__ __launch_bounds__(256) void calibrate_copy_kernel(const f32x4 *__restrict__ src, f32x4 *__restrict__ dst,
                                                             int64_t n16) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (int64_t)gridDim.x * 256) dst[i] = src[i];
}

}  // namespace mtnlg

using namespace mtnlg;

extern "C" {

size_t mtnlg_calibrate_mfma_operand_bytes(int workgroups) {
  return workgroups > 0 ? (size_t)workgroups * 64 * CAL_WAVES * (CAL_KSTEPS * (CAL_NA + CAL_NB)) * 16 : 0;
}

int64_t mtnlg_calibrate_mfma_flops(int workgroups, int iters) {
  if (workgroups <= 0 || iters <= 0) return 0;
  return (int64_t)workgroups * CAL_WAVES * iters * (CAL_NA * CAL_NB * CAL_KSTEPS) * (2LL * 16 * 16 * 32);
}

int mtnlg_calibrate_mfma(int workgroups, int iters, const void *operands, float *out, void *stream) {
  if (!operands || !out) return MTNLG_NULL_POINTER;
  if (workgroups <= 0 || iters <= 0 || workgroups > (1 << 20)) return MTNLG_INVALID_ARG;
  calibrate_mfma_kernel<<<dim3((unsigned)workgroups), 64 * CAL_WAVES, 0, (hipStream_t)stream>>>((const bf16 *)operands,
                                                                                               iters, out);
  return check_launch();
}

int mtnlg_calibrate_copy(void *dst, const void *src, int64_t bytes, void *stream) {
  if (!dst || !src) return MTNLG_NULL_POINTER;
  if (bytes <= 0 || bytes % 16 || ((uintptr_t)dst | (uintptr_t)src) % 16) return MTNLG_INVALID_ARG;
  calibrate_copy_kernel<<<dim3(256 * 8), 256, 0, (hipStream_t)stream>>>((const f32x4 *)src, (f32x4 *)dst, bytes / 16);
  return check_launch();
}

}  // extern "C"
