// Measurement aids: what this chip sustains on the two resources the layer's kernels are bound by, measured
// with the same data and in the same process as the benchmark.
//
//  * mtnlg_calibrate_mfma: a loop of nothing but v_mfma_f32_16x16x32_bf16 (the instruction of the GEMM and
//    attention kernels) on the caller's operands, 8 waves per compute unit (two per SIMD, as in the GEMM), every
//    wave cycling through 4 x 2 fragments and 8 accumulator blocks so that operands change from one
//    instruction to the next.  No LDS, no memory traffic inside the loop: its rate is the matrix pipes' rate
//    at the clock the board's power limit allows for this data.
//  * mtnlg_calibrate_copy: a plain streaming copy, 16 bytes per lane: the HBM rate a kernel of this library
//    can expect, and a kernel of known size to scale the profiler's byte counters by.
#include "common.h"

namespace mtnlg {

constexpr int CAL_WAVES = 8, CAL_NA = 4, CAL_NB = 2;

__global__ __launch_bounds__(64 * CAL_WAVES, 1) void calibrate_mfma_kernel(const bf16 *__restrict__ operands, int iters,
                                                                           float *__restrict__ out) {
  // every thread takes its own 6 fragments of 8 values from the operand buffer
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const bf16x8 *src = reinterpret_cast<const bf16x8 *>(operands) + t * (CAL_NA + CAL_NB);
  bf16x8 a[CAL_NA], b[CAL_NB];
#pragma unroll
  for (int i = 0; i < CAL_NA; ++i) a[i] = src[i];
#pragma unroll
  for (int j = 0; j < CAL_NB; ++j) b[j] = src[CAL_NA + j];
  f32x4 acc[CAL_NA][CAL_NB];
#pragma unroll
  for (int i = 0; i < CAL_NA; ++i)
#pragma unroll
    for (int j = 0; j < CAL_NB; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.0f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < CAL_NA; ++i)
#pragma unroll
      for (int j = 0; j < CAL_NB; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
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
  return workgroups > 0 ? (size_t)workgroups * 64 * CAL_WAVES * (CAL_NA + CAL_NB) * 16 : 0;
}

int64_t mtnlg_calibrate_mfma_flops(int workgroups, int iters) {
  if (workgroups <= 0 || iters <= 0) return 0;
  return (int64_t)workgroups * CAL_WAVES * iters * (CAL_NA * CAL_NB) * (2LL * 16 * 16 * 32);
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
