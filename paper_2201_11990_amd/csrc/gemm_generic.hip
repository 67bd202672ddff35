// Shape-agnostic GEMM with fp32 accumulation on the vector ALUs: the fp32 path of
// the library and the fallback for bf16 problems whose sizes the MFMA kernel does
// not take.  64x64 output tile per 256-thread workgroup, 4x4 outputs per thread,
// operands staged through LDS in K-slabs of 16.  Any layout is expressed by
// element strides, every access is bounds-checked.
#include "common.h"

namespace mtnlg {

constexpr int GT = 64, GK = 16;

template <typename E>
__global__ __launch_bounds__(256) void gemm_generic_kernel(int64_t M, int64_t N, int64_t K,
                                                           const E *__restrict__ A, int64_t sam,
                                                           int64_t sak, const E *__restrict__ B,
                                                           int64_t sbn, int64_t sbk, void *C,
                                                           EpiArgs ea) {
  __shared__ float As[GK][GT + 1];
  __shared__ float Bs[GK][GT + 1];
  const int tid = threadIdx.x;
  const int tx = tid % 16, ty = tid / 16;
  const int64_t m0 = (int64_t)blockIdx.y * GT, n0 = (int64_t)blockIdx.x * GT;
  float acc[4][4] = {};
  for (int64_t k0 = 0; k0 < K; k0 += GK) {
    // 64x16 elements per operand, 4 per thread; walk the contiguous axis fastest
    for (int i = tid; i < GT * GK; i += 256) {
      int r, kk;
      if (sak == 1) { kk = i % GK; r = i / GK; } else { r = i % GT; kk = i / GT; }
      int64_t m = m0 + r, k = k0 + kk;
      As[kk][r] = (m < M && k < K) ? to_f32(A[m * sam + k * sak]) : 0.0f;
    }
    for (int i = tid; i < GT * GK; i += 256) {
      int r, kk;
      if (sbk == 1) { kk = i % GK; r = i / GK; } else { r = i % GT; kk = i / GT; }
      int64_t n = n0 + r, k = k0 + kk;
      Bs[kk][r] = (n < N && k < K) ? to_f32(B[n * sbn + k * sbk]) : 0.0f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < GK; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = As[kk][ty * 4 + i]; b[i] = Bs[kk][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int64_t m = m0 + ty * 4 + i, n = n0 + tx * 4 + j;
      if (m < M && n < N) epilogue_store<E>(ea, C, N, m, n, acc[i][j]);
    }
}

int gemm_generic(int dtype, int layout, int64_t M, int64_t N, int64_t K, const void *A,
                 const void *B, void *C, const void *bias, void *aux, uint32_t epi,
                 hipStream_t stream) {
  int64_t sam, sak, sbn, sbk;
  switch (layout) {
    case MTNLG_GEMM_NT: sam = K; sak = 1; sbn = K; sbk = 1; break;
    case MTNLG_GEMM_NN: sam = K; sak = 1; sbn = 1; sbk = N; break;
    case MTNLG_GEMM_TN: sam = 1; sak = M; sbn = 1; sbk = N; break;
    default: return MTNLG_INVALID_ARG;
  }
  dim3 grid((unsigned)((N + GT - 1) / GT), (unsigned)((M + GT - 1) / GT));
  if (grid.y > 65535) return MTNLG_UNSUPPORTED_SHAPE;
  EpiArgs ea{bias, aux, epi};
  LaunchScope scope(MTNLG_K_GEMM_NT + layout, stream);
  if (dtype == MTNLG_F32)
    gemm_generic_kernel<float><<<grid, 256, 0, stream>>>(M, N, K, (const float *)A, sam, sak,
                                                         (const float *)B, sbn, sbk, C, ea);
  else
    gemm_generic_kernel<bf16><<<grid, 256, 0, stream>>>(M, N, K, (const bf16 *)A, sam, sak,
                                                        (const bf16 *)B, sbn, sbk, C, ea);
  return check_launch();
}

}  // namespace mtnlg
