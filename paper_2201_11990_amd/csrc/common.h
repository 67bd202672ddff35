// Shared declarations of the gfx950 layer-slice library: element types, status
// handling, launch bookkeeping.  Internal to the GPU library.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/mtnlg.h"

namespace mtnlg {

typedef __bf16 bf16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

// Storage <-> fp32.  float -> bf16 is round-to-nearest-even (v_cvt_pk_bf16_f32).
__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16 v) { return (float)v; }
template <typename E> __device__ __forceinline__ E from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16 from_f32<bf16>(float v) { return (bf16)v; }

// 8 consecutive elements as one unit (16 B for bf16, 32 B for float).
template <typename E> struct Vec8 { E v[8]; };
template <typename E> __device__ __forceinline__ void load8(const E *p, float (&out)[8]) {
  if constexpr (sizeof(E) == 2) {
    bf16x8 t = *reinterpret_cast<const bf16x8 *>(p);
#pragma unroll
    for (int i = 0; i < 8; ++i) out[i] = (float)t[i];
  } else {
    f32x4 a = *reinterpret_cast<const f32x4 *>(p);
    f32x4 b = *reinterpret_cast<const f32x4 *>(p + 4);
#pragma unroll
    for (int i = 0; i < 4; ++i) { out[i] = a[i]; out[4 + i] = b[i]; }
  }
}
template <typename E> __device__ __forceinline__ void store8(E *p, const float (&in)[8]) {
  if constexpr (sizeof(E) == 2) {
    bf16x8 t;
#pragma unroll
    for (int i = 0; i < 8; ++i) t[i] = (bf16)in[i];
    *reinterpret_cast<bf16x8 *>(p) = t;
  } else {
    f32x4 a, b;
#pragma unroll
    for (int i = 0; i < 4; ++i) { a[i] = in[i]; b[i] = in[4 + i]; }
    *reinterpret_cast<f32x4 *>(p) = a;
    *reinterpret_cast<f32x4 *>(p + 4) = b;
  }
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
  return v;
}

// Global -> LDS DMA (buffer_load ... lds): every lane moves 16 (or 4) bytes from base + its byte
// offset to LDS byte address lds_dst + 16 (or 4) * lane; lds_dst is the same for the whole wave.  Issued as
// inline assembly on purpose: once the compiler has seen such a write to LDS it makes the next LDS
// read it cannot tell apart from it wait for all outstanding memory operations, which empties a
// ring of several stages at every tile.  Kernels that use these count their outstanding DMAs
// themselves (s_waitcnt vmcnt(N) before the barrier that publishes a stage).  The LDS address
// travels in M0, which each statement declares as clobbered.
typedef __attribute__((ext_vector_type(4))) int dma_rsrc_t;
__device__ __forceinline__ dma_rsrc_t dma_rsrc(const void *base) {   // base: the same in every lane
  const uint64_t a = (uint64_t)base;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)a), hi = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32));
  return dma_rsrc_t{(int)lo, (int)(hi & 0xFFFF), -1, 0x00020000};
}
// LDS byte address of a pointer into shared memory (what M0 takes)
__device__ __forceinline__ uint32_t lds_address(const void *p) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void *)p;
}
// The compiler keeps M0 out of register allocation ("reserved") and warns about it in a clobber list; the
// clobber is still what tells it that its own M0 initialisations do not survive these statements.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
// TAG only tells call sites apart: the compiler merges identical asm statements on the two sides
// of a branch into one burst in front of it, which is exactly what spreading them tries to avoid.
template <int TAG = 0>
__device__ __forceinline__ void dma16(dma_rsrc_t rs, uint32_t lds_dst, uint32_t byte_offset) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds ; site %3" ::"s"(
                   __builtin_amdgcn_readfirstlane(lds_dst)),
               "v"(byte_offset), "s"(rs), "n"(TAG)
               : "memory", "m0");
}
// ... with a further byte offset that is the same in every lane (a scalar register: instructions whose lane offsets
// differ by uniform amounts share one vector register)
template <int TAG = 0>
__device__ __forceinline__ void dma16(dma_rsrc_t rs, uint32_t lds_dst, uint32_t byte_offset, uint32_t uniform_offset) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %4 offen lds ; site %3" ::"s"(
                   __builtin_amdgcn_readfirstlane(lds_dst)),
               "v"(byte_offset), "s"(rs), "n"(TAG), "s"(__builtin_amdgcn_readfirstlane(uniform_offset))
               : "memory", "m0");
}
template <int TAG = 0>
__device__ __forceinline__ void dma4(dma_rsrc_t rs, uint32_t lds_dst, uint32_t byte_offset) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, 0 offen lds ; site %3" ::"s"(
                   __builtin_amdgcn_readfirstlane(lds_dst)),
               "v"(byte_offset), "s"(rs), "n"(TAG)
               : "memory", "m0");
}

#pragma clang diagnostic pop

// GeLU in fp32.  tanh form: 0.5 z (1 + tanh(sqrt(2/pi) (z + 0.044715 z^3))); erf form:
// 0.5 z (1 + erf(z / sqrt 2)).
__device__ __forceinline__ float gelu_f(float z, bool erf_form) {
  if (erf_form) return 0.5f * z * (1.0f + erff(z * 0.70710678118654752f));
  float inner = 0.79788456080286536f * (z + 0.044715f * z * z * z);
  return 0.5f * z * (1.0f + tanhf(inner));
}
__device__ __forceinline__ float gelu_grad_f(float z, bool erf_form) {
  if (erf_form) {
    float cdf = 0.5f * (1.0f + erff(z * 0.70710678118654752f));
    float pdf = __expf(-0.5f * z * z) * 0.39894228040143268f;
    return cdf + z * pdf;
  }
  float inner = 0.79788456080286536f * (z + 0.044715f * z * z * z);
  float th = tanhf(inner);
  float dinner = 0.79788456080286536f * (1.0f + 3.0f * 0.044715f * z * z);
  return 0.5f * (1.0f + th) + 0.5f * z * (1.0f - th * th) * dinner;
}

// The tanh form again for the epilogue of the bf16 MFMA GEMMs, where the library tanhf (some 40 instructions an
// element) would cost a 256 x 320 tile 25 us of vector ALU time with the matrix pipes idle.  With
// s = 1 / (1 + exp(-2 u)), u = sqrt(2/pi) (z + 0.044715 z^3):  0.5 (1 + tanh u) = s, so GeLU(z) = z s and
// GeLU'(z) = s + 2 z u' s (1 - s), 1 - s = exp(-2 u) s.  Hardware exp2 and reciprocal (1 ulp each): relative error
// of a few 1e-7, two orders below the rounding of the bf16 result; no cancellation for very negative z, unlike
// 1 + tanh.  The exponent is clamped so that exp(-2 u) s stays finite.  8 and 13 instructions an element.
__device__ __forceinline__ float gelu_sigmoid_f(float z, float z2, float &e) {   // returns s, e = exp(-2 u)
  constexpr float K1 = -2.0f * 1.4426950408889634f * 0.79788456080286536f, K3 = K1 * 0.044715f;   // -2 u log2(e) = z (K1 + K3 z^2)
  e = __builtin_amdgcn_exp2f(fminf(z * (K1 + K3 * z2), 115.0f));
  return __builtin_amdgcn_rcpf(1.0f + e);
}
__device__ __forceinline__ float gelu_tanh_fast_f(float z) {
  float e;
  return z * gelu_sigmoid_f(z, z * z, e);
}
__device__ __forceinline__ float gelu_tanh_grad_fast_f(float z) {
  constexpr float D1 = 2.0f * 0.79788456080286536f, D3 = D1 * 3.0f * 0.044715f;   // 2 u' = D1 + D3 z^2
  const float z2 = z * z;
  float e;
  const float s = gelu_sigmoid_f(z, z2, e);
  return s + (z * (D1 + D3 * z2)) * (e * s) * s;
}

// GEMM epilogue shared by the GEMM kernels: bias, GeLU (pre-activation kept in aux),
// residual from aux, accumulate, fp32 or storage-dtype output.  One element at a time.
struct EpiArgs {
  const void *bias;
  void *aux;
  uint32_t flags;
};

template <typename E>
__device__ __forceinline__ void epilogue_store(const EpiArgs &ea, void *C, int64_t ldc, int64_t m,
                                               int64_t n, float acc) {
  if (ea.flags & MTNLG_EPI_BIAS) acc += to_f32(static_cast<const E *>(ea.bias)[n]);
  if (ea.flags & MTNLG_EPI_GELU) {
    static_cast<E *>(ea.aux)[m * ldc + n] = from_f32<E>(acc);
    acc = gelu_f(acc, (ea.flags & MTNLG_EPI_GELU_ERF) != 0);
  }
  if (ea.flags & MTNLG_EPI_RESIDUAL) acc += to_f32(static_cast<const E *>(ea.aux)[m * ldc + n]);
  if (ea.flags & MTNLG_EPI_GELU_GRAD)
    acc *= gelu_grad_f(to_f32(static_cast<const E *>(ea.aux)[m * ldc + n]), (ea.flags & MTNLG_EPI_GELU_ERF) != 0);
  if (ea.flags & MTNLG_EPI_OUT_F32) {
    float *c = static_cast<float *>(C) + m * ldc + n;
    *c = (ea.flags & MTNLG_EPI_ACCUMULATE) ? *c + acc : acc;
  } else {
    E *c = static_cast<E *>(C) + m * ldc + n;
    *c = from_f32<E>((ea.flags & MTNLG_EPI_ACCUMULATE) ? to_f32(*c) + acc : acc);
  }
}

// ---- host side -------------------------------------------------------------
// Brackets a launch with HIP events when per-class timing is on (profile.cpp).
struct LaunchScope {
  int cls;
  hipStream_t stream;
  long idx;  // slot in the record list, -1 when timing is off
  LaunchScope(int cls_, hipStream_t s);
  ~LaunchScope();
};

inline int check_launch() { return hipGetLastError() == hipSuccess ? MTNLG_OK : MTNLG_HIP_ERROR; }

// Kernel attributes (dynamic LDS size) are set once per device and kernel: `done` is a bit mask of
// the devices on which the attribute of one kernel has been set (devices beyond 63 set it every time).
// Thread-safe; a race sets the attribute twice, which is harmless.
inline bool attr_is_set(unsigned long long &done, int *device) {
  if (hipGetDevice(device) != hipSuccess) { *device = -1; return false; }
  if (*device < 0 || *device > 63) return false;
  return (__atomic_load_n(&done, __ATOMIC_ACQUIRE) >> *device) & 1ull;
}
inline void attr_mark_set(unsigned long long &done, int device) {
  if (device >= 0 && device <= 63) __atomic_fetch_or(&done, 1ull << device, __ATOMIC_RELEASE);
}

#define MTNLG_TRY(expr)            \
  do {                             \
    int st__ = (expr);             \
    if (st__ != MTNLG_OK) return st__; \
  } while (0)

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// internal launchers shared between translation units
int gemm_generic(int dtype, int layout, int64_t M, int64_t N, int64_t K, const void *A,
                 const void *B, void *C, const void *bias, void *aux, uint32_t epi,
                 hipStream_t stream);
// returns MTNLG_UNSUPPORTED_SHAPE when the MFMA kernel cannot take this problem
// ws (nullable): scratch for the split-K tail, see gemm_mfma_workspace_bytes
// prof_class: kernel class the launch is timed under (-1: MTNLG_K_GEMM_NT + layout)
// tile: one of gemm_tile, or -1 to let gemm_mfma_pick_tile choose (what every product call does)
enum gemm_tile { GEMM_TILE_GENERAL_256 = 0, GEMM_TILE_GENERAL_128, GEMM_TILE_STREAM_256x256, GEMM_TILE_STREAM_256x320 };
int gemm_mfma_bf16(int layout, int64_t M, int64_t N, int64_t K, const void *A, const void *B,
                   void *C, const void *bias, void *aux, uint32_t epi, void *ws, size_t ws_bytes,
                   hipStream_t stream, int prof_class = -1, int tile = -1);
int gemm_mfma_pick_tile(int layout, int64_t M, int64_t N, int64_t K, bool have_workspace);
size_t gemm_mfma_workspace_bytes(int layout, int64_t M, int64_t N, int64_t K);
int attention_fwd_simple(int dtype, int b, int s, int n, int d, float scale, const void *qkv,
                         void *a, float *lse, hipStream_t stream);
int attention_bwd_simple(int dtype, int b, int s, int n, int d, float scale, const void *qkv,
                         const void *a, const float *lse, const void *da, void *dqkv, void *ws,
                         hipStream_t stream);

// MFMA attention (bf16): which head sizes it takes, its scratch need, its launchers
bool attention_mfma_supported(int dtype, int d);
// ... and whether it takes this problem (grid limits, 32-bit byte offsets inside one sequence)
bool attention_mfma_takes(int dtype, int b, int s, int n, int d);
constexpr int ATTENTION_SIMPLE_MAX_SEQ = 4096;   // the vector-ALU kernels hold one row of scores in LDS
size_t attention_bwd_workspace_bytes(int b, int s, int n, int d);
int attention_fwd_mfma(int b, int s, int n, int d, float scale, const void *qkv, void *a, float *lse,
                       hipStream_t stream);
int attention_bwd_mfma(int b, int s, int n, int d, float scale, const void *qkv, const void *a,
                       const float *lse, const void *da, void *dqkv, void *ws, hipStream_t stream);

}  // namespace mtnlg
