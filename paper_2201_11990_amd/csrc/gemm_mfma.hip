// bf16 GEMM on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16), fp32 accumulate.
//
//   C[M,N] = op(A) * op(B)   with both operands brought into LDS as [row][k] tiles
//   ("row" = m for A, n for B; 64 k per tile = 128 bytes per row), whatever their
//   layout in memory:
//     K-contiguous operand (x in x W^T, W in x W^T, dY in dY W): 16-byte global loads
//       land in LDS unchanged;
//     row-contiguous operand (W in dY W, dY and X in dY^T X): each thread loads an
//       8(k) x 8(row) block with 16-byte loads along the row axis, transposes it in
//       registers and writes 16-byte k-runs.
//   Inside a tile, the 16-byte chunk c of row r sits at chunk position
//   c ^ (r & 7) ^ ((r >> 3) & 7), which keeps both kinds of LDS writes and the
//   MFMA operand reads (32 rows x one chunk per half-wave) free of bank conflicts.
//
// Workgroup = 256 threads = 2 x 2 waves; workgroup tile BM x BN, wave tile
// (BM/2) x (BN/2) built from 32x32 MFMA blocks; K advances 64 at a time through two
// LDS stages (global loads for tile i+1 are in flight while tile i is multiplied).
// Workgroups are numbered so that the 8 XCDs (workgroup id mod 8) each own a
// contiguous run of column-major tiles: neighbours in an XCD's L2 share B panels.
//
// Requirements: K % 8 == 0 and N % 8 == 0; a row-contiguous A also needs M % 8 == 0
// (16-byte accesses never straddle an edge).  Other edges are handled by clamped
// loads and masked stores.
#include "common.h"

namespace mtnlg {

namespace {

constexpr int BK = 64;

struct GemmArgs {
  int64_t M, N, K;
  const bf16 *A, *B;
  int64_t lda, ldb;
  void *C;
  int64_t ldc;
  EpiArgs ea;
  int tiles_m, tiles_n, per_xcd;
};

__device__ __forceinline__ int swz(int r, int c) { return (c ^ (r & 7) ^ ((r >> 3) & 7)) << 4; }

typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(8))) short i16x8;
typedef __attribute__((ext_vector_type(4))) short i16x4;

// ---- global -> registers -> LDS for one ROWS x 64 operand tile ----------------
// K-contiguous source: ROWS*8 chunks of 16 B, ROWS/32 per thread.
template <int ROWS>
struct LoadK {
  static constexpr int N = ROWS / 32;
  i32x4 r[N];
  template <bool KTAIL>
  __device__ __forceinline__ void fetch(const bf16 *base, int64_t ld, int64_t rows_valid, int64_t k0, int64_t K) {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      int q = threadIdx.x + 256 * i;
      int row = q >> 3, c = q & 7;
      int64_t rr = row < rows_valid ? row : rows_valid - 1;
      int64_t k = k0 + c * 8;
      if constexpr (KTAIL) {
        i32x4 v = {0, 0, 0, 0};
        if (k < K) v = *reinterpret_cast<const i32x4 *>(base + rr * ld + k);
        r[i] = v;
      } else {
        r[i] = *reinterpret_cast<const i32x4 *>(base + rr * ld + k);
      }
    }
  }
  __device__ __forceinline__ void stash(char *lds) const {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      int q = threadIdx.x + 256 * i;
      int row = q >> 3, c = q & 7;
      *reinterpret_cast<i32x4 *>(lds + row * 128 + swz(row, c)) = r[i];
    }
  }
};

// Row-contiguous source ([k][row] in memory): each thread owns KB k-rows x 8 rows.
template <int ROWS>
struct LoadT {
  static constexpr int KB = ROWS / 32;  // 8 for 256 rows, 4 for 128
  static constexpr int RB = ROWS / 8;   // row blocks
  i16x8 r[KB];
  template <bool KTAIL>
  __device__ __forceinline__ void fetch(const bf16 *base, int64_t ld, int64_t rows_valid, int64_t k0, int64_t K) {
    const int rb = threadIdx.x % RB, kb = threadIdx.x / RB;
    int64_t row = rb * 8;
    if (row + 8 > rows_valid) row = rows_valid - 8;  // rows_valid >= 8 and a multiple of 8
#pragma unroll
    for (int j = 0; j < KB; ++j) {
      int64_t k = k0 + kb * KB + j;
      if constexpr (KTAIL) {
        i16x8 v = {0, 0, 0, 0, 0, 0, 0, 0};
        if (k < K) v = *reinterpret_cast<const i16x8 *>(base + k * ld + row);
        r[j] = v;
      } else {
        r[j] = *reinterpret_cast<const i16x8 *>(base + k * ld + row);
      }
    }
  }
  __device__ __forceinline__ void stash(char *lds) const {
    const int rb = threadIdx.x % RB, kb = threadIdx.x / RB;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int row = rb * 8 + i;
      if constexpr (KB == 8) {
        i16x8 t;
#pragma unroll
        for (int j = 0; j < 8; ++j) t[j] = r[j][i];
        *reinterpret_cast<i16x8 *>(lds + row * 128 + swz(row, kb)) = t;
      } else {
        i16x4 t;
#pragma unroll
        for (int j = 0; j < 4; ++j) t[j] = r[j][i];
        *reinterpret_cast<i16x4 *>(lds + row * 128 + swz(row, kb >> 1) + (kb & 1) * 8) = t;
      }
    }
  }
};

template <int ROWS, bool T>
struct Loader;
template <int ROWS>
struct Loader<ROWS, false> : LoadK<ROWS> {};
template <int ROWS>
struct Loader<ROWS, true> : LoadT<ROWS> {};

// KTAIL: K is not a multiple of 64, so the last K-slab is partly zero-filled.
template <int BM, int BN, bool AT, bool BT, bool KTAIL>
__global__ __launch_bounds__(256, 1) void gemm_bf16_kernel(GemmArgs g) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  constexpr int WM = BM / 2, WN = BN / 2, TM = WM / 32, TN = WN / 32;
  constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2, STAGE = A_BYTES + B_BYTES;

  // XCD-aware tile numbering
  const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
  const int tile = xcd * g.per_xcd + local;
  if (local >= g.per_xcd || tile >= g.tiles_m * g.tiles_n) return;
  const int tm = tile % g.tiles_m, tn = tile / g.tiles_m;
  const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * BN;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  const bf16 *Abase = AT ? g.A + m0 : g.A + m0 * g.lda;
  const bf16 *Bbase = BT ? g.B + n0 : g.B + n0 * g.ldb;
  const int64_t a_rows = g.M - m0, b_rows = g.N - n0;

  Loader<BM, AT> la;
  Loader<BN, BT> lb;

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

  const int nk = (int)((g.K + BK - 1) / BK);
  la.template fetch<KTAIL>(Abase, g.lda, a_rows, 0, g.K);
  lb.template fetch<KTAIL>(Bbase, g.ldb, b_rows, 0, g.K);
  la.stash(smem);
  lb.stash(smem + A_BYTES);
  __syncthreads();

  // per-lane fragment addressing: row (lane & 31) of a 32-row block, chunk 2*kk + (lane >> 5)
  const int frow = lane & 31, fchunk = lane >> 5;
  for (int it = 0; it < nk; ++it) {
    char *cur = smem + (it & 1) * STAGE;
    char *nxt = smem + ((it + 1) & 1) * STAGE;
    const bool more = it + 1 < nk;
    if (more) {
      la.template fetch<KTAIL>(Abase, g.lda, a_rows, (int64_t)(it + 1) * BK, g.K);
      lb.template fetch<KTAIL>(Bbase, g.ldb, b_rows, (int64_t)(it + 1) * BK, g.K);
    }
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      bf16x8 af[TM], bfr[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        int row = wm * WM + i * 32 + frow;
        af[i] = *reinterpret_cast<const bf16x8 *>(cur + row * 128 + swz(row, kk * 2 + fchunk));
      }
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        int row = wn * WN + j * 32 + frow;
        bfr[j] = *reinterpret_cast<const bf16x8 *>(cur + A_BYTES + row * 128 + swz(row, kk * 2 + fchunk));
      }
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    if (more) {
      la.stash(nxt);
      lb.stash(nxt + A_BYTES);
    }
    __syncthreads();
  }

  // Epilogue through LDS, one half (wm) of the tile at a time: accumulators are
  // written as a [BM/2][BN] fp32 image (element e of lane l is row 8*(e/4) + 4*(l/32)
  // + e%4, column l%32 of its 32x32 block), then every thread walks the image in
  // 8-element row segments and applies bias / GeLU / residual / accumulate with
  // 16-byte global accesses.
  float *img = reinterpret_cast<float *>(smem);
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    if (wm == half) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int row = i * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
            const int col = wn * WN + j * 32 + (lane & 31);
            img[row * BN + col] = acc[i][j][e];
          }
    }
    __syncthreads();
    const uint32_t flags = g.ea.flags;
    for (int idx = threadIdx.x; idx < (BM / 2) * (BN / 8); idx += 256) {
      const int row = idx / (BN / 8), cv = idx % (BN / 8);
      const int64_t m = m0 + half * (BM / 2) + row, n = n0 + cv * 8;
      if (m >= g.M || n >= g.N) continue;
      float v[8], t[8];
      const f32x4 lo = *reinterpret_cast<const f32x4 *>(img + row * BN + cv * 8);
      const f32x4 hi = *reinterpret_cast<const f32x4 *>(img + row * BN + cv * 8 + 4);
#pragma unroll
      for (int e = 0; e < 4; ++e) { v[e] = lo[e]; v[4 + e] = hi[e]; }
      const int64_t off = m * g.ldc + n;
      if (flags & MTNLG_EPI_BIAS) {
        load8(static_cast<const bf16 *>(g.ea.bias) + n, t);
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] += t[e];
      }
      if (flags & MTNLG_EPI_GELU) {
        store8(static_cast<bf16 *>(g.ea.aux) + off, v);
        const bool erf_form = (flags & MTNLG_EPI_GELU_ERF) != 0;
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = gelu_f(v[e], erf_form);
      }
      if (flags & MTNLG_EPI_RESIDUAL) {
        load8(static_cast<const bf16 *>(g.ea.aux) + off, t);
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] += t[e];
      }
      if (flags & MTNLG_EPI_OUT_F32) {
        float *c = static_cast<float *>(g.C) + off;
        if (flags & MTNLG_EPI_ACCUMULATE) {
          load8(c, t);
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] += t[e];
        }
        store8(c, v);
      } else {
        bf16 *c = static_cast<bf16 *>(g.C) + off;
        if (flags & MTNLG_EPI_ACCUMULATE) {
          load8(c, t);
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] += t[e];
        }
        store8(c, v);
      }
    }
    __syncthreads();
  }
}

template <int BM, int BN, bool AT, bool BT, bool KTAIL>
int launch_k(const GemmArgs &in, hipStream_t st) {
  GemmArgs g = in;
  g.tiles_m = (int)((g.M + BM - 1) / BM);
  g.tiles_n = (int)((g.N + BN - 1) / BN);
  const int64_t tiles = (int64_t)g.tiles_m * g.tiles_n;
  if (tiles > (1 << 28)) return MTNLG_UNSUPPORTED_SHAPE;
  g.per_xcd = (int)((tiles + 7) / 8);
  constexpr int smem = 2 * (BM + BN) * BK * 2;
  static bool attr_set = false;
  if (!attr_set) {
    if (hipFuncSetAttribute((const void *)gemm_bf16_kernel<BM, BN, AT, BT, KTAIL>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, smem) != hipSuccess)
      return MTNLG_HIP_ERROR;
    attr_set = true;
  }
  gemm_bf16_kernel<BM, BN, AT, BT, KTAIL><<<dim3((unsigned)(g.per_xcd * 8)), 256, smem, st>>>(g);
  return check_launch();
}

template <int BM, int BN, bool AT, bool BT>
int launch(const GemmArgs &g, hipStream_t st) {
  return g.K % BK ? launch_k<BM, BN, AT, BT, true>(g, st) : launch_k<BM, BN, AT, BT, false>(g, st);
}

template <bool AT, bool BT>
int pick_tile(const GemmArgs &g, hipStream_t st) {
  // Few large tiles when the problem fills the chip several times over, smaller ones
  // otherwise so that the last round of workgroups is not mostly idle.
  auto rounds_eff = [&](int bm, int bn) {
    double tiles = (double)((g.M + bm - 1) / bm) * (double)((g.N + bn - 1) / bn);
    double rounds = ceil(tiles / 256.0);
    return tiles / (rounds * 256.0);
  };
  const double e256 = rounds_eff(256, 256), e128 = rounds_eff(128, 128) * 0.85;
  if (e256 >= e128) return launch<256, 256, AT, BT>(g, st);
  return launch<128, 128, AT, BT>(g, st);
}

}  // namespace

int gemm_mfma_bf16(int layout, int64_t M, int64_t N, int64_t K, const void *A, const void *B, void *C,
                   const void *bias, void *aux, uint32_t epi, hipStream_t stream) {
  if (K % 8 || N % 8) return MTNLG_UNSUPPORTED_SHAPE;
  const bool at = layout == MTNLG_GEMM_TN, bt = layout != MTNLG_GEMM_NT;
  if ((at && (M % 8 || M < 8)) || (bt && (N % 8 || N < 8))) return MTNLG_UNSUPPORTED_SHAPE;
  GemmArgs g;
  g.M = M; g.N = N; g.K = K;
  g.A = (const bf16 *)A; g.B = (const bf16 *)B;
  g.lda = at ? M : K;
  g.ldb = bt ? N : K;
  g.C = C; g.ldc = N;
  g.ea = EpiArgs{bias, aux, epi};
  g.tiles_m = g.tiles_n = g.per_xcd = 0;
  LaunchScope scope(MTNLG_K_GEMM_NT + layout, stream);
  if (!at && !bt) return pick_tile<false, false>(g, stream);
  if (!at && bt) return pick_tile<false, true>(g, stream);
  return pick_tile<true, true>(g, stream);
}

}  // namespace mtnlg
