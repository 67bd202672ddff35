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
// Workgroup = WGM x WGN waves (256x256 tile on 2 x 4 waves by default, 128x128 on 2 x 2
// for small problems); wave tile built from 32x32 MFMA blocks; K advances 64 at a time
// through two LDS stages (global loads for slab i+1 are in flight while slab i is
// multiplied), with the LDS traffic interleaved between the MFMAs by scheduling hints.
// Workgroups are numbered so that the 8 XCDs (workgroup id mod 8) each own a
// contiguous run of column-major tiles: neighbours in an XCD's L2 share B panels.
//
// Requirements: K % 8 == 0 and N % 8 == 0; a row-contiguous A also needs M % 8 == 0
// (16-byte accesses never straddle an edge).  Other edges are handled by clamped
// loads and masked stores.
#include <stdlib.h>

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
// K-contiguous source: ROWS*8 chunks of 16 B spread over NTHR threads.
template <int ROWS, int NTHR>
struct LoadK {
  static constexpr int N = ROWS * 8 / NTHR;
  i32x4 r[N];
  template <bool KTAIL>
  __device__ __forceinline__ void fetch(const bf16 *base, int64_t ld, int64_t rows_valid, int64_t k0, int64_t K) {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      int q = threadIdx.x + NTHR * i;
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
      int q = threadIdx.x + NTHR * i;
      int row = q >> 3, c = q & 7;
      *reinterpret_cast<i32x4 *>(lds + row * 128 + swz(row, c)) = r[i];
    }
  }
};

// Row-contiguous source ([k][row] in memory): each thread owns KB k-rows x 8 rows.
// A wave covers 8 row-blocks x 8 k-blocks, which spreads its transposed LDS writes
// evenly over the banks.
template <int ROWS, int NTHR>
struct LoadT {
  static constexpr int KB = ROWS * 8 / NTHR;  // k-rows per thread: 8, 4 or 2
  static constexpr int RBH = ROWS / 64;       // groups of 8 row-blocks
  i16x8 r[KB];
  __device__ __forceinline__ static int row_block() {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    return (wave % RBH) * 8 + (lane & 7);
  }
  __device__ __forceinline__ static int k_block() {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    return (wave / RBH) * 8 + (lane >> 3);
  }
  template <bool KTAIL>
  __device__ __forceinline__ void fetch(const bf16 *base, int64_t ld, int64_t rows_valid, int64_t k0, int64_t K) {
    const int rb = row_block(), kb = k_block();
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
    const int rb = row_block(), kb = k_block();
    const int chunk = (kb * KB) >> 3, off = ((kb * KB) & 7) * 2;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int row = rb * 8 + i;
      typedef __attribute__((ext_vector_type(KB))) short vec_t;
      vec_t t;
#pragma unroll
      for (int j = 0; j < KB; ++j) t[j] = r[j][i];
      *reinterpret_cast<vec_t *>(lds + row * 128 + swz(row, chunk) + off) = t;
    }
  }
};

// Scheduling hints: REP times {NA instructions of class MASK_A, then NB of class MASK_B}.
constexpr int SCHED_MFMA = 0x008, SCHED_DS_READ = 0x100, SCHED_DS_WRITE = 0x200;
template <int MASK_A, int NA, int MASK_B, int NB, int REP>
__device__ __forceinline__ void sched_pairs() {
  if constexpr (REP > 0) {
    __builtin_amdgcn_sched_group_barrier(MASK_A, NA, 0);
    __builtin_amdgcn_sched_group_barrier(MASK_B, NB, 0);
    sched_pairs<MASK_A, NA, MASK_B, NB, REP - 1>();
  }
}

template <int ROWS, int NTHR, bool T>
struct Loader;
template <int ROWS, int NTHR>
struct Loader<ROWS, NTHR, false> : LoadK<ROWS, NTHR> {};
template <int ROWS, int NTHR>
struct Loader<ROWS, NTHR, true> : LoadT<ROWS, NTHR> {};

// Tile order: tiles are numbered so that 32 consecutive ids form an 8 (m) x 4 (n)
// block; XCD x (workgroup id mod 8) owns ids [x*per_xcd, (x+1)*per_xcd), so the
// workgroups resident on one XCD at a time share A and B panels in its L2.
__device__ __forceinline__ void tile_coords(const GemmArgs &g, int pid, int &tm, int &tn) {
  constexpr int GM = 8;
  const int per_group = GM * g.tiles_n;
  const int group = pid / per_group, first_m = group * GM;
  const int gsz = g.tiles_m - first_m < GM ? g.tiles_m - first_m : GM;
  tm = first_m + (pid % per_group) % gsz;
  tn = (pid % per_group) / gsz;
}

// WGM x WGN waves per workgroup.  KTAIL: K is not a multiple of 64, so the last
// K-slab is partly zero-filled.
template <int BM, int BN, int WGM, int WGN, bool AT, bool BT, bool KTAIL>
__global__ __launch_bounds__(64 * WGM * WGN, 1) void gemm_bf16_kernel(GemmArgs g) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  constexpr int NTHR = 64 * WGM * WGN;
  constexpr int WM = BM / WGM, WN = BN / WGN, TM = WM / 32, TN = WN / 32, KS = BK / 16;
  constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2, STAGE = A_BYTES + B_BYTES;

  const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
  const int pid = xcd * g.per_xcd + local;
  if (local >= g.per_xcd || pid >= g.tiles_m * g.tiles_n) return;
  int tm, tn;
  tile_coords(g, pid, tm, tn);
  const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * BN;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave / WGN, wn = wave % WGN;

  const bf16 *Abase = AT ? g.A + m0 : g.A + m0 * g.lda;
  const bf16 *Bbase = BT ? g.B + n0 : g.B + n0 * g.ldb;
  const int64_t a_rows = g.M - m0, b_rows = g.N - n0;

  Loader<BM, NTHR, AT> la;
  Loader<BN, NTHR, BT> lb;

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

  // per-lane fragment addressing: row (lane & 31) of a 32-row block, chunk 2*kk + (lane >> 5)
  const int frow = lane & 31, fchunk = lane >> 5;
  bf16x8 af[2][TM], bfr[2][TN];
  auto read_frags = [&](const char *buf, int kk, bf16x8(&fa)[TM], bf16x8(&fb)[TN]) {
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      int row = wm * WM + i * 32 + frow;
      fa[i] = *reinterpret_cast<const bf16x8 *>(buf + row * 128 + swz(row, kk * 2 + fchunk));
    }
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      int row = wn * WN + j * 32 + frow;
      fb[j] = *reinterpret_cast<const bf16x8 *>(buf + A_BYTES + row * 128 + swz(row, kk * 2 + fchunk));
    }
  };

  const int nk = (int)((g.K + BK - 1) / BK);
  la.template fetch<KTAIL>(Abase, g.lda, a_rows, 0, g.K);
  lb.template fetch<KTAIL>(Bbase, g.ldb, b_rows, 0, g.K);
  la.stash(smem);
  lb.stash(smem + A_BYTES);
  __syncthreads();
  read_frags(smem, 0, af[0], bfr[0]);

  // Software pipeline, pinned with scheduling barriers so that the compiler keeps it:
  //   top      : global loads of slab it+1 (16-byte, into registers)
  //   k-step kk: the LDS reads of k-step kk+1 are interleaved with the MFMAs of kk
  //   last step: first half of its MFMAs interleaved with the LDS writes of the new
  //              slab, workgroup barrier, then the first fragment reads of the new
  //              slab are issued under the second half of the MFMAs.
  // The final iteration reloads the last slab instead of branching; nobody reads it.
  constexpr int NM = TM * TN, NR = TM + TN;
  constexpr int NW = (AT ? 8 : BM * 8 / NTHR) + (BT ? 8 : BN * 8 / NTHR);  // LDS writes per slab
  auto mfma_rows = [&](int buf, int i_begin, int i_end) {
#pragma unroll
    for (int i = i_begin; i < i_end; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[buf][i], bfr[buf][j], acc[i][j], 0, 0, 0);
  };
  for (int it = 0; it < nk; ++it) {
    const char *cur = smem + (it & 1) * STAGE;
    char *nxt = smem + ((it + 1) & 1) * STAGE;
    const int64_t k_next = (int64_t)(it + 1 < nk ? it + 1 : it) * BK;
    la.template fetch<KTAIL>(Abase, g.lda, a_rows, k_next, g.K);
    lb.template fetch<KTAIL>(Bbase, g.ldb, b_rows, k_next, g.K);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int kk = 0; kk < KS - 1; ++kk) {
      read_frags(cur, kk + 1, af[(kk + 1) & 1], bfr[(kk + 1) & 1]);
      mfma_rows(kk & 1, 0, TM);
      if constexpr (NM % NR == 0) {
        sched_pairs<SCHED_DS_READ, 1, SCHED_MFMA, NM / NR, NR>();
      } else {  // 6 reads, 8 MFMAs
        sched_pairs<SCHED_DS_READ, 1, SCHED_MFMA, 1, NR - (NM - NR)>();
        sched_pairs<SCHED_DS_READ, 1, SCHED_MFMA, 2, NM - NR>();
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    la.stash(nxt);
    lb.stash(nxt + A_BYTES);
    mfma_rows((KS - 1) & 1, 0, TM / 2);
    sched_pairs<SCHED_MFMA, 1, SCHED_DS_WRITE, NW / (NM / 2), NM / 2>();
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();
    __builtin_amdgcn_sched_barrier(0);
    read_frags(nxt, 0, af[0], bfr[0]);
    mfma_rows((KS - 1) & 1, TM / 2, TM);
    __builtin_amdgcn_sched_barrier(0);
  }
  __syncthreads();

  // Epilogue through LDS, one wave-row (wm) of the tile at a time: accumulators are
  // written as a [WM][BN] fp32 image (element e of lane l is row 8*(e/4) + 4*(l/32)
  // + e%4, column l%32 of its 32x32 block), then every thread walks the image in
  // 8-element row segments and applies bias / GeLU / residual / accumulate with
  // 16-byte global accesses.
  float *img = reinterpret_cast<float *>(smem);
#pragma unroll
  for (int half = 0; half < WGM; ++half) {
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
    for (int idx = threadIdx.x; idx < WM * (BN / 8); idx += NTHR) {
      const int row = idx / (BN / 8), cv = idx % (BN / 8);
      const int64_t m = m0 + half * WM + row, n = n0 + cv * 8;
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

template <int BM, int BN, int WGM, int WGN, bool AT, bool BT, bool KTAIL>
int launch_k(const GemmArgs &in, hipStream_t st) {
  GemmArgs g = in;
  g.tiles_m = (int)((g.M + BM - 1) / BM);
  g.tiles_n = (int)((g.N + BN - 1) / BN);
  const int64_t tiles = (int64_t)g.tiles_m * g.tiles_n;
  if (tiles > (1 << 28)) return MTNLG_UNSUPPORTED_SHAPE;
  g.per_xcd = (int)((tiles + 7) / 8);
  constexpr int stages = 2 * (BM + BN) * BK * 2, image = (BM / WGM) * BN * 4;
  constexpr int smem = stages > image ? stages : image;
  static bool attr_set = false;
  if (!attr_set) {
    if (hipFuncSetAttribute((const void *)gemm_bf16_kernel<BM, BN, WGM, WGN, AT, BT, KTAIL>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, smem) != hipSuccess)
      return MTNLG_HIP_ERROR;
    attr_set = true;
  }
  gemm_bf16_kernel<BM, BN, WGM, WGN, AT, BT, KTAIL>
      <<<dim3((unsigned)(g.per_xcd * 8)), 64 * WGM * WGN, smem, st>>>(g);
  return check_launch();
}

template <int BM, int BN, int WGM, int WGN, bool AT, bool BT>
int launch(const GemmArgs &g, hipStream_t st) {
  return g.K % BK ? launch_k<BM, BN, WGM, WGN, AT, BT, true>(g, st)
                  : launch_k<BM, BN, WGM, WGN, AT, BT, false>(g, st);
}

// Tile shapes on offer: {BM, BN, waves_m, waves_n}
enum TileConfig { T256x256_2x2 = 0, T128x128_2x2, T256x256_2x4, T256x128_2x2, T128x256_2x2, TILE_CONFIGS };

template <bool AT, bool BT>
int launch_config(int cfg, const GemmArgs &g, hipStream_t st) {
  switch (cfg) {
    case T256x256_2x2: return launch<256, 256, 2, 2, AT, BT>(g, st);
    case T128x128_2x2: return launch<128, 128, 2, 2, AT, BT>(g, st);
    case T256x256_2x4: return launch<256, 256, 2, 4, AT, BT>(g, st);
    case T256x128_2x2: return launch<256, 128, 2, 2, AT, BT>(g, st);
    case T128x256_2x2: return launch<128, 256, 2, 2, AT, BT>(g, st);
    default: return MTNLG_INVALID_ARG;
  }
}

template <bool AT, bool BT>
int pick_tile(const GemmArgs &g, hipStream_t st) {
  // MTNLG_GEMM_TILE=<0..4> forces one tile shape (tuning aid).
  static const int forced = [] {
    const char *e = getenv("MTNLG_GEMM_TILE");
    return e ? atoi(e) : -1;
  }();
  if (forced >= 0 && forced < TILE_CONFIGS) return launch_config<AT, BT>(forced, g, st);
  // 256x256 tiles on 8 waves measure fastest per tile; problems too small to give
  // most of the 256 CUs one such tile take 128x128 tiles (two workgroups per CU).
  const int64_t tiles256 = ((g.M + 255) / 256) * ((g.N + 255) / 256);
  return launch_config<AT, BT>(tiles256 < 160 ? T128x128_2x2 : T256x256_2x4, g, st);
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
