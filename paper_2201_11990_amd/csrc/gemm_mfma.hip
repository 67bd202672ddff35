// bf16 GEMM on the gfx950 matrix cores, fp32 accumulate:  C[M,N] = op(A) * op(B).
//
// Two kernels share the tile numbering, the split-K tail and the epilogue:
//
//  * gemm_stream_kernel (aligned problems: M, N multiples of 256, K of 64 -- every GEMM of the
//    MT-NLG slice): 256x256 tile on 2 x 4 waves, v_mfma_f32_16x16x32_bf16, both operands moved
//    global -> LDS by DMA through a ring of 2 + 3 stages with the loads spread over the slab,
//    transposing LDS reads for row-contiguous operands.  Described at its definition.
//
//  * gemm_bf16_kernel (everything else: ragged edges, K tails, small problems):
//    v_mfma_f32_32x32x16_bf16, both operands brought into LDS as [row][k] tiles ("row" = m for
//    A, n for B; 64 k per tile = 128 bytes per row), whatever their layout in memory:
//      K-contiguous operand (x in x W^T, W in x W^T, dY in dY W): 16-byte global loads land in
//        LDS unchanged (by DMA when K has no tail);
//      row-contiguous operand (W in dY W, dY and X in dY^T X): each thread loads an 8(k) x 8(row)
//        block with 16-byte loads along the row axis, transposes it in registers and writes
//        16-byte k-runs.
//    Inside a tile, the 16-byte chunk c of row r sits at chunk position
//    c ^ (r & 7) ^ ((r >> 3) & 7), chosen from a bank model (an LDS pass serving 16 consecutive
//    lanes) for both kinds of LDS writes and the 32-row MFMA operand reads; unlike the streaming
//    kernel's placement it has not been measured.  Workgroup = WGM x WGN waves (256x256 tile on 2 x 4 waves by
//    default, 128x128 on 2 x 2 for small problems); K advances 64 at a time through two LDS
//    stages, with the LDS traffic interleaved between the MFMAs by scheduling hints.
//    Requirements: K % 8 == 0 and N % 8 == 0; a row-contiguous A also needs M % 8 == 0 (16-byte
//    accesses never straddle an edge).  Other edges are handled by clamped loads and masked stores.
//
// Workgroups are numbered so that the 8 XCDs (workgroup id mod 8) each own a contiguous run of
// column-major tiles: neighbours in an XCD's L2 share A and B panels.
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
  // split-K tail: tiles [whole_tiles, tiles) are each computed by `split` workgroups,
  // `part_slabs` K-slabs apiece, which leave fp32 partial tiles in `partial`
  int whole_tiles, split, part_slabs;
  float *partial;
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
  static constexpr int LDS_WRITES = N;
  template <bool KTAIL>
  __device__ __forceinline__ void fetch(const bf16 *base, int64_t ld, int64_t rows_valid, int64_t k0, int64_t K,
                                        char *) {
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

// K-contiguous source, straight into LDS (global_load_lds_dwordx4): a wave instruction
// fills 1 KB = 8 tile rows; lane l supplies the address of the chunk that belongs at
// LDS slot l of that KB under the tile's swizzle.  No registers, no LDS write
// instructions; completion is tracked by vmcnt.  K % 64 == 0 only.
template <int ROWS, int NTHR>
struct LoadKDirect {
  static constexpr int NI = ROWS / 8 / (NTHR / 64);  // instructions per wave
  static constexpr int LDS_WRITES = 0;
  template <bool KTAIL>
  __device__ __forceinline__ void fetch(const bf16 *base, int64_t ld, int64_t rows_valid, int64_t k0, int64_t,
                                        char *lds) {
    static_assert(!KTAIL, "direct-to-LDS loads cannot zero-fill a K tail");
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int q = wave * NI + i;
      const int row = 8 * q + (lane >> 3);
      const int c = (lane & 7) ^ (lane >> 3) ^ (q & 7);
      const int64_t rr = row < rows_valid ? row : rows_valid - 1;
      __builtin_amdgcn_global_load_lds(
          (const __attribute__((address_space(1))) void *)(base + rr * ld + k0 + c * 8),
          (__attribute__((address_space(3))) void *)(lds + q * 1024), 16, 0, 0);
    }
  }
  __device__ __forceinline__ void stash(char *) const {}
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
  static constexpr int LDS_WRITES = 8;
  template <bool KTAIL>
  __device__ __forceinline__ void fetch(const bf16 *base, int64_t ld, int64_t rows_valid, int64_t k0, int64_t K,
                                        char *) {
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

// Scheduling pipeline of one k-step of the streaming kernel: NM MFMAs, NR LDS fragment reads and NV
// DMA instructions, spread as evenly as the counts allow (one item after each MFMA).
template <int NM, int NR, int NV, int M = 0, int R = 0, int V = 0>
__device__ __forceinline__ void stream_sched() {
  if constexpr (M < NM) {
    __builtin_amdgcn_sched_group_barrier(SCHED_MFMA, 1, 0);
    // after MFMA number M+1: reads so far should be ceil((M+1) NR / NM), loads ceil((M+1) NV / NM) - offset
    constexpr int r_target = ((M + 1) * NR + NM - 1) / NM;
    constexpr int v_target = ((2 * M + 1) * NV) / (2 * NM);   // loads trail the reads by half a slot
    constexpr int dr = r_target - R, dv = v_target - V;
    if constexpr (dr > 0) __builtin_amdgcn_sched_group_barrier(SCHED_DS_READ, dr, 0);
    if constexpr (dv > 0) __builtin_amdgcn_sched_group_barrier(0x020, dv, 0);
    stream_sched<NM, NR, NV, M + 1, R + (dr > 0 ? dr : 0), V + (dv > 0 ? dv : 0)>();
  } else {
    if constexpr (R < NR) __builtin_amdgcn_sched_group_barrier(SCHED_DS_READ, NR - R, 0);
    if constexpr (V < NV) __builtin_amdgcn_sched_group_barrier(0x020, NV - V, 0);
  }
}

template <int ROWS, int NTHR, bool T, bool DIRECT>
struct Loader;
template <int ROWS, int NTHR>
struct Loader<ROWS, NTHR, false, false> : LoadK<ROWS, NTHR> {};
template <int ROWS, int NTHR>
struct Loader<ROWS, NTHR, false, true> : LoadKDirect<ROWS, NTHR> {};
template <int ROWS, int NTHR, bool D>
struct Loader<ROWS, NTHR, true, D> : LoadT<ROWS, NTHR> {};

// Bias / GeLU / residual / accumulate / store for 8 consecutive outputs of row m at column n.
__device__ __forceinline__ void epilogue8(const GemmArgs &g, int64_t m, int64_t n, float (&v)[8]) {
  const uint32_t flags = g.ea.flags;
  const int64_t off = m * g.ldc + n;
  float t[8];
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

  // Workgroups [0, 8*per_xcd) take whole tiles (XCD-aware numbering); the rest take
  // one K-part of a tail tile each.
  const int nk_all = (int)((g.K + BK - 1) / BK);
  int pid, slab0 = 0, slab1 = nk_all, part_id = -1;
  if ((int)blockIdx.x < 8 * g.per_xcd) {
    const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
    pid = xcd * g.per_xcd + local;
    if (pid >= g.whole_tiles) return;
  } else {
    part_id = blockIdx.x - 8 * g.per_xcd;
    pid = g.whole_tiles + part_id / g.split;
    slab0 = (part_id % g.split) * g.part_slabs;
    slab1 = slab0 + g.part_slabs < nk_all ? slab0 + g.part_slabs : nk_all;
  }
  int tm, tn;
  tile_coords(g, pid, tm, tn);
  const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * BN;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave / WGN, wn = wave % WGN;

  const bf16 *Abase = AT ? g.A + m0 : g.A + m0 * g.lda;
  const bf16 *Bbase = BT ? g.B + n0 : g.B + n0 * g.ldb;
  const int64_t a_rows = g.M - m0, b_rows = g.N - n0;

  // K-contiguous operands go straight to LDS when K has no tail
  constexpr bool DIRECT_A = !AT && !KTAIL, DIRECT_B = !BT && !KTAIL;
  Loader<BM, NTHR, AT, DIRECT_A> la;
  Loader<BN, NTHR, BT, DIRECT_B> lb;

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

  const int nk = slab1 - slab0;
  la.template fetch<KTAIL>(Abase, g.lda, a_rows, (int64_t)slab0 * BK, g.K, smem);
  lb.template fetch<KTAIL>(Bbase, g.ldb, b_rows, (int64_t)slab0 * BK, g.K, smem + A_BYTES);
  la.stash(smem);
  lb.stash(smem + A_BYTES);
  if constexpr (DIRECT_A || DIRECT_B) __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): direct loads landed
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
  constexpr int NW = decltype(la)::LDS_WRITES + decltype(lb)::LDS_WRITES;  // LDS write instructions per slab
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
    const int64_t k_next = (int64_t)(slab0 + (it + 1 < nk ? it + 1 : it)) * BK;
    la.template fetch<KTAIL>(Abase, g.lda, a_rows, k_next, g.K, nxt);
    lb.template fetch<KTAIL>(Bbase, g.ldb, b_rows, k_next, g.K, nxt + A_BYTES);
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
    if constexpr (NW > 0) sched_pairs<SCHED_MFMA, 1, SCHED_DS_WRITE, (NW + NM / 2 - 1) / (NM / 2), NM / 2>();
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (DIRECT_A || DIRECT_B) __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
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
    for (int idx = threadIdx.x; idx < WM * (BN / 8); idx += NTHR) {
      const int row = idx / (BN / 8), cv = idx % (BN / 8);
      float v[8];
      const f32x4 lo = *reinterpret_cast<const f32x4 *>(img + row * BN + cv * 8);
      const f32x4 hi = *reinterpret_cast<const f32x4 *>(img + row * BN + cv * 8 + 4);
#pragma unroll
      for (int e = 0; e < 4; ++e) { v[e] = lo[e]; v[4 + e] = hi[e]; }
      if (part_id >= 0) {  // K-part of a tail tile: raw fp32 partial, summed by splitk_reduce_kernel
        store8(g.partial + (int64_t)part_id * (BM * BN) + (half * WM + row) * BN + cv * 8, v);
      } else {
        const int64_t m = m0 + half * WM + row, n = n0 + cv * 8;
        if (m < g.M && n < g.N) epilogue8(g, m, n, v);
      }
    }
    __syncthreads();
  }
}

// =======================================================================================
// Streaming kernel: 256x256 tile, BK = 64, both operands brought global -> LDS by DMA
// (buffer_load ... lds), no register staging, no LDS store instructions; MFMA 16x16x32.
//   A lives in a ring of two 32 KB stages, B in a ring of three (B is the operand that comes
//   from HBM for the first time: the weights); the DMA instructions of a slab are spread over
//   the four phases of a slab (two per phase and wave) so that the texture path never sees a burst.
//   K-contiguous operand: stage = [256 rows][128 B], 16-byte chunk c of row r at chunk position
//     c ^ (r & 7); MFMA fragments are 16-byte LDS reads (this placement measured conflict-free for the
//     fragment pattern -- 16 rows x one chunk per 16 lanes -- at 4.5-4.9 cycles per wave instruction;
//     with a further ^ (r >> 3), which a model of 16 consecutive lanes per LDS pass asks for, the
//     same reads take 7.8).
//   Row-contiguous operand ([k][row] in memory): stage = [64 k][512 B] as in memory, with the
//     16-byte unit u of k-row k at unit position (((u >> 2) ^ (k & 3)) << 2) | ((u & 3) ^ ((k >> 2) & 2));
//     MFMA fragments are two transposing 8-byte LDS reads (ds_read_b64_tr_b16: a 16-lane group reads
//     4 k-rows x 16 rows and every lane receives the 4 k values of its own row).
//   A slab is four phases of 16 MFMAs: (k-step 0, rows 0-63 of the wave tile), (0, rows 64-127),
//   (1, rows 0-63), (1, rows 64-127); each phase loads the fragments of the next one.  The one
//   workgroup barrier per slab sits before the last phase (whose fragments are already in
//   registers) so that the first fragment reads of the next slab hide behind a phase of MFMAs.
//   Aligned problems only: M, N multiples of 256, K of 64.
template <bool AT, bool BT, bool PLAIN16>
__global__ __launch_bounds__(512, 1) void gemm_stream_kernel(GemmArgs g) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  constexpr int BM = 256, BN = 256, WGM = 2, WGN = 4, NWAVES = WGM * WGN;
  constexpr int WM = BM / WGM, WN = BN / WGN, TM = WM / 16, TN = WN / 16, HM = TM / 2;
  constexpr int STAGE = 256 * BK * 2, A_RING = 2 * STAGE, B_RING = 3 * STAGE;
  constexpr int NI = 32 / NWAVES;   // DMA instructions per wave per operand and slab
  const int nk_all = (int)(g.K / BK);
  int pid, slab0 = 0, slab1 = nk_all, part_id = -1;
  if ((int)blockIdx.x < 8 * g.per_xcd) {
    const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
    pid = xcd * g.per_xcd + local;
    if (pid >= g.whole_tiles) return;
  } else {
    part_id = blockIdx.x - 8 * g.per_xcd;
    pid = g.whole_tiles + part_id / g.split;
    slab0 = (part_id % g.split) * g.part_slabs;
    slab1 = slab0 + g.part_slabs < nk_all ? slab0 + g.part_slabs : nk_all;
  }
  int tm, tn;
  tile_coords(g, pid, tm, tn);
  const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * BN;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  const bf16 *Abase = AT ? g.A + m0 : g.A + m0 * g.lda;
  const bf16 *Bbase = BT ? g.B + n0 : g.B + n0 * g.ldb;

  // DMA addressing.  Wave w issues instructions q = NI w .. NI w + NI - 1 of each operand; instruction
  // q fills LDS bytes [1024 q, 1024 q + 1024) of the stage, lane l the 16 bytes at 16 l.
  auto dma_offset = [&](int q, int64_t ld, bool transposed) -> uint32_t {
    if (!transposed) {   // rows 8q .. 8q+7, lane l: row 8q + l/8, chunk position l%8
      const int row = 8 * q + (lane >> 3), c = (lane & 7) ^ (lane >> 3);   // row % 8 == lane / 8
      return (uint32_t)(row * ld * 2 + c * 16);
    } else {             // k-rows 2q, 2q+1, lane l: k = 2q + l/32, unit position l%32
      const int k = 2 * q + (lane >> 5), p = lane & 31;
      const int u = (((p >> 2) ^ (k & 3)) << 2) | ((p & 3) ^ ((k >> 2) & 2));
      return (uint32_t)(k * ld * 2 + u * 16);
    }
  };
  uint32_t a_off[NI], b_off[NI];
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    a_off[i] = dma_offset(wave * NI + i, g.lda, AT);
    b_off[i] = dma_offset(wave * NI + i, g.ldb, BT);
  }
  // With a transposing LDS read in the loop the DMA goes out as inline assembly (see dma16: the
  // compiler would put a wait for all memory operations in front of those reads); otherwise
  // through the builtin, which the scheduling hints below can place.
  auto issue = [&](const bf16 *base, const uint32_t(&off)[NI], char *stage, int i0, int i1) {
    char *dst = stage + wave * (NI * 1024);
    if constexpr (AT || BT) {
      const dma_rsrc_t rs = dma_rsrc(base);
      const uint32_t dst_addr = lds_address(dst);
#pragma unroll
      for (int i = 0; i < NI; ++i)
        if (i >= i0 && i < i1) dma16(rs, dst_addr + i * 1024, off[i]);
    } else {
      const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16 *>(base), 0, 0xFFFFFFFFu, 0x00020000);
#pragma unroll
      for (int i = 0; i < NI; ++i)
        if (i >= i0 && i < i1)
          __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (__attribute__((address_space(3))) void *)(dst + i * 1024), 16,
                                                   (int)off[i], 0, 0, 0);
    }
  };
  auto a_at = [&](int64_t k0) { return AT ? Abase + k0 * g.lda : Abase + k0; };
  auto b_at = [&](int64_t k0) { return BT ? Bbase + k0 * g.ldb : Bbase + k0; };

  f32x4 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.0f;

  // MFMA 16x16x32 operand of the 16-row block at r0 for k-step kk (32 k): lane l holds row
  // r0 + l%16, k = 32 kk + 8 (l/16) .. + 7
  auto frag = [&](const char *stage, int r0, int kk, bool transposed) -> bf16x8 {
    if (!transposed) {
      const int row = r0 + (lane & 15);
      return *reinterpret_cast<const bf16x8 *>(stage + row * 128 + (((kk * 4 + (lane >> 4)) ^ (row & 7)) << 4));
    } else {
      // as address supplier lane 16 grp + L covers k-row kbase + L/4, rows r0 + 4 (L%4) .. + 3
      const int grp = lane >> 4, L = lane & 15;
      const int nb = r0 + 4 * (L & 3);
      const int kbase = 32 * kk + 8 * grp + (L >> 2);
      auto addr = [&](int k) {
        const int u = nb >> 3;                                    // 16-byte unit of the row
        const int p = (((u >> 2) ^ (k & 3)) << 2) | ((u & 3) ^ ((k >> 2) & 2));
        return stage + k * 512 + p * 16 + (nb & 7) * 2;
      };
      const i16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4 *)addr(kbase));
      const i16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4 *)addr(kbase + 4));
      i16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
      return __builtin_bit_cast(bf16x8, v);
    }
  };
  bf16x8 af[2][HM], bfr[2][TN];   // A: one buffer per half of the wave tile; B: one per k-step parity
  auto read_a = [&](const char *abuf, int kk, int h) {
#pragma unroll
    for (int i = 0; i < HM; ++i) af[h][i] = frag(abuf, wm * WM + (h * HM + i) * 16, kk, AT);
  };
  auto read_b = [&](const char *bbuf, int kk) {
#pragma unroll
    for (int j = 0; j < TN; ++j) bfr[kk & 1][j] = frag(bbuf, wn * WN + j * 16, kk, BT);
  };
  auto mfma_phase = [&](int kk, int h) {
#pragma unroll
    for (int i = 0; i < HM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
        acc[h * HM + i][j] =   // B fragment first: the block comes out transposed, see the epilogue
            __builtin_amdgcn_mfma_f32_16x16x32_bf16(bfr[kk & 1][j], af[h][i], acc[h * HM + i][j], 0, 0, 0);
  };

  const int nk = slab1 - slab0;
  auto slab_k = [&](int it) { return (int64_t)(slab0 + (it < nk ? it : nk - 1)) * BK; };
  char *const aring = smem, *const bring = smem + A_RING;
  // prologue: A slab 0, B slabs 0 and 1, first half of A slab 1
  issue(a_at(slab_k(0)), a_off, aring, 0, NI);
  issue(b_at(slab_k(0)), b_off, bring, 0, NI);
  issue(b_at(slab_k(1)), b_off, bring + STAGE, 0, NI);
  issue(a_at(slab_k(1)), a_off, aring + STAGE, 0, NI / 2);
  asm volatile("s_waitcnt vmcnt(6)\n\ts_barrier" ::: "memory");   // A 0, B 0 landed
  read_a(aring, 0, 0);
  read_b(bring, 0);

  constexpr int RA = (AT ? 2 : 1) * HM, RB = (BT ? 2 : 1) * TN;   // LDS read instructions of an A half / of B
  int a_cur = 0, b_cur = 0;   // ring offsets of slab `it`
  for (int it = 0; it < nk; ++it) {
    const int a_nxt = a_cur ^ STAGE;
    const int b_nxt = b_cur + STAGE >= B_RING ? b_cur + STAGE - B_RING : b_cur + STAGE;
    const int b_nn = b_nxt + STAGE >= B_RING ? b_nxt + STAGE - B_RING : b_nxt + STAGE;
    // phase 0: second half of A slab it+1 (into the stage slab it-1 left at the last barrier)
    // phases 1, 2: B slab it+2 into the ring stage that held slab it-1
    // phase 3 (after the barrier): first half of A slab it+2 into the stage slab it just left
#pragma unroll
    for (int ph = 0; ph < 4; ++ph) {
      const int kk = ph >> 1, h = ph & 1;
      // The two waves of a SIMD take turns on the matrix pipe one phase at a time: the wave that
      // is behind (counted from the barrier) has the higher issue priority.
      if (ph == 0) __builtin_amdgcn_s_setprio(2);
      else if (ph == 1) __builtin_amdgcn_s_setprio(1);
      else if (ph == 2) __builtin_amdgcn_s_setprio(0);
      if (ph == 3) {
        // slab it+1 is complete once only the DMAs of B slab it+2 are outstanding
        asm volatile("s_waitcnt vmcnt(4) lgkmcnt(0)\n\ts_barrier" ::: "memory");
        __builtin_amdgcn_s_setprio(3);
        __builtin_amdgcn_sched_barrier(0);
        read_a(aring + a_nxt, 0, 0);
        read_b(bring + b_nxt, 0);
      } else if (h == 0) {
        read_a(aring + a_cur, kk, 1);
      } else {
        read_a(aring + a_cur, kk + 1, 0);
        read_b(bring + b_cur, kk + 1);
      }
      if (ph == 0) issue(a_at(slab_k(it + 1)), a_off, aring + a_nxt, NI / 2, NI);
      else if (ph < 3) issue(b_at(slab_k(it + 2)), b_off, bring + b_nn, (ph - 1) * (NI / 2), ph * (NI / 2));
      else issue(a_at(slab_k(it + 2)), a_off, aring + a_cur, 0, NI / 2);
      mfma_phase(kk, h);
      if (h == 0) stream_sched<HM * TN, RA, NI / 2>();
      else stream_sched<HM * TN, RA + RB, NI / 2>();
      __builtin_amdgcn_sched_barrier(0);
    }
    a_cur = a_nxt;
    b_cur = b_nxt;
  }
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
  __builtin_amdgcn_s_setprio(0);

  // Epilogue, wave by wave with no workgroup barrier.  The MFMAs took the B fragment as their first
  // operand, so block (i, j) of the wave tile sits transposed in the registers: lane l holds row
  // 16 i + l % 16 and the four consecutive columns 16 j + 4 (l / 16) .. + 3.  Each wave turns its
  // 128 x 64 tile, 64 rows at a time, through a private 64 x 68-float LDS patch (16-byte stores,
  // conflict-free at that pitch) into 8-column row segments, so that every global access is 16
  // bytes of a row and a wave instruction covers whole 128-byte lines.
  if (PLAIN16 && part_id < 0) {
    // bf16 output with at most a bias: round before the transposition, which halves the LDS
    // traffic of the patch and leaves the second half of the epilogue a plain 16-byte copy.
    // Patch = 64 rows x 128 B per wave, 16-byte unit u of row r at unit position u ^ ((r >> 1) & 7)
    // (8-byte block stores and 16-byte row reads both conflict-free).
    char *patch = smem + wave * 8192;
    const int g4 = lane >> 4;
    f32x4 bias4[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
#pragma unroll
      for (int e = 0; e < 4; ++e) bias4[j][e] = 0.0f;
      if (g.ea.flags & MTNLG_EPI_BIAS) {
        const bf16x4 bv = *reinterpret_cast<const bf16x4 *>(static_cast<const bf16 *>(g.ea.bias) + n0 + wn * WN + j * 16 + 4 * g4);
#pragma unroll
        for (int e = 0; e < 4; ++e) bias4[j][e] = (float)bv[e];
      }
    }
    bf16 *cbase = static_cast<bf16 *>(g.C) + (m0 + wm * WM) * g.ldc + n0 + wn * WN;
#pragma unroll
    for (int p = 0; p < TM / 4; ++p) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          const int row = (lane & 15) + i * 16, unit = 2 * j + (g4 >> 1);
          bf16x4 h;
#pragma unroll
          for (int e = 0; e < 4; ++e) h[e] = (bf16)(acc[p * 4 + i][j][e] + bias4[j][e]);
          *reinterpret_cast<bf16x4 *>(patch + row * 128 + ((unit ^ ((row >> 1) & 7)) << 4) + (g4 & 1) * 8) = h;
        }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        const int row = t * 8 + (lane >> 3), cv = lane & 7;   // 8 rows x 8 segments per instruction
        const bf16x8 o = *reinterpret_cast<const bf16x8 *>(patch + row * 128 + ((cv ^ ((row >> 1) & 7)) << 4));
        *reinterpret_cast<bf16x8 *>(cbase + (int64_t)(p * 64 + row) * g.ldc + cv * 8) = o;
      }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // patch is rewritten by the next pass
    }
  } else {
    constexpr int PITCH = WN + 4;
    float *patch = reinterpret_cast<float *>(smem) + wave * (64 * PITCH);
#pragma unroll
    for (int p = 0; p < TM / 4; ++p) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          *reinterpret_cast<f32x4 *>(patch + ((lane & 15) + i * 16) * PITCH + j * 16 + 4 * (lane >> 4)) = acc[p * 4 + i][j];
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        const int row = t * 8 + (lane >> 3), cv = lane & 7;   // 8 rows x 8 segments per instruction
        float v[8];
        const f32x4 lo = *reinterpret_cast<const f32x4 *>(patch + row * PITCH + cv * 8);
        const f32x4 hi = *reinterpret_cast<const f32x4 *>(patch + row * PITCH + cv * 8 + 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) { v[e] = lo[e]; v[4 + e] = hi[e]; }
        const int trow = wm * WM + p * 64 + row, tcol = wn * WN + cv * 8;   // position in the 256 x 256 tile
        if (part_id >= 0) {  // K-part of a tail tile: raw fp32 partial, summed by splitk_reduce_kernel
          store8(g.partial + (int64_t)part_id * (BM * BN) + trow * BN + tcol, v);
        } else {
          epilogue8(g, m0 + trow, n0 + tcol, v);
        }
      }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // patch is rewritten by the next pass
    }
  }
}

// Sum the `split` fp32 partial tiles of each tail tile in a fixed order and run the epilogue.
template <int BM, int BN>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(GemmArgs g) {
  const int tail = blockIdx.y;  // tail tile index
  int tm, tn;
  tile_coords(g, g.whole_tiles + tail, tm, tn);
  const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * BN;
  for (int idx = blockIdx.x * 256 + threadIdx.x; idx < BM * (BN / 8); idx += gridDim.x * 256) {
    const int row = idx / (BN / 8), cv = idx % (BN / 8);
    const int64_t m = m0 + row, n = n0 + cv * 8;
    if (m >= g.M || n >= g.N) continue;
    float v[8] = {}, t[8];
    for (int s = 0; s < g.split; ++s) {
      load8(g.partial + ((int64_t)tail * g.split + s) * (BM * BN) + row * BN + cv * 8, t);
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] += t[e];
    }
    epilogue8(g, m, n, v);
  }
}

// How the tiles of a problem are covered: `whole` tiles by one workgroup each, the
// remaining tail tiles by `split` workgroups each (split == 1: no tail).
struct SplitPlan {
  int whole, tail, split, part_slabs;
  size_t workspace;
};
inline SplitPlan plan_split(int64_t tiles, int nk, int bm, int bn, size_t ws_bytes) {
  SplitPlan p{(int)tiles, 0, 1, nk, 0};
  const int cus = 256;
  const int tail = (int)(tiles % cus);
  if (tail == 0 || tail > 176) return p;  // the last round is full enough
  if (tiles >= 4 * cus) return p;          // many rounds: an idle tail costs little, splitting costs more
  int split = cus / tail;
  if (split > 8) split = 8;
  while (split > 1 && nk / split < 8) --split;  // keep K-parts long enough to pipeline
  while (split > 1 && (split - 1) * ((nk + split - 1) / split) >= nk) --split;  // no empty K-part
  if (split <= 1) return p;
  const size_t need = (size_t)tail * split * bm * bn * sizeof(float);
  p.workspace = need;
  if (ws_bytes < need) return p;  // caller gave no room: whole tiles only
  p.whole = (int)(tiles - tail);
  p.tail = tail;
  p.split = split;
  p.part_slabs = (nk + split - 1) / split;
  return p;
}

template <int BM, int BN, int WGM, int WGN, bool AT, bool BT, bool KTAIL>
int launch_k(const GemmArgs &in, void *ws, size_t ws_bytes, hipStream_t st) {
  GemmArgs g = in;
  g.tiles_m = (int)((g.M + BM - 1) / BM);
  g.tiles_n = (int)((g.N + BN - 1) / BN);
  const int64_t tiles = (int64_t)g.tiles_m * g.tiles_n;
  if (tiles > (1 << 28)) return MTNLG_UNSUPPORTED_SHAPE;
  const int nk = (int)((g.K + BK - 1) / BK);
  const SplitPlan plan = plan_split(tiles, nk, BM, BN, ws ? ws_bytes : 0);
  const bool split = plan.tail > 0;
  g.whole_tiles = split ? plan.whole : (int)tiles;
  g.split = split ? plan.split : 1;
  g.part_slabs = split ? plan.part_slabs : nk;
  g.partial = (float *)ws;
  g.per_xcd = (g.whole_tiles + 7) / 8;
  const unsigned grid = (unsigned)(g.per_xcd * 8 + (split ? plan.tail * plan.split : 0));
  constexpr int stages = 2 * (BM + BN) * BK * 2, image = (BM / WGM) * BN * 4;
  constexpr int smem = stages > image ? stages : image;
  static unsigned long long attr_done = 0;
  int device;
  if (!attr_is_set(attr_done, &device)) {
    if (hipFuncSetAttribute((const void *)gemm_bf16_kernel<BM, BN, WGM, WGN, AT, BT, KTAIL>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, smem) != hipSuccess)
      return MTNLG_HIP_ERROR;
    attr_mark_set(attr_done, device);
  }
  // Aligned problems on the default tile shape take the streaming kernel (all operands by DMA).
  if constexpr (BM == 256 && BN == 256 && WGM == 2 && WGN == 4 && !KTAIL) {
    if (g.M % 256 == 0 && g.N % 256 == 0) {
      constexpr int stream_smem = 5 * 256 * BK * 2;
      static unsigned long long stream_attr_done = 0;
      if (!attr_is_set(stream_attr_done, &device)) {
        if (hipFuncSetAttribute((const void *)gemm_stream_kernel<AT, BT, false>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, stream_smem) != hipSuccess ||
            hipFuncSetAttribute((const void *)gemm_stream_kernel<AT, BT, true>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, stream_smem) != hipSuccess)
          return MTNLG_HIP_ERROR;
        attr_mark_set(stream_attr_done, device);
      }
      // bf16 output with nothing but an optional bias: the epilogue that rounds before it transposes
      if ((g.ea.flags & ~(uint32_t)MTNLG_EPI_BIAS) == 0)
        gemm_stream_kernel<AT, BT, true><<<dim3(grid), 64 * WGM * WGN, stream_smem, st>>>(g);
      else
        gemm_stream_kernel<AT, BT, false><<<dim3(grid), 64 * WGM * WGN, stream_smem, st>>>(g);
      MTNLG_TRY(check_launch());
      if (split) {
        splitk_reduce_kernel<BM, BN><<<dim3(8, plan.tail), 256, 0, st>>>(g);
        MTNLG_TRY(check_launch());
      }
      return MTNLG_OK;
    }
  }
  gemm_bf16_kernel<BM, BN, WGM, WGN, AT, BT, KTAIL><<<dim3(grid), 64 * WGM * WGN, smem, st>>>(g);
  MTNLG_TRY(check_launch());
  if (split) {
    splitk_reduce_kernel<BM, BN><<<dim3(8, plan.tail), 256, 0, st>>>(g);
    MTNLG_TRY(check_launch());
  }
  return MTNLG_OK;
}

template <int BM, int BN, int WGM, int WGN, bool AT, bool BT>
int launch(const GemmArgs &g, void *ws, size_t ws_bytes, hipStream_t st) {
  return g.K % BK ? launch_k<BM, BN, WGM, WGN, AT, BT, true>(g, ws, ws_bytes, st)
                  : launch_k<BM, BN, WGM, WGN, AT, BT, false>(g, ws, ws_bytes, st);
}

// Tile shapes on offer: {BM, BN, waves_m, waves_n}
enum TileConfig { T256x256_2x2 = 0, T128x128_2x2, T256x256_2x4, T256x128_2x2, T128x256_2x2, TILE_CONFIGS };

template <bool AT, bool BT>
int launch_config(int cfg, const GemmArgs &g, void *ws, size_t ws_bytes, hipStream_t st) {
  switch (cfg) {
    case T256x256_2x2: return launch<256, 256, 2, 2, AT, BT>(g, ws, ws_bytes, st);
    case T128x128_2x2: return launch<128, 128, 2, 2, AT, BT>(g, ws, ws_bytes, st);
    case T256x256_2x4: return launch<256, 256, 2, 4, AT, BT>(g, ws, ws_bytes, st);
    case T256x128_2x2: return launch<256, 128, 2, 2, AT, BT>(g, ws, ws_bytes, st);
    case T128x256_2x2: return launch<128, 256, 2, 2, AT, BT>(g, ws, ws_bytes, st);
    default: return MTNLG_INVALID_ARG;
  }
}

template <bool AT, bool BT>
int pick_tile(const GemmArgs &g, void *ws, size_t ws_bytes, hipStream_t st) {
  // 256x256 tiles on 8 waves measure fastest per tile.  A last round that would leave
  // most CUs idle is split along K instead (needs workspace); without workspace, problems
  // too small to give most CUs one big tile take 128x128 tiles (two workgroups per CU).
  const int64_t tiles256 = ((g.M + 255) / 256) * ((g.N + 255) / 256);
  const int nk = (int)((g.K + BK - 1) / BK);
  const SplitPlan plan = plan_split(tiles256, nk, 256, 256, ws ? ws_bytes : 0);
  if (plan.tail == 0 && tiles256 < 160) return launch_config<AT, BT>(T128x128_2x2, g, ws, ws_bytes, st);
  return launch_config<AT, BT>(T256x256_2x4, g, ws, ws_bytes, st);
}

}  // namespace

size_t gemm_mfma_workspace_bytes(int64_t M, int64_t N, int64_t K) {
  if (M <= 0 || N <= 0 || K <= 0) return 0;
  const int64_t tiles256 = ((M + 255) / 256) * ((N + 255) / 256);
  return plan_split(tiles256, (int)((K + BK - 1) / BK), 256, 256, 0).workspace;
}

bool gemm_mfma_streams(int64_t M, int64_t N, int64_t K) {
  if (M <= 0 || N <= 0 || K <= 0 || M % 256 || N % 256 || K % BK) return false;
  // same choice as pick_tile: small problems take 128x128 tiles
  const int64_t tiles256 = (M / 256) * (N / 256);
  return tiles256 >= 160 || plan_split(tiles256, (int)(K / BK), 256, 256, ~(size_t)0).tail > 0;
}

int gemm_mfma_bf16(int layout, int64_t M, int64_t N, int64_t K, const void *A, const void *B, void *C,
                   const void *bias, void *aux, uint32_t epi, void *ws, size_t ws_bytes, hipStream_t stream,
                   int prof_class) {
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
  g.whole_tiles = 0; g.split = 1; g.part_slabs = 0; g.partial = nullptr;
  LaunchScope scope(prof_class >= 0 ? prof_class : MTNLG_K_GEMM_NT + layout, stream);
  if (!at && !bt) return pick_tile<false, false>(g, ws, ws_bytes, stream);
  if (!at && bt) return pick_tile<false, true>(g, ws, ws_bytes, stream);
  return pick_tile<true, true>(g, ws, ws_bytes, stream);
}

}  // namespace mtnlg
