// bf16 GEMM on the gfx950 matrix cores, fp32 accumulate:  C[M,N] = op(A) * op(B).
//
// Two kernels share the tile numbering, the split-K tail and the epilogue:
//
//  * gemm_stream_kernel (aligned problems: M a multiple of 256, N of the tile width, K of 64 -- every
//    GEMM of the MT-NLG slice): 256x256 or 256x320 tile on 2 x 4 waves, v_mfma_f32_16x16x32_bf16, both
//    operands moved global -> LDS by DMA through a ring of 2 + 3 (or 2 + 2) stages with the loads spread
//    over the slab, transposing LDS reads for row-contiguous operands.  Described at its definition;
//    gemm_mfma_pick_tile chooses kernel and tile shape per problem.
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
#include <type_traits>

#include "common.h"

namespace mtnlg {

namespace {

constexpr int BK = 64;
// Relative cost per FLOP of the wider streaming tile against 256 x 256 (measured on the MT-NLG slice's shapes).
constexpr double GEMM_COST_256x320 = 0.97;

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

// LDS reads that should have been issued after MFMA number m + 1 of a phase of nm MFMAs with nr reads.
//   rbj == 0: spread evenly.
//   rbj > 0 (last phase of a slab; MFMAs in groups of 4 per column block): the first group carries the nr - (nm / 4) rbj
//   reads of the next A fragments, group g > 0 the rbj reads that refill the B fragments of column block g - 1, whose
//   registers group g - 1 has just released; the last block's refill follows the last MFMA.
constexpr int sched_reads_after(int m, int nm, int nr, int rbj) {
  if (rbj == 0) return ((m + 1) * nr + nm - 1) / nm;
  const int ra = nr - (nm / 4) * rbj, grp = m / 4, s = m % 4;
  return grp == 0 ? ((s + 1) * ra + 3) / 4 : ra + (grp - 1) * rbj + ((s + 1) * rbj + 3) / 4;
}

// Scheduling pipeline of one phase of the streaming kernel: NM MFMAs, NR LDS fragment reads and NV
// DMA instructions (spread as evenly as the counts allow, one item after each MFMA).
template <int NM, int NR, int NV, int RBJ = 0, int M = 0, int R = 0, int V = 0>
__device__ __forceinline__ void stream_sched() {
  if constexpr (M < NM) {
    __builtin_amdgcn_sched_group_barrier(SCHED_MFMA, 1, 0);
    constexpr int r_target = sched_reads_after(M, NM, NR, RBJ);
    constexpr int v_target = ((2 * M + 1) * NV) / (2 * NM);   // loads trail the reads by half a slot
    constexpr int dr = r_target - R, dv = v_target - V;
    if constexpr (dr > 0) __builtin_amdgcn_sched_group_barrier(SCHED_DS_READ, dr, 0);
    if constexpr (dv > 0) __builtin_amdgcn_sched_group_barrier(0x020, dv, 0);
    stream_sched<NM, NR, NV, RBJ, M + 1, R + (dr > 0 ? dr : 0), V + (dv > 0 ? dv : 0)>();
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
// flags: the epilogue flags to apply (a caller that has added the bias already passes them without it);
// aux_in: the 8 aux values of this position if the caller has loaded them already, else nullptr.
__device__ __forceinline__ void epilogue8(const GemmArgs &g, int64_t m, int64_t n, float (&v)[8], uint32_t flags,
                                          const bf16x8 *aux_in = nullptr) {
  const int64_t off = m * g.ldc + n;
  float t[8];
  if (flags & MTNLG_EPI_BIAS) {
    load8(static_cast<const bf16 *>(g.ea.bias) + n, t);
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] += t[e];
  }
  if (flags & MTNLG_EPI_GELU) {
    store8(static_cast<bf16 *>(g.ea.aux) + off, v);
    if (flags & MTNLG_EPI_GELU_ERF) {   // the form is chosen per group of 8, not per element
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = gelu_f(v[e], true);
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = gelu_tanh_fast_f(v[e]);
    }
  }
  if (flags & (MTNLG_EPI_RESIDUAL | MTNLG_EPI_GELU_GRAD)) {
    if (aux_in) {
#pragma unroll
      for (int e = 0; e < 8; ++e) t[e] = (float)(*aux_in)[e];
    } else {
      load8(static_cast<const bf16 *>(g.ea.aux) + off, t);
    }
    if (flags & MTNLG_EPI_RESIDUAL) {
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] += t[e];
    } else {
      if (flags & MTNLG_EPI_GELU_ERF) {
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] *= gelu_grad_f(t[e], true);
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] *= gelu_tanh_grad_fast_f(t[e]);
      }
    }
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
__device__ __forceinline__ void epilogue8(const GemmArgs &g, int64_t m, int64_t n, float (&v)[8]) {
  epilogue8(g, m, n, v, g.ea.flags);
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
// Streaming kernel: 256 x BN tile (BN 256 or 320) on 2 x 4 waves, BK = 64, both operands brought
// global -> LDS by DMA (buffer_load ... lds), no register staging, no LDS store instructions; MFMA 16x16x32.
//   Tile shapes and LDS rings (160 KB per compute unit; a stage is ROWS x 128 bytes):
//     256 x 256: A in a ring of two 32 KB stages, B in a ring of three (B is the operand that comes from HBM
//                for the first time: the weights); 160 KB.
//     256 x 320: A two stages of 32 KB, B two of 40 KB; 144 KB.   N a multiple of 320.
//   The wider tile moves 10 % fewer operand bytes per FLOP from L2 into LDS ((BM + BN) / (BM BN)), which is
//   what holds the clock down under the board's power limit, and it covers the layer's forward, input-gradient
//   and FC weight-gradient shapes in whole rounds of 256 tiles; it pays with a ring one stage shorter and with
//   160 of a wave's 256 registers in accumulators (a 320 x 320 tile would need 200 and does not fit), which
//   leaves about 20 for addresses: hence the scalar DMA offsets and the XOR-derived fragment addresses below.
//   The DMA instructions of a slab are spread over the phases of a slab so that the texture path never sees a burst.
//   K-contiguous operand: stage = [ROWS][128 B], 16-byte chunk c of row r at chunk position
//     c ^ (r & 7); MFMA fragments are 16-byte LDS reads (this placement measured conflict-free for the
//     fragment pattern -- 16 rows x one chunk per 16 lanes -- at 4.5-4.9 cycles per wave instruction;
//     with a further ^ (r >> 3), which a model of 16 consecutive lanes per LDS pass asks for, the
//     same reads take 7.8).
//   Row-contiguous operand ([k][row] in memory): stage = [64 k][ROWS x 2 B] as in memory, with the 16-byte units
//     of a k-row permuted (tr_pos below) so that the fragment reads spread over all banks;
//     MFMA fragments are two transposing 8-byte LDS reads (ds_read_b64_tr_b16: a 16-lane group reads
//     4 k-rows x 16 rows and every lane receives the 4 k values of its own row).
//   A slab (two k-steps of 32) is four phases, one per pair of 16-row blocks of the wave tile, each issuing
//   both k-steps of its 2 x TN accumulator blocks back to back and loading the A fragments of the next phase;
//   the B fragments are held for the whole slab.  The one workgroup barrier per slab sits before the last
//   phase (whose fragments are already in registers), which then reads the first A fragments and, block by
//   block as its MFMAs release the registers, the B fragments of the next slab.
//   Aligned problems only: M a multiple of BM, N of BN, K of 64.

// Position of the 16-byte unit u of k-row k inside a row-contiguous stage's k-row of UPR units (an involution
// in u for every k).  A transposing fragment read touches, per 16-lane group, k-rows k0 .. k0+3 (k0 a multiple
// of 4) at two neighbouring units, and the four groups of a wave sit 8 k-rows apart.
//   32 units (512-byte k-rows, every k-row starts on the same bank): k & 3 moves the 64-byte group, k bit 3 the
//     32-byte pair inside it.
//   40 units (640-byte k-rows: consecutive k-rows already sit half the bank space apart): k bit 1 and k bit 3
//     move the 32-byte pair inside the aligned 128-byte group, which keeps units 32 .. 39 in place.
template <int UPR>
__device__ __forceinline__ int tr_pos(int u, int k) {
  if constexpr (UPR == 32) return (((u >> 2) ^ (k & 3)) << 2) | ((u & 3) ^ ((k >> 2) & 2));
  else return (u & ~7) | ((u & 7) ^ ((k & 2) | ((k >> 1) & 4)));
}

template <int N>
__device__ __forceinline__ void wait_dma_and_barrier() {   // at most N of this wave's DMAs still in flight
  asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
}

template <int BM, int BN, bool AT, bool BT, bool PLAIN16>
__global__ __launch_bounds__(512, 1) void gemm_stream_kernel(GemmArgs g) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  constexpr int WGM = 2, WGN = 4, NWAVES = WGM * WGN;
  constexpr int WM = BM / WGM, WN = BN / WGN, TM = WM / 16, TN = WN / 16;
  static_assert(TM == 8, "four phases of two 16-row blocks");
  constexpr int A_STAGE = BM * BK * 2, B_STAGE = BN * BK * 2;
  constexpr int RING_B = (BM == 256 && BN == 256) ? 3 : 2;
  constexpr int A_RING = 2 * A_STAGE, B_RING = RING_B * B_STAGE;
  constexpr int NIA = BM / 8 / NWAVES, NIB = BN / 8 / NWAVES;   // DMA instructions (1 KB each) per wave, operand and slab
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
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave: a scalar
  const int wm = wave / WGN, wn = wave % WGN;
  const bf16 *Abase = AT ? g.A + m0 : g.A + m0 * g.lda;
  const bf16 *Bbase = BT ? g.B + n0 : g.B + n0 * g.ldb;

  // DMA addressing.  Instruction q of an operand fills LDS bytes [1024 q, 1024 q + 1024) of the stage, lane l
  // the 16 bytes at 16 l; wave w issues the instructions NI w .. NI w + NI - 1.
  //   K-contiguous operand: rows 8q .. 8q+7, lane l: row 8q + l/8, chunk position l%8.  A wave's instructions
  //   differ by 8 rows, the same amount in every lane: one vector offset, the rest in the scalar offset.
  //   Row-contiguous operand: unit 64 q + l of the stage, k-row (64 q + l) / UPR, position (64 q + l) % UPR.
  //   32 units per k-row: instruction i of a wave covers k-rows 8 w + 2 i, + 1 and the permutation depends on the
  //   k-row through k & 3 and bit 3 only, so instructions i and i + 2 differ by 4 k-rows in every lane: two vector
  //   offsets, the rest in the scalar offset.  40 units per k-row: one vector offset per instruction.
  auto dma_offset_k = [&](int q, int64_t ld) -> uint32_t {
    const int row = 8 * q + (lane >> 3), c = (lane & 7) ^ (lane >> 3);   // row % 8 == lane / 8
    return (uint32_t)(row * ld * 2 + c * 16);
  };
  auto dma_offset_t = [&](int q, int64_t ld, int rows) -> uint32_t {
    const int upr = rows / 8, i = 64 * q + lane;
    const int k = i / upr, pos = i % upr;
    const int u = upr == 32 ? tr_pos<32>(pos, k) : tr_pos<40>(pos, k);
    return (uint32_t)(k * ld * 2 + u * 16);
  };
  constexpr int A_NOFF = !AT ? 1 : 2, B_NOFF = !BT ? 1 : BN == 256 ? 2 : NIB;
  static_assert(BM == 256 && NIA == 4, "the A side assumes 256 rows");
  uint32_t a_off[A_NOFF], b_off[B_NOFF];
#pragma unroll
  for (int i = 0; i < A_NOFF; ++i) a_off[i] = AT ? dma_offset_t(wave * NIA + i, g.lda, BM) : dma_offset_k(wave * NIA, g.lda);
#pragma unroll
  for (int i = 0; i < B_NOFF; ++i) b_off[i] = BT ? dma_offset_t(wave * NIB + i, g.ldb, BN) : dma_offset_k(wave * NIB, g.ldb);
  // scalar offset of instruction i: K-contiguous 8 i rows; row-contiguous with 32 units 4 (i / 2) k-rows
  const uint32_t a_step = (uint32_t)((AT ? 8 : 16) * g.lda), b_step = (uint32_t)((BT ? 8 : 16) * g.ldb);
  // With a transposing LDS read in the loop the DMA goes out as inline assembly (see dma16: the
  // compiler would put a wait for all memory operations in front of those reads); otherwise
  // through the builtin, which the scheduling hints below can place.
  auto issue = [&](const bf16 *base, const auto &off, uint32_t step, int ni, char *stage, int i0, int i1) {
    constexpr int NOFF = sizeof(off) / sizeof(off[0]);
    char *dst = stage + wave * (ni * 1024);
    if constexpr (AT || BT) {
      const dma_rsrc_t rs = dma_rsrc(base);
      const uint32_t dst_addr = lds_address(dst);
#pragma unroll
      for (int i = 0; i < 8; ++i)
        if (i < ni && i >= i0 && i < i1) {
          if constexpr (NOFF == 1) dma16(rs, dst_addr + i * 1024, off[0], i * step);
          else if constexpr (NOFF == 2) dma16(rs, dst_addr + i * 1024, off[i & 1], (i >> 1) * step);
          else dma16(rs, dst_addr + i * 1024, off[i < NOFF ? i : 0]);
        }
    } else {
      const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16 *>(base), 0, 0xFFFFFFFFu, 0x00020000);
#pragma unroll
      for (int i = 0; i < 8; ++i)
        if (i < ni && i >= i0 && i < i1)
          __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (__attribute__((address_space(3))) void *)(dst + i * 1024), 16,
                                                   (int)off[0], (int)(i * step), 0, 0);
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
  auto frag = [&](const char *stage, int r0, int kk, bool transposed, int rows) -> bf16x8 {
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
        const int p = rows == 256 ? tr_pos<32>(u, k) : tr_pos<40>(u, k);
        return stage + k * (rows * 2) + p * 16 + (nb & 7) * 2;
      };
      const i16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4 *)addr(kbase));
      const i16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4 *)addr(kbase + 4));
      i16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
      return __builtin_bit_cast(bf16x8, v);
    }
  };
  // Row-contiguous operand in a 256-row stage (32 units per k-row): tr_pos<32>(u, k) = u ^ mask(k), the mask is the
  // same for every k-row a lane ever reads (k mod 4 and k bit 3 do not change with the k-step or the half), and
  // the unit of block b of the wave tile is that of block 0 with 2 b in bits 1 .. 3, which block 0 leaves empty.
  // So all of a lane's fragment addresses in a stage are ONE per-lane offset XOR a value that is the same in every
  // lane (32 b, and the stage's offset, whose bits lie above), plus a constant: one address register per operand
  // instead of one per block.  The uniform value passes through an empty asm statement so that the XOR stays
  // inside the loop (hoisted, the eight results would occupy the registers this saves).
  auto tr256_base = [&](int r0) -> uint32_t {   // block 0 at row r0 of the stage, k-step 0, low half
    const int grp = lane >> 4, L = lane & 15;
    const int nb = r0 + 4 * (L & 3), k = 8 * grp + (L >> 2);
    return (uint32_t)(k * 512 + tr_pos<32>(nb >> 3, k) * 16 + (nb & 7) * 2);
  };
  typedef __attribute__((address_space(3))) const char *lds_ptr;
  auto tr256_block = [&](uint32_t lane_off, uint32_t stage_off, int blk) -> lds_ptr {   // address of (block, k-step 0, low half)
    uint32_t uni = stage_off ^ (uint32_t)(blk * 32);
    asm volatile("" : "+s"(uni));
    return (lds_ptr)(__attribute__((address_space(3))) const char *)smem + (lane_off ^ uni);
  };
  auto frag_tr256 = [&](lds_ptr block, int kk) -> bf16x8 {
    typedef __attribute__((address_space(3))) i16x4 *lds_i16x4_ptr;
    const i16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4_ptr)(block + kk * (32 * 512)));
    const i16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4_ptr)(block + kk * (32 * 512) + 4 * 512));
    i16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8, v);
  };
  constexpr bool A_TR256 = AT, B_TR256 = BT && BN == 256;
  const uint32_t tr_a = A_TR256 ? tr256_base(wm * WM) : 0u, tr_b = B_TR256 ? tr256_base(wn * WN) : 0u;
  // offset of a stage from the start of the rings (a multiple of 32 KB), the same in every lane
  auto stage_offset = [&](const char *stage) { return (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)(stage - smem)); };
  // A slab (two k-steps of 32) is four phases, one per pair of 16-row blocks of the wave tile; a phase issues both
  // k-steps of each of its 2 x TN accumulator blocks back to back.  Two consecutive MFMAs on one accumulator, and
  // beyond that consecutive MFMAs that share an operand, cost measurably less power than the same instructions
  // in another order (a loop of nothing but MFMAs runs 4.5 % faster under the board's power limit with the pairs
  // adjacent, 3 % faster with a shared operand than without), so the order below is a snake through
  // (column block, row block, k-step) in which every step keeps the accumulator or one operand.
  bf16x8 aq[2][2][2];   // A: [buffer = phase parity][row block of the pair][k-step]
  bf16x8 bf[2][TN];     // B: [k-step][column block], all of the slab's
  auto read_aq = [&](const char *abuf, int q) {   // A fragments of phase q (q == 4: phase 0 of the next slab)
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
      if constexpr (A_TR256) {
        const lds_ptr block = tr256_block(tr_a, stage_offset(abuf), 2 * (q & 3) + rb);
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) aq[q & 1][rb][kk] = frag_tr256(block, kk);
      } else {
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) aq[q & 1][rb][kk] = frag(abuf, wm * WM + (2 * (q & 3) + rb) * 16, kk, AT, BM);
      }
    }
  };
  auto read_bj = [&](const char *bbuf, int j) {
    if constexpr (B_TR256) {
      const lds_ptr block = tr256_block(tr_b, stage_offset(bbuf), j);
#pragma unroll
      for (int kk = 0; kk < 2; ++kk) bf[kk][j] = frag_tr256(block, kk);
    } else {
#pragma unroll
      for (int kk = 0; kk < 2; ++kk) bf[kk][j] = frag(bbuf, wn * WN + j * 16, kk, BT, BN);
    }
  };
  auto mfma_col = [&](int q, int j) {   // the 4 MFMAs of column block j in phase q
#pragma unroll
    for (int step = 0; step < 4; ++step) {
      const int t = (j & 1) ? 3 - step : step;   // (rb, kk): (0,0) (0,1) (1,1) (1,0), backwards for odd j
      const int rb = t >> 1, kk = (t & 1) ^ rb;
      acc[2 * q + rb][j] =   // B fragment first: the block comes out transposed, see the epilogue
          __builtin_amdgcn_mfma_f32_16x16x32_bf16(bf[kk][j], aq[q & 1][rb][kk], acc[2 * q + rb][j], 0, 0, 0);
    }
  };

  const int nk = slab1 - slab0;
  auto slab_k = [&](int it) { return (int64_t)(slab0 + (it < nk ? it : nk - 1)) * BK; };
  char *const aring = smem, *const bring = smem + A_RING;
  constexpr int NM = 4 * TN;                                  // MFMAs of a phase
  constexpr int RAQ = (AT ? 2 : 1) * 4, RBJ = (BT ? 2 : 1) * 2;   // LDS read instructions of read_aq / read_bj
  int a_cur = 0, b_cur = 0;   // ring offsets of slab `it`

  // Phases 0 .. 2 read the A fragments of the next phase; phase 3, after the slab's one barrier, those of phase 0
  // of the next slab and, column block by column block as its MFMAs release the registers, the next slab's B
  // fragments.  dma(): the phase's share of the DMA instructions.
  auto phase = [&](auto PH, const char *a_stage, const char *a_next, const char *b_next, auto dma, auto NDMA) {
    constexpr int q = decltype(PH)::value, ndma = decltype(NDMA)::value;
    if constexpr (q < 3) {
      // The two waves of a SIMD take turns on the matrix pipe one phase at a time: the wave that
      // is behind (counted from the barrier) has the higher issue priority.
      __builtin_amdgcn_s_setprio(2 - q);
      read_aq(a_stage, q + 1);
      dma();
#pragma unroll
      for (int j = 0; j < TN; ++j) mfma_col(q, j);
      stream_sched<NM, RAQ, ndma>();
    } else {
      __builtin_amdgcn_s_setprio(3);
      __builtin_amdgcn_sched_barrier(0);
      read_aq(a_next, 4);
      dma();
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        mfma_col(3, j);
        read_bj(b_next, j);
      }
      stream_sched<NM, RAQ + TN * RBJ, ndma, RBJ>();
    }
    __builtin_amdgcn_sched_barrier(0);
  };
  using std::integral_constant;

  if constexpr (RING_B == 3) {
    // prologue: A slab 0, B slabs 0 and 1, first half of A slab 1
    issue(a_at(slab_k(0)), a_off, a_step, NIA, aring, 0, NIA);
    issue(b_at(slab_k(0)), b_off, b_step, NIB, bring, 0, NIB);
    issue(b_at(slab_k(1)), b_off, b_step, NIB, bring + B_STAGE, 0, NIB);
    issue(a_at(slab_k(1)), a_off, a_step, NIA, aring + A_STAGE, 0, NIA / 2);
    wait_dma_and_barrier<NIB + NIA / 2>();   // A 0, B 0 landed
    read_aq(aring, 0);
#pragma unroll
    for (int j = 0; j < TN; ++j) read_bj(bring, j);
    for (int it = 0; it < nk; ++it) {
      const int a_nxt = a_cur ^ A_STAGE;
      const int b_nxt = b_cur + B_STAGE >= B_RING ? b_cur + B_STAGE - B_RING : b_cur + B_STAGE;
      const int b_nn = b_nxt + B_STAGE >= B_RING ? b_nxt + B_STAGE - B_RING : b_nxt + B_STAGE;
      // phase 0: second half of A slab it+1 (into the stage slab it-1 left at the last barrier)
      // phases 1, 2: B slab it+2 into the ring stage that held slab it-1
      // phase 3 (after the barrier): first half of A slab it+2 into the stage slab it just left
      phase(integral_constant<int, 0>{}, aring + a_cur, nullptr, nullptr,
            [&] { issue(a_at(slab_k(it + 1)), a_off, a_step, NIA, aring + a_nxt, NIA / 2, NIA); }, integral_constant<int, NIA / 2>{});
      phase(integral_constant<int, 1>{}, aring + a_cur, nullptr, nullptr,
            [&] { issue(b_at(slab_k(it + 2)), b_off, b_step, NIB, bring + b_nn, 0, NIB / 2); }, integral_constant<int, NIB / 2>{});
      phase(integral_constant<int, 2>{}, aring + a_cur, nullptr, nullptr,
            [&] { issue(b_at(slab_k(it + 2)), b_off, b_step, NIB, bring + b_nn, NIB / 2, NIB); }, integral_constant<int, NIB / 2>{});
      // slab it+1 is complete once only the DMAs of B slab it+2 are outstanding
      wait_dma_and_barrier<NIB>();
      phase(integral_constant<int, 3>{}, nullptr, aring + a_nxt, bring + b_nxt,
            [&] { issue(a_at(slab_k(it + 2)), a_off, a_step, NIA, aring + a_cur, 0, NIA / 2); }, integral_constant<int, NIA / 2>{});
      a_cur = a_nxt;
      b_cur = b_nxt;
    }
  } else {
    // Two stages each way: the stages of slab `it` are free from the barrier of slab `it` on (every wave has
    // read its last fragments of it), and slab it+2 goes there in three groups: all of B right after that
    // barrier (phase 3), A in phases 0 and 1 of slab it+1; slab it+1 has to be complete at the barrier of
    // slab it+1, when nothing else is in flight.
    constexpr int A_FIRST = (NIA + 1) / 2;
    issue(a_at(slab_k(0)), a_off, a_step, NIA, aring, 0, NIA);
    issue(b_at(slab_k(0)), b_off, b_step, NIB, bring, 0, NIB);
    issue(b_at(slab_k(1)), b_off, b_step, NIB, bring + B_STAGE, 0, NIB);
    wait_dma_and_barrier<NIB>();   // A 0, B 0 landed
    read_aq(aring, 0);
#pragma unroll
    for (int j = 0; j < TN; ++j) read_bj(bring, j);
    for (int it = 0; it < nk; ++it) {
      const int a_nxt = a_cur ^ A_STAGE, b_nxt = b_cur ^ B_STAGE;
      phase(integral_constant<int, 0>{}, aring + a_cur, nullptr, nullptr,
            [&] { issue(a_at(slab_k(it + 1)), a_off, a_step, NIA, aring + a_nxt, 0, A_FIRST); }, integral_constant<int, A_FIRST>{});
      phase(integral_constant<int, 1>{}, aring + a_cur, nullptr, nullptr,
            [&] { issue(a_at(slab_k(it + 1)), a_off, a_step, NIA, aring + a_nxt, A_FIRST, NIA); }, integral_constant<int, NIA - A_FIRST>{});
      phase(integral_constant<int, 2>{}, aring + a_cur, nullptr, nullptr, [] {}, integral_constant<int, 0>{});
      wait_dma_and_barrier<0>();   // slab it+1 complete
      phase(integral_constant<int, 3>{}, nullptr, aring + a_nxt, bring + b_nxt,
            [&] { issue(b_at(slab_k(it + 2)), b_off, b_step, NIB, bring + b_cur, 0, NIB); }, integral_constant<int, NIB>{});
      a_cur = a_nxt;
      b_cur = b_nxt;
    }
  }
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
  __builtin_amdgcn_s_setprio(0);

  // Epilogue, wave by wave with no workgroup barrier.  The MFMAs took the B fragment as their first
  // operand, so block (i, j) of the wave tile sits transposed in the registers: lane l holds row
  // 16 i + l % 16 and the four consecutive columns 16 j + 4 (l / 16) .. + 3.  Each wave turns its
  // WM x WN tile, RP rows at a time, through a private LDS patch (16-byte stores,
  // conflict-free at its pitch) into 8-column row segments, so that every global access is 16
  // bytes of a row and a wave instruction covers whole lines.
  // The lane and wave numbers pass through an empty asm statement here: the epilogue's addresses then cannot be
  // computed ahead of the main loop, where they would occupy registers the loop needs (the 320-column tile has
  // 160 of 256 in accumulators).
  int elane = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u)), ewave = wave;
  asm volatile("" : "+v"(elane), "+s"(ewave));
  const int ewm = ewave / WGN, ewn = ewave % WGN;
  constexpr int RP = WN == 80 ? 32 : 64;        // rows per pass
  constexpr int SEG = WN / 8;                   // 8-column segments per row
  constexpr int NRD = RP * SEG / 64;            // read instructions per pass
  static_assert(WM % RP == 0 && (RP * SEG) % 64 == 0, "epilogue passes must tile the wave tile");
  if (PLAIN16 && part_id < 0) {
    // bf16 output with at most a bias: round before the transposition, which halves the LDS
    // traffic of the patch and leaves the second half of the epilogue a plain 16-byte copy.
    // Patch = RP rows per wave; 64 columns: 128 B per row, 16-byte unit u of row r at unit position
    // u ^ ((r >> 1) & 7); 80 columns: 256 B per row (10 units used), unit u at u ^ (r & 15)
    // (8-byte block stores and 16-byte row reads both conflict-free).
    constexpr int PROW = WN == 64 ? 128 : 256;
    char *patch = smem + ewave * (RP * PROW);
    auto unit_pos = [](int unit, int row) { return WN == 64 ? (unit ^ ((row >> 1) & 7)) : (unit ^ (row & 15)); };
    static_assert(WN == 64 || WN == 80, "patch layouts exist for these wave tile widths");
    const int g4 = elane >> 4;
    f32x4 bias4[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
#pragma unroll
      for (int e = 0; e < 4; ++e) bias4[j][e] = 0.0f;
      if (g.ea.flags & MTNLG_EPI_BIAS) {
        const bf16x4 bv = *reinterpret_cast<const bf16x4 *>(static_cast<const bf16 *>(g.ea.bias) + n0 + ewn * WN + j * 16 + 4 * g4);
#pragma unroll
        for (int e = 0; e < 4; ++e) bias4[j][e] = (float)bv[e];
      }
    }
    bf16 *cbase = static_cast<bf16 *>(g.C) + (m0 + ewm * WM) * g.ldc + n0 + ewn * WN;
#pragma unroll
    for (int p = 0; p < WM / RP; ++p) {
#pragma unroll
      for (int i = 0; i < RP / 16; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          const int row = (elane & 15) + i * 16, unit = 2 * j + (g4 >> 1);
          bf16x4 h;
#pragma unroll
          for (int e = 0; e < 4; ++e) h[e] = (bf16)(acc[p * (RP / 16) + i][j][e] + bias4[j][e]);
          *reinterpret_cast<bf16x4 *>(patch + row * PROW + (unit_pos(unit, row) << 4) + (g4 & 1) * 8) = h;
        }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
      for (int t = 0; t < NRD; ++t) {
        const int q = t * 64 + elane, row = q / SEG, cv = q % SEG;
        const bf16x8 o = *reinterpret_cast<const bf16x8 *>(patch + row * PROW + (unit_pos(cv, row) << 4));
        *reinterpret_cast<bf16x8 *>(cbase + (int64_t)(p * RP + row) * g.ldc + cv * 8) = o;
      }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // patch is rewritten by the next pass
    }
  } else {
    constexpr int PITCH = WN + 4;   // floats; 68 and 84 both leave 16-byte block stores of 16 rows conflict-free
    constexpr int NP = WM / RP;
    float *patch = reinterpret_cast<float *>(smem) + ewave * (RP * PITCH);
    const bool whole = part_id < 0;
    // The bias joins in the accumulator layout (4 consecutive columns per lane), and the values a residual or a
    // GeLU' read from aux are fetched two passes ahead, in the registers the accumulators of finished passes
    // leave: no pass waits for global memory except the first.
    const uint32_t flags = whole ? g.ea.flags : 0u;
    bf16x4 bias_h[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
#pragma unroll
      for (int e = 0; e < 4; ++e) bias_h[j][e] = (bf16)0.0f;
      if (flags & MTNLG_EPI_BIAS)
        bias_h[j] = *reinterpret_cast<const bf16x4 *>(static_cast<const bf16 *>(g.ea.bias) + n0 + ewn * WN + j * 16 + 4 * (elane >> 4));
    }
    const bool pre_aux = (flags & (MTNLG_EPI_RESIDUAL | MTNLG_EPI_GELU_GRAD)) != 0;
    const bf16 *aux_base = static_cast<const bf16 *>(g.ea.aux) + (m0 + ewm * WM) * g.ldc + n0 + ewn * WN;
    bf16x8 pre[NP][NRD];
    auto preload = [&](auto P) {
      constexpr int p = decltype(P)::value;
      if constexpr (p < NP) {
        if (pre_aux) {
#pragma unroll
          for (int t = 0; t < NRD; ++t) {
            const int q = t * 64 + elane, row = q / SEG, cv = q % SEG;
            pre[p][t] = *reinterpret_cast<const bf16x8 *>(aux_base + (int64_t)(p * RP + row) * g.ldc + cv * 8);
          }
        }
      }
    };
    preload(std::integral_constant<int, 0>{});
    preload(std::integral_constant<int, 1>{});
    // one pass; instantiated per pass number so that the accumulator blocks are always named at compile time
    // (a pass loop this large is not unrolled on request, and a rolled one would index the registers dynamically)
    auto pass = [&](auto P) {
      constexpr int p = decltype(P)::value;
#pragma unroll
      for (int i = 0; i < RP / 16; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          f32x4 o = acc[p * (RP / 16) + i][j];
#pragma unroll
          for (int e = 0; e < 4; ++e) o[e] += (float)bias_h[j][e];
          *reinterpret_cast<f32x4 *>(patch + ((elane & 15) + i * 16) * PITCH + j * 16 + 4 * (elane >> 4)) = o;
        }
      preload(std::integral_constant<int, p + 2>{});
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
      for (int t = 0; t < NRD; ++t) {
        const int q = t * 64 + elane, row = q / SEG, cv = q % SEG;
        float v[8];
        const f32x4 lo = *reinterpret_cast<const f32x4 *>(patch + row * PITCH + cv * 8);
        const f32x4 hi = *reinterpret_cast<const f32x4 *>(patch + row * PITCH + cv * 8 + 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) { v[e] = lo[e]; v[4 + e] = hi[e]; }
        const int trow = ewm * WM + p * RP + row, tcol = ewn * WN + cv * 8;   // position in the tile
        if (!whole) {  // K-part of a tail tile: raw fp32 partial, summed by splitk_reduce_kernel
          store8(g.partial + (int64_t)part_id * (BM * BN) + trow * BN + tcol, v);
        } else {
          epilogue8(g, m0 + trow, n0 + tcol, v, flags & ~MTNLG_EPI_BIAS, pre_aux ? &pre[p][t] : nullptr);
        }
      }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // patch is rewritten by the next pass
    };
    static_assert(WM / RP == 2 || WM / RP == 4 || WM / RP == 5, "passes are written out below");
    pass(std::integral_constant<int, 0>{});
    pass(std::integral_constant<int, 1>{});
    if constexpr (WM / RP > 2) {
      pass(std::integral_constant<int, 2>{});
      pass(std::integral_constant<int, 3>{});
    }
    if constexpr (WM / RP > 4) pass(std::integral_constant<int, 4>{});
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

// Tile numbering, XCD slices and the split-K plan of one launch.
template <int BM, int BN>
int plan_launch(GemmArgs &g, void *ws, size_t ws_bytes, bool allow_split, unsigned *grid, SplitPlan *plan_out) {
  g.tiles_m = (int)((g.M + BM - 1) / BM);
  g.tiles_n = (int)((g.N + BN - 1) / BN);
  const int64_t tiles = (int64_t)g.tiles_m * g.tiles_n;
  if (tiles > (1 << 28)) return MTNLG_UNSUPPORTED_SHAPE;
  const int nk = (int)((g.K + BK - 1) / BK);
  SplitPlan plan = plan_split(tiles, nk, BM, BN, (ws && allow_split) ? ws_bytes : 0);
  const bool split = plan.tail > 0;
  g.whole_tiles = split ? plan.whole : (int)tiles;
  g.split = split ? plan.split : 1;
  g.part_slabs = split ? plan.part_slabs : nk;
  g.partial = (float *)ws;
  g.per_xcd = (g.whole_tiles + 7) / 8;
  *grid = (unsigned)(g.per_xcd * 8 + (split ? plan.tail * plan.split : 0));
  *plan_out = plan;
  return MTNLG_OK;
}

// General kernel: any shape within its alignment rules.
template <int BM, int BN, int WGM, int WGN, bool AT, bool BT, bool KTAIL>
int launch_k(const GemmArgs &in, void *ws, size_t ws_bytes, hipStream_t st) {
  GemmArgs g = in;
  unsigned grid;
  SplitPlan plan;
  MTNLG_TRY((plan_launch<BM, BN>(g, ws, ws_bytes, true, &grid, &plan)));
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
  gemm_bf16_kernel<BM, BN, WGM, WGN, AT, BT, KTAIL><<<dim3(grid), 64 * WGM * WGN, smem, st>>>(g);
  MTNLG_TRY(check_launch());
  if (plan.tail > 0) {
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

// Streaming kernel: M a multiple of BM, N of BN, K of 64.  Only 256 x 256 tiles split a last round along K.
template <int BM, int BN, bool AT, bool BT>
int launch_stream(const GemmArgs &in, void *ws, size_t ws_bytes, hipStream_t st) {
  GemmArgs g = in;
  if (g.M % BM || g.N % BN || g.K % BK) return MTNLG_UNSUPPORTED_SHAPE;
  unsigned grid;
  SplitPlan plan;
  MTNLG_TRY((plan_launch<BM, BN>(g, ws, ws_bytes, BM == 256 && BN == 256, &grid, &plan)));
  constexpr int ring_b = (BM == 256 && BN == 256) ? 3 : 2;
  constexpr int smem = (2 * BM + ring_b * BN) * BK * 2;
  static unsigned long long attr_done = 0;
  int device;
  if (!attr_is_set(attr_done, &device)) {
    if (hipFuncSetAttribute((const void *)gemm_stream_kernel<BM, BN, AT, BT, false>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, smem) != hipSuccess ||
        hipFuncSetAttribute((const void *)gemm_stream_kernel<BM, BN, AT, BT, true>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, smem) != hipSuccess)
      return MTNLG_HIP_ERROR;
    attr_mark_set(attr_done, device);
  }
  // bf16 output with nothing but an optional bias: the epilogue that rounds before it transposes
  if ((g.ea.flags & ~(uint32_t)MTNLG_EPI_BIAS) == 0)
    gemm_stream_kernel<BM, BN, AT, BT, true><<<dim3(grid), 512, smem, st>>>(g);
  else
    gemm_stream_kernel<BM, BN, AT, BT, false><<<dim3(grid), 512, smem, st>>>(g);
  MTNLG_TRY(check_launch());
  if (plan.tail > 0) {
    splitk_reduce_kernel<BM, BN><<<dim3(8, plan.tail), 256, 0, st>>>(g);
    MTNLG_TRY(check_launch());
  }
  return MTNLG_OK;
}

template <bool AT, bool BT>
int launch_tile(int tile, const GemmArgs &g, void *ws, size_t ws_bytes, hipStream_t st) {
  switch (tile) {
    case GEMM_TILE_GENERAL_256: return launch<256, 256, 2, 4, AT, BT>(g, ws, ws_bytes, st);
    case GEMM_TILE_GENERAL_128: return launch<128, 128, 2, 2, AT, BT>(g, ws, ws_bytes, st);
    case GEMM_TILE_STREAM_256x256: return launch_stream<256, 256, AT, BT>(g, ws, ws_bytes, st);
    case GEMM_TILE_STREAM_256x320: return launch_stream<256, 320, AT, BT>(g, ws, ws_bytes, st);
    default: return MTNLG_INVALID_ARG;
  }
}

// Rounds of 256 workgroups a tiling needs, counting a last round that is split along K by its share.
double rounds_of(int64_t tiles, bool can_split, int nk) {
  const int cus = 256;
  if (can_split && plan_split(tiles, nk, 256, 256, ~(size_t)0).tail > 0) return (double)tiles / cus + 0.15;
  return (double)((tiles + cus - 1) / cus);
}

}  // namespace

// Which kernel and tile shape take a problem.  Aligned problems go to the streaming kernel; among its tile
// shapes the one with the least estimated time wins: rounds of 256 tiles x tile area x a measured relative
// cost per FLOP of the shape (wider tiles move fewer operand bytes per FLOP).  Without workspace a last
// round cannot be split along K and counts in full.
int gemm_mfma_pick_tile(int layout, int64_t M, int64_t N, int64_t K, bool have_workspace) {
  if (M <= 0 || N <= 0 || K <= 0) return GEMM_TILE_GENERAL_256;
  const int nk = (int)((K + BK - 1) / BK);
  if (K % BK == 0 && M % 256 == 0) {
    double best = 1e300;
    int pick = -1;
    auto offer = [&](int tile, int64_t bm, int64_t bn, double cost_per_flop, bool can_split) {
      if (M % bm || N % bn) return;
      const int64_t tiles = (M / bm) * (N / bn);
      const double t = rounds_of(tiles, can_split && have_workspace, nk) * (double)(bm * bn) * cost_per_flop;
      if (t < best) { best = t; pick = tile; }
    };
    const int64_t tiles256 = N % 256 == 0 ? (M / 256) * (N / 256) : 0;
    // small problems: 128 x 128 tiles of the general kernel (two workgroups per compute unit)
    const bool small = tiles256 > 0 && tiles256 < 160 && !(have_workspace && plan_split(tiles256, nk, 256, 256, ~(size_t)0).tail > 0);
    if (!small || N % 256) {
      offer(GEMM_TILE_STREAM_256x256, 256, 256, 1.00, true);
      offer(GEMM_TILE_STREAM_256x320, 256, 320, GEMM_COST_256x320, false);
      if (pick >= 0) return pick;
    }
  }
  const int64_t tiles256 = ((M + 255) / 256) * ((N + 255) / 256);
  const SplitPlan plan = plan_split(tiles256, nk, 256, 256, have_workspace ? ~(size_t)0 : 0);
  if (plan.tail == 0 && tiles256 < 160) return GEMM_TILE_GENERAL_128;
  return GEMM_TILE_GENERAL_256;
}

size_t gemm_mfma_workspace_bytes(int layout, int64_t M, int64_t N, int64_t K) {
  if (M <= 0 || N <= 0 || K <= 0) return 0;
  const int tile = gemm_mfma_pick_tile(layout, M, N, K, true);
  if (tile != GEMM_TILE_STREAM_256x256 && tile != GEMM_TILE_GENERAL_256) return 0;
  const int64_t tiles256 = ((M + 255) / 256) * ((N + 255) / 256);
  return plan_split(tiles256, (int)((K + BK - 1) / BK), 256, 256, 0).workspace;
}

int gemm_mfma_bf16(int layout, int64_t M, int64_t N, int64_t K, const void *A, const void *B, void *C,
                   const void *bias, void *aux, uint32_t epi, void *ws, size_t ws_bytes, hipStream_t stream,
                   int prof_class, int tile) {
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
  if (tile < 0)
    tile = gemm_mfma_pick_tile(layout, M, N, K, ws != nullptr && ws_bytes >= gemm_mfma_workspace_bytes(layout, M, N, K));
  LaunchScope scope(prof_class >= 0 ? prof_class : MTNLG_K_GEMM_NT + layout, stream);
  if (!at && !bt) return launch_tile<false, false>(tile, g, ws, ws_bytes, stream);
  if (!at && bt) return launch_tile<false, true>(tile, g, ws, ws_bytes, stream);
  return launch_tile<true, true>(tile, g, ws, ws_bytes, stream);
}

}  // namespace mtnlg
