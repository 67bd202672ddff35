// Fused causal softmax attention on the gfx950 matrix cores (bf16 in, fp32 softmax
// and accumulation), forward and backward, for head sizes 64, 128 and 160.
//
//   S = scale * q k^T (causal),  P = rowsoftmax(S),  a = P v,  lse = log sum exp(S)
//   backward with D_t = da_t . a_t :  dP = da v^T,  dS = P o (dP - D),
//   dq = scale dS k,  dk = scale dS^T q,  dv = P^T da.
//
// Three kernels, one geometry.  A workgroup owns 128 (or, forward only, 256) rows of one side (queries for
// forward and dq, keys for dk/dv), 16 or 32 per wave on eight waves, held in registers as MFMA
// B operands (groups of 16, one row per lane column); the other side streams through
// LDS in tiles of 64 rows, brought in by LDS DMA (buffer_load ... lds, no staging
// registers) three tiles deep, one workgroup barrier per tile.
//
// All products are v_mfma_f32_16x16x32_bf16 with the streamed tile as the A operand, so a
// product block comes out as C[tile row 4 (lane/16) + i][own row lane%16], i = 0..3:
//   forward : S^T = K Q^T; the softmax statistics of a query live in the four lanes that
//             share lane%16; P^T packed to bf16 is directly the B operand of O^T += V^T P^T.
//   dq      : S^T and dP^T = V dO^T the same way, dQ^T += K^T dS^T.
//   dk / dv : S = Q K^T, dP = dO V^T with the key on the lane column,
//             dV^T += dO^T P, dK^T += Q^T dS.
// The second product of each chain contracts over the tile's rows.  Its A operand is read
// from the same natural [row][D] tile with the transposing LDS read (ds_read_b64_tr_b16: a
// 16-lane group reads 4 tile rows x 16 columns, each lane receives the 4 row values of its
// column); the k slots of that MFMA are ordered to match the accumulator layout of the
// first product (slot (g, e) of a 32-row step = tile row 4g + e for e < 4, 16 + 4g + e - 4
// otherwise), so P and dS never leave the registers and nothing is transposed in software.
// No atomics: every output element has one owner, results are run-to-run identical.
#include <math.h>

#include "common.h"

namespace mtnlg {

namespace {

typedef __attribute__((ext_vector_type(8))) short i16x8;
typedef __attribute__((ext_vector_type(4))) short i16x4;
typedef __attribute__((address_space(3))) i16x4 *lds_i16x4_ptr;

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

#define MFMA16(a, b, c) __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0)

// 2^x on the transcendental unit (v_exp_f32): no denormal fix-up, 2^-inf = 0.
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// A 64-row x D-column bf16 tile in LDS, rows as in memory, the 16-byte units of a row
// permuted by an XOR that depends on the row.  The masks are the ones a micro-benchmark of the
// two fragment read patterns found fastest (cycles per wave instruction, two waves per SIMD):
// head size 160: 4.5-4.9 for the 16-byte reads and 3.0 for the transposing reads (no conflicts);
// 64: the same; 128: 4.5 and 4.0 (no mask of this form is conflict-free for both at a row of
// exactly 256 bytes).  The masks look at the low four bits of the row only.
template <int D>
struct Tile {
  static constexpr int UPR = D / 8;        // 16-byte units per row
  static constexpr int BYTES = 64 * D * 2;
  static constexpr int NI = D / 32;        // DMA instructions per wave and tile (16 rows)
  static __device__ __forceinline__ int mask(int row) {
    if constexpr (D == 160) return (row >> 1) & 3;
    else if constexpr (D == 128) return row & 15;
    else return row & 7;
  }
  static __device__ __forceinline__ int off(int row, int u) { return (row * UPR + (u ^ mask(row))) * 16; }

  // Wave `wave` brings rows 16 wave .. 16 wave + 15 of the tile whose first row is row0 of the
  // matrix behind rs (row pitch ld_bytes) to LDS byte address `stage` with NI DMA instructions;
  // rows past the end repeat the last row.  Instruction i fills 1024 consecutive LDS bytes, lane l
  // the 16 bytes at 16 l.
  template <int TAG>
  static __device__ __forceinline__ void dma_one(dma_rsrc_t rs, int row0, int rows_total, uint32_t ld_bytes,
                                                 uint32_t stage, int wave, int lane, int i) {
    const int p = i * 64 + lane;
    const int r = 16 * wave + p / UPR, u = (p % UPR) ^ mask(16 * wave + p / UPR);
    int gr = row0 + r;
    gr = gr < rows_total ? gr : rows_total - 1;
    dma16<TAG>(rs, stage + (wave * NI + i) * 1024, gr * ld_bytes + u * 16);
  }
  // Byte offsets of a lane's fragment reads inside a tile.  mask() looks at the low four bits of a
  // row only, so a block of 16 rows further down is a constant distance away.
  struct Lane {
    int nat[D / 32];   // row lane%16, 16-byte unit 4 kk + lane/16
    int tr[D / 16];    // as address supplier of a transposing read: row 4 (lane/16) + L/4, columns 16 cblk + 4 (L%4) .. + 3, L = lane%16
    __device__ __forceinline__ explicit Lane(int lane) {
      const int g = lane >> 4, L = lane & 15;
#pragma unroll
      for (int kk = 0; kk < D / 32; ++kk) nat[kk] = off(L, 4 * kk + g);
#pragma unroll
      for (int cb = 0; cb < D / 16; ++cb) {
        const int col = cb * 16 + 4 * (L & 3);
        tr[cb] = off(4 * g + (L >> 2), col >> 3) + (col & 7) * 2;
      }
    }
  };
  static constexpr int ROWS16 = 16 * UPR * 16;   // bytes of 16 tile rows
  // A operand contracting over columns: lane l holds row 16 blk + l%16, columns 32 kk + 8 (l/16) .. + 7
  static __device__ __forceinline__ bf16x8 nat(const char *t, const Lane &ln, int blk, int kk) {
    return *reinterpret_cast<const bf16x8 *>(t + ln.nat[kk] + blk * ROWS16);
  }
  // A operand contracting over tile rows 32 ks .. 32 ks + 31: lane l holds column 16 cblk + l%16 and,
  // with g = l/16, tile rows 32 ks + 4 g .. + 3 (elements 0-3) and 32 ks + 16 + 4 g .. + 3 (4-7).
  static __device__ __forceinline__ bf16x8 tr(const char *t, const Lane &ln, int cblk, int ks) {
    const char *p = t + ln.tr[cblk] + 2 * ks * ROWS16;
    const i16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4_ptr)p);
    const i16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4_ptr)(p + ROWS16));
    const i16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8, v);
  }
};

// call-site tags of the DMA helpers
struct Burst { static constexpr int value = 0; };
struct Spread { static constexpr int value = 1; };

// two accumulator blocks (tile rows 32 ks + 4g + i and 32 ks + 16 + 4g + i) as the bf16 B operand
__device__ __forceinline__ bf16x8 pack2(const f32x4 &lo, const f32x4 &hi) {
  bf16x8 o;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    o[i] = (bf16)lo[i];
    o[4 + i] = (bf16)hi[i];
  }
  return o;
}

// Steps 0 .. N-1 of a run of MFMAs whose A operands come from LDS: load(i) fetches the fragments
// of step i, mma(i) multiplies with them, extra(i) is whatever else should issue during step i.
// The loads run P steps ahead of the MFMAs, and nothing may be scheduled across a step boundary:
// left alone, the compiler issues each LDS read right in front of its MFMA and the wave (one per
// SIMD in these kernels) sits out the LDS latency each time.
template <int N, int P, typename L>
__device__ __forceinline__ void pipelined_start(L &&load) {
#pragma unroll
  for (int i = 0; i < P && i < N; ++i) load(i);
  __builtin_amdgcn_sched_barrier(0);
}
template <int N, int P, typename L, typename M, typename X>
__device__ __forceinline__ void pipelined_run(L &&load, M &&mma, X &&extra) {
#pragma unroll
  for (int i = 0; i < N; ++i) {
    if (i + P < N) load(i + P);
    extra(i);
    mma(i);
    __builtin_amdgcn_sched_barrier(0);
  }
}
template <int N, int P, typename L, typename M, typename X>
__device__ __forceinline__ void pipelined(L &&load, M &&mma, X &&extra) {
  pipelined_start<N, P>(load);
  pipelined_run<N, P>(load, mma, extra);
}
template <int N, int P, typename L, typename M>
__device__ __forceinline__ void pipelined(L &&load, M &&mma) {
  pipelined<N, P>(load, mma, [](int) {});
}

// wait until at most N of this wave's memory operations are outstanding, then the workgroup barrier
template <int N>
__device__ __forceinline__ void wait_and_barrier() {
  asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
}

// The value is needed "now": makes the compiler wait for the global load behind v here, before the
// main loop, rather than at the first use inside it -- a wait for ordinary loads inside the loop
// would also drain the DMAs in flight, which the compiler does not know about.
template <typename V>
__device__ __forceinline__ void arrive(V &v) {
  asm volatile("" : "+v"(v));
}
// An accumulator block that only MFMAs touch inside the main loop stays in the accumulation
// registers: without this hint at the top of the loop body the compiler moves every block to the
// ordinary registers and back once per tile.
__device__ __forceinline__ void keep_acc(f32x4 &v) {
  asm volatile("" : "+a"(v));
}

// sum / maximum over the four lanes that share lane % 16
__device__ __forceinline__ float quad_sum(float v) {
  v += __shfl_xor(v, 16, 64);
  return v + __shfl_xor(v, 32, 64);
}
__device__ __forceinline__ float quad_max(float v) {
  v = fmaxf(v, __shfl_xor(v, 16, 64));
  return fmaxf(v, __shfl_xor(v, 32, 64));
}

// Which rows (queries in the forward and dq kernels, keys in the dk/dv kernel) a wave owns.
// Under the causal mask a 64-row block b works on b + 1 of the 64-row tiles the workgroup streams
// (or, for keys, on all tiles from b on), so blocks taken in order would leave the workgroups of a
// head with 1 .. s/64 tiles of work.  With eight waves the two halves of a workgroup therefore take
// blocks p and nb - 1 - p (nb blocks in the sequence): every workgroup then computes nb + 1 wave-halves
// of tiles, and while only one half has work in a tile it has the compute unit to itself.  With an
// odd nb the middle block is alone in its workgroup and the other half only helps to move tiles.
// Four waves of 32 rows (G = 2) keep consecutive 128-row blocks.
template <int G, int W = 8 / G>
struct RowBlocks {
  int row0;        // first row of this wave
  int first_tile;  // lowest and highest 64-row block of the workgroup: the tile range that the
  int last_tile;   //   forward / dq kernels (0 .. last) and the dk/dv kernel (first .. end) stream
  bool idle;       // wave-uniform: this wave owns no rows
  __device__ RowBlocks(int s, int pair, int wave) {
    const int nb = (s + 63) / 64;
    if (W == 4) {
      row0 = pair * 128 + wave * 32;
      first_tile = 2 * pair;
      last_tile = 2 * pair + 1 < nb ? 2 * pair + 1 : nb - 1;
      idle = false;
    } else {
      // eight waves: the two halves own blocks lo and hi of 64 G rows from opposite ends of the sequence
      constexpr int TPB = G;   // 64-row tiles per block
      const int nblk = (nb + TPB - 1) / TPB;
      const int lo = pair, hi = nblk - 1 - pair, half = wave >> 2;
      row0 = (half ? hi : lo) * (64 * G) + (wave & 3) * (16 * G);
      first_tile = lo * TPB;
      last_tile = hi * TPB + TPB - 1 < nb ? hi * TPB + TPB - 1 : nb - 1;
      idle = half && hi == lo;
    }
  }
  // workgroups along x for a sequence of s rows
  static int grid(int s) {
    const int nb = (s + 63) / 64;
    return W == 4 ? (s + 127) / 128 : ((nb + G - 1) / G + 1) / 2;
  }
};

// ------------------------------------------------------------------ forward
template <int D, int G, int W = 8 / G>
__global__ __launch_bounds__(64 * W) void attn_fwd_kernel(int s, int n, float scale, const bf16 *__restrict__ qkv,
                                                      bf16 *__restrict__ a, float *__restrict__ lse) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  using T = Tile<D>;
  constexpr int KK = D / 32, DB = D / 16, STAGE = 2 * T::BYTES;
  const int j = blockIdx.y, bi = blockIdx.z;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, g = lane >> 4, lr = lane & 15;
  const int64_t ld = (int64_t)n * 3 * D;
  const bf16 *base = qkv + (int64_t)bi * s * ld + (int64_t)j * 3 * D;
  const RowBlocks<G, W> rb(s, blockIdx.x, wave);
  const int qw = rb.row0;
  const float c = scale * kLog2e;
  const typename T::Lane ln(lane);
  const uint32_t smem_addr = lds_address(smem);

  int qc[G];
  bf16x8 qf[G][KK];
#pragma unroll
  for (int qg = 0; qg < G; ++qg) {
    const int q = qw + 16 * qg + lr;
    qc[qg] = q < s ? q : s - 1;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk)
      qf[qg][kk] = *reinterpret_cast<const bf16x8 *>(base + (int64_t)qc[qg] * ld + 32 * kk + 8 * g);
  }
  f32x4 o[G][DB];
#pragma unroll
  for (int qg = 0; qg < G; ++qg)
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int e = 0; e < 4; ++e) o[qg][db][e] = 0.0f;
  float m[G], l[G];   // l: this lane's share of the row sum
#pragma unroll
  for (int qg = 0; qg < G; ++qg) {
    m[qg] = -INFINITY;
    l[qg] = 0.0f;
  }

  const int ntiles = rb.last_tile + 1;
  // Who brings what: with four waves wave w brings rows 16 w .. 16 w + 15 of the K tile and of
  // the V tile; with eight, waves 0-3 bring the K tile, waves 4-7 the V tile.
  constexpr int IPW = (W == 4 ? 2 : 1) * T::NI;   // DMA instructions per wave and tile
  const int quarter = W == 4 ? wave : (wave & 3), half = W == 4 ? 0 : (wave >> 2);
  const dma_rsrc_t rk = dma_rsrc(base + D + half * D), rv = dma_rsrc(base + 2 * D);
  // DMA instruction i (of IPW) of tile t (clamped to the last one) into ring stage st.  A tile's
  // DMAs go out one per step of the first MFMA run of the tile before: a burst of them would hold
  // the waves at the issue port of the texture path.
  auto issue_one = [&](auto tag, int t, int st, int i) {
    constexpr int TAG = decltype(tag)::value;
    const int tt = t < ntiles ? t : ntiles - 1;
    if (W == 8 || i < T::NI)
      T::template dma_one<TAG>(rk, tt * 64, s, (uint32_t)(ld * 2), smem_addr + st * STAGE + half * T::BYTES, quarter, lane, i);
    else
      T::template dma_one<TAG>(rv, tt * 64, s, (uint32_t)(ld * 2), smem_addr + st * STAGE + T::BYTES, quarter, lane, i - T::NI);
  };
  auto issue = [&](int t, int st) {
#pragma unroll
    for (int i = 0; i < IPW; ++i) issue_one(Burst{}, t, st, i);
  };
  issue(0, 0);
  issue(1, 1);
#pragma unroll
  for (int qg = 0; qg < G; ++qg)
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) arrive(qf[qg][kk]);
  int cur = 0;
  for (int it = 0; it < ntiles; ++it) {
    wait_and_barrier<IPW>();   // tile it landed everywhere, tile it-1 no longer read
    const int nn = cur == 0 ? 2 : cur - 1;   // stage of tile it + 2
    const char *Kt = smem + cur * STAGE, *Vt = Kt + T::BYTES;
    const int kv0 = it * 64;
    if (rb.idle || kv0 > qw + (16 * G - 1)) {  // wave-uniform: every (query, key) pair of this wave is masked
      issue(it + 2, nn);
    } else {
      f32x4 sc[G][4];
#pragma unroll
      for (int qg = 0; qg < G; ++qg)
#pragma unroll
        for (int kb = 0; kb < 4; ++kb)
#pragma unroll
          for (int e = 0; e < 4; ++e) sc[qg][kb][e] = 0.0f;
      {  // step i: k-step i / 2, key blocks 2 (i % 2) and 2 (i % 2) + 1
        bf16x8 kfr[4][2];
        pipelined<2 * KK, 3>(
            [&](int i) {
#pragma unroll
              for (int h = 0; h < 2; ++h) kfr[i & 3][h] = T::nat(Kt, ln, 2 * (i & 1) + h, i >> 1);
            },
            [&](int i) {
#pragma unroll
              for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int qg = 0; qg < G; ++qg)
                  sc[qg][2 * (i & 1) + h] = MFMA16(kfr[i & 3][h], qf[qg][i >> 1], sc[qg][2 * (i & 1) + h]);
            },
            [&](int i) {
              if (i < IPW) issue_one(Spread{}, it + 2, nn, i);
            });
      }
      // element (qg, kb, e): key kv0 + 16 kb + 4 g + e, query qc[qg]
      if (kv0 + 63 > qw) {  // wave-uniform: this tile crosses the diagonal for some row
#pragma unroll
        for (int qg = 0; qg < G; ++qg)
#pragma unroll
          for (int kb = 0; kb < 4; ++kb)
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (kv0 + 16 * kb + 4 * g + e > qc[qg]) sc[qg][kb][e] = -INFINITY;
      }
      // m tracks the running maximum of the raw scores; exponents are taken in base 2 with the
      // scale folded in: p = 2^(s c - m c).
      float alpha[G];
#pragma unroll
      for (int qg = 0; qg < G; ++qg) {
        float mx = -INFINITY;
#pragma unroll
        for (int kb = 0; kb < 4; ++kb)
#pragma unroll
          for (int e = 0; e < 4; ++e) mx = fmaxf(mx, sc[qg][kb][e]);
        mx = quad_max(mx);
        // The reference maximum only follows when the row maximum has outgrown it by more than
        // 2^8 in the exponent's units (any reference gives the same sums; this one keeps p <= 256
        // and makes rescaling O rare).  Finite from the first tile on: key 0 is never masked.
        const float m_new = mx * c > m[qg] * c + 8.0f ? mx : m[qg];
        const float mc = m_new * c;
        float rs = 0.0f;
#pragma unroll
        for (int kb = 0; kb < 4; ++kb)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float p = fast_exp2(fmaf(sc[qg][kb][e], c, -mc));
            sc[qg][kb][e] = p;
            rs += p;
          }
        alpha[qg] = fast_exp2((m[qg] - m_new) * c);
        l[qg] = l[qg] * alpha[qg] + rs;
        m[qg] = m_new;
      }
      bool moved = false;
#pragma unroll
      for (int qg = 0; qg < G; ++qg) moved = moved || alpha[qg] != 1.0f;
      if (__builtin_amdgcn_ballot_w64(moved) != 0) {  // a reference maximum moved: rescale O
#pragma unroll
        for (int qg = 0; qg < G; ++qg)
#pragma unroll
          for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int e = 0; e < 4; ++e) o[qg][db][e] *= alpha[qg];
      }
      {  // step i: key half i / (DB / 2), output blocks 2 (i % (DB / 2)) and + 1
        bf16x8 pf[2][G], vfr[4][2];
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
          for (int qg = 0; qg < G; ++qg) pf[ks][qg] = pack2(sc[qg][2 * ks], sc[qg][2 * ks + 1]);
        constexpr int HB = DB / 2;
        pipelined<2 * HB, 3>(
            [&](int i) {
#pragma unroll
              for (int h = 0; h < 2; ++h) vfr[i & 3][h] = T::tr(Vt, ln, 2 * (i % HB) + h, i / HB);
            },
            [&](int i) {
#pragma unroll
              for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int qg = 0; qg < G; ++qg)
                  o[qg][2 * (i % HB) + h] = MFMA16(vfr[i & 3][h], pf[i / HB][qg], o[qg][2 * (i % HB) + h]);
            });
      }
    }
    cur = cur == 2 ? 0 : cur + 1;
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the clamped look-ahead tiles

#pragma unroll
  for (int qg = 0; qg < G; ++qg) {
    const int q = qw + 16 * qg + lr;
    const float lsum = quad_sum(l[qg]);
    if (q < s && !rb.idle) {
      const float inv = 1.0f / lsum;
      bf16 *out = a + ((int64_t)bi * s + q) * ((int64_t)n * D) + (int64_t)j * D;
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        bf16x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = (bf16)(o[qg][db][e] * inv);
        *reinterpret_cast<bf16x4 *>(out + db * 16 + 4 * g) = v;
      }
      if (g == 0) lse[((int64_t)bi * n + j) * s + q] = (m[qg] * c + log2f(lsum)) * kLn2;
    }
  }
}

// ------------------------------------------------------------------ backward: dq (and D)
template <int D, int G, int W = 8 / G>
__global__ __launch_bounds__(64 * W) void attn_bwd_dq_kernel(int s, int n, float scale, const bf16 *__restrict__ qkv,
                                                         const bf16 *__restrict__ a, const float *__restrict__ lse,
                                                         const bf16 *__restrict__ da, bf16 *__restrict__ dqkv,
                                                         float *__restrict__ Dvec) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  using T = Tile<D>;
  constexpr int KK = D / 32, DB = D / 16, STAGE = 2 * T::BYTES;
  const int j = blockIdx.y, bi = blockIdx.z;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, g = lane >> 4, lr = lane & 15;
  const int64_t ld = (int64_t)n * 3 * D, pld = (int64_t)n * D;
  const bf16 *base = qkv + (int64_t)bi * s * ld + (int64_t)j * 3 * D;
  const RowBlocks<G, W> rb(s, blockIdx.x, wave);
  const int qw = rb.row0;
  const float c = scale * kLog2e;
  const typename T::Lane ln(lane);
  const uint32_t smem_addr = lds_address(smem);

  int qc[G];
  bf16x8 qf[G][KK], dof[G][KK];
  float dsum[G], lse2[G];
#pragma unroll
  for (int qg = 0; qg < G; ++qg) {
    const int q = qw + 16 * qg + lr;
    qc[qg] = q < s ? q : s - 1;
    const bf16 *dar = da + ((int64_t)bi * s + qc[qg]) * pld + (int64_t)j * D;
    const bf16 *ar = a + ((int64_t)bi * s + qc[qg]) * pld + (int64_t)j * D;
    float ds = 0.0f;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      qf[qg][kk] = *reinterpret_cast<const bf16x8 *>(base + (int64_t)qc[qg] * ld + 32 * kk + 8 * g);
      dof[qg][kk] = *reinterpret_cast<const bf16x8 *>(dar + 32 * kk + 8 * g);
      const bf16x8 av = *reinterpret_cast<const bf16x8 *>(ar + 32 * kk + 8 * g);
#pragma unroll
      for (int i = 0; i < 8; ++i) ds += (float)dof[qg][kk][i] * (float)av[i];
    }
    dsum[qg] = quad_sum(ds);
    lse2[qg] = lse[((int64_t)bi * n + j) * s + qc[qg]] * kLog2e;
    if (q < s && g == 0 && !rb.idle) Dvec[((int64_t)bi * n + j) * s + q] = dsum[qg];
  }

  f32x4 dq[G][DB];
#pragma unroll
  for (int qg = 0; qg < G; ++qg)
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int e = 0; e < 4; ++e) dq[qg][db][e] = 0.0f;

  const int ntiles = rb.last_tile + 1;
  // tile DMAs as in the forward kernel
  constexpr int IPW = (W == 4 ? 2 : 1) * T::NI;
  const int quarter = W == 4 ? wave : (wave & 3), half = W == 4 ? 0 : (wave >> 2);
  const dma_rsrc_t rk = dma_rsrc(base + D + half * D), rv = dma_rsrc(base + 2 * D);
  auto issue_one = [&](auto tag, int t, int st, int i) {
    constexpr int TAG = decltype(tag)::value;
    const int tt = t < ntiles ? t : ntiles - 1;
    if (W == 8 || i < T::NI)
      T::template dma_one<TAG>(rk, tt * 64, s, (uint32_t)(ld * 2), smem_addr + st * STAGE + half * T::BYTES, quarter, lane, i);
    else
      T::template dma_one<TAG>(rv, tt * 64, s, (uint32_t)(ld * 2), smem_addr + st * STAGE + T::BYTES, quarter, lane, i - T::NI);
  };
  auto issue = [&](int t, int st) {
#pragma unroll
    for (int i = 0; i < IPW; ++i) issue_one(Burst{}, t, st, i);
  };
  issue(0, 0);
  issue(1, 1);
#pragma unroll
  for (int qg = 0; qg < G; ++qg) {
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      arrive(qf[qg][kk]);
      arrive(dof[qg][kk]);
    }
    arrive(lse2[qg]);
    arrive(dsum[qg]);
  }
  int cur = 0;
  for (int it = 0; it < ntiles; ++it) {
    wait_and_barrier<IPW>();
#pragma unroll
    for (int qg = 0; qg < G; ++qg)
#pragma unroll
      for (int db = 0; db < DB; ++db) keep_acc(dq[qg][db]);
    const int nn = cur == 0 ? 2 : cur - 1;
    const char *Kt = smem + cur * STAGE, *Vt = Kt + T::BYTES;
    const int kv0 = it * 64;
    if (rb.idle || kv0 > qw + (16 * G - 1)) {
      issue(it + 2, nn);
    } else {
      f32x4 sc[G][4], pc[G][4];
#pragma unroll
      for (int qg = 0; qg < G; ++qg)
#pragma unroll
        for (int kb = 0; kb < 4; ++kb)
#pragma unroll
          for (int e = 0; e < 4; ++e) sc[qg][kb][e] = pc[qg][kb][e] = 0.0f;
      {  // step i: k-step i / 2, key blocks 2 (i % 2) and + 1
        bf16x8 kfr[2][2], vfr[2][2];
        pipelined<2 * KK, 1>(
            [&](int i) {
#pragma unroll
              for (int h = 0; h < 2; ++h) {
                kfr[i & 1][h] = T::nat(Kt, ln, 2 * (i & 1) + h, i >> 1);
                vfr[i & 1][h] = T::nat(Vt, ln, 2 * (i & 1) + h, i >> 1);
              }
            },
            [&](int i) {
#pragma unroll
              for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int qg = 0; qg < G; ++qg) {
                  sc[qg][2 * (i & 1) + h] = MFMA16(kfr[i & 1][h], qf[qg][i >> 1], sc[qg][2 * (i & 1) + h]);
                  pc[qg][2 * (i & 1) + h] = MFMA16(vfr[i & 1][h], dof[qg][i >> 1], pc[qg][2 * (i & 1) + h]);
                }
            },
            [&](int i) {
              if (i < IPW) issue_one(Spread{}, it + 2, nn, i);
            });
      }
      // dS^T = P^T o (dP^T - D); element (qg, kb, e): key kv0 + 16 kb + 4 g + e, query qc[qg]
      const bool diag = kv0 + 63 > qw;  // wave-uniform: diagonal (or past-the-end keys) in this tile
      // one half of the tile's keys at a time: dS of key blocks 2 ks, 2 ks + 1, then their 2 DB
      // MFMAs, step i = output blocks 2 i, 2 i + 1
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        bf16x8 df[G], ktr[4][2];
        auto load = [&](int i) {
#pragma unroll
          for (int h = 0; h < 2; ++h) ktr[i & 3][h] = T::tr(Kt, ln, 2 * i + h, ks);
        };
        pipelined_start<DB / 2, 3>(load);
#pragma unroll
        for (int qg = 0; qg < G; ++qg)
#pragma unroll
          for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const int kb = 2 * ks + h;
              float p = fast_exp2(fmaf(sc[qg][kb][e], c, -lse2[qg]));
              if (diag && kv0 + 16 * kb + 4 * g + e > qc[qg]) p = 0.0f;
              sc[qg][kb][e] = p * (pc[qg][kb][e] - dsum[qg]);
            }
#pragma unroll
        for (int qg = 0; qg < G; ++qg) df[qg] = pack2(sc[qg][2 * ks], sc[qg][2 * ks + 1]);
        pipelined_run<DB / 2, 3>(
            load,
            [&](int i) {
#pragma unroll
              for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int qg = 0; qg < G; ++qg) dq[qg][2 * i + h] = MFMA16(ktr[i & 3][h], df[qg], dq[qg][2 * i + h]);
            },
            [](int) {});
      }
    }
    cur = cur == 2 ? 0 : cur + 1;
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

#pragma unroll
  for (int qg = 0; qg < G; ++qg) {
    const int q = qw + 16 * qg + lr;
    if (q < s && !rb.idle) {
      bf16 *out = dqkv + ((int64_t)bi * s + q) * ld + (int64_t)j * 3 * D;
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        bf16x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = (bf16)(dq[qg][db][e] * scale);
        *reinterpret_cast<bf16x4 *>(out + db * 16 + 4 * g) = v;
      }
    }
  }
}

// ------------------------------------------------------------------ backward: dk, dv
template <int D, int G>
__global__ __launch_bounds__(512 / G) void attn_bwd_dkv_kernel(int s, int n, float scale, const bf16 *__restrict__ qkv,
                                                           const float *__restrict__ lse,
                                                           const float *__restrict__ Dvec,
                                                           const bf16 *__restrict__ da, bf16 *__restrict__ dqkv) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  using T = Tile<D>;
  constexpr int KK = D / 32, DB = D / 16, STAGE = 2 * T::BYTES + 512;   // Q tile, dO tile, lse[64], D[64]
  const int j = blockIdx.y, bi = blockIdx.z;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, g = lane >> 4, lr = lane & 15;
  const int64_t ld = (int64_t)n * 3 * D, pld = (int64_t)n * D;
  const bf16 *base = qkv + (int64_t)bi * s * ld + (int64_t)j * 3 * D;
  const bf16 *dab = da + (int64_t)bi * s * pld + (int64_t)j * D;
  const RowBlocks<G> rb(s, blockIdx.x, wave);
  // a wave without keys gets a first key beyond any sequence: every tile test below then skips it,
  // and no register is spent on a flag (this kernel has none to spare at head size 160)
  const int kw = rb.idle ? (1 << 30) : rb.row0;
  const float c = scale * kLog2e;
  const typename T::Lane ln(lane);
  const uint32_t smem_addr = lds_address(smem);

  int key[G];
  bf16x8 kf[G][KK], vf[G][KK];
#pragma unroll
  for (int kg = 0; kg < G; ++kg) {
    key[kg] = kw + 16 * kg + lr;
    const int keyc = key[kg] < s ? key[kg] : s - 1;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      kf[kg][kk] = *reinterpret_cast<const bf16x8 *>(base + (int64_t)keyc * ld + D + 32 * kk + 8 * g);
      vf[kg][kk] = *reinterpret_cast<const bf16x8 *>(base + (int64_t)keyc * ld + 2 * D + 32 * kk + 8 * g);
    }
  }
  f32x4 dk[G][DB], dv[G][DB];
#pragma unroll
  for (int kg = 0; kg < G; ++kg)
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int e = 0; e < 4; ++e) dk[kg][db][e] = dv[kg][db][e] = 0.0f;

  const int t_first = rb.first_tile, ntiles = (s + 63) / 64 - t_first;
  // tile DMAs as in the forward kernel (Q tile and dO tile), plus one instruction per wave for the
  // tile's lse values (even waves) or D values (odd waves); those arrive two or four times over, so
  // that every wave issues the same number of memory operations, which the counted waits rely on
  constexpr int IPW = G * T::NI;
  const int quarter = G == 2 ? wave : (wave & 3), half = G == 2 ? 0 : (wave >> 2);
  const dma_rsrc_t rq = dma_rsrc(half ? dab : base), ro = dma_rsrc(dab);
  const uint32_t pitch_q = (uint32_t)((half ? pld : ld) * 2);
  const dma_rsrc_t rstat = dma_rsrc(((wave & 1) ? Dvec : lse) + ((int64_t)bi * n + j) * s);
  auto issue_one = [&](auto tag, int t, int st, int i) {   // i == IPW: the statistics
    constexpr int TAG = decltype(tag)::value;
    const int tt = t < ntiles ? t : ntiles - 1;
    const int row0 = (t_first + tt) * 64;
    const uint32_t stage = smem_addr + st * STAGE;
    if (i == IPW) {
      int qq = row0 + lane;
      qq = qq < s ? qq : s - 1;
      dma4<TAG>(rstat, stage + 2 * T::BYTES + (wave & 1) * 256, qq * 4);
    } else if (G == 1 || i < T::NI) {
      T::template dma_one<TAG>(rq, row0, s, pitch_q, stage + half * T::BYTES, quarter, lane, i);
    } else {
      T::template dma_one<TAG>(ro, row0, s, (uint32_t)(pld * 2), stage + T::BYTES, quarter, lane, i - T::NI);
    }
  };
  auto issue = [&](int t, int st) {
#pragma unroll
    for (int i = 0; i <= IPW; ++i) issue_one(Burst{}, t, st, i);
  };
  issue(0, 0);
  issue(1, 1);
#pragma unroll
  for (int kg = 0; kg < G; ++kg)
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      arrive(kf[kg][kk]);
      arrive(vf[kg][kk]);
    }
  int cur = 0;
  for (int it = 0; it < ntiles; ++it) {
    wait_and_barrier<IPW + 1>();
    const int nn = cur == 0 ? 2 : cur - 1;
    const char *Qt = smem + cur * STAGE, *Ot = Qt + T::BYTES;
    const float *stat = reinterpret_cast<const float *>(Qt + 2 * T::BYTES);
    const int q0 = (t_first + it) * 64;
    if (q0 + 63 < kw) {  // wave-uniform: no query of the tile sees a key of this wave
      issue(it + 2, nn);
    } else {
      f32x4 sc[G][4], pc[G][4];
#pragma unroll
      for (int kg = 0; kg < G; ++kg)
#pragma unroll
        for (int qb = 0; qb < 4; ++qb)
#pragma unroll
          for (int e = 0; e < 4; ++e) sc[kg][qb][e] = pc[kg][qb][e] = 0.0f;
      {  // step i: k-step i / 2, query blocks 2 (i % 2) and + 1
        bf16x8 qfr[3][2], ofr[3][2];
        pipelined<2 * KK, 2>(
            [&](int i) {
#pragma unroll
              for (int h = 0; h < 2; ++h) {
                qfr[i % 3][h] = T::nat(Qt, ln, 2 * (i & 1) + h, i >> 1);
                ofr[i % 3][h] = T::nat(Ot, ln, 2 * (i & 1) + h, i >> 1);
              }
            },
            [&](int i) {
#pragma unroll
              for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int kg = 0; kg < G; ++kg) {
                  sc[kg][2 * (i & 1) + h] = MFMA16(qfr[i % 3][h], kf[kg][i >> 1], sc[kg][2 * (i & 1) + h]);
                  pc[kg][2 * (i & 1) + h] = MFMA16(ofr[i % 3][h], vf[kg][i >> 1], pc[kg][2 * (i & 1) + h]);
                }
            },
            [&](int i) {
              if (i < IPW) issue_one(Spread{}, it + 2, nn, i);
              if (i == 2 * KK - 1) issue_one(Spread{}, it + 2, nn, IPW);
            });
      }
      // element (kg, qb, e): query q0 + 16 qb + 4 g + e, key key[kg]
      const bool edge = q0 < kw + 16 * G || q0 + 63 >= s;  // wave-uniform: diagonal or past-the-end queries
#pragma unroll
      for (int qb = 0; qb < 4; ++qb) {
        const f32x4 ls = *reinterpret_cast<const f32x4 *>(stat + 16 * qb + 4 * g);
        const f32x4 dd = *reinterpret_cast<const f32x4 *>(stat + 64 + 16 * qb + 4 * g);
#pragma unroll
        for (int kg = 0; kg < G; ++kg)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int qq = q0 + 16 * qb + 4 * g + e;
            float p = fast_exp2(fmaf(sc[kg][qb][e], c, -ls[e] * kLog2e));
            if (edge && (qq < key[kg] || qq >= s)) p = 0.0f;
            sc[kg][qb][e] = p;
            pc[kg][qb][e] = p * (pc[kg][qb][e] - dd[e]);
          }
      }
      {  // step i: query half i / DB, output block i % DB
        bf16x8 pf[2][G], df[2][G], otr[4], qtr[4];
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
          for (int kg = 0; kg < G; ++kg) {
            pf[ks][kg] = pack2(sc[kg][2 * ks], sc[kg][2 * ks + 1]);
            df[ks][kg] = pack2(pc[kg][2 * ks], pc[kg][2 * ks + 1]);
          }
        pipelined<2 * DB, 3>(
            [&](int i) {
              otr[i & 3] = T::tr(Ot, ln, i % DB, i / DB);
              qtr[i & 3] = T::tr(Qt, ln, i % DB, i / DB);
            },
            [&](int i) {
#pragma unroll
              for (int kg = 0; kg < G; ++kg) {
                dv[kg][i % DB] = MFMA16(otr[i & 3], pf[i / DB][kg], dv[kg][i % DB]);
                dk[kg][i % DB] = MFMA16(qtr[i & 3], df[i / DB][kg], dk[kg][i % DB]);
              }
            });
      }
    }
    cur = cur == 2 ? 0 : cur + 1;
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

#pragma unroll
  for (int kg = 0; kg < G; ++kg) {
    if (key[kg] < s) {
      bf16 *out = dqkv + ((int64_t)bi * s + key[kg]) * ld + (int64_t)j * 3 * D;
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        bf16x4 ok, ov;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          ok[e] = (bf16)(dk[kg][db][e] * scale);
          ov[e] = (bf16)dv[kg][db][e];
        }
        *reinterpret_cast<bf16x4 *>(out + D + db * 16 + 4 * g) = ok;
        *reinterpret_cast<bf16x4 *>(out + 2 * D + db * 16 + 4 * g) = ov;
      }
    }
  }
}

// Row groups of 16 per wave and waves per workgroup.  Four waves of 32 rows (every LDS fragment feeds two MFMAs, one
// wave per SIMD with 512 registers) measured slower than eight waves of 16 rows (twice the LDS reads, two waves per
// SIMD to overlap the softmax arithmetic with the MFMAs) at head size 160, sequence 2048: forward 69 against 54 us,
// dk/dv 119 against 86 us, dq 77 against 69 us.  Eight waves of 32 rows need 256 rows per workgroup: the forward
// kernel takes that shape when the problem has enough workgroups (see fwd_launch); the backward kernels do not fit
// the 256 registers a wave has at eight waves.
constexpr int DKV_G = 1;

// Forward with 32 rows per wave on eight waves (256 rows per workgroup): every K / V fragment read from LDS feeds two
// MFMAs, which halves the kernel's LDS traffic -- its bound: each of the eight waves reads the whole K and V tile, the
// V tile through half-rate transposing reads -- but halves the number of workgroups as well.  Taken when that still
// leaves at least one workgroup per compute unit (the MT-NLG slice at micro-batch 1 has 16 heads x 8 = 128: it stays
// with 16 rows per wave) and the head size is 128 or 160 (at 64 the variant measures 17 % slower).  Measured: 1.3B-shaped
// layer (4 x 16 heads x 128) 168 -> 123 us, slice at micro-batch 4 167 -> 129 us, whole layer (128 heads) 326 -> 250 us.
template <int D, int G>
int fwd_launch_g(int b, int s, int n, float scale, const void *qkv, void *a, float *lse, hipStream_t st) {
  constexpr int smem = 3 * 2 * 64 * D * 2;
  static unsigned long long attr_done = 0;
  int device;
  if (!attr_is_set(attr_done, &device)) {
    if (hipFuncSetAttribute((const void *)attn_fwd_kernel<D, G, 8>, hipFuncAttributeMaxDynamicSharedMemorySize, smem) !=
        hipSuccess)
      return MTNLG_HIP_ERROR;
    attr_mark_set(attr_done, device);
  }
  LaunchScope scope(MTNLG_K_ATTN_FWD, st);
  attn_fwd_kernel<D, G, 8><<<dim3(RowBlocks<G, 8>::grid(s), n, b), 512, smem, st>>>(s, n, scale, (const bf16 *)qkv, (bf16 *)a, lse);
  return check_launch();
}

template <int D>
int fwd_launch(int b, int s, int n, float scale, const void *qkv, void *a, float *lse, hipStream_t st) {
  if (D >= 128 && (int64_t)RowBlocks<2, 8>::grid(s) * n * b >= 256) return fwd_launch_g<D, 2>(b, s, n, scale, qkv, a, lse, st);
  return fwd_launch_g<D, 1>(b, s, n, scale, qkv, a, lse, st);
}

template <int D, int G>
int bwd_dq_launch_g(int b, int s, int n, float scale, const void *qkv, const void *a, const float *lse, const void *da,
                    void *dqkv, float *Dvec, hipStream_t st) {
  constexpr int smem_dq = 3 * 2 * 64 * D * 2;
  static unsigned long long attr_done = 0;
  int device;
  if (!attr_is_set(attr_done, &device)) {
    if (hipFuncSetAttribute((const void *)attn_bwd_dq_kernel<D, G, 8>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            smem_dq) != hipSuccess)
      return MTNLG_HIP_ERROR;
    attr_mark_set(attr_done, device);
  }
  attn_bwd_dq_kernel<D, G, 8><<<dim3(RowBlocks<G, 8>::grid(s), n, b), 512, smem_dq, st>>>(
      s, n, scale, (const bf16 *)qkv, (const bf16 *)a, lse, (const bf16 *)da, (bf16 *)dqkv, Dvec);
  return check_launch();
}

template <int D>
int bwd_launch(int b, int s, int n, float scale, const void *qkv, const void *a, const float *lse, const void *da,
               void *dqkv, void *ws, hipStream_t st) {
  constexpr int smem_dkv = 3 * (2 * 64 * D * 2 + 512);
  static unsigned long long attr_done = 0;
  int device;
  if (!attr_is_set(attr_done, &device)) {
    if (hipFuncSetAttribute((const void *)attn_bwd_dkv_kernel<D, DKV_G>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            smem_dkv) != hipSuccess)
      return MTNLG_HIP_ERROR;
    attr_mark_set(attr_done, device);
  }
  float *Dvec = (float *)ws;
  LaunchScope scope(MTNLG_K_ATTN_BWD, st);
  // 16 rows per wave in both backward kernels: with 32 the dq kernel spills at head size 128 (256 registers and 256
  // bytes of scratch) and the dk/dv kernel does not fit at any
  MTNLG_TRY((bwd_dq_launch_g<D, 1>(b, s, n, scale, qkv, a, lse, da, dqkv, Dvec, st)));
  attn_bwd_dkv_kernel<D, DKV_G><<<dim3(RowBlocks<DKV_G>::grid(s), n, b), 512 / DKV_G, smem_dkv, st>>>(
      s, n, scale, (const bf16 *)qkv, lse, Dvec, (const bf16 *)da, (bf16 *)dqkv);
  return check_launch();
}

// The DMA addresses a sequence's rows with 32-bit byte offsets from its first row.
bool fits(int s, int n, int d) { return (int64_t)s * n * 3 * d * 2 < ((int64_t)1 << 31); }

}  // namespace

bool attention_mfma_supported(int dtype, int d) { return dtype == MTNLG_BF16 && (d == 64 || d == 128 || d == 160); }

bool attention_mfma_takes(int dtype, int b, int s, int n, int d) {
  return attention_mfma_supported(dtype, d) && n <= 65535 && b <= 65535 && fits(s, n, d);
}

size_t attention_bwd_workspace_bytes(int b, int s, int n, int) { return (size_t)b * n * s * sizeof(float); }

int attention_fwd_mfma(int b, int s, int n, int d, float scale, const void *qkv, void *a, float *lse,
                       hipStream_t stream) {
  if (n > 65535 || b > 65535 || !fits(s, n, d)) return MTNLG_UNSUPPORTED_SHAPE;
  switch (d) {
    case 64: return fwd_launch<64>(b, s, n, scale, qkv, a, lse, stream);
    case 128: return fwd_launch<128>(b, s, n, scale, qkv, a, lse, stream);
    case 160: return fwd_launch<160>(b, s, n, scale, qkv, a, lse, stream);
    default: return MTNLG_UNSUPPORTED_SHAPE;
  }
}

int attention_bwd_mfma(int b, int s, int n, int d, float scale, const void *qkv, const void *a, const float *lse,
                       const void *da, void *dqkv, void *ws, hipStream_t stream) {
  if (n > 65535 || b > 65535 || !fits(s, n, d)) return MTNLG_UNSUPPORTED_SHAPE;
  switch (d) {
    case 64: return bwd_launch<64>(b, s, n, scale, qkv, a, lse, da, dqkv, ws, stream);
    case 128: return bwd_launch<128>(b, s, n, scale, qkv, a, lse, da, dqkv, ws, stream);
    case 160: return bwd_launch<160>(b, s, n, scale, qkv, a, lse, da, dqkv, ws, stream);
    default: return MTNLG_UNSUPPORTED_SHAPE;
  }
}

}  // namespace mtnlg
