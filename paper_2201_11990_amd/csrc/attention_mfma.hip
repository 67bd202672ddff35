// Fused causal softmax attention on the gfx950 matrix cores (bf16 in, fp32 softmax
// and accumulation), forward and backward, for head sizes 64, 128 and 160.
//
//   S = scale * q k^T (causal),  P = rowsoftmax(S),  a = P v,  lse = log sum exp(S)
//   backward with D_t = da_t . a_t :  dP = da v^T,  dS = P o (dP - D),
//   dq = scale dS k,  dk = scale dS^T q,  dv = P^T da.
//
// All three kernels keep "their" rows in registers as MFMA B operands and stream
// the other side through LDS in 64-row tiles:
//   forward  : workgroup = 128 queries (32 per wave); K and V tiles streamed.
//              S^T = K Q^T puts one query per lane (column of the 32x32 MFMA block)
//              and keys along the accumulator registers, so the softmax statistics
//              are lane-local and P^T is already in B-operand form for
//              O^T += V^T P^T.  V is transposed on its way into LDS.
//   dq       : same geometry; dQ^T += K^T dS^T with K also kept transposed in LDS.
//              Also emits D_t for the dk/dv kernel.
//   dk / dv  : workgroup = 128 keys (32 per wave); Q and dO tiles streamed, both in
//              natural and transposed form;  dV^T += dO^T P,  dK^T += Q^T dS.
// No atomics: every output element has one owner, results are run-to-run identical.
//
// Transposed tiles are [D][64] with the 64 "k" positions of a row permuted (bits 2
// and 3 of the index swapped inside each group of 16) so that the 8 values a lane
// needs for one MFMA step -- the ones matching accumulator registers 8t..8t+7 of
// the producing block -- are one 16-byte LDS read.
#include <math.h>

#include "common.h"

namespace mtnlg {

namespace {

typedef __attribute__((ext_vector_type(8))) short i16x8;
typedef __attribute__((ext_vector_type(4))) short i16x4;

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// chunk position inside a natural [rows][D] tile (row = 2*D bytes)
template <int D>
__device__ __forceinline__ int nat_off(int r, int c) {
  if constexpr ((2 * D) % 128 == 0)
    return r * (2 * D) + ((c ^ (r & 7)) << 4);
  else  // 2*D = 64 mod 128 (D = 160): rows alternate between two bank halves
    return r * (2 * D) + ((c ^ ((r >> 1) & 3)) << 4);
}
// chunk position inside a transposed [D][64] tile (row = 128 bytes)
__device__ __forceinline__ int tr_off(int r, int c) { return r * 128 + ((c ^ (r & 7) ^ ((r >> 3) & 7)) << 4); }

// One 8(rows) x 8(cols) block of a 64-row x D-column bf16 tile per thread.
template <int D>
struct Block64 {
  static constexpr int DB = D / 8;       // column blocks
  static constexpr int NB = 8 * DB;      // blocks in the tile
  static_assert(NB <= 256, "one block per thread");
  i16x8 r[8];
  // rows row0.. of a matrix with leading dimension ld; rows >= rows_total are clamped
  __device__ __forceinline__ void fetch(const bf16 *base, int64_t ld, int row0, int rows_total) {
    if (threadIdx.x < NB) {
      const int rb = threadIdx.x / DB, db = threadIdx.x % DB;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        int row = row0 + rb * 8 + i;
        row = row < rows_total ? row : rows_total - 1;
        r[i] = *reinterpret_cast<const i16x8 *>(base + (int64_t)row * ld + db * 8);
      }
    }
  }
  __device__ __forceinline__ void stash_natural(char *lds) const {
    if (threadIdx.x < NB) {
      const int rb = threadIdx.x / DB, db = threadIdx.x % DB;
#pragma unroll
      for (int i = 0; i < 8; ++i) *reinterpret_cast<i16x8 *>(lds + nat_off<D>(rb * 8 + i, db)) = r[i];
    }
  }
  __device__ __forceinline__ void stash_transposed(char *lds) const {
    if (threadIdx.x < NB) {
      const int rb = threadIdx.x / DB, db = threadIdx.x % DB;
      const int c0 = 2 * (rb >> 1), half = (rb & 1) * 8;  // 16-group rb/2, element offset 4*(rb&1)
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int row = db * 8 + e;
        i16x4 lo, hi;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          lo[j] = r[j][e];
          hi[j] = r[4 + j][e];
        }
        *reinterpret_cast<i16x4 *>(lds + tr_off(row, c0) + half) = lo;
        *reinterpret_cast<i16x4 *>(lds + tr_off(row, c0 + 1) + half) = hi;
      }
    }
  }
};

template <int D>
__device__ __forceinline__ bf16x8 frag_nat(const char *lds, int row, int c) {
  return *reinterpret_cast<const bf16x8 *>(lds + nat_off<D>(row, c));
}
__device__ __forceinline__ bf16x8 frag_tr(const char *lds, int row, int c) {
  return *reinterpret_cast<const bf16x8 *>(lds + tr_off(row, c));
}
// accumulator registers 8t..8t+7 of a 32x32 block as a bf16 B operand
__device__ __forceinline__ bf16x8 pack8(const f32x16 &v, int t) {
  bf16x8 o;
#pragma unroll
  for (int i = 0; i < 8; ++i) o[i] = (bf16)v[8 * t + i];
  return o;
}
// row index inside a 32x32 block of accumulator register e for lane group g
__device__ __forceinline__ int acc_row(int e, int g) { return 8 * (e >> 2) + 4 * g + (e & 3); }

// 2^x on the transcendental unit (v_exp_f32): no denormal fix-up, 2^-inf = 0.
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

#define MFMA(a, b, c) __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0)

// ------------------------------------------------------------------ forward
template <int D>
__global__ __launch_bounds__(256) void attn_fwd_kernel(int s, int n, float scale, const bf16 *__restrict__ qkv,
                                                       bf16 *__restrict__ a, float *__restrict__ lse) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  constexpr int KK = D / 16, DBK = D / 32, TILE = 64 * D * 2, STAGE = 2 * TILE;
  const int qt = gridDim.x - 1 - blockIdx.x, j = blockIdx.y, bi = blockIdx.z;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, g = lane >> 5;
  const int64_t ld = (int64_t)n * 3 * D;
  const bf16 *base = qkv + (int64_t)bi * s * ld + (int64_t)j * 3 * D;
  const int q0 = qt * 128, qw = q0 + wave * 32;
  const int q = qw + (lane & 31), qc = q < s ? q : s - 1;
  const float c = scale * kLog2e;

  bf16x8 qf[KK];
#pragma unroll
  for (int kk = 0; kk < KK; ++kk)
    qf[kk] = *reinterpret_cast<const bf16x8 *>(base + (int64_t)qc * ld + (2 * kk + g) * 8);

  f32x16 oacc[DBK];
#pragma unroll
  for (int db = 0; db < DBK; ++db)
#pragma unroll
    for (int e = 0; e < 16; ++e) oacc[db][e] = 0.0f;
  float m = -INFINITY, l = 0.0f;

  int last = q0 + 127 < s - 1 ? q0 + 127 : s - 1;
  const int ntiles = last / 64 + 1;
  Block64<D> kb, vb;
  kb.fetch(base + D, ld, 0, s);
  vb.fetch(base + 2 * D, ld, 0, s);
  kb.stash_natural(smem);
  vb.stash_transposed(smem + TILE);
  __syncthreads();

  for (int it = 0; it < ntiles; ++it) {
    const char *Kt = smem + (it & 1) * STAGE, *Vt = Kt + TILE;
    char *nxt = smem + ((it + 1) & 1) * STAGE;
    const bool more = it + 1 < ntiles;
    const int kv0 = it * 64;
    if (more) {
      kb.fetch(base + D, ld, kv0 + 64, s);
      vb.fetch(base + 2 * D, ld, kv0 + 64, s);
    }
    if (kv0 <= qw + 31) {  // wave-uniform: some (query, key) pair of this wave is unmasked
      f32x16 sacc[2];
#pragma unroll
      for (int blk = 0; blk < 2; ++blk)
#pragma unroll
        for (int e = 0; e < 16; ++e) sacc[blk][e] = 0.0f;
#pragma unroll
      for (int kk = 0; kk < KK; ++kk)
#pragma unroll
        for (int blk = 0; blk < 2; ++blk)
          sacc[blk] = MFMA(frag_nat<D>(Kt, blk * 32 + (lane & 31), 2 * kk + g), qf[kk], sacc[blk]);
      // m tracks the running maximum of the raw scores; exponents are taken in base 2
      // with the scale folded in: p = 2^(s*c - m*c).
      if (kv0 + 63 > qw) {  // wave-uniform: this tile crosses the diagonal for some row
#pragma unroll
        for (int blk = 0; blk < 2; ++blk)
#pragma unroll
          for (int e = 0; e < 16; ++e)
            if (kv0 + blk * 32 + acc_row(e, g) > qc) sacc[blk][e] = -INFINITY;
      }
      float mx = -INFINITY;
#pragma unroll
      for (int blk = 0; blk < 2; ++blk)
#pragma unroll
        for (int e = 0; e < 16; ++e) mx = fmaxf(mx, sacc[blk][e]);
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float m_new = fmaxf(m, mx);  // finite from the first tile on (key 0 is never masked)
      const float mc = m_new * c;
      float rs = 0.0f;
#pragma unroll
      for (int blk = 0; blk < 2; ++blk)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const float p = fast_exp2(fmaf(sacc[blk][e], c, -mc));
          sacc[blk][e] = p;
          rs += p;
        }
      rs += __shfl_xor(rs, 32, 64);
      const float alpha = fast_exp2((m - m_new) * c);
      l = l * alpha + rs;
      if (__builtin_amdgcn_ballot_w64(m_new > m) != 0) {  // some row's maximum moved: rescale O
#pragma unroll
        for (int db = 0; db < DBK; ++db)
#pragma unroll
          for (int e = 0; e < 16; ++e) oacc[db][e] *= alpha;
      }
      m = m_new;
#pragma unroll
      for (int blk = 0; blk < 2; ++blk)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          const bf16x8 pf = pack8(sacc[blk], t);
#pragma unroll
          for (int db = 0; db < DBK; ++db)
            oacc[db] = MFMA(frag_tr(Vt, db * 32 + (lane & 31), 2 * (2 * blk + t) + g), pf, oacc[db]);
        }
    }
    if (more) {
      kb.stash_natural(nxt);
      vb.stash_transposed(nxt + TILE);
    }
    __syncthreads();
  }

  if (q < s) {
    const float inv = 1.0f / l;
    bf16 *out = a + ((int64_t)bi * s + q) * ((int64_t)n * D) + (int64_t)j * D;
#pragma unroll
    for (int db = 0; db < DBK; ++db)
#pragma unroll
      for (int e4 = 0; e4 < 4; ++e4) {
        bf16x4 o;
#pragma unroll
        for (int i = 0; i < 4; ++i) o[i] = (bf16)(oacc[db][4 * e4 + i] * inv);
        *reinterpret_cast<bf16x4 *>(out + db * 32 + 8 * e4 + 4 * g) = o;
      }
    if (g == 0) lse[((int64_t)bi * n + j) * s + q] = (m * c + log2f(l)) * kLn2;
  }
}

// ------------------------------------------------------------------ backward: dq (and D)
template <int D>
__global__ __launch_bounds__(256) void attn_bwd_dq_kernel(int s, int n, float scale, const bf16 *__restrict__ qkv,
                                                          const bf16 *__restrict__ a, const float *__restrict__ lse,
                                                          const bf16 *__restrict__ da, bf16 *__restrict__ dqkv,
                                                          float *__restrict__ Dvec) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  constexpr int KK = D / 16, DBK = D / 32, TILE = 64 * D * 2;
  const int qt = gridDim.x - 1 - blockIdx.x, j = blockIdx.y, bi = blockIdx.z;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, g = lane >> 5;
  const int64_t ld = (int64_t)n * 3 * D, pld = (int64_t)n * D;
  const bf16 *base = qkv + (int64_t)bi * s * ld + (int64_t)j * 3 * D;
  const int q0 = qt * 128, qw = q0 + wave * 32;
  const int q = qw + (lane & 31), qc = q < s ? q : s - 1;
  const float c = scale * kLog2e;

  bf16x8 qf[KK], dof[KK];
  float dsum = 0.0f;
  {
    const bf16 *dar = da + ((int64_t)bi * s + qc) * pld + (int64_t)j * D;
    const bf16 *ar = a + ((int64_t)bi * s + qc) * pld + (int64_t)j * D;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      qf[kk] = *reinterpret_cast<const bf16x8 *>(base + (int64_t)qc * ld + (2 * kk + g) * 8);
      dof[kk] = *reinterpret_cast<const bf16x8 *>(dar + (2 * kk + g) * 8);
      const bf16x8 av = *reinterpret_cast<const bf16x8 *>(ar + (2 * kk + g) * 8);
#pragma unroll
      for (int i = 0; i < 8; ++i) dsum += (float)dof[kk][i] * (float)av[i];
    }
  }
  dsum += __shfl_xor(dsum, 32, 64);
  const float lse2 = lse[((int64_t)bi * n + j) * s + qc] * kLog2e;
  if (q < s && g == 0) Dvec[((int64_t)bi * n + j) * s + q] = dsum;

  f32x16 dq[DBK];
#pragma unroll
  for (int db = 0; db < DBK; ++db)
#pragma unroll
    for (int e = 0; e < 16; ++e) dq[db][e] = 0.0f;

  int last = q0 + 127 < s - 1 ? q0 + 127 : s - 1;
  const int ntiles = last / 64 + 1;
  char *Kn = smem, *Vn = smem + TILE, *Kt = smem + 2 * TILE;
  Block64<D> kb, vb;
  kb.fetch(base + D, ld, 0, s);
  vb.fetch(base + 2 * D, ld, 0, s);

  for (int it = 0; it < ntiles; ++it) {
    const int kv0 = it * 64;
    __syncthreads();  // previous tile fully consumed
    kb.stash_natural(Kn);
    kb.stash_transposed(Kt);
    vb.stash_natural(Vn);
    __syncthreads();
    if (it + 1 < ntiles) {
      kb.fetch(base + D, ld, kv0 + 64, s);
      vb.fetch(base + 2 * D, ld, kv0 + 64, s);
    }
    if (kv0 <= qw + 31) {
      f32x16 sacc[2], pacc[2];
#pragma unroll
      for (int blk = 0; blk < 2; ++blk)
#pragma unroll
        for (int e = 0; e < 16; ++e) sacc[blk][e] = pacc[blk][e] = 0.0f;
#pragma unroll
      for (int kk = 0; kk < KK; ++kk)
#pragma unroll
        for (int blk = 0; blk < 2; ++blk) {
          sacc[blk] = MFMA(frag_nat<D>(Kn, blk * 32 + (lane & 31), 2 * kk + g), qf[kk], sacc[blk]);
          pacc[blk] = MFMA(frag_nat<D>(Vn, blk * 32 + (lane & 31), 2 * kk + g), dof[kk], pacc[blk]);
        }
      // dS^T = P^T o (dP^T - D)
      if (kv0 + 63 > qw) {  // wave-uniform: diagonal (or past-the-end keys) in this tile
#pragma unroll
        for (int blk = 0; blk < 2; ++blk)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int kv = kv0 + blk * 32 + acc_row(e, g);
            const float p = kv > qc ? 0.0f : fast_exp2(fmaf(sacc[blk][e], c, -lse2));
            sacc[blk][e] = p * (pacc[blk][e] - dsum);
          }
      } else {
#pragma unroll
        for (int blk = 0; blk < 2; ++blk)
#pragma unroll
          for (int e = 0; e < 16; ++e)
            sacc[blk][e] = fast_exp2(fmaf(sacc[blk][e], c, -lse2)) * (pacc[blk][e] - dsum);
      }
#pragma unroll
      for (int blk = 0; blk < 2; ++blk)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          const bf16x8 df = pack8(sacc[blk], t);
#pragma unroll
          for (int db = 0; db < DBK; ++db)
            dq[db] = MFMA(frag_tr(Kt, db * 32 + (lane & 31), 2 * (2 * blk + t) + g), df, dq[db]);
        }
    }
  }
  if (q < s) {
    bf16 *out = dqkv + ((int64_t)bi * s + q) * ld + (int64_t)j * 3 * D;
#pragma unroll
    for (int db = 0; db < DBK; ++db)
#pragma unroll
      for (int e4 = 0; e4 < 4; ++e4) {
        bf16x4 o;
#pragma unroll
        for (int i = 0; i < 4; ++i) o[i] = (bf16)(dq[db][4 * e4 + i] * scale);
        *reinterpret_cast<bf16x4 *>(out + db * 32 + 8 * e4 + 4 * g) = o;
      }
  }
}

// ------------------------------------------------------------------ backward: dk, dv
template <int D>
__global__ __launch_bounds__(256) void attn_bwd_dkv_kernel(int s, int n, float scale, const bf16 *__restrict__ qkv,
                                                           const float *__restrict__ lse,
                                                           const float *__restrict__ Dvec,
                                                           const bf16 *__restrict__ da, bf16 *__restrict__ dqkv) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  constexpr int KK = D / 16, DBK = D / 32, TILE = 64 * D * 2;
  const int kt = blockIdx.x, j = blockIdx.y, bi = blockIdx.z;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, g = lane >> 5;
  const int64_t ld = (int64_t)n * 3 * D, pld = (int64_t)n * D;
  const bf16 *base = qkv + (int64_t)bi * s * ld + (int64_t)j * 3 * D;
  const bf16 *dab = da + (int64_t)bi * s * pld + (int64_t)j * D;
  const int k0 = kt * 128, kw = k0 + wave * 32;
  const int key = kw + (lane & 31), keyc = key < s ? key : s - 1;
  const float c = scale * kLog2e;

  bf16x8 kf[KK], vf[KK];
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) {
    kf[kk] = *reinterpret_cast<const bf16x8 *>(base + (int64_t)keyc * ld + D + (2 * kk + g) * 8);
    vf[kk] = *reinterpret_cast<const bf16x8 *>(base + (int64_t)keyc * ld + 2 * D + (2 * kk + g) * 8);
  }
  f32x16 dk[DBK], dv[DBK];
#pragma unroll
  for (int db = 0; db < DBK; ++db)
#pragma unroll
    for (int e = 0; e < 16; ++e) dk[db][e] = dv[db][e] = 0.0f;

  char *Qn = smem, *On = smem + TILE, *Qt = smem + 2 * TILE, *Ot = smem + 3 * TILE;
  float *stat = reinterpret_cast<float *>(smem + 4 * TILE);  // [0..63] lse*log2e, [64..127] D
  const float *lrow = lse + ((int64_t)bi * n + j) * s, *drow = Dvec + ((int64_t)bi * n + j) * s;

  const int t_first = k0 / 64, t_end = (s + 63) / 64;
  Block64<D> qb, ob;
  qb.fetch(base, ld, t_first * 64, s);
  ob.fetch(dab, pld, t_first * 64, s);

  for (int it = t_first; it < t_end; ++it) {
    const int q0 = it * 64;
    __syncthreads();
    qb.stash_natural(Qn);
    qb.stash_transposed(Qt);
    ob.stash_natural(On);
    ob.stash_transposed(Ot);
    if (threadIdx.x < 64) {
      int qq = q0 + threadIdx.x;
      qq = qq < s ? qq : s - 1;
      stat[threadIdx.x] = lrow[qq] * kLog2e;
      stat[64 + threadIdx.x] = drow[qq];
    }
    __syncthreads();
    if (it + 1 < t_end) {
      qb.fetch(base, ld, q0 + 64, s);
      ob.fetch(dab, pld, q0 + 64, s);
    }
    if (q0 + 63 >= kw) {  // wave-uniform: some query of the tile sees a key of this wave
      f32x16 sacc[2], pacc[2];
#pragma unroll
      for (int qb2 = 0; qb2 < 2; ++qb2)
#pragma unroll
        for (int e = 0; e < 16; ++e) sacc[qb2][e] = pacc[qb2][e] = 0.0f;
#pragma unroll
      for (int kk = 0; kk < KK; ++kk)
#pragma unroll
        for (int qb2 = 0; qb2 < 2; ++qb2) {
          sacc[qb2] = MFMA(frag_nat<D>(Qn, qb2 * 32 + (lane & 31), 2 * kk + g), kf[kk], sacc[qb2]);
          pacc[qb2] = MFMA(frag_nat<D>(On, qb2 * 32 + (lane & 31), 2 * kk + g), vf[kk], pacc[qb2]);
        }
      // element (register e, lane) is query q0 + 32*qb2 + acc_row(e,g), key = this lane's key
      if (q0 < kw + 32 || q0 + 63 >= s) {  // wave-uniform: diagonal or past-the-end queries
#pragma unroll
        for (int qb2 = 0; qb2 < 2; ++qb2)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int ql = qb2 * 32 + acc_row(e, g);
            const int qq = q0 + ql;
            const float p = (qq < key || qq >= s) ? 0.0f : fast_exp2(fmaf(sacc[qb2][e], c, -stat[ql]));
            sacc[qb2][e] = p;
            pacc[qb2][e] = p * (pacc[qb2][e] - stat[64 + ql]);
          }
      } else {
#pragma unroll
        for (int qb2 = 0; qb2 < 2; ++qb2)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int ql = qb2 * 32 + acc_row(e, g);
            const float p = fast_exp2(fmaf(sacc[qb2][e], c, -stat[ql]));
            sacc[qb2][e] = p;
            pacc[qb2][e] = p * (pacc[qb2][e] - stat[64 + ql]);
          }
      }
#pragma unroll
      for (int qb2 = 0; qb2 < 2; ++qb2)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          const bf16x8 pf = pack8(sacc[qb2], t), df = pack8(pacc[qb2], t);
#pragma unroll
          for (int db = 0; db < DBK; ++db) {
            dv[db] = MFMA(frag_tr(Ot, db * 32 + (lane & 31), 2 * (2 * qb2 + t) + g), pf, dv[db]);
            dk[db] = MFMA(frag_tr(Qt, db * 32 + (lane & 31), 2 * (2 * qb2 + t) + g), df, dk[db]);
          }
        }
    }
  }
  if (key < s) {
    bf16 *out = dqkv + ((int64_t)bi * s + key) * ld + (int64_t)j * 3 * D;
#pragma unroll
    for (int db = 0; db < DBK; ++db)
#pragma unroll
      for (int e4 = 0; e4 < 4; ++e4) {
        bf16x4 ok, ov;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          ok[i] = (bf16)(dk[db][4 * e4 + i] * scale);
          ov[i] = (bf16)dv[db][4 * e4 + i];
        }
        *reinterpret_cast<bf16x4 *>(out + D + db * 32 + 8 * e4 + 4 * g) = ok;
        *reinterpret_cast<bf16x4 *>(out + 2 * D + db * 32 + 8 * e4 + 4 * g) = ov;
      }
  }
}

template <int D>
int fwd_launch(int b, int s, int n, float scale, const void *qkv, void *a, float *lse, hipStream_t st) {
  constexpr int smem = 2 * 2 * 64 * D * 2;
  static bool attr = false;
  if (!attr) {
    if (hipFuncSetAttribute((const void *)attn_fwd_kernel<D>, hipFuncAttributeMaxDynamicSharedMemorySize, smem) !=
        hipSuccess)
      return MTNLG_HIP_ERROR;
    attr = true;
  }
  LaunchScope scope(MTNLG_K_ATTN_FWD, st);
  attn_fwd_kernel<D><<<dim3((s + 127) / 128, n, b), 256, smem, st>>>(s, n, scale, (const bf16 *)qkv, (bf16 *)a, lse);
  return check_launch();
}

template <int D>
int bwd_launch(int b, int s, int n, float scale, const void *qkv, const void *a, const float *lse, const void *da,
               void *dqkv, void *ws, hipStream_t st) {
  constexpr int smem_dq = 3 * 64 * D * 2, smem_dkv = 4 * 64 * D * 2 + 128 * 4;
  static bool attr = false;
  if (!attr) {
    if (hipFuncSetAttribute((const void *)attn_bwd_dq_kernel<D>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            smem_dq) != hipSuccess ||
        hipFuncSetAttribute((const void *)attn_bwd_dkv_kernel<D>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            smem_dkv) != hipSuccess)
      return MTNLG_HIP_ERROR;
    attr = true;
  }
  float *Dvec = (float *)ws;
  LaunchScope scope(MTNLG_K_ATTN_BWD, st);
  attn_bwd_dq_kernel<D><<<dim3((s + 127) / 128, n, b), 256, smem_dq, st>>>(
      s, n, scale, (const bf16 *)qkv, (const bf16 *)a, lse, (const bf16 *)da, (bf16 *)dqkv, Dvec);
  MTNLG_TRY(check_launch());
  attn_bwd_dkv_kernel<D><<<dim3((s + 127) / 128, n, b), 256, smem_dkv, st>>>(
      s, n, scale, (const bf16 *)qkv, lse, Dvec, (const bf16 *)da, (bf16 *)dqkv);
  return check_launch();
}

}  // namespace

bool attention_mfma_supported(int dtype, int d) { return dtype == MTNLG_BF16 && (d == 64 || d == 128 || d == 160); }

size_t attention_bwd_workspace_bytes(int b, int s, int n, int) { return (size_t)b * n * s * sizeof(float); }

int attention_fwd_mfma(int b, int s, int n, int d, float scale, const void *qkv, void *a, float *lse,
                       hipStream_t stream) {
  if (n > 65535 || b > 65535) return MTNLG_UNSUPPORTED_SHAPE;
  switch (d) {
    case 64: return fwd_launch<64>(b, s, n, scale, qkv, a, lse, stream);
    case 128: return fwd_launch<128>(b, s, n, scale, qkv, a, lse, stream);
    case 160: return fwd_launch<160>(b, s, n, scale, qkv, a, lse, stream);
    default: return MTNLG_UNSUPPORTED_SHAPE;
  }
}

int attention_bwd_mfma(int b, int s, int n, int d, float scale, const void *qkv, const void *a, const float *lse,
                       const void *da, void *dqkv, void *ws, hipStream_t stream) {
  if (n > 65535 || b > 65535) return MTNLG_UNSUPPORTED_SHAPE;
  switch (d) {
    case 64: return bwd_launch<64>(b, s, n, scale, qkv, a, lse, da, dqkv, ws, stream);
    case 128: return bwd_launch<128>(b, s, n, scale, qkv, a, lse, da, dqkv, ws, stream);
    case 160: return bwd_launch<160>(b, s, n, scale, qkv, a, lse, da, dqkv, ws, stream);
    default: return MTNLG_UNSUPPORTED_SHAPE;
  }
}

}  // namespace mtnlg
