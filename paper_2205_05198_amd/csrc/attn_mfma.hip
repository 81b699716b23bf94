// bf16 attention core with selective recomputation (Section 5) on gfx950 matrix cores.
//
// Everything is built from 32x32x16 bf16 MFMA tiles (v_mfma_f32_32x32x16_bf16).  Operand and result
// layout of one tile D[32x32] += A[32x16] B[16x32] on a 64-lane wavefront, lane = 32*hh + li:
//   A: lane holds row li, k = 8*hh .. 8*hh+7        B: lane holds column li, k = 8*hh .. 8*hh+7
//   D: lane holds column li, rows 8*g + 4*hh + r for acc[4*g + r], g, r in 0..3
// so a result tile keeps ONE column per lane.  Scores are therefore produced transposed,
// S^T[j][i] = K Q^T, which puts one query row i in each lane: row max / row sum / log-sum-exp / the
// Philox counter of a row are lane-local, and the same registers, rounded to bf16, are directly the B
// operand (k = j) of the second product O^T[c][i] = V^T P^T.  K rows are stored in LDS with bits 2 and 3
// of the row index swapped, which makes the 8 values a lane feeds to that second product 8 CONSECUTIVE
// keys j (= exactly one 8-element Philox call, and one 16-byte operand).  V^T operands are read from the
// row-major V tile with the LDS transpose load ds_read_b64_tr_b16.
//
// Workgroups have 4 waves on one block of 64 query rows (or 64 keys): two waves per 32-row group, which split
// the keys (or, in the column pass, the query tiles) between them and merge their partial results through LDS
// at the end.  One workgroup fills a CU (one wave per SIMD, accumulators in registers), and the grid lists the
// heaviest causal blocks first, so the dispatcher balances the triangular work over the CUs.
//
// Forward   : O, LSE from Q, K, V             (2 contractions per score tile)
// Backward 1: dQ and delta = rowsum(dO o O)    (row-stationary; S^T, dD^T recomputed, dQ = dS K)
// Backward 2: dK, dV                           (column-stationary; S^T, dD^T recomputed again,
//                                               dS / D moved to the transposed layout by an identity MFMA)
// No s x s tensor is ever written; the dropout mask is regenerated from (seed, offset) in all three.
#include "sar_device.h"
#include "sar_internal.h"

namespace sar {

static constexpr float kLog2e = 1.4426950408889634f;
static constexpr float kLn2 = 0.6931471805599453f;

typedef __attribute__((address_space(3))) short4_t lds_short4_t;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4_t;

#ifdef SAR_EXP_NOMFMA
__device__ __forceinline__ float16_t mfma32(bf16x8_t a, bf16x8_t b, float16_t c) { c[0] += (float)a[0] + (float)b[0]; return c; }
#else
__device__ __forceinline__ float16_t mfma32(bf16x8_t a, bf16x8_t b, float16_t c) { return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0); }
#endif
#ifdef SAR_EXP_NOEXP
#define SAR_EXP2(x) ((x) * 0.001f)
#else
#define SAR_EXP2(x) __builtin_amdgcn_exp2f(x)
#endif
#ifdef SAR_EXP_NOPHILOX
#define keep_bits8(G, site, k0, k1, T) ((uint32_t)(G) | 0xFFu)
#endif

// 16-byte operand from LDS / global (8 consecutive bf16)
__device__ __forceinline__ bf16x8_t ld_frag(const uint16_t* p) { return *reinterpret_cast<const bf16x8_t*>(p); }

// Transposed operand: from a row-major tile T[k][c] (pitch in elements) return, for this lane,
// T[k0 + 8*hh + e][c0 + li], e = 0..7, as one MFMA operand.
__device__ __forceinline__ bf16x8_t ld_frag_tr(const uint16_t* tile, int pitch, int k0, int c0, int lane) {
  const int lam = lane & 15, blk = lane >> 4;  // 16-lane block: li = 16*(blk&1) + lam, hh = blk >> 1
  const uint16_t* p = tile + (k0 + 8 * (blk >> 1) + (lam >> 2)) * pitch + c0 + 16 * (blk & 1) + 4 * (lam & 3);
  union { short4_t h[2]; bf16x8_t v; } u;
  u.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_t*)(p));
  u.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_t*)(p + 4 * pitch));
  return u.v;
}

__device__ __forceinline__ bf16x8_t pack8(const float* f) {
  union { uint32_t w[4]; bf16x8_t v; } u;
  u.w[0] = pack_bf16x2(f[0], f[1]);
  u.w[1] = pack_bf16x2(f[2], f[3]);
  u.w[2] = pack_bf16x2(f[4], f[5]);
  u.w[3] = pack_bf16x2(f[6], f[7]);
  return u.v;
}

// LDS row that holds row r (0..63) of a K tile: bits 2 and 3 swapped inside each group of 32 rows
__device__ __forceinline__ int perm_row(int r) { return (r & ~12) | ((r & 4) << 1) | ((r & 8) >> 1); }

// ---------------------------------------------------------------------------------------------------
// Tile staging: a tile is 64 rows x D bf16.  Each of the 256 threads moves ITER 16-byte chunks; the global
// loads land in registers (tile_fetch) long before they are written to LDS (tile_commit), so that they fly
// during the previous tile's math.
// ---------------------------------------------------------------------------------------------------
template <int D>
struct TileMap {
  static constexpr int ROWS = 64, NT = 256, CPR = D / 8, NCH = ROWS * CPR, ITER = NCH / NT;
  static_assert(NCH % NT == 0, "tile must split evenly over 256 threads");
  int goff[ITER];  // element offset of the chunk from the tile's first row in global memory
  int loff[ITER];  // element offset of the chunk inside the LDS tile
  __device__ __forceinline__ void init(int tid, int gstride, int pitch, bool perm) {
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
      const int c = tid + it * NT, r = c / CPR, cc = c - r * CPR;
      goff[it] = r * gstride + 8 * cc;
      loff[it] = (perm ? perm_row(r) : r) * pitch + 8 * cc;
    }
  }
};
template <int D>
struct TileBuf { u32x4_t r[TileMap<D>::ITER]; };

// gtile points at the tile's first row (uniform); rows_valid = rows of the tensor left from there (clamped reads)
template <int D>
__device__ __forceinline__ void tile_fetch(TileBuf<D>& buf, const TileMap<D>& map, const uint16_t* gtile, int gstride, int rows_valid, int tid) {
#ifdef SAR_EXP_NOFETCH
  if (rows_valid > -1000000) return;
#endif
  if (rows_valid >= TileMap<D>::ROWS) {
#pragma unroll
    for (int it = 0; it < TileMap<D>::ITER; ++it) buf.r[it] = *reinterpret_cast<const u32x4_t*>(gtile + map.goff[it]);
  } else {
#pragma unroll
    for (int it = 0; it < TileMap<D>::ITER; ++it) {
      const int c = tid + it * TileMap<D>::NT, r = c / TileMap<D>::CPR, cc = c - r * TileMap<D>::CPR;
      const int rr = r < rows_valid ? r : rows_valid - 1;
      buf.r[it] = *reinterpret_cast<const u32x4_t*>(gtile + rr * gstride + 8 * cc);
    }
  }
}
template <int D>
__device__ __forceinline__ void tile_commit(const TileBuf<D>& buf, const TileMap<D>& map, uint16_t* lds) {
#pragma unroll
  for (int it = 0; it < TileMap<D>::ITER; ++it) *reinterpret_cast<u32x4_t*>(lds + map.loff[it]) = buf.r[it];
}

// Same as ld_frag_tr but for the k order that the swapped rows and the identity-transposed tiles use:
// slot e of lane half hh <-> tile row k0 + 8*(e>>2) + 4*hh + (e&3).
__device__ __forceinline__ bf16x8_t ld_frag_tr_perm(const uint16_t* tile, int pitch, int k0, int c0, int lane) {
  const int lam = lane & 15, blk = lane >> 4;
  const uint16_t* p = tile + (k0 + 4 * (blk >> 1) + (lam >> 2)) * pitch + c0 + 16 * (blk & 1) + 4 * (lam & 3);
  union { short4_t h[2]; bf16x8_t v; } u;
  u.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_t*)(p));
  u.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_t*)(p + 8 * pitch));
  return u.v;
}

// dot product of two 8-element bf16 fragments in fp32
__device__ __forceinline__ float dot8(bf16x8_t a, bf16x8_t b) {
  union { bf16x8_t v; uint32_t w[4]; } ua, ub;
  ua.v = a;
  ub.v = b;
  float acc = 0.f;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    acc = fmaf(__uint_as_float(ua.w[e] << 16), __uint_as_float(ub.w[e] << 16), acc);
    acc = fmaf(__uint_as_float(ua.w[e] & 0xffff0000u), __uint_as_float(ub.w[e] & 0xffff0000u), acc);
  }
  return acc;
}

// store one accumulator set (rows = head-dim columns 32*dt + 8g + 4hh + r of tensor row `row`) as bf16
template <int DT>
__device__ __forceinline__ void store_acc_row(uint16_t* row, const float16_t (&acc)[DT], float mul, int hh) {
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      uint2 w;
      w.x = pack_bf16x2(acc[dt][4 * g + 0] * mul, acc[dt][4 * g + 1] * mul);
      w.y = pack_bf16x2(acc[dt][4 * g + 2] * mul, acc[dt][4 * g + 3] * mul);
      *reinterpret_cast<uint2*>(row + 32 * dt + 8 * g + 4 * hh) = w;
    }
}

static constexpr float kLazyRescale = 60.0f;  // the running reference exponent moves only when the row maximum grew by > 2^60

// ===================================================================================================
// Forward.  Workgroup = 64 query rows: wave = (rg, ks), rg = 32-row group, ks = which 32 keys of each 64-key
// tile.  K and V tiles are staged in LDS, both with swapped rows.
// ===================================================================================================
template <int D>
__global__ __launch_bounds__(256) void attn_fwd_mfma_kernel(AttnParams P, const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
                                                           const uint16_t* __restrict__ v, uint16_t* __restrict__ o, float* __restrict__ lse) {
  constexpr int BM = 64, BN = 64, KP = D + 8, KC = D / 16, DT = D / 32;
  __shared__ __attribute__((aligned(16))) uint16_t smem[2 * BN * KP];
  uint16_t* Ks = smem;
  uint16_t* Vs = smem + BN * KP;

  const int N = P.b * P.A;
  const int nrb = (P.s + BM - 1) / BM;
  const int rb = nrb - 1 - (int)(blockIdx.x / N);  // heaviest row blocks first
  const int bn = blockIdx.x % N, beta = bn / P.A, n = bn % P.A;
  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, li = lane & 31, hh = lane >> 5;
  const int rg = wave & 1, ks = wave >> 1;
  const int64_t base = (int64_t)beta * P.stride_b + (int64_t)n * P.stride_a;
  const int gstride = (int)P.stride_s;
  const int iw0 = rb * BM + rg * 32;  // first row of this wave
  const int i = iw0 + li;
  const int i_ld = i < P.s ? i : P.s - 1;

  bf16x8_t qf[KC];
#pragma unroll
  for (int kc = 0; kc < KC; ++kc) qf[kc] = ld_frag(q + base + (int64_t)i_ld * P.stride_s + 16 * kc + 8 * hh);

  // Philox call index of (row i, key 0): offset + e/8 with e = ((beta*a + head)*s + i)*s
  const uint64_t rowG = P.offset + (((uint64_t)beta * (uint64_t)P.a_global + (uint64_t)(P.head0 + n)) * (uint64_t)P.s + (uint64_t)i_ld) * (uint64_t)(P.s >> 3);

  float16_t oacc[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int e = 0; e < 16; ++e) oacc[dt][e] = 0.f;
  float m_ref = -INFINITY, l_run = 0.f;
  const float sc2 = P.scale * kLog2e;

  const int last_row = min(rb * BM + BM - 1, P.s - 1);
  const int ntile = last_row / BN + 1;
  TileMap<D> map;
  map.init(tid, gstride, KP, true);
  TileBuf<D> kbuf, vbuf;
  const uint16_t* kg = k + base;
  const uint16_t* vg = v + base;
  tile_fetch(kbuf, map, kg, gstride, P.s, tid);
  tile_fetch(vbuf, map, vg, gstride, P.s, tid);
  for (int jt = 0; jt < ntile; ++jt) {
    const int j0 = jt * BN;
    __syncthreads();  // every wave is done reading the previous tile
    tile_commit(kbuf, map, Ks);
    tile_commit(vbuf, map, Vs);
    __syncthreads();
    if (jt + 1 < ntile) {  // next tile's global loads fly while this one is computed
      tile_fetch(kbuf, map, kg + (int64_t)(j0 + BN) * gstride, gstride, P.s - (j0 + BN), tid);
      tile_fetch(vbuf, map, vg + (int64_t)(j0 + BN) * gstride, gstride, P.s - (j0 + BN), tid);
    }
    const int j0w = j0 + 32 * ks;  // this wave's 32 keys
    if (j0w <= iw0 + 31) {
      // ---- S^T = K Q^T ----
      float16_t st;
#pragma unroll
      for (int e = 0; e < 16; ++e) st[e] = 0.f;
#pragma unroll
      for (int kc = 0; kc < KC; ++kc) st = mfma32(ld_frag(Ks + (32 * ks + li) * KP + 16 * kc + 8 * hh), qf[kc], st);
      // st[8*c + e] is the score of key j0w + 16*c + 8*hh + e against query row i
      const bool diag = (j0w + 31 > iw0);
      float mt = -INFINITY;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        float x = st[e] * sc2;
        if (diag && (j0w + 16 * (e >> 3) + 8 * hh + (e & 7) > i)) x = -INFINITY;
        st[e] = x;
        mt = fmaxf(mt, x);
      }
      mt = fmaxf(mt, __shfl_xor(mt, 32, 64));
      if (__builtin_expect(__builtin_amdgcn_ballot_w64(mt > m_ref + kLazyRescale) != 0, 0)) {
        const float m_new = fmaxf(m_ref, mt);
        const float corr = __builtin_amdgcn_exp2f(m_ref - m_new);
        m_ref = m_new;
        l_run *= corr;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
          for (int e = 0; e < 16; ++e) oacc[dt][e] *= corr;
      }
      float psum = 0.f;
      bf16x8_t pf[2];
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        const uint32_t keep = keep_bits8(rowG + (uint64_t)((j0w + 16 * c + 8 * hh) >> 3), 0u, P.key0, P.key1, P.thresh);
        float pd[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float pe = SAR_EXP2(st[8 * c + e] - m_ref);
          psum += pe;
          pd[e] = ((keep >> e) & 1u) ? pe : 0.f;
        }
        pf[c] = pack8(pd);
      }
      l_run += psum;
      // ---- O^T += V^T P^T ----
#pragma unroll
      for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) oacc[dt] = mfma32(ld_frag_tr_perm(Vs, KP, 32 * ks + 16 * c, 32 * dt, lane), pf[c], oacc[dt]);
    }
  }

  // ---- merge the two key halves of each row group, then O = O^T^T / ((1-p) l), LSE = m + ln l ----
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  __syncthreads();
  float* mg = reinterpret_cast<float*>(smem) + rg * (64 * (16 * DT + 2));
  if (ks == 1) {
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int e = 0; e < 16; ++e) mg[(16 * dt + e) * 64 + lane] = oacc[dt][e];
    mg[(16 * DT) * 64 + lane] = m_ref;
    mg[(16 * DT + 1) * 64 + lane] = l_tot;
  }
  __syncthreads();
  if (ks == 0) {
    const float m1 = mg[(16 * DT) * 64 + lane], l1 = mg[(16 * DT + 1) * 64 + lane];
    const float m = fmaxf(m_ref, m1);
    const float w0 = __builtin_amdgcn_exp2f(m_ref - m), w1 = __builtin_amdgcn_exp2f(m1 - m);
    const float l = l_tot * w0 + l1 * w1;
    const float inv = P.keep_scale / l;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int e = 0; e < 16; ++e) oacc[dt][e] = oacc[dt][e] * w0 + mg[(16 * dt + e) * 64 + lane] * w1;
    if (i < P.s) {
      store_acc_row<DT>(o + base + (int64_t)i * P.stride_s, oacc, inv, hh);
      if (hh == 0) lse[(size_t)bn * P.s + i] = (m + __builtin_amdgcn_logf(l)) * kLn2;
    }
  }
}

// ===================================================================================================
// Backward, row-stationary pass: delta_i = dO_i . O_i and dQ_i = alpha sum_j dS_ij K_j, with
// P_ij = exp(alpha q_i.k_j - LSE_i), dP = (dO V^T) o M/(1-p), dS = P o (dP - delta) recomputed per tile.
// Same workgroup shape as the forward.
// ===================================================================================================
template <int D>
__global__ __launch_bounds__(256) void attn_bwd_dq_mfma_kernel(AttnParams P, const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
                                                              const uint16_t* __restrict__ v, const uint16_t* __restrict__ o,
                                                              const float* __restrict__ lse, const uint16_t* __restrict__ dO,
                                                              uint16_t* __restrict__ dq, float* __restrict__ delta) {
  constexpr int BM = 64, BN = 64, KP = D + 8, KC = D / 16, DT = D / 32;
  __shared__ __attribute__((aligned(16))) uint16_t smem[2 * BN * KP];
  uint16_t* Ks = smem;
  uint16_t* Vs = smem + BN * KP;

  const int N = P.b * P.A;
  const int nrb = (P.s + BM - 1) / BM;
  const int rb = nrb - 1 - (int)(blockIdx.x / N);
  const int bn = blockIdx.x % N, beta = bn / P.A, n = bn % P.A;
  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, li = lane & 31, hh = lane >> 5;
  const int rg = wave & 1, ks = wave >> 1;
  const int64_t base = (int64_t)beta * P.stride_b + (int64_t)n * P.stride_a;
  const int gstride = (int)P.stride_s;
  const int iw0 = rb * BM + rg * 32;
  const int i = iw0 + li;
  const int i_ld = i < P.s ? i : P.s - 1;

  bf16x8_t qf[KC], dof[KC];
  float dpart = 0.f;
#pragma unroll
  for (int kc = 0; kc < KC; ++kc) {
    const int64_t off = base + (int64_t)i_ld * P.stride_s + 16 * kc + 8 * hh;
    qf[kc] = ld_frag(q + off);
    dof[kc] = ld_frag(dO + off);
    dpart += dot8(dof[kc], ld_frag(o + off));
  }
  const float dl = dpart + __shfl_xor(dpart, 32, 64);
  if (ks == 0 && hh == 0 && i < P.s) delta[(size_t)bn * P.s + i] = dl;
  const float lse2 = lse[(size_t)bn * P.s + i_ld] * kLog2e;
  const uint64_t rowG = P.offset + (((uint64_t)beta * (uint64_t)P.a_global + (uint64_t)(P.head0 + n)) * (uint64_t)P.s + (uint64_t)i_ld) * (uint64_t)(P.s >> 3);
  const float sc2 = P.scale * kLog2e;

  float16_t dqacc[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int e = 0; e < 16; ++e) dqacc[dt][e] = 0.f;

  const int last_row = min(rb * BM + BM - 1, P.s - 1);
  const int ntile = last_row / BN + 1;
  TileMap<D> map;
  map.init(tid, gstride, KP, true);
  TileBuf<D> kbuf, vbuf;
  const uint16_t* kg = k + base;
  const uint16_t* vg = v + base;
  tile_fetch(kbuf, map, kg, gstride, P.s, tid);
  tile_fetch(vbuf, map, vg, gstride, P.s, tid);
  for (int jt = 0; jt < ntile; ++jt) {
    const int j0 = jt * BN;
    __syncthreads();
    tile_commit(kbuf, map, Ks);
    tile_commit(vbuf, map, Vs);
    __syncthreads();
    if (jt + 1 < ntile) {
      tile_fetch(kbuf, map, kg + (int64_t)(j0 + BN) * gstride, gstride, P.s - (j0 + BN), tid);
      tile_fetch(vbuf, map, vg + (int64_t)(j0 + BN) * gstride, gstride, P.s - (j0 + BN), tid);
    }
    const int j0w = j0 + 32 * ks;
    if (j0w <= iw0 + 31) {
      const bool diag = (j0w + 31 > iw0);
      float16_t st, dd;
#pragma unroll
      for (int e = 0; e < 16; ++e) { st[e] = 0.f; dd[e] = 0.f; }
#pragma unroll
      for (int kc = 0; kc < KC; ++kc) {
        st = mfma32(ld_frag(Ks + (32 * ks + li) * KP + 16 * kc + 8 * hh), qf[kc], st);
        dd = mfma32(ld_frag(Vs + (32 * ks + li) * KP + 16 * kc + 8 * hh), dof[kc], dd);
      }
      bf16x8_t dsf[2];
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        const int jc = j0w + 16 * c + 8 * hh;
        const uint32_t keep = keep_bits8(rowG + (uint64_t)(jc >> 3), 0u, P.key0, P.key1, P.thresh);
        float ds[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float pex = SAR_EXP2(fmaf(st[8 * c + e], sc2, -lse2));
          const float pe = (diag && (jc + e > i)) ? 0.f : pex;
          const float dp = ((keep >> e) & 1u) ? dd[8 * c + e] * P.keep_scale : 0.f;
          ds[e] = pe * (dp - dl);
        }
        dsf[c] = pack8(ds);
      }
#pragma unroll
      for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) dqacc[dt] = mfma32(ld_frag_tr_perm(Ks, KP, 32 * ks + 16 * c, 32 * dt, lane), dsf[c], dqacc[dt]);
    }
  }
  // ---- sum the two key halves, scale, store ----
  __syncthreads();
  float* mg = reinterpret_cast<float*>(smem) + rg * (64 * 16 * DT);
  if (ks == 1) {
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int e = 0; e < 16; ++e) mg[(16 * dt + e) * 64 + lane] = dqacc[dt][e];
  }
  __syncthreads();
  if (ks == 0) {
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int e = 0; e < 16; ++e) dqacc[dt][e] += mg[(16 * dt + e) * 64 + lane];
    if (i < P.s) store_acc_row<DT>(dq + base + (int64_t)i * P.stride_s, dqacc, P.scale, hh);
  }
}

// ===================================================================================================
// Backward, column-stationary pass.  Workgroup = 64 keys: wave = (kgp, is), kgp = 32-key group whose dK, dV
// accumulators it keeps in registers, is = which 32 query rows of each 64-row tile it sweeps.
//   dV_j = sum_i D_ij dO_i,  dK_j = alpha sum_i dS_ij q_i.
// P, D, dS are produced with one query row per lane; the two products above contract over i, so the bf16
// tiles are first moved to the one-key-per-lane layout by multiplying with an identity on the matrix core.
// ===================================================================================================
template <int D>
__global__ __launch_bounds__(256) void attn_bwd_dkdv_mfma_kernel(AttnParams P, const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
                                                                const uint16_t* __restrict__ v, const float* __restrict__ lse,
                                                                const uint16_t* __restrict__ dO, const float* __restrict__ delta,
                                                                uint16_t* __restrict__ dk, uint16_t* __restrict__ dv) {
  constexpr int BN = 64, BI = 64, KP = D + 8, KC = D / 16, DT = D / 32;
  __shared__ __attribute__((aligned(16))) uint16_t smem[4 * 64 * KP];
  __shared__ float lse_s[BI], delta_s[BI];
  uint16_t* Ksm = smem;                 // this workgroup's keys, rows swapped inside groups of 32
  uint16_t* Vsm = smem + 64 * KP;
  uint16_t* Qs = smem + 2 * 64 * KP;    // current 64 query rows, natural order
  uint16_t* dOs = smem + 3 * 64 * KP;

  const int N = P.b * P.A;
  const int kb = (int)(blockIdx.x / N);  // key block 0 sweeps the most rows: heaviest first
  const int bn = blockIdx.x % N, beta = bn / P.A, n = bn % P.A;
  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, li = lane & 31, hh = lane >> 5;
  const int kgp = wave & 1, is = wave >> 1;
  const int64_t base = (int64_t)beta * P.stride_b + (int64_t)n * P.stride_a;
  const int gstride = (int)P.stride_s;
  const int jw0 = kb * BN + kgp * 32;  // first key of this wave

  TileMap<D> map;
  map.init(tid, gstride, KP, true);
  {
    TileBuf<D> kbuf, vbuf;
    tile_fetch(kbuf, map, k + base + (int64_t)(kb * BN) * gstride, gstride, P.s - kb * BN, tid);
    tile_fetch(vbuf, map, v + base + (int64_t)(kb * BN) * gstride, gstride, P.s - kb * BN, tid);
    tile_commit(kbuf, map, Ksm);
    tile_commit(vbuf, map, Vsm);
  }
  map.init(tid, gstride, KP, false);
  // A operands of S^T and dD^T: LDS row 32*kgp + li holds key jw0 + perm_row(li)
  const uint16_t* kw = Ksm + (32 * kgp + li) * KP + 8 * hh;
  const uint16_t* vw = Vsm + (32 * kgp + li) * KP + 8 * hh;
  // identity operands: ident[c] has a one where this lane's column li equals key 16*c + 8*hh + e
  bf16x8_t ident[2];
#pragma unroll
  for (int c = 0; c < 2; ++c) {
    union { uint16_t h[8]; bf16x8_t v; } u;
#pragma unroll
    for (int e = 0; e < 8; ++e) u.h[e] = (li == 16 * c + 8 * hh + e) ? (uint16_t)0x3F80 : (uint16_t)0;
    ident[c] = u.v;
  }
  float16_t dkacc[DT], dvacc[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int e = 0; e < 16; ++e) { dkacc[dt][e] = 0.f; dvacc[dt][e] = 0.f; }

  const uint64_t headG = P.offset + (((uint64_t)beta * (uint64_t)P.a_global + (uint64_t)(P.head0 + n)) * (uint64_t)P.s) * (uint64_t)(P.s >> 3);
  const float sc2 = P.scale * kLog2e;
  const int nit = (P.s + BI - 1) / BI;
  const int it0 = kb;  // BI == BN: the first tile with rows >= this block's keys
  const uint16_t* qg = q + base;
  const uint16_t* dog = dO + base;
  TileBuf<D> qbuf, dobuf;
  float lse_n = 0.f, delta_n = 0.f;
  tile_fetch(qbuf, map, qg + (int64_t)(it0 * BI) * gstride, gstride, P.s - it0 * BI, tid);
  tile_fetch(dobuf, map, dog + (int64_t)(it0 * BI) * gstride, gstride, P.s - it0 * BI, tid);
  if (tid < BI) {
    const int ir = min(it0 * BI + tid, P.s - 1);
    lse_n = lse[(size_t)bn * P.s + ir];
    delta_n = delta[(size_t)bn * P.s + ir];
  }
  for (int it = it0; it < nit; ++it) {
    const int i0 = it * BI;
    __syncthreads();
    tile_commit(qbuf, map, Qs);
    tile_commit(dobuf, map, dOs);
    if (tid < BI) {
      lse_s[tid] = lse_n * kLog2e;
      delta_s[tid] = delta_n;
    }
    __syncthreads();
    if (it + 1 < nit) {  // next tile's global loads fly while this one is computed
      tile_fetch(qbuf, map, qg + (int64_t)(i0 + BI) * gstride, gstride, P.s - (i0 + BI), tid);
      tile_fetch(dobuf, map, dog + (int64_t)(i0 + BI) * gstride, gstride, P.s - (i0 + BI), tid);
      if (tid < BI) {
        const int ir = min(i0 + BI + tid, P.s - 1);
        lse_n = lse[(size_t)bn * P.s + ir];
        delta_n = delta[(size_t)bn * P.s + ir];
      }
    }
    const int i0w = i0 + 32 * is;  // this wave's 32 rows
    if (i0w + 31 >= jw0) {         // otherwise every row precedes this wave's keys
      const bool diag = (i0w < jw0 + 31);
      float16_t st, dd;
#pragma unroll
      for (int e = 0; e < 16; ++e) { st[e] = 0.f; dd[e] = 0.f; }
#pragma unroll
      for (int kc = 0; kc < KC; ++kc) {
        st = mfma32(ld_frag(kw + 16 * kc), ld_frag(Qs + (32 * is + li) * KP + 16 * kc + 8 * hh), st);
        dd = mfma32(ld_frag(vw + 16 * kc), ld_frag(dOs + (32 * is + li) * KP + 16 * kc + 8 * hh), dd);
      }
      const int i = i0w + li;
      const float lse2 = lse_s[32 * is + li], dl = delta_s[32 * is + li];
      const uint64_t rowG = headG + (uint64_t)min(i, P.s - 1) * (uint64_t)(P.s >> 3);
      const bool row_ok = i < P.s;
      bf16x8_t df[2], dsf[2];
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        const int jc = jw0 + 16 * c + 8 * hh;
        const uint32_t keep = keep_bits8(rowG + (uint64_t)(jc >> 3), 0u, P.key0, P.key1, P.thresh);
        float dvv[8], ds[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float pex = SAR_EXP2(fmaf(st[8 * c + e], sc2, -lse2));
          const bool dead = !row_ok || (diag && (jc + e > i));
          const float pe = dead ? 0.f : pex;
          const float km = ((keep >> e) & 1u) ? P.keep_scale : 0.f;
          dvv[e] = pe * km;
          ds[e] = pe * (dd[8 * c + e] * km - dl);
        }
        df[c] = pack8(dvv);
        dsf[c] = pack8(ds);
      }
      // one-key-per-lane copies: T[i][key] = sum_k tile[i][k] I[k][key]
      float16_t tD, tS;
#pragma unroll
      for (int e = 0; e < 16; ++e) { tD[e] = 0.f; tS[e] = 0.f; }
      tD = mfma32(df[0], ident[0], tD);
      tS = mfma32(dsf[0], ident[0], tS);
      tD = mfma32(df[1], ident[1], tD);
      tS = mfma32(dsf[1], ident[1], tS);
      // acc[4g + r] <-> row 8g + 4hh + r: operand X takes g in {2X, 2X+1}, i.e. rows 16X + 8*(e>>2) + 4hh + (e&3)
#pragma unroll
      for (int X = 0; X < 2; ++X) {
        float td[8], ts[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) { td[e] = tD[8 * X + e]; ts[e] = tS[8 * X + e]; }
        const bf16x8_t dT = pack8(td), sT = pack8(ts);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
          dvacc[dt] = mfma32(ld_frag_tr_perm(dOs, KP, 32 * is + 16 * X, 32 * dt, lane), dT, dvacc[dt]);
          dkacc[dt] = mfma32(ld_frag_tr_perm(Qs, KP, 32 * is + 16 * X, 32 * dt, lane), sT, dkacc[dt]);
        }
      }
    }
  }
  // ---- sum the two row halves, scale, store ----
  __syncthreads();
  float* mg = reinterpret_cast<float*>(smem) + kgp * (64 * 32 * DT);
  if (is == 1) {
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        mg[(32 * dt + e) * 64 + lane] = dkacc[dt][e];
        mg[(32 * dt + 16 + e) * 64 + lane] = dvacc[dt][e];
      }
  }
  __syncthreads();
  if (is == 0) {
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        dkacc[dt][e] += mg[(32 * dt + e) * 64 + lane];
        dvacc[dt][e] += mg[(32 * dt + 16 + e) * 64 + lane];
      }
    const int key = jw0 + li;
    if (key < P.s) {
      store_acc_row<DT>(dk + base + (int64_t)key * P.stride_s, dkacc, P.scale, hh);
      store_acc_row<DT>(dv + base + (int64_t)key * P.stride_s, dvacc, 1.0f, hh);
    }
  }
}

bool attn_mfma_supported(int d) { return d == 64 || d == 96 || d == 128 || d == 160; }

template <int D>
static hipError_t fwd_d(const AttnParams& P, const void* q, const void* k, const void* v, void* o, float* lse, hipStream_t st) {
  const int N = P.b * P.A, nrb = (P.s + 63) / 64;
  hipLaunchKernelGGL((attn_fwd_mfma_kernel<D>), dim3((unsigned)(nrb * N)), dim3(256), 0, st, P, (const uint16_t*)q, (const uint16_t*)k,
                     (const uint16_t*)v, (uint16_t*)o, lse);
  return hipGetLastError();
}

hipError_t launch_attn_fwd_mfma(const AttnParams& P, const void* q, const void* k, const void* v, void* o, float* lse, hipStream_t st) {
  switch (P.d) {
    case 64: return fwd_d<64>(P, q, k, v, o, lse, st);
    case 96: return fwd_d<96>(P, q, k, v, o, lse, st);
    case 128: return fwd_d<128>(P, q, k, v, o, lse, st);
    case 160: return fwd_d<160>(P, q, k, v, o, lse, st);
    default: return hipErrorInvalidValue;
  }
}

template <int D>
static hipError_t bwd_d(const AttnParams& P, const void* q, const void* k, const void* v, const void* o, const float* lse, const void* dO, void* dq,
                        void* dk, void* dv, float* delta, int passes, hipStream_t st) {
  const int N = P.b * P.A, nb = (P.s + 63) / 64;
  if (passes & 1)
    hipLaunchKernelGGL((attn_bwd_dq_mfma_kernel<D>), dim3((unsigned)(nb * N)), dim3(256), 0, st, P, (const uint16_t*)q, (const uint16_t*)k,
                       (const uint16_t*)v, (const uint16_t*)o, lse, (const uint16_t*)dO, (uint16_t*)dq, delta);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (passes & 2)
    hipLaunchKernelGGL((attn_bwd_dkdv_mfma_kernel<D>), dim3((unsigned)(nb * N)), dim3(256), 0, st, P, (const uint16_t*)q, (const uint16_t*)k,
                       (const uint16_t*)v, lse, (const uint16_t*)dO, (const float*)delta, (uint16_t*)dk, (uint16_t*)dv);
  return hipGetLastError();
}

hipError_t launch_attn_bwd_mfma(const AttnParams& P, const void* q, const void* k, const void* v, const void* o, const float* lse, const void* dO,
                                void* dq, void* dk, void* dv, float* delta, int passes, hipStream_t st) {
  switch (P.d) {
    case 64: return bwd_d<64>(P, q, k, v, o, lse, dO, dq, dk, dv, delta, passes, st);
    case 96: return bwd_d<96>(P, q, k, v, o, lse, dO, dq, dk, dv, delta, passes, st);
    case 128: return bwd_d<128>(P, q, k, v, o, lse, dO, dq, dk, dv, delta, passes, st);
    case 160: return bwd_d<160>(P, q, k, v, o, lse, dO, dq, dk, dv, delta, passes, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace sar
