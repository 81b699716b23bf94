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

__device__ __forceinline__ float16_t mfma32(bf16x8_t a, bf16x8_t b, float16_t c) { return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0); }

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

// cooperative copy of `nrows` rows x D bf16 from global (row stride gstride, rows clamped to row_max) to LDS
template <int D, int NT, bool PERM>
__device__ __forceinline__ void load_tile(uint16_t* lds, int pitch, const uint16_t* g, int64_t gstride, int row0, int nrows, int row_max, int tid) {
  constexpr int CPR = D / 8;  // 16-byte chunks per row
  for (int c = tid; c < nrows * CPR; c += NT) {
    const int r = c / CPR, cc = c - r * CPR;
    int gr = row0 + r;
    gr = gr > row_max ? row_max : gr;
    const uint4 val = *reinterpret_cast<const uint4*>(g + (int64_t)gr * gstride + 8 * cc);
    const int lr = PERM ? perm_row(r) : r;
    *reinterpret_cast<uint4*>(lds + lr * pitch + 8 * cc) = val;
  }
}

// ===================================================================================================
// Forward.  Workgroup = NW waves x 32 query rows; K/V tiles of 64 keys staged in LDS.
// ===================================================================================================
template <int D, int NW>
__global__ __launch_bounds__(NW * 64) void attn_fwd_mfma_kernel(AttnParams P, const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
                                                               const uint16_t* __restrict__ v, uint16_t* __restrict__ o, float* __restrict__ lse) {
  constexpr int BM = 32 * NW, BN = 64, KP = D + 8, KC = D / 16, DT = D / 32, NT = NW * 64;
  __shared__ __attribute__((aligned(16))) uint16_t Ks[BN * KP];
  __shared__ __attribute__((aligned(16))) uint16_t Vs[BN * KP];

  const int N = P.b * P.A;
  const int nrb = (P.s + BM - 1) / BM;
  const int rb = nrb - 1 - (int)(blockIdx.x / N);  // heaviest row blocks first
  const int bn = blockIdx.x % N, beta = bn / P.A, n = bn % P.A;
  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, li = lane & 31, hh = lane >> 5;
  const int64_t base = (int64_t)beta * P.stride_b + (int64_t)n * P.stride_a;
  const int iw0 = rb * BM + wave * 32;  // first row of this wave
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
  float m_run = -INFINITY, l_run = 0.f;
  const float sc2 = P.scale * kLog2e;

  const int last_row = min(rb * BM + BM - 1, P.s - 1);
  const int ntile = last_row / BN + 1;
  for (int jt = 0; jt < ntile; ++jt) {
    const int j0 = jt * BN;
    __syncthreads();
    load_tile<D, NT, true>(Ks, KP, k + base, P.stride_s, j0, BN, P.s - 1, tid);
    load_tile<D, NT, false>(Vs, KP, v + base, P.stride_s, j0, BN, P.s - 1, tid);
    __syncthreads();
    if (j0 > iw0 + 31) continue;  // whole tile above this wave's diagonal (barriers are at the loop head)
    const bool two = (j0 + 32 <= iw0 + 31);  // second 32-key sub-tile has unmasked entries for this wave

    // ---- S^T = K Q^T for the two 32-key sub-tiles ----
    float16_t st[2];
#pragma unroll
    for (int e = 0; e < 16; ++e) { st[0][e] = 0.f; st[1][e] = 0.f; }
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) {
      st[0] = mfma32(ld_frag(Ks + li * KP + 16 * kc + 8 * hh), qf[kc], st[0]);
      if (two) st[1] = mfma32(ld_frag(Ks + (32 + li) * KP + 16 * kc + 8 * hh), qf[kc], st[1]);
    }
    // st[u][8*c + e] is the score of key j0 + 32*u + 16*c + 8*hh + e against query row i
    const bool diag = (j0 + BN - 1 > iw0);
    float mt = -INFINITY;
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        float x = st[u][e] * sc2;
        if (diag) {
          const int j = j0 + 32 * u + 16 * (e >> 3) + 8 * hh + (e & 7);
          if (j > i) x = -INFINITY;
        }
        if (u == 1 && !two) x = -INFINITY;
        st[u][e] = x;
        mt = fmaxf(mt, x);
      }
    mt = fmaxf(mt, __shfl_xor(mt, 32, 64));
    const float m_new = fmaxf(m_run, mt);
    const float corr = __builtin_amdgcn_exp2f(m_run - m_new);
    m_run = m_new;
    float psum = 0.f;
    bf16x8_t pf[2][2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      if (u == 0 || two) {
#pragma unroll
        for (int c = 0; c < 2; ++c) {
          const uint32_t keep = keep_bits8(rowG + (uint64_t)((j0 + 32 * u + 16 * c + 8 * hh) >> 3), 0u, P.key0, P.key1, P.thresh);
          float pd[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const float pe = __builtin_amdgcn_exp2f(st[u][8 * c + e] - m_new);
            psum += pe;
            pd[e] = ((keep >> e) & 1u) ? pe : 0.f;
          }
          pf[u][c] = pack8(pd);
        }
      }
    }
    l_run = l_run * corr + psum;
    if (__builtin_amdgcn_ballot_w64(corr != 1.0f)) {
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int e = 0; e < 16; ++e) oacc[dt][e] *= corr;
    }
    // ---- O^T += V^T P^T ----
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      if (u == 0 || two) {
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
          for (int dt = 0; dt < DT; ++dt) oacc[dt] = mfma32(ld_frag_tr(Vs, KP, 32 * u + 16 * c, 32 * dt, lane), pf[u][c], oacc[dt]);
      }
    }
  }

  // ---- epilogue: O = O^T^T * (1/(1-p)) / l, LSE = m + ln l ----
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  const float inv = P.keep_scale / l_tot;
  if (i < P.s) {
    uint16_t* orow = o + base + (int64_t)i * P.stride_s;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        uint2 w;
        w.x = pack_bf16x2(oacc[dt][4 * g + 0] * inv, oacc[dt][4 * g + 1] * inv);
        w.y = pack_bf16x2(oacc[dt][4 * g + 2] * inv, oacc[dt][4 * g + 3] * inv);
        *reinterpret_cast<uint2*>(orow + 32 * dt + 8 * g + 4 * hh) = w;
      }
    if (hh == 0) lse[(size_t)bn * P.s + i] = (m_run + __builtin_amdgcn_logf(l_tot)) * kLn2;
  }
}


// Same as ld_frag_tr but for the k order that the swapped K rows and the identity-transposed tiles use:
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

// ===================================================================================================
// Backward, row-stationary pass: delta_i = dO_i . O_i and dQ_i = alpha sum_j dS_ij K_j, with
// P_ij = exp(alpha q_i.k_j - LSE_i), dP = (dO V^T) o M/(1-p), dS = P o (dP - delta) recomputed per tile.
// ===================================================================================================
template <int D, int NW>
__global__ __launch_bounds__(NW * 64) void attn_bwd_dq_mfma_kernel(AttnParams P, const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
                                                                  const uint16_t* __restrict__ v, const uint16_t* __restrict__ o,
                                                                  const float* __restrict__ lse, const uint16_t* __restrict__ dO,
                                                                  uint16_t* __restrict__ dq, float* __restrict__ delta) {
  constexpr int BM = 32 * NW, BN = 64, KP = D + 8, KC = D / 16, DT = D / 32, NT = NW * 64;
  __shared__ __attribute__((aligned(16))) uint16_t Ks[BN * KP];
  __shared__ __attribute__((aligned(16))) uint16_t Vs[BN * KP];

  const int N = P.b * P.A;
  const int nrb = (P.s + BM - 1) / BM;
  const int rb = nrb - 1 - (int)(blockIdx.x / N);
  const int bn = blockIdx.x % N, beta = bn / P.A, n = bn % P.A;
  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, li = lane & 31, hh = lane >> 5;
  const int64_t base = (int64_t)beta * P.stride_b + (int64_t)n * P.stride_a;
  const int iw0 = rb * BM + wave * 32;
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
  if (hh == 0 && i < P.s) delta[(size_t)bn * P.s + i] = dl;
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
  for (int jt = 0; jt < ntile; ++jt) {
    const int j0 = jt * BN;
    __syncthreads();
    load_tile<D, NT, true>(Ks, KP, k + base, P.stride_s, j0, BN, P.s - 1, tid);
    load_tile<D, NT, true>(Vs, KP, v + base, P.stride_s, j0, BN, P.s - 1, tid);
    __syncthreads();
    if (j0 > iw0 + 31) continue;
    const bool two = (j0 + 32 <= iw0 + 31);
    const bool diag = (j0 + BN - 1 > iw0);
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      if (u == 0 || two) {
        float16_t st, dd;
#pragma unroll
        for (int e = 0; e < 16; ++e) { st[e] = 0.f; dd[e] = 0.f; }
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) {
          st = mfma32(ld_frag(Ks + (32 * u + li) * KP + 16 * kc + 8 * hh), qf[kc], st);
          dd = mfma32(ld_frag(Vs + (32 * u + li) * KP + 16 * kc + 8 * hh), dof[kc], dd);
        }
        bf16x8_t dsf[2];
#pragma unroll
        for (int c = 0; c < 2; ++c) {
          const int jc = j0 + 32 * u + 16 * c + 8 * hh;
          const uint32_t keep = keep_bits8(rowG + (uint64_t)(jc >> 3), 0u, P.key0, P.key1, P.thresh);
          float ds[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            float pe = __builtin_amdgcn_exp2f(fmaf(st[8 * c + e], sc2, -lse2));
            if (diag && (jc + e > i)) pe = 0.f;
            const float dp = ((keep >> e) & 1u) ? dd[8 * c + e] * P.keep_scale : 0.f;
            ds[e] = pe * (dp - dl);
          }
          dsf[c] = pack8(ds);
        }
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
          for (int dt = 0; dt < DT; ++dt) dqacc[dt] = mfma32(ld_frag_tr_perm(Ks, KP, 32 * u + 16 * c, 32 * dt, lane), dsf[c], dqacc[dt]);
      }
    }
  }
  if (i < P.s) {
    uint16_t* row = dq + base + (int64_t)i * P.stride_s;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        uint2 w;
        w.x = pack_bf16x2(dqacc[dt][4 * g + 0] * P.scale, dqacc[dt][4 * g + 1] * P.scale);
        w.y = pack_bf16x2(dqacc[dt][4 * g + 2] * P.scale, dqacc[dt][4 * g + 3] * P.scale);
        *reinterpret_cast<uint2*>(row + 32 * dt + 8 * g + 4 * hh) = w;
      }
  }
}

// ===================================================================================================
// Backward, column-stationary pass: each wave owns 32 keys (K_j, V_j operands and the dK_j, dV_j
// accumulators stay in registers) and sweeps the query rows i >= j in tiles of 32 staged in LDS.
//   dV_j = sum_i D_ij dO_i,  dK_j = alpha sum_i dS_ij q_i.
// P, D, dS are produced with one query row per lane; the two products above contract over i, so the bf16
// tiles are first moved to the one-key-per-lane layout by multiplying with an identity on the matrix core.
// ===================================================================================================
template <int D, int NW>
__global__ __launch_bounds__(NW * 64) void attn_bwd_dkdv_mfma_kernel(AttnParams P, const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
                                                                    const uint16_t* __restrict__ v, const float* __restrict__ lse,
                                                                    const uint16_t* __restrict__ dO, const float* __restrict__ delta,
                                                                    uint16_t* __restrict__ dk, uint16_t* __restrict__ dv) {
  constexpr int BN = 32 * NW, BI = 32, KP = D + 8, KC = D / 16, DT = D / 32, NT = NW * 64;
  __shared__ __attribute__((aligned(16))) uint16_t Qs[BI * KP];
  __shared__ __attribute__((aligned(16))) uint16_t dOs[BI * KP];
  __shared__ float lse_s[BI], delta_s[BI];

  const int N = P.b * P.A;
  const int kb = (int)(blockIdx.x / N);  // key block 0 sweeps the most rows: heaviest first
  const int bn = blockIdx.x % N, beta = bn / P.A, n = bn % P.A;
  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, li = lane & 31, hh = lane >> 5;
  const int64_t base = (int64_t)beta * P.stride_b + (int64_t)n * P.stride_a;
  const int jw0 = kb * BN + wave * 32;  // first key of this wave

  // A operands: MFMA row li <-> key jw0 + perm_row(li)
  bf16x8_t kf[KC], vf[KC];
  {
    int jr = jw0 + perm_row(li);
    jr = jr < P.s ? jr : P.s - 1;
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) {
      const int64_t off = base + (int64_t)jr * P.stride_s + 16 * kc + 8 * hh;
      kf[kc] = ld_frag(k + off);
      vf[kc] = ld_frag(v + off);
    }
  }
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
  for (int it = (kb * BN) / BI; it < nit; ++it) {
    const int i0 = it * BI;
    __syncthreads();
    load_tile<D, NT, false>(Qs, KP, q + base, P.stride_s, i0, BI, P.s - 1, tid);
    load_tile<D, NT, false>(dOs, KP, dO + base, P.stride_s, i0, BI, P.s - 1, tid);
    if (tid < BI) {
      const int ir = min(i0 + tid, P.s - 1);
      lse_s[tid] = lse[(size_t)bn * P.s + ir] * kLog2e;
      delta_s[tid] = delta[(size_t)bn * P.s + ir];
    }
    __syncthreads();
    if (i0 + BI - 1 < jw0) continue;  // every row of the tile precedes this wave's keys
    const bool diag = (i0 < jw0 + 31);
    float16_t st, dd;
#pragma unroll
    for (int e = 0; e < 16; ++e) { st[e] = 0.f; dd[e] = 0.f; }
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) {
      st = mfma32(kf[kc], ld_frag(Qs + li * KP + 16 * kc + 8 * hh), st);
      dd = mfma32(vf[kc], ld_frag(dOs + li * KP + 16 * kc + 8 * hh), dd);
    }
    const int i = i0 + li;
    const float lse2 = lse_s[li], dl = delta_s[li];
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
        float pe = __builtin_amdgcn_exp2f(fmaf(st[8 * c + e], sc2, -lse2));
        if (!row_ok || (diag && (jc + e > i))) pe = 0.f;
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
        dvacc[dt] = mfma32(ld_frag_tr_perm(dOs, KP, 16 * X, 32 * dt, lane), dT, dvacc[dt]);
        dkacc[dt] = mfma32(ld_frag_tr_perm(Qs, KP, 16 * X, 32 * dt, lane), sT, dkacc[dt]);
      }
    }
  }
  const int key = jw0 + li;
  if (key < P.s) {
    uint16_t* krow = dk + base + (int64_t)key * P.stride_s;
    uint16_t* vrow = dv + base + (int64_t)key * P.stride_s;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        uint2 w;
        w.x = pack_bf16x2(dkacc[dt][4 * g + 0] * P.scale, dkacc[dt][4 * g + 1] * P.scale);
        w.y = pack_bf16x2(dkacc[dt][4 * g + 2] * P.scale, dkacc[dt][4 * g + 3] * P.scale);
        *reinterpret_cast<uint2*>(krow + 32 * dt + 8 * g + 4 * hh) = w;
        w.x = pack_bf16x2(dvacc[dt][4 * g + 0], dvacc[dt][4 * g + 1]);
        w.y = pack_bf16x2(dvacc[dt][4 * g + 2], dvacc[dt][4 * g + 3]);
        *reinterpret_cast<uint2*>(vrow + 32 * dt + 8 * g + 4 * hh) = w;
      }
  }
}

bool attn_mfma_supported(int d) { return d == 64 || d == 96 || d == 128 || d == 160; }

template <int D>
static hipError_t fwd_d(const AttnParams& P, const void* q, const void* k, const void* v, void* o, float* lse, hipStream_t st) {
  constexpr int NW = 2;
  const int N = P.b * P.A, nrb = (P.s + 32 * NW - 1) / (32 * NW);
  hipLaunchKernelGGL((attn_fwd_mfma_kernel<D, NW>), dim3((unsigned)(nrb * N)), dim3(NW * 64), 0, st, P, (const uint16_t*)q, (const uint16_t*)k,
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
  constexpr int NWQ = 2, NWK = 2;
  const int N = P.b * P.A;
  const int nrb = (P.s + 32 * NWQ - 1) / (32 * NWQ), nkb = (P.s + 32 * NWK - 1) / (32 * NWK);
  if (passes & 1)
    hipLaunchKernelGGL((attn_bwd_dq_mfma_kernel<D, NWQ>), dim3((unsigned)(nrb * N)), dim3(NWQ * 64), 0, st, P, (const uint16_t*)q, (const uint16_t*)k,
                       (const uint16_t*)v, (const uint16_t*)o, lse, (const uint16_t*)dO, (uint16_t*)dq, delta);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (passes & 2)
  hipLaunchKernelGGL((attn_bwd_dkdv_mfma_kernel<D, NWK>), dim3((unsigned)(nkb * N)), dim3(NWK * 64), 0, st, P, (const uint16_t*)q, (const uint16_t*)k,
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
