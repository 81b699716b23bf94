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
#include "attn_mfma_common.h"

namespace sar {

static constexpr float kLazyRescale = 60.0f;  // the running reference exponent moves only when the row maximum grew by > 2^60

// ===================================================================================================
// Forward.  Workgroup = 64 query rows: wave = (rg, ks), rg = 32-row group, ks = which 32 keys of each 64-key
// tile.  K and V tiles (both with swapped rows) go from global memory straight into one of two LDS stages;
// the loads of tile j+1 are issued right after the single barrier of step j and land while tile j is computed.
// ===================================================================================================
template <int D>
__global__ __launch_bounds__(256) void attn_fwd_mfma_kernel(AttnParams P, const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
                                                           const uint16_t* __restrict__ v, uint16_t* __restrict__ o, float* __restrict__ lse) {
  constexpr int BM = 64, BN = 64, KP = D + 8, KC = D / 16, DT = D / 32;
  constexpr int TILE = BN * KP;
  __shared__ __attribute__((aligned(16))) uint16_t smem[4 * TILE];  // stage 0: K, V; stage 1: K, V

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
  DmaMap<D> map;
  map.init(wave, lane, gstride, true);
  const uint16_t* kg = k + base;
  const uint16_t* vg = v + base;
  if (P.s >= BN) {
    dma_tile<D>(map, kg, smem, wave);
    dma_tile<D>(map, vg, smem + TILE, wave);
  } else {
    dma_tile_ragged<D>(map, kg, smem, wave, lane, gstride, P.s);
    dma_tile_ragged<D>(map, vg, smem + TILE, wave, lane, gstride, P.s);
  }
  for (int jt = 0; jt < ntile; ++jt) {
    const int j0 = jt * BN;
    __syncthreads();  // tile jt has landed (every wave waited for its own loads); nobody reads the other stage any more
    if (jt + 1 < ntile) {
      uint16_t* nxt = smem + ((jt + 1) & 1) * 2 * TILE;
      const int left = P.s - (j0 + BN);
      if (left >= BN) {
        dma_tile<D>(map, kg + (int64_t)(j0 + BN) * gstride, nxt, wave);
        dma_tile<D>(map, vg + (int64_t)(j0 + BN) * gstride, nxt + TILE, wave);
      } else {
        dma_tile_ragged<D>(map, kg + (int64_t)(j0 + BN) * gstride, nxt, wave, lane, gstride, left);
        dma_tile_ragged<D>(map, vg + (int64_t)(j0 + BN) * gstride, nxt + TILE, wave, lane, gstride, left);
      }
    }
    const uint16_t* Ks = smem + (jt & 1) * 2 * TILE;
    const uint16_t* Vs = Ks + TILE;
    const int j0w = j0 + 32 * ks;  // this wave's 32 keys
    if (j0w <= iw0 + 31) {
      // ---- S^T = K Q^T ----
      float16_t st;
#pragma unroll
      for (int e = 0; e < 16; ++e) st[e] = 0.f;
#pragma unroll
      for (int kc = 0; kc < KC; ++kc) st = mfma32(ld_frag(Ks + (32 * ks + li) * KP + 16 * kc + 8 * hh), qf[kc], st);
      // st[8*c + e] is the score of key j0w + 16*c + 8*hh + e against query row i
      if (j0w + 31 > iw0) {  // tile touches the diagonal (uniform per wave): mask keys j > i
        asm volatile("" ::: "memory");  // keep this a branch: most tiles skip it
#pragma unroll
        for (int e = 0; e < 16; ++e)
          if (j0w + 16 * (e >> 3) + 8 * hh + (e & 7) > i) st[e] = -INFINITY;
      }
      // the softmax runs on alpha*log2(e)*score; alpha > 0, so the maximum can be taken on the raw scores
      float mt = fmaxf(fmaxf(st[0], st[1]), st[2]);
#pragma unroll
      for (int e = 3; e < 15; e += 2) mt = fmaxf(fmaxf(mt, st[e]), st[e + 1]);
      mt = fmaxf(mt, st[15]);
      mt = fmaxf(mt, __shfl_xor(mt, 32, 64)) * sc2;
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
          const float pe = __builtin_amdgcn_exp2f(fmaf(st[8 * c + e], sc2, -m_ref));
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
  constexpr int TILE = BN * KP;
  __shared__ __attribute__((aligned(16))) uint16_t smem[4 * TILE];  // stage 0: K, V; stage 1: K, V

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
  DmaMap<D> map;
  map.init(wave, lane, gstride, true);
  const uint16_t* kg = k + base;
  const uint16_t* vg = v + base;
  if (P.s >= BN) {
    dma_tile<D>(map, kg, smem, wave);
    dma_tile<D>(map, vg, smem + TILE, wave);
  } else {
    dma_tile_ragged<D>(map, kg, smem, wave, lane, gstride, P.s);
    dma_tile_ragged<D>(map, vg, smem + TILE, wave, lane, gstride, P.s);
  }
  for (int jt = 0; jt < ntile; ++jt) {
    const int j0 = jt * BN;
    __syncthreads();  // tile jt has landed (every wave waited for its own loads); nobody reads the other stage any more
    if (jt + 1 < ntile) {
      uint16_t* nxt = smem + ((jt + 1) & 1) * 2 * TILE;
      const int left = P.s - (j0 + BN);
      if (left >= BN) {
        dma_tile<D>(map, kg + (int64_t)(j0 + BN) * gstride, nxt, wave);
        dma_tile<D>(map, vg + (int64_t)(j0 + BN) * gstride, nxt + TILE, wave);
      } else {
        dma_tile_ragged<D>(map, kg + (int64_t)(j0 + BN) * gstride, nxt, wave, lane, gstride, left);
        dma_tile_ragged<D>(map, vg + (int64_t)(j0 + BN) * gstride, nxt + TILE, wave, lane, gstride, left);
      }
    }
    const uint16_t* Ks = smem + (jt & 1) * 2 * TILE;
    const uint16_t* Vs = Ks + TILE;
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
      if (diag) {  // uniform per wave: keys j > i get probability exp2(-inf) = 0
        asm volatile("" ::: "memory");  // keep this a branch: most tiles skip it
#pragma unroll
        for (int e = 0; e < 16; ++e)
          if (j0w + 16 * (e >> 3) + 8 * hh + (e & 7) > i) st[e] = -INFINITY;
      }
      bf16x8_t dsf[2];
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        const int jc = j0w + 16 * c + 8 * hh;
        const uint32_t keep = keep_bits8(rowG + (uint64_t)(jc >> 3), 0u, P.key0, P.key1, P.thresh);
        float ds[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float pe = __builtin_amdgcn_exp2f(fmaf(st[8 * c + e], sc2, -lse2));
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
static hipError_t bwd_dq_d(const AttnParams& P, const void* q, const void* k, const void* v, const void* o, const float* lse, const void* dO, void* dq,
                           float* delta, hipStream_t st) {
  const int N = P.b * P.A, nb = (P.s + 63) / 64;
  hipLaunchKernelGGL((attn_bwd_dq_mfma_kernel<D>), dim3((unsigned)(nb * N)), dim3(256), 0, st, P, (const uint16_t*)q, (const uint16_t*)k,
                     (const uint16_t*)v, (const uint16_t*)o, lse, (const uint16_t*)dO, (uint16_t*)dq, delta);
  return hipGetLastError();
}

hipError_t launch_attn_bwd_mfma(const AttnParams& P, const void* q, const void* k, const void* v, const void* o, const float* lse, const void* dO,
                                void* dq, void* dk, void* dv, float* delta, int passes, hipStream_t st) {
  hipError_t e = hipSuccess;
  if (passes & 1) {
    switch (P.d) {
      case 64: e = bwd_dq_d<64>(P, q, k, v, o, lse, dO, dq, delta, st); break;
      case 96: e = bwd_dq_d<96>(P, q, k, v, o, lse, dO, dq, delta, st); break;
      case 128: e = bwd_dq_d<128>(P, q, k, v, o, lse, dO, dq, delta, st); break;
      case 160: e = bwd_dq_d<160>(P, q, k, v, o, lse, dO, dq, delta, st); break;
      default: return hipErrorInvalidValue;
    }
    if (e != hipSuccess) return e;
  }
  if (passes & 2) e = launch_attn_bwd_dkdv_mfma(P, q, k, v, lse, dO, delta, dk, dv, st);
  return e;
}

}  // namespace sar
