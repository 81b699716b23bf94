// bf16 attention core, forward in its producer / consumer form (included by attn_mfma_rows.hip, which documents the tile
// layouts): a workgroup of 64 query rows runs eight waves, two per SIMD, and each (32 rows x 32 keys) block of a step is
// divided between them:
//   producer (waves 0..3)  scores S^T = K Q^T of the next tile between this tile's exponentials, keep selects and row sums,
//                          then the next tile's Philox words, mask and row maximum; it owns the row statistics (running
//                          reference exponent and sum) and hands P, rounded to bf16, to the consumer through LDS together
//                          with the factor by which the running output has to be rescaled first (1 unless the reference
//                          exponent moved);
//   consumer (waves 4..7)  O^T += V^T P^T one tile behind, and every direct-to-LDS load of the workgroup.
// A wave issues in order, so the waves of a pair fill each other's issue slots: the producer is vector-bound, the consumer
// waits for the matrix pipe and for its loads to be accepted.  One workgroup barrier per step.
#pragma once
#include "attn_mfma_common.h"

namespace sar {

template <int D, bool DROP>
__global__ __launch_bounds__(512, 1) void attn_fwd_split_kernel(AttnParams P, const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
                                                               const uint16_t* __restrict__ v, uint16_t* __restrict__ o, float* __restrict__ lse) {
  constexpr int BM = 64, BN = 64, KP = D + 8, KC = D / 16, DT = D / 32;
  constexpr int TILE = BN * KP;
  constexpr float kRescale = 60.0f;  // the running reference exponent moves only when the row maximum grew by > 2^60
  __shared__ __attribute__((aligned(16))) uint16_t smem[4 * TILE];   // K tile jt in stage jt & 1, then V likewise; afterwards the epilogue's buffers
  __shared__ __attribute__((aligned(16))) uint16_t xb[2][4][2][512];  // exchange: [tile parity][wave pair][key group c][16 bytes per lane]
  __shared__ float xc[2][4][64];                                      // ... and the rescaling factor per row
  uint16_t* Kst = smem;
  uint16_t* Vst = smem + 2 * TILE;

  const int N = P.b * P.A;
  const int nrb = (P.s + BM - 1) / BM;
  const int rb = nrb - 1 - (int)(blockIdx.x / N);  // heaviest row blocks first
  const int bn = blockIdx.x % N, beta = bn / P.A, n = bn % P.A;
  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, li = lane & 31, hh = lane >> 5;
  const bool producer = wave < 4;
  const int w = wave & 3;  // the pair: waves w and w + 4 sit on SIMD w
  const int rg = w & 1, ks = w >> 1;
  const int64_t base = (int64_t)beta * P.stride_b + (int64_t)n * P.stride_a;
  const int gstride = (int)P.stride_s;
  const int last_row = min(rb * BM + BM - 1, P.s - 1);
  const int nt = P.causal ? last_row / BN + 1 : (P.s + BN - 1) / BN;  // tiles the workgroup streams; the last one needs the mask
  const int i = rb * BM + rg * 32 + li;                               // this lane's query row

  float16_t oacc[DT];  // consumer
  float m_ref = 0.f, l_tot = 0.f;  // producer
  if (producer) {
    const int i_ld = i < P.s ? i : P.s - 1;
    const int jlim = P.causal ? i : P.s - 1;  // last key row i attends to
    bf16x8_t qf[KC];
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) qf[kc] = ld_frag(q + base + (int64_t)i_ld * P.stride_s + 16 * kc + 8 * hh);
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) asm volatile("" : "+v"(qf[kc]));
    // Philox call index of (row i, key 0): offset + e/8 with e = ((beta*a + head)*s + i)*s
    const uint64_t rowG = P.offset + (((uint64_t)beta * (uint64_t)P.a_global + (uint64_t)(P.head0 + n)) * (uint64_t)P.s + (uint64_t)i_ld) * (uint64_t)(P.s >> 3);
    const float sc2 = P.scale * kLog2e;
    float l_run = 0.f;
    auto philox_begin = [&](Philox4 (&r)[2], const int jt) __attribute__((always_inline)) {
#pragma unroll
      for (int c = 0; c < 2; ++c) r[c] = philox_start(rowG + (uint64_t)((jt * BN + 32 * ks + 16 * c + 8 * hh) >> 3), 0u);
    };
    auto mask_diag = [&](float16_t& st, const int jt) __attribute__((always_inline)) {
      const int j0w = jt * BN + 32 * ks;
#pragma unroll
      for (int e = 0; e < 16; ++e)
        if (j0w + 16 * (e >> 3) + 8 * hh + (e & 7) > jlim) st[e] = -INFINITY;
    };
    // row maximum of a score tile in the softmax's units, floored so that a fully masked tile stays finite
    auto tile_max = [&](const float16_t& st) __attribute__((always_inline)) {
      float mt = fmaxf(fmaxf(st[0], st[1]), st[2]);
#pragma unroll
      for (int e = 3; e < 15; e += 2) mt = fmaxf(fmaxf(mt, st[e]), st[e + 1]);
      mt = fmaxf(mt, st[15]);
      return fmaxf(xhalf_max(mt) * sc2, -1.0e30f);
    };
    Philox4 rnd[2] = {{0u, 0u, 0u, 0u}, {0u, 0u, 0u, 0u}};
    if (DROP) {  // the first tile's, while the first K tiles are on their way
      philox_begin(rnd, 0);
#pragma unroll
      for (int r = 0; r < 10; ++r) {
        philox_round(rnd[0], P.key0, P.key1, r);
        philox_round(rnd[1], P.key0, P.key1, r);
      }
    }
    __syncthreads();  // K tile 0 (and 1) are there
    float16_t st;
    {
      const uint16_t* Ks = Kst + (32 * ks + li) * KP + 8 * hh;
#pragma unroll
      for (int e = 0; e < 16; ++e) st[e] = 0.f;
#pragma unroll
      for (int kc = 0; kc < KC; ++kc) st = mfma32(ld_frag(Ks + 16 * kc), qf[kc], st);
      if (nt == 1) mask_diag(st, 0);
    }
    m_ref = tile_max(st);
    float corr = 1.0f;  // what the running output is multiplied by before tile jt is added

    // One step: tile jt's probabilities (to the consumer), and (NEXT != 0) the scores, Philox words, mask and maximum of
    // tile jt+1; NEXT == 2: that tile is the diagonal one.
    auto step = [&](const int jt, auto next) __attribute__((always_inline)) {
      constexpr int NEXT = decltype(next)::value;
      constexpr int kAhead = 3;
      __syncthreads();  // K tile jt+1 is there; the consumer has read exchange buffer jt & 1 (tile jt - 2)
      const uint16_t* Ksn = Kst + ((jt + 1) & 1) * TILE + (32 * ks + li) * KP + 8 * hh;
      float16_t stn;
#pragma unroll
      for (int e = 0; e < 16; ++e) stn[e] = 0.f;
      bf16x8_t kfr[kAhead];
      if (NEXT != 0) {
#pragma unroll
        for (int a = 0; a < kAhead && a < KC; ++a) kfr[a] = ld_frag(Ksn + 16 * a);
      }
      float psum = 0.f;
      float pd[16];
#pragma unroll
      for (int kc = 0; kc < KC; ++kc) {
        if (NEXT != 0) {
          stn = mfma32(kfr[kc % kAhead], qf[kc], stn);
          if (kc + kAhead < KC) kfr[kc % kAhead] = ld_frag(Ksn + 16 * (kc + kAhead));
        }
#pragma unroll
        for (int e = (16 * kc) / KC; e < (16 * (kc + 1)) / KC; ++e) {
          const float pe = __builtin_amdgcn_exp2f(fmaf(st[e], sc2, -m_ref));
          psum += pe;
          pd[e] = (!DROP || keep_field(rnd[e >> 3], e & 7, P.thresh)) ? pe : 0.f;
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      l_run += psum;
      {
        bf16x8_t* x = reinterpret_cast<bf16x8_t*>(&xb[jt & 1][w][0][0]) + lane;
        x[0] = pack8(pd);
        x[64] = pack8(pd + 8);
        xc[jt & 1][w][lane] = corr;
      }
      corr = 1.0f;
      if (NEXT != 0) {
        if (DROP) {
          philox_begin(rnd, jt + 1);
#pragma unroll
          for (int r = 0; r < 10; ++r) {
            philox_round(rnd[0], P.key0, P.key1, r);
            philox_round(rnd[1], P.key0, P.key1, r);
          }
        }
        if (NEXT == 2) mask_diag(stn, jt + 1);
        st = stn;
        const float mt = tile_max(stn);
        if (__builtin_expect(__builtin_amdgcn_ballot_w64(mt > m_ref + kRescale) != 0, 0)) {
          const float m_new = fmaxf(m_ref, mt);
          corr = __builtin_amdgcn_exp2f(m_ref - m_new);
          m_ref = m_new;
          l_run *= corr;
        }
      }
    };
    {
      int jt = 0;
      for (; jt + 2 < nt; ++jt) step(jt, std::integral_constant<int, 1>{});
      if (jt + 1 < nt) step(jt++, std::integral_constant<int, 2>{});
      step(jt++, std::integral_constant<int, 0>{});
    }
    __syncthreads();  // the consumer's last step
    l_tot = l_run + __shfl_xor(l_run, 32, 64);
  } else {
    // ---- consumer ----
    DmaMap<D, 4> lmap;
    lmap.init(w, lane, gstride, true);
    auto fetch = [&](const uint16_t* g, uint16_t* st2, int jt) __attribute__((always_inline)) {
      const int left = P.s - jt * BN;  // only the last tile of the sequence can end before its 64th row
      if (left >= BN) dma_tile<D>(lmap, g + (int64_t)(jt * BN) * gstride, st2 + (jt & 1) * TILE, w);
      else dma_tile_ragged<D>(lmap, g + (int64_t)(jt * BN) * gstride, st2 + (jt & 1) * TILE, w, lane, gstride, left);
    };
    fetch(k + base, Kst, 0);
    if (nt > 1) fetch(k + base, Kst, 1);
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int e = 0; e < 16; ++e) oacc[dt][e] = 0.f;
    dma_wait();
    __syncthreads();  // K tile 0 (and 1) are there
    for (int jt = 0; jt <= nt; ++jt) {
      dma_wait();       // this wave's share of K tile jt+1 and V tile jt-1 has landed
      __syncthreads();  // ... and everybody's; nobody reads K tile jt or V tile jt-2 any more
      if (jt + 2 < nt) fetch(k + base, Kst, jt + 2);
      if (jt < nt) fetch(v + base, Vst, jt);
      if (jt == 0) continue;
      const int t = jt - 1;
      const uint16_t* Vs = Vst + (t & 1) * TILE;
      const bf16x8_t* x = reinterpret_cast<const bf16x8_t*>(&xb[t & 1][w][0][0]) + lane;
      bf16x8_t pf[2] = {x[0], x[64]};
      const float corr = xc[t & 1][w][lane];
      if (__builtin_expect(__builtin_amdgcn_ballot_w64(corr != 1.0f) != 0, 0)) {
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
          for (int e = 0; e < 16; ++e) oacc[dt][e] *= corr;
      }
      constexpr int kAhead = 3, NPV = 2 * DT;
      auto v_frag = [&](const int idx) __attribute__((always_inline)) {
        return ld_frag_tr_perm(Vs, KP, 32 * ks + 16 * (idx / DT), 32 * (idx % DT), lane);
      };
      bf16x8_t vfr[kAhead];
#pragma unroll
      for (int a = 0; a < kAhead && a < NPV; ++a) vfr[a] = v_frag(a);
#pragma unroll
      for (int idx = 0; idx < NPV; ++idx) {
        oacc[idx % DT] = mfma32(vfr[idx % kAhead], pf[idx / DT], oacc[idx % DT]);
        if (idx + kAhead < NPV) vfr[idx % kAhead] = v_frag(idx + kAhead);
      }
    }
  }

  // ---- merge the two key halves of each row group, then O = O^T^T / ((1-p) l), LSE = m + ln l ----
  __syncthreads();  // everybody is done with the tiles
  float* mg = reinterpret_cast<float*>(smem) + rg * (64 * 16 * DT);
  float* stat = reinterpret_cast<float*>(smem) + 2 * (64 * 16 * DT);  // [pair][m, l][lane]
  if (producer) {
    stat[(2 * w) * 64 + lane] = m_ref;
    stat[(2 * w + 1) * 64 + lane] = l_tot;
  } else if (ks == 1) {
    acc_put<DT>(mg, oacc, lane);
  }
  __syncthreads();
  if (!producer && ks == 0) {
    const float m0 = stat[(2 * w) * 64 + lane], l0 = stat[(2 * w + 1) * 64 + lane];
    const float m1 = stat[(2 * (w + 2)) * 64 + lane], l1 = stat[(2 * (w + 2) + 1) * 64 + lane];
    const float m = fmaxf(m0, m1);
    const float w0 = __builtin_amdgcn_exp2f(m0 - m), w1 = __builtin_amdgcn_exp2f(m1 - m);
    const float l = l0 * w0 + l1 * w1;
    const float inv = P.keep_scale / l;
    acc_combine<DT>(mg, oacc, w0, w1, lane);
    if (i < P.s && hh == 0) lse[(size_t)bn * P.s + i] = (m + __builtin_amdgcn_logf(l)) * kLn2;
    acc_to_lds_rows<DT>(smem + 2 * TILE, KP, 32 * rg + li, oacc, inv, hh);  // behind the exchange buffers and the statistics
  }
  __syncthreads();
  if (tid < 256) lds_rows_to_global<D>(smem + 2 * TILE, o + base + (int64_t)(rb * BM) * P.stride_s, gstride, P.s - rb * BM, tid);
}

}  // namespace sar
