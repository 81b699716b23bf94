// bf16 attention core, forward with tile-fetching waves (included by attn_mfma_rows.hip, which documents the tile layouts and
// the step), in its persistent form: fewer workgroups than row blocks, each working through a fixed list of them.
//
// Why: a workgroup spends about 2.4 us before its first step (Q operands and the first K tile on their way from memory,
// the first Philox words, the first scores) and 1.6 us after its last one, and a CU runs two or more workgroups one after
// the other (LDS allows one at a time): at s = 2048 a quarter of the kernel's time.  Here the next row block's Q operands,
// first Philox words and first K / V tiles are requested during the last step of the current one (its registers for Q
// and the Philox words, both K stages and one V stage are idle then) and land while the epilogue runs in LDS buffers of
// its own.
//
// Work list: the grid is R x N workgroups (N = b x heads, R row blocks of each head at a time, R x N <= number of CUs);
// workgroup (wq, head) takes, of its head's row blocks ranked heaviest first, rank wq, 2R-1-wq, 2R+wq, 4R-1-wq, ...: a
// heavy block is followed by a light one, all blocks of a head stay on the workgroups (and, with heads dealt round-robin
// to the XCDs, on the L2) that work on that head.
#pragma once
#include "attn_mfma_common.h"

namespace sar {

template <int D, bool DROP>
__global__ __launch_bounds__(512) void attn_fwd_pers_kernel(AttnParams P, const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
                                                             const uint16_t* __restrict__ v, uint16_t* __restrict__ o, float* __restrict__ lse) {
  constexpr int BM = 64, BN = 64, KP = D + 8, KC = D / 16, DT = D / 32;
  constexpr int TILE = BN * KP;
  constexpr float kRescale = 60.0f;  // the running reference exponent moves only when the row maximum grew by > 2^60
  constexpr int MGW = 64 * (16 * DT + 4);  // floats per row group in the merge buffer: DT accumulator tiles, (m, l) of both key halves
  __shared__ __attribute__((aligned(16))) uint16_t smem[4 * TILE];
  __shared__ __attribute__((aligned(16))) float mgbuf[2 * MGW];     // the epilogue's buffers: partial outputs and statistics of the upper key half
  __shared__ __attribute__((aligned(16))) uint16_t otile[TILE];     // ... and the output tile on its way to memory
  uint16_t* Kst = smem;             // K tile jt of a row block lives in Kst + (jt & 1) * TILE
  uint16_t* Vst = smem + 2 * TILE;  // V tile jt lives in Vst + ((jt + voff) & 1) * TILE, voff per row block

  const int N = P.b * P.A;
  const int nrb = (P.s + BM - 1) / BM;
  const int R = (int)gridDim.x / N;
  const int wq = (int)blockIdx.x / N;
  const int bn = blockIdx.x % N, beta = bn / P.A, n = bn % P.A;
  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, li = lane & 31, hh = lane >> 5;
  const int64_t base = (int64_t)beta * P.stride_b + (int64_t)n * P.stride_a;
  const int gstride = (int)P.stride_s;
  // rank (0 = heaviest = last row block) of this workgroup's j-th row block; >= nrb: the list has ended
  auto rank_of = [&](const int j) __attribute__((always_inline)) { return (j & 1) ? (j + 1) * R - 1 - wq : j * R + wq; };
  auto tiles_of = [&](const int rb) __attribute__((always_inline)) {
    const int last_row = min(rb * BM + BM - 1, P.s - 1);
    return P.causal ? last_row / BN + 1 : (P.s + BN - 1) / BN;
  };

  if (wave >= 4) {  // a loader (one per SIMD): same barriers as the others
    const int lw = wave - 4;
    constexpr int C1 = DmaMap<D, 4>::PER - 1;  // a tile is at least this many loads of a wave
    DmaMap<D, 4> lmap;
    lmap.init(lw, lane, gstride, true);
    auto fetch = [&](const uint16_t* g, uint16_t* stage, const int jt) __attribute__((always_inline)) {
      const int left = P.s - jt * BN;
      if (left >= BN) dma_tile<D>(lmap, g + (int64_t)(jt * BN) * gstride, stage, lw);
      else dma_tile_ragged<D>(lmap, g + (int64_t)(jt * BN) * gstride, stage, lw, lane, gstride, left);
    };
    int j = 0, voff = 0;
    int nt = tiles_of(nrb - 1 - rank_of(0));
    fetch(k + base, Kst, 0);
    fetch(v + base, Vst, 0);
    if (nt > 1) fetch(k + base, Kst + TILE, 1);
    for (;;) {
      // the first scores need K tile 0 only: the loads of the one or two tiles issued after it may still be in flight
      if (nt > 1) dma_wait_keep<2 * C1>();
      else dma_wait_keep<C1>();
      __syncthreads();  // K tile 0 is there
      dma_wait();       // V tile 0 and K tile 1, before the first step's barrier
      const int rank_n = rank_of(j + 1);
      const bool has_next = rank_n < nrb;
      const int nt_n = has_next ? tiles_of(nrb - 1 - rank_n) : 0;
      for (int jt = 0; jt < nt; ++jt) {
        __syncthreads();  // top of step jt: K tile jt and V tile jt-1 are free
        if (jt + 2 < nt) fetch(k + base, Kst + (jt & 1) * TILE, jt + 2);
        if (jt + 1 < nt) fetch(v + base, Vst + ((jt + 1 + voff) & 1) * TILE, jt + 1);
        if (jt + 1 < nt) {
          dma_wait();
        } else if (has_next) {
          // the last step reads V tile nt-1 only: both K stages and the other V stage take the next row block's first tiles,
          // which have until that block's first barrier (after this block's epilogue) to land
          fetch(k + base, Kst, 0);
          fetch(v + base, Vst + ((nt + voff) & 1) * TILE, 0);
          if (nt_n > 1) fetch(k + base, Kst + TILE, 1);
        }
      }
      __syncthreads();  // the two barriers of the others' epilogue
      __syncthreads();
      if (!has_next) break;
      voff = (nt + voff) & 1;
      nt = nt_n;
      ++j;
    }
    return;
  }

  const int rg = wave & 1, ks = wave >> 1;
  const float sc2 = P.scale * kLog2e;
  const uint64_t headG = P.offset + (((uint64_t)beta * (uint64_t)P.a_global + (uint64_t)(P.head0 + n)) * (uint64_t)P.s) * (uint64_t)(P.s >> 3);
  // per row block
  int rb = nrb - 1 - rank_of(0);
  int nt = tiles_of(rb);
  int i = rb * BM + rg * 32 + li;                  // this lane's query row
  int i_ld = i < P.s ? i : P.s - 1;
  int jlim = P.causal ? i : P.s - 1;               // last key row i attends to
  uint64_t rowG = headG + (uint64_t)i_ld * (uint64_t)(P.s >> 3);  // Philox call index of (row i, key 0)
  int voff = 0;

  bf16x8_t qf[KC];
#pragma unroll
  for (int kc = 0; kc < KC; ++kc) qf[kc] = ld_frag(q + base + (int64_t)i_ld * P.stride_s + 16 * kc + 8 * hh);
#pragma unroll
  for (int kc = 0; kc < KC; ++kc) asm volatile("" : "+v"(qf[kc]));

  float16_t oacc[DT];
  float l_run = 0.f, m_ref = 0.f;
  float16_t st;

  auto scores = [&](const int jt, auto diag) __attribute__((always_inline)) {
    const uint16_t* Ks = Kst + (jt & 1) * TILE;
    float16_t s0;
#pragma unroll
    for (int e = 0; e < 16; ++e) s0[e] = 0.f;
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) s0 = mfma32(ld_frag(Ks + (32 * ks + li) * KP + 16 * kc + 8 * hh), qf[kc], s0);
    if (decltype(diag)::value) {
      const int j0w = jt * BN + 32 * ks;
#pragma unroll
      for (int e = 0; e < 16; ++e)
        if (j0w + 16 * (e >> 3) + 8 * hh + (e & 7) > jlim) s0[e] = -INFINITY;
    }
    return s0;
  };
  auto tile_max = [&](const float16_t& t) __attribute__((always_inline)) {
    float mt = fmaxf(fmaxf(t[0], t[1]), t[2]);
#pragma unroll
    for (int e = 3; e < 15; e += 2) mt = fmaxf(fmaxf(mt, t[e]), t[e + 1]);
    mt = fmaxf(mt, t[15]);
    return fmaxf(xhalf_max(mt) * sc2, -1.0e30f);
  };
  Philox4 rnd[2] = {{0u, 0u, 0u, 0u}, {0u, 0u, 0u, 0u}};
  auto philox_begin = [&](Philox4 (&r)[2], const uint64_t row, const int jt) __attribute__((always_inline)) {
#pragma unroll
    for (int c = 0; c < 2; ++c) r[c] = philox_start(row + (uint64_t)((jt * BN + 32 * ks + 16 * c + 8 * hh) >> 3), 0u);
  };
  if (DROP) {
    philox_begin(rnd, rowG, 0);
#pragma unroll
    for (int r = 0; r < 10; ++r) {
      philox_round(rnd[0], P.key0, P.key1, r);
      philox_round(rnd[1], P.key0, P.key1, r);
    }
  }

  // what the last step of a row block prepares for the next one
  bool has_next = false;
  int rb_n = 0, i_ld_n = 0;
  uint64_t rowG_n = 0;

  // One step (see the step of attn_fwd_mfma_kernel).  NEXT != 0: there is a tile jt+1; NEXT == 2: it is the diagonal one;
  // NEXT == 0: the row block's last step, which requests the next row block's Q operands and draws its first Philox words.
  auto step = [&](const int jt, auto next) __attribute__((always_inline)) {
    constexpr int NEXT = decltype(next)::value;
    constexpr int kAhead = 3, NPV = 2 * DT;
    __syncthreads();  // K tile jt+1 and V tile jt are there; nobody reads K tile jt or V tile jt-1 any more
    if (NEXT == 0) {
      if (has_next) {
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) qf[kc] = ld_frag(q + base + (int64_t)i_ld_n * P.stride_s + 16 * kc + 8 * hh);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    const uint16_t* Ksn = Kst + ((jt + 1) & 1) * TILE + (32 * ks + li) * KP + 8 * hh;
    const uint16_t* Vs = Vst + ((jt + voff) & 1) * TILE;
    float16_t stn;
#pragma unroll
    for (int e = 0; e < 16; ++e) stn[e] = 0.f;
    bf16x8_t kfr[kAhead], vfr[kAhead];
    if (NEXT != 0) {
#pragma unroll
      for (int a = 0; a < kAhead && a < KC; ++a) kfr[a] = ld_frag(Ksn + 16 * a);
    }
    auto v_frag = [&](const int idx) __attribute__((always_inline)) {
      return ld_frag_tr_perm(Vs, KP, 32 * ks + 16 * (idx / DT), 32 * (idx % DT), lane);
    };
    float psum = 0.f;
    float pd[16];
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) {
      if (NEXT != 0) {
        stn = mfma32(kfr[kc % kAhead], qf[kc], stn);
        if (kc + kAhead < KC) kfr[kc % kAhead] = ld_frag(Ksn + 16 * (kc + kAhead));
      }
      if (kc >= KC - kAhead && kc - (KC - kAhead) < NPV) vfr[kc - (KC - kAhead)] = v_frag(kc - (KC - kAhead));
#pragma unroll
      for (int e = (16 * kc) / KC; e < (16 * (kc + 1)) / KC; ++e) {
        const float pe = __builtin_amdgcn_exp2f(fmaf(st[e], sc2, -m_ref));
        psum += pe;
        pd[e] = (!DROP || keep_field(rnd[e >> 3], e & 7, P.thresh)) ? pe : 0.f;
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    l_run += psum;
    bf16x8_t pf[2];
    pf[0] = pack8(pd);
    pf[1] = pack8(pd + 8);
    Philox4 rn[2] = {{0u, 0u, 0u, 0u}, {0u, 0u, 0u, 0u}};
    if (DROP) {
      if (NEXT != 0) philox_begin(rn, rowG, jt + 1);
      else philox_begin(rn, rowG_n, 0);  // (drawn in vain after the last row block)
    }
    __builtin_amdgcn_sched_barrier(0);
    float mt = 0.f;
#pragma unroll
    for (int idx = 0; idx < NPV; ++idx) {
      oacc[idx % DT] = mfma32(vfr[idx % kAhead], pf[idx / DT], oacc[idx % DT]);
      if (idx + kAhead < NPV) vfr[idx % kAhead] = v_frag(idx + kAhead);
      if (NEXT == 2 && idx == 1) {  // the diagonal tile: keys beyond jlim are masked
        const int j0n = (jt + 1) * BN + 32 * ks;
#pragma unroll
        for (int e = 0; e < 16; ++e)
          if (j0n + 16 * (e >> 3) + 8 * hh + (e & 7) > jlim) stn[e] = -INFINITY;
      }
      if (NEXT != 0 && idx == 2) mt = tile_max(stn);
      if (DROP) {
#pragma unroll
        for (int u = (20 * idx) / NPV; u < (20 * (idx + 1)) / NPV; ++u) philox_round(rn[u & 1], P.key0, P.key1, u >> 1);
#pragma unroll
        for (int c = 0; c < 2; ++c) asm volatile("" : "+v"(rn[c].x), "+v"(rn[c].y), "+v"(rn[c].z), "+v"(rn[c].w));
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    rnd[0] = rn[0];
    rnd[1] = rn[1];
    if (NEXT != 0) {
      st = stn;
      if (__builtin_expect(__builtin_amdgcn_ballot_w64(mt > m_ref + kRescale) != 0, 0)) {
        const float m_new = fmaxf(m_ref, mt);
        const float corr = __builtin_amdgcn_exp2f(m_ref - m_new);
        m_ref = m_new;
        l_run *= corr;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
          for (int e = 0; e < 16; ++e) oacc[dt][e] *= corr;
      }
    }
  };

  for (int j = 0;; ++j) {
    {
      const int rank_n = rank_of(j + 1);
      has_next = rank_n < nrb;
      rb_n = has_next ? nrb - 1 - rank_n : rb;
      const int i_n = rb_n * BM + rg * 32 + li;
      i_ld_n = i_n < P.s ? i_n : P.s - 1;
      rowG_n = headG + (uint64_t)i_ld_n * (uint64_t)(P.s >> 3);
    }
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int e = 0; e < 16; ++e) oacc[dt][e] = 0.f;
    l_run = 0.f;
    __syncthreads();  // K tile 0 is there
    st = nt == 1 ? scores(0, std::true_type{}) : scores(0, std::false_type{});
    m_ref = tile_max(st);
    {
      int jt = 0;
      for (; jt + 2 < nt; ++jt) step(jt, std::integral_constant<int, 1>{});
      if (jt + 1 < nt) step(jt++, std::integral_constant<int, 2>{});
      step(jt++, std::integral_constant<int, 0>{});
    }
    // ---- merge the two key halves of each row group, then O = O^T^T / ((1-p) l), LSE = m + ln l ----
    // (the merge buffer and the output tile are touched by nothing else: no barrier between the last step and the hand-over; the
    // row block before this one left them two barriers and a whole tile loop ago)
    // Both waves of a row group work in both phases: the lower key half (ks = 0) hands over its accumulator tiles DH .. DT-1
    // and finishes tiles 0 .. DH-1, the upper half the other way round; each leaves its statistics for the other.
    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    float* mg = mgbuf + rg * MGW;
    constexpr int DH = (DT + 1) / 2;
    {
      f32x4_t* bq = reinterpret_cast<f32x4_t*>(mg) + lane;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
        if ((dt < DH) == (ks == 1)) {
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const f32x4_t t4 = {oacc[dt][4 * g], oacc[dt][4 * g + 1], oacc[dt][4 * g + 2], oacc[dt][4 * g + 3]};
            bq[(4 * dt + g) * 64] = t4;
          }
        }
      mg[(16 * DT) * 64 + 128 * ks + lane] = m_ref;
      mg[(16 * DT) * 64 + 128 * ks + 64 + lane] = l_tot;
    }
    __syncthreads();
    {
      const float mo = mg[(16 * DT) * 64 + 128 * (1 - ks) + lane], lo = mg[(16 * DT) * 64 + 128 * (1 - ks) + 64 + lane];
      const float m0 = ks ? mo : m_ref, m1 = ks ? m_ref : mo, l0 = ks ? lo : l_tot, l1 = ks ? l_tot : lo;
      const float m = fmaxf(m0, m1);
      const float w0 = __builtin_amdgcn_exp2f(m0 - m), w1 = __builtin_amdgcn_exp2f(m1 - m);
      const float l = l0 * w0 + l1 * w1;
      const float inv = P.keep_scale / l;
      const float wown = ks ? w1 : w0, woth = ks ? w0 : w1;
      const f32x4_t* bq = reinterpret_cast<const f32x4_t*>(mg) + lane;
      uint16_t* orow = otile + (32 * rg + li) * KP + 4 * hh;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
        if ((dt < DH) == (ks == 0)) {
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const f32x4_t t4 = bq[(4 * dt + g) * 64];
            float r4[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) r4[r] = (oacc[dt][4 * g + r] * wown + t4[r] * woth) * inv;
            uint2 w2;
            w2.x = pack_bf16x2(r4[0], r4[1]);
            w2.y = pack_bf16x2(r4[2], r4[3]);
            *reinterpret_cast<uint2*>(orow + 32 * dt + 8 * g) = w2;
          }
        }
      if (ks == 0 && i < P.s && hh == 0) lse[(size_t)bn * P.s + i] = (m + __builtin_amdgcn_logf(l)) * kLn2;
    }
    __syncthreads();
    {
      // the copy's per-thread row / column offsets are recomputed for every row block on purpose: kept across the tile loop they
      // do not fit the register file, and reloading spilled ones costs a memory round trip each
      int t = tid;
      asm volatile("" : "+v"(t));
      lds_rows_to_global<D>(otile, o + base + (int64_t)(rb * BM) * P.stride_s, gstride, P.s - rb * BM, t);
    }
    if (!has_next) break;
    voff = (nt + voff) & 1;
    rb = rb_n;
    nt = tiles_of(rb);
    i = rb * BM + rg * 32 + li;
    i_ld = i_ld_n;
    jlim = P.causal ? i : P.s - 1;
    rowG = rowG_n;
  }
}

}  // namespace sar
