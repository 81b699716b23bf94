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
#include <atomic>
#include <type_traits>
#include "attn_mfma_fwd_split.h"
#include "attn_mfma_fwd_pers.h"

namespace sar {

static constexpr float kLazyRescale = 60.0f;  // the running reference exponent moves only when the row maximum grew by > 2^60

// ===================================================================================================
// Forward.  Workgroup = 32 NRG query rows, 2 NRG waves: wave = (rg, ks), rg = 32-row group, ks = which 32 keys of
// each 64-key tile.  NRG = 2: 64 rows, one wave per SIMD.  NRG = 4: 128 rows, two waves per SIMD, a K / V tile
// serves twice the rows (half the tile bytes through the L1 per unit of work); under the causal mask the two lower
// row groups stop one tile before the two upper ones.
// K and V tiles (both with swapped rows) go from global memory straight into LDS, two stages each.
// The score tile and the Philox words run one step ahead of the rest: step j computes S_{j+1} between the exponentials and
// keep decisions of tile j, then P_j V_j between the Philox rounds, the mask and the row maximum of tile j+1 (the order
// is laid out by hand, see the step).  A wave issues in order, so a step costs the sum of its instructions' issue times
// whichever pipe executes them: measured at d = 160 per 64 x 64 step, 1700 cycles = ~1130 of vector instructions
// (16 exponentials at quarter rate are 256 of them, two Philox calls 320) + ~240 for issuing 20 matrix instructions +
// ~260 for 30 LDS reads + ~80 at the barrier; with the vector work removed the first half takes 562 cycles, with the
// matrix work and its reads removed 627, both together 946.  The (rare) rescaling of the running maximum for tile j+1
// is decided at the end of step j.
// ===================================================================================================
// DROP = false is the p = 0 variant: no random numbers are drawn at all.
// LW (64-row workgroups only): four more waves, one per SIMD, that do nothing but fetch the K / V tiles.  A wave-wide
// 16-byte load occupies its wave for about 64 cycles (16 bytes per cycle per SIMD; four SIMDs are the CU's 64 B/clk), so
// 42 loads per step cost each computing wave some 650 cycles of a 2200-cycle step; in a wave of their own those cycles
// run beside the arithmetic of the SIMD's other wave.  The price: every wave must fit half the register file.
template <int D, bool DROP, int NRG, bool LW = false>
__global__ __launch_bounds__(128 * NRG + (LW ? 256 : 0)) void attn_fwd_mfma_kernel(AttnParams P, const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
                                                           const uint16_t* __restrict__ v, uint16_t* __restrict__ o, float* __restrict__ lse) {
  constexpr int BM = 32 * NRG, BN = 64, KP = D + 8, KC = D / 16, DT = D / 32, NW = 2 * NRG;
  constexpr int TILE = BN * KP;
  __shared__ __attribute__((aligned(16))) uint16_t smem[4 * TILE];
  uint16_t* Kst = smem;             // K tile jt lives in Kst + (jt & 1) * TILE
  uint16_t* Vst = smem + 2 * TILE;  // V tile jt lives in Vst + (jt & 1) * TILE

  const int N = P.b * P.A;
  const int nrb = (P.s + BM - 1) / BM;
  const int rb = nrb - 1 - (int)(blockIdx.x / N);  // heaviest row blocks first
  const int bn = blockIdx.x % N, beta = bn / P.A, n = bn % P.A;
  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, li = lane & 31, hh = lane >> 5;
  const int rg = wave % NRG, ks = wave / NRG;
  const int64_t base = (int64_t)beta * P.stride_b + (int64_t)n * P.stride_a;
  const int gstride = (int)P.stride_s;
  if constexpr (LW) {
    static_assert(NRG == 2, "the loader wave goes with 64-row workgroups");
    if (wave >= NW) {  // a loader (one per SIMD): same barriers as the others
      const int lw = wave - NW;
      const int last_row_l = min(rb * BM + BM - 1, P.s - 1);
      const int nt = P.causal ? last_row_l / BN + 1 : (P.s + BN - 1) / BN;
      DmaMap<D, 4> lmap;
      lmap.init(lw, lane, gstride, true);
      auto fetch = [&](const uint16_t* g, uint16_t* st2, int jt) __attribute__((always_inline)) {
        const int left = P.s - jt * BN;
        if (left >= BN) dma_tile<D>(lmap, g + (int64_t)(jt * BN) * gstride, st2 + (jt & 1) * TILE, lw);
        else dma_tile_ragged<D>(lmap, g + (int64_t)(jt * BN) * gstride, st2 + (jt & 1) * TILE, lw, lane, gstride, left);
      };
      fetch(k + base, Kst, 0);
      fetch(v + base, Vst, 0);
      if (nt > 1) fetch(k + base, Kst, 1);
      // the first scores need K tile 0 only: the loads of the one or two tiles issued after it (at least PER - 1 per wave and
      // tile) may still be in flight at the first barrier
      if (nt > 1) dma_wait_keep<2 * (DmaMap<D, 4>::PER - 1)>();
      else dma_wait_keep<DmaMap<D, 4>::PER - 1>();
      __syncthreads();  // K tile 0 is there
      dma_wait();       // V tile 0 and K tile 1, before the first step's barrier
      for (int jt = 0; jt < nt; ++jt) {
        __syncthreads();  // top of step jt: K tile jt and V tile jt-1 are free
        if (jt + 2 < nt) fetch(k + base, Kst, jt + 2);
        if (jt + 1 < nt) fetch(v + base, Vst, jt + 1);
        dma_wait();
      }
      __syncthreads();  // the three barriers of the others' epilogue
      __syncthreads();
      __syncthreads();
      return;
    }
  }
  const int iw0 = rb * BM + rg * 32;  // first row of this wave
  const int i = iw0 + li;
  const int i_ld = i < P.s ? i : P.s - 1;
  const int jlim = P.causal ? i : P.s - 1;  // last key row i attends to

  bf16x8_t qf[KC];
#pragma unroll
  for (int kc = 0; kc < KC; ++kc) qf[kc] = ld_frag(q + base + (int64_t)i_ld * P.stride_s + 16 * kc + 8 * hh);
  // These must have arrived before the tile loop: a wait left inside the loop would also wait for the direct
  // loads in flight there, which the compiler does not know about.
#pragma unroll
  for (int kc = 0; kc < KC; ++kc) asm volatile("" : "+v"(qf[kc]));

  // Philox call index of (row i, key 0): offset + e/8 with e = ((beta*a + head)*s + i)*s
  const uint64_t rowG = P.offset + (((uint64_t)beta * (uint64_t)P.a_global + (uint64_t)(P.head0 + n)) * (uint64_t)P.s + (uint64_t)i_ld) * (uint64_t)(P.s >> 3);

  float16_t oacc[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int e = 0; e < 16; ++e) oacc[dt][e] = 0.f;
  float l_run = 0.f;
  const float sc2 = P.scale * kLog2e;

  const int last_row = min(rb * BM + BM - 1, P.s - 1);
  const int ntile = P.causal ? last_row / BN + 1 : (P.s + BN - 1) / BN;  // tiles the workgroup streams
  // tiles this wave has rows for: the two lower row groups stop one tile before the two upper ones under the causal
  // mask; a wave's last tile is the only one that needs a mask
  const int nt_w = (NRG > 2 && P.causal) ? min(iw0 + 31, P.s - 1) / BN + 1 : ntile;
  DmaMap<D, NW> map;
  map.init(wave, lane, gstride, true);
  const uint16_t* kg = k + base;
  const uint16_t* vg = v + base;
  auto load_tile = [&](const uint16_t* g, uint16_t* st2, int jt) __attribute__((always_inline)) {
    const int left = P.s - jt * BN;  // only the last tile of the sequence can end before its 64th row
    if (left >= BN) dma_tile<D>(map, g + (int64_t)(jt * BN) * gstride, st2 + (jt & 1) * TILE, wave);
    else dma_tile_ragged<D>(map, g + (int64_t)(jt * BN) * gstride, st2 + (jt & 1) * TILE, wave, lane, gstride, left);
  };
  // S^T tile of this wave's 32 keys of tile jt against its 32 rows; st[8*c + e] is the score of key
  // jt*64 + 32*ks + 16*c + 8*hh + e.  DIAG: the last tile of the row block: keys beyond jlim (above the diagonal, or past the end) are masked.
  auto scores = [&](const int jt, auto diag) __attribute__((always_inline)) {
    const uint16_t* Ks = Kst + (jt & 1) * TILE;
    float16_t st;
#pragma unroll
    for (int e = 0; e < 16; ++e) st[e] = 0.f;
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) st = mfma32(ld_frag(Ks + (32 * ks + li) * KP + 16 * kc + 8 * hh), qf[kc], st);
    if (decltype(diag)::value) {
      const int j0w = jt * BN + 32 * ks;
#pragma unroll
      for (int e = 0; e < 16; ++e)
        if (j0w + 16 * (e >> 3) + 8 * hh + (e & 7) > jlim) st[e] = -INFINITY;
    }
    return st;
  };
  // row maximum of a score tile in the softmax's units (alpha*log2(e)*score; alpha > 0), floored so that a fully
  // masked tile (the upper wave of the first row group on the diagonal) stays finite
  auto tile_max = [&](const float16_t& st) __attribute__((always_inline)) {
    float mt = fmaxf(fmaxf(st[0], st[1]), st[2]);
#pragma unroll
    for (int e = 3; e < 15; e += 2) mt = fmaxf(fmaxf(mt, st[e]), st[e + 1]);
    mt = fmaxf(mt, st[15]);
    return fmaxf(xhalf_max(mt) * sc2, -1.0e30f);
  };

  if constexpr (!LW) {
    load_tile(kg, Kst, 0);
    load_tile(vg, Vst, 0);
    if (ntile > 1) load_tile(kg, Kst, 1);
  }
  // Philox words of the tile whose probabilities are formed next: rnd[c] covers this lane's keys 16 c + 8 hh .. + 7 of
  // its wave's half of the tile.  They do not depend on the scores, so they are drawn one step ahead (the first tile's while the first K / V tiles are on
  // their way).
  Philox4 rnd[2] = {{0u, 0u, 0u, 0u}, {0u, 0u, 0u, 0u}};
  auto philox_begin = [&](Philox4 (&r)[2], const int jt) __attribute__((always_inline)) {
#pragma unroll
    for (int c = 0; c < 2; ++c) r[c] = philox_start(rowG + (uint64_t)((jt * BN + 32 * ks + 16 * c + 8 * hh) >> 3), 0u);
  };
  if (DROP) {
    philox_begin(rnd, 0);
#pragma unroll
    for (int r = 0; r < 10; ++r) {
      philox_round(rnd[0], P.key0, P.key1, r);
      philox_round(rnd[1], P.key0, P.key1, r);
    }
  }

  if constexpr (!LW) dma_wait();
  __syncthreads();
  float16_t st = nt_w == 1 ? scores(0, std::true_type{}) : scores(0, std::false_type{});
  float m_ref = tile_max(st);

  // One step, laid out by hand in two halves so that the matrix pipe and the vector pipe of the SIMD run side by side
  // (the scheduler left to itself puts most of the vector work between the two groups of matrix instructions):
  //   first half : the KC matrix instructions of the scores of tile jt+1 (K operands read kAhead instructions ahead), and
  //                between them tile jt's exponentials, keep decisions and sums, dealt out evenly;
  //   second half: the 2 DT matrix instructions of O^T += V^T P^T for tile jt (V^T operands read kAhead ahead), and
  //                between them the twenty Philox rounds (two calls) of tile jt+1.
  // NEXT != 0: there is a tile jt+1; NEXT == 2: it is the diagonal one.
  auto step = [&](const int jt, auto next) __attribute__((always_inline)) {
    constexpr int NEXT = decltype(next)::value;
    constexpr int kAhead = 3, NPV = 2 * DT;
    if constexpr (!LW) dma_wait();  // this wave's loads of K tile jt+1 and V tile jt have landed
    __syncthreads();                // ... and everybody's; nobody reads K tile jt or V tile jt-1 any more
    if constexpr (!LW) {
      if (jt + 2 < ntile) load_tile(kg, Kst, jt + 2);
      if (jt + 1 < ntile) load_tile(vg, Vst, jt + 1);
    }
    const uint16_t* Ksn = Kst + ((jt + 1) & 1) * TILE + (32 * ks + li) * KP + 8 * hh;
    const uint16_t* Vs = Vst + (jt & 1) * TILE;
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
    if (DROP && NEXT != 0) philox_begin(rn, jt + 1);
    __builtin_amdgcn_sched_barrier(0);
    // ---- O^T += V^T P^T; beside it the next tile's mask, maximum and Philox rounds ----
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
      if (DROP && NEXT != 0) {
#pragma unroll
        for (int u = (20 * idx) / NPV; u < (20 * (idx + 1)) / NPV; ++u) philox_round(rn[u & 1], P.key0, P.key1, u >> 1);
        // the words are next needed in the following step: without a use here the rounds sink below the matrix instructions
#pragma unroll
        for (int c = 0; c < 2; ++c) asm volatile("" : "+v"(rn[c].x), "+v"(rn[c].y), "+v"(rn[c].z), "+v"(rn[c].w));
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    if (NEXT != 0) {
      st = stn;
      rnd[0] = rn[0];
      rnd[1] = rn[1];
      // the running reference exponent only moves when the next tile's maximum exceeds it by more than 2^60
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
    }
  };
  {
    int jt = 0;
    for (; jt + 2 < nt_w; ++jt) step(jt, std::integral_constant<int, 1>{});
    if (jt + 1 < nt_w) step(jt++, std::integral_constant<int, 2>{});
    step(jt++, std::integral_constant<int, 0>{});
    if constexpr (NRG > 2)
      for (; jt < ntile; ++jt) {  // a tile above this wave's rows: keep pace with the workgroup's barriers and loads
        dma_wait();
        __syncthreads();
        if (jt + 2 < ntile) load_tile(kg, Kst, jt + 2);
        if (jt + 1 < ntile) load_tile(vg, Vst, jt + 1);
      }
  }

  // ---- merge the two key halves of each row group, then O = O^T^T / ((1-p) l), LSE = m + ln l ----
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  __syncthreads();
  float* mg = reinterpret_cast<float*>(smem) + rg * (64 * (16 * DT + 2));
  if (ks == 1) {
    acc_put<DT>(mg, oacc, lane);
    mg[(16 * DT) * 64 + lane] = m_ref;
    mg[(16 * DT + 1) * 64 + lane] = l_tot;
  }
  __syncthreads();
  float inv = 0.f;
  if (ks == 0) {
    const float m1 = mg[(16 * DT) * 64 + lane], l1 = mg[(16 * DT + 1) * 64 + lane];
    const float m = fmaxf(m_ref, m1);
    const float w0 = __builtin_amdgcn_exp2f(m_ref - m), w1 = __builtin_amdgcn_exp2f(m1 - m);
    const float l = l_tot * w0 + l1 * w1;
    inv = P.keep_scale / l;
    acc_combine<DT>(mg, oacc, w0, w1, lane);
    if (i < P.s && hh == 0) lse[(size_t)bn * P.s + i] = (m + __builtin_amdgcn_logf(l)) * kLn2;
  }
  if constexpr (NRG == 2) {  // 64 rows: the output tile sits behind the exchange buffers
    if (ks == 0) acc_to_lds_rows<DT>(smem + 2 * TILE, KP, 32 * rg + li, oacc, inv, hh);
    __syncthreads();
    lds_rows_to_global<D>(smem + 2 * TILE, o + base + (int64_t)(rb * BM) * P.stride_s, gstride, P.s - rb * BM, tid);
  } else {  // 128 rows: two output tiles that overlap the exchange buffers
    __syncthreads();
    if (ks == 0) acc_to_lds_rows<DT>(smem + (rg >> 1) * TILE, KP, 32 * (rg & 1) + li, oacc, inv, hh);
    __syncthreads();
    const int half = tid >> 8;  // threads 0..255 copy rows 0..63 out, threads 256..511 rows 64..127
    lds_rows_to_global<D>(smem + half * TILE, o + base + (int64_t)(rb * BM + 64 * half) * P.stride_s, gstride, P.s - rb * BM - 64 * half, tid & 255);
  }
}

// ===================================================================================================
// Backward, row-stationary pass: delta_i = dO_i . O_i and dQ_i = alpha sum_j dS_ij K_j, with
// P_ij = exp(alpha q_i.k_j - LSE_i), dP = (dO V^T) o M/(1-p), dS = P o (dP - delta) recomputed per tile.
// Same workgroup shape as the forward.
// ===================================================================================================
// LW: four more waves that fetch the tiles, as in the forward.  Its Q / dO operands are pinned in vector registers, not
// accumulation registers: a kernel that uses none of the latter gets all 256 registers of a wave as vector registers
// (253 used at d = 160, no spills), otherwise the file is split 128 + 128 and the arithmetic is squeezed into half.
template <int D, bool DROP, bool LW = false>
__global__ __launch_bounds__(LW ? 512 : 256) void attn_bwd_dq_mfma_kernel(AttnParams P, const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
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
  if constexpr (LW) {
    if (wave >= 4) {  // a loader (one per SIMD): same barriers as the others
      const int lw = wave - 4;
      const int last_row_l = min(rb * BM + BM - 1, P.s - 1);
      const int nt = P.causal ? last_row_l / BN + 1 : (P.s + BN - 1) / BN;
      DmaMap<D> lmap;
      lmap.init(lw, lane, gstride, true);
      auto fetch = [&](int jt) __attribute__((always_inline)) {
        uint16_t* st2 = smem + (jt & 1) * 2 * TILE;
        const int left = P.s - jt * BN;
        if (left >= BN) {
          dma_tile<D>(lmap, k + base + (int64_t)(jt * BN) * gstride, st2, lw);
          dma_tile<D>(lmap, v + base + (int64_t)(jt * BN) * gstride, st2 + TILE, lw);
        } else {
          dma_tile_ragged<D>(lmap, k + base + (int64_t)(jt * BN) * gstride, st2, lw, lane, gstride, left);
          dma_tile_ragged<D>(lmap, v + base + (int64_t)(jt * BN) * gstride, st2 + TILE, lw, lane, gstride, left);
        }
      };
      fetch(0);
      for (int jt = 0; jt < nt; ++jt) {
        dma_wait();
        __syncthreads();  // top of step jt: tile jt is there, the other stage is free
        if (jt + 1 < nt) fetch(jt + 1);
      }
      __syncthreads();  // the three barriers of the others' epilogue
      __syncthreads();
      __syncthreads();
      return;
    }
  }
  const int iw0 = rb * BM + rg * 32;
  const int i = iw0 + li;
  const int i_ld = i < P.s ? i : P.s - 1;
  const int jlim = P.causal ? i : P.s - 1;                     // last key row i attends to
  const int lim_lo = P.causal ? iw0 : P.s - 1, lim_hi = P.causal ? iw0 + 31 : P.s - 1;  // its range over the wave's rows

  bf16x8_t qf[KC], dof[KC];
  float dpart = 0.f;
#pragma unroll
  for (int kc = 0; kc < KC; ++kc) {
    const int64_t off = base + (int64_t)i_ld * P.stride_s + 16 * kc + 8 * hh;
    qf[kc] = ld_frag(q + off);
    dof[kc] = ld_frag(dO + off);
    dpart += dot8(dof[kc], ld_frag(o + off));
  }
  // These must have arrived before the tile loop: a wait left inside the loop would also wait for the direct
  // loads in flight there, which the compiler does not know about.
#pragma unroll
  for (int kc = 0; kc < KC; ++kc) {
    if constexpr (LW) asm volatile("" : "+v"(qf[kc]), "+v"(dof[kc]));  // two waves per SIMD: no accumulation registers, so that all 256 are vector registers
    else asm volatile("" : "+a"(qf[kc]), "+a"(dof[kc]));
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
  const int ntile = P.causal ? last_row / BN + 1 : (P.s + BN - 1) / BN;
  DmaMap<D> map;
  map.init(wave, lane, gstride, true);
  const uint16_t* kg = k + base;
  const uint16_t* vg = v + base;
  if constexpr (!LW) {
    if (P.s >= BN) {
      dma_tile<D>(map, kg, smem, wave);
      dma_tile<D>(map, vg, smem + TILE, wave);
    } else {
      dma_tile_ragged<D>(map, kg, smem, wave, lane, gstride, P.s);
      dma_tile_ragged<D>(map, vg, smem + TILE, wave, lane, gstride, P.s);
    }
  }
  // One tile step.  MODE says how tile jt+1 is loaded into the other stage meanwhile: 0 = there is none,
  // 1 = loads spread between the matrix instructions below, 2 = the next tile ends before its 64th row: loads with
  // clamped rows, all issued up front.
  auto step = [&](const int jt, auto mode) __attribute__((always_inline)) {
    constexpr int MODE = LW ? 0 : decltype(mode)::value;  // with loader waves the computing waves fetch nothing
    const int j0 = jt * BN;
    if constexpr (!LW) dma_wait();  // this wave's share of tile jt has landed
    __syncthreads();  // ... and everybody's; nobody reads the other stage any more
    uint16_t* nxt = smem + ((jt + 1) & 1) * 2 * TILE;
    const uint16_t* kn = kg + (int64_t)(j0 + BN) * gstride;
    const uint16_t* vn = vg + (int64_t)(j0 + BN) * gstride;
    if (MODE == 2) {
      dma_tile_ragged<D>(map, kn, nxt, wave, lane, gstride, P.s - (j0 + BN));
      dma_tile_ragged<D>(map, vn, nxt + TILE, wave, lane, gstride, P.s - (j0 + BN));
    }
    const uint16_t* Ks = smem + (jt & 1) * 2 * TILE;
    const uint16_t* Vs = Ks + TILE;
    // MODE 1: the four waves issue their shares of the next tile's loads at four different points of the step
    if (MODE == 1 && wave == 0) {
      dma_tile<D>(map, kn, nxt, wave);
      dma_tile<D>(map, vn, nxt + TILE, wave);
    }
    const int j0w = j0 + 32 * ks;
    {
      // a wave whose keys all lie past its rows (upper half of the diagonal tile) runs the step fully masked: the
      // other waves of the tile work meanwhile, so skipping would gain nothing, and one path through the step
      // keeps the accumulators in place
      const bool diag = (j0w + 31 > lim_lo);  // some of the wave's keys are masked for some of its rows
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
          if (j0w + 16 * (e >> 3) + 8 * hh + (e & 7) > jlim) st[e] = -INFINITY;
      }
      if (MODE == 1 && wave == 1) {  // pinned after the score tile
        float tok = st[0];
        dma_tile<D>(map, kn, nxt, wave, tok);
        dma_tile<D>(map, vn, nxt + TILE, wave, tok);
        st[0] = tok;
      }
      bf16x8_t dsf[2];
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        const int jc = j0w + 16 * c + 8 * hh;
        Philox4 rnd = {0u, 0u, 0u, 0u};
        if (DROP) rnd = philox_call8(rowG + (uint64_t)(jc >> 3), 0u, P.key0, P.key1);
        // waves 2 and 3 issue their loads of the next tile after the first / second random-number block
        if (MODE == 1 && wave == 2 + c) {
          if (DROP) {
            dma_tile<D>(map, kn, nxt, wave, rnd.x);
            dma_tile<D>(map, vn, nxt + TILE, wave, rnd.x);
          } else {
            float tok = st[8 * c];
            dma_tile<D>(map, kn, nxt, wave, tok);
            dma_tile<D>(map, vn, nxt + TILE, wave, tok);
            st[8 * c] = tok;
          }
        }
        float ds[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float pe = __builtin_amdgcn_exp2f(fmaf(st[8 * c + e], sc2, -lse2));
          const float dp = (!DROP || keep_field(rnd, e, P.thresh)) ? dd[8 * c + e] * P.keep_scale : 0.f;
          ds[e] = pe * (dp - dl);
        }
        dsf[c] = pack8(ds);
      }
#pragma unroll
      for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) dqacc[dt] = mfma32(ld_frag_tr_perm(Ks, KP, 32 * ks + 16 * c, 32 * dt, lane), dsf[c], dqacc[dt]);
    }
  };
  {
    const bool last_full = P.s - (ntile - 1) * BN >= BN;  // only the last tile can be ragged
    const int nspread = last_full ? ntile - 1 : ntile - 2;
    int jt = 0;
    for (; jt < nspread; ++jt) step(jt, std::integral_constant<int, 1>{});
    if (jt + 1 < ntile) step(jt++, std::integral_constant<int, 2>{});
    step(jt, std::integral_constant<int, 0>{});
  }
  // ---- sum the two key halves, scale, store ----
  __syncthreads();
  float* mg = reinterpret_cast<float*>(smem) + rg * (64 * 16 * DT);
  if (ks == 1) acc_put<DT>(mg, dqacc, lane);
  __syncthreads();
  if (ks == 0) {
    acc_combine<DT>(mg, dqacc, 1.f, 1.f, lane);
    acc_to_lds_rows<DT>(smem + 2 * TILE, KP, 32 * rg + li, dqacc, P.scale, hh);
  }
  __syncthreads();
  lds_rows_to_global<D>(smem + 2 * TILE, dq + base + (int64_t)(rb * BM) * P.stride_s, gstride, P.s - rb * BM, tid);
}

bool attn_mfma_supported(int d) { return d == 64 || d == 96 || d == 128 || d == 160; }

// 128-row workgroups pay when there are more of them than CUs (256 on this chip), so that the heaviest one does not set the pace,
// and at the largest head dimension only (measured at d = 160: -19 % at s = 4096, -20 % at s = 8192, -21 % without the
// mask, -14 % for 20 heads, -20 % for 32 heads; +14 % at the 16-head s = 2048 shape with its 256 workgroups; at d = 128
// +4 % and +10 % with 768 and 384 workgroups, at d = 96 +9 % with 512).
// sar_test_force_variants (tests, measurements) overrides the choice.
static std::atomic<int> g_force_fwd128{-1}, g_force_fwdlw{-1}, g_force_dqlw{-1};  // -1: the library chooses; 0 / 1: forced
void attn_mfma_force_variants(int fwd128, int fwdlw, int dqlw) {
  g_force_fwd128 = fwd128;
  g_force_fwdlw = fwdlw;
  g_force_dqlw = dqlw;
}

// compute units of the current device, asked once
int attn_mfma_cu_count() {
  static std::atomic<int> cached{0};
  int n = cached.load();
  if (n > 0) return n;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
  cached = n;
  return n;
}

static int cu_count() { return attn_mfma_cu_count(); }

static bool fwd_use_128(const AttnParams& P) {
  if (P.s < 128) return false;
  const int f = g_force_fwd128.load();
  if (f == 0 || f == 1) return f == 1;
  const int64_t wgs = (int64_t)((P.s + 127) / 128) * P.b * P.A;
  const int cus = cu_count();
  return P.d >= 160 && (P.causal ? wgs > cus : wgs >= cus);
}

template <int D>
static hipError_t fwd_d(const AttnParams& P, const void* q, const void* k, const void* v, void* o, float* lse, hipStream_t st) {
  if (fwd_use_128(P)) {
    const int N128 = P.b * P.A, nrb128 = (P.s + 127) / 128;
    if (P.thresh != 0)
      hipLaunchKernelGGL((attn_fwd_mfma_kernel<D, true, 4>), dim3((unsigned)(nrb128 * N128)), dim3(512), 0, st, P, (const uint16_t*)q,
                         (const uint16_t*)k, (const uint16_t*)v, (uint16_t*)o, lse);
    else
      hipLaunchKernelGGL((attn_fwd_mfma_kernel<D, false, 4>), dim3((unsigned)(nrb128 * N128)), dim3(512), 0, st, P, (const uint16_t*)q,
                         (const uint16_t*)k, (const uint16_t*)v, (uint16_t*)o, lse);
    return hipGetLastError();
  }
  const int N = P.b * P.A, nrb = (P.s + 63) / 64;
  {
    // loader waves: measured -10 % at d = 160 (530B shard), -9 % at d = 128 (175B), -8 % at d = 64, +15 % at d = 96 (22B
    // shard: three 4-wave workgroups share a CU there and fill each other's stalls).
    const int lw = g_force_fwdlw.load();
    // producer / consumer pairs: measured against the tile-fetching waves -16 % at d = 64 (22B shard), +2 % at d = 160,
    // +12 % at d = 128: where the head dimension is small the matrix and LDS work that moves to the second wave is a larger
    // share of a step, at d >= 128 the vector work that stays is the step
    if (lw == 2 || (lw < 0 && D == 64)) {
      if (P.thresh != 0)
        hipLaunchKernelGGL((attn_fwd_split_kernel<D, true>), dim3((unsigned)(nrb * N)), dim3(512), 0, st, P, (const uint16_t*)q, (const uint16_t*)k,
                           (const uint16_t*)v, (uint16_t*)o, lse);
      else
        hipLaunchKernelGGL((attn_fwd_split_kernel<D, false>), dim3((unsigned)(nrb * N)), dim3(512), 0, st, P, (const uint16_t*)q, (const uint16_t*)k,
                           (const uint16_t*)v, (uint16_t*)o, lse);
      return hipGetLastError();
    }
    const bool use_lw = (lw == 0 || lw == 1 || lw == 3) ? lw != 0 : D != 96;
    // persistent form of the same kernel (each workgroup works through a list of row blocks and overlaps a block's start with
    // the end of the one before): needs a grid of (row blocks at a time) x (heads) within the CU count; chosen when every
    // workgroup then gets at least two row blocks (measured at s = 2048: 16 heads of 160 -5 % .. -2.5 %; 12 heads of 128, where
    // 21 of the 32 blocks of a head start at once and only some workgroups get a second one, +1 %); forced by 3
    const int cus = cu_count();
    const bool pers = use_lw && N <= cus && (lw == 3 || (lw < 0 && nrb >= 2 * std::min(nrb, cus / N)));
    if (pers) {
      const int R = std::min(nrb, cus / N);
      if (P.thresh != 0)
        hipLaunchKernelGGL((attn_fwd_pers_kernel<D, true>), dim3((unsigned)(R * N)), dim3(512), 0, st, P, (const uint16_t*)q, (const uint16_t*)k,
                           (const uint16_t*)v, (uint16_t*)o, lse);
      else
        hipLaunchKernelGGL((attn_fwd_pers_kernel<D, false>), dim3((unsigned)(R * N)), dim3(512), 0, st, P, (const uint16_t*)q, (const uint16_t*)k,
                           (const uint16_t*)v, (uint16_t*)o, lse);
      return hipGetLastError();
    }
    if (use_lw) {
      if (P.thresh != 0)
        hipLaunchKernelGGL((attn_fwd_mfma_kernel<D, true, 2, true>), dim3((unsigned)(nrb * N)), dim3(512), 0, st, P, (const uint16_t*)q,
                           (const uint16_t*)k, (const uint16_t*)v, (uint16_t*)o, lse);
      else
        hipLaunchKernelGGL((attn_fwd_mfma_kernel<D, false, 2, true>), dim3((unsigned)(nrb * N)), dim3(512), 0, st, P, (const uint16_t*)q,
                           (const uint16_t*)k, (const uint16_t*)v, (uint16_t*)o, lse);
      return hipGetLastError();
    }
  }
  if (P.thresh != 0)
    hipLaunchKernelGGL((attn_fwd_mfma_kernel<D, true, 2>), dim3((unsigned)(nrb * N)), dim3(256), 0, st, P, (const uint16_t*)q, (const uint16_t*)k,
                       (const uint16_t*)v, (uint16_t*)o, lse);
  else  // every element is kept: the variant that draws no random numbers
    hipLaunchKernelGGL((attn_fwd_mfma_kernel<D, false, 2>), dim3((unsigned)(nrb * N)), dim3(256), 0, st, P, (const uint16_t*)q, (const uint16_t*)k,
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
  {
    // loader waves: -12 % at d = 128 (175B shard), -3 % at d = 160 (530B shard; -6 % at s = 4096), nothing at d = 64, +16 %
    // at d = 96, where several workgroups share a CU anyway.
    const int lw = g_force_dqlw.load();
    const bool use_lw = (lw == 0 || lw == 1) ? lw == 1 : D >= 128;
    if (use_lw) {
      if (P.thresh != 0)
        hipLaunchKernelGGL((attn_bwd_dq_mfma_kernel<D, true, true>), dim3((unsigned)(nb * N)), dim3(512), 0, st, P, (const uint16_t*)q, (const uint16_t*)k,
                           (const uint16_t*)v, (const uint16_t*)o, lse, (const uint16_t*)dO, (uint16_t*)dq, delta);
      else
        hipLaunchKernelGGL((attn_bwd_dq_mfma_kernel<D, false, true>), dim3((unsigned)(nb * N)), dim3(512), 0, st, P, (const uint16_t*)q, (const uint16_t*)k,
                           (const uint16_t*)v, (const uint16_t*)o, lse, (const uint16_t*)dO, (uint16_t*)dq, delta);
      return hipGetLastError();
    }
  }
  if (P.thresh != 0)
    hipLaunchKernelGGL((attn_bwd_dq_mfma_kernel<D, true>), dim3((unsigned)(nb * N)), dim3(256), 0, st, P, (const uint16_t*)q, (const uint16_t*)k,
                       (const uint16_t*)v, (const uint16_t*)o, lse, (const uint16_t*)dO, (uint16_t*)dq, delta);
  else
    hipLaunchKernelGGL((attn_bwd_dq_mfma_kernel<D, false>), dim3((unsigned)(nb * N)), dim3(256), 0, st, P, (const uint16_t*)q, (const uint16_t*)k,
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
  if (passes & 2) e = launch_attn_bwd_dkdv_mfma(P, q, k, v, lse, dO, delta, dk, dv, nullptr, st);
  return e;
}

}  // namespace sar
