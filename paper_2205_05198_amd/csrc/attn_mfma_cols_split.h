// bf16 attention core, backward column pass (dK, dV) in its two-waves-per-SIMD form: the work of a (32 keys x 32 query rows)
// block of every step is divided between a producing and a consuming wave that share a SIMD.
//
// Why: a wave issues its instructions in order, so with one wave per SIMD a step of the column pass costs the sum of the issue
// times of its vector instructions, matrix instructions, LDS reads and direct-to-LDS loads (about 3700 cycles at d = 160 for
// 1400 cycles of matrix-pipe time and 1650 of vector-unit time), and a second wave of the same kind does not fit the register
// file (two accumulator sets of d/32 x 16 registers plus the arithmetic's working set).  Divided in two, each half fits 256
// registers, and the halves use different units:
//   producer (waves 0..3)  S^T = K Q^T and dD^T = V dO^T with K and V operands held in registers, then the vector arithmetic:
//                          P = exp2(alpha log2e S - LSE), Philox mask, D = M P / (1-p), dS = P (dD M / (1-p) - delta); the two
//                          results go, rounded to bf16, as row-major [32 rows][32 keys] tiles to an exchange buffer in LDS
//                          (and, WDS, dS to the tiles that the dQ product reads);
//   consumer (waves 4..7)  reads them one key per lane (transposing LDS reads) and accumulates dV^T += dO^T D (two of the
//                          waves, one per 32 keys, over all 64 rows of the tile) or dK^T += Q^T dS (the other two), and
//                          issues every direct-to-LDS load of the workgroup.
// The consumer works one tile behind the producer; (Q, dO) tiles live in three stages: tile m is loaded during step m-1, read
// by the producer in step m and by the consumer in step m+1.  One workgroup barrier per step.
// Needs s % 64 == 0.  Everything is in vector registers (compiled with -amdgpu-mfma-vgpr-form): no copies out of
// accumulation registers.
#pragma once
#include "attn_mfma_cols_kernel.h"

namespace sar {

template <int D, bool DROP, bool WDS, bool PERS = false>
__global__ __launch_bounds__(512, 1) void attn_bwd_dkdv_split_kernel(AttnParams P, const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
                                                                    const uint16_t* __restrict__ v, const float* __restrict__ lse,
                                                                    const uint16_t* __restrict__ dO, const float* __restrict__ delta,
                                                                    uint16_t* __restrict__ dk, uint16_t* __restrict__ dv, uint16_t* __restrict__ ds_ws) {
  constexpr int BN = 64, BI = 64, KP = D + 8, KC = D / 16, DT = D / 32, NST = 3;
  constexpr int TILE = 64 * KP;
  __shared__ __attribute__((aligned(16))) uint16_t smem[2 * NST * TILE];  // stage s: Q at 2 s TILE, dO at (2 s + 1) TILE; afterwards the epilogue's buffers
  __shared__ __attribute__((aligned(16))) uint16_t xb[2][4][4][512];      // exchange: [step parity][wave pair][D rows 0..15, D rows 16..31, dS likewise][16 rows x 32 keys]
  __shared__ float lse_s[NST][BI], delta_s[NST][BI];

  const int N = P.b * P.A;
  const int nb = P.s / BN;
  // Which key blocks this workgroup takes.  Plain: one, block blockIdx / N (key block 0 sweeps the most rows: heaviest
  // first).  PERS: the grid is R x N workgroups (R x N <= number of CUs) and workgroup (wq, head) takes its head's key blocks
  // wq, 2R-1-wq, 2R+wq, 4R-1-wq, ...: a heavy block, then a light one; the next block's K, V and first (Q, dO) tile are
  // requested during the last step of the block before and land while its epilogue runs.
  const int Rr = PERS ? (int)gridDim.x / N : nb;
  const int wq = (int)(blockIdx.x / N);
  auto block_of = [&](const int j) __attribute__((always_inline)) { return (j & 1) ? (j + 1) * Rr - 1 - wq : j * Rr + wq; };  // >= nb: none
  int kb = wq;
  const int bn = blockIdx.x % N, beta = bn / P.A, n = bn % P.A;
  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, li = lane & 31, hh = lane >> 5;
  const bool producer = wave < 4;
  const int w = wave & 3;  // the pair: waves w and w + 4 sit on SIMD w
  const int kgp = w & 1, is = w >> 1;
  const int64_t base = (int64_t)beta * P.stride_b + (int64_t)n * P.stride_a;
  const int gstride = (int)P.stride_s;
  int jw0 = kb * BN + kgp * 32;  // first key of this pair
  const int nit = P.s / BI;
  int it0 = P.causal ? kb : 0;
  // (Q, dO) tile m of the current key block lives in stage (m - it0 + off) % NST; its K and V blocks are staged where tile
  // it0 + 1 will go; its output tiles go where its last tile was
  int off = 0;
  auto stage_of = [&](const int m) __attribute__((always_inline)) { return (m - it0 + off) % NST; };
  const uint16_t* qg = q + base;
  const uint16_t* dog = dO + base;

  if (producer) {
    // ---- K and V operands of this wave's 32 keys, for the whole kernel: lane li holds key jw0 + perm_row(li).  They come
    // through LDS (coalesced direct loads into the stage that tile it0 + 1 will take; rows swapped inside groups of 32):
    // fetched straight into registers, every lane reads 20 separate 16-byte pieces of its own row ----
    bf16x8_t kf[KC], vf[KC];
    DmaMap<D> kvmap;
    kvmap.init(w, lane, gstride, true);
    {
      uint16_t* Kst = smem + stage_of(it0 + 1) * 2 * TILE;
      dma_tile<D>(kvmap, k + base + (int64_t)(kb * BN) * gstride, Kst, w);
      dma_tile<D>(kvmap, v + base + (int64_t)(kb * BN) * gstride, Kst + TILE, w);
      dma_wait();
      __syncthreads();  // the K and V blocks are staged
    }
    const uint64_t headG = P.offset + (((uint64_t)beta * (uint64_t)P.a_global + (uint64_t)(P.head0 + n)) * (uint64_t)P.s) * (uint64_t)(P.s >> 3);
    const float sc2 = P.scale * kLog2e;
    const float log2_keep_scale = __builtin_amdgcn_logf(P.keep_scale), inv_keep_scale = 1.0f / P.keep_scale;  // v_log_f32 is log2
    for (int j = 0;; ++j) {  // key blocks of this workgroup
    {
      const uint16_t* kw = smem + stage_of(it0 + 1) * 2 * TILE + (32 * kgp + li) * KP + 8 * hh;
#pragma unroll
      for (int kc = 0; kc < KC; ++kc) {
        kf[kc] = ld_frag(kw + 16 * kc);
        vf[kc] = ld_frag(kw + TILE + 16 * kc);
      }
#pragma unroll
      for (int kc = 0; kc < KC; ++kc) asm volatile("" : "+v"(kf[kc]), "+v"(vf[kc]));  // read before the barrier that frees the stage
    }
    const int kb_n = PERS ? block_of(j + 1) : nb;
    const bool has_next = kb_n < nb;
    uint16_t* ds_tile = nullptr;  // uniform: the wave's 2 KB of the dS tile (it, kb)
    int64_t ds_step = 0;
    if constexpr (WDS) {
      ds_tile = ds_ws + ((int64_t)bn * ds_tiles_per_head(P) + ds_tile_index(P, it0, kb)) * kDsTileElems + (2 * is + kgp) * 1024;
      ds_step = (P.causal ? (int64_t)(it0 + 1) : (int64_t)nit) * kDsTileElems;
    }
    for (int m = it0; m <= nit; ++m) {
      __syncthreads();  // tile m is in its stage; the consumer has read exchange buffer m & 1 (tile m - 2)
      if (m == nit) break;
      const int sg = stage_of(m);
      const uint16_t* Qs = smem + sg * 2 * TILE;
      const uint16_t* qrow = Qs + (32 * is + li) * KP + 8 * hh;
      const uint16_t* drow = qrow + TILE;
      float16_t st, dd;
#pragma unroll
      for (int e = 0; e < 16; ++e) { st[e] = 0.f; dd[e] = 0.f; }
      const int i = m * BI + 32 * is + li;
      // lse2q: the row's LSE in log2 units minus log2 of 1/(1-p); dlq: delta (1-p)
      const float lse2q = lse_s[sg][32 * is + li] * kLog2e - log2_keep_scale, dlq = delta_s[sg][32 * is + li] * inv_keep_scale;
      // The wave's instructions are ordered by hand so that its matrix instructions always have vector work of the same
      // wave beside them:
      //   1. S^T = K Q^T            between its matrix instructions: the two Philox calls of the tile (indices only);
      //   2. dD^T = V dO^T          between them: P = exp2(..), the keep decisions, D = P M / (1-p) (need S only);
      //   3. dS = P (dD M / (1-p) - delta), rounding to bf16.
      Philox4 rnd[2] = {{0u, 0u, 0u, 0u}, {0u, 0u, 0u, 0u}};
      if (DROP) {
        const uint64_t rowG = headG + (uint64_t)i * (uint64_t)(P.s >> 3);
#pragma unroll
        for (int c = 0; c < 2; ++c) rnd[c] = philox_start(rowG + (uint64_t)((jw0 + 16 * c + 8 * hh) >> 3), 0u);
      }
      constexpr int kAhead = 3;
      bf16x8_t qa[kAhead], da[kAhead];
#pragma unroll
      for (int a = 0; a < kAhead; ++a) qa[a] = ld_frag(qrow + 16 * a);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int kc = 0; kc < KC; ++kc) {
        st = mfma32(kf[kc], qa[kc % kAhead], st);
        if (kc + kAhead < KC) qa[kc % kAhead] = ld_frag(qrow + 16 * (kc + kAhead));
        if (kc >= KC - kAhead) da[kc - (KC - kAhead)] = ld_frag(drow + 16 * (kc - (KC - kAhead)));
        if (DROP) {
#pragma unroll
          for (int u = (20 * kc) / KC; u < (20 * (kc + 1)) / KC; ++u) philox_round(rnd[u & 1], P.key0, P.key1, u >> 1);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      if (P.causal && m == kb) {  // the diagonal tile: keys j > i get probability exp2(-inf) = 0
        asm volatile("" ::: "memory");  // keep this a branch: all other tiles skip it
#pragma unroll
        for (int e = 0; e < 16; ++e)
          if (jw0 + 16 * (e >> 3) + 8 * hh + (e & 7) > i) st[e] = -INFINITY;
      }
      // Q = P / (1-p) comes straight out of the exponential (log2 of the scale folded into the row's LSE term), so that
      // D = M Q is one select and dS = P (dD M / (1-p) - delta) = D dD - Q delta (1-p) two more operations per element.
      float pq[16], dvv[16];
#pragma unroll
      for (int kc = 0; kc < KC; ++kc) {
        dd = mfma32(vf[kc], da[kc % kAhead], dd);
        if (kc + kAhead < KC) da[kc % kAhead] = ld_frag(drow + 16 * (kc + kAhead));
        // 16 exponent arguments, 16 exponentials, the two blocks of eight keep selects, 16 products, dealt out in this order
        // over the windows: a window then holds one kind of operation on different elements (dependent instructions would
        // run at their latency)
        constexpr int NOPS = 50;  // 16 + 16 + 2 + 16
#pragma unroll
        for (int o = (NOPS * kc) / KC; o < (NOPS * (kc + 1)) / KC; ++o) {
          if (o < 16) pq[o] = fmaf(st[o], sc2, -lse2q);
          else if (o < 32) pq[o - 16] = __builtin_amdgcn_exp2f(pq[o - 16]);
          else if (o < 34) {
            const int c = o - 32;
            if (DROP) {
              keep_select8(rnd[c], P.thresh, reinterpret_cast<const float(&)[8]>(pq[8 * c]), reinterpret_cast<float(&)[8]>(dvv[8 * c]));
            } else {
#pragma unroll
              for (int e = 0; e < 8; ++e) dvv[8 * c + e] = pq[8 * c + e];
            }
          } else pq[o - 34] *= dlq;  // Q delta (1-p)
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      bf16x8_t df[2], dsf[2];
      df[0] = pack8(dvv);
      df[1] = pack8(dvv + 8);
      {
        float ds[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) ds[e] = fmaf(dvv[e], dd[e], -pq[e]);
        dsf[0] = pack8(ds);
        dsf[1] = pack8(ds + 8);
      }
      if constexpr (WDS) {
        ds_store2(ds_tile, lane, dsf[0], dsf[1]);
        ds_tile += ds_step;
        if (P.causal) ds_step += kDsTileElems;
      }
      // exchange tiles [32 rows][32 keys], 64 bytes per row; the 16-byte piece q of row r sits at piece q ^ 2 (r>>2 & 1), which
      // spreads the writes of a wave over all banks
      uint16_t* x = &xb[m & 1][w][0][0] + 32 * li;
      const int sw = 2 * ((li >> 2) & 1);
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        *reinterpret_cast<bf16x8_t*>(x + 8 * ((2 * c + hh) ^ sw)) = df[c];
        *reinterpret_cast<bf16x8_t*>(x + 1024 + 8 * ((2 * c + hh) ^ sw)) = dsf[c];
      }
    }
    // The consumers' last step and epilogue.  The stage of the last tile becomes the output tiles; of the other two, the
    // one after it takes the next key block's first (Q, dO) tile (fetched by the consumers), the one after that its K and V.
    const int so = stage_of(nit - 1);
    if (has_next) {
      uint16_t* Kst = smem + ((so + 2) % NST) * 2 * TILE;
      dma_tile<D>(kvmap, k + base + (int64_t)(kb_n * BN) * gstride, Kst, w);
      dma_tile<D>(kvmap, v + base + (int64_t)(kb_n * BN) * gstride, Kst + TILE, w);
    }
    __syncthreads();  // the consumers are done with the last tile
    if (has_next) dma_wait();
    __syncthreads();  // the output tiles are complete (and the next K and V blocks staged)
    lds_rows_to_global<D>(smem + so * 2 * TILE, dk + base + (int64_t)(kb * BN) * P.stride_s, gstride, P.s - kb * BN, tid);
    if (!has_next) break;
    kb = kb_n;
    jw0 = kb * BN + kgp * 32;
    off = (so + 1) % NST;  // before it0 changes: stage_of(new it0) = off
    it0 = P.causal ? kb : 0;
    }  // key blocks
  } else {
    // ---- consumer ----
    DmaMap<D> map;
    map.init(w, lane, gstride, false);
    auto fetch_to = [&](int it, int round, int sg) __attribute__((always_inline)) {  // rounds 0 .. 2 PER - 1 of tile `it`, into stage sg
      constexpr int PER = DmaMap<D>::PER;
      uint16_t* dst = smem + sg * 2 * TILE;
      if (round < PER) dma_one<D>(map, qg + (int64_t)(it * BI) * gstride, dst, w, round);
      else dma_one<D>(map, dog + (int64_t)(it * BI) * gstride, dst + TILE, w, round - PER);
    };
    auto fetch_stats_to = [&](int it, int sg) __attribute__((always_inline)) {  // one float per row, straight into LDS
      dma4(lse + (size_t)bn * P.s + it * BI + lane, lds_addr(lse_s[sg]));
      dma4(delta + (size_t)bn * P.s + it * BI + lane, lds_addr(delta_s[sg]));
    };
    auto fetch = [&](int it, int round) __attribute__((always_inline)) { fetch_to(it, round, stage_of(it)); };
    auto fetch_stats = [&](int it) __attribute__((always_inline)) { fetch_stats_to(it, stage_of(it)); };
    constexpr int NR = 2 * DmaMap<D>::PER;
#pragma unroll
    for (int r = 0; r < NR; ++r) fetch(it0, r);
    if (w == 0) fetch_stats(it0);
    __syncthreads();  // the producers have staged K and V (they read them before the first barrier of the loop)
    // Consumer w = (kgp, role): role 0 accumulates dV^T of the pair of producers with key group kgp (both row halves of the
    // tile) from D and dO, role 1 dK^T from dS and Q.  One accumulator set per wave, complete at the end: no merging.
    const int role = is;
    float16_t acc[DT];
    // this lane's address inside a [32 rows][32 keys] exchange tile for the transposing read of rows 0..3 / 4..7 (hh)
    const int lam = lane & 15, blk = lane >> 4;
    const int xoff = 1024 * role + (4 * (blk >> 1) + (lam >> 2)) * 32 + 8 * ((2 * (blk & 1) + ((lam & 3) >> 1)) ^ (2 * (blk >> 1))) + 4 * (lam & 1);

    for (int j = 0;; ++j) {  // key blocks of this workgroup
    const int kb_n = PERS ? block_of(j + 1) : nb;
    const bool has_next = kb_n < nb;
    const int it0_n = P.causal ? kb_n : 0;
    const int so = stage_of(nit - 1);  // the last tile's stage, then the output tiles
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[dt][e] = 0.f;
    for (int m = it0; m <= nit; ++m) {
      dma_wait();       // this wave's share of tile m has landed
      __syncthreads();  // ... and everybody's; the producers have written exchange buffer (m - 1) & 1 and read tile m - 1
      const bool more = m + 1 < nit;
      if (more && w == 0) fetch_stats(m + 1);
      if (m == it0) {  // nothing to consume yet
        if (more) {
#pragma unroll
          for (int r = 0; r < NR; ++r) fetch(m + 1, r);
        }
        continue;
      }
      const int t = m - 1;
      const uint16_t* Ts = smem + stage_of(t) * 2 * TILE + (role ? 0 : TILE);  // Q for dK, dO for dV
      // one-key-per-lane operands straight from the exchange tiles (transposing LDS reads): slot e of lane (li, hh) <-> key li,
      // row 32 h + 16 X + 8 (e>>2) + 4 hh + (e&3), the row order of the transposed Q / dO operands
      bf16x8_t bT[2][2];  // [row half h][X]
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const uint16_t* xp = &xb[t & 1][2 * h + kgp][0][0] + xoff;
#pragma unroll
        for (int X = 0; X < 2; ++X) {
          union { short4_t q[2]; bf16x8_t v; } u;
          u.q[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_t*)(xp + 512 * X));
          u.q[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_t*)(xp + 512 * X + 256));
          bT[h][X] = u.v;
        }
      }
      if (more) { fetch(m + 1, 0); fetch(m + 1, 1); }
      if (PERS && m == nit && has_next) {  // the next key block's first (Q, dO) tile and row statistics, into the stage after this one
#pragma unroll
        for (int r = 0; r < NR; ++r) fetch_to(it0_n, r, (so + 1) % NST);
        if (w == 0) fetch_stats_to(it0_n, (so + 1) % NST);
      }
      constexpr int kAhead = 3, NP = 4 * DT;
      bf16x8_t ta[kAhead];
      auto tr = [&](int p) __attribute__((always_inline)) {  // product p: rows 16 (p / DT) .. + 15 of the tile, columns 32 (p % DT) ..
        return ld_frag_tr_perm(Ts, KP, 16 * (p / DT), 32 * (p % DT), lane);
      };
#pragma unroll
      for (int a = 0; a < kAhead; ++a) ta[a] = tr(a);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int p = 0; p < NP; ++p) {
        acc[p % DT] = mfma32(ta[p % kAhead], bT[p / (2 * DT)][(p / DT) & 1], acc[p % DT]);
        if (p + kAhead < NP) ta[p % kAhead] = tr(p + kAhead);
        // the rest of the next tile's loads, one after each of the first products: they have the rest of the step to land
        if (more && 2 + p < NR) fetch(m + 1, 2 + p);
        __builtin_amdgcn_sched_barrier(0);
      }
      static_assert(NR - 2 <= NP, "more load rounds than products");
    }
    // ---- scale, round, rows through LDS (the producers' threads copy dK out, the consumers' dV) ----
    __syncthreads();  // every consumer is done with the last tile (the output tiles take its stage)
    acc_to_lds_rows<DT>(smem + (2 * so + (role ? 0 : 1)) * TILE, KP, 32 * kgp + li, acc, role ? P.scale : 1.0f, hh);
    __syncthreads();
    lds_rows_to_global<D>(smem + (2 * so + 1) * TILE, dv + base + (int64_t)(kb * BN) * P.stride_s, gstride, P.s - kb * BN, tid - 256);
    if (!has_next) break;
    kb = kb_n;
    off = (so + 1) % NST;  // before it0 changes: the new first tile's stage
    it0 = it0_n;
    }  // key blocks
  }
}

}  // namespace sar
