// bf16 attention core, backward column pass (dK, dV) on gfx950 matrix cores: the kernel, included by the two translation
// units that instantiate it.  See attn_mfma_rows.hip for the tile layouts shared by the three kernels.
//   attn_mfma_cols.hip        d = 128, 160: compiled WITHOUT -amdgpu-mfma-vgpr-form.  One wave per SIMD; the two accumulator
//                             sets (2 x d/32 x 16 registers) live in accumulation registers (AGPRs) so that the 256 vector
//                             registers stay free for operands.                                   SAR_COLS_ACC = "a"
//   attn_mfma_cols_small.hip  d = 64, 96: compiled WITH it.  Two workgroups per CU, i.e. 256 registers per wave; a kernel that
//                             uses no AGPRs gets all of them as vector registers (otherwise the file is split 128 + 128) and
//                             the matrix instructions write where the vector arithmetic reads (22B shard -4.5 %, d = 64
//                             -16 %).                                                               SAR_COLS_ACC = "v"
#pragma once
#include "attn_mfma_common.h"

namespace sar {

// Two 16-byte stores per lane at (uniform base) + 16 lane and + 1 KB more: the wave's two dS operands of a step.  Written
// with a scalar base so that the only vector register the addresses cost is a short-lived one (the kernel is within a
// few registers of its limit, and a spilled or recomputed tile address sits on the critical path of every load).
__device__ __forceinline__ void ds_store2(uint16_t* base, int lane, bf16x8_t a, bf16x8_t b) {
  const uint32_t off = 16u * (uint32_t)lane;
  asm volatile("global_store_dwordx4 %0, %1, %3\n\tglobal_store_dwordx4 %0, %2, %3 offset:1024" : : "v"(off), "v"(a), "v"(b), "s"(base) : "memory");
}

// ===================================================================================================
// Backward, column-stationary pass.  Workgroup = 64 keys: wave = (kgp, is), kgp = 32-key group whose dK, dV
// accumulators it keeps in registers, is = which 32 query rows of each 64-row tile it sweeps.
//   dV_j = sum_i D_ij dO_i,  dK_j = alpha sum_i dS_ij q_i.
// P, D, dS are produced with one query row per lane; the two products above contract over i, so the bf16
// tiles are first moved to the one-key-per-lane layout by multiplying with an identity on the matrix core.
// ===================================================================================================
// DROP = false is the p = 0 variant: no random numbers are drawn at all.
// Up to d = 96 two workgroups fit a CU (LDS), if the compiler keeps a wave within half the register file: second
// argument = waves per SIMD.
// EVEN: s is a multiple of 64, every query tile is full.  Then the loads of the next (Q, dO) block are dealt out one
// per pair of score-tile matrix instructions instead of all at the top of the step: the L1 accepts one wave-wide
// load per 16 cycles per CU, a pair of 32x32x16 instructions keeps a SIMD busy for 64, so four waves that each issue
// one load per pair never queue behind each other (issued back to back, all four sit through all 44 loads).
// WDS: the bf16 dS tiles are also written to ds_ws (layout: ds_tile_index / kDsTileElems of sar_internal.h; inside a tile
// wave (kgp, is) owns two runs of 1 KB, one per 16-key group c, 16 bytes per lane), for the pass that forms dQ = alpha dS K
// from them without recomputing anything.
template <int D, bool DROP, bool EVEN, bool WDS = false>
__global__ __launch_bounds__(256, D <= 96 ? 2 : 1) void attn_bwd_dkdv_mfma_kernel(AttnParams P, const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
                                                                const uint16_t* __restrict__ v, const float* __restrict__ lse,
                                                                const uint16_t* __restrict__ dO, const float* __restrict__ delta,
                                                                uint16_t* __restrict__ dk, uint16_t* __restrict__ dv, uint16_t* __restrict__ ds_ws) {
  constexpr int BN = 64, BI = 64, KP = D + 8, KC = D / 16, DT = D / 32;
  constexpr int TILE = 64 * KP;
  __shared__ __attribute__((aligned(16))) uint16_t smem[6 * TILE];
  __shared__ float lse_s[2][BI], delta_s[2][BI];
  uint16_t* Ksm = smem;          // this workgroup's keys, rows swapped inside groups of 32
  uint16_t* Vsm = smem + TILE;
  uint16_t* stages = smem + 2 * TILE;  // two stages of (Q, dO): 64 query rows each, natural order; global -> LDS directly

  const int N = P.b * P.A;
  const int kb = (int)(blockIdx.x / N);  // key block 0 sweeps the most rows: heaviest first
  const int bn = blockIdx.x % N, beta = bn / P.A, n = bn % P.A;
  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, li = lane & 31, hh = lane >> 5;
  const int kgp = wave & 1, is = wave >> 1;
  const int64_t base = (int64_t)beta * P.stride_b + (int64_t)n * P.stride_a;
  const int gstride = (int)P.stride_s;
  const int jw0 = kb * BN + kgp * 32;  // first key of this wave

  const int nit = (P.s + BI - 1) / BI;
  const int it0 = P.causal ? kb : 0;  // BI == BN: the first tile with rows that attend to this block's keys
  const uint16_t* qg = q + base;
  const uint16_t* dog = dO + base;
  DmaMap<D> map;
  {
    const int left = P.s - kb * BN;
    map.init(wave, lane, gstride, true, left);
    dma_tile<D>(map, k + base + (int64_t)(kb * BN) * gstride, Ksm, wave);
    dma_tile<D>(map, v + base + (int64_t)(kb * BN) * gstride, Vsm, wave);
    map.init(wave, lane, gstride, false);
    const int leftq = P.s - it0 * BI;  // rows left from the first query tile
    if (leftq >= BI) {
      dma_tile<D>(map, qg + (int64_t)(it0 * BI) * gstride, stages + (it0 & 1) * 2 * TILE, wave);
      dma_tile<D>(map, dog + (int64_t)(it0 * BI) * gstride, stages + (it0 & 1) * 2 * TILE + TILE, wave);
    } else {
      dma_tile_ragged<D>(map, qg + (int64_t)(it0 * BI) * gstride, stages + (it0 & 1) * 2 * TILE, wave, lane, gstride, leftq);
      dma_tile_ragged<D>(map, dog + (int64_t)(it0 * BI) * gstride, stages + (it0 & 1) * 2 * TILE + TILE, wave, lane, gstride, leftq);
    }
  }
  // Row statistics (LSE, delta) of a query tile travel like the tile itself: wave 0 sends one float per row straight
  // into LDS.  Through registers, the wait for them would also wait for all of wave 0's tile loads in flight (the
  // counter is in order), and the other three waves would wait for wave 0 at the next barrier.
  auto load_stats = [&](int i_first, int stage) __attribute__((always_inline)) {
    const int ir = min(i_first + lane, P.s - 1);
    dma4(lse + (size_t)bn * P.s + ir, lds_addr(lse_s[stage]));
    dma4(delta + (size_t)bn * P.s + ir, lds_addr(delta_s[stage]));
  };
  if (wave == 0) load_stats(it0 * BI, it0 & 1);
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
  if constexpr (WDS) dma_wait();  // the first loads; inside the loop only "all but the last two operations" is waited for
  // WDS: this lane's 16 bytes of key group 0 in tile (it, kb) (key group 1: + 512 elements); the tile index grows by it + 1
  // per step under the causal mask, by the number of key blocks without it
  uint16_t* ds_tile = nullptr;                               // uniform: the wave's 2 KB of the tile
  int64_t ds_step = 0;
  if constexpr (WDS) {
    ds_tile = ds_ws + ((int64_t)bn * ds_tiles_per_head(P) + ds_tile_index(P, it0, kb)) * kDsTileElems + (2 * is + kgp) * 1024;
    ds_step = (P.causal ? (int64_t)(it0 + 1) : (int64_t)nit) * kDsTileElems;
  }
  for (int it = it0; it < nit; ++it) {
    const int i0 = it * BI;
    // This wave's share of tile `it` (and, the first time, of K and V) has landed.  WDS: every step ends with exactly two
    // dS stores per wave, issued after the step's loads; they need not have completed (waiting for them would cost the
    // write latency in every step).
    if constexpr (WDS) dma_wait_keep<2>();
    else dma_wait();
    __syncthreads();  // ... and everybody's; nobody reads the other stage any more
    // EVEN: the first round of the next block's loads; the last step fetches its own block again (into the stage
    // that nobody reads any more) so that the step has one path
    const int inx = min(it + 1, nit - 1) * BI;
    uint16_t* nxt = stages + ((it + 1) & 1) * 2 * TILE;
    if constexpr (EVEN) {
      dma_one<D>(map, qg + (int64_t)inx * gstride, nxt, wave, 0);
      dma_one<D>(map, dog + (int64_t)inx * gstride, nxt + TILE, wave, 0);
      if (wave == 0) load_stats(inx, (it + 1) & 1);
    } else if (it + 1 < nit) {  // next tile's loads fly while this one is computed
      const int left = P.s - (i0 + BI);
      if (left >= BI) {
        dma_tile<D>(map, qg + (int64_t)(i0 + BI) * gstride, nxt, wave);
        dma_tile<D>(map, dog + (int64_t)(i0 + BI) * gstride, nxt + TILE, wave);
      } else {
        dma_tile_ragged<D>(map, qg + (int64_t)(i0 + BI) * gstride, nxt, wave, lane, gstride, left);
        dma_tile_ragged<D>(map, dog + (int64_t)(i0 + BI) * gstride, nxt + TILE, wave, lane, gstride, left);
      }
      if (wave == 0) load_stats(i0 + BI, (it + 1) & 1);
    }
    const uint16_t* Qs = stages + (it & 1) * 2 * TILE;
    const uint16_t* dOs = Qs + TILE;
    const float* lse_c = lse_s[it & 1];
    const float* delta_c = delta_s[it & 1];
    const int i0w = i0 + 32 * is;  // this wave's 32 rows
    // i0w + 31 < jw0 (the upper right quarter of the diagonal tile): every row precedes this wave's keys.  EVEN: the
    // wave runs the tile fully masked rather than skipping it (its share of the loads sits inside)
    if (EVEN || !P.causal || i0w + 31 >= jw0) {
      const bool diag = P.causal && (i0w < jw0 + 31);
      float16_t st, dd;
#pragma unroll
      for (int e = 0; e < 16; ++e) { st[e] = 0.f; dd[e] = 0.f; }
      if constexpr (EVEN) {  // loads between the matrix instructions: keep the accumulators where they are around them
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
          asm volatile("" : "+" SAR_COLS_ACC(dkacc[dt]));
          asm volatile("" : "+" SAR_COLS_ACC(dvacc[dt]));
        }
      }
      // The operand reads run kAhead pairs of matrix instructions ahead, written out: the loads below are opaque
      // memory operations to the compiler, which therefore never moves an LDS read up across one of them, and a
      // read issued right before its matrix instruction leaves the whole LDS latency exposed, KC times.
      constexpr int kAhead = 2;
      bf16x8_t ka[kAhead], qa[kAhead], va[kAhead], da[kAhead];
      const uint16_t* qrow = Qs + (32 * is + li) * KP + 8 * hh;
      const uint16_t* drow = dOs + (32 * is + li) * KP + 8 * hh;
#pragma unroll
      for (int a = 0; a < kAhead; ++a) {
        ka[a] = ld_frag(kw + 16 * a), qa[a] = ld_frag(qrow + 16 * a);
        va[a] = ld_frag(vw + 16 * a), da[a] = ld_frag(drow + 16 * a);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int kc = 0; kc < KC; ++kc) {
        st = mfma32(ka[kc % kAhead], qa[kc % kAhead], st);
        dd = mfma32(va[kc % kAhead], da[kc % kAhead], dd);
        if (kc + kAhead < KC) {
          ka[kc % kAhead] = ld_frag(kw + 16 * (kc + kAhead)), qa[kc % kAhead] = ld_frag(qrow + 16 * (kc + kAhead));
          va[kc % kAhead] = ld_frag(vw + 16 * (kc + kAhead)), da[kc % kAhead] = ld_frag(drow + 16 * (kc + kAhead));
        }
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (EVEN) {  // rounds 1 .. PER-1 of the Q tile, then of the dO tile
          constexpr int PER = DmaMap<D>::PER;
          static_assert(2 * (PER - 1) <= KC, "more load rounds than pairs of matrix instructions");
          if (1 + kc < PER) dma_one<D>(map, qg + (int64_t)inx * gstride, nxt, wave, 1 + kc);
          else if (2 + kc - PER < PER) dma_one<D>(map, dog + (int64_t)inx * gstride, nxt + TILE, wave, 2 + kc - PER);
        }
      }
      if constexpr (EVEN) {
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
          asm volatile("" : "+" SAR_COLS_ACC(dkacc[dt]));
          asm volatile("" : "+" SAR_COLS_ACC(dvacc[dt]));
        }
      }
      const int i = i0w + li;
      const float lse2 = lse_c[32 * is + li] * kLog2e, dl = delta_c[32 * is + li];
      const uint64_t rowG = headG + (uint64_t)min(i, P.s - 1) * (uint64_t)(P.s >> 3);
      // uniform per wave: keys j > i, rows past the end and (WDS: their dS must be zero) keys past the end get
      // probability exp2(-inf) = 0
      if (diag || i0w + 31 >= P.s || (WDS && jw0 + 31 >= P.s)) {
        asm volatile("" ::: "memory");  // keep this a branch: most tiles skip it
        const int jlim = i >= P.s ? -1 : (P.causal ? i : P.s - 1);  // last key that row i attends to
#pragma unroll
        for (int e = 0; e < 16; ++e)
          if (jw0 + 16 * (e >> 3) + 8 * hh + (e & 7) > jlim) st[e] = -INFINITY;
      }
      bf16x8_t df[2], dsf[2];
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        const int jc = jw0 + 16 * c + 8 * hh;
        Philox4 rnd = {0u, 0u, 0u, 0u};
        if (DROP) rnd = philox_call8(rowG + (uint64_t)(jc >> 3), 0u, P.key0, P.key1);
        float dvv[8], ds[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float pe = __builtin_amdgcn_exp2f(fmaf(st[8 * c + e], sc2, -lse2));
          // the 16-bit field compared where it lies (no 8-bit mask in between: 60 fewer vector instructions per step)
          const float km = (!DROP || keep_field(rnd, e, P.thresh)) ? P.keep_scale : 0.f;
          dvv[e] = pe * km;
          ds[e] = pe * (dd[8 * c + e] * km - dl);
        }
        df[c] = pack8(dvv);
        dsf[c] = pack8(ds);
      }
      if constexpr (WDS) ds_store2(ds_tile, lane, dsf[0], dsf[1]);
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
    } else if constexpr (WDS) {  // a quarter above the diagonal: its dS is zero (and the step still ends with two stores)
      const u32x4_t zero = {0u, 0u, 0u, 0u};
      ds_store2(ds_tile, lane, __builtin_bit_cast(bf16x8_t, zero), __builtin_bit_cast(bf16x8_t, zero));
    }
    if constexpr (WDS) {
      ds_tile += ds_step;
      if (P.causal) ds_step += kDsTileElems;
    }
    // Keep the loop-carried accumulators in the accumulation registers (AGPRs) across the back-edge; without
    // this the compiler copies all of them to VGPRs and back on every trip.
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      asm volatile("" : "+" SAR_COLS_ACC(dkacc[dt]));
      asm volatile("" : "+" SAR_COLS_ACC(dvacc[dt]));
    }
  }
  // ---- sum the two row halves, scale, store ----
  dma_wait();  // EVEN: the last step's loads still target the stages that the exchange buffers overlap
  __syncthreads();
  // each wave of a pair gives one accumulator set away and finishes the other: the upper half completes dV, the lower dK
  float* mg = reinterpret_cast<float*>(smem) + kgp * (64 * 32 * DT);
  if (is == 1) acc_put<DT>(mg, dkacc, lane);
  else acc_put<DT>(mg + 16 * DT * 64, dvacc, lane);
  __syncthreads();
  if (is == 0) {
    acc_combine<DT>(mg, dkacc, 1.f, 1.f, lane);
    acc_to_lds_rows<DT>(smem + 4 * TILE, KP, 32 * kgp + li, dkacc, P.scale, hh);
  } else {
    acc_combine<DT>(mg + 16 * DT * 64, dvacc, 1.f, 1.f, lane);
    acc_to_lds_rows<DT>(smem + 5 * TILE, KP, 32 * kgp + li, dvacc, 1.0f, hh);
  }
  __syncthreads();
  lds_rows_to_global<D>(smem + 4 * TILE, dk + base + (int64_t)(kb * BN) * P.stride_s, gstride, P.s - kb * BN, tid);
  lds_rows_to_global<D>(smem + 5 * TILE, dv + base + (int64_t)(kb * BN) * P.stride_s, gstride, P.s - kb * BN, tid);
}

template <int D>
static hipError_t bwd_dkdv_d(const AttnParams& P, const void* q, const void* k, const void* v, const float* lse, const void* dO, const float* delta,
                             void* dk, void* dv, uint16_t* ds_ws, hipStream_t st) {
  const int N = P.b * P.A, nb = (P.s + 63) / 64;
  auto go = [&](auto kern) {
    hipLaunchKernelGGL(kern, dim3((unsigned)(nb * N)), dim3(256), 0, st, P, (const uint16_t*)q, (const uint16_t*)k, (const uint16_t*)v, lse,
                       (const uint16_t*)dO, delta, (uint16_t*)dk, (uint16_t*)dv, ds_ws);
  };
  // interleaved loads pay at d = 160 only (530B shard -3 %, 1T -6 %, s = 4096 -3 %; d = 128 unchanged; d = 96, where two
  // workgroups share a CU and fill each other's stalls anyway, +2 %)
  constexpr bool kInterleave = D >= 160;
  const bool even = kInterleave && P.s % 64 == 0;
  if (ds_ws) {
    if (P.thresh != 0) {
      if (even) go(attn_bwd_dkdv_mfma_kernel<D, true, kInterleave, true>);
      else go(attn_bwd_dkdv_mfma_kernel<D, true, false, true>);
    } else {
      if (even) go(attn_bwd_dkdv_mfma_kernel<D, false, kInterleave, true>);
      else go(attn_bwd_dkdv_mfma_kernel<D, false, false, true>);
    }
  } else if (P.thresh != 0) {
    if (even) go(attn_bwd_dkdv_mfma_kernel<D, true, kInterleave>);
    else go(attn_bwd_dkdv_mfma_kernel<D, true, false>);
  } else {
    if (even) go(attn_bwd_dkdv_mfma_kernel<D, false, kInterleave>);
    else go(attn_bwd_dkdv_mfma_kernel<D, false, false>);
  }
  return hipGetLastError();
}

}  // namespace sar
