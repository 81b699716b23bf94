// bf16 attention core, backward column pass (dK, dV), software-pipelined form for the large head dimensions (one wave per
// SIMD, so nothing but the wave's own instruction stream can overlap its matrix and vector work).
//
// Same decomposition, tile layouts and results as attn_bwd_dkdv_mfma_kernel (attn_mfma_cols_kernel.h): workgroup = 64 keys,
// wave = (kgp, is).  What differs is the order of a step.  There, a step runs scores -> softmax / dropout arithmetic ->
// products, one after the other, and during the ~1800 cycles of vector arithmetic the matrix pipe is idle.  Here the score
// tiles (S^T, dD^T) of query tile it + 1 are computed during the vector arithmetic of tile it: each pair of score-tile
// matrix instructions is followed by one round of the tile's two Philox calls and a share of its exponentials, which run
// in the shadow of those matrix instructions.  That needs three (Q, dO) stages in LDS (tile it for the products, it + 1 for
// the scores, it + 2 in flight), so K leaves LDS: each wave keeps the K operands of its 32 keys in 40 accumulation
// registers (matrix instructions read them there), V stays in LDS: 7 tiles = 147 KB.
// Needs s % 64 == 0 (every query tile is full) and is instantiated for d = 128 and 160.  Measured (rocprofv3, once-form):
// d = 128 (175B shard) 59.1 against 70.4 us; d = 160 (530B shard) 80.2 against 79.1 us: there a step is the sum of its
// vector arithmetic (~1700 cycles), the issue of its ten direct loads (64 cycles each, which overlap the score tiles'
// matrix instructions but not vector instructions of the same wave) and the products (~1100), and hiding the score tiles
// behind the arithmetic only trades one overlap for another.  The library therefore picks it for d = 128.
#pragma once
#include "attn_mfma_cols_kernel.h"

namespace sar {

template <int D, bool DROP, bool WDS>
__global__ __launch_bounds__(256, 1) void attn_bwd_dkdv_pipe_kernel(AttnParams P, const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
                                                                  const uint16_t* __restrict__ v, const float* __restrict__ lse,
                                                                  const uint16_t* __restrict__ dO, const float* __restrict__ delta,
                                                                  uint16_t* __restrict__ dk, uint16_t* __restrict__ dv, uint16_t* __restrict__ ds_ws) {
  constexpr int BN = 64, BI = 64, KP = D + 8, KC = D / 16, DT = D / 32, NST = 3;
  constexpr int TILE = 64 * KP;
  __shared__ __attribute__((aligned(16))) uint16_t smem[7 * TILE];
  __shared__ float lse_s[NST][BI], delta_s[NST][BI];
  uint16_t* Vsm = smem;             // this workgroup's V rows, swapped inside groups of 32
  uint16_t* stages = smem + TILE;   // three stages of (Q, dO): stage g holds Q at + 2 g TILE, dO one tile behind it

  const int N = P.b * P.A;
  const int kb = (int)(blockIdx.x / N);  // key block 0 sweeps the most rows: heaviest first
  const int bn = blockIdx.x % N, beta = bn / P.A, n = bn % P.A;
  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, li = lane & 31, hh = lane >> 5;
  const int kgp = wave & 1, is = wave >> 1;
  const int64_t base = (int64_t)beta * P.stride_b + (int64_t)n * P.stride_a;
  const int gstride = (int)P.stride_s;
  const int jw0 = kb * BN + kgp * 32;  // first key of this wave

  const int nit = P.s / BI;
  const int it0 = P.causal ? kb : 0;
  const uint16_t* qg = q + base;
  const uint16_t* dog = dO + base;
  auto stage_q = [&](int it) __attribute__((always_inline)) { return stages + (it % NST) * 2 * TILE; };
  auto load_stats = [&](int it, int stage) __attribute__((always_inline)) {
    dma4(lse + (size_t)bn * P.s + it * BI + lane, lds_addr(lse_s[stage]));
    dma4(delta + (size_t)bn * P.s + it * BI + lane, lds_addr(delta_s[stage]));
  };
  DmaMap<D> map;
  uint16_t* Ktmp = stage_q(it0 + 2);  // K passes through the stage that the first step's loads will fill
  {
    map.init(wave, lane, gstride, true);
    dma_tile<D>(map, k + base + (int64_t)(kb * BN) * gstride, Ktmp, wave);
    dma_tile<D>(map, v + base + (int64_t)(kb * BN) * gstride, Vsm, wave);
    map.init(wave, lane, gstride, false);
    const int it1 = min(it0 + 1, nit - 1);
    dma_tile<D>(map, qg + (int64_t)(it0 * BI) * gstride, stage_q(it0), wave);
    dma_tile<D>(map, dog + (int64_t)(it0 * BI) * gstride, stage_q(it0) + TILE, wave);
    dma_tile<D>(map, qg + (int64_t)(it1 * BI) * gstride, stage_q(it0 + 1), wave);
    dma_tile<D>(map, dog + (int64_t)(it1 * BI) * gstride, stage_q(it0 + 1) + TILE, wave);
    if (wave == 0) {
      load_stats(it0, it0 % NST);
      load_stats(it1, (it0 + 1) % NST);
    }
  }
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
  const uint16_t* vw = Vsm + (32 * kgp + li) * KP + 8 * hh;

  dma_wait();
  __syncthreads();
  // the K operands of this wave's keys, for the whole kernel (LDS row 32 kgp + li holds key jw0 + perm_row(li))
  bf16x8_t kf[KC];
#pragma unroll
  for (int kc = 0; kc < KC; ++kc) kf[kc] = ld_frag(Ktmp + (32 * kgp + li) * KP + 16 * kc + 8 * hh);
#pragma unroll
  for (int kc = 0; kc < KC; ++kc) asm volatile("" : "+a"(kf[kc]));
  __syncthreads();  // everybody has its K operands: the stage may be overwritten

  // score tiles of query tile `it` against this wave's keys, rows 32 is .. 32 is + 31 of the tile (no interleaving: used once)
  auto scores_plain = [&](int it, float16_t& st, float16_t& dd) __attribute__((always_inline)) {
    const uint16_t* qrow = stage_q(it) + (32 * is + li) * KP + 8 * hh;
    const uint16_t* drow = qrow + TILE;
#pragma unroll
    for (int e = 0; e < 16; ++e) { st[e] = 0.f; dd[e] = 0.f; }
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) {
      st = mfma32(kf[kc], ld_frag(qrow + 16 * kc), st);
      dd = mfma32(ld_frag(vw + 16 * kc), ld_frag(drow + 16 * kc), dd);
    }
  };
  float16_t st, dd;  // score tiles of the tile whose arithmetic is next
  scores_plain(it0, st, dd);

  uint16_t* ds_tile = nullptr;
  int64_t ds_step = 0;
  if constexpr (WDS) {
    ds_tile = ds_ws + ((int64_t)bn * ds_tiles_per_head(P) + ds_tile_index(P, it0, kb)) * kDsTileElems + (2 * is + kgp) * 1024;
    ds_step = (P.causal ? (int64_t)(it0 + 1) : (int64_t)nit) * kDsTileElems;
  }

  for (int it = it0; it < nit; ++it) {
    // Tile it + 1 (requested one step ago) has landed.  WDS: every step ends with exactly two dS stores per wave, issued
    // after the step's loads; they need not have completed.
    if constexpr (WDS) dma_wait_keep<2>();
    else dma_wait();
    __syncthreads();  // ... for everybody; nobody reads tile it - 1 any more, whose stage tile it + 2 takes
    const int itn = min(it + 1, nit - 1), it2 = min(it + 2, nit - 1);  // past the end: the last tile again (results unused)
    uint16_t* nxt = stage_q(it + 2);
    dma_one<D>(map, qg + (int64_t)(it2 * BI) * gstride, nxt, wave, 0);
    dma_one<D>(map, dog + (int64_t)(it2 * BI) * gstride, nxt + TILE, wave, 0);
    if (wave == 0) load_stats(it2, (it + 2) % NST);

    const int i0w = it * BI + 32 * is;
    const int i = i0w + li;
    const float lse2 = lse_s[it % NST][32 * is + li] * kLog2e, dl = delta_s[it % NST][32 * is + li];
    // this tile's scores, in vector registers from here on; keys j > i of the diagonal tile get probability exp2(-inf) = 0
    asm volatile("" : "+v"(st), "+v"(dd));
    if (P.causal && i0w < jw0 + 31) {
      asm volatile("" ::: "memory");  // keep this a branch: most tiles skip it
#pragma unroll
      for (int e = 0; e < 16; ++e)
        if (jw0 + 16 * (e >> 3) + 8 * hh + (e & 7) > i) st[e] = -INFINITY;
    }
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      asm volatile("" : "+" SAR_COLS_ACC(dkacc[dt]));
      asm volatile("" : "+" SAR_COLS_ACC(dvacc[dt]));
    }
    // ---- phase A: score tiles of tile it + 1 on the matrix pipe, the vector arithmetic of tile it beside them ----
    Philox4 rnd[2] = {{0u, 0u, 0u, 0u}, {0u, 0u, 0u, 0u}};
    if constexpr (DROP) {
      const uint64_t rowG = headG + (uint64_t)i * (uint64_t)(P.s >> 3);
      rnd[0] = philox_start(rowG + (uint64_t)((jw0 + 8 * hh) >> 3), 0u);
      rnd[1] = philox_start(rowG + (uint64_t)((jw0 + 16 + 8 * hh) >> 3), 0u);
    }
    float dvv[16], ds[16];  // D = P o M / (1 - p) and dS of this lane's row, key slot e
    float16_t stn, ddn;
#pragma unroll
    for (int e = 0; e < 16; ++e) { stn[e] = 0.f; ddn[e] = 0.f; }
    {
      constexpr int kAhead = 2, KH = KC / 2;  // first half of the pairs: Philox; second half: exponentials, dropout, dS
      bf16x8_t qa[kAhead], va[kAhead], da[kAhead];
      const uint16_t* qrow = stage_q(itn) + (32 * is + li) * KP + 8 * hh;
      const uint16_t* drow = qrow + TILE;
#pragma unroll
      for (int a = 0; a < kAhead; ++a) {
        qa[a] = ld_frag(qrow + 16 * a);
        va[a] = ld_frag(vw + 16 * a), da[a] = ld_frag(drow + 16 * a);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int kc = 0; kc < KC; ++kc) {
        stn = mfma32(kf[kc], qa[kc % kAhead], stn);
        ddn = mfma32(va[kc % kAhead], da[kc % kAhead], ddn);
        if (kc + kAhead < KC) {
          qa[kc % kAhead] = ld_frag(qrow + 16 * (kc + kAhead));
          va[kc % kAhead] = ld_frag(vw + 16 * (kc + kAhead)), da[kc % kAhead] = ld_frag(drow + 16 * (kc + kAhead));
        }
        {  // rounds 1 .. PER-1 of the Q tile, then of the dO tile, of the block two steps ahead
          constexpr int PER = DmaMap<D>::PER;
          static_assert(2 * (PER - 1) <= KC, "more load rounds than pairs of matrix instructions");
          if (1 + kc < PER) dma_one<D>(map, qg + (int64_t)(it2 * BI) * gstride, nxt, wave, 1 + kc);
          else if (2 + kc - PER < PER) dma_one<D>(map, dog + (int64_t)(it2 * BI) * gstride, nxt + TILE, wave, 2 + kc - PER);
        }
        // this pair's share of tile it's vector work
        if (kc < KH) {
          if constexpr (DROP) {
#pragma unroll
            for (int r = 10 * kc / KH; r < 10 * (kc + 1) / KH; ++r) {
              philox_round(rnd[0], P.key0, P.key1, r);
              philox_round(rnd[1], P.key0, P.key1, r);
            }
          }
        } else {
#pragma unroll
          for (int e = 16 * (kc - KH) / (KC - KH); e < 16 * (kc - KH + 1) / (KC - KH); ++e) {
            const float pe = __builtin_amdgcn_exp2f(fmaf(st[e], sc2, -lse2));
            const float km = (!DROP || keep_field(rnd[e >> 3], e & 7, P.thresh)) ? P.keep_scale : 0.f;
            dvv[e] = pe * km;
            ds[e] = pe * (dd[e] * km - dl);
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    // ---- phase B: the one-key-per-lane copies and the dV / dK products of tile it ----
    bf16x8_t df[2], dsf[2];
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      df[c] = pack8(dvv + 8 * c);
      dsf[c] = pack8(ds + 8 * c);
    }
    if constexpr (WDS) ds_store2(ds_tile, lane, dsf[0], dsf[1]);
    float16_t tD, tS;
#pragma unroll
    for (int e = 0; e < 16; ++e) { tD[e] = 0.f; tS[e] = 0.f; }
    tD = mfma32(df[0], ident[0], tD);
    tS = mfma32(dsf[0], ident[0], tS);
    tD = mfma32(df[1], ident[1], tD);
    tS = mfma32(dsf[1], ident[1], tS);
    const uint16_t* Qs = stage_q(it);
    const uint16_t* dOs = Qs + TILE;
    {
      // acc[4g + r] <-> row 8g + 4hh + r: operand X takes g in {2X, 2X+1}, i.e. rows 16X + 8*(e>>2) + 4hh + (e&3).
      // The transposed operand reads run kAhead pairs of products ahead, written out (left to the compiler at this register
      // pressure, every product waits for a read issued just before it).
      bf16x8_t dT[2], sT[2];
#pragma unroll
      for (int X = 0; X < 2; ++X) {
        float td[8], ts[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) { td[e] = tD[8 * X + e]; ts[e] = tS[8 * X + e]; }
        dT[X] = pack8(td);
        sT[X] = pack8(ts);
      }
      constexpr int kAhead = 2, NP = 2 * DT;
      bf16x8_t fo[kAhead], fq[kAhead];
#pragma unroll
      for (int a = 0; a < kAhead; ++a) {
        fo[a] = ld_frag_tr_perm(dOs, KP, 32 * is + 16 * (a / DT), 32 * (a % DT), lane);
        fq[a] = ld_frag_tr_perm(Qs, KP, 32 * is + 16 * (a / DT), 32 * (a % DT), lane);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int pidx = 0; pidx < NP; ++pidx) {
        const int X = pidx / DT, dt = pidx % DT;
        dvacc[dt] = mfma32(fo[pidx % kAhead], dT[X], dvacc[dt]);
        dkacc[dt] = mfma32(fq[pidx % kAhead], sT[X], dkacc[dt]);
        if (pidx + kAhead < NP) {
          const int X2 = (pidx + kAhead) / DT, dt2 = (pidx + kAhead) % DT;
          fo[pidx % kAhead] = ld_frag_tr_perm(dOs, KP, 32 * is + 16 * X2, 32 * dt2, lane);
          fq[pidx % kAhead] = ld_frag_tr_perm(Qs, KP, 32 * is + 16 * X2, 32 * dt2, lane);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    if constexpr (WDS) {
      ds_tile += ds_step;
      if (P.causal) ds_step += kDsTileElems;
    }
    st = stn;
    dd = ddn;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      asm volatile("" : "+" SAR_COLS_ACC(dkacc[dt]));
      asm volatile("" : "+" SAR_COLS_ACC(dvacc[dt]));
    }
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) asm volatile("" : "+a"(kf[kc]));
  }
  // ---- sum the two row halves, scale, store ----
  dma_wait();  // the last steps' loads still target stages that the exchange buffers overlap
  __syncthreads();
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

// whether the pipelined kernel takes this shape; force: -1 = the library's choice, 0 / 1 = never / whenever possible
template <int D>
static inline bool bwd_dkdv_use_pipe(const AttnParams& P, int force) {
  if (D < 128 || P.s % 64 != 0 || force == 0) return false;
  return force == 1 || D == 128;
}

template <int D>
static hipError_t bwd_dkdv_pipe_d(const AttnParams& P, const void* q, const void* k, const void* v, const float* lse, const void* dO, const float* delta,
                                  void* dk, void* dv, uint16_t* ds_ws, hipStream_t st) {
  const int N = P.b * P.A, nb = P.s / 64;
  auto go = [&](auto kern) {
    hipLaunchKernelGGL(kern, dim3((unsigned)(nb * N)), dim3(256), 0, st, P, (const uint16_t*)q, (const uint16_t*)k, (const uint16_t*)v, lse,
                       (const uint16_t*)dO, delta, (uint16_t*)dk, (uint16_t*)dv, ds_ws);
  };
  if (ds_ws) {
    if (P.thresh != 0) go(attn_bwd_dkdv_pipe_kernel<D, true, true>);
    else go(attn_bwd_dkdv_pipe_kernel<D, false, true>);
  } else {
    if (P.thresh != 0) go(attn_bwd_dkdv_pipe_kernel<D, true, false>);
    else go(attn_bwd_dkdv_pipe_kernel<D, false, false>);
  }
  return hipGetLastError();
}

}  // namespace sar
