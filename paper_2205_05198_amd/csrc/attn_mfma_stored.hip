// bf16 attention core, stored-activation baseline on gfx950 matrix cores (Section 4.1): the same 64 x 64 tiles as
// the recompute kernels, but the softmax output P, the dropout mask M and the dropout output D are written to
// global memory by the forward and read back by the backward instead of being recomputed.
//   forward  = the recompute forward (O, LSE) followed by attn_store_pmd_mfma_kernel (P, M, D from Q, K, LSE)
//   backward = attn_bwd_dq_stored_mfma_kernel (dQ, delta) + attn_bwd_dkdv_stored_mfma_kernel (dK, dV)
// Needs s % 64 == 0 (every P / M / D tile is a full 64 x 64 block with 128-byte rows).  See attn_mfma_rows.hip for
// the operand layouts.  This file is compiled without -amdgpu-mfma-vgpr-form, like the dK/dV pass.
#include "attn_mfma_common.h"

namespace sar {

static constexpr int kSP = 72;  // pitch (bf16 elements) of a 64 x 64 P or D tile in LDS: 8 data chunks + 1 of padding
static constexpr int kSM = 80;  // pitch (bytes) of a 64 x 64 M tile in LDS: 4 data chunks + 1 of padding

__device__ __forceinline__ void unpack8(bf16x8_t f, float* out) {
  union { bf16x8_t v; uint32_t w[4]; } u;
  u.v = f;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    out[2 * e] = __uint_as_float(u.w[e] << 16);
    out[2 * e + 1] = __uint_as_float(u.w[e] & 0xffff0000u);
  }
}

// ===================================================================================================
// P, M, D of one block of 64 query rows against every key tile.  wave = (rg, ks) as in the forward; one query
// row per lane, so a lane holds 8 consecutive keys of its row per register group: 16 bytes of P and D, 8 of M.
// They go through an LDS tile and leave with 16-byte accesses that run along the rows (128 bytes of P and D and
// 64 of M per row and tile).  Tiles above the diagonal are written as zeros.
// ===================================================================================================
template <int D, bool DROP>
__global__ __launch_bounds__(256) void attn_store_pmd_mfma_kernel(AttnParams P, const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
                                                                 const float* __restrict__ lse, uint16_t* __restrict__ Pst, uint8_t* __restrict__ Mst,
                                                                 uint16_t* __restrict__ Dst) {
  constexpr int BM = 64, BN = 64, KP = D + 8, KC = D / 16;
  constexpr int TILE = BN * KP;
  __shared__ __attribute__((aligned(16))) uint16_t smem[2 * TILE + 2 * 64 * kSP + 64 * kSM / 2];
  uint16_t* Pt = smem + 2 * TILE;
  uint16_t* Dt = Pt + 64 * kSP;
  uint8_t* Mt = reinterpret_cast<uint8_t*>(Dt + 64 * kSP);

  const int N = P.b * P.A;
  const int rb = (int)(blockIdx.x / N);
  const int bn = blockIdx.x % N, beta = bn / P.A, n = bn % P.A;
  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, li = lane & 31, hh = lane >> 5;
  const int rg = wave & 1, ks = wave >> 1;
  const int64_t base = (int64_t)beta * P.stride_b + (int64_t)n * P.stride_a;
  const int gstride = (int)P.stride_s;
  const int i = rb * BM + rg * 32 + li;  // < s: s is a multiple of 64

  bf16x8_t qf[KC];
#pragma unroll
  for (int kc = 0; kc < KC; ++kc) qf[kc] = ld_frag(q + base + (int64_t)i * P.stride_s + 16 * kc + 8 * hh);
#pragma unroll
  for (int kc = 0; kc < KC; ++kc) asm volatile("" : "+v"(qf[kc]));
  const float lse2 = lse[(size_t)bn * P.s + i] * kLog2e;
  const uint64_t rowG = P.offset + (((uint64_t)beta * (uint64_t)P.a_global + (uint64_t)(P.head0 + n)) * (uint64_t)P.s + (uint64_t)i) * (uint64_t)(P.s >> 3);
  const float sc2 = P.scale * kLog2e;

  const int nt_all = P.s / BN, nt = P.causal ? rb + 1 : nt_all;
  DmaMap<D> map;
  map.init(wave, lane, gstride, true);
  const uint16_t* kg = k + base;
  dma_tile<D>(map, kg, smem, wave);
  const size_t srow0 = ((size_t)bn * P.s + (size_t)rb * BM) * (size_t)P.s;  // element index of (row rb*64, key 0)
  for (int jt = 0; jt < nt_all; ++jt) {
    const int j0 = jt * BN;
    if (jt < nt) {
      dma_wait();
      __syncthreads();  // K tile jt is complete; everybody has copied the previous tile out of the staging tiles
      if (jt + 1 < nt) dma_tile<D>(map, kg + (int64_t)(j0 + BN) * gstride, smem + ((jt + 1) & 1) * TILE, wave);
      const uint16_t* Ks = smem + (jt & 1) * TILE;
      float16_t st;
#pragma unroll
      for (int e = 0; e < 16; ++e) st[e] = 0.f;
#pragma unroll
      for (int kc = 0; kc < KC; ++kc) st = mfma32(ld_frag(Ks + (32 * ks + li) * KP + 16 * kc + 8 * hh), qf[kc], st);
      const int j0w = j0 + 32 * ks;
      const bool diag = P.causal && jt == nt - 1;
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        const int jc = j0w + 16 * c + 8 * hh;
        Philox4 rnd = {0u, 0u, 0u, 0u};
        if (DROP) rnd = philox_call8(rowG + (uint64_t)(jc >> 3), 0u, P.key0, P.key1);
        float pv[8], dv[8];
        uint32_t mlo = 0, mhi = 0;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const bool in = !diag || jc + e <= i;
          const float pe = in ? __builtin_amdgcn_exp2f(fmaf(st[8 * c + e], sc2, -lse2)) : 0.f;
          const bool kp = in && (!DROP || keep_field(rnd, e, P.thresh));
          pv[e] = pe;
          dv[e] = kp ? pe * P.keep_scale : 0.f;
          if (e < 4) mlo |= (kp ? 1u : 0u) << (8 * e);
          else mhi |= (kp ? 1u : 0u) << (8 * (e - 4));
        }
        const int col = 32 * ks + 16 * c + 8 * hh;
        *reinterpret_cast<bf16x8_t*>(Pt + (32 * rg + li) * kSP + col) = pack8(pv);
        *reinterpret_cast<bf16x8_t*>(Dt + (32 * rg + li) * kSP + col) = pack8(dv);
        *reinterpret_cast<uint2*>(Mt + (32 * rg + li) * kSM + col) = make_uint2(mlo, mhi);
      }
      __syncthreads();
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int c = tid + 256 * u, r = c >> 3, cc = c & 7;
        const size_t g = srow0 + (size_t)r * P.s + j0 + 8 * cc;
        *reinterpret_cast<u32x4_t*>(Pst + g) = *reinterpret_cast<const u32x4_t*>(Pt + r * kSP + 8 * cc);
        *reinterpret_cast<u32x4_t*>(Dst + g) = *reinterpret_cast<const u32x4_t*>(Dt + r * kSP + 8 * cc);
      }
      {
        const int r = tid >> 2, cc = tid & 3;
        *reinterpret_cast<u32x4_t*>(Mst + srow0 + (size_t)r * P.s + j0 + 16 * cc) = *reinterpret_cast<const u32x4_t*>(Mt + r * kSM + 16 * cc);
      }
    } else {  // above the diagonal
      const u32x4_t z = {0u, 0u, 0u, 0u};
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int c = tid + 256 * u, r = c >> 3, cc = c & 7;
        const size_t g = srow0 + (size_t)r * P.s + j0 + 8 * cc;
        *reinterpret_cast<u32x4_t*>(Pst + g) = z;
        *reinterpret_cast<u32x4_t*>(Dst + g) = z;
      }
      const int r = tid >> 2, cc = tid & 3;
      *reinterpret_cast<u32x4_t*>(Mst + srow0 + (size_t)r * P.s + j0 + 16 * cc) = z;
    }
  }
}

// ===================================================================================================
// Backward, row pass with stored P, M: dP = (dO V^T) o M/(1-p), dS = P o (dP - delta), dQ = alpha dS K,
// delta_i = dO_i . O_i.  Same workgroup shape as the recompute pass; each stage holds a K, a V, a P and an M tile.
// ===================================================================================================
template <int D>
__global__ __launch_bounds__(256) void attn_bwd_dq_stored_mfma_kernel(AttnParams P, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
                                                                     const uint16_t* __restrict__ o, const uint16_t* __restrict__ dO,
                                                                     const uint16_t* __restrict__ Pst, const uint8_t* __restrict__ Mst,
                                                                     uint16_t* __restrict__ dq, float* __restrict__ delta) {
  constexpr int BM = 64, BN = 64, KP = D + 8, KC = D / 16, DT = D / 32;
  constexpr int TILE = BN * KP, STG = 2 * TILE + 64 * kSP + 64 * kSM / 2;
  __shared__ __attribute__((aligned(16))) uint16_t smem[2 * STG];

  const int N = P.b * P.A;
  const int nrb = P.s / BM;
  const int rb = nrb - 1 - (int)(blockIdx.x / N);
  const int bn = blockIdx.x % N, beta = bn / P.A, n = bn % P.A;
  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, li = lane & 31, hh = lane >> 5;
  const int rg = wave & 1, ks = wave >> 1;
  const int64_t base = (int64_t)beta * P.stride_b + (int64_t)n * P.stride_a;
  const int gstride = (int)P.stride_s;
  const int i = rb * BM + rg * 32 + li;

  bf16x8_t dof[KC];
  float dpart = 0.f;
#pragma unroll
  for (int kc = 0; kc < KC; ++kc) {
    const int64_t off = base + (int64_t)i * P.stride_s + 16 * kc + 8 * hh;
    dof[kc] = ld_frag(dO + off);
    dpart += dot8(dof[kc], ld_frag(o + off));
  }
#pragma unroll
  for (int kc = 0; kc < KC; ++kc) asm volatile("" : "+v"(dof[kc]));
  const float dl = dpart + __shfl_xor(dpart, 32, 64);
  if (ks == 0 && hh == 0) delta[(size_t)bn * P.s + i] = dl;

  float16_t dqacc[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int e = 0; e < 16; ++e) dqacc[dt][e] = 0.f;

  const int ntile = P.causal ? rb + 1 : P.s / BN;
  DmaMap<D> mapkv;
  mapkv.init(wave, lane, gstride, true);
  DmaMap<64> mapp;
  mapp.init(wave, lane, P.s, false);
  DmaMap<32> mapm;
  mapm.init(wave, lane, P.s / 2, false);
  const uint16_t* kg = k + base;
  const uint16_t* vg = v + base;
  const size_t srow0 = ((size_t)bn * P.s + (size_t)rb * BM) * (size_t)P.s;
  auto load = [&](int jt) __attribute__((always_inline)) {
    uint16_t* st = smem + (jt & 1) * STG;
    dma_tile<D>(mapkv, kg + (int64_t)(jt * BN) * gstride, st, wave);
    dma_tile<D>(mapkv, vg + (int64_t)(jt * BN) * gstride, st + TILE, wave);
    dma_tile<64>(mapp, Pst + srow0 + (size_t)jt * BN, st + 2 * TILE, wave);
    dma_tile<32>(mapm, reinterpret_cast<const uint16_t*>(Mst + srow0 + (size_t)jt * BN), st + 2 * TILE + 64 * kSP, wave);
  };
  load(0);
  for (int jt = 0; jt < ntile; ++jt) {
    dma_wait();
    __syncthreads();
    if (jt + 1 < ntile) load(jt + 1);
    const uint16_t* Ks = smem + (jt & 1) * STG;
    const uint16_t* Vs = Ks + TILE;
    const uint16_t* Pt = Ks + 2 * TILE;
    const uint8_t* Mt = reinterpret_cast<const uint8_t*>(Pt + 64 * kSP);
    float16_t dd;
#pragma unroll
    for (int e = 0; e < 16; ++e) dd[e] = 0.f;
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) dd = mfma32(ld_frag(Vs + (32 * ks + li) * KP + 16 * kc + 8 * hh), dof[kc], dd);
    bf16x8_t dsf[2];
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      const int col = 32 * ks + 16 * c + 8 * hh;
      float pv[8], ds[8];
      unpack8(ld_frag(Pt + (32 * rg + li) * kSP + col), pv);
      const uint2 m = *reinterpret_cast<const uint2*>(Mt + (32 * rg + li) * kSM + col);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const uint32_t kp = ((e < 4 ? m.x : m.y) >> (8 * (e & 3))) & 0xffu;
        const float dp = kp ? dd[8 * c + e] * P.keep_scale : 0.f;
        ds[e] = pv[e] * (dp - dl);
      }
      dsf[c] = pack8(ds);
    }
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) dqacc[dt] = mfma32(ld_frag_tr_perm(Ks, KP, 32 * ks + 16 * c, 32 * dt, lane), dsf[c], dqacc[dt]);
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
  lds_rows_to_global<D>(smem + 2 * TILE, dq + base + (int64_t)(rb * BM) * P.stride_s, gstride, BM, tid);
}

// ===================================================================================================
// Backward, column pass with stored P, M, D: dV_j = sum_i D_ij dO_i with the D tile read transposed straight from
// LDS; dK_j = alpha sum_i dS_ij q_i with dS rebuilt from P, M and dO V^T and moved to the transposed layout by an
// identity MFMA, as in the recompute pass.  wave = (kgp, is).
// ===================================================================================================
template <int D>
__global__ __launch_bounds__(256) void attn_bwd_dkdv_stored_mfma_kernel(AttnParams P, const uint16_t* __restrict__ q, const uint16_t* __restrict__ v,
                                                                       const uint16_t* __restrict__ dO, const float* __restrict__ delta,
                                                                       const uint16_t* __restrict__ Pst, const uint8_t* __restrict__ Mst,
                                                                       const uint16_t* __restrict__ Dst, uint16_t* __restrict__ dk,
                                                                       uint16_t* __restrict__ dv) {
  constexpr int BN = 64, BI = 64, KP = D + 8, KC = D / 16, DT = D / 32;
  constexpr int TILE = 64 * KP, STG = 2 * TILE + 2 * 64 * kSP + 64 * kSM / 2;
  constexpr int SMEM = (TILE + 2 * STG) > 6 * TILE ? (TILE + 2 * STG) : 6 * TILE;  // the epilogue uses six tiles' worth
  __shared__ __attribute__((aligned(16))) uint16_t smem[SMEM];
  __shared__ float delta_s[2][BI];
  uint16_t* Vsm = smem;
  uint16_t* stages = smem + TILE;  // two stages of (Q, dO, P, D, M)

  const int N = P.b * P.A;
  const int kb = (int)(blockIdx.x / N);
  const int bn = blockIdx.x % N, beta = bn / P.A, n = bn % P.A;
  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, li = lane & 31, hh = lane >> 5;
  const int kgp = wave & 1, is = wave >> 1;
  const int64_t base = (int64_t)beta * P.stride_b + (int64_t)n * P.stride_a;
  const int gstride = (int)P.stride_s;

  const int nit = P.s / BI;
  const int it0 = P.causal ? kb : 0;
  const uint16_t* qg = q + base;
  const uint16_t* dog = dO + base;
  DmaMap<D> mapv, mapq;
  mapv.init(wave, lane, gstride, true);
  mapq.init(wave, lane, gstride, false);
  DmaMap<64> mapp;
  mapp.init(wave, lane, P.s, false);
  DmaMap<32> mapm;
  mapm.init(wave, lane, P.s / 2, false);
  const size_t scol0 = (size_t)bn * P.s * (size_t)P.s + (size_t)kb * BN;  // element index of (row 0, key kb*64)
  auto load = [&](int it) __attribute__((always_inline)) {
    uint16_t* st = stages + (it & 1) * STG;
    const size_t g = scol0 + (size_t)it * BI * (size_t)P.s;
    dma_tile<D>(mapq, qg + (int64_t)(it * BI) * gstride, st, wave);
    dma_tile<D>(mapq, dog + (int64_t)(it * BI) * gstride, st + TILE, wave);
    dma_tile<64>(mapp, Pst + g, st + 2 * TILE, wave);
    dma_tile<64>(mapp, Dst + g, st + 2 * TILE + 64 * kSP, wave);
    dma_tile<32>(mapm, reinterpret_cast<const uint16_t*>(Mst + g), st + 2 * TILE + 2 * 64 * kSP, wave);
  };
  dma_tile<D>(mapv, v + base + (int64_t)(kb * BN) * gstride, Vsm, wave);
  load(it0);
  // delta of the tile's rows goes straight into LDS like the tile (a register load would make wave 0 wait for its tile loads)
  if (wave == 0) dma4(delta + (size_t)bn * P.s + it0 * BI + lane, lds_addr(delta_s[it0 & 1]));
  const uint16_t* vw = Vsm + (32 * kgp + li) * KP + 8 * hh;  // LDS row 32*kgp + li holds key kb*64 + 32*kgp + perm_row(li)
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

  for (int it = it0; it < nit; ++it) {
    dma_wait();
    __syncthreads();
    if (it + 1 < nit) {
      load(it + 1);
      if (wave == 0) dma4(delta + (size_t)bn * P.s + (it + 1) * BI + lane, lds_addr(delta_s[(it + 1) & 1]));
    }
    const uint16_t* Qs = stages + (it & 1) * STG;
    const uint16_t* dOs = Qs + TILE;
    const uint16_t* Pt = Qs + 2 * TILE;
    const uint16_t* Dt = Pt + 64 * kSP;
    const uint8_t* Mt = reinterpret_cast<const uint8_t*>(Dt + 64 * kSP);
    float16_t dd;
#pragma unroll
    for (int e = 0; e < 16; ++e) dd[e] = 0.f;
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) dd = mfma32(ld_frag(vw + 16 * kc), ld_frag(dOs + (32 * is + li) * KP + 16 * kc + 8 * hh), dd);
    const float dl = delta_s[it & 1][32 * is + li];
    bf16x8_t dsf[2];
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      const int col = 32 * kgp + 16 * c + 8 * hh;
      float pv[8], ds[8];
      unpack8(ld_frag(Pt + (32 * is + li) * kSP + col), pv);
      const uint2 m = *reinterpret_cast<const uint2*>(Mt + (32 * is + li) * kSM + col);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const uint32_t kp = ((e < 4 ? m.x : m.y) >> (8 * (e & 3))) & 0xffu;
        const float dp = kp ? dd[8 * c + e] * P.keep_scale : 0.f;
        ds[e] = pv[e] * (dp - dl);
      }
      dsf[c] = pack8(ds);
    }
    float16_t tS;
#pragma unroll
    for (int e = 0; e < 16; ++e) tS[e] = 0.f;
    tS = mfma32(dsf[0], ident[0], tS);
    tS = mfma32(dsf[1], ident[1], tS);
#pragma unroll
    for (int X = 0; X < 2; ++X) {
      float ts[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) ts[e] = tS[8 * X + e];
      const bf16x8_t sT = pack8(ts);
      const bf16x8_t dT = ld_frag_tr_perm(Dt, kSP, 32 * is + 16 * X, 32 * kgp, lane);  // D[rows of this operand][this wave's keys], transposed
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        dvacc[dt] = mfma32(ld_frag_tr_perm(dOs, KP, 32 * is + 16 * X, 32 * dt, lane), dT, dvacc[dt]);
        dkacc[dt] = mfma32(ld_frag_tr_perm(Qs, KP, 32 * is + 16 * X, 32 * dt, lane), sT, dkacc[dt]);
      }
    }
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      asm volatile("" : "+a"(dkacc[dt]));
      asm volatile("" : "+a"(dvacc[dt]));
    }
  }
  // ---- sum the two row halves, scale, store ----
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
  lds_rows_to_global<D>(smem + 4 * TILE, dk + base + (int64_t)(kb * BN) * P.stride_s, gstride, BN, tid);
  lds_rows_to_global<D>(smem + 5 * TILE, dv + base + (int64_t)(kb * BN) * P.stride_s, gstride, BN, tid);
}

bool attn_mfma_stored_supported(const AttnParams& P) { return attn_mfma_supported(P.d) && P.s % 64 == 0 && P.scale > 0.f; }

template <int D>
static hipError_t stored_fwd_d(const AttnParams& P, const void* q, const void* k, const float* lse, void* Pst, uint8_t* Mst, void* Dst, hipStream_t st) {
  const int N = P.b * P.A, nrb = P.s / 64;
  if (P.thresh != 0)
    hipLaunchKernelGGL((attn_store_pmd_mfma_kernel<D, true>), dim3((unsigned)(nrb * N)), dim3(256), 0, st, P, (const uint16_t*)q, (const uint16_t*)k, lse,
                       (uint16_t*)Pst, Mst, (uint16_t*)Dst);
  else
    hipLaunchKernelGGL((attn_store_pmd_mfma_kernel<D, false>), dim3((unsigned)(nrb * N)), dim3(256), 0, st, P, (const uint16_t*)q, (const uint16_t*)k, lse,
                       (uint16_t*)Pst, Mst, (uint16_t*)Dst);
  return hipGetLastError();
}

hipError_t launch_attn_store_pmd_mfma(const AttnParams& P, const void* q, const void* k, const float* lse, void* Pst, uint8_t* Mst, void* Dst,
                                      hipStream_t st) {
  switch (P.d) {
    case 64: return stored_fwd_d<64>(P, q, k, lse, Pst, Mst, Dst, st);
    case 96: return stored_fwd_d<96>(P, q, k, lse, Pst, Mst, Dst, st);
    case 128: return stored_fwd_d<128>(P, q, k, lse, Pst, Mst, Dst, st);
    case 160: return stored_fwd_d<160>(P, q, k, lse, Pst, Mst, Dst, st);
    default: return hipErrorInvalidValue;
  }
}

template <int D>
static hipError_t stored_bwd_d(const AttnParams& P, const void* q, const void* k, const void* v, const void* o, const void* dO, const void* Pst,
                               const uint8_t* Mst, const void* Dst, void* dq, void* dk, void* dv, float* delta, hipStream_t st) {
  const int N = P.b * P.A, nb = P.s / 64;
  hipLaunchKernelGGL((attn_bwd_dq_stored_mfma_kernel<D>), dim3((unsigned)(nb * N)), dim3(256), 0, st, P, (const uint16_t*)k, (const uint16_t*)v,
                     (const uint16_t*)o, (const uint16_t*)dO, (const uint16_t*)Pst, Mst, (uint16_t*)dq, delta);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((attn_bwd_dkdv_stored_mfma_kernel<D>), dim3((unsigned)(nb * N)), dim3(256), 0, st, P, (const uint16_t*)q, (const uint16_t*)v,
                     (const uint16_t*)dO, (const float*)delta, (const uint16_t*)Pst, Mst, (const uint16_t*)Dst, (uint16_t*)dk, (uint16_t*)dv);
  return hipGetLastError();
}

hipError_t launch_attn_bwd_stored_mfma(const AttnParams& P, const void* q, const void* k, const void* v, const void* o, const void* dO, const void* Pst,
                                       const uint8_t* Mst, const void* Dst, void* dq, void* dk, void* dv, float* delta, hipStream_t st) {
  switch (P.d) {
    case 64: return stored_bwd_d<64>(P, q, k, v, o, dO, Pst, Mst, Dst, dq, dk, dv, delta, st);
    case 96: return stored_bwd_d<96>(P, q, k, v, o, dO, Pst, Mst, Dst, dq, dk, dv, delta, st);
    case 128: return stored_bwd_d<128>(P, q, k, v, o, dO, Pst, Mst, Dst, dq, dk, dv, delta, st);
    case 160: return stored_bwd_d<160>(P, q, k, v, o, dO, Pst, Mst, Dst, dq, dk, dv, delta, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace sar
