// bf16 attention core, the backward that recomputes the region of Section 5 once.
//
// The two-pass backward (attn_mfma_rows.hip row pass + column pass) regenerates softmax, the dropout mask and dO V^T in
// both passes, because dQ sums over keys and dK / dV over queries.  Here the column pass, which has every dS tile in
// registers anyway, also writes it out as bf16 (a backward-only scratch: nothing of it is kept from the forward), and dQ
// becomes a plain batched product over those tiles:
//   1. attn_bwd_delta_kernel      delta_i = sum_x dO_ix O_ix                      (reads dO, O once)
//   2. attn_bwd_dkdv_mfma_kernel  dK, dV, and dS tiles          (attn_mfma_cols_kernel.h, WDS = true)
//   3. attn_bwd_dq_gemm_kernel    dQ = alpha dS K                                  (reads the tiles and K)
// 5 contractions are executed instead of 7, and Philox and the exponentials run once per backward instead of twice.
#include "attn_mfma_common.h"

namespace sar {

// ---------------------------------------------------------------------------------------------------
// delta: one workgroup per 64 rows of one (batch, head).  Thread t takes the 16-byte chunks t, t + 256, ... of the
// block (chunk c = row c / CPR, piece c % CPR), the partial dot products meet in LDS and 64 threads add each row's
// CPR pieces in a fixed order (deterministic).
// ---------------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void attn_bwd_delta_kernel(AttnParams P, const uint16_t* __restrict__ o, const uint16_t* __restrict__ dO,
                                                            float* __restrict__ delta) {
  constexpr int CPR = D / 8, NCH = 64 * CPR;
  __shared__ float part[NCH];
  const int bn = blockIdx.y, beta = bn / P.A, n = bn % P.A;
  const int i0 = blockIdx.x * 64;
  const int64_t base = (int64_t)beta * P.stride_b + (int64_t)n * P.stride_a;
#pragma unroll
  for (int u = 0; u < (NCH + 255) / 256; ++u) {
    const int c = threadIdx.x + 256 * u;
    if (c < NCH) {
      const int r = c / CPR, cc = c - r * CPR;
      const int i = min(i0 + r, P.s - 1);
      const int64_t off = base + (int64_t)i * P.stride_s + 8 * cc;
      part[c] = dot8(ld_frag(dO + off), ld_frag(o + off));
    }
  }
  __syncthreads();
  if (threadIdx.x < 64 && i0 + (int)threadIdx.x < P.s) {
    float t = 0.f;
#pragma unroll
    for (int cc = 0; cc < CPR; ++cc) t += part[threadIdx.x * CPR + cc];
    delta[(size_t)bn * P.s + i0 + threadIdx.x] = t;
  }
}

// ---------------------------------------------------------------------------------------------------
// dQ = alpha dS K.  Workgroup = 64 query rows: 4 computing waves = 2 row groups x 2 key halves of each 64-key tile (summed
// through LDS at the end, as in the row pass of the two-pass backward) and 4 waves, one per SIMD, that only fetch the K
// tiles (rows swapped inside groups of 32, see attn_mfma_rows.hip) global -> LDS in pairs (one barrier per two tiles: the fixed cost of a barrier-to-barrier section, about 600 cycles
// beside 320 of matrix work per tile, is paid half as often), three stages of a pair each, two pairs ahead.
// The dS operand of a computing wave is 16 bytes per lane and 16-key group, read straight from the tile in the order
// the column pass wrote it, kDsAhead tiles ahead: the pass does little arithmetic per byte, so what bounds it is how many
// bytes a CU keeps in flight.  The computing waves issue no direct-to-LDS loads, so the compiler's own bookkeeping of
// their outstanding loads is exact and each step waits for its own operands only.
// ---------------------------------------------------------------------------------------------------
static constexpr int kDsAhead = 6;  // even: a round of the register ring is a whole number of tile pairs

template <int D>
__global__ __launch_bounds__(512, 1) void attn_bwd_dq_gemm_kernel(AttnParams P, const uint16_t* __restrict__ k, const uint16_t* __restrict__ ds_ws,
                                                                 uint16_t* __restrict__ dq) {
  constexpr int BM = 64, BN = 64, KP = D + 8, DT = D / 32, NS = 3;
  constexpr int TILE = BN * KP;
  // K stages of two tiles each (one barrier per pair of tiles); afterwards the exchange buffers, then the output tile
  __shared__ __attribute__((aligned(16))) uint16_t smem[NS * 2 * TILE];
  auto stage = [&](int jt) __attribute__((always_inline)) { return smem + (((jt >> 1) % NS) * 2 + (jt & 1)) * TILE; };

  const int N = P.b * P.A;
  const int nrb = (P.s + BM - 1) / BM;
  const int rb = nrb - 1 - (int)(blockIdx.x / N);  // heaviest row blocks first
  const int bn = blockIdx.x % N, beta = bn / P.A, n = bn % P.A;
  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, li = lane & 31, hh = lane >> 5;
  const int64_t base = (int64_t)beta * P.stride_b + (int64_t)n * P.stride_a;
  const int gstride = (int)P.stride_s;
  const int ntile = P.causal ? rb + 1 : nrb;
  if (wave >= 4) {  // a loader: same barriers as the computing waves
    const int lw = wave - 4;
    const uint16_t* kg = k + base;
    DmaMap<D> map;
    map.init(lw, lane, gstride, true);
    auto fetch = [&](int jt) __attribute__((always_inline)) {
      const int left = P.s - jt * BN;
      uint16_t* st2 = stage(jt);
      if (left >= BN) dma_tile<D>(map, kg + (int64_t)(jt * BN) * gstride, st2, lw);
      else dma_tile_ragged<D>(map, kg + (int64_t)(jt * BN) * gstride, st2, lw, lane, gstride, left);
    };
    for (int jt = 0; jt < 4 && jt < ntile; ++jt) fetch(jt);  // pairs 0 and 1
    for (int jt = 0; jt < ntile; jt += 2) {
      // the pair (jt, jt + 1) has landed; the loads of the next pair (at least DmaMap::PER - 1 per wave and tile) may
      // still be in flight
      const int later = ntile - (jt + 2);
      if (later >= 2) dma_wait_keep<2 * (DmaMap<D>::PER - 1)>();
      else if (later == 1) dma_wait_keep<DmaMap<D>::PER - 1>();
      else dma_wait();
      __syncthreads();  // top of the pair: its tiles are there, and nobody reads the pair before it (whose stage the pair after next takes) any more
      if (jt + 4 < ntile) fetch(jt + 4);
      if (jt + 5 < ntile) fetch(jt + 5);
    }
    __syncthreads();  // the four barriers of the others' epilogue
    __syncthreads();
    __syncthreads();
    __syncthreads();
    return;
  }
  const int rg = wave & 1, ks = wave >> 1;
  // this wave's 2 KB of tile (it = rb, kb = jt): key group c at + 512 c
  const uint16_t* dsw = ds_ws + (int64_t)bn * ds_tiles_per_head(P) * kDsTileElems + (2 * rg + ks) * 1024 + 8 * lane;
  auto ds_tile = [&](int jt) __attribute__((always_inline)) { return dsw + ds_tile_index(P, rb, jt) * kDsTileElems; };

  float16_t dqacc[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int e = 0; e < 16; ++e) dqacc[dt][e] = 0.f;

  // One step: K tile jt against this wave's dS operands.  The operand reads run kAhead matrix instructions ahead, written
  // out (left to the compiler, every matrix instruction waits for a read issued just before it).
  auto step = [&](const int jt, bf16x8_t d0, bf16x8_t d1) __attribute__((always_inline)) {
    // the upper right quarter of the diagonal tile lies above the diagonal
    if (P.causal && jt == rb && rg == 0 && ks == 1) {
      const u32x4_t zero = {0u, 0u, 0u, 0u};
      d0 = __builtin_bit_cast(bf16x8_t, zero);
      d1 = __builtin_bit_cast(bf16x8_t, zero);
    }
    const uint16_t* Ks = stage(jt);
    constexpr int kAhead = 3, NF = 2 * DT;
    bf16x8_t fr[kAhead];
#pragma unroll
    for (int a = 0; a < kAhead; ++a) fr[a] = ld_frag_tr_perm(Ks, KP, 32 * ks + 16 * (a / DT), 32 * (a % DT), lane);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int f = 0; f < NF; ++f) {
      dqacc[f % DT] = mfma32(fr[f % kAhead], f < DT ? d0 : d1, dqacc[f % DT]);
      if (f + kAhead < NF) fr[f % kAhead] = ld_frag_tr_perm(Ks, KP, 32 * ks + 16 * ((f + kAhead) / DT), 32 * ((f + kAhead) % DT), lane);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // dS operands kDsAhead tiles ahead, in a ring of registers with compile-time slots.  The main loop takes whole rounds of
  // the ring and has no condition inside (a load past the last tile re-reads the last tile); the remaining steps follow
  // without further loads.
  bf16x8_t ring[kDsAhead][2];
#pragma unroll
  for (int u = 0; u < kDsAhead; ++u) {
    const uint16_t* t = ds_tile(min(u, ntile - 1));
    ring[u][0] = ld_frag(t);
    ring[u][1] = ld_frag(t + 512);
  }
  int jt0 = 0;
  for (; jt0 + kDsAhead <= ntile; jt0 += kDsAhead) {
#pragma unroll
    for (int u = 0; u < kDsAhead; ++u) {
      if ((u & 1) == 0) __syncthreads();  // K tiles jt0 + u and jt0 + u + 1 are in their stage
      step(jt0 + u, ring[u][0], ring[u][1]);
      // refilled only now, when its last reader has been issued: the new load can then land in the same registers (loaded
      // at the top of the step it needs registers of its own, and the compiler moves every slot's value, load waited
      // for, around the back-edge)
      const uint16_t* t = ds_tile(min(jt0 + u + kDsAhead, ntile - 1));
      ring[u][0] = ld_frag(t);
      ring[u][1] = ld_frag(t + 512);
    }
  }
#pragma unroll
  for (int u = 0; u < kDsAhead - 1; ++u)
    if (jt0 + u < ntile) {
      if ((u & 1) == 0) __syncthreads();
      step(jt0 + u, ring[u][0], ring[u][1]);
    }
  // ---- sum the two key halves, scale, store ----
  __syncthreads();
  float* mg = reinterpret_cast<float*>(smem) + rg * (64 * 16 * DT);
  if (ks == 1) acc_put<DT>(mg, dqacc, lane);
  __syncthreads();
  if (ks == 0) acc_combine<DT>(mg, dqacc, 1.f, 1.f, lane);
  __syncthreads();  // the output tile overlaps both exchange buffers
  if (ks == 0) acc_to_lds_rows<DT>(smem, KP, 32 * rg + li, dqacc, P.scale, hh);
  __syncthreads();
  lds_rows_to_global<D>(smem, dq + base + (int64_t)(rb * BM) * P.stride_s, gstride, P.s - rb * BM, tid);
}

template <int D>
static hipError_t bwd_once_d(const AttnParams& P, const void* q, const void* k, const void* v, const void* o, const float* lse, const void* dO, void* dq,
                             void* dk, void* dv, float* delta, uint16_t* ds_ws, int stages, hipStream_t st) {
  const int N = P.b * P.A, nb = (P.s + 63) / 64;
  hipError_t e = hipSuccess;
  if (stages & 1) {
    hipLaunchKernelGGL((attn_bwd_delta_kernel<D>), dim3((unsigned)nb, (unsigned)N), dim3(256), 0, st, P, (const uint16_t*)o, (const uint16_t*)dO, delta);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  if (stages & 2) {
    if ((e = launch_attn_bwd_dkdv_mfma(P, q, k, v, lse, dO, delta, dk, dv, ds_ws, st)) != hipSuccess) return e;
  }
  if (stages & 4) {
    hipLaunchKernelGGL((attn_bwd_dq_gemm_kernel<D>), dim3((unsigned)(nb * N)), dim3(512), 0, st, P, (const uint16_t*)k, (const uint16_t*)ds_ws,
                       (uint16_t*)dq);
    e = hipGetLastError();
  }
  return e;
}

hipError_t launch_attn_bwd_once_mfma(const AttnParams& P, const void* q, const void* k, const void* v, const void* o, const float* lse,
                                     const void* dO, void* dq, void* dk, void* dv, float* delta, uint16_t* ds_ws, int stages, hipStream_t st) {
  switch (P.d) {
    case 64: return bwd_once_d<64>(P, q, k, v, o, lse, dO, dq, dk, dv, delta, ds_ws, stages, st);
    case 96: return bwd_once_d<96>(P, q, k, v, o, lse, dO, dq, dk, dv, delta, ds_ws, stages, st);
    case 128: return bwd_once_d<128>(P, q, k, v, o, lse, dO, dq, dk, dv, delta, ds_ws, stages, st);
    case 160: return bwd_once_d<160>(P, q, k, v, o, lse, dO, dq, dk, dv, delta, ds_ws, stages, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace sar
