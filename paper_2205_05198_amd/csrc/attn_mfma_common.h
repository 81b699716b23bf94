// Shared pieces of the bf16 matrix-core attention kernels (attn_mfma_rows.hip, attn_mfma_cols.hip, attn_mfma_stored.hip): MFMA wrapper,
// LDS operand loads, direct global -> LDS tile loads, output staging.
#pragma once
#include "sar_device.h"
#include "sar_internal.h"

namespace sar {


static constexpr float kLog2e = 1.4426950408889634f;
static constexpr float kLn2 = 0.6931471805599453f;

typedef __attribute__((address_space(3))) short4_t lds_short4_t;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4_t;

__device__ __forceinline__ float16_t mfma32(bf16x8_t a, bf16x8_t b, float16_t c) { return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0); }

// 16-byte operand from LDS / global (8 consecutive bf16)
__device__ __forceinline__ bf16x8_t ld_frag(const uint16_t* p) { return *reinterpret_cast<const bf16x8_t*>(p); }

__device__ __forceinline__ bf16x8_t pack8(const float* f) {
  union { uint32_t w[4]; bf16x8_t v; } u;
  u.w[0] = pack_bf16x2(f[0], f[1]);
  u.w[1] = pack_bf16x2(f[2], f[3]);
  u.w[2] = pack_bf16x2(f[4], f[5]);
  u.w[3] = pack_bf16x2(f[6], f[7]);
  return u.v;
}

// max of a value with the one held 32 lanes away (v_permlane32_swap exchanges the upper half of one register with the lower
// half of the other: afterwards one holds the lower half's values in both halves, the other the upper half's)
__device__ __forceinline__ float xhalf_max(float v) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// LDS row that holds row r (0..63) of a K tile: bits 2 and 3 swapped inside each group of 32 rows
__device__ __forceinline__ int perm_row(int r) { return (r & ~12) | ((r & 4) << 1) | ((r & 8) >> 1); }

// ---------------------------------------------------------------------------------------------------
// Direct global -> LDS tile loads (global_load_lds_dwordx4): lane L of a wave-wide load writes its 16 bytes
// at (wave-uniform LDS base, in M0) + 16 L, without passing through registers.  A tile of 64 rows whose LDS
// pitch is D + 8 elements = CPR + 1 chunks of 16 bytes (the last chunk of a row is padding) is exactly CPR + 1
// such loads of 64 consecutive chunks; wave w of the workgroup issues loads w, w + 4, ...  Lanes that fall
// on a padding chunk re-read the row's last chunk.  Several tiles with the same row stride (K and V, or Q and
// dO) share one offset table.
//
// The load is written as inline assembly on purpose.  Through the compiler's builtin every later LDS read is
// preceded by a wait for ALL outstanding direct loads (the compiler cannot tell the stage being filled from the
// stage being read), which serialises the pipeline.  The price: the compiler does not know about these loads, so
// the kernels wait for them explicitly (dma_wait) before the barrier that publishes a stage.
// ---------------------------------------------------------------------------------------------------
typedef __attribute__((address_space(3))) void lds_void_t;

__device__ __forceinline__ uint32_t lds_addr(const void* p) { return (uint32_t)(uintptr_t)(lds_void_t*)p; }
// The global address is a wave-uniform base (the tile's first row, in scalar registers) plus this lane's 32-bit byte
// offset: no 64-bit vector addition per load.
__device__ __forceinline__ void dma16(const void* gbase, uint32_t goff, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(goff), "s"(gbase), "s"(lds_base) : "m0");
}
// Same, pinned in the instruction stream: issued after `token` has been computed and before anything that uses
// `token` afterwards (the statement pretends to modify it).
template <typename T>
__device__ __forceinline__ void dma16(const void* gbase, uint32_t goff, uint32_t lds_base, T& token) {
  asm volatile("s_mov_b32 m0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" : "+v"(token) : "v"(goff), "s"(gbase), "s"(lds_base) : "m0");
}
// 4 bytes per lane: lane L writes at (LDS base) + 4 L (per-row statistics of a tile: one float per row)
__device__ __forceinline__ void dma4(const void* gaddr, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %0, off" : : "v"(gaddr), "s"(lds_base) : "m0");
}
// every direct load this wave has issued has landed in LDS
__device__ __forceinline__ void dma_wait() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
// all but the N most recent vector-memory operations of this wave have completed (the counter covers loads and stores
// alike and they complete in issue order): waits for direct loads without waiting for N stores or loads issued after them
template <int N>
__device__ __forceinline__ void dma_wait_keep() { asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory"); }

// NW = number of waves that share the loads of a tile (the whole workgroup)
template <int D, int NW = 4>
struct DmaMap {
  static constexpr int ROWS = 64, CPR = D / 8, NL = CPR + 1, PER = (NL + NW - 1) / NW;
  static constexpr int TILE = ROWS * (D + 8);  // elements of one LDS tile
  uint32_t goff[PER];                          // byte offset of this lane's chunk from the tile's first row
  bool perm;
  // rows_valid: rows of the tensor left from the tile's first row (reads of later rows are clamped to the last one)
  __device__ __forceinline__ void init(int wave, int lane, int gstride, bool perm_rows, int rows_valid = ROWS) {
    perm = perm_rows;
#pragma unroll
    for (int u = 0; u < PER; ++u) {
      const int L = 64 * (wave + NW * u) + lane, r0 = (L / NL) & (ROWS - 1), c0 = L - (L / NL) * NL;
      int r = perm_rows ? perm_row(r0) : r0;
      r = r < rows_valid ? r : rows_valid - 1;
      goff[u] = 2u * (uint32_t)(r * gstride + 8 * (c0 < CPR ? c0 : CPR - 1));
    }
  }
};

// gtile: first row of the tile in global memory (uniform); lds: the tile's place in LDS (uniform).
// dma_one issues round u (0 .. PER-1) of this wave's loads, so that callers can spread them between matrix
// instructions: the texture path accepts one such load every 16 cycles per CU, and a wave that issues its whole
// share back to back stalls until they are accepted.
template <int D, int NW>
__device__ __forceinline__ void dma_one(const DmaMap<D, NW>& map, const uint16_t* gtile, uint16_t* lds, int wave, int u) {
  const int l = wave + NW * u;
  if (u < DmaMap<D, NW>::PER - 1 || l < DmaMap<D, NW>::NL)  // only the last round can run past the tile
    dma16(gtile, map.goff[u], lds_addr(lds) + 1024u * (uint32_t)l);
}
template <int D, int NW>
__device__ __forceinline__ void dma_tile(const DmaMap<D, NW>& map, const uint16_t* gtile, uint16_t* lds, int wave) {
#pragma unroll
  for (int u = 0; u < DmaMap<D, NW>::PER; ++u) dma_one<D, NW>(map, gtile, lds, wave, u);
}
template <int D, int NW, typename T>
__device__ __forceinline__ void dma_tile(const DmaMap<D, NW>& map, const uint16_t* gtile, uint16_t* lds, int wave, T& token) {
#pragma unroll
  for (int u = 0; u < DmaMap<D, NW>::PER; ++u) {
    const int l = wave + NW * u;
    if (u < DmaMap<D, NW>::PER - 1 || l < DmaMap<D, NW>::NL)
      dma16(gtile, map.goff[u], lds_addr(lds) + 1024u * (uint32_t)l, token);
  }
}
// the same for a tile that ends before its 64th row: offsets recomputed with clamped rows
template <int D, int NW>
__device__ __forceinline__ void dma_tile_ragged(const DmaMap<D, NW>& map, const uint16_t* gtile, uint16_t* lds, int wave, int lane, int gstride, int rows_valid) {
  DmaMap<D, NW> m2;
  m2.init(wave, lane, gstride, map.perm, rows_valid);
  dma_tile<D, NW>(m2, gtile, lds, wave);
}

// Transposed operand through the LDS transpose load (ds_read_b64_tr_b16): from a row-major tile T[k][c] (pitch in
// elements) this lane gets column c0 + li of 8 rows, in the k order that the swapped K rows and the
// identity-transposed tiles use: slot e of lane half hh <-> tile row k0 + 8*(e>>2) + 4*hh + (e&3).
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

// ---------------------------------------------------------------------------------------------------
// Output through LDS.  An accumulator set keeps one tensor row per lane, so storing it directly writes 8-byte
// pieces of 32 different rows per instruction.  Instead the waves that hold results put them, as bf16, into a
// 64-row LDS tile (pitch D + 8), and after a barrier all 256 threads copy the tile out with 16-byte accesses that
// run along the rows.
// ---------------------------------------------------------------------------------------------------
template <int DT>
__device__ __forceinline__ void acc_to_lds_rows(uint16_t* tile, int pitch, int row, const float16_t (&acc)[DT], float mul, int hh) {
  uint16_t* r = tile + row * pitch + 4 * hh;
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      uint2 w;
      w.x = pack_bf16x2(acc[dt][4 * g + 0] * mul, acc[dt][4 * g + 1] * mul);
      w.y = pack_bf16x2(acc[dt][4 * g + 2] * mul, acc[dt][4 * g + 3] * mul);
      *reinterpret_cast<uint2*>(r + 32 * dt + 8 * g) = w;
    }
}
// rows 0 .. rows_valid-1 of the LDS tile -> global rows g0, g0 + gstride, ...
template <int D>
__device__ __forceinline__ void lds_rows_to_global(const uint16_t* tile, uint16_t* g0, int gstride, int rows_valid, int tid) {
  constexpr int CPR = D / 8, NCH = 64 * CPR, KP = D + 8;
#pragma unroll
  for (int it = 0; it < (NCH + 255) / 256; ++it) {
    const int c = tid + 256 * it, r = c / CPR, cc = c - r * CPR;
    if (c < NCH && r < rows_valid)
      *reinterpret_cast<u32x4_t*>(g0 + (int64_t)r * gstride + 8 * cc) = *reinterpret_cast<const u32x4_t*>(tile + r * KP + 8 * cc);
  }
}

// Exchange of accumulator sets between two waves through LDS, 16 bytes per lane and access: slot (4*dt + g) of
// lane `lane` holds acc[dt][4g .. 4g+3].  buf must hold 16 * DT * 64 floats.
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;
template <int DT>
__device__ __forceinline__ void acc_put(float* buf, const float16_t (&acc)[DT], int lane) {
  f32x4_t* b = reinterpret_cast<f32x4_t*>(buf) + lane;
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      f32x4_t v = {acc[dt][4 * g], acc[dt][4 * g + 1], acc[dt][4 * g + 2], acc[dt][4 * g + 3]};
      b[(4 * dt + g) * 64] = v;
    }
}
// acc = acc * w0 + other * w1
template <int DT>
__device__ __forceinline__ void acc_combine(const float* buf, float16_t (&acc)[DT], float w0, float w1, int lane) {
  const f32x4_t* b = reinterpret_cast<const f32x4_t*>(buf) + lane;
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const f32x4_t v = b[(4 * dt + g) * 64];
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[dt][4 * g + r] = acc[dt][4 * g + r] * w0 + v[r] * w1;
    }
}

}  // namespace sar
