// Device-side helpers shared by the HIP kernels of libsar (gfx950 only): bf16 conversion, Philox4x32-10,
// wavefront reductions.  Nothing here is used by, or shared with, the CPU oracle.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sar {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;   // MFMA A/B operand (8 bf16)
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short short4_t;     // ds_read_b64_tr_b16 result
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float float16_t;   // 32x32 MFMA accumulator
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float float4_t;

// ---- bf16 <-> fp32 (round to nearest even), on raw 16-bit patterns ----
__device__ __forceinline__ float bf16_to_f32(uint16_t v) { return __uint_as_float(((uint32_t)v) << 16); }
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);  // NaN stays NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
// two floats -> packed bf16 pair (lo = a, hi = b)
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
  typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;
  typedef __attribute__((__vector_size__(2 * sizeof(float)))) float float2_t;
  float2_t f = {a, b};
  bf16x2_t r = __builtin_convertvector(f, bf16x2_t);  // v_cvt_pk_bf16_f32, RNE
  return __builtin_bit_cast(uint32_t, r);
}

// element load/store abstraction for the generic (non-MFMA) kernels
template <typename T> struct Elem;
template <> struct Elem<float> {
  static __device__ __forceinline__ float load(const float* p) { return *p; }
  static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
  static __device__ __forceinline__ float round(float v) { return v; }  // the value as it would be stored
};
template <> struct Elem<uint16_t> {  // bf16 bit pattern
  static __device__ __forceinline__ float load(const uint16_t* p) { return bf16_to_f32(*p); }
  static __device__ __forceinline__ void store(uint16_t* p, float v) { *p = f32_to_bf16(v); }
  static __device__ __forceinline__ float round(float v) { return bf16_to_f32(f32_to_bf16(v)); }
};

// ---- Philox4x32-10 (Salmon et al., SC'11); the four output words for counter (g_lo, g_hi, 0, site) ----
struct Philox4 { uint32_t x, y, z, w; };
// a ^ b ^ c in one instruction (v_bitop3_b32, truth table 0x96)
__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c) { return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96); }
__device__ __forceinline__ Philox4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    uint32_t n0 = xor3((uint32_t)(p1 >> 32), c1, k0);
    uint32_t n2 = xor3((uint32_t)(p0 >> 32), c3, k1);
    c1 = (uint32_t)p1;
    c3 = (uint32_t)p0;
    c0 = n0;
    c2 = n2;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  Philox4 o = {c0, c1, c2, c3};
  return o;
}
// The same generator one round at a time, for kernels that spread a call's ten rounds between other instructions.
// Round r (0 .. 9) uses the key (k0 + r * 0x9E3779B9, k1 + r * 0xBB67AE85).
__device__ __forceinline__ Philox4 philox_start(uint64_t G, uint32_t site) {
  Philox4 s = {(uint32_t)G, (uint32_t)(G >> 32), 0u, site};
  return s;
}
__device__ __forceinline__ void philox_round(Philox4& s, uint32_t k0, uint32_t k1, int r) {
  const uint64_t p0 = (uint64_t)0xD2511F53u * s.x;
  const uint64_t p1 = (uint64_t)0xCD9E8D57u * s.z;
  const uint32_t n0 = xor3((uint32_t)(p1 >> 32), s.y, k0 + (uint32_t)r * 0x9E3779B9u);
  const uint32_t n2 = xor3((uint32_t)(p0 >> 32), s.w, k1 + (uint32_t)r * 0xBB67AE85u);
  s.y = (uint32_t)p1;
  s.w = (uint32_t)p0;
  s.x = n0;
  s.z = n2;
}
// the eight 16-bit fields of one call, for elements 8G .. 8G+7, as keep bits (bit r set = element r kept)
__device__ __forceinline__ uint32_t keep_bits8(uint64_t G, uint32_t site, uint32_t k0, uint32_t k1, uint32_t T) {
  Philox4 o = philox4x32_10((uint32_t)G, (uint32_t)(G >> 32), 0u, site, k0, k1);
  uint32_t m = 0;
  m |= ((o.x & 0xFFFFu) >= T) ? 1u : 0u;
  m |= ((o.x >> 16) >= T) ? 2u : 0u;
  m |= ((o.y & 0xFFFFu) >= T) ? 4u : 0u;
  m |= ((o.y >> 16) >= T) ? 8u : 0u;
  m |= ((o.z & 0xFFFFu) >= T) ? 16u : 0u;
  m |= ((o.z >> 16) >= T) ? 32u : 0u;
  m |= ((o.w & 0xFFFFu) >= T) ? 64u : 0u;
  m |= ((o.w >> 16) >= T) ? 128u : 0u;
  return m;
}
// the same decision for element r (0..7) of one call, straight from the raw output words
__device__ __forceinline__ Philox4 philox_call8(uint64_t G, uint32_t site, uint32_t k0, uint32_t k1) {
  return philox4x32_10((uint32_t)G, (uint32_t)(G >> 32), 0u, site, k0, k1);
}
__device__ __forceinline__ bool keep_field(const Philox4& o, int r, uint32_t T) {
  const uint32_t w = (r >> 1) == 0 ? o.x : (r >> 1) == 1 ? o.y : (r >> 1) == 2 ? o.z : o.w;
  return ((r & 1) ? (w >> 16) : (w & 0xFFFFu)) >= T;
}
// The same decisions for all eight elements of a call at once, as selects: out[r] = kept(r) ? val[r] : 0.  Written out as
// eight compares into eight scalar register pairs followed by eight selects: through the one condition register that the
// compiler uses for a compare-and-select, each pair waits for the one before it (measured 18 cycles per pair against 10).
// The compares sit at least seven instructions before the select that reads them.
__device__ __forceinline__ void keep_select8(const Philox4& o, uint32_t T, const float (&val)[8], float (&out)[8]) {
  uint64_t m0, m1, m2, m3, m4, m5, m6, m7;
  asm("v_cmp_ge_u32_sdwa %8, %16, %20 src0_sel:WORD_0 src1_sel:DWORD\n\t"
      "v_cmp_ge_u32_sdwa %9, %16, %20 src0_sel:WORD_1 src1_sel:DWORD\n\t"
      "v_cmp_ge_u32_sdwa %10, %17, %20 src0_sel:WORD_0 src1_sel:DWORD\n\t"
      "v_cmp_ge_u32_sdwa %11, %17, %20 src0_sel:WORD_1 src1_sel:DWORD\n\t"
      "v_cmp_ge_u32_sdwa %12, %18, %20 src0_sel:WORD_0 src1_sel:DWORD\n\t"
      "v_cmp_ge_u32_sdwa %13, %18, %20 src0_sel:WORD_1 src1_sel:DWORD\n\t"
      "v_cmp_ge_u32_sdwa %14, %19, %20 src0_sel:WORD_0 src1_sel:DWORD\n\t"
      "v_cmp_ge_u32_sdwa %15, %19, %20 src0_sel:WORD_1 src1_sel:DWORD\n\t"
      "v_cndmask_b32_e64 %0, 0, %21, %8\n\t"
      "v_cndmask_b32_e64 %1, 0, %22, %9\n\t"
      "v_cndmask_b32_e64 %2, 0, %23, %10\n\t"
      "v_cndmask_b32_e64 %3, 0, %24, %11\n\t"
      "v_cndmask_b32_e64 %4, 0, %25, %12\n\t"
      "v_cndmask_b32_e64 %5, 0, %26, %13\n\t"
      "v_cndmask_b32_e64 %6, 0, %27, %14\n\t"
      "v_cndmask_b32_e64 %7, 0, %28, %15"
      : "=&v"(out[0]), "=&v"(out[1]), "=&v"(out[2]), "=&v"(out[3]), "=&v"(out[4]), "=&v"(out[5]), "=&v"(out[6]), "=&v"(out[7]),
        "=&s"(m0), "=&s"(m1), "=&s"(m2), "=&s"(m3), "=&s"(m4), "=&s"(m5), "=&s"(m6), "=&s"(m7)
      : "v"(o.x), "v"(o.y), "v"(o.z), "v"(o.w), "s"(T),
        "v"(val[0]), "v"(val[1]), "v"(val[2]), "v"(val[3]), "v"(val[4]), "v"(val[5]), "v"(val[6]), "v"(val[7]));
}
// out[r] = kept(r) ? val : 0 with one value for all eight
__device__ __forceinline__ void keep_scale8(const Philox4& o, uint32_t T, float val, float (&out)[8]) {
  uint64_t m0, m1, m2, m3, m4, m5, m6, m7;
  asm("v_cmp_ge_u32_sdwa %8, %16, %20 src0_sel:WORD_0 src1_sel:DWORD\n\t"
      "v_cmp_ge_u32_sdwa %9, %16, %20 src0_sel:WORD_1 src1_sel:DWORD\n\t"
      "v_cmp_ge_u32_sdwa %10, %17, %20 src0_sel:WORD_0 src1_sel:DWORD\n\t"
      "v_cmp_ge_u32_sdwa %11, %17, %20 src0_sel:WORD_1 src1_sel:DWORD\n\t"
      "v_cmp_ge_u32_sdwa %12, %18, %20 src0_sel:WORD_0 src1_sel:DWORD\n\t"
      "v_cmp_ge_u32_sdwa %13, %18, %20 src0_sel:WORD_1 src1_sel:DWORD\n\t"
      "v_cmp_ge_u32_sdwa %14, %19, %20 src0_sel:WORD_0 src1_sel:DWORD\n\t"
      "v_cmp_ge_u32_sdwa %15, %19, %20 src0_sel:WORD_1 src1_sel:DWORD\n\t"
      "v_cndmask_b32_e64 %0, 0, %21, %8\n\t"
      "v_cndmask_b32_e64 %1, 0, %21, %9\n\t"
      "v_cndmask_b32_e64 %2, 0, %21, %10\n\t"
      "v_cndmask_b32_e64 %3, 0, %21, %11\n\t"
      "v_cndmask_b32_e64 %4, 0, %21, %12\n\t"
      "v_cndmask_b32_e64 %5, 0, %21, %13\n\t"
      "v_cndmask_b32_e64 %6, 0, %21, %14\n\t"
      "v_cndmask_b32_e64 %7, 0, %21, %15"
      : "=&v"(out[0]), "=&v"(out[1]), "=&v"(out[2]), "=&v"(out[3]), "=&v"(out[4]), "=&v"(out[5]), "=&v"(out[6]), "=&v"(out[7]),
        "=&s"(m0), "=&s"(m1), "=&s"(m2), "=&s"(m3), "=&s"(m4), "=&s"(m5), "=&s"(m6), "=&s"(m7)
      : "v"(o.x), "v"(o.y), "v"(o.z), "v"(o.w), "s"(T), "v"(val));
}
// keep bit of a single element e
__device__ __forceinline__ uint32_t keep_bit1(uint64_t e, uint64_t offset, uint32_t site, uint32_t k0, uint32_t k1, uint32_t T) {
  uint32_t m = keep_bits8(offset + (e >> 3), site, k0, k1, T);
  return (m >> (uint32_t)(e & 7u)) & 1u;
}

// ---- wavefront (64 lanes) reductions ----
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

}  // namespace sar
