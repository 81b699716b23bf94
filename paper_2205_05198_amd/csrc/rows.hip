// Memory-bound operators of the sequence-parallel region (Section 4.2.2, Eq. 3) on one rank's rows:
// LayerNorm forward / backward and dropout(+bias)+residual.  One pass over HBM per tensor, 128-bit accesses.
#include "sar_device.h"
#include "sar_internal.h"

namespace sar {

// 8 consecutive elements (one 16-byte access for bf16, two for fp32) <-> 8 floats
template <typename T> struct Vec8;
template <> struct Vec8<uint16_t> {
  static __device__ __forceinline__ void load(const uint16_t* p, float (&f)[8]) {
    uint4 u = *reinterpret_cast<const uint4*>(p);
    uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      f[2 * e] = __uint_as_float(w[e] << 16);
      f[2 * e + 1] = __uint_as_float(w[e] & 0xffff0000u);
    }
  }
  static __device__ __forceinline__ void store(uint16_t* p, const float (&f)[8]) {
    uint4 u;
    u.x = pack_bf16x2(f[0], f[1]);
    u.y = pack_bf16x2(f[2], f[3]);
    u.z = pack_bf16x2(f[4], f[5]);
    u.w = pack_bf16x2(f[6], f[7]);
    *reinterpret_cast<uint4*>(p) = u;
  }
};
template <> struct Vec8<float> {
  static __device__ __forceinline__ void load(const float* p, float (&f)[8]) {
    float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
    f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w; f[4] = b.x; f[5] = b.y; f[6] = b.z; f[7] = b.w;
  }
  static __device__ __forceinline__ void store(float* p, const float (&f)[8]) {
    *reinterpret_cast<float4*>(p) = make_float4(f[0], f[1], f[2], f[3]);
    *reinterpret_cast<float4*>(p + 4) = make_float4(f[4], f[5], f[6], f[7]);
  }
};

// block-wide sum of two values; every thread gets the totals.  red must hold 2 * 16 floats.
__device__ __forceinline__ void block_sum2(float& a, float& b, float* red) {
  a = wave_sum(a);
  b = wave_sum(b);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, nw = (blockDim.x + 63) >> 6;
  if (lane == 0) { red[wave] = a; red[16 + wave] = b; }
  __syncthreads();
  float ta = 0.f, tb = 0.f;
  for (int w = 0; w < nw; ++w) { ta += red[w]; tb += red[16 + w]; }
  a = ta;
  b = tb;
  __syncthreads();
}

// ---------------------------------------------------------------------------------------------------
// LayerNorm forward: one workgroup per row, the row lives in registers (VPT chunks of 8 per thread).
// Statistics in fp32 with the row's first element as shift, so one reduction gives mean and variance.
// ---------------------------------------------------------------------------------------------------
template <typename T, int VPT>
__global__ __launch_bounds__(1024) void ln_fwd_kernel(RowsParams P, const T* __restrict__ x, const T* __restrict__ gamma, const T* __restrict__ beta,
                                                     T* __restrict__ y, float* __restrict__ mean, float* __restrict__ rstd) {
  __shared__ float red[32];
  const int64_t r = blockIdx.x;
  const int nchunk = (int)(P.h >> 3);
  const T* xr = x + r * P.h;
  float xv[VPT][8];
  const float shift = Elem<T>::load(xr);
  float s1 = 0.f, s2 = 0.f;
#pragma unroll
  for (int u = 0; u < VPT; ++u) {
    const int c = threadIdx.x + u * blockDim.x;
    if (c < nchunk) {
      Vec8<T>::load(xr + 8 * c, xv[u]);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        float dlt = xv[u][e] - shift;
        s1 += dlt;
        s2 = fmaf(dlt, dlt, s2);
      }
    }
  }
  block_sum2(s1, s2, red);
  const float invh = 1.f / (float)P.h;
  const float m1 = s1 * invh;
  const float var = fmaxf(s2 * invh - m1 * m1, 0.f);
  const float mu = shift + m1;
  const float rs = rsqrtf(var + P.eps);
#pragma unroll
  for (int u = 0; u < VPT; ++u) {
    const int c = threadIdx.x + u * blockDim.x;
    if (c < nchunk) {
      float g[8], bt[8], out[8];
      Vec8<T>::load(gamma + 8 * c, g);
      Vec8<T>::load(beta + 8 * c, bt);
#pragma unroll
      for (int e = 0; e < 8; ++e) out[e] = fmaf((xv[u][e] - mu) * rs, g[e], bt[e]);
      Vec8<T>::store(y + r * P.h + 8 * c, out);
    }
  }
  if (threadIdx.x == 0) { mean[r] = mu; rstd[r] = rs; }
}

// ---------------------------------------------------------------------------------------------------
// LayerNorm backward, one launch with two kinds of workgroups (dgamma / dbeta do not depend on the row sums, so
// nothing orders the two kinds):
//   blockIdx <  rows: one row, kept in registers: c1 = mean_c(g), c2 = mean_c(g xhat) with g = dy*gamma, then
//                     dx = rstd (g - c1 - xhat c2);
//   blockIdx >= rows: a slab of kLnSlab columns and a contiguous range of rows (kLnSlab/8 lanes cover one row segment,
//                     8 blockDim/kLnSlab segments per trip): dgamma = sum_r dy xhat, dbeta = sum_r dy of the slab, summed in
//                     registers, across the lanes of a wave, then across waves in LDS.  The second read of x and dy
//                     comes out of the caches: the row workgroups stream the same bytes at the same time.
// part[split][0][h] = dgamma partial, part[split][1][h] = dbeta partial (or the final arrays if there is 1 split).
// ---------------------------------------------------------------------------------------------------
constexpr int kLnSlab = 64;  // columns of a slab workgroup: 8 lanes x 16 bytes (bf16) per row segment; 128 measured slower

template <typename T, int VPT>
__global__ __launch_bounds__(1024) void ln_bwd_kernel(RowsParams P, const T* __restrict__ dy, const T* __restrict__ x,
                                                     const float* __restrict__ mean, const float* __restrict__ rstd,
                                                     const T* __restrict__ gamma, T* __restrict__ dx, float* __restrict__ dg_out,
                                                     float* __restrict__ db_out, int nslab, int rows_per_split) {
  __shared__ float red[32];
  __shared__ float sacc[2][16][kLnSlab];
  if ((int64_t)blockIdx.x < P.rows) {
    const int64_t r = blockIdx.x;
    const int nchunk = (int)(P.h >> 3);
    const float mu = mean[r], rs = rstd[r];
    float xh[VPT][8], gg[VPT][8];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int u = 0; u < VPT; ++u) {
      const int c = threadIdx.x + u * blockDim.x;
      if (c < nchunk) {
        float xv[8], dv[8], g[8];
        Vec8<T>::load(x + r * P.h + 8 * c, xv);
        Vec8<T>::load(dy + r * P.h + 8 * c, dv);
        Vec8<T>::load(gamma + 8 * c, g);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          xh[u][e] = (xv[e] - mu) * rs;
          gg[u][e] = dv[e] * g[e];
          s1 += gg[u][e];
          s2 = fmaf(gg[u][e], xh[u][e], s2);
        }
      }
    }
    block_sum2(s1, s2, red);
    const float c1 = s1 / (float)P.h, c2 = s2 / (float)P.h;
#pragma unroll
    for (int u = 0; u < VPT; ++u) {
      const int c = threadIdx.x + u * blockDim.x;
      if (c < nchunk) {
        float out[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) out[e] = rs * (gg[u][e] - c1 - xh[u][e] * c2);
        Vec8<T>::store(dx + r * P.h + 8 * c, out);
      }
    }
    return;
  }
  const int idx = (int)((int64_t)blockIdx.x - P.rows);
  const int slab = idx % nslab, split = idx / nslab;
  constexpr int LPS = kLnSlab / 8;  // lanes per row segment
  const int nseg = (int)(blockDim.x / LPS), seg = threadIdx.x / LPS, ls = threadIdx.x % LPS;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, nw = (int)(blockDim.x >> 6);
  const int64_t col = (int64_t)slab * kLnSlab + 8 * ls;
  const bool colok = col < P.h;
  const int64_t r_lo = (int64_t)split * rows_per_split;
  const int64_t r_hi = min(P.rows, r_lo + rows_per_split);
  float ag[8], ab[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) { ag[e] = 0.f; ab[e] = 0.f; }
  if (colok) {
    for (int64_t r = r_lo + seg; r < r_hi; r += nseg) {
      float xv[8], dv[8];
      Vec8<T>::load(x + r * P.h + col, xv);
      Vec8<T>::load(dy + r * P.h + col, dv);
      const float mu = mean[r], rs = rstd[r];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        ag[e] = fmaf(dv[e], (xv[e] - mu) * rs, ag[e]);
        ab[e] += dv[e];
      }
    }
  }
  // lanes ls, ls + LPS, ... of a wave hold the same columns
#pragma unroll
  for (int e = 0; e < 8; ++e) {
#pragma unroll
    for (int m = LPS; m < 64; m <<= 1) {
      ag[e] += __shfl_xor(ag[e], m);
      ab[e] += __shfl_xor(ab[e], m);
    }
  }
  if (lane < LPS) {
#pragma unroll
    for (int e = 0; e < 8; ++e) { sacc[0][wave][8 * ls + e] = ag[e]; sacc[1][wave][8 * ls + e] = ab[e]; }
  }
  __syncthreads();
  // thread t sums array t / kLnSlab, column t % kLnSlab over the waves
  for (int t = threadIdx.x; t < 2 * kLnSlab; t += blockDim.x) {
    const int c = t % kLnSlab, which = t / kLnSlab;
    float tot = 0.f;
    for (int q = 0; q < nw; ++q) tot += sacc[which][q][c];
    const int64_t cc = (int64_t)slab * kLnSlab + c;
    if (cc < P.h) (which ? db_out : dg_out)[(size_t)split * 2 * P.h + cc] = tot;
  }
}

// sums the row-split partials: part[nsplit][2][h] -> dgamma[h], dbeta[h]
__global__ void ln_bwd_finish_kernel(const float* __restrict__ part, int nsplit, int64_t h, float* __restrict__ dgamma, float* __restrict__ dbeta) {
  const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= h) return;
  float tg = 0.f, tb = 0.f;
  for (int q = 0; q < nsplit; ++q) {
    tg += part[(size_t)q * 2 * h + c];
    tb += part[(size_t)q * 2 * h + h + c];
  }
  dgamma[c] = tg;
  dbeta[c] = tb;
}

// ---------------------------------------------------------------------------------------------------
// bias-dropout-add: out = resid + M (x + bias) / (1-p); one thread per 8 elements = one Philox call.
// ---------------------------------------------------------------------------------------------------
template <typename T, bool HAS_BIAS, bool HAS_MASK>
__global__ __launch_bounds__(256) void bias_dropout_add_kernel(RowsParams P, const T* __restrict__ x, const T* __restrict__ bias, const T* resid,
                                                              T* out, uint8_t* __restrict__ mask) {
  const int64_t r = blockIdx.x, c = ((int64_t)blockIdx.y * 256 + threadIdx.x) << 3;  // grid = (rows, chunks of a row / 256): no index division
  if (c >= P.h) return;
  float xv[8], rv[8], bv[8], o[8];
  Vec8<T>::load(x + r * P.h + c, xv);
  Vec8<T>::load(resid + r * P.h + c, rv);
  if (HAS_BIAS) Vec8<T>::load(bias + c, bv);
  const uint64_t e = (uint64_t)(P.row_offset + r) * (uint64_t)P.h + (uint64_t)c;
  const uint32_t keep = keep_bits8(P.offset + (e >> 3), 1u, P.key0, P.key1, P.thresh);
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    float xb = HAS_BIAS ? xv[q] + bv[q] : xv[q];
    o[q] = ((keep >> q) & 1u) ? fmaf(xb, P.keep_scale, rv[q]) : rv[q];
  }
  Vec8<T>::store(out + r * P.h + c, o);
  if (HAS_MASK) {
    uint2 m;
    m.x = (keep & 1u) | ((keep & 2u) << 7) | ((keep & 4u) << 14) | ((keep & 8u) << 21);
    m.y = ((keep >> 4) & 1u) | ((keep & 32u) << 3) | ((keep & 64u) << 10) | ((keep & 128u) << 17);
    *reinterpret_cast<uint2*>(mask + r * P.h + c) = m;
  }
}

// ---------------------------------------------------------------------------------------------------
// Fused bias-dropout-add + LayerNorm forward (last line of Eq. 3 feeding the next layer's first line):
//   out = resid + M (x + bias)/(1-p),  y = LayerNorm(out).
// One workgroup per row, as ln_fwd: the row is read once instead of twice (8 instead of 10 bytes per element).
// The statistics are taken from `out` as it is stored (rounded to T), so that a later ln_bwd, which re-reads the
// stored row, sees exactly the values mean and rstd belong to.
// ---------------------------------------------------------------------------------------------------
template <typename T, int VPT, bool HAS_BIAS>
__global__ __launch_bounds__(1024) void bda_ln_fwd_kernel(RowsParams P, const T* __restrict__ x, const T* __restrict__ bias, const T* resid,
                                                         const T* __restrict__ gamma, const T* __restrict__ beta, T* out, T* __restrict__ y,
                                                         float* __restrict__ mean, float* __restrict__ rstd) {
  __shared__ float red[32];
  const int64_t r = blockIdx.x;
  const int nchunk = (int)(P.h >> 3);
  float ov[VPT][8];
  float s1 = 0.f, s2 = 0.f, shift = 0.f;
#pragma unroll
  for (int u = 0; u < VPT; ++u) {
    const int c = threadIdx.x + u * blockDim.x;
    if (c < nchunk) {
      float xv[8], rv[8], bv[8];
      Vec8<T>::load(x + r * P.h + 8 * c, xv);
      Vec8<T>::load(resid + r * P.h + 8 * c, rv);
      if (HAS_BIAS) Vec8<T>::load(bias + 8 * c, bv);
      const uint64_t e = (uint64_t)(P.row_offset + r) * (uint64_t)P.h + (uint64_t)(8 * c);
      const uint32_t keep = keep_bits8(P.offset + (e >> 3), 1u, P.key0, P.key1, P.thresh);
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const float xb = HAS_BIAS ? xv[q] + bv[q] : xv[q];
        ov[u][q] = Elem<T>::round(((keep >> q) & 1u) ? fmaf(xb, P.keep_scale, rv[q]) : rv[q]);
      }
      Vec8<T>::store(out + r * P.h + 8 * c, ov[u]);
    }
  }
  // shift = the row's first element, held by thread 0: broadcast through LDS
  if (threadIdx.x == 0) red[0] = ov[0][0];
  __syncthreads();
  shift = red[0];
  __syncthreads();
#pragma unroll
  for (int u = 0; u < VPT; ++u) {
    const int c = threadIdx.x + u * blockDim.x;
    if (c < nchunk) {
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const float dlt = ov[u][q] - shift;
        s1 += dlt;
        s2 = fmaf(dlt, dlt, s2);
      }
    }
  }
  block_sum2(s1, s2, red);
  const float invh = 1.f / (float)P.h;
  const float m1 = s1 * invh;
  const float var = fmaxf(s2 * invh - m1 * m1, 0.f);
  const float mu = shift + m1;
  const float rs = rsqrtf(var + P.eps);
#pragma unroll
  for (int u = 0; u < VPT; ++u) {
    const int c = threadIdx.x + u * blockDim.x;
    if (c < nchunk) {
      float g[8], bt[8], o[8];
      Vec8<T>::load(gamma + 8 * c, g);
      Vec8<T>::load(beta + 8 * c, bt);
#pragma unroll
      for (int q = 0; q < 8; ++q) o[q] = fmaf((ov[u][q] - mu) * rs, g[q], bt[q]);
      Vec8<T>::store(y + r * P.h + 8 * c, o);
    }
  }
  if (threadIdx.x == 0) { mean[r] = mu; rstd[r] = rs; }
}

// ---------------------------------------------------------------------------------------------------
// bias-dropout-add backward: dx = M dout/(1-p) with M regenerated from Philox; the residual branch's gradient is
// dout itself and is not written.  Without dbias this is elementwise (one thread per 8 elements).  With dbias
// (the column sums of dx) a workgroup owns a slab of 64 columns and a range of rows, as ln_bwd's second pass:
// part[split][h] partial sums, or dbias itself if there is one split.
// ---------------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void bda_bwd_kernel(RowsParams P, const T* __restrict__ dout, T* __restrict__ dx) {
  const int64_t r = blockIdx.x, c = ((int64_t)blockIdx.y * 256 + threadIdx.x) << 3;  // grid = (rows, chunks of a row / 256): no index division
  if (c >= P.h) return;
  float dv[8], o[8];
  Vec8<T>::load(dout + r * P.h + c, dv);
  const uint64_t e = (uint64_t)(P.row_offset + r) * (uint64_t)P.h + (uint64_t)c;
  const uint32_t keep = keep_bits8(P.offset + (e >> 3), 1u, P.key0, P.key1, P.thresh);
#pragma unroll
  for (int q = 0; q < 8; ++q) o[q] = ((keep >> q) & 1u) ? dv[q] * P.keep_scale : 0.f;
  Vec8<T>::store(dx + r * P.h + c, o);
}

template <typename T>
__global__ __launch_bounds__(256) void bda_bwd_slab_kernel(RowsParams P, const T* __restrict__ dout, T* __restrict__ dx, float* __restrict__ db_out,
                                                          int rows_per_split) {
  __shared__ float sb[32][65];
  const int slab = blockIdx.x, split = blockIdx.y;
  const int seg = threadIdx.x >> 3, l8 = threadIdx.x & 7;
  const int64_t col = (int64_t)slab * 64 + 8 * l8;
  const bool colok = col < P.h;
  const int64_t r_lo = (int64_t)split * rows_per_split;
  const int64_t r_hi = min(P.rows, r_lo + rows_per_split);
  float ab[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) ab[e] = 0.f;
  for (int64_t r = r_lo + seg; r < r_hi; r += 32) {
    if (colok) {
      float dv[8], o[8];
      Vec8<T>::load(dout + r * P.h + col, dv);
      const uint64_t e = (uint64_t)(P.row_offset + r) * (uint64_t)P.h + (uint64_t)col;
      const uint32_t keep = keep_bits8(P.offset + (e >> 3), 1u, P.key0, P.key1, P.thresh);
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        o[q] = ((keep >> q) & 1u) ? dv[q] * P.keep_scale : 0.f;
        ab[q] += o[q];
      }
      Vec8<T>::store(dx + r * P.h + col, o);
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) sb[seg][8 * l8 + e] = ab[e];
  __syncthreads();
  if (threadIdx.x < 64) {
    const int c = threadIdx.x;
    float t = 0.f;
    for (int q = 0; q < 32; ++q) t += sb[q][c];
    const int64_t cc = (int64_t)slab * 64 + c;
    if (cc < P.h) db_out[(size_t)split * P.h + cc] = t;
  }
}

// sums row-split partials: part[nsplit][h] -> dbias[h]
__global__ void bda_bwd_finish_kernel(const float* __restrict__ part, int nsplit, int64_t h, float* __restrict__ dbias) {
  const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= h) return;
  float t = 0.f;
  for (int q = 0; q < nsplit; ++q) t += part[(size_t)q * h + c];
  dbias[c] = t;
}

// ---------------------------------------------------------------------------------------------------
// bias + GeLU of the MLP block (Section 4.1): y = z Phi(z), z = x + bias, Phi the standard normal CDF (exact form,
// through erf).  Backward: dx = dy (Phi(z) + z phi(z)) from the stored input, dbias = column sums of dx.
// One thread per 8 elements; with dbias, column slabs of 64 as in bias_dropout_add_bwd.
// ---------------------------------------------------------------------------------------------------
// Phi(z) and phi(z) from one exponential: erf by the rational approximation 7.1.26 of Abramowitz & Stegun,
// erf(x) = 1 - (a1 t + ... + a5 t^5) exp(-x^2), t = 1 / (1 + p x), x >= 0, |error| <= 1.5e-7, with x = |z| / sqrt 2,
// so that exp(-x^2) = exp(-z^2 / 2) also gives the density.  (The library erff costs about three times as many
// vector instructions and made both kernels ALU-bound.)
__device__ __forceinline__ void gelu_parts(float z, float& Phi, float& pdf) {
  const float x = fabsf(z) * 0.70710678118654752f;
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, x, 1.f));  // 1 ulp; a correctly rounded reciprocal costs ten more instructions
  const float e = __expf(-x * x);
  const float poly = t * fmaf(t, fmaf(t, fmaf(t, fmaf(t, 1.061405429f, -1.453152027f), 1.421413741f), -0.284496736f), 0.254829592f);
  const float erfa = fmaf(-poly, e, 1.f);
  Phi = 0.5f * (1.f + copysignf(erfa, z));
  pdf = 0.3989422804014327f * e;
}
__device__ __forceinline__ float gelu_phi_cdf(float z) {
  float Phi, pdf;
  gelu_parts(z, Phi, pdf);
  return Phi;
}
__device__ __forceinline__ float gelu_grad(float z) {
  float Phi, pdf;
  gelu_parts(z, Phi, pdf);
  return fmaf(z, pdf, Phi);
}

// One chunk of 8 elements per thread; grid = (rows, chunks of a row / 256): no index division in the kernel (it cost
// four instructions per element of a kernel that is bound by its vector arithmetic).  More chunks per thread were slower.
template <typename T, bool HAS_BIAS>
__global__ __launch_bounds__(256) void bias_gelu_fwd_kernel(RowsParams P, const T* __restrict__ x, const T* __restrict__ bias, T* __restrict__ y) {
  const int64_t c = ((int64_t)blockIdx.y * 256 + threadIdx.x) << 3;
  if (c >= P.h) return;
  const int64_t at = (int64_t)blockIdx.x * P.h + c;
  float xv[8], bv[8], o[8];
  Vec8<T>::load(x + at, xv);
  if (HAS_BIAS) Vec8<T>::load(bias + c, bv);
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    const float z = HAS_BIAS ? xv[q] + bv[q] : xv[q];
    o[q] = z * gelu_phi_cdf(z);
  }
  Vec8<T>::store(y + at, o);
}

template <typename T, bool HAS_BIAS>
__global__ __launch_bounds__(256) void bias_gelu_bwd_kernel(RowsParams P, const T* __restrict__ dy, const T* __restrict__ x,
                                                           const T* __restrict__ bias, T* __restrict__ dx) {
  const int64_t c = ((int64_t)blockIdx.y * 256 + threadIdx.x) << 3;
  if (c >= P.h) return;
  const int64_t at = (int64_t)blockIdx.x * P.h + c;
  float xv[8], dv[8], bv[8], o[8];
  Vec8<T>::load(x + at, xv);
  Vec8<T>::load(dy + at, dv);
  if (HAS_BIAS) Vec8<T>::load(bias + c, bv);
#pragma unroll
  for (int q = 0; q < 8; ++q) o[q] = dv[q] * gelu_grad(HAS_BIAS ? xv[q] + bv[q] : xv[q]);
  Vec8<T>::store(dx + at, o);
}

// with dbias: a workgroup owns 64 columns and a range of rows, as bda_bwd_slab_kernel
template <typename T, bool HAS_BIAS>
__global__ __launch_bounds__(256) void bias_gelu_bwd_slab_kernel(RowsParams P, const T* __restrict__ dy, const T* __restrict__ x,
                                                                const T* __restrict__ bias, T* __restrict__ dx, float* __restrict__ db_out,
                                                                int rows_per_split) {
  __shared__ float sb[32][65];
  const int slab = blockIdx.x, split = blockIdx.y;
  const int seg = threadIdx.x >> 3, l8 = threadIdx.x & 7;
  const int64_t col = (int64_t)slab * 64 + 8 * l8;
  const bool colok = col < P.h;
  const int64_t r_lo = (int64_t)split * rows_per_split;
  const int64_t r_hi = min(P.rows, r_lo + rows_per_split);
  float ab[8], bv[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) { ab[e] = 0.f; bv[e] = 0.f; }
  if (HAS_BIAS && colok) Vec8<T>::load(bias + col, bv);
  for (int64_t r = r_lo + seg; r < r_hi; r += 32) {
    if (colok) {
      float xv[8], dv[8], o[8];
      Vec8<T>::load(x + r * P.h + col, xv);
      Vec8<T>::load(dy + r * P.h + col, dv);
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        o[q] = dv[q] * gelu_grad(xv[q] + bv[q]);
        ab[q] += o[q];
      }
      Vec8<T>::store(dx + r * P.h + col, o);
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) sb[seg][8 * l8 + e] = ab[e];
  __syncthreads();
  if (threadIdx.x < 64) {
    const int c = threadIdx.x;
    float t = 0.f;
    for (int q = 0; q < 32; ++q) t += sb[q][c];
    const int64_t cc = (int64_t)slab * 64 + c;
    if (cc < P.h) db_out[(size_t)split * P.h + cc] = t;
  }
}

// ------------------------------------------------------------------------------------------------ launchers
static inline int pick_vpt(int64_t h, int& threads) {
  const int nchunk = (int)(h >> 3);
  int vpt = (nchunk + 1023) / 1024;
  if (vpt < 1) vpt = 1;
  threads = (nchunk + vpt - 1) / vpt;
  threads = (threads + 63) / 64 * 64;
  return vpt;
}

template <typename T>
static hipError_t ln_fwd_t(const RowsParams& P, const void* x, const void* gamma, const void* beta, void* y, float* mean, float* rstd, hipStream_t st) {
  int threads;
  const int vpt = pick_vpt(P.h, threads);
  dim3 grid((unsigned)P.rows), block(threads);
#define SAR_LN_FWD(V) hipLaunchKernelGGL((ln_fwd_kernel<T, V>), grid, block, 0, st, P, (const T*)x, (const T*)gamma, (const T*)beta, (T*)y, mean, rstd)
  switch (vpt) {
    case 1: SAR_LN_FWD(1); break;
    case 2: SAR_LN_FWD(2); break;
    case 3: SAR_LN_FWD(3); break;
    default: SAR_LN_FWD(4); break;
  }
#undef SAR_LN_FWD
  return hipGetLastError();
}

hipError_t launch_ln_fwd(const RowsParams& P, bool bf16, const void* x, const void* gamma, const void* beta, void* y, float* mean, float* rstd,
                         hipStream_t st) {
  return bf16 ? ln_fwd_t<uint16_t>(P, x, gamma, beta, y, mean, rstd, st) : ln_fwd_t<float>(P, x, gamma, beta, y, mean, rstd, st);
}

// target: slab workgroups to aim at (256 = one per CU); min_trips: trips of a slab workgroup over its rows at least
static inline void ln_bwd_plan(int64_t rows, int64_t h, int threads, int slabw, int& nslab, int& nsplit, int& rows_per_split, int target = 256,
                               int min_trips = 1) {
  nslab = (int)((h + slabw - 1) / slabw);
  const int nseg = threads / (slabw / 8);                // row segments per trip of a slab workgroup
  int want = (target + nslab - 1) / nslab;
  int maxsplit = (int)((rows + (int64_t)nseg * min_trips - 1) / ((int64_t)nseg * min_trips));
  nsplit = want < 1 ? 1 : (want > maxsplit ? maxsplit : want);
  if (nsplit < 1) nsplit = 1;
  rows_per_split = (int)((rows + nsplit - 1) / nsplit);
  nsplit = (int)((rows + rows_per_split - 1) / rows_per_split);
}

size_t ln_bwd_workspace_bytes(int64_t rows, int64_t h) {
  int nslab, nsplit, rps, threads;
  pick_vpt(h, threads);
  ln_bwd_plan(rows, h, threads, kLnSlab, nslab, nsplit, rps);
  return nsplit > 1 ? (size_t)nsplit * 2 * (size_t)h * sizeof(float) : 256;
}

template <typename T>
static hipError_t ln_bwd_t(const RowsParams& P, const void* dy, const void* x, const float* mean, const float* rstd, const void* gamma, void* dx,
                           float* dgamma, float* dbeta, void* ws, hipStream_t st) {
  int nslab, nsplit, rps, threads;
  const int vpt = pick_vpt(P.h, threads);
  ln_bwd_plan(P.rows, P.h, threads, kLnSlab, nslab, nsplit, rps);
  float* part = (float*)ws;
  // one split: the slab workgroups see every row and write dgamma / dbeta themselves; else partials [split][2][h]
  float* dg_out = nsplit == 1 ? dgamma : part;
  float* db_out = nsplit == 1 ? dbeta : part + P.h;
  dim3 grid((unsigned)(P.rows + (int64_t)nslab * nsplit)), block(threads);
#define SAR_LN_BWD(V) hipLaunchKernelGGL((ln_bwd_kernel<T, V>), grid, block, 0, st, P, (const T*)dy, (const T*)x, mean, rstd, (const T*)gamma, (T*)dx, dg_out, db_out, nslab, rps)
  switch (vpt) {
    case 1: SAR_LN_BWD(1); break;
    case 2: SAR_LN_BWD(2); break;
    case 3: SAR_LN_BWD(3); break;
    default: SAR_LN_BWD(4); break;
  }
#undef SAR_LN_BWD
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || nsplit == 1) return e;
  hipLaunchKernelGGL(ln_bwd_finish_kernel, dim3((unsigned)((P.h + 255) / 256)), dim3(256), 0, st, (const float*)part, nsplit, P.h, dgamma, dbeta);
  return hipGetLastError();
}

hipError_t launch_ln_bwd(const RowsParams& P, bool bf16, const void* dy, const void* x, const float* mean, const float* rstd, const void* gamma,
                         void* dx, float* dgamma, float* dbeta, void* ws, hipStream_t st) {
  return bf16 ? ln_bwd_t<uint16_t>(P, dy, x, mean, rstd, gamma, dx, dgamma, dbeta, ws, st)
              : ln_bwd_t<float>(P, dy, x, mean, rstd, gamma, dx, dgamma, dbeta, ws, st);
}

template <typename T>
static hipError_t bda_t(const RowsParams& P, const void* x, const void* bias, const void* resid, void* out, uint8_t* mask, hipStream_t st) {
  dim3 grid((unsigned)P.rows, (unsigned)(((P.h >> 3) + 255) / 256)), block(256);
#define SAR_BDA(B, M) hipLaunchKernelGGL((bias_dropout_add_kernel<T, B, M>), grid, block, 0, st, P, (const T*)x, (const T*)bias, (const T*)resid, (T*)out, mask)
  if (bias && mask) SAR_BDA(true, true);
  else if (bias) SAR_BDA(true, false);
  else if (mask) SAR_BDA(false, true);
  else SAR_BDA(false, false);
#undef SAR_BDA
  return hipGetLastError();
}

hipError_t launch_bias_dropout_add(const RowsParams& P, bool bf16, const void* x, const void* bias, const void* resid, void* out, uint8_t* mask,
                                   hipStream_t st) {
  return bf16 ? bda_t<uint16_t>(P, x, bias, resid, out, mask, st) : bda_t<float>(P, x, bias, resid, out, mask, st);
}

template <typename T>
static hipError_t bda_ln_t(const RowsParams& P, const void* x, const void* bias, const void* resid, const void* gamma, const void* beta, void* out,
                           void* y, float* mean, float* rstd, hipStream_t st) {
  int threads;
  const int vpt = pick_vpt(P.h, threads);
  dim3 grid((unsigned)P.rows), block(threads);
#define SAR_BDA_LN(V, B) hipLaunchKernelGGL((bda_ln_fwd_kernel<T, V, B>), grid, block, 0, st, P, (const T*)x, (const T*)bias, (const T*)resid, \
                                            (const T*)gamma, (const T*)beta, (T*)out, (T*)y, mean, rstd)
#define SAR_BDA_LN_V(V) do { if (bias) SAR_BDA_LN(V, true); else SAR_BDA_LN(V, false); } while (0)
  switch (vpt) {
    case 1: SAR_BDA_LN_V(1); break;
    case 2: SAR_BDA_LN_V(2); break;
    case 3: SAR_BDA_LN_V(3); break;
    default: SAR_BDA_LN_V(4); break;
  }
#undef SAR_BDA_LN_V
#undef SAR_BDA_LN
  return hipGetLastError();
}

hipError_t launch_bias_dropout_add_ln_fwd(const RowsParams& P, bool bf16, const void* x, const void* bias, const void* resid, const void* gamma,
                                          const void* beta, void* out, void* y, float* mean, float* rstd, hipStream_t st) {
  return bf16 ? bda_ln_t<uint16_t>(P, x, bias, resid, gamma, beta, out, y, mean, rstd, st)
              : bda_ln_t<float>(P, x, bias, resid, gamma, beta, out, y, mean, rstd, st);
}

// The bias-GeLU backward has many rows (s b of them, not s b / t): a slab workgroup does one dependent load -> arithmetic
// -> store chain per trip, so the bytes in flight are what the resident waves hold; eight workgroups per CU instead of
// one or two (2048 x 10240: 320 -> 2080 workgroups) take it from 45 to 32 us.  (Finer splits, or two rows per trip, are slower.)
static constexpr int kGeluTarget = 2048, kGeluMinTrips = 2;
size_t bias_gelu_bwd_workspace_bytes(int64_t rows, int64_t h) {
  int nslab, nsplit, rps;
  ln_bwd_plan(rows, h, 256, 64, nslab, nsplit, rps, kGeluTarget, kGeluMinTrips);
  return nsplit > 1 ? (size_t)nsplit * (size_t)h * sizeof(float) : 0;
}

size_t bda_bwd_workspace_bytes(int64_t rows, int64_t h) {
  int nslab, nsplit, rps;
  ln_bwd_plan(rows, h, 256, 64, nslab, nsplit, rps);
  return nsplit > 1 ? (size_t)nsplit * (size_t)h * sizeof(float) : 0;
}

template <typename T>
static hipError_t bda_bwd_t(const RowsParams& P, const void* dout, void* dx, float* dbias, void* ws, hipStream_t st) {
  if (!dbias) {
    hipLaunchKernelGGL((bda_bwd_kernel<T>), dim3((unsigned)P.rows, (unsigned)(((P.h >> 3) + 255) / 256)), dim3(256), 0, st, P, (const T*)dout, (T*)dx);
    return hipGetLastError();
  }
  int nslab, nsplit, rps;
  ln_bwd_plan(P.rows, P.h, 256, 64, nslab, nsplit, rps);
  if (nsplit == 1) {
    hipLaunchKernelGGL((bda_bwd_slab_kernel<T>), dim3(nslab, 1), dim3(256), 0, st, P, (const T*)dout, (T*)dx, dbias, rps);
    return hipGetLastError();
  }
  float* part = (float*)ws;
  hipLaunchKernelGGL((bda_bwd_slab_kernel<T>), dim3(nslab, nsplit), dim3(256), 0, st, P, (const T*)dout, (T*)dx, part, rps);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(bda_bwd_finish_kernel, dim3((unsigned)((P.h + 255) / 256)), dim3(256), 0, st, (const float*)part, nsplit, P.h, dbias);
  return hipGetLastError();
}

hipError_t launch_bias_dropout_add_bwd(const RowsParams& P, bool bf16, const void* dout, void* dx, float* dbias, void* ws, hipStream_t st) {
  return bf16 ? bda_bwd_t<uint16_t>(P, dout, dx, dbias, ws, st) : bda_bwd_t<float>(P, dout, dx, dbias, ws, st);
}

template <typename T>
static hipError_t bias_gelu_fwd_t(const RowsParams& P, const void* x, const void* bias, void* y, hipStream_t st) {
  dim3 grid((unsigned)P.rows, (unsigned)(((P.h >> 3) + 255) / 256)), block(256);
  if (bias) hipLaunchKernelGGL((bias_gelu_fwd_kernel<T, true>), grid, block, 0, st, P, (const T*)x, (const T*)bias, (T*)y);
  else hipLaunchKernelGGL((bias_gelu_fwd_kernel<T, false>), grid, block, 0, st, P, (const T*)x, (const T*)bias, (T*)y);
  return hipGetLastError();
}

hipError_t launch_bias_gelu_fwd(const RowsParams& P, bool bf16, const void* x, const void* bias, void* y, hipStream_t st) {
  return bf16 ? bias_gelu_fwd_t<uint16_t>(P, x, bias, y, st) : bias_gelu_fwd_t<float>(P, x, bias, y, st);
}

template <typename T>
static hipError_t bias_gelu_bwd_t(const RowsParams& P, const void* dy, const void* x, const void* bias, void* dx, float* dbias, void* ws,
                                  hipStream_t st) {
  if (!dbias) {
    dim3 grid((unsigned)P.rows, (unsigned)(((P.h >> 3) + 255) / 256)), block(256);
    if (bias) hipLaunchKernelGGL((bias_gelu_bwd_kernel<T, true>), grid, block, 0, st, P, (const T*)dy, (const T*)x, (const T*)bias, (T*)dx);
    else hipLaunchKernelGGL((bias_gelu_bwd_kernel<T, false>), grid, block, 0, st, P, (const T*)dy, (const T*)x, (const T*)bias, (T*)dx);
    return hipGetLastError();
  }
  int nslab, nsplit, rps;
  ln_bwd_plan(P.rows, P.h, 256, 64, nslab, nsplit, rps, kGeluTarget, kGeluMinTrips);
  float* out = nsplit == 1 ? dbias : (float*)ws;
  if (bias)
    hipLaunchKernelGGL((bias_gelu_bwd_slab_kernel<T, true>), dim3(nslab, nsplit), dim3(256), 0, st, P, (const T*)dy, (const T*)x, (const T*)bias, (T*)dx,
                       out, rps);
  else
    hipLaunchKernelGGL((bias_gelu_bwd_slab_kernel<T, false>), dim3(nslab, nsplit), dim3(256), 0, st, P, (const T*)dy, (const T*)x, (const T*)bias, (T*)dx,
                       out, rps);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || nsplit == 1) return e;
  hipLaunchKernelGGL(bda_bwd_finish_kernel, dim3((unsigned)((P.h + 255) / 256)), dim3(256), 0, st, (const float*)ws, nsplit, P.h, dbias);
  return hipGetLastError();
}

hipError_t launch_bias_gelu_bwd(const RowsParams& P, bool bf16, const void* dy, const void* x, const void* bias, void* dx, float* dbias, void* ws,
                                hipStream_t st) {
  return bf16 ? bias_gelu_bwd_t<uint16_t>(P, dy, x, bias, dx, dbias, ws, st) : bias_gelu_bwd_t<float>(P, dy, x, bias, dx, dbias, ws, st);
}

}  // namespace sar
