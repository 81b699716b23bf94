// Attention core in plain fp32 arithmetic, one wavefront per score row (forward, dQ) or per score column
// (dK, dV).  Serves (i) the fp32 dtype, (ii) the stored-activation baseline of Section 4.1 (P, M, D written
// in the forward and read back in the backward), for any head dimension d % 4 == 0 up to 256.
// The bf16 recompute path of Section 5 at the benchmark head dimensions lives in attn_mfma_rows.hip (forward, dQ pass) and attn_mfma_cols_kernel.h (dK/dV pass).
#include "sar_device.h"
#include "sar_internal.h"

namespace sar {

static constexpr int kWavesPerBlock = 4;
static constexpr int kMaxD = 256;

__device__ __forceinline__ uint64_t score_elem(const AttnParams& P, int beta, int n, int i, int j) {
  return (((uint64_t)beta * (uint64_t)P.a_global + (uint64_t)(P.head0 + n)) * (uint64_t)P.s + (uint64_t)i) * (uint64_t)P.s + (uint64_t)j;
}

// ---------------------------------------------------------------------------------------------------
// forward: row i of (batch beta, head n).  Section 4.1: S = alpha q.k, causal softmax, dropout, times V.
// ---------------------------------------------------------------------------------------------------
template <typename T, bool STORED>
__global__ __launch_bounds__(kWavesPerBlock * 64) void attn_fwd_simple_kernel(AttnParams P, const T* __restrict__ q, const T* __restrict__ k,
                                                                              const T* __restrict__ v, T* __restrict__ o, float* __restrict__ lse,
                                                                              T* __restrict__ Pst, uint8_t* __restrict__ Mst, T* __restrict__ Dst) {
  extern __shared__ float smem[];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int i = blockIdx.x * kWavesPerBlock + wave;
  const int bn = blockIdx.y, beta = bn / P.A, n = bn % P.A;
  const bool valid = i < P.s;
  float* prow = smem + (size_t)wave * (P.s + kMaxD);
  float* qrow = prow + P.s;
  const int64_t base = (int64_t)beta * P.stride_b + (int64_t)n * P.stride_a;
  const int ic = valid ? i : 0;
  const int jend = P.causal ? i : P.s - 1;  // last key this row attends to
  for (int x = lane; x < P.d; x += 64) qrow[x] = Elem<T>::load(q + base + (int64_t)ic * P.stride_s + x);
  __syncthreads();
  float mx = -INFINITY;
  if (valid)
    for (int j = lane; j <= jend; j += 64) {
      const T* kj = k + base + (int64_t)j * P.stride_s;
      float acc = 0.f;
      for (int x = 0; x < P.d; ++x) acc = fmaf(qrow[x], Elem<T>::load(kj + x), acc);
      float sc = P.scale * acc;
      prow[j] = sc;
      mx = fmaxf(mx, sc);
    }
  mx = wave_max(mx);
  float sum = 0.f;
  if (valid)
    for (int j = lane; j <= jend; j += 64) {
      float e = expf(prow[j] - mx);
      prow[j] = e;
      sum += e;
    }
  sum = wave_sum(sum);
  const float inv = 1.f / sum;
  if (valid) {
    const size_t srow = ((size_t)bn * P.s + i) * P.s;
    for (int j = lane; j < P.s; j += 64) {
      if (j <= jend) {
        float pj = prow[j] * inv;
        uint32_t keep = keep_bit1(score_elem(P, beta, n, i, j), P.offset, 0u, P.key0, P.key1, P.thresh);
        float dj = keep ? pj * P.keep_scale : 0.f;
        if (STORED) {
          Elem<T>::store(Pst + srow + j, pj);
          Mst[srow + j] = (uint8_t)keep;
          Elem<T>::store(Dst + srow + j, dj);
          dj = Elem<T>::load(Dst + srow + j);  // the stored path multiplies the rounded D by V
        }
        prow[j] = dj;
      } else if (STORED) {
        Elem<T>::store(Pst + srow + j, 0.f);
        Mst[srow + j] = 0;
        Elem<T>::store(Dst + srow + j, 0.f);
      }
    }
  }
  __syncthreads();
  if (valid) {
    for (int x = lane; x < P.d; x += 64) {
      float acc = 0.f;
      for (int j = 0; j <= jend; ++j) acc = fmaf(prow[j], Elem<T>::load(v + base + (int64_t)j * P.stride_s + x), acc);
      Elem<T>::store(o + base + (int64_t)i * P.stride_s + x, acc);
    }
    if (lane == 0 && lse) lse[(size_t)bn * P.s + i] = mx + logf(sum);
  }
}

// ---------------------------------------------------------------------------------------------------
// backward, row pass: dS row i and dQ_i = alpha dS_i K; also emits the row term delta_i.
// Recompute mode (Section 5): P_ij = exp(alpha q_i.k_j - lse_i), mask regenerated, delta_i = dO_i . O_i.
// Stored mode: P, M read back; delta_i = sum_j P_ij dP_ij.
// ---------------------------------------------------------------------------------------------------
template <typename T, bool STORED>
__global__ __launch_bounds__(kWavesPerBlock * 64) void attn_bwd_rows_simple_kernel(AttnParams P, const T* __restrict__ q, const T* __restrict__ k,
                                                                                   const T* __restrict__ v, const T* __restrict__ o,
                                                                                   const float* __restrict__ lse, const T* __restrict__ dO,
                                                                                   T* __restrict__ dq, float* __restrict__ delta,
                                                                                   const T* __restrict__ Pst, const uint8_t* __restrict__ Mst) {
  extern __shared__ float smem[];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int i = blockIdx.x * kWavesPerBlock + wave;
  const int bn = blockIdx.y, beta = bn / P.A, n = bn % P.A;
  const bool valid = i < P.s;
  float* prow = smem + (size_t)wave * (2 * P.s + 2 * kMaxD);
  float* dsrow = prow + P.s;
  float* qrow = dsrow + P.s;
  float* dorow = qrow + kMaxD;
  const int64_t base = (int64_t)beta * P.stride_b + (int64_t)n * P.stride_a;
  const int ic = valid ? i : 0;
  const int jend = P.causal ? i : P.s - 1;  // last key this row attends to
  float dsum = 0.f;
  for (int x = lane; x < P.d; x += 64) {
    qrow[x] = Elem<T>::load(q + base + (int64_t)ic * P.stride_s + x);
    dorow[x] = Elem<T>::load(dO + base + (int64_t)ic * P.stride_s + x);
    if (!STORED) dsum = fmaf(dorow[x], Elem<T>::load(o + base + (int64_t)ic * P.stride_s + x), dsum);
  }
  __syncthreads();
  const float lse_i = STORED ? 0.f : lse[(size_t)bn * P.s + ic];
  const size_t srow = ((size_t)bn * P.s + ic) * P.s;
  float psum = 0.f;
  if (valid)
    for (int j = lane; j <= jend; j += 64) {
      const T* kj = k + base + (int64_t)j * P.stride_s;
      const T* vj = v + base + (int64_t)j * P.stride_s;
      float accd = 0.f;
      for (int x = 0; x < P.d; ++x) accd = fmaf(dorow[x], Elem<T>::load(vj + x), accd);
      float pj;
      uint32_t keep;
      if (STORED) {
        pj = Elem<T>::load(Pst + srow + j);
        keep = Mst[srow + j];
      } else {
        float accs = 0.f;
        for (int x = 0; x < P.d; ++x) accs = fmaf(qrow[x], Elem<T>::load(kj + x), accs);
        pj = expf(P.scale * accs - lse_i);
        keep = keep_bit1(score_elem(P, beta, n, i, j), P.offset, 0u, P.key0, P.key1, P.thresh);
      }
      float dp = keep ? accd * P.keep_scale : 0.f;
      prow[j] = pj;
      dsrow[j] = dp;
      psum = fmaf(pj, dp, psum);
    }
  const float dl = STORED ? wave_sum(psum) : wave_sum(dsum);
  if (valid) {
    for (int j = lane; j <= jend; j += 64) dsrow[j] = prow[j] * (dsrow[j] - dl);
    if (lane == 0) delta[(size_t)bn * P.s + i] = dl;
  }
  __syncthreads();
  if (valid)
    for (int x = lane; x < P.d; x += 64) {
      float acc = 0.f;
      for (int j = 0; j <= jend; ++j) acc = fmaf(dsrow[j], Elem<T>::load(k + base + (int64_t)j * P.stride_s + x), acc);
      Elem<T>::store(dq + base + (int64_t)i * P.stride_s + x, P.scale * acc);
    }
}

// ---------------------------------------------------------------------------------------------------
// backward, column pass: dK_j = alpha sum_i dS_ij q_i, dV_j = sum_i D_ij dO_i, over the rows i that attend to key j.
// ---------------------------------------------------------------------------------------------------
template <typename T, bool STORED>
__global__ __launch_bounds__(kWavesPerBlock * 64) void attn_bwd_cols_simple_kernel(AttnParams P, const T* __restrict__ q, const T* __restrict__ k,
                                                                                   const T* __restrict__ v, const float* __restrict__ lse,
                                                                                   const T* __restrict__ dO, const float* __restrict__ delta,
                                                                                   T* __restrict__ dk, T* __restrict__ dv,
                                                                                   const T* __restrict__ Pst, const uint8_t* __restrict__ Mst,
                                                                                   const T* __restrict__ Dst) {
  __shared__ float sk[kWavesPerBlock][kMaxD], sv[kWavesPerBlock][kMaxD], sds[kWavesPerBlock][64], sdd[kWavesPerBlock][64];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int j = blockIdx.x * kWavesPerBlock + wave;
  const int bn = blockIdx.y, beta = bn / P.A, n = bn % P.A;
  const bool valid = j < P.s;
  const int jc = valid ? j : 0;
  const int64_t base = (int64_t)beta * P.stride_b + (int64_t)n * P.stride_a;
  for (int x = lane; x < P.d; x += 64) {
    sk[wave][x] = Elem<T>::load(k + base + (int64_t)jc * P.stride_s + x);
    sv[wave][x] = Elem<T>::load(v + base + (int64_t)jc * P.stride_s + x);
  }
  __syncthreads();
  float acck[kMaxD / 64] = {0.f, 0.f, 0.f, 0.f}, accv[kMaxD / 64] = {0.f, 0.f, 0.f, 0.f};
  // every wave of the block runs the same number of chunk iterations so that the barriers match
  const int j_first = P.causal ? blockIdx.x * kWavesPerBlock : 0;
  for (int i0 = j_first; i0 < P.s; i0 += 64) {
    const int i = i0 + lane;
    float ds = 0.f, dd = 0.f;
    if (valid && (i >= j || !P.causal) && i < P.s) {
      const T* doi = dO + base + (int64_t)i * P.stride_s;
      float accd = 0.f;
      for (int x = 0; x < P.d; ++x) accd = fmaf(Elem<T>::load(doi + x), sv[wave][x], accd);
      float pij;
      uint32_t keep;
      const size_t sidx = ((size_t)bn * P.s + i) * P.s + j;
      if (STORED) {
        pij = Elem<T>::load(Pst + sidx);
        keep = Mst[sidx];
        dd = Elem<T>::load(Dst + sidx);
      } else {
        const T* qi = q + base + (int64_t)i * P.stride_s;
        float accs = 0.f;
        for (int x = 0; x < P.d; ++x) accs = fmaf(Elem<T>::load(qi + x), sk[wave][x], accs);
        pij = expf(P.scale * accs - lse[(size_t)bn * P.s + i]);
        keep = keep_bit1(score_elem(P, beta, n, i, j), P.offset, 0u, P.key0, P.key1, P.thresh);
        dd = keep ? pij * P.keep_scale : 0.f;
      }
      float dp = keep ? accd * P.keep_scale : 0.f;
      ds = pij * (dp - delta[(size_t)bn * P.s + i]);
    }
    sds[wave][lane] = ds;
    sdd[wave][lane] = dd;
    __syncthreads();
    const int cnt = min(64, P.s - i0);
#pragma unroll
    for (int c = 0; c < kMaxD / 64; ++c) {
      const int x = lane + 64 * c;
      if (x < P.d)
        for (int ii = 0; ii < cnt; ++ii) {
          acck[c] = fmaf(sds[wave][ii], Elem<T>::load(q + base + (int64_t)(i0 + ii) * P.stride_s + x), acck[c]);
          accv[c] = fmaf(sdd[wave][ii], Elem<T>::load(dO + base + (int64_t)(i0 + ii) * P.stride_s + x), accv[c]);
        }
    }
    __syncthreads();
  }
  if (valid) {
#pragma unroll
    for (int c = 0; c < kMaxD / 64; ++c) {
      const int x = lane + 64 * c;
      if (x < P.d) {
        Elem<T>::store(dk + base + (int64_t)j * P.stride_s + x, P.scale * acck[c]);
        Elem<T>::store(dv + base + (int64_t)j * P.stride_s + x, accv[c]);
      }
    }
  }
}

size_t attn_simple_lds_bytes(int s) { return (size_t)kWavesPerBlock * (2 * (size_t)s + 2 * kMaxD) * sizeof(float); }

template <typename T>
static hipError_t fwd_t(const AttnParams& P, const void* q, const void* k, const void* v, void* o, float* lse, void* Pst, uint8_t* Mst, void* Dst,
                        hipStream_t st) {
  dim3 grid((P.s + kWavesPerBlock - 1) / kWavesPerBlock, P.b * P.A), block(kWavesPerBlock * 64);
  size_t lds = (size_t)kWavesPerBlock * ((size_t)P.s + kMaxD) * sizeof(float);
  if (Pst) {
    auto kern = attn_fwd_simple_kernel<T, true>;
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, grid, block, lds, st, P, (const T*)q, (const T*)k, (const T*)v, (T*)o, lse, (T*)Pst, Mst, (T*)Dst);
  } else {
    auto kern = attn_fwd_simple_kernel<T, false>;
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, grid, block, lds, st, P, (const T*)q, (const T*)k, (const T*)v, (T*)o, lse, (T*)nullptr, (uint8_t*)nullptr, (T*)nullptr);
  }
  return hipGetLastError();
}

hipError_t launch_attn_fwd_simple(const AttnParams& P, bool bf16, const void* q, const void* k, const void* v, void* o, float* lse, void* Pst,
                                  uint8_t* Mst, void* Dst, hipStream_t st) {
  return bf16 ? fwd_t<uint16_t>(P, q, k, v, o, lse, Pst, Mst, Dst, st) : fwd_t<float>(P, q, k, v, o, lse, Pst, Mst, Dst, st);
}

template <typename T>
static hipError_t bwd_t(const AttnParams& P, const void* q, const void* k, const void* v, const void* o, const float* lse, const void* dO, void* dq,
                        void* dk, void* dv, float* delta, const void* Pst, const uint8_t* Mst, const void* Dst, int passes, hipStream_t st) {
  dim3 grid((P.s + kWavesPerBlock - 1) / kWavesPerBlock, P.b * P.A), block(kWavesPerBlock * 64);
  size_t lds = attn_simple_lds_bytes(P.s);
  hipError_t e;
  if (Pst) {
    auto ka = attn_bwd_rows_simple_kernel<T, true>;
    e = hipFuncSetAttribute((const void*)ka, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    if (passes & 1)
      hipLaunchKernelGGL(ka, grid, block, lds, st, P, (const T*)q, (const T*)k, (const T*)v, (const T*)o, lse, (const T*)dO, (T*)dq, delta,
                         (const T*)Pst, Mst);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (passes & 2)
    hipLaunchKernelGGL((attn_bwd_cols_simple_kernel<T, true>), grid, block, 0, st, P, (const T*)q, (const T*)k, (const T*)v, lse, (const T*)dO,
                       (const float*)delta, (T*)dk, (T*)dv, (const T*)Pst, Mst, (const T*)Dst);
  } else {
    auto ka = attn_bwd_rows_simple_kernel<T, false>;
    e = hipFuncSetAttribute((const void*)ka, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    if (passes & 1)
      hipLaunchKernelGGL(ka, grid, block, lds, st, P, (const T*)q, (const T*)k, (const T*)v, (const T*)o, lse, (const T*)dO, (T*)dq, delta,
                         (const T*)nullptr, (const uint8_t*)nullptr);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (passes & 2)
    hipLaunchKernelGGL((attn_bwd_cols_simple_kernel<T, false>), grid, block, 0, st, P, (const T*)q, (const T*)k, (const T*)v, lse, (const T*)dO,
                       (const float*)delta, (T*)dk, (T*)dv, (const T*)nullptr, (const uint8_t*)nullptr, (const T*)nullptr);
  }
  return hipGetLastError();
}

hipError_t launch_attn_bwd_simple(const AttnParams& P, bool bf16, const void* q, const void* k, const void* v, const void* o, const float* lse,
                                  const void* dO, void* dq, void* dk, void* dv, float* delta, const void* Pst, const uint8_t* Mst, const void* Dst,
                                  int passes, hipStream_t st) {
  return bf16 ? bwd_t<uint16_t>(P, q, k, v, o, lse, dO, dq, dk, dv, delta, Pst, Mst, Dst, passes, st)
              : bwd_t<float>(P, q, k, v, o, lse, dO, dq, dk, dv, delta, Pst, Mst, Dst, passes, st);
}

}  // namespace sar
