// Measurement hooks (not part of the method): what this GPU attains on the two rooflines that bound the library's kernels,
// measured with kernels as simple as possible.
//   sar_bench_mfma   a register-resident loop of v_mfma_f32_32x32x16_bf16 on constant operands, four independent
//                    accumulator chains per wave, two waves per SIMD on every CU: the matrix cores' attainable rate
//   sar_bench_copy   a grid-stride copy, 16 bytes per lane and access: the attainable HBM read + write rate
#include "../../include/sar.h"
#include "attn_mfma_common.h"

namespace sar {

__global__ __launch_bounds__(512) void mfma_peak_kernel(int iters, float* __restrict__ sink) {
  bf16x8_t a, b;
  {
    union { uint16_t h[8]; bf16x8_t v; } u;
#pragma unroll
    for (int e = 0; e < 8; ++e) u.h[e] = (uint16_t)(0x3C00 + ((threadIdx.x + e) & 15));  // small positive values
    a = u.v;
    b = u.v;
  }
  float16_t acc[4];
#pragma unroll
  for (int c = 0; c < 4; ++c)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[c][e] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int c = 0; c < 4; ++c) acc[c] = mfma32(a, b, acc[c]);
  }
  float t = 0.f;
#pragma unroll
  for (int c = 0; c < 4; ++c) t += acc[c][0] + acc[c][15];
  if (t == 12345.678f) sink[0] = t;  // keeps the loop alive; never true for these operands
}

// four loads in flight per lane before the first store
__global__ __launch_bounds__(256) void copy_kernel(const u32x4_t* __restrict__ src, u32x4_t* __restrict__ dst, size_t n16) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  for (; i + 3 * stride < n16; i += 4 * stride) {
    const u32x4_t a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
    dst[i] = a;
    dst[i + stride] = b;
    dst[i + 2 * stride] = c;
    dst[i + 3 * stride] = d;
  }
  for (; i < n16; i += stride) dst[i] = src[i];
}

}  // namespace sar

extern "C" {

sar_status sar_bench_mfma(int iters, float* sink, double* flops_out, void* stream) {
  if (iters <= 0 || !sink || !flops_out) return SAR_ERR_NULL;
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) return SAR_ERR_HIP;
  // one workgroup of 8 waves per CU: two waves per SIMD
  hipLaunchKernelGGL(sar::mfma_peak_kernel, dim3((unsigned)cus), dim3(512), 0, (hipStream_t)stream, iters, sink);
  if (hipGetLastError() != hipSuccess) return SAR_ERR_HIP;
  *flops_out = (double)cus * 8.0 * 4.0 * (double)iters * 2.0 * 32.0 * 32.0 * 16.0;
  return SAR_OK;
}

sar_status sar_bench_copy(const void* src, void* dst, size_t bytes, void* stream) {
  if (!src || !dst) return SAR_ERR_NULL;
  if (bytes == 0 || bytes % 16 || (reinterpret_cast<uintptr_t>(src) & 15u) || (reinterpret_cast<uintptr_t>(dst) & 15u)) return SAR_ERR_ALIGN;
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) return SAR_ERR_HIP;
  hipLaunchKernelGGL(sar::copy_kernel, dim3((unsigned)(cus * 8)), dim3(256), 0, (hipStream_t)stream, (const sar::u32x4_t*)src, (sar::u32x4_t*)dst, bytes / 16);
  return hipGetLastError() == hipSuccess ? SAR_OK : SAR_ERR_HIP;
}

}  // extern "C"
