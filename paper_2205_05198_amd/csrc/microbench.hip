// Measurement hooks (not part of the method): what this GPU attains on the two rooflines that bound the library's kernels,
// measured with kernels as simple as possible.
//   sar_bench_mfma   a register-resident loop of v_mfma_f32_32x32x16_bf16 on constant operands, four independent
//                    accumulator chains per wave, two waves per SIMD on every CU: the matrix cores' attainable rate
//   sar_bench_copy   a grid-stride copy, 16 bytes per lane and access: the attainable HBM read + write rate
//   sar_bench_issue  what one instruction costs the wave that issues it (cycles of s_memtime between the first and the last of
//                    a long unrolled run), alone on its SIMD or beside a second wave: the attention kernels run one or two
//                    waves per SIMD, a wave issues in order, and a step costs it the sum of these
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


// ---- issue costs ----
#define SAR_REP8(x) x x x x x x x x
enum IssueOp { OP_FMA_IND, OP_FMA_DEP, OP_MAD64_IND, OP_EXP_IND, OP_CMP_VCC, OP_CMP_SGPR, OP_MFMA, OP_FMA8_MFMA, OP_LDS_B128, OP_IDLE };
// one iteration of a probe; instructions per iteration in kIssueInsts
template <int OP>
__device__ __forceinline__ void issue_body(float (&f)[8], uint32_t (&u)[8], uint64_t (&q)[4], float16_t (&acc)[4], bf16x8_t a, bf16x8_t b, uint32_t lds) {
  if constexpr (OP == OP_FMA_IND) {  // 64 independent fused multiply-adds
    SAR_REP8(asm volatile("v_fma_f32 %0, %0, %8, %8\n v_fma_f32 %1, %1, %8, %8\n v_fma_f32 %2, %2, %8, %8\n v_fma_f32 %3, %3, %8, %8\n v_fma_f32 %4, %4, %8, %8\n v_fma_f32 %5, %5, %8, %8\n v_fma_f32 %6, %6, %8, %8\n v_fma_f32 %7, %7, %8, %8" : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]), "+v"(f[4]), "+v"(f[5]), "+v"(f[6]), "+v"(f[7]) : "v"(1.0001f));)
  } else if constexpr (OP == OP_FMA_DEP) {  // 64, each on the result of the one before
    SAR_REP8(SAR_REP8(asm volatile("v_fma_f32 %0, %0, %1, %1" : "+v"(f[0]) : "v"(1.0001f));))
  } else if constexpr (OP == OP_MAD64_IND) {  // 64 independent 32 x 32 -> 64 bit multiplies (the Philox round's)
    SAR_REP8(asm volatile("v_mad_u64_u32 %0, vcc, %4, %5, 0\n v_mad_u64_u32 %1, vcc, %4, %6, 0\n v_mad_u64_u32 %2, vcc, %4, %7, 0\n v_mad_u64_u32 %3, vcc, %4, %8, 0\n v_mad_u64_u32 %0, vcc, %4, %5, 0\n v_mad_u64_u32 %1, vcc, %4, %6, 0\n v_mad_u64_u32 %2, vcc, %4, %7, 0\n v_mad_u64_u32 %3, vcc, %4, %8, 0" : "+v"(q[0]), "+v"(q[1]), "+v"(q[2]), "+v"(q[3]) : "v"(0xD2511F53u), "v"(u[0]), "v"(u[1]), "v"(u[2]), "v"(u[3]) : "vcc");)
  } else if constexpr (OP == OP_EXP_IND) {  // 64 independent exponentials
    SAR_REP8(asm volatile("v_exp_f32 %0, %0\n v_exp_f32 %1, %1\n v_exp_f32 %2, %2\n v_exp_f32 %3, %3\n v_exp_f32 %4, %4\n v_exp_f32 %5, %5\n v_exp_f32 %6, %6\n v_exp_f32 %7, %7" : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]), "+v"(f[4]), "+v"(f[5]), "+v"(f[6]), "+v"(f[7]));)
  } else if constexpr (OP == OP_CMP_VCC) {  // 32 keep decisions as the compiler writes them: compare into vcc, two idle states, select
    SAR_REP8(asm volatile("v_cmp_ge_u32_sdwa vcc, %4, %5 src0_sel:WORD_0 src1_sel:DWORD\n s_nop 1\n v_cndmask_b32 %0, 0, %6, vcc\n v_cmp_ge_u32_sdwa vcc, %4, %5 src0_sel:WORD_1 src1_sel:DWORD\n s_nop 1\n v_cndmask_b32 %1, 0, %6, vcc\n v_cmp_ge_u32_sdwa vcc, %7, %5 src0_sel:WORD_0 src1_sel:DWORD\n s_nop 1\n v_cndmask_b32 %2, 0, %6, vcc\n v_cmp_ge_u32_sdwa vcc, %7, %5 src0_sel:WORD_1 src1_sel:DWORD\n s_nop 1\n v_cndmask_b32 %3, 0, %6, vcc" : "=v"(f[0]), "=v"(f[1]), "=v"(f[2]), "=v"(f[3]) : "v"(u[0]), "s"(0x1999u), "v"(f[4]), "v"(u[1]) : "vcc");)
  } else if constexpr (OP == OP_CMP_SGPR) {  // 32 keep decisions as keep_select8 writes them: four compares into four scalar register pairs, four selects
    uint64_t m0, m1, m2, m3;
    SAR_REP8(asm volatile("v_cmp_ge_u32_sdwa %4, %8, %9 src0_sel:WORD_0 src1_sel:DWORD\n v_cmp_ge_u32_sdwa %5, %8, %9 src0_sel:WORD_1 src1_sel:DWORD\n v_cmp_ge_u32_sdwa %6, %10, %9 src0_sel:WORD_0 src1_sel:DWORD\n v_cmp_ge_u32_sdwa %7, %10, %9 src0_sel:WORD_1 src1_sel:DWORD\n v_cndmask_b32_e64 %0, 0, %11, %4\n v_cndmask_b32_e64 %1, 0, %11, %5\n v_cndmask_b32_e64 %2, 0, %11, %6\n v_cndmask_b32_e64 %3, 0, %11, %7" : "=&v"(f[0]), "=&v"(f[1]), "=&v"(f[2]), "=&v"(f[3]), "=&s"(m0), "=&s"(m1), "=&s"(m2), "=&s"(m3) : "v"(u[0]), "s"(0x1999u), "v"(u[1]), "v"(f[4]));)
  } else if constexpr (OP == OP_MFMA) {  // 64 matrix instructions on four accumulator chains
#pragma unroll
    for (int r = 0; r < 64; ++r) acc[r & 3] = mfma32(a, b, acc[r & 3]);
  } else if constexpr (OP == OP_FMA8_MFMA) {  // 8 x (one matrix instruction, eight independent fused multiply-adds) of the same wave
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      acc[r & 3] = mfma32(a, b, acc[r & 3]);
      asm volatile("v_fma_f32 %0, %0, %8, %8\n v_fma_f32 %1, %1, %8, %8\n v_fma_f32 %2, %2, %8, %8\n v_fma_f32 %3, %3, %8, %8\n v_fma_f32 %4, %4, %8, %8\n v_fma_f32 %5, %5, %8, %8\n v_fma_f32 %6, %6, %8, %8\n v_fma_f32 %7, %7, %8, %8" : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]), "+v"(f[4]), "+v"(f[5]), "+v"(f[6]), "+v"(f[7]) : "v"(1.0001f));
    }
  } else if constexpr (OP == OP_LDS_B128) {  // 8 x (eight 16-byte LDS reads, then a wait for all of them)
    u32x4_t r0, r1, r2, r3;
    SAR_REP8(asm volatile("ds_read_b128 %0, %4\n ds_read_b128 %1, %4 offset:1024\n ds_read_b128 %2, %4 offset:2048\n ds_read_b128 %3, %4 offset:3072\n ds_read_b128 %0, %4 offset:4096\n ds_read_b128 %1, %4 offset:5120\n ds_read_b128 %2, %4 offset:6144\n ds_read_b128 %3, %4 offset:7168\n s_waitcnt lgkmcnt(0)" : "=&v"(r0), "=&v"(r1), "=&v"(r2), "=&v"(r3) : "v"(lds));)
    u[0] ^= r0[0] ^ r1[0] ^ r2[0] ^ r3[0];
  }
}
__host__ __device__ constexpr int issue_insts(int op) { return op == OP_CMP_VCC || op == OP_CMP_SGPR ? 64 : op == OP_FMA8_MFMA ? 72 : op == OP_IDLE ? 0 : 64; }

// waves 0..3 of a workgroup run OPA, waves 4..7 (if launched) OPB; cycles[workgroup * 8 + wave] = cycles for `iters` iterations
template <int OPA, int OPB>
__global__ __launch_bounds__(512, 1) void issue_kernel(unsigned long long* __restrict__ cycles, float* __restrict__ sink, int iters) {
  __shared__ uint32_t lds[4096];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  float f[8];
  uint32_t u[8];
  uint64_t q[4];
  float16_t acc[4];
#pragma unroll
  for (int i = 0; i < 8; ++i) { f[i] = 0.5f + 0.001f * (float)(lane + i); u[i] = 0x9E3779B9u * (uint32_t)(lane + i + 1); }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    q[i] = u[i];
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
  }
  bf16x8_t a, b;
  {
    union { uint16_t h[8]; bf16x8_t v; } w;
#pragma unroll
    for (int e = 0; e < 8; ++e) w.h[e] = (uint16_t)(0x3A00 + ((lane + e) & 15));
    a = w.v;
    b = w.v;
  }
  for (int i = threadIdx.x; i < 4096; i += blockDim.x) lds[i] = (uint32_t)i;
  __syncthreads();
  const uint32_t lp = lds_addr(lds) + 16u * (uint32_t)lane;  // + 7168 + 16 <= 16 KB
  const uint64_t t0 = __builtin_amdgcn_s_memtime();
  if (wave < 4) for (int it = 0; it < iters; ++it) issue_body<OPA>(f, u, q, acc, a, b, lp);
  else for (int it = 0; it < iters; ++it) issue_body<OPB>(f, u, q, acc, a, b, lp);
  const uint64_t t1 = __builtin_amdgcn_s_memtime();
  float t = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) t += f[i] + (float)u[i];
#pragma unroll
  for (int i = 0; i < 4; ++i) t += (float)q[i] + acc[i][0] + acc[i][5];
  if (t == 12345.678f) sink[0] = t;  // keeps the probes alive
  if (lane == 0) cycles[blockIdx.x * 8 + wave] = t1 - t0;
}

struct IssueProbe { const char* name; int opa, opb; void (*kern)(unsigned long long*, float*, int); };
#define SAR_PROBE(n, A, B) {n, A, B, issue_kernel<A, B>}
static const IssueProbe kIssueProbes[] = {
    SAR_PROBE("vector instruction, independent", OP_FMA_IND, OP_IDLE),
    SAR_PROBE("vector instruction, dependent on the one before", OP_FMA_DEP, OP_IDLE),
    SAR_PROBE("32x32->64 multiply (Philox), independent", OP_MAD64_IND, OP_IDLE),
    SAR_PROBE("exponential, independent", OP_EXP_IND, OP_IDLE),
    SAR_PROBE("keep decision through vcc (compare, 2 idle, select), per instruction of the pair", OP_CMP_VCC, OP_IDLE),
    SAR_PROBE("keep decision through scalar register pairs (4 compares, 4 selects), per instruction of the pair", OP_CMP_SGPR, OP_IDLE),
    SAR_PROBE("matrix instruction 32x32x16 bf16", OP_MFMA, OP_IDLE),
    SAR_PROBE("one matrix instruction + eight independent vector instructions, per instruction", OP_FMA8_MFMA, OP_IDLE),
    SAR_PROBE("LDS read of 16 bytes per lane, eight in flight", OP_LDS_B128, OP_IDLE),
    SAR_PROBE("two waves: vector | vector", OP_FMA_IND, OP_FMA_IND),
    SAR_PROBE("two waves: dependent vector | dependent vector", OP_FMA_DEP, OP_FMA_DEP),
    SAR_PROBE("two waves: matrix | vector", OP_MFMA, OP_FMA_IND),
    SAR_PROBE("two waves: matrix | exponential", OP_MFMA, OP_EXP_IND),
    SAR_PROBE("two waves: matrix | matrix", OP_MFMA, OP_MFMA),
    SAR_PROBE("two waves: matrix | LDS read", OP_MFMA, OP_LDS_B128),
};
constexpr int kNumIssueProbes = (int)(sizeof(kIssueProbes) / sizeof(kIssueProbes[0]));

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

const char* sar_bench_issue_name(int probe) { return probe >= 0 && probe < sar::kNumIssueProbes ? sar::kIssueProbes[probe].name : nullptr; }

sar_status sar_bench_issue(int probe, int iters, unsigned long long* cycles, int workgroups, float* sink, int* insts_a, int* insts_b, void* stream) {
  if (probe < 0 || probe >= sar::kNumIssueProbes || iters <= 0 || workgroups <= 0) return SAR_ERR_SHAPE;
  if (!cycles || !sink || !insts_a || !insts_b) return SAR_ERR_NULL;
  const sar::IssueProbe& p = sar::kIssueProbes[probe];
  const bool two = p.opb != sar::OP_IDLE;
  hipLaunchKernelGGL(p.kern, dim3((unsigned)workgroups), dim3(two ? 512 : 256), 0, (hipStream_t)stream, cycles, sink, iters);
  if (hipGetLastError() != hipSuccess) return SAR_ERR_HIP;
  *insts_a = sar::issue_insts(p.opa);
  *insts_b = two ? sar::issue_insts(p.opb) : 0;
  return SAR_OK;
}

}  // extern "C"
