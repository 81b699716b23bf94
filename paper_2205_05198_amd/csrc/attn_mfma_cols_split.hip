// bf16 attention core, backward column pass (dK, dV) in its producer / consumer form (two waves per SIMD, each within
// 256 vector registers; compiled WITH -amdgpu-mfma-vgpr-form): every head dimension of the matrix-core path, s % 64 == 0.
#define SAR_COLS_ACC "v"
#include "attn_mfma_cols_split.h"

#include <algorithm>

namespace sar {

template <int D>
static hipError_t bwd_dkdv_split_d(const AttnParams& P, const void* q, const void* k, const void* v, const float* lse, const void* dO, const float* delta,
                                   void* dk, void* dv, uint16_t* ds_ws, int pers, hipStream_t st) {
  const int N = P.b * P.A, nb = P.s / 64;
  // Persistent workgroups (each takes several key blocks of its head, a heavy one then a light one, and overlaps a block's
  // start with the end of the one before): needs (key blocks at a time) x (heads) workgroups within the CU count; chosen
  // when every workgroup then gets at least two key blocks.
  const int cus = attn_mfma_cu_count();
  const int R = N <= cus ? std::min(nb, cus / N) : 0;
  const bool use_pers = R > 0 && (pers == 1 || (pers < 0 && nb >= 2 * R));
  const unsigned grid = use_pers ? (unsigned)(R * N) : (unsigned)(nb * N);
  auto go = [&](auto kern) {
    hipLaunchKernelGGL(kern, dim3(grid), dim3(512), 0, st, P, (const uint16_t*)q, (const uint16_t*)k, (const uint16_t*)v, lse,
                       (const uint16_t*)dO, delta, (uint16_t*)dk, (uint16_t*)dv, ds_ws);
  };
  if (use_pers) {
    if (ds_ws) {
      if (P.thresh != 0) go(attn_bwd_dkdv_split_kernel<D, true, true, true>);
      else go(attn_bwd_dkdv_split_kernel<D, false, true, true>);
    } else {
      if (P.thresh != 0) go(attn_bwd_dkdv_split_kernel<D, true, false, true>);
      else go(attn_bwd_dkdv_split_kernel<D, false, false, true>);
    }
  } else if (ds_ws) {
    if (P.thresh != 0) go(attn_bwd_dkdv_split_kernel<D, true, true>);
    else go(attn_bwd_dkdv_split_kernel<D, false, true>);
  } else {
    if (P.thresh != 0) go(attn_bwd_dkdv_split_kernel<D, true, false>);
    else go(attn_bwd_dkdv_split_kernel<D, false, false>);
  }
  return hipGetLastError();
}

hipError_t launch_attn_bwd_dkdv_mfma_split(const AttnParams& P, const void* q, const void* k, const void* v, const float* lse, const void* dO,
                                           const float* delta, void* dk, void* dv, uint16_t* ds_ws, int pers, hipStream_t st) {
  if (P.s % 64 != 0) return hipErrorInvalidValue;
  switch (P.d) {
    case 64: return bwd_dkdv_split_d<64>(P, q, k, v, lse, dO, delta, dk, dv, ds_ws, pers, st);
    case 96: return bwd_dkdv_split_d<96>(P, q, k, v, lse, dO, delta, dk, dv, ds_ws, pers, st);
    case 128: return bwd_dkdv_split_d<128>(P, q, k, v, lse, dO, delta, dk, dv, ds_ws, pers, st);
    case 160: return bwd_dkdv_split_d<160>(P, q, k, v, lse, dO, delta, dk, dv, ds_ws, pers, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace sar
