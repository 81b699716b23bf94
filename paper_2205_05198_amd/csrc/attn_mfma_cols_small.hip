// bf16 attention core, backward column pass (dK, dV): head dimensions 64 and 96 (two workgroups per CU, everything in
// vector registers; compiled WITH -amdgpu-mfma-vgpr-form).
#define SAR_COLS_ACC "v"
#include "attn_mfma_cols_kernel.h"

namespace sar {

hipError_t launch_attn_bwd_dkdv_mfma_small(const AttnParams& P, const void* q, const void* k, const void* v, const float* lse, const void* dO,
                                           const float* delta, void* dk, void* dv, uint16_t* ds_ws, hipStream_t st) {
  switch (P.d) {
    case 64: return bwd_dkdv_d<64>(P, q, k, v, lse, dO, delta, dk, dv, ds_ws, st);
    case 96: return bwd_dkdv_d<96>(P, q, k, v, lse, dO, delta, dk, dv, ds_ws, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace sar
