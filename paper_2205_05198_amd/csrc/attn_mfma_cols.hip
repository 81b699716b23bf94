// bf16 attention core, backward column pass (dK, dV): head dimensions 128 and 160 (one wave per SIMD, accumulators in
// AGPRs; compiled WITHOUT -amdgpu-mfma-vgpr-form) and the dispatch over the head dimension.
#define SAR_COLS_ACC "a"
#include "attn_mfma_cols_pipe.h"

#include <atomic>

namespace sar {

static std::atomic<int> g_force_pipe{-1};
void attn_mfma_force_dkdv_pipelined(int force) { g_force_pipe = force; }

hipError_t launch_attn_bwd_dkdv_mfma_small(const AttnParams& P, const void* q, const void* k, const void* v, const float* lse, const void* dO,
                                           const float* delta, void* dk, void* dv, uint16_t* ds_ws, hipStream_t st);  // attn_mfma_cols_small.hip

hipError_t launch_attn_bwd_dkdv_mfma(const AttnParams& P, const void* q, const void* k, const void* v, const float* lse, const void* dO,
                                     const float* delta, void* dk, void* dv, uint16_t* ds_ws, hipStream_t st) {
  switch (P.d) {
    case 64:
    case 96: return launch_attn_bwd_dkdv_mfma_small(P, q, k, v, lse, dO, delta, dk, dv, ds_ws, st);
    case 128: return bwd_dkdv_use_pipe<128>(P, g_force_pipe.load()) ? bwd_dkdv_pipe_d<128>(P, q, k, v, lse, dO, delta, dk, dv, ds_ws, st)
                                               : bwd_dkdv_d<128>(P, q, k, v, lse, dO, delta, dk, dv, ds_ws, st);
    case 160: return bwd_dkdv_use_pipe<160>(P, g_force_pipe.load()) ? bwd_dkdv_pipe_d<160>(P, q, k, v, lse, dO, delta, dk, dv, ds_ws, st)
                                               : bwd_dkdv_d<160>(P, q, k, v, lse, dO, delta, dk, dv, ds_ws, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace sar
