// bf16 attention core, backward column pass (dK, dV): head dimensions 128 and 160 (one wave per SIMD, accumulators in
// AGPRs; compiled WITHOUT -amdgpu-mfma-vgpr-form) and the dispatch over the head dimension.
#define SAR_COLS_ACC "a"
#include "attn_mfma_cols_pipe.h"

#include <atomic>

namespace sar {

// form of the column pass at d = 128, 160 and s % 64 == 0: -1 = the library's choice; 0 plain, 1 software-pipelined,
// 2 producer / consumer waves, 3 the same with persistent workgroups (forced forms fall back where they do not exist: 1 to
// the plain one, 3 to 2)
static std::atomic<int> g_force_form{-1};
void attn_mfma_force_dkdv_pipelined(int force) { g_force_form = force; }

hipError_t launch_attn_bwd_dkdv_mfma_small(const AttnParams& P, const void* q, const void* k, const void* v, const float* lse, const void* dO,
                                           const float* delta, void* dk, void* dv, uint16_t* ds_ws, hipStream_t st);  // attn_mfma_cols_small.hip
hipError_t launch_attn_bwd_dkdv_mfma_split(const AttnParams& P, const void* q, const void* k, const void* v, const float* lse, const void* dO,
                                           const float* delta, void* dk, void* dv, uint16_t* ds_ws, int pers, hipStream_t st);  // attn_mfma_cols_split.hip

// the form that runs: 0 plain, 1 software-pipelined, 2 producer / consumer (3: forced persistent)
template <int D>
static int dkdv_form(const AttnParams& P, const uint16_t* ds_ws) {
  if (P.s % 64 != 0) return 0;
  const int force = g_force_form.load();
  if (force >= 0) return (D < 128 && force == 1) ? 0 : force;  // the software-pipelined form exists for d = 128, 160 only
  // d = 64 (22B shard): 101.5 against 107.1 us with the dS stores of the once-form, 90.2 against 86.2 without
  if (D < 128) return ds_ws ? 2 : 0;
  // measured (once-form, us): 530B shard 78.6 / 80.2 / 69.6, 175B 70.4 / 60.5 / 48.1, 1T 98.3 / - / 90.0 for forms 0 / 1 / 2
  return 2;
}

// persistent workgroups in the producer / consumer form: -1 the launcher decides by shape, 0 / 1 forced
static int split_pers() {
  const int force = g_force_form.load();
  return force == 2 ? 0 : force == 3 ? 1 : -1;
}

hipError_t launch_attn_bwd_dkdv_mfma(const AttnParams& P, const void* q, const void* k, const void* v, const float* lse, const void* dO,
                                     const float* delta, void* dk, void* dv, uint16_t* ds_ws, hipStream_t st) {
  switch (P.d) {
    case 64:
      if (dkdv_form<64>(P, ds_ws) >= 2) return launch_attn_bwd_dkdv_mfma_split(P, q, k, v, lse, dO, delta, dk, dv, ds_ws, split_pers(), st);
      return launch_attn_bwd_dkdv_mfma_small(P, q, k, v, lse, dO, delta, dk, dv, ds_ws, st);
    case 96:
      if (dkdv_form<96>(P, ds_ws) >= 2) return launch_attn_bwd_dkdv_mfma_split(P, q, k, v, lse, dO, delta, dk, dv, ds_ws, split_pers(), st);
      return launch_attn_bwd_dkdv_mfma_small(P, q, k, v, lse, dO, delta, dk, dv, ds_ws, st);
    case 128:
      switch (dkdv_form<128>(P, ds_ws)) {
        case 2:
        case 3: return launch_attn_bwd_dkdv_mfma_split(P, q, k, v, lse, dO, delta, dk, dv, ds_ws, split_pers(), st);
        case 1: return bwd_dkdv_pipe_d<128>(P, q, k, v, lse, dO, delta, dk, dv, ds_ws, st);
        default: return bwd_dkdv_d<128>(P, q, k, v, lse, dO, delta, dk, dv, ds_ws, st);
      }
    case 160:
      switch (dkdv_form<160>(P, ds_ws)) {
        case 2:
        case 3: return launch_attn_bwd_dkdv_mfma_split(P, q, k, v, lse, dO, delta, dk, dv, ds_ws, split_pers(), st);
        case 1: return bwd_dkdv_pipe_d<160>(P, q, k, v, lse, dO, delta, dk, dv, ds_ws, st);
        default: return bwd_dkdv_d<160>(P, q, k, v, lse, dO, delta, dk, dv, ds_ws, st);
      }
    default: return hipErrorInvalidValue;
  }
}

}  // namespace sar
