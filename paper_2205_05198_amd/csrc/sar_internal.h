// Host-side declarations shared by the translation units of libsar: kernel parameter blocks and the
// launchers each .hip file exports to the C-ABI layer (sar_api.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace sar {

struct AttnParams {
  int s, b, A, d;               // per-GPU share: A = a/t local heads, d = h/a
  int causal;                   // 1: keys j <= i only (decoder); 0: every key (encoder)
  int a_global, head0;          // global head count and global index of local head 0 (Philox indexing)
  int64_t stride_s, stride_b, stride_a;
  float scale;                  // alpha
  float p, keep_scale;          // dropout probability and 1/(1-p) in fp32
  uint32_t thresh;              // keep iff 16-bit field >= thresh
  uint32_t key0, key1;          // Philox key = seed
  uint64_t offset;              // Philox counter base
};

// dS tiles of the backward that recomputes the region once: one 64 x 64 bf16 tile per (batch*head, 64-row query tile `it`,
// 64-key block `kb`), kDsTileElems elements each; under the causal mask only the tiles with kb <= it exist.
static constexpr int kDsTileElems = 64 * 64;
__host__ __device__ inline int64_t ds_tiles_per_head(const AttnParams& P) {
  const int64_t nt = (P.s + 63) / 64;
  return P.causal ? nt * (nt + 1) / 2 : nt * nt;
}
__host__ __device__ inline int64_t ds_tile_index(const AttnParams& P, int it, int kb) {
  return P.causal ? (int64_t)it * (it + 1) / 2 + kb : (int64_t)it * ((P.s + 63) / 64) + kb;
}

struct RowsParams {
  int64_t rows, h, row_offset;
  float eps, p, keep_scale;
  uint32_t thresh, key0, key1;
  uint64_t offset;
};

// attn_simple.hip: one-wave-per-row kernels in plain fp32 arithmetic, any d % 4 == 0 up to 256; also the
// stored-activation baseline (P, M, D written / read).
hipError_t launch_attn_fwd_simple(const AttnParams& P, bool bf16, const void* q, const void* k, const void* v, void* o, float* lse,
                                  void* Pst, uint8_t* Mst, void* Dst, hipStream_t st);
// passes: bit 0 = row pass (dq, writes delta), bit 1 = column pass (dk, dv, reads delta)
hipError_t launch_attn_bwd_simple(const AttnParams& P, bool bf16, const void* q, const void* k, const void* v, const void* o,
                                  const float* lse, const void* dO, void* dq, void* dk, void* dv, float* delta,
                                  const void* Pst, const uint8_t* Mst, const void* Dst, int passes, hipStream_t st);
size_t attn_simple_lds_bytes(int s);

// attn_mfma_rows.hip (forward, dQ pass) and attn_mfma_cols.hip (dK/dV pass): bf16 MFMA kernels, d in {64, 96, 128, 160}
bool attn_mfma_supported(int d);
// attn_mfma_stored.hip: the stored-activation baseline on the same tiles (needs s % 64 == 0): P, M, D from Q, K, LSE after
// the forward; backward passes that read them back
bool attn_mfma_stored_supported(const AttnParams& P);
hipError_t launch_attn_store_pmd_mfma(const AttnParams& P, const void* q, const void* k, const float* lse, void* Pst, uint8_t* Mst, void* Dst,
                                      hipStream_t st);
hipError_t launch_attn_bwd_stored_mfma(const AttnParams& P, const void* q, const void* k, const void* v, const void* o, const void* dO, const void* Pst,
                                       const uint8_t* Mst, const void* Dst, void* dq, void* dk, void* dv, float* delta, hipStream_t st);
hipError_t launch_attn_fwd_mfma(const AttnParams& P, const void* q, const void* k, const void* v, void* o, float* lse, hipStream_t st);
hipError_t launch_attn_bwd_mfma(const AttnParams& P, const void* q, const void* k, const void* v, const void* o, const float* lse,
                                const void* dO, void* dq, void* dk, void* dv, float* delta, int passes, hipStream_t st);

// ds_ws != nullptr: the dS tiles are written there as well
hipError_t launch_attn_bwd_dkdv_mfma(const AttnParams& P, const void* q, const void* k, const void* v, const float* lse, const void* dO,
                                     const float* delta, void* dk, void* dv, uint16_t* ds_ws, hipStream_t st);
// attn_mfma_dsgemm.hip: the backward that recomputes the region once.  stages: bit 0 = delta_i = dO_i . O_i, bit 1 = column
// pass (dK, dV, and the dS tiles into ds_ws), bit 2 = dQ = alpha dS K from the tiles.
hipError_t launch_attn_bwd_once_mfma(const AttnParams& P, const void* q, const void* k, const void* v, const void* o, const float* lse,
                                     const void* dO, void* dq, void* dk, void* dv, float* delta, uint16_t* ds_ws, int stages, hipStream_t st);
// test hook: force kernel variants (-1 = the library's choice, 0 / 1 = off / on)
void attn_mfma_force_variants(int fwd128, int fwdlw, int dqlw);
void attn_mfma_force_dkdv_pipelined(int force);
int attn_mfma_cu_count();  // compute units of the current device, asked once

// rows.hip: LayerNorm forward/backward and bias-dropout-add on [rows, h]
hipError_t launch_ln_fwd(const RowsParams& P, bool bf16, const void* x, const void* gamma, const void* beta, void* y, float* mean,
                         float* rstd, hipStream_t st);
size_t ln_bwd_workspace_bytes(int64_t rows, int64_t h);
hipError_t launch_ln_bwd(const RowsParams& P, bool bf16, const void* dy, const void* x, const float* mean, const float* rstd,
                         const void* gamma, void* dx, float* dgamma, float* dbeta, void* ws, hipStream_t st);
hipError_t launch_bias_dropout_add(const RowsParams& P, bool bf16, const void* x, const void* bias, const void* resid, void* out,
                                   uint8_t* mask, hipStream_t st);
hipError_t launch_bias_dropout_add_ln_fwd(const RowsParams& P, bool bf16, const void* x, const void* bias, const void* resid, const void* gamma,
                                          const void* beta, void* out, void* y, float* mean, float* rstd, hipStream_t st);
size_t bda_bwd_workspace_bytes(int64_t rows, int64_t h);
hipError_t launch_bias_dropout_add_bwd(const RowsParams& P, bool bf16, const void* dout, void* dx, float* dbias, void* ws, hipStream_t st);
// bias + GeLU (the MLP block's non-linearity)
size_t bias_gelu_bwd_workspace_bytes(int64_t rows, int64_t h);
hipError_t launch_bias_gelu_fwd(const RowsParams& P, bool bf16, const void* x, const void* bias, void* y, hipStream_t st);
hipError_t launch_bias_gelu_bwd(const RowsParams& P, bool bf16, const void* dy, const void* x, const void* bias, void* dx, float* dbias, void* ws,
                                hipStream_t st);

}  // namespace sar
