// C-ABI layer of libsar: argument validation on the host, then kernel launches on the caller's stream.
// See include/sar.h for the contract of every entry point.
#include "../../include/sar.h"

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <mutex>

#include "sar_internal.h"

namespace {

thread_local char g_err[256] = "";

sar_status fail(sar_status st, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return st;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Dropout threshold on 16 random bits: floor(p * 65536 + 0.5) from the float p.
inline uint32_t dropout_threshold(float p) { return (uint32_t)std::floor((double)p * 65536.0 + 0.5); }

sar_status check_attn_desc(const sar_attn_desc* c, sar::AttnParams* P) {
  if (!c) return fail(SAR_ERR_NULL, "descriptor is NULL");
  if (c->s <= 0 || c->b <= 0 || c->a <= 0 || c->t <= 0 || c->h <= 0) return fail(SAR_ERR_SHAPE, "s, b, a, t, h must be positive");
  if (c->a % c->t != 0) return fail(SAR_ERR_SHAPE, "a (%d) is not a multiple of t (%d)", c->a, c->t);
  if (c->h % c->a != 0) return fail(SAR_ERR_SHAPE, "h (%d) is not a multiple of a (%d)", c->h, c->a);
  if (c->rank < 0 || c->rank >= c->t) return fail(SAR_ERR_SHAPE, "rank %d outside [0, t)", c->rank);
  if (c->dtype != SAR_F32 && c->dtype != SAR_BF16) return fail(SAR_ERR_UNSUPPORTED, "dtype %d", c->dtype);
  if (c->causal != 0 && c->causal != 1) return fail(SAR_ERR_SHAPE, "causal must be 0 or 1 (got %d)", c->causal);
  if (!(c->p >= 0.f && c->p < 1.f)) return fail(SAR_ERR_PROB, "dropout probability %g outside [0, 1)", (double)c->p);
  if (!std::isfinite(c->scale)) return fail(SAR_ERR_SHAPE, "scale is not finite");
  const int d = c->h / c->a, A = c->a / c->t;
  if (c->s % 8 != 0) return fail(SAR_ERR_UNSUPPORTED, "s (%d) must be a multiple of 8", c->s);
  if (c->s > 32768) return fail(SAR_ERR_UNSUPPORTED, "s (%d) above 32768", c->s);
  if (d % 4 != 0 || d > 256) return fail(SAR_ERR_UNSUPPORTED, "head dimension %d (need a multiple of 4, at most 256)", d);
  if (c->dtype == SAR_BF16 && d % 8 != 0) return fail(SAR_ERR_UNSUPPORTED, "bf16 head dimension %d must be a multiple of 8", d);
  const int64_t esz = c->dtype == SAR_BF16 ? 2 : 4;
  if (c->stride_a < d || c->stride_b < 0 || c->stride_s < 0) return fail(SAR_ERR_SHAPE, "strides must be non-negative and stride_a >= d");
  if ((c->stride_s * esz) % 16 || (c->stride_b * esz) % 16 || (c->stride_a * esz) % 16) return fail(SAR_ERR_ALIGN, "strides must be multiples of 16 bytes");
  if ((int64_t)c->b * A > 65535) return fail(SAR_ERR_UNSUPPORTED, "b * a/t above 65535");
  if (P) {
    P->s = c->s; P->b = c->b; P->A = A; P->d = d;
    P->a_global = c->a; P->head0 = c->rank * A;
    P->stride_s = c->stride_s; P->stride_b = c->stride_b; P->stride_a = c->stride_a;
    P->causal = c->causal;
    P->scale = c->scale; P->p = c->p; P->keep_scale = 1.0f / (1.0f - c->p);
    P->thresh = dropout_threshold(c->p);
    P->key0 = (uint32_t)(c->seed & 0xFFFFFFFFu); P->key1 = (uint32_t)(c->seed >> 32);
    P->offset = c->offset;
  }
  return SAR_OK;
}

bool use_mfma(const sar_attn_desc* c, const sar::AttnParams& P) { return c->dtype == SAR_BF16 && sar::attn_mfma_supported(P.d) && c->scale > 0.f; }

// The matrix-core kernels address a 64-row tile with 32-bit byte offsets from the tile's first row.
sar_status check_mfma_limits(const sar::AttnParams& P) {
  if (63 * P.stride_s * 2 + 2 * (int64_t)P.d >= (1ll << 31)) return fail(SAR_ERR_UNSUPPORTED, "stride_s (%lld) too large for the bf16 kernels", (long long)P.stride_s);
  return SAR_OK;
}

// workspace of the backward: delta (one float per row) and, for the path that recomputes the region once, the dS tiles
size_t delta_bytes(const sar::AttnParams& P) { return ((size_t)P.b * P.A * P.s * sizeof(float) + 255) / 256 * 256; }
size_t ds_bytes(const sar::AttnParams& P) { return (size_t)P.b * P.A * (size_t)sar::ds_tiles_per_head(P) * sar::kDsTileElems * 2; }
constexpr size_t kDsWorkspaceCap = 8ull << 30;  // above this attn_core_bwd_workspace asks for the two-pass backward's scratch only

sar_status check_simple_limits(const sar::AttnParams& P) {
  if (sar::attn_simple_lds_bytes(P.s) > 160 * 1024) return fail(SAR_ERR_UNSUPPORTED, "s (%d) too long for this dtype / head dimension", P.s);
  return SAR_OK;
}

sar_status hip_fail(hipError_t e, const char* what) { return fail(SAR_ERR_HIP, "%s: %s", what, hipGetErrorString(e)); }

sar_status check_rows_desc(const sar_rows_desc* c, sar::RowsParams* P) {
  if (!c) return fail(SAR_ERR_NULL, "descriptor is NULL");
  if (c->rows <= 0 || c->h <= 0 || c->row_offset < 0) return fail(SAR_ERR_SHAPE, "rows, h must be positive and row_offset non-negative");
  if (c->dtype != SAR_F32 && c->dtype != SAR_BF16) return fail(SAR_ERR_UNSUPPORTED, "dtype %d", c->dtype);
  if (c->h % 8 != 0) return fail(SAR_ERR_UNSUPPORTED, "h (%lld) must be a multiple of 8", (long long)c->h);
  if (c->h > 32768) return fail(SAR_ERR_UNSUPPORTED, "h (%lld) above 32768", (long long)c->h);
  if (c->rows > 0x7fffffffLL) return fail(SAR_ERR_UNSUPPORTED, "rows above 2^31-1");
  if (!(c->p >= 0.f && c->p < 1.f)) return fail(SAR_ERR_PROB, "dropout probability %g outside [0, 1)", (double)c->p);
  if (!(c->eps >= 0.f) || !std::isfinite(c->eps)) return fail(SAR_ERR_SHAPE, "eps must be finite and non-negative");
  if (P) {
    P->rows = c->rows; P->h = c->h; P->row_offset = c->row_offset;
    P->eps = c->eps; P->p = c->p; P->keep_scale = 1.0f / (1.0f - c->p);
    P->thresh = dropout_threshold(c->p);
    P->key0 = (uint32_t)(c->seed & 0xFFFFFFFFu); P->key1 = (uint32_t)(c->seed >> 32);
    P->offset = c->offset;
  }
  return SAR_OK;
}

// Scratch of attn_core_bwd_recompute_noalloc: one array per GPU, part of the loaded code object, held until the process
// ends.  In host code the array's name is only a handle; its device address on the current GPU comes from
// hipGetSymbolAddress, asked once per device, and is what the kernels get.
constexpr size_t kStaticScratchBytes = 1u << 20;
constexpr int kMaxDevices = 64;
}  // namespace

static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

sar_status static_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
  if (dev < 0 || dev >= kMaxDevices) return fail(SAR_ERR_UNSUPPORTED, "device index %d outside [0, %d)", dev, kMaxDevices);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) return hip_fail(e, "hipGetSymbolAddress(scratch)");
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return SAR_OK;
}
}  // namespace

extern "C" {

const char* sar_last_error(void) { return g_err; }

sar_status attn_core_fwd(const sar_attn_desc* desc, const void* q, const void* k, const void* v, void* o, float* lse, void* stream) {
  sar::AttnParams P;
  sar_status st = check_attn_desc(desc, &P);
  if (st != SAR_OK) return st;
  if (!q || !k || !v || !o || !lse) return fail(SAR_ERR_NULL, "attn_core_fwd: NULL tensor pointer");
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(lse)) return fail(SAR_ERR_ALIGN, "attn_core_fwd: pointer not 16-byte aligned");
  hipError_t e;
  if (use_mfma(desc, P)) {
    if ((st = check_mfma_limits(P)) != SAR_OK) return st;
    e = sar::launch_attn_fwd_mfma(P, q, k, v, o, lse, (hipStream_t)stream);
  } else {
    if ((st = check_simple_limits(P)) != SAR_OK) return st;
    e = sar::launch_attn_fwd_simple(P, desc->dtype == SAR_BF16, q, k, v, o, lse, nullptr, nullptr, nullptr, (hipStream_t)stream);
  }
  return e == hipSuccess ? SAR_OK : hip_fail(e, "attn_core_fwd launch");
}

size_t attn_core_bwd_workspace_min(const sar_attn_desc* desc) {
  sar::AttnParams P;
  if (check_attn_desc(desc, &P) != SAR_OK) return 0;
  return delta_bytes(P);  // delta_i = dO_i . O_i per row
}

size_t attn_core_bwd_workspace(const sar_attn_desc* desc) {
  sar::AttnParams P;
  if (check_attn_desc(desc, &P) != SAR_OK) return 0;
  if (use_mfma(desc, P) && ds_bytes(P) <= kDsWorkspaceCap) return delta_bytes(P) + ds_bytes(P);
  return delta_bytes(P);
}

void sar_test_force_variants(int fwd_128_rows, int fwd_loader_waves, int dq_loader_waves, int dkdv_pipelined) {
  sar::attn_mfma_force_variants(fwd_128_rows, fwd_loader_waves, dq_loader_waves);
  sar::attn_mfma_force_dkdv_pipelined(dkdv_pipelined);
}

// passes: two-pass backward, bit 0 = row pass, bit 1 = column pass.  stages (passes == 0): the backward that recomputes the
// region once, bit 0 = delta, bit 1 = column pass + dS tiles, bit 2 = dQ from the tiles.  passes == 3 and stages == 7: the
// whole backward, by whichever of the two the workspace allows.
static sar_status bwd_recompute_impl(const char* who, const sar_attn_desc* desc, const void* q, const void* k, const void* v, const void* o,
                                     const float* lse, const void* d_o, void* dq, void* dk, void* dv, void* workspace, size_t workspace_bytes,
                                     int passes, int stages, void* stream) {
  sar::AttnParams P;
  sar_status st = check_attn_desc(desc, &P);
  if (st != SAR_OK) return st;
  const bool mfma = use_mfma(desc, P);
  if (passes && stages) {  // the whole backward
    if (mfma && workspace && workspace_bytes >= delta_bytes(P) + ds_bytes(P)) passes = 0;
    else stages = 0;
  }
  if (stages && !mfma) return fail(SAR_ERR_UNSUPPORTED, "%s: the single-recompute backward needs bf16 and a head dimension of 64, 96, 128 or 160", who);
  const bool rowp = (passes & 1) || (stages & 5), colp = (passes & 2) || (stages & 2);
  const bool need_o = (passes & 1) || (stages & 1), need_dq = (passes & 1) || (stages & 4);
  if (!k || !v || !lse || !d_o || ((passes || (stages & 2)) && !q) || (need_o && !o) || (need_dq && !dq) || (colp && (!dk || !dv)))
    return fail(SAR_ERR_NULL, "%s: NULL tensor pointer", who);
  (void)rowp;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(lse) || !aligned16(d_o) || !aligned16(dq) || !aligned16(dk) ||
      !aligned16(dv))
    return fail(SAR_ERR_ALIGN, "%s: pointer not 16-byte aligned", who);
  const void* ins[5] = {q, k, v, o, d_o};
  void* outs[3] = {need_dq ? dq : nullptr, colp ? dk : nullptr, colp ? dv : nullptr};
  for (int x = 0; x < 3; ++x) {
    if (!outs[x]) continue;
    for (int y = 0; y < 5; ++y)
      if (outs[x] == ins[y]) return fail(SAR_ERR_SHAPE, "%s: outputs may not alias inputs", who);
    for (int y = x + 1; y < 3; ++y)
      if (outs[x] == outs[y]) return fail(SAR_ERR_SHAPE, "%s: outputs may not alias each other", who);
  }
  const size_t need = stages ? delta_bytes(P) + ds_bytes(P) : delta_bytes(P);
  if (!workspace || workspace_bytes < need) return fail(SAR_ERR_WORKSPACE, "workspace needs %zu bytes, got %zu", need, workspace_bytes);
  if (!aligned16(workspace)) return fail(SAR_ERR_ALIGN, "workspace not 16-byte aligned");
  hipError_t e;
  if (mfma) {
    if ((st = check_mfma_limits(P)) != SAR_OK) return st;
    if (stages)
      e = sar::launch_attn_bwd_once_mfma(P, q, k, v, o, lse, d_o, dq, dk, dv, (float*)workspace,
                                         reinterpret_cast<uint16_t*>(static_cast<char*>(workspace) + delta_bytes(P)), stages, (hipStream_t)stream);
    else
      e = sar::launch_attn_bwd_mfma(P, q, k, v, o, lse, d_o, dq, dk, dv, (float*)workspace, passes, (hipStream_t)stream);
  } else {
    if ((st = check_simple_limits(P)) != SAR_OK) return st;
    e = sar::launch_attn_bwd_simple(P, desc->dtype == SAR_BF16, q, k, v, o, lse, d_o, dq, dk, dv, (float*)workspace, nullptr, nullptr, nullptr, passes,
                                    (hipStream_t)stream);
  }
  return e == hipSuccess ? SAR_OK : hip_fail(e, who);
}

sar_status attn_core_bwd_recompute(const sar_attn_desc* desc, const void* q, const void* k, const void* v, const void* o, const float* lse,
                                   const void* d_o, void* dq, void* dk, void* dv, void* workspace, size_t workspace_bytes, void* stream) {
  return bwd_recompute_impl("attn_core_bwd_recompute", desc, q, k, v, o, lse, d_o, dq, dk, dv, workspace, workspace_bytes, 3, 7, stream);
}

size_t attn_core_bwd_noalloc_max_bytes(void) { return kStaticScratchBytes; }

sar_status attn_core_bwd_recompute_noalloc(const sar_attn_desc* desc, const void* q, const void* k, const void* v, const void* o, const float* lse,
                                           const void* d_o, void* dq, void* dk, void* dv, void* stream) {
  sar::AttnParams P;
  sar_status st = check_attn_desc(desc, &P);
  if (st != SAR_OK) return st;
  const size_t need = delta_bytes(P);
  if (need > kStaticScratchBytes)
    return fail(SAR_ERR_UNSUPPORTED, "attn_core_bwd_recompute_noalloc: b * a/t * s = %lld rows need %zu bytes of scratch, the built-in buffer holds %zu",
                (long long)P.b * P.A * P.s, need, kStaticScratchBytes);
  void* ws = nullptr;
  if ((st = static_scratch(&ws)) != SAR_OK) return st;
  // the two-pass form: its only scratch is one float per query row, written by the row pass before the column pass reads it
  return bwd_recompute_impl("attn_core_bwd_recompute_noalloc", desc, q, k, v, o, lse, d_o, dq, dk, dv, ws, need, 3, 0, stream);
}

sar_status attn_core_bwd_recompute_stages(const sar_attn_desc* desc, int stages, const void* q, const void* k, const void* v, const void* o,
                                          const float* lse, const void* d_o, void* dq, void* dk, void* dv, void* workspace, size_t workspace_bytes,
                                          void* stream) {
  if (stages < 1 || stages > 7) return fail(SAR_ERR_SHAPE, "attn_core_bwd_recompute_stages: stages must be a non-empty subset of 1 | 2 | 4");
  return bwd_recompute_impl("attn_core_bwd_recompute_stages", desc, q, k, v, o, lse, d_o, dq, dk, dv, workspace, workspace_bytes, 0, stages, stream);
}

sar_status attn_core_bwd_recompute_dq(const sar_attn_desc* desc, const void* q, const void* k, const void* v, const void* o, const float* lse,
                                      const void* d_o, void* dq, void* workspace, size_t workspace_bytes, void* stream) {
  return bwd_recompute_impl("attn_core_bwd_recompute_dq", desc, q, k, v, o, lse, d_o, dq, nullptr, nullptr, workspace, workspace_bytes, 1, 0, stream);
}

sar_status attn_core_bwd_recompute_dkdv(const sar_attn_desc* desc, const void* q, const void* k, const void* v, const float* lse, const void* d_o,
                                        void* dk, void* dv, void* workspace, size_t workspace_bytes, void* stream) {
  return bwd_recompute_impl("attn_core_bwd_recompute_dkdv", desc, q, k, v, nullptr, lse, d_o, nullptr, dk, dv, workspace, workspace_bytes, 2, 0, stream);
}

sar_status attn_core_fwd_stored(const sar_attn_desc* desc, const void* q, const void* k, const void* v, void* o, float* lse, void* Pst, uint8_t* Mst,
                                void* Dst, void* stream) {
  sar::AttnParams P;
  sar_status st = check_attn_desc(desc, &P);
  if (st != SAR_OK) return st;
  if (!q || !k || !v || !o || !lse || !Pst || !Mst || !Dst) return fail(SAR_ERR_NULL, "attn_core_fwd_stored: NULL tensor pointer");
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(lse) || !aligned16(Pst) || !aligned16(Mst) || !aligned16(Dst))
    return fail(SAR_ERR_ALIGN, "attn_core_fwd_stored: pointer not 16-byte aligned");
  hipError_t e;
  if (use_mfma(desc, P) && sar::attn_mfma_stored_supported(P)) {
    if ((st = check_mfma_limits(P)) != SAR_OK) return st;
    e = sar::launch_attn_fwd_mfma(P, q, k, v, o, lse, (hipStream_t)stream);
    if (e == hipSuccess) e = sar::launch_attn_store_pmd_mfma(P, q, k, lse, Pst, Mst, Dst, (hipStream_t)stream);
  } else {
    if ((st = check_simple_limits(P)) != SAR_OK) return st;
    e = sar::launch_attn_fwd_simple(P, desc->dtype == SAR_BF16, q, k, v, o, lse, Pst, Mst, Dst, (hipStream_t)stream);
  }
  return e == hipSuccess ? SAR_OK : hip_fail(e, "attn_core_fwd_stored launch");
}

sar_status attn_core_bwd_stored(const sar_attn_desc* desc, const void* q, const void* k, const void* v, const void* o, const void* Pst,
                                const uint8_t* Mst, const void* Dst, const void* d_o, void* dq, void* dk, void* dv, void* workspace,
                                size_t workspace_bytes, void* stream) {
  sar::AttnParams P;
  sar_status st = check_attn_desc(desc, &P);
  if (st != SAR_OK) return st;
  if (!q || !k || !v || !o || !Pst || !Mst || !Dst || !d_o || !dq || !dk || !dv) return fail(SAR_ERR_NULL, "attn_core_bwd_stored: NULL tensor pointer");
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(Pst) || !aligned16(Mst) || !aligned16(Dst) || !aligned16(d_o) ||
      !aligned16(dq) || !aligned16(dk) || !aligned16(dv))
    return fail(SAR_ERR_ALIGN, "attn_core_bwd_stored: pointer not 16-byte aligned");
  const size_t need = delta_bytes(P);
  if (!workspace || workspace_bytes < need) return fail(SAR_ERR_WORKSPACE, "workspace needs %zu bytes, got %zu", need, workspace_bytes);
  if (!aligned16(workspace)) return fail(SAR_ERR_ALIGN, "workspace not 16-byte aligned");
  hipError_t e;
  if (use_mfma(desc, P) && sar::attn_mfma_stored_supported(P)) {
    if ((st = check_mfma_limits(P)) != SAR_OK) return st;
    e = sar::launch_attn_bwd_stored_mfma(P, q, k, v, o, d_o, Pst, Mst, Dst, dq, dk, dv, (float*)workspace, (hipStream_t)stream);
  } else {
    if ((st = check_simple_limits(P)) != SAR_OK) return st;
    e = sar::launch_attn_bwd_simple(P, desc->dtype == SAR_BF16, q, k, v, nullptr, nullptr, d_o, dq, dk, dv, (float*)workspace, Pst, Mst, Dst, 3,
                                    (hipStream_t)stream);
  }
  return e == hipSuccess ? SAR_OK : hip_fail(e, "attn_core_bwd_stored launch");
}

uint64_t attn_core_saved_bytes(const sar_attn_desc* desc, int selective) {
  sar::AttnParams P;
  if (check_attn_desc(desc, &P) != SAR_OK) return 0;
  const uint64_t esz = desc->dtype == SAR_BF16 ? 2 : 4;
  const uint64_t qkvo = 4ull * esz * (uint64_t)P.s * P.b * P.A * P.d;       // Q, K, V (6sbh/t) + O (2sbh/t)
  if (selective) return qkvo;                                               // Section 5: no s^2 term
  return qkvo + (2ull * esz + 1ull) * (uint64_t)P.A * P.s * P.s * P.b;      // + softmax out, mask, dropout out
}

uint64_t attn_core_small_buffer_bytes(const sar_attn_desc* desc) {
  sar::AttnParams P;
  if (check_attn_desc(desc, &P) != SAR_OK) return 0;
  return 4ull * (uint64_t)P.A * P.s * P.b + 16ull;
}

uint64_t attn_core_philox_count(const sar_attn_desc* desc) {
  if (check_attn_desc(desc, nullptr) != SAR_OK) return 0;
  return (uint64_t)desc->b * (uint64_t)desc->a * (uint64_t)desc->s * (uint64_t)desc->s / 8ull;
}

sar_status ln_fwd(const sar_rows_desc* desc, const void* x, const void* gamma, const void* beta, void* y, float* mean, float* rstd, void* stream) {
  sar::RowsParams P;
  sar_status st = check_rows_desc(desc, &P);
  if (st != SAR_OK) return st;
  if (!x || !gamma || !beta || !y || !mean || !rstd) return fail(SAR_ERR_NULL, "ln_fwd: NULL tensor pointer");
  if (!aligned16(x) || !aligned16(gamma) || !aligned16(beta) || !aligned16(y)) return fail(SAR_ERR_ALIGN, "ln_fwd: pointer not 16-byte aligned");
  hipError_t e = sar::launch_ln_fwd(P, desc->dtype == SAR_BF16, x, gamma, beta, y, mean, rstd, (hipStream_t)stream);
  return e == hipSuccess ? SAR_OK : hip_fail(e, "ln_fwd launch");
}

size_t ln_bwd_workspace(const sar_rows_desc* desc) {
  if (check_rows_desc(desc, nullptr) != SAR_OK) return 0;
  return sar::ln_bwd_workspace_bytes(desc->rows, desc->h);
}

sar_status ln_bwd(const sar_rows_desc* desc, const void* dy, const void* x, const float* mean, const float* rstd, const void* gamma, void* dx,
                  float* dgamma, float* dbeta, void* workspace, size_t workspace_bytes, void* stream) {
  sar::RowsParams P;
  sar_status st = check_rows_desc(desc, &P);
  if (st != SAR_OK) return st;
  if (!dy || !x || !mean || !rstd || !gamma || !dx || !dgamma || !dbeta) return fail(SAR_ERR_NULL, "ln_bwd: NULL tensor pointer");
  if (!aligned16(dy) || !aligned16(x) || !aligned16(gamma) || !aligned16(dx)) return fail(SAR_ERR_ALIGN, "ln_bwd: pointer not 16-byte aligned");
  const size_t need = sar::ln_bwd_workspace_bytes(P.rows, P.h);
  if (!workspace || workspace_bytes < need) return fail(SAR_ERR_WORKSPACE, "workspace needs %zu bytes, got %zu", need, workspace_bytes);
  if (!aligned16(workspace)) return fail(SAR_ERR_ALIGN, "workspace not 16-byte aligned");
  hipError_t e = sar::launch_ln_bwd(P, desc->dtype == SAR_BF16, dy, x, mean, rstd, gamma, dx, dgamma, dbeta, workspace, (hipStream_t)stream);
  return e == hipSuccess ? SAR_OK : hip_fail(e, "ln_bwd launch");
}

sar_status bias_dropout_add(const sar_rows_desc* desc, const void* x, const void* bias, const void* resid, void* out, uint8_t* mask_out, void* stream) {
  sar::RowsParams P;
  sar_status st = check_rows_desc(desc, &P);
  if (st != SAR_OK) return st;
  if (!x || !resid || !out) return fail(SAR_ERR_NULL, "bias_dropout_add: NULL tensor pointer");
  if (!aligned16(x) || !aligned16(resid) || !aligned16(out) || (bias && !aligned16(bias)) || (mask_out && (reinterpret_cast<uintptr_t>(mask_out) & 7u)))
    return fail(SAR_ERR_ALIGN, "bias_dropout_add: pointer not aligned (16 bytes; mask 8 bytes)");
  if (out == x) return fail(SAR_ERR_SHAPE, "bias_dropout_add: out may alias resid only");
  hipError_t e = sar::launch_bias_dropout_add(P, desc->dtype == SAR_BF16, x, bias, resid, out, mask_out, (hipStream_t)stream);
  return e == hipSuccess ? SAR_OK : hip_fail(e, "bias_dropout_add launch");
}

sar_status bias_dropout_add_ln_fwd(const sar_rows_desc* desc, const void* x, const void* bias, const void* resid, const void* gamma, const void* beta,
                                   void* out, void* y, float* mean, float* rstd, void* stream) {
  sar::RowsParams P;
  sar_status st = check_rows_desc(desc, &P);
  if (st != SAR_OK) return st;
  if (!x || !resid || !gamma || !beta || !out || !y || !mean || !rstd) return fail(SAR_ERR_NULL, "bias_dropout_add_ln_fwd: NULL tensor pointer");
  if (!aligned16(x) || !aligned16(resid) || !aligned16(gamma) || !aligned16(beta) || !aligned16(out) || !aligned16(y) || (bias && !aligned16(bias)))
    return fail(SAR_ERR_ALIGN, "bias_dropout_add_ln_fwd: pointer not 16-byte aligned");
  if (out == x || y == x || y == resid || y == out) return fail(SAR_ERR_SHAPE, "bias_dropout_add_ln_fwd: out may alias resid only; y aliases nothing");
  hipError_t e = sar::launch_bias_dropout_add_ln_fwd(P, desc->dtype == SAR_BF16, x, bias, resid, gamma, beta, out, y, mean, rstd, (hipStream_t)stream);
  return e == hipSuccess ? SAR_OK : hip_fail(e, "bias_dropout_add_ln_fwd launch");
}

size_t bias_dropout_add_bwd_workspace(const sar_rows_desc* desc) {
  if (check_rows_desc(desc, nullptr) != SAR_OK) return 0;
  return sar::bda_bwd_workspace_bytes(desc->rows, desc->h);
}

sar_status bias_dropout_add_bwd(const sar_rows_desc* desc, const void* dout, void* dx, float* dbias, void* workspace, size_t workspace_bytes,
                                void* stream) {
  sar::RowsParams P;
  sar_status st = check_rows_desc(desc, &P);
  if (st != SAR_OK) return st;
  if (!dout || !dx) return fail(SAR_ERR_NULL, "bias_dropout_add_bwd: NULL tensor pointer");
  if (!aligned16(dout) || !aligned16(dx)) return fail(SAR_ERR_ALIGN, "bias_dropout_add_bwd: pointer not 16-byte aligned");
  if (dbias) {
    const size_t need = sar::bda_bwd_workspace_bytes(P.rows, P.h);
    if (need && (!workspace || workspace_bytes < need)) return fail(SAR_ERR_WORKSPACE, "workspace needs %zu bytes, got %zu", need, workspace_bytes);
    if (need && !aligned16(workspace)) return fail(SAR_ERR_ALIGN, "workspace not 16-byte aligned");
  }
  hipError_t e = sar::launch_bias_dropout_add_bwd(P, desc->dtype == SAR_BF16, dout, dx, dbias, workspace, (hipStream_t)stream);
  return e == hipSuccess ? SAR_OK : hip_fail(e, "bias_dropout_add_bwd launch");
}

sar_status bias_gelu_fwd(const sar_rows_desc* desc, const void* x, const void* bias, void* y, void* stream) {
  sar::RowsParams P;
  sar_status st = check_rows_desc(desc, &P);
  if (st != SAR_OK) return st;
  if (!x || !y) return fail(SAR_ERR_NULL, "bias_gelu_fwd: NULL tensor pointer");
  if (!aligned16(x) || !aligned16(y) || (bias && !aligned16(bias))) return fail(SAR_ERR_ALIGN, "bias_gelu_fwd: pointer not 16-byte aligned");
  hipError_t e = sar::launch_bias_gelu_fwd(P, desc->dtype == SAR_BF16, x, bias, y, (hipStream_t)stream);
  return e == hipSuccess ? SAR_OK : hip_fail(e, "bias_gelu_fwd launch");
}

size_t bias_gelu_bwd_workspace(const sar_rows_desc* desc) {
  if (check_rows_desc(desc, nullptr) != SAR_OK) return 0;
  return sar::bias_gelu_bwd_workspace_bytes(desc->rows, desc->h);
}

sar_status bias_gelu_bwd(const sar_rows_desc* desc, const void* dy, const void* x, const void* bias, void* dx, float* dbias, void* workspace,
                         size_t workspace_bytes, void* stream) {
  sar::RowsParams P;
  sar_status st = check_rows_desc(desc, &P);
  if (st != SAR_OK) return st;
  if (!dy || !x || !dx) return fail(SAR_ERR_NULL, "bias_gelu_bwd: NULL tensor pointer");
  if (!aligned16(dy) || !aligned16(x) || !aligned16(dx) || (bias && !aligned16(bias)))
    return fail(SAR_ERR_ALIGN, "bias_gelu_bwd: pointer not 16-byte aligned");
  if (dbias) {
    const size_t need = sar::bias_gelu_bwd_workspace_bytes(P.rows, P.h);
    if (need && (!workspace || workspace_bytes < need)) return fail(SAR_ERR_WORKSPACE, "workspace needs %zu bytes, got %zu", need, workspace_bytes);
    if (need && !aligned16(workspace)) return fail(SAR_ERR_ALIGN, "workspace not 16-byte aligned");
  }
  hipError_t e = sar::launch_bias_gelu_bwd(P, desc->dtype == SAR_BF16, dy, x, bias, dx, dbias, workspace, (hipStream_t)stream);
  return e == hipSuccess ? SAR_OK : hip_fail(e, "bias_gelu_bwd launch");
}

}  // extern "C"
