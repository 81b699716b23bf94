/*
 * sar.h -- C ABI of the selective-activation-recomputation hot path for MI355X (gfx950).
 *
 * Method: "Reducing Activation Recomputation in Large Transformer Models" (arXiv 2205.05198).
 * The library implements, as hand-written HIP kernels,
 *   - the attention core that Section 5 selects for recomputation (QK^T, softmax, softmax dropout,
 *     attention over V; Section 4.1), in a form whose forward keeps only Q, K, V, O and a per-row
 *     log-sum-exp and whose backward regenerates softmax and the dropout mask on the fly, and
 *   - the memory-bound operators of the sequence-parallel region (Section 4.2.2, Eq. 3): LayerNorm
 *     forward/backward and dropout(+bias)+residual on one rank's s/t rows.
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller.  The library never allocates,
 *     frees or synchronises: each call validates its arguments on the host, enqueues its kernels on
 *     `stream` (a hipStream_t passed as void*, NULL = the default stream) and returns.
 *   - Return value: SAR_OK or a negative sar_status.  On any non-OK return nothing has been
 *     enqueued and no output byte is written; sar_last_error() gives a thread-local description.
 *   - Names follow the paper's Table 1: s sequence length, b microbatch, h hidden size, a attention
 *     heads, t tensor-parallel size; p is the dropout probability here (the paper's pipeline size
 *     does not appear in this library).
 *   - Attention tensors are the paper's s x b x h activations seen by one tensor-parallel rank:
 *     [s, b, A, d] with A = a/t local heads and d = h/a, d contiguous, element strides given in the
 *     descriptor.  Q, K, V, O and all gradients share the same strides.
 *   - Dropout masks are a pure function of (seed, offset, global element index): Philox4x32-10,
 *     key = seed, counter = (G lo, G hi, 0, site) with G = offset + (e >> 3); element e uses the
 *     16-bit field (e & 7) of the 128 output bits and is kept iff field >= floor(p*65536 + 0.5).
 *     Site 0 (softmax dropout): e = ((beta*a + rank*A + n)*s + i)*s + j.  Site 1 (bias-dropout-add):
 *     e = (row_offset + r)*h + c.  A shard therefore reproduces its slice of the unsharded mask.
 *   - Supported shapes: d in {64, 96, 128, 160} for bf16 (any multiple of 4 up to 256 for f32);
 *     s % 8 == 0; a % t == 0; h % a == 0; rows-kernels need h % 8 == 0 and h <= 32768.  Base pointers and
 *     row strides must be 16-byte aligned.  Anything else returns SAR_ERR_UNSUPPORTED / SAR_ERR_ALIGN.
 */
#ifndef SAR_H_
#define SAR_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  SAR_OK = 0,
  SAR_ERR_NULL = -1,        /* a required pointer is NULL                                  */
  SAR_ERR_SHAPE = -2,       /* a size is non-positive or inconsistent (a % t, h % a, ...)   */
  SAR_ERR_UNSUPPORTED = -3, /* a shape or option the kernels do not cover                   */
  SAR_ERR_ALIGN = -4,       /* pointer or stride not 16-byte aligned                        */
  SAR_ERR_PROB = -5,        /* dropout probability outside [0, 1)                           */
  SAR_ERR_WORKSPACE = -6,   /* workspace NULL or smaller than *_workspace() reports         */
  SAR_ERR_HIP = -7          /* a HIP runtime call failed (launch error)                     */
} sar_status;

typedef enum { SAR_F32 = 0, SAR_BF16 = 1 } sar_dtype;

/* Attention-core descriptor (paper notation, Table 1). */
typedef struct {
  int32_t s, b;            /* sequence length, microbatch                                          */
  int32_t a, t, rank;      /* global heads, tensor-parallel size, this GPU's rank in [0, t):
                              local head n has global index rank*(a/t) + n (used by Philox only)  */
  int32_t h;               /* hidden size; head dimension d = h / a                                */
  int32_t dtype;           /* sar_dtype of Q, K, V, O, dO, dQ, dK, dV                              */
  int32_t causal;          /* 1: decoder mask, keys j <= i (Section 6's models); 0: every key      */
  float scale;             /* alpha applied to QK^T; pass 1/sqrt(d)                                */
  float p;                 /* softmax-dropout probability, 0 <= p < 1                              */
  uint64_t seed, offset;   /* Philox key and counter base                                          */
  int64_t stride_s, stride_b, stride_a; /* element strides of [s, b, A, d]; packed layout:
                              stride_a = d, stride_b = A*d, stride_s = b*A*d                       */
} sar_attn_desc;

/*
 * attn_core_fwd -- Section 4.1 (QK^T, softmax, softmax dropout, attention over V) computed as in
 * Section 5: nothing of size s x s is written.
 *   q, k, v : in,  device, [s, b, A, d] in desc->dtype
 *   o       : out, device, same layout; O = (softmax(alpha QK^T, causal) o M / (1-p)) V
 *   lse     : out, device, float [b, A, s]; natural-log-sum-exp of row i's scaled scores
 * Saved set for the backward = {q, k, v, o, lse, seed, offset}.
 */
sar_status attn_core_fwd(const sar_attn_desc* desc, const void* q, const void* k, const void* v,
                         void* o, float* lse, void* stream);

/*
 * Scratch of attn_core_bwd_recompute (0 on error).  The backward exists in two forms, chosen by the workspace it is given:
 *   - workspace_bytes >= attn_core_bwd_workspace(desc): the region is recomputed ONCE.  The pass that forms dK, dV also
 *     writes the bf16 dS tiles (2 bytes per score pair that the mask allows, in 64 x 64 tiles: 2 A b s^2 bytes, about half
 *     of it under the causal mask) and dQ = alpha dS K is formed from them.  This scratch lives only inside the call;
 *     nothing of size s x s is kept from the forward (Section 5).  bf16 with head dimension 64 / 96 / 128 / 160 only.
 *   - workspace_bytes >= attn_core_bwd_workspace_min(desc) (one float per query row): the region is recomputed TWICE, once
 *     per query block for dQ and once per key block for dK, dV; scratch is O(s).
 * attn_core_bwd_workspace returns the first size while it stays below 8 GiB (16 heads: s = 8192 1.1 GB, s = 16384 4.3 GB,
 * s = 32768 17 GB), else the second.
 */
size_t attn_core_bwd_workspace(const sar_attn_desc* desc);
size_t attn_core_bwd_workspace_min(const sar_attn_desc* desc);

/*
 * attn_core_bwd_recompute -- backward of the region of Section 5: softmax P and the dropout mask are
 * regenerated from q, k, lse and (seed, offset); dq, dk, dv follow the chain rule through
 * Section 4.1's four operations.
 *   q, k, v, o, lse : in, exactly what attn_core_fwd received / produced
 *   d_o             : in, gradient of o, same layout and dtype
 *   dq, dk, dv      : out, same layout and dtype (may not alias inputs or each other)
 *   workspace       : device scratch of at least attn_core_bwd_workspace_min(desc) bytes, 16-byte
 *                     aligned; contents on entry are irrelevant, contents on exit unspecified.  Its size
 *                     selects the form of the backward (see attn_core_bwd_workspace).
 * Results are deterministic (no atomics).
 */
sar_status attn_core_bwd_recompute(const sar_attn_desc* desc, const void* q, const void* k, const void* v,
                                   const void* o, const float* lse, const void* d_o,
                                   void* dq, void* dk, void* dv,
                                   void* workspace, size_t workspace_bytes, void* stream);

/*
 * attn_core_bwd_recompute_noalloc -- for callers that cannot allocate device memory or bring a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  The same backward as attn_core_bwd_recompute in
 * its recompute-twice form (same kernels, same results bit for bit), with the scratch (one float per query row) in a
 * buffer that is built into the library: attn_core_bwd_noalloc_max_bytes() bytes (1 MiB) per GPU, held until the process
 * ends.  The call allocates and frees nothing.  b * (a/t) * s * 4 bytes (rounded up to 256) beyond that size return
 * SAR_ERR_UNSUPPORTED (530B shard: 131 072 bytes).  Every call on a GPU uses that GPU's one buffer: calls that overlap in
 * time on one GPU (different streams, or different threads) race; calls on one stream are ordered and safe.  The buffer's
 * earlier contents do not matter (every byte read is written first by the same call).
 */
size_t attn_core_bwd_noalloc_max_bytes(void);
sar_status attn_core_bwd_recompute_noalloc(const sar_attn_desc* desc, const void* q, const void* k, const void* v,
                                           const void* o, const float* lse, const void* d_o,
                                           void* dq, void* dk, void* dv, void* stream);

/*
 * The three launches of the recompute-once backward as separate calls (for timing each of them): `stages` is a subset of
 *   1  delta_i = sum_k dO_ik O_ik into the workspace          (needs o, d_o)
 *   2  dk, dv and the dS tiles into the workspace             (needs q, k, v, lse, d_o; reads delta)
 *   4  dq from the dS tiles                                   (needs k; reads the tiles)
 * run in this order on one stream with the same workspace (at least attn_core_bwd_workspace bytes of the once-form; see
 * above) they equal attn_core_bwd_recompute.  Pointers that the chosen stages do not need may be NULL.
 */
sar_status attn_core_bwd_recompute_stages(const sar_attn_desc* desc, int stages, const void* q, const void* k, const void* v,
                                          const void* o, const float* lse, const void* d_o, void* dq, void* dk, void* dv,
                                          void* workspace, size_t workspace_bytes, void* stream);

/*
 * The two passes of the recompute-twice backward as separate calls (same kernels, same arguments): the row
 * pass recomputes the region per query block and writes dq and the per-row term sum_k dO_ik O_ik into the
 * workspace; the column pass recomputes it per key block, reads that term back and writes dk, dv.
 * Row pass then column pass on one stream, with the same workspace, equals attn_core_bwd_recompute.
 */
sar_status attn_core_bwd_recompute_dq(const sar_attn_desc* desc, const void* q, const void* k, const void* v,
                                      const void* o, const float* lse, const void* d_o, void* dq,
                                      void* workspace, size_t workspace_bytes, void* stream);
sar_status attn_core_bwd_recompute_dkdv(const sar_attn_desc* desc, const void* q, const void* k, const void* v,
                                        const float* lse, const void* d_o, void* dk, void* dv,
                                        void* workspace, size_t workspace_bytes, void* stream);

/*
 * Stored-activation baseline (what Section 4.1 itemises and Section 5 avoids): the forward also
 * writes the softmax output P, the dropout mask M and the dropout output D, and the backward reads
 * them back instead of recomputing.  Used for the recompute-vs-stored timing ratio and to expose the
 * mask bit for bit.
 *   P, D : desc->dtype [b, A, s, s];  M : uint8 [b, A, s, s]; entries with j > i are written as 0.
 *   lse  : out, float [b, A, s], as attn_core_fwd;  o : the forward's output (in, for the backward's
 *          per-row term delta_i = dO_i . O_i; the plain-kernel path rebuilds that term from P and ignores o).
 * Exactly (2*elem + 1) * A * s^2 * b extra bytes = the paper's 5 a s^2 b / t for 16-bit elements.
 * bf16 with head dimension 64 / 96 / 128 / 160 and s % 64 == 0 runs on the matrix cores with the tiles of
 * the recompute kernels (the forward computes the scores twice: once for O and the row statistics, once
 * to write the normalised P); everything else on the plain kernels.
 * attn_core_bwd_stored takes the same workspace as attn_core_bwd_recompute (per-row softmax term).
 */
sar_status attn_core_fwd_stored(const sar_attn_desc* desc, const void* q, const void* k, const void* v,
                                void* o, float* lse, void* P, uint8_t* M, void* D, void* stream);
sar_status attn_core_bwd_stored(const sar_attn_desc* desc, const void* q, const void* k, const void* v, const void* o,
                                const void* P, const uint8_t* M, const void* D, const void* d_o,
                                void* dq, void* dk, void* dv,
                                void* workspace, size_t workspace_bytes, void* stream);

/* Bytes held from forward to backward by the attention core on this rank: Q, K, V, O and, when
 * selective == 0, the three s x s tensors (Section 4.1; Table 2 rows with / without selective
 * recomputation).  The fp32 log-sum-exp and the 16 bytes of (seed, offset) are "small buffers" in the
 * paper's sense and are reported by attn_core_small_buffer_bytes.  0 on an invalid descriptor. */
uint64_t attn_core_saved_bytes(const sar_attn_desc* desc, int selective);
uint64_t attn_core_small_buffer_bytes(const sar_attn_desc* desc);

/* Number of Philox calls one attention call may consume (b*a*s*s/8, the global score tensor, so
 * ranks need not coordinate); advance `offset` by at least this between calls. */
uint64_t attn_core_philox_count(const sar_attn_desc* desc);

/* Rows descriptor for the sequence-parallel region: rows = (s/t)*b local rows of width h. */
typedef struct {
  int64_t rows, h;
  int64_t row_offset;      /* global index of local row 0 = rank*(s/t)*b (feeds Philox only)  */
  int32_t dtype;           /* sar_dtype of x, y, dy, dx, resid, out, gamma, beta, bias         */
  float eps;               /* LayerNorm epsilon (1e-5)                                         */
  float p;                 /* dropout probability of bias_dropout_add, 0 <= p < 1              */
  uint64_t seed, offset;   /* Philox key and counter base of bias_dropout_add                  */
} sar_rows_desc;

/*
 * ln_fwd -- LayerNorm of Eq. 3's first line on this rank's rows: per row mu, biased variance,
 * rstd = 1/sqrt(var + eps), y = (x - mu) rstd gamma + beta.
 *   x [rows, h], gamma [h], beta [h] : in, desc->dtype;  y [rows, h] : out, desc->dtype
 *   mean [rows], rstd [rows] : out, float (the "small buffers" of Section 4)
 */
sar_status ln_fwd(const sar_rows_desc* desc, const void* x, const void* gamma, const void* beta,
                  void* y, float* mean, float* rstd, void* stream);

/* Bytes of scratch ln_bwd needs (per-workgroup partial sums of dgamma / dbeta). */
size_t ln_bwd_workspace(const sar_rows_desc* desc);

/*
 * ln_bwd -- gradient of ln_fwd.  dx in desc->dtype; dgamma, dbeta are float [h], summed over this
 * rank's rows only (the sum over ranks is the caller's all-reduce).
 */
sar_status ln_bwd(const sar_rows_desc* desc, const void* dy, const void* x, const float* mean, const float* rstd,
                  const void* gamma, void* dx, float* dgamma, float* dbeta,
                  void* workspace, size_t workspace_bytes, void* stream);

/*
 * bias_dropout_add -- last line of Eq. 3 plus the residual connection:
 *   out = resid + M o (x + bias) / (1 - p),  M from Philox site 1.
 *   bias [h] may be NULL (the paper's Dropout(W)); mask_out uint8 [rows, h] may be NULL (the paper
 *   stores this mask, sbh bytes; Philox can regenerate it); out may alias resid (in-place residual).
 */
sar_status bias_dropout_add(const sar_rows_desc* desc, const void* x, const void* bias, const void* resid,
                            void* out, uint8_t* mask_out, void* stream);

/*
 * bias_dropout_add_ln_fwd -- the step above fused with the LayerNorm that consumes it (Eq. 3: the last line of
 * one block feeds the first line of the next), one pass over the row instead of two:
 *   out = resid + M o (x + bias) / (1 - p),   y = LayerNorm(out) with gamma, beta, eps.
 *   x, resid [rows, h], bias [h] or NULL, gamma, beta [h] : in;  out, y [rows, h] : out (desc->dtype);
 *   mean, rstd [rows] : out, float, the statistics of `out` as stored (so ln_bwd on the stored row matches).
 *   out may alias resid; y may alias nothing.  Same Philox stream as bias_dropout_add (site 1).
 */
sar_status bias_dropout_add_ln_fwd(const sar_rows_desc* desc, const void* x, const void* bias, const void* resid,
                                   const void* gamma, const void* beta, void* out, void* y, float* mean, float* rstd,
                                   void* stream);

/* Bytes of scratch bias_dropout_add_bwd needs when dbias is requested (row-split partial sums; may be 0). */
size_t bias_dropout_add_bwd_workspace(const sar_rows_desc* desc);

/*
 * bias_dropout_add_bwd -- gradient of bias_dropout_add (Eq. 3, last line): the mask is regenerated from
 * (seed, offset), nothing of the forward is needed.
 *   dout [rows, h] : in;  dx = M o dout / (1 - p) [rows, h] : out (desc->dtype; may alias dout)
 *   dbias [h] : out, float, column sums of dx over this rank's rows, or NULL (then no workspace is needed).
 *   The gradient of the residual branch is dout itself and is not written.
 */
sar_status bias_dropout_add_bwd(const sar_rows_desc* desc, const void* dout, void* dx, float* dbias,
                                void* workspace, size_t workspace_bytes, void* stream);

/*
 * bias_gelu_fwd / bias_gelu_bwd -- the non-linearity of the MLP block with its bias (Section 4.1: the GeLU
 * keeps its input, 8sbh bytes without tensor parallelism, for the backward).  The paper names the function
 * only; the exact form is taken: GeLU(z) = z Phi(z), Phi the standard normal CDF.
 *   x [rows, h] (the first linear layer's output on this rank: rows = s*b, h = 4h/t), bias [h] or NULL : in
 *   y = GeLU(x + bias) [rows, h] : out (desc->dtype; may alias x only if the caller keeps x elsewhere)
 *   backward: dy, x, bias as above : in;  dx = dy GeLU'(x + bias) [rows, h] : out (may alias dy);
 *   dbias [h] : out, float, column sums of dx, or NULL (then no workspace is needed).
 * Only rows, h and dtype of the descriptor are used.
 */
sar_status bias_gelu_fwd(const sar_rows_desc* desc, const void* x, const void* bias, void* y, void* stream);
size_t bias_gelu_bwd_workspace(const sar_rows_desc* desc);
sar_status bias_gelu_bwd(const sar_rows_desc* desc, const void* dy, const void* x, const void* bias, void* dx, float* dbias,
                         void* workspace, size_t workspace_bytes, void* stream);

/*
 * Test and measurement hook, not part of the method: forces kernel variants that the library otherwise picks by shape
 * (every variant computes the same result).  Each argument: -1 = the library's choice, 0 = off, 1 = on.
 *   fwd_128_rows      forward with 128 instead of 64 query rows per workgroup (needs s >= 128)
 *   fwd_loader_waves  forward (64-row workgroups) with four extra waves that only fetch K / V tiles (1), or as producer /
 *                     consumer wave pairs (2: one wave computes scores and softmax, the other accumulates P V and fetches),
 *                     or 3: as 1 with persistent workgroups, each working through a list of row blocks (used only when
 *                     b x heads does not exceed the number of compute units; otherwise 3 behaves as 1)
 *   dq_loader_waves   the same for the row pass of the recompute-twice backward
 *   dkdv_pipelined    form of the column pass where s % 64 == 0: 0 plain; 1 software-pipelined (head dimension 128 and 160
 *                     only: score tiles of the next query tile computed beside this tile's vector arithmetic); 2 producer /
 *                     consumer (two waves per SIMD: one computes scores, softmax, mask and dS, the other accumulates dK, dV),
 *                     one key block per workgroup; 3 the same with persistent workgroups that each take several key blocks
 *                     (only when b x heads does not exceed the number of compute units; otherwise 3 behaves as 2)
 * Process-wide; not meant to be changed while another thread launches.
 */
void sar_test_force_variants(int fwd_128_rows, int fwd_loader_waves, int dq_loader_waves, int dkdv_pipelined);

/*
 * Measurement hooks, not part of the method: the rates this GPU attains on the two rooflines that bound the kernels above.
 *   sar_bench_mfma  enqueues a register-resident loop of `iters` x 4 independent 32x32x16 bf16 matrix instructions per wave,
 *                   8 waves on every CU; *flops_out (host) receives the floating-point operations the launch performs;
 *                   sink: device, at least 4 bytes, never written in practice.
 *   sar_bench_copy  enqueues a plain copy of `bytes` (a multiple of 16, 16-byte aligned device pointers) from src to dst:
 *                   `bytes` read and `bytes` written.
 * The caller times them (events on `stream`).  They set no sar_last_error text.
 */
sar_status sar_bench_mfma(int iters, float* sink, double* flops_out, void* stream);
sar_status sar_bench_copy(const void* src, void* dst, size_t bytes, void* stream);
/*
 *   sar_bench_issue  enqueues probe number `probe` (0 .. until sar_bench_issue_name returns NULL) on `workgroups` workgroups:
 *                    waves 0..3 of a workgroup (one per SIMD) run `iters` iterations of one unrolled instruction sequence, and in
 *                    the two-wave probes waves 4..7 run a second one beside them.  cycles: device, workgroups x 8 values, written
 *                    at [workgroup * 8 + wave] with the wave's s_memtime cycles for all its iterations; insts_a / insts_b
 *                    (host, out): instructions per iteration of the two sequences (0 if there is no second).  sink: device, one
 *                    float, never written.  Cycles per instruction = cycles / (iters x insts).
 */
const char* sar_bench_issue_name(int probe);
sar_status sar_bench_issue(int probe, int iters, unsigned long long* cycles, int workgroups, float* sink, int* insts_a, int* insts_b, void* stream);

/* Thread-local text describing the last non-OK status returned on this thread ("" if none). */
const char* sar_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* SAR_H_ */
