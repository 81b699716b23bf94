/*
 * fp64 CPU oracle for the selective-activation-recomputation hot path of
 * "Reducing Activation Recomputation in Large Transformer Models" (arXiv 2205.05198).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the GPU library is
 * checked against.  It shares no code, header, table or helper with the HIP path and nothing
 * in the product path may call it.
 *
 * What is written out here, straight from the definitions (no tiling, no online softmax, no
 * fusion; every s x s intermediate is materialised on purpose, because the stored-activation
 * computation is exactly what selective recomputation must reproduce, Section 5):
 *
 *   attention core (Section 4.1, the four operations inside the recomputed region of
 *   Section 5):  S = alpha Q K^T, causal fill, row softmax P, Bernoulli mask M from a
 *   counter-based Philox4x32-10 stream, D = P*M/(1-p), O = D V; and the chain rule through
 *   those steps for dQ, dK, dV.
 *   LayerNorm and dropout(+bias)+residual of the sequence-parallel region (Section 4.2.2,
 *   Eq. 3): per-row statistics, y = xhat*gamma+beta; out = resid + M*(x+bias)/(1-p).
 *
 * The paper does not define the scale, the mask fill, the RNG or the LayerNorm epsilon; the
 * readings used are listed next to each function.  Pins for every function live in
 * tests/test_oracle_*.py (finite differences, library special cases, closed forms, published
 * Philox known-answer vectors).  The index->bit mapping of the dropout mask is this build's own
 * definition and has no external pin: "parity unpinned" for that mapping alone (it is pinned
 * only by an independent big-integer re-implementation and statistical invariants).
 *
 * Tensor layout: the paper's s x b x h activations (Section 3) seen per GPU as [s, b, A, d]
 * with A = a/t local heads and d = h/a, addressed through element strides.
 * All values are double; callers pass inputs already rounded to the device dtype.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
  int32_t s, b;          /* sequence length, microbatch (Table 1)                         */
  int32_t a, t, rank;    /* global heads, tensor-parallel size, this shard's rank         */
  int32_t h;             /* hidden size; d = h / a                                        */
  int32_t causal;        /* 1: S_ij = -inf for j > i                                      */
  float scale;           /* alpha, as the float the device receives                       */
  float p;               /* dropout probability, as the float the device receives         */
  uint64_t seed, offset; /* Philox key and counter base                                   */
  int64_t stride_s, stride_b, stride_a; /* element strides of [s, b, A, d]; d contiguous   */
} orc_attn_desc;

int orc_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* ---------------------------------------------------------------------------------------
 * Philox4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw, SC'11).  One round multiplies
 * counter words 0 and 2 by two fixed constants, and mixes the high halves with the other
 * two words and the key; the key is bumped by the Weyl constants between rounds.
 * ------------------------------------------------------------------------------------- */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; ++round) {
    uint64_t prod0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
    uint64_t prod1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
    uint32_t hi0 = (uint32_t)(prod0 >> 32), lo0 = (uint32_t)prod0;
    uint32_t hi1 = (uint32_t)(prod1 >> 32), lo1 = (uint32_t)prod1;
    uint32_t n0 = hi1 ^ c1 ^ k0;
    uint32_t n1 = lo1;
    uint32_t n2 = hi0 ^ c3 ^ k1;
    uint32_t n3 = lo0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Dropout threshold on 16 random bits: T = floor(p*65536 + 0.5), p taken as the float it is. */
uint32_t orc_dropout_threshold(float p) { return (uint32_t)floor((double)p * 65536.0 + 0.5); }

/*
 * Keep-bit of element e of dropout site `site` (0 = softmax dropout, 1 = bias-dropout-add).
 * Eight consecutive elements share one Philox call: call index G = offset + (e >> 3) is the
 * 64-bit counter (low word, high word, 0, site); the key is the seed; element e takes the
 * 16-bit field number (e & 7) of the 128 output bits, low half of word (e&7)>>1 first.
 * Kept iff field >= T.  (The paper only says that a dropout mask exists, one byte per
 * element, Section 4; generator, bit budget and tie rule are this build's reading.)
 */
uint8_t orc_keep_bit(uint64_t seed, uint64_t offset, uint64_t e, uint32_t site, uint32_t T) {
  uint64_t G = offset + (e >> 3);
  uint32_t ctr[4] = {(uint32_t)(G & 0xFFFFFFFFu), (uint32_t)(G >> 32), 0u, site};
  uint32_t key[2] = {(uint32_t)(seed & 0xFFFFFFFFu), (uint32_t)(seed >> 32)};
  uint32_t out[4];
  orc_philox4x32_10(ctr, key, out);
  uint32_t r = (uint32_t)(e & 7u);
  uint32_t u = (out[r >> 1] >> (16u * (r & 1u))) & 0xFFFFu;
  return (uint8_t)(u >= T);
}

/* Element index of score (beta, n_global, i, j) in the global [b, a, s, s] score tensor. */
static uint64_t score_index(const orc_attn_desc* c, int beta, int n_global, int i, int j) {
  return (((uint64_t)beta * (uint64_t)c->a + (uint64_t)n_global) * (uint64_t)c->s + (uint64_t)i) * (uint64_t)c->s + (uint64_t)j;
}

/* Raw softmax-dropout mask for this shard, M[b][A][s][s], every (i, j) including j > i. */
void orc_attn_mask(const orc_attn_desc* c, uint8_t* M) {
  const int A = c->a / c->t;
  const uint32_t T = orc_dropout_threshold(c->p);
  for (int beta = 0; beta < c->b; ++beta)
    for (int n = 0; n < A; ++n)
      for (int i = 0; i < c->s; ++i)
        for (int j = 0; j < c->s; ++j)
          M[(((size_t)beta * A + n) * c->s + i) * c->s + j] =
              orc_keep_bit(c->seed, c->offset, score_index(c, beta, c->rank * A + n, i, j), 0u, T);
}

/* How many Philox calls one attention call may consume: the whole global score tensor / 8. */
uint64_t orc_attn_philox_count(const orc_attn_desc* c) {
  return (uint64_t)c->b * (uint64_t)c->a * (uint64_t)c->s * (uint64_t)c->s / 8u;
}

/* ---------------------------------------------------------------------------------------
 * Attention core, forward (Section 4.1 items QK^T, softmax, softmax dropout, attention over
 * V), for the flattened (batch, local head) indices [head_lo, head_hi).
 *   1. S_ij = alpha * sum_k Q_ik K_jk           (alpha: reading, the paper is silent)
 *   2. S_ij = -inf for j > i when causal         (reading: GPT-style decoder)
 *   3. m_i = max_j S_ij, l_i = sum_j exp(S_ij - m_i), P_ij = exp(S_ij - m_i) / l_i,
 *      LSE_i = m_i + ln l_i
 *   4. D_ij = P_ij * M_ij / (1 - p)              (inverted dropout on the normalised P)
 *   5. O_ik = sum_j D_ij V_jk
 * Optional outputs (may be NULL): P, D as double [head_hi - head_lo][s][s], M as bytes (0 above the
 * diagonal when causal) -- the tensors the non-selective path would have to store.
 * ------------------------------------------------------------------------------------- */
int orc_attn_fwd(const orc_attn_desc* c, const double* q, const double* k, const double* v,
                 double* o, double* lse, double* Pout, uint8_t* Mout, double* Dout,
                 int head_lo, int head_hi) {
  const int s = c->s, A = c->a / c->t, d = c->h / c->a;
  const double alpha = (double)c->scale;
  const double keep_scale = 1.0 / (1.0 - (double)c->p);
  const uint32_t T = orc_dropout_threshold(c->p);
  int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
  for (int bn = head_lo; bn < head_hi; ++bn) {
    const int beta = bn / A, n = bn % A;
    const int64_t base = (int64_t)beta * c->stride_b + (int64_t)n * c->stride_a;
    double* S = (double*)malloc((size_t)s * s * sizeof(double));
    double* P = (double*)malloc((size_t)s * s * sizeof(double));
    double* D = (double*)malloc((size_t)s * s * sizeof(double));
    uint8_t* M = (uint8_t*)malloc((size_t)s * s);
    if (!S || !P || !D || !M) { failed = 1; free(S); free(P); free(D); free(M); continue; }
    for (int i = 0; i < s; ++i) {
      const double* qi = q + base + (int64_t)i * c->stride_s;
      /* steps 1-2 */
      for (int j = 0; j < s; ++j) {
        if (c->causal && j > i) { S[(size_t)i * s + j] = -INFINITY; continue; }
        const double* kj = k + base + (int64_t)j * c->stride_s;
        double acc = 0.0;
        for (int x = 0; x < d; ++x) acc += qi[x] * kj[x];
        S[(size_t)i * s + j] = alpha * acc;
      }
      /* step 3 */
      double m = -INFINITY;
      for (int j = 0; j < s; ++j) if (S[(size_t)i * s + j] > m) m = S[(size_t)i * s + j];
      double l = 0.0;
      for (int j = 0; j < s; ++j) l += exp(S[(size_t)i * s + j] - m);
      for (int j = 0; j < s; ++j) P[(size_t)i * s + j] = exp(S[(size_t)i * s + j] - m) / l;
      lse[(size_t)bn * s + i] = m + log(l);
      /* step 4 */
      for (int j = 0; j < s; ++j) {
        uint8_t keep = 0;
        if (!(c->causal && j > i)) keep = orc_keep_bit(c->seed, c->offset, score_index(c, beta, c->rank * A + n, i, j), 0u, T);
        M[(size_t)i * s + j] = keep;
        D[(size_t)i * s + j] = P[(size_t)i * s + j] * (double)keep * keep_scale;
      }
      /* step 5 */
      double* oi = o + base + (int64_t)i * c->stride_s;
      for (int x = 0; x < d; ++x) oi[x] = 0.0;
      for (int j = 0; j < s; ++j) {
        const double* vj = v + base + (int64_t)j * c->stride_s;
        for (int x = 0; x < d; ++x) oi[x] += D[(size_t)i * s + j] * vj[x];
      }
    }
    if (Pout) memcpy(Pout + (size_t)(bn - head_lo) * s * s, P, (size_t)s * s * sizeof(double));
    if (Dout) memcpy(Dout + (size_t)(bn - head_lo) * s * s, D, (size_t)s * s * sizeof(double));
    if (Mout) memcpy(Mout + (size_t)(bn - head_lo) * s * s, M, (size_t)s * s);
    free(S); free(P); free(D); free(M);
  }
  return failed ? -1 : 0;
}

/* ---------------------------------------------------------------------------------------
 * Attention core, backward: the chain rule through steps 1-5 above, given dO.  Everything is
 * recomputed from Q, K, V by the definition (the oracle takes neither O nor LSE).
 *   dD_ij = sum_k dO_ik V_jk        dP_ij = dD_ij * M_ij / (1-p)
 *   delta_i = sum_j P_ij dP_ij      dS_ij = P_ij (dP_ij - delta_i)
 *   dV_jk = sum_i D_ij dO_ik        dQ_ik = alpha sum_j dS_ij K_jk     dK_jk = alpha sum_i dS_ij Q_ik
 * Optional outputs: delta [b][A][s], dS [head_hi - head_lo][s][s] (for the invariant tests).
 * ------------------------------------------------------------------------------------- */
int orc_attn_bwd(const orc_attn_desc* c, const double* q, const double* k, const double* v, const double* dO,
                 double* dq, double* dk, double* dv, double* delta_out, double* dS_out,
                 int head_lo, int head_hi) {
  const int s = c->s, A = c->a / c->t, d = c->h / c->a;
  const double alpha = (double)c->scale;
  const double keep_scale = 1.0 / (1.0 - (double)c->p);
  const uint32_t T = orc_dropout_threshold(c->p);
  int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
  for (int bn = head_lo; bn < head_hi; ++bn) {
    const int beta = bn / A, n = bn % A;
    const int64_t base = (int64_t)beta * c->stride_b + (int64_t)n * c->stride_a;
    double* P = (double*)malloc((size_t)s * s * sizeof(double));
    double* dS = (double*)malloc((size_t)s * s * sizeof(double));
    double* Mk = (double*)malloc((size_t)s * s * sizeof(double)); /* M_ij / (1-p) */
    double* row = (double*)malloc((size_t)s * sizeof(double));
    if (!P || !dS || !Mk || !row) { failed = 1; free(P); free(dS); free(Mk); free(row); continue; }
    /* recompute P and M exactly as the forward defines them */
    for (int i = 0; i < s; ++i) {
      const double* qi = q + base + (int64_t)i * c->stride_s;
      double m = -INFINITY;
      for (int j = 0; j < s; ++j) {
        if (c->causal && j > i) { row[j] = -INFINITY; continue; }
        const double* kj = k + base + (int64_t)j * c->stride_s;
        double acc = 0.0;
        for (int x = 0; x < d; ++x) acc += qi[x] * kj[x];
        row[j] = alpha * acc;
        if (row[j] > m) m = row[j];
      }
      double l = 0.0;
      for (int j = 0; j < s; ++j) l += exp(row[j] - m);
      for (int j = 0; j < s; ++j) {
        P[(size_t)i * s + j] = exp(row[j] - m) / l;
        uint8_t keep = 0;
        if (!(c->causal && j > i)) keep = orc_keep_bit(c->seed, c->offset, score_index(c, beta, c->rank * A + n, i, j), 0u, T);
        Mk[(size_t)i * s + j] = (double)keep * keep_scale;
      }
    }
    /* dS */
    for (int i = 0; i < s; ++i) {
      const double* doi = dO + base + (int64_t)i * c->stride_s;
      double delta = 0.0;
      for (int j = 0; j < s; ++j) {
        const double* vj = v + base + (int64_t)j * c->stride_s;
        double dD = 0.0;
        for (int x = 0; x < d; ++x) dD += doi[x] * vj[x];
        row[j] = dD * Mk[(size_t)i * s + j]; /* dP_ij */
        delta += P[(size_t)i * s + j] * row[j];
      }
      for (int j = 0; j < s; ++j) dS[(size_t)i * s + j] = P[(size_t)i * s + j] * (row[j] - delta);
      if (delta_out) delta_out[(size_t)bn * s + i] = delta;
    }
    /* dQ */
    for (int i = 0; i < s; ++i) {
      double* dqi = dq + base + (int64_t)i * c->stride_s;
      for (int x = 0; x < d; ++x) dqi[x] = 0.0;
      for (int j = 0; j < s; ++j) {
        const double* kj = k + base + (int64_t)j * c->stride_s;
        for (int x = 0; x < d; ++x) dqi[x] += dS[(size_t)i * s + j] * kj[x];
      }
      for (int x = 0; x < d; ++x) dqi[x] *= alpha;
    }
    /* dK, dV */
    for (int j = 0; j < s; ++j) {
      double* dkj = dk + base + (int64_t)j * c->stride_s;
      double* dvj = dv + base + (int64_t)j * c->stride_s;
      for (int x = 0; x < d; ++x) { dkj[x] = 0.0; dvj[x] = 0.0; }
      for (int i = 0; i < s; ++i) {
        const double* qi = q + base + (int64_t)i * c->stride_s;
        const double* doi = dO + base + (int64_t)i * c->stride_s;
        const double dS_ij = dS[(size_t)i * s + j];
        const double D_ij = P[(size_t)i * s + j] * Mk[(size_t)i * s + j];
        for (int x = 0; x < d; ++x) { dkj[x] += dS_ij * qi[x]; dvj[x] += D_ij * doi[x]; }
      }
      for (int x = 0; x < d; ++x) dkj[x] *= alpha;
    }
    if (dS_out) memcpy(dS_out + (size_t)(bn - head_lo) * s * s, dS, (size_t)s * s * sizeof(double));
    free(P); free(dS); free(Mk); free(row);
  }
  return failed ? -1 : 0;
}

/* ---------------------------------------------------------------------------------------
 * LayerNorm over the last dimension of x[rows][h] (Section 4.1 "Layer norm": its input, mean
 * and variance are what the backward needs).  Reading: biased variance, eps inside the root.
 *   mu_r = mean_c x_rc, var_r = mean_c (x_rc - mu_r)^2, rstd_r = 1/sqrt(var_r + eps),
 *   xhat = (x - mu) rstd, y = xhat*gamma + beta.
 * ------------------------------------------------------------------------------------- */
void orc_ln_fwd(int64_t rows, int64_t h, double eps, const double* x, const double* gamma, const double* beta,
                double* y, double* mean, double* rstd) {
#pragma omp parallel for
  for (int64_t r = 0; r < rows; ++r) {
    const double* xr = x + r * h;
    double mu = 0.0;
    for (int64_t c = 0; c < h; ++c) mu += xr[c];
    mu /= (double)h;
    double var = 0.0;
    for (int64_t c = 0; c < h; ++c) var += (xr[c] - mu) * (xr[c] - mu);
    var /= (double)h;
    double rs = 1.0 / sqrt(var + eps);
    for (int64_t c = 0; c < h; ++c) y[r * h + c] = (xr[c] - mu) * rs * gamma[c] + beta[c];
    mean[r] = mu;
    rstd[r] = rs;
  }
}

/*
 * LayerNorm backward, from the definition above:  g = dy*gamma,
 *   dx_rc = rstd_r (g_rc - mean_c g_r - xhat_rc mean_c(g_r xhat_r)),
 *   dgamma_c = sum_r dy_rc xhat_rc,  dbeta_c = sum_r dy_rc.
 * Statistics are recomputed from x.
 */
void orc_ln_bwd(int64_t rows, int64_t h, double eps, const double* dy, const double* x, const double* gamma,
                double* dx, double* dgamma, double* dbeta) {
  for (int64_t c = 0; c < h; ++c) { dgamma[c] = 0.0; dbeta[c] = 0.0; }
  double* xhat = (double*)malloc((size_t)h * sizeof(double));
  for (int64_t r = 0; r < rows; ++r) {
    const double* xr = x + r * h;
    const double* dyr = dy + r * h;
    double mu = 0.0;
    for (int64_t c = 0; c < h; ++c) mu += xr[c];
    mu /= (double)h;
    double var = 0.0;
    for (int64_t c = 0; c < h; ++c) var += (xr[c] - mu) * (xr[c] - mu);
    var /= (double)h;
    double rs = 1.0 / sqrt(var + eps);
    double mg = 0.0, mgx = 0.0;
    for (int64_t c = 0; c < h; ++c) {
      xhat[c] = (xr[c] - mu) * rs;
      double g = dyr[c] * gamma[c];
      mg += g;
      mgx += g * xhat[c];
    }
    mg /= (double)h;
    mgx /= (double)h;
    for (int64_t c = 0; c < h; ++c) {
      double g = dyr[c] * gamma[c];
      dx[r * h + c] = rs * (g - mg - xhat[c] * mgx);
      dgamma[c] += dyr[c] * xhat[c];
      dbeta[c] += dyr[c];
    }
  }
  free(xhat);
}

/* ---------------------------------------------------------------------------------------
 * Dropout (+ optional bias) + residual add on the sequence-parallel shard (last line of
 * Eq. 3, plus the residual connection of the transformer layer):
 *   out_rc = resid_rc + M_rc (x_rc + bias_c) / (1-p),   M from Philox site 1 at element
 *   index (row_offset + r) * h + c, so a shard's mask is the matching slice of the global one.
 * bias may be NULL (the paper's form).  mask (bytes) may be NULL.
 * ------------------------------------------------------------------------------------- */
void orc_bias_dropout_add(int64_t rows, int64_t h, int64_t row_offset, float p, uint64_t seed, uint64_t offset,
                          const double* x, const double* bias, const double* resid, double* out, uint8_t* mask) {
  const uint32_t T = orc_dropout_threshold(p);
  const double keep_scale = 1.0 / (1.0 - (double)p);
#pragma omp parallel for
  for (int64_t r = 0; r < rows; ++r)
    for (int64_t c = 0; c < h; ++c) {
      uint64_t e = (uint64_t)(row_offset + r) * (uint64_t)h + (uint64_t)c;
      uint8_t keep = orc_keep_bit(seed, offset, e, 1u, T);
      double xb = x[r * h + c] + (bias ? bias[c] : 0.0);
      out[r * h + c] = resid[r * h + c] + (double)keep * xb * keep_scale;
      if (mask) mask[r * h + c] = keep;
    }
}

/* Backward of the above: dx = dout*M/(1-p), dresid = dout, dbias_c = sum_r dx_rc. */
void orc_bias_dropout_add_bwd(int64_t rows, int64_t h, int64_t row_offset, float p, uint64_t seed, uint64_t offset,
                              const double* dout, double* dx, double* dresid, double* dbias) {
  const uint32_t T = orc_dropout_threshold(p);
  const double keep_scale = 1.0 / (1.0 - (double)p);
  for (int64_t c = 0; c < h; ++c) dbias[c] = 0.0;
  for (int64_t r = 0; r < rows; ++r)
    for (int64_t c = 0; c < h; ++c) {
      uint64_t e = (uint64_t)(row_offset + r) * (uint64_t)h + (uint64_t)c;
      double keep = (double)orc_keep_bit(seed, offset, e, 1u, T);
      dx[r * h + c] = dout[r * h + c] * keep * keep_scale;
      dresid[r * h + c] = dout[r * h + c];
      dbias[c] += dx[r * h + c];
    }
}

/* ---------------------------------------------------------------------------------------------------
 * Bias + GeLU of the MLP block (Section 4.1: "the GeLU non-linearity also needs its input ... for
 * back-propagation").  The paper names the non-linearity only; the definition taken is the exact one of
 * Hendrycks & Gimpel, GeLU(z) = z Phi(z) with Phi the standard normal CDF, written with erf:
 *   y_rc  = z Phi(z),  z = x_rc + bias_c,  Phi(z) = (1 + erf(z / sqrt 2)) / 2
 *   dx_rc = dy_rc (Phi(z) + z phi(z)),  phi(z) = exp(-z^2 / 2) / sqrt(2 pi);  dbias_c = sum_r dx_rc.
 * bias may be NULL.
 * --------------------------------------------------------------------------------------------------- */
void orc_bias_gelu_fwd(int64_t rows, int64_t h, const double* x, const double* bias, double* y) {
  for (int64_t r = 0; r < rows; ++r)
    for (int64_t c = 0; c < h; ++c) {
      const double z = x[r * h + c] + (bias ? bias[c] : 0.0);
      y[r * h + c] = z * 0.5 * (1.0 + erf(z / sqrt(2.0)));
    }
}

void orc_bias_gelu_bwd(int64_t rows, int64_t h, const double* dy, const double* x, const double* bias, double* dx, double* dbias) {
  const double inv_sqrt_2pi = 1.0 / sqrt(2.0 * 3.14159265358979323846);
  for (int64_t c = 0; c < h; ++c) dbias[c] = 0.0;
  for (int64_t r = 0; r < rows; ++r)
    for (int64_t c = 0; c < h; ++c) {
      const double z = x[r * h + c] + (bias ? bias[c] : 0.0);
      const double Phi = 0.5 * (1.0 + erf(z / sqrt(2.0)));
      const double phi = exp(-0.5 * z * z) * inv_sqrt_2pi;
      dx[r * h + c] = dy[r * h + c] * (Phi + z * phi);
      dbias[c] += dx[r * h + c];
    }
}
