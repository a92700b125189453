/*
 * CPU oracle for the BlockFFN layer: TEST INFRASTRUCTURE, not a product path.
 *
 * Only the tests, the smoke check and the benchmark's cpu_baseline leg may call this
 * file.  It shares no code with the HIP library and includes none of its headers.
 *
 * What it computes is the plain definition, written as loops, in fp64:
 *
 *   Eq. 1   FFN(x)   = sum_{i=1..N_e} A_i(x) * E_i(x)
 *   Eq. 2   E_i(x)   = W_down^(i)T Swish(W_up^(i)T x)                  (non-gated expert)
 *   Table 1 E_i(x)   = W_down^(i)T [ Swish(W_gate^(i)T x) . W_up^(i)T x ]   (gated variant,
 *                      the DeepSeek-V3 row; Swish with beta = 1 is SiLU)
 *   Eq. 3   A^0 = W_router^T x (+ b),  A^1 = ReLU(A^0),  A = RMSNorm(A^1)
 *   Sec. 2.1  TLS / CLS_L: share of experts with zero activation for a token / for every
 *             token of a chunk of L consecutive tokens
 *   Sec. 3.3  Union(x): index union of the experts activated by the n tokens of a chunk;
 *             only those experts are evaluated, and per token only the ones that token
 *             activates contribute.
 *
 * The chunk-sparse path reaches exactly the value of Eq. 1: it only leaves out terms
 * whose A_i(x) is exactly zero.  So oracle_sparse_ffn and oracle_dense_ffn are the same
 * sum, the first skipping experts outside the union / outside the token's mask, the
 * second visiting every expert.
 *
 * Readings where the paper is silent (kept in step with the design notes):
 *   - RMSNorm is the textbook one: mean of squares over all N_e entries (zeros
 *     included), eps inside the square root, element-wise gain g.  An all-zero row
 *     stays all-zero for any eps >= 0.
 *   - "activated" means A^0 > 0 strictly (the ReLU's exact zero), decided on the value
 *     rounded to fp32, which keeps the sign of the fp64 sum.
 *   - the mask follows A^1: a zero gain g_i gives a zero score but leaves the bit set.
 *   - the union list is in ascending expert index; unused tail entries are -1.
 *   - chunks are the disjoint windows [c*k, (c+1)*k).
 *
 * Storage: every matrix is stored one row per OUTPUT feature, i.e. as the transposes
 * that appear in Eq. 2-3: w_router [E][d], w_up / w_gate [E][d_e][d], w_down [E][d][d_e].
 * wdtype 0 = fp32, 1 = bf16 bit patterns (uint16), widened exactly.
 *
 * Parity pins (tests/test_oracle_pins.py): hand-worked router values, the RMSNorm
 * sum-of-squares identity, scale invariance, set-based brute force of masks / unions /
 * counts, one-hot-weight closed forms, the single-expert case against a two-matmul MLP,
 * the W_gate = W_up identity tying the gated to the non-gated expert, sparse == dense.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

typedef struct {
  int32_t d, n_experts, d_e;
  int32_t wdtype;       /* 0 fp32, 1 bf16 */
  int32_t gated;        /* 0: Eq. 2, 1: gated variant */
  int32_t pad_;
  double eps;           /* RMSNorm epsilon */
  const void *w_router; /* [E][d] */
  const float *b_router;/* [E] or NULL */
  const float *g_rms;   /* [E] or NULL (all ones) */
  const void *w_up;     /* [E][d_e][d] */
  const void *w_gate;   /* [E][d_e][d], NULL unless gated */
  const void *w_down;   /* [E][d][d_e] */
} oracle_layer;

static double widen(const void *w, int wdtype, size_t idx) {
  if (wdtype == 0) return (double)((const float *)w)[idx];
  uint32_t bits = (uint32_t)((const uint16_t *)w)[idx] << 16;
  float f;
  memcpy(&f, &bits, sizeof f);
  return (double)f;
}

static double swish(double u) { return u / (1.0 + exp(-u)); }

/* Eq. 3 for n_tok tokens.  a0_out (optional) receives the fp64 pre-activations. */
int oracle_router(const oracle_layer *L, const float *x, int64_t n_tok, float *scores,
                  uint64_t *token_mask, double *a0_out) {
  const int d = L->d, E = L->n_experts, W = (E + 63) / 64;
#pragma omp parallel for schedule(static)
  for (int64_t t = 0; t < n_tok; ++t) {
    double a1[1024];
    double sumsq = 0.0;
    for (int w = 0; w < W; ++w) token_mask[t * W + w] = 0;
    for (int i = 0; i < E; ++i) {
      double a0 = L->b_router ? (double)L->b_router[i] : 0.0;
      for (int j = 0; j < d; ++j)
        a0 += (double)x[t * d + j] * widen(L->w_router, L->wdtype, (size_t)i * d + j);
      if (a0_out) a0_out[t * E + i] = a0;
      int active = (float)a0 > 0.0f;
      a1[i] = active ? a0 : 0.0;
      sumsq += a1[i] * a1[i];
      if (active) token_mask[t * W + i / 64] |= (uint64_t)1 << (i % 64);
    }
    double rms = sqrt(sumsq / (double)E + L->eps);
    for (int i = 0; i < E; ++i) {
      double g = L->g_rms ? (double)L->g_rms[i] : 1.0;
      scores[t * E + i] = a1[i] > 0.0 ? (float)(g * a1[i] / rms) : 0.0f;
    }
  }
  return 0;
}

/* Union(x) per chunk, its ascending index list, and the TLS / CLS inactive counts
 * (stats[0] += inactive (token, expert) pairs, stats[1] += inactive (chunk, expert) pairs). */
int oracle_chunk_union(const uint64_t *token_mask, int64_t n_chunks, int32_t k, int32_t E,
                       uint64_t *union_mask, int32_t *active_idx, int32_t *n_active,
                       int64_t *stats) {
  const int W = (E + 63) / 64;
  int64_t tls_inactive = 0, cls_inactive = 0;
  for (int64_t c = 0; c < n_chunks; ++c) {
    for (int w = 0; w < W; ++w) union_mask[c * W + w] = 0;
    for (int t = 0; t < k; ++t)
      for (int i = 0; i < E; ++i) {
        int bit = (int)((token_mask[(c * k + t) * W + i / 64] >> (i % 64)) & 1);
        if (bit) union_mask[c * W + i / 64] |= (uint64_t)1 << (i % 64);
        else tls_inactive += 1;
      }
    int n = 0;
    for (int i = 0; i < E; ++i)
      if ((union_mask[c * W + i / 64] >> (i % 64)) & 1) active_idx[c * E + n++] = i;
    n_active[c] = n;
    cls_inactive += E - n;
    for (int s = n; s < E; ++s) active_idx[c * E + s] = -1;
  }
  if (stats) {
    stats[0] += tls_inactive;
    stats[1] += cls_inactive;
  }
  return 0;
}

/* y[0..d) += a * E_i(x_t)   (Eq. 2, or the gated variant) */
static void add_expert(const oracle_layer *L, const float *xt, int i, double a, double *y,
                       double *h /* scratch [d_e] */) {
  const int d = L->d, de = L->d_e;
  for (int j = 0; j < de; ++j) {
    size_t row = ((size_t)i * de + j) * d;
    double u = 0.0;
    for (int c = 0; c < d; ++c) u += (double)xt[c] * widen(L->w_up, L->wdtype, row + c);
    if (L->gated) {
      double g = 0.0;
      for (int c = 0; c < d; ++c) g += (double)xt[c] * widen(L->w_gate, L->wdtype, row + c);
      h[j] = swish(g) * u;
    } else {
      h[j] = swish(u);
    }
  }
  for (int c = 0; c < d; ++c) {
    size_t row = ((size_t)i * d + c) * de;
    double e = 0.0;
    for (int j = 0; j < de; ++j) e += h[j] * widen(L->w_down, L->wdtype, row + j);
    y[c] += a * e;
  }
}

/* Sec. 3.3: per chunk only the experts in the union list are visited; per token only the
 * ones in that token's mask contribute (a masked term contributes nothing). */
int oracle_sparse_ffn(const oracle_layer *L, const float *x, const float *scores,
                      const uint64_t *token_mask, const int32_t *active_idx,
                      const int32_t *n_active, int64_t n_chunks, int32_t k, double *y) {
  const int d = L->d, E = L->n_experts, W = (E + 63) / 64;
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t c = 0; c < n_chunks; ++c) {
    double h[4096];
    for (int t = 0; t < k; ++t) {
      int64_t tok = c * k + t;
      double *yt = y + tok * d;
      for (int j = 0; j < d; ++j) yt[j] = 0.0;
      for (int s = 0; s < n_active[c]; ++s) {
        int i = active_idx[c * E + s];
        if (!((token_mask[tok * W + i / 64] >> (i % 64)) & 1)) continue;
        add_expert(L, x + tok * d, i, (double)scores[tok * E + i], yt, h);
      }
    }
  }
  return 0;
}

/* Eq. 1 with every expert evaluated (no skipping at all). */
int oracle_dense_ffn(const oracle_layer *L, const float *x, const float *scores, int64_t n_tok,
                     double *y) {
  const int d = L->d, E = L->n_experts;
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t t = 0; t < n_tok; ++t) {
    double h[4096];
    double *yt = y + t * d;
    for (int j = 0; j < d; ++j) yt[j] = 0.0;
    for (int i = 0; i < E; ++i)
      add_expert(L, x + t * d, i, (double)scores[t * E + i], yt, h);
  }
  return 0;
}

int oracle_max_experts(void) { return 1024; }
int oracle_max_d_e(void) { return 4096; }
