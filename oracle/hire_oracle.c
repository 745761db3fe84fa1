/*
 * HiRE CPU oracle.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, step-by-step CPU
 * statement of what the HiRE decode-step path computes.  It exists so that
 * the GPU library can be checked against something that was written from the
 * paper alone.  It shares no code, header, table or helper with the GPU
 * library and must never be called from the product path: only the tests,
 * the smoke check and the benchmark's cpu_baseline leg may use it.
 *
 * What it follows (arXiv 2402.09360):
 *   - Algorithm 1 (HiRE): S' = TopInd_k'(phi(Zapprox^T x)); then the exact
 *     phi(Z|S'^T x) and its top-k.  The prose under Algorithm 1 applies phi
 *     before the exact top-k; eq. (5) does too; that reading is used.
 *   - HiRE-Q (Sec. 3.2): Zapprox is an int4 copy of Z.  The paper names no
 *     quantiser; the one here is symmetric, one scale per row (amax/7, codes
 *     in [-7,7], round-half-even), activations int8 per token (amax/127).
 *     Parity with the quantiser the authors used is unpinned.
 *   - HiRE-LR (Sec. 3.2): Zapprox = Z1 Z2^T, Z1 [d,r], Z2 [l,r].
 *   - Sec. 3.4.1, dynamic overlap: the per-token candidate sets are unioned
 *     across the batch and the exact stage runs on the union for every token.
 *   - eq. (4): FF_k(x) = sum_{j in S(x)} phi(<u_j,x>) v_j.
 *   - eq. (2): Softmax_k = softmax restricted to and renormalised over the
 *     k largest logits.
 *   - Algorithm 2 (DA-TOP-k): Algorithm 1 run shard by shard with the quotas
 *     k'/s and k/s (rounded up), here with all shards on one device.
 *   - eq. (7), Sec. 3.4.1: CommonPath, a dense set of units next to the
 *     group-sparse ones.
 *   - eq. (6), Sec. 3.4: the group-sparse FFN (groups of g adjacent units
 *     shortlisted and selected by the sum of their absolute activations).
 *   - eq. (1), eq. (3), eq. (4) written out densely as independent pins.
 *
 *   - HiRE-LRQ (Sec. 4.1): both low-rank factors in int4; a reading, see
 *     hire_oracle_scorer_lrq.
 *
 * Scorer arguments of the step functions: kind INT4 uses (q, qscale);
 * LOWRANK uses (z1, z2, r); LRQ uses (q1, s1) for Z1^T [r, d], (q, qscale)
 * for Z2 [N, r], and r.
 *
 * Conventions: every floating-point accumulation is in double.  All matrices
 * are row-major and "unit-major": row j of w1u is u_j, row j of w2u is v_j,
 * row j of the classifier is class j.  bf16 values are uint16 bit patterns.
 * Ties are always broken toward the lower index.  NaN inputs are unsupported.
 *
 * Pins (tests/test_oracle_*.py): brute-force top-k on tiny inputs; k'=N, k=N
 * equals a library fp64 matmul / softmax; k'=N equals eq. (4); output equals
 * the dense FFN under the selected mask; recall = k when the scorer is exact;
 * nested candidate sets; quantiser error bounds; integer scorer equals an
 * int64 library matmul.  Unpinned: the paper's own quantiser (see above) and
 * all of the paper's quality tables (need its weights and data).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define HIRE_ORACLE_SCORER_INT4 0
#define HIRE_ORACLE_SCORER_LOWRANK 1
#define HIRE_ORACLE_SCORER_LRQ 2

static float bf16_to_float(uint16_t h) {
  uint32_t u = (uint32_t)h << 16;
  float f;
  memcpy(&f, &u, sizeof f);
  return f;
}

/* Nearest bf16 (8 significant bits, round-half-even) of a double, returned as
 * the value it denotes.  Done directly on the double: going through float
 * first would round twice. */
static double round_to_bf16_value(double v) {
  if (v == 0.0 || isnan(v) || isinf(v)) return v;
  int e;
  (void)frexp(v, &e); /* |v| in [2^(e-1), 2^e) */
  int ulp_exp = e - 8; /* 8 significant bits */
  if (ulp_exp < -133) ulp_exp = -133; /* bf16 subnormal spacing 2^-133 */
  double q = ldexp(v, -ulp_exp);      /* |q| < 2^8, exact scaling */
  q = rint(q);                        /* default mode: half-to-even */
  return ldexp(q, ulp_exp);
}

static uint16_t double_to_bf16_bits(double v) {
  float f = (float)round_to_bf16_value(v); /* exact: value is a bf16 */
  uint32_t u;
  memcpy(&u, &f, sizeof u);
  return (uint16_t)(u >> 16);
}

/* ---------------------------------------------------------------------- */
/* HiRE-Q preparation: int4 copy of a unit-major matrix, one scale per row. */
void hire_oracle_quantize_rows_int4(const uint16_t* w, int rows, int cols, int8_t* q, float* scale) {
  for (int j = 0; j < rows; ++j) {
    float amax = 0.0f;
    for (int i = 0; i < cols; ++i) {
      float a = fabsf(bf16_to_float(w[(size_t)j * cols + i]));
      if (a > amax) amax = a;
    }
    float s = amax / 7.0f;
    if (amax == 0.0f) s = 1.0f;
    scale[j] = s;
    for (int i = 0; i < cols; ++i) {
      float r = rintf(bf16_to_float(w[(size_t)j * cols + i]) / s);
      if (r > 7.0f) r = 7.0f;
      if (r < -7.0f) r = -7.0f;
      q[(size_t)j * cols + i] = (int8_t)r;
    }
  }
}

/* Per-token int8 activations for the int4 scorer. */
void hire_oracle_quantize_tokens_int8(const uint16_t* x, int B, int d, int8_t* xq, float* sx) {
  for (int b = 0; b < B; ++b) {
    float amax = 0.0f;
    for (int i = 0; i < d; ++i) {
      float a = fabsf(bf16_to_float(x[(size_t)b * d + i]));
      if (a > amax) amax = a;
    }
    float s = amax / 127.0f;
    if (amax == 0.0f) s = 1.0f;
    sx[b] = s;
    for (int i = 0; i < d; ++i) {
      float r = rintf(bf16_to_float(x[(size_t)b * d + i]) / s);
      if (r > 127.0f) r = 127.0f;
      if (r < -127.0f) r = -127.0f;
      xq[(size_t)b * d + i] = (int8_t)r;
    }
  }
}

/* Algorithm 1 line 1, HiRE-Q: integer scores of every row, then one fp32
 * multiply by the row scale, then phi.  The token scale is a positive
 * constant per token and cannot change the ranking; it is left out. */
void hire_oracle_scorer_int4(const int8_t* q, const float* scale, const int8_t* xq, int B, int N, int d,
                             int relu, int32_t* acc_out, float* key_out) {
#pragma omp parallel for schedule(static)
  for (int j = 0; j < N; ++j) {
    for (int b = 0; b < B; ++b) {
      int32_t acc = 0;
      for (int i = 0; i < d; ++i) acc += (int32_t)q[(size_t)j * d + i] * (int32_t)xq[(size_t)b * d + i];
      float key = (float)acc * scale[j];
      if (relu && !(key > 0.0f)) key = 0.0f;
      if (key == 0.0f) key = 0.0f; /* -0 -> +0 */
      if (acc_out) acc_out[(size_t)b * N + j] = acc;
      key_out[(size_t)b * N + j] = key;
    }
  }
}

/* Algorithm 1 line 1, HiRE-LR: t = Z1^T x (an r-vector, stored as a bf16
 * activation), score_j = <Z2[j,:], t>, key = phi(score) kept in double. */
void hire_oracle_scorer_lowrank(const uint16_t* z1, const uint16_t* z2, const uint16_t* x, int B, int N, int d,
                                int r, int relu, uint16_t* t_out, double* key_out) {
  uint16_t* t = (uint16_t*)malloc((size_t)B * r * sizeof(uint16_t));
  for (int b = 0; b < B; ++b) {
    for (int p = 0; p < r; ++p) {
      double s = 0.0;
      for (int i = 0; i < d; ++i)
        s += (double)bf16_to_float(z1[(size_t)i * r + p]) * (double)bf16_to_float(x[(size_t)b * d + i]);
      t[(size_t)b * r + p] = double_to_bf16_bits(s);
    }
  }
#pragma omp parallel for schedule(static)
  for (int j = 0; j < N; ++j) {
    for (int b = 0; b < B; ++b) {
      double s = 0.0;
      for (int p = 0; p < r; ++p)
        s += (double)bf16_to_float(z2[(size_t)j * r + p]) * (double)bf16_to_float(t[(size_t)b * r + p]);
      if (relu && !(s > 0.0)) s = 0.0;
      if (s == 0.0) s = 0.0;
      key_out[(size_t)b * N + j] = s;
    }
  }
  if (t_out) memcpy(t_out, t, (size_t)B * r * sizeof(uint16_t));
  free(t);
}

/* Algorithm 1 line 1, HiRE-LRQ (Sec. 4.1: low rank and int4 together; the paper gives no further detail, the
 * reading here chains two HiRE-Q products): both factors are int4 with one scale per row, Z1 stored transposed
 * (q1 [r, d], row p = column p of Z1, scales s1 [r]) and Z2 as q2 [N, r] with scales s2 [N].
 *   xq = int8(x);  t_p = float(sum_i q1[p,i] xq[i]) * s1[p]  -> stored as a bf16 activation
 *   tq = int8(t);  key_j = phi(float(sum_p q2[j,p] tq[p]) * s2[j])
 * The per-token scales of x and t are positive constants and are left out, as in HiRE-Q. */
void hire_oracle_scorer_lrq(const int8_t* q1, const float* s1, const int8_t* q2, const float* s2, const uint16_t* x,
                            int B, int N, int d, int r, int relu, uint16_t* t_out, float* key_out) {
  int8_t* xq = (int8_t*)malloc((size_t)B * d);
  float* sx = (float*)malloc((size_t)B * sizeof(float));
  float* tf = (float*)malloc((size_t)B * r * sizeof(float));
  uint16_t* tb = (uint16_t*)malloc((size_t)B * r * sizeof(uint16_t));
  int8_t* tq = (int8_t*)malloc((size_t)B * r);
  float* st = (float*)malloc((size_t)B * sizeof(float));
  hire_oracle_quantize_tokens_int8(x, B, d, xq, sx);
  hire_oracle_scorer_int4(q1, s1, xq, B, r, d, 0, NULL, tf);
  for (size_t i = 0; i < (size_t)B * r; ++i) tb[i] = double_to_bf16_bits((double)tf[i]);
  hire_oracle_quantize_tokens_int8(tb, B, r, tq, st);
  hire_oracle_scorer_int4(q2, s2, tq, B, N, r, relu, NULL, key_out);
  if (t_out) memcpy(t_out, tb, (size_t)B * r * sizeof(uint16_t));
  free(st);
  free(tq);
  free(tb);
  free(tf);
  free(sx);
  free(xq);
}

/* The scorers whose keys are fp32 numbers (HiRE-Q, HiRE-LRQ): keys of all N rows for B tokens. */
static void fp32_scorer_keys(int scorer_kind, const int8_t* q, const float* qscale, const int8_t* q1, const float* s1,
                             int r, const uint16_t* x, int B, int N, int d, int relu, int32_t* acc_out, float* kf) {
  if (scorer_kind == HIRE_ORACLE_SCORER_INT4) {
    int8_t* xq = (int8_t*)malloc((size_t)B * d);
    float* sx = (float*)malloc((size_t)B * sizeof(float));
    hire_oracle_quantize_tokens_int8(x, B, d, xq, sx);
    hire_oracle_scorer_int4(q, qscale, xq, B, N, d, relu, acc_out, kf);
    free(sx);
    free(xq);
  } else {
    hire_oracle_scorer_lrq(q1, s1, q, qscale, x, B, N, d, r, relu, NULL, kf);
  }
}

/* ---------------------------------------------------------------------- */
/* TopInd_k: indices of the k largest values, ties to the lower index.     */
typedef struct {
  double v;
  int32_t i;
} ranked_t;

static int ranked_cmp(const void* a, const void* b) {
  const ranked_t* x = (const ranked_t*)a;
  const ranked_t* y = (const ranked_t*)b;
  if (x->v > y->v) return -1;
  if (x->v < y->v) return 1;
  return (x->i > y->i) - (x->i < y->i);
}

static int int32_cmp(const void* a, const void* b) {
  int32_t x = *(const int32_t*)a, y = *(const int32_t*)b;
  return (x > y) - (x < y);
}

/* rank_order != 0: output in rank order (value descending, index ascending);
 * otherwise ascending by index.  margin (optional) receives the relative gap
 * between the k-th and (k+1)-th ranked values (inf if k == n). */
void hire_oracle_topk(const double* v, int n, int k, int rank_order, int32_t* idx_out, double* margin) {
  ranked_t* a = (ranked_t*)malloc((size_t)(n > 0 ? n : 1) * sizeof(ranked_t));
  for (int i = 0; i < n; ++i) {
    a[i].v = v[i];
    a[i].i = i;
  }
  qsort(a, (size_t)n, sizeof(ranked_t), ranked_cmp); /* total order: no ties left to chance */
  for (int t = 0; t < k; ++t) idx_out[t] = a[t].i;
  if (margin) {
    if (k >= n || k == 0) {
      *margin = INFINITY;
    } else {
      double hi = a[k - 1].v, lo = a[k].v, den = fabs(hi) > fabs(lo) ? fabs(hi) : fabs(lo);
      *margin = den > 0.0 ? (hi - lo) / den : 0.0;
    }
  }
  if (!rank_order) qsort(idx_out, (size_t)k, sizeof(int32_t), int32_cmp);
  free(a);
}

/* Same on float input (each float is exactly a double). */
void hire_oracle_topk_f32(const float* v, int n, int k, int relu, int rank_order, int32_t* idx_out) {
  double* w = (double*)malloc((size_t)(n > 0 ? n : 1) * sizeof(double));
  for (int i = 0; i < n; ++i) {
    double t = (double)v[i];
    if (relu && !(t > 0.0)) t = 0.0;
    w[i] = t;
  }
  hire_oracle_topk(w, n, k, rank_order, idx_out, NULL);
  free(w);
}

/* Sec. 3.4.1 dynamic overlap: ascending union of B index sets of size m. */
int hire_oracle_union(const int32_t* sets, int B, int m, int N, int32_t* U) {
  uint8_t* seen = (uint8_t*)calloc((size_t)(N > 0 ? N : 1), 1);
  for (int b = 0; b < B; ++b)
    for (int t = 0; t < m; ++t) seen[sets[(size_t)b * m + t]] = 1;
  int n = 0;
  for (int j = 0; j < N; ++j)
    if (seen[j]) U[n++] = j;
  free(seen);
  return n;
}

/* Algorithm 1 line 2, first half: exact phi(<z_j, x_b>) for j in U. */
void hire_oracle_exact_scores(const uint16_t* W, const uint16_t* x, const int32_t* U, int nU, int B, int d, int relu,
                              double* h) {
#pragma omp parallel for schedule(static)
  for (int t = 0; t < nU; ++t) {
    const uint16_t* row = W + (size_t)U[t] * d;
    for (int b = 0; b < B; ++b) {
      double s = 0.0;
      for (int i = 0; i < d; ++i) s += (double)bf16_to_float(row[i]) * (double)bf16_to_float(x[(size_t)b * d + i]);
      if (relu && !(s > 0.0)) s = 0.0;
      if (s == 0.0) s = 0.0;
      h[(size_t)b * nU + t] = s;
    }
  }
}

/* Shared front half of both steps: scorer -> per-token top-k' -> union ->
 * exact scores on the union.  Returns n_U; h is [B, n_U] with row stride
 * n_U (allocated here, caller frees). */
static int hire_candidates(int scorer_kind, const int8_t* q, const float* qscale, const uint16_t* z1,
                           const uint16_t* z2, int r, const int8_t* q1, const float* s1, const uint16_t* Z, const uint16_t* x, int B, int d, int N,
                           int kprime, int relu, int32_t* U, int32_t* acc_out, double* margin_kprime, double** h_out) {
  double* key = (double*)malloc((size_t)B * N * sizeof(double));
  if (scorer_kind != HIRE_ORACLE_SCORER_LOWRANK) {
    float* kf = (float*)malloc((size_t)B * N * sizeof(float));
    fp32_scorer_keys(scorer_kind, q, qscale, q1, s1, r, x, B, N, d, relu, acc_out, kf);
    for (size_t i = 0; i < (size_t)B * N; ++i) key[i] = (double)kf[i];
    free(kf);
  } else {
    hire_oracle_scorer_lowrank(z1, z2, x, B, N, d, r, relu, NULL, key);
  }
  int32_t* cand = (int32_t*)malloc((size_t)B * kprime * sizeof(int32_t));
  for (int b = 0; b < B; ++b)
    hire_oracle_topk(key + (size_t)b * N, N, kprime, 0, cand + (size_t)b * kprime,
                     margin_kprime ? margin_kprime + b : NULL);
  int nU = hire_oracle_union(cand, B, kprime, N, U);
  double* h = (double*)malloc((size_t)B * (nU > 0 ? nU : 1) * sizeof(double));
  hire_oracle_exact_scores(Z, x, U, nU, B, d, relu, h);
  free(cand);
  free(key);
  *h_out = h;
  return nU;
}

/* HiRE-FFN decode step (Sec. 3.4 with Algorithm 1, eq. (4), batch union).
 *   w1u, w2u : bf16 [N, d]          x : bf16 [B, d]
 *   y        : float [B, d]         topk_idx : [B, k] ascending unit index
 *   topk_val : double [B, k]        U : ascending union, capacity min(B*k', N)
 * Returns n_U. */
int hire_oracle_ffn_step(const uint16_t* w1u, const uint16_t* w2u, int scorer_kind, const int8_t* q,
                         const float* qscale, const uint16_t* z1, const uint16_t* z2, int r, const int8_t* q1, const float* s1,
                         const uint16_t* x, int B,
                         int d, int N, int k, int kprime, float* y, int32_t* topk_idx, double* topk_val, int32_t* U,
                         int32_t* acc_out, double* margin_kprime, double* margin_k) {
  double* h;
  int nU = hire_candidates(scorer_kind, q, qscale, z1, z2, r, q1, s1, w1u, x, B, d, N, kprime, 1, U, acc_out, margin_kprime, &h);
  int32_t* pos = (int32_t*)malloc((size_t)k * sizeof(int32_t));
  double* acc = (double*)malloc((size_t)d * sizeof(double));
  for (int b = 0; b < B; ++b) {
    /* positions within U are in unit order, so "lower position" = "lower unit index" */
    hire_oracle_topk(h + (size_t)b * nU, nU, k, 0, pos, margin_k ? margin_k + b : NULL);
    for (int i = 0; i < d; ++i) acc[i] = 0.0;
    for (int t = 0; t < k; ++t) {
      int j = U[pos[t]];
      double hv = h[(size_t)b * nU + pos[t]];
      if (topk_idx) topk_idx[(size_t)b * k + t] = j;
      if (topk_val) topk_val[(size_t)b * k + t] = hv;
      for (int i = 0; i < d; ++i) acc[i] += hv * (double)bf16_to_float(w2u[(size_t)j * d + i]);
    }
    for (int i = 0; i < d; ++i) y[(size_t)b * d + i] = (float)acc[i];
  }
  free(acc);
  free(pos);
  free(h);
  return nU;
}

/* HiRE-Softmax decode step (Sec. 3.3 with Algorithm 1, phi = identity, eq. (2)).
 *   W : bf16 [c, d]   top_idx : [B, k] rank order   top_prob, top_logit : double [B, k]
 * Returns n_U. */
int hire_oracle_softmax_step(const uint16_t* W, int scorer_kind, const int8_t* q, const float* qscale,
                             const uint16_t* z1, const uint16_t* z2, int r, const int8_t* q1, const float* s1,
                         const uint16_t* x, int B, int d, int c,
                             int k, int kprime, int32_t* top_idx, double* top_prob, double* top_logit, int32_t* U,
                             int32_t* acc_out, double* margin_kprime, double* margin_k) {
  double* z;
  int nU = hire_candidates(scorer_kind, q, qscale, z1, z2, r, q1, s1, W, x, B, d, c, kprime, 0, U, acc_out, margin_kprime, &z);
  int32_t* pos = (int32_t*)malloc((size_t)k * sizeof(int32_t));
  for (int b = 0; b < B; ++b) {
    const double* zb = z + (size_t)b * nU;
    hire_oracle_topk(zb, nU, k, 1, pos, margin_k ? margin_k + b : NULL);
    double zmax = zb[pos[0]], sum = 0.0;
    for (int t = 0; t < k; ++t) sum += exp(zb[pos[t]] - zmax);
    for (int t = 0; t < k; ++t) {
      top_idx[(size_t)b * k + t] = U[pos[t]];
      top_prob[(size_t)b * k + t] = exp(zb[pos[t]] - zmax) / sum;
      if (top_logit) top_logit[(size_t)b * k + t] = zb[pos[t]];
    }
  }
  free(pos);
  free(z);
  return nU;
}

/* Group-sparse HiRE-FFN decode step (Sec. 3.4, eq. (6), with Algorithm 1 and the batch union of Sec. 3.4.1).
 * The N hidden units form N/g groups of g adjacent units.  k and k' count units, so k'/g groups are shortlisted
 * and k/g groups survive (the subscripts of eq. (6)); the inner sum of eq. (6) runs over the g units of a group.
 *   approximate group activation  Phi[b, J] = sum_{l<g} |key[b, gJ+l]|, key = the scorer's phi(approximate score)
 *   S'_g(b) = TopInd_{k'/g}(Phi[b, :]);  U_g = union over the batch (ascending)
 *   exact group activation        E[b, J] = sum_{l<g} |phi(<u_{gJ+l}, x_b>)|  for J in U_g
 *   S~_g(b) = TopInd_{k/g}(E[b, :]) over U_g      (GroupTopInd_{g, k/g})
 *   y_b = sum_{J in S~_g(b)} sum_{l<g} phi(<u_{gJ+l}, x_b>) v_{gJ+l}
 * The int4 scorer's keys are fp32 numbers, and its group sums are formed in fp32, units in index order: the
 * decision "which groups" is then taken on the same numbers by anyone who follows this rule.  All else in double.
 *   topk_group : [B, k/g] ascending group index     topk_val : double [B, k], units of the chosen groups in order
 *   Ug         : ascending union of groups, capacity min(B*k'/g, N/g)
 * Returns |U_g|, or -1 if g does not divide N, k and k'. */
static int ffn_group_step_wide(const uint16_t* w1u, const uint16_t* w2u, int scorer_kind, const int8_t* q,
                               const float* qscale, const uint16_t* z1, const uint16_t* z2, int r, const int8_t* q1, const float* s1,
                         const uint16_t* x,
                               int B, int d, int N, int k, int kprime, int g, double* y, int32_t* topk_group,
                               double* topk_val, int32_t* Ug, int32_t* acc_out, double* margin_kprime,
                               double* margin_k) {
  if (g < 1 || N % g || k % g || kprime % g) return -1;
  const int G = N / g, kg = k / g, kpg = kprime / g;
  double* Phi = (double*)malloc((size_t)B * G * sizeof(double));
  if (scorer_kind != HIRE_ORACLE_SCORER_LOWRANK) {
    float* kf = (float*)malloc((size_t)B * N * sizeof(float));
    fp32_scorer_keys(scorer_kind, q, qscale, q1, s1, r, x, B, N, d, 1, acc_out, kf);
    for (int b = 0; b < B; ++b)
      for (int J = 0; J < G; ++J) {
        float sum = 0.0f;
        for (int l = 0; l < g; ++l) sum += fabsf(kf[(size_t)b * N + (size_t)J * g + l]);
        Phi[(size_t)b * G + J] = (double)sum;
      }
    free(kf);
  } else {
    double* key = (double*)malloc((size_t)B * N * sizeof(double));
    hire_oracle_scorer_lowrank(z1, z2, x, B, N, d, r, 1, NULL, key);
    for (int b = 0; b < B; ++b)
      for (int J = 0; J < G; ++J) {
        double sum = 0.0;
        for (int l = 0; l < g; ++l) sum += fabs(key[(size_t)b * N + (size_t)J * g + l]);
        Phi[(size_t)b * G + J] = sum;
      }
    free(key);
  }
  int32_t* shortlist = (int32_t*)malloc((size_t)B * kpg * sizeof(int32_t));
  for (int b = 0; b < B; ++b)
    hire_oracle_topk(Phi + (size_t)b * G, G, kpg, 0, shortlist + (size_t)b * kpg,
                     margin_kprime ? margin_kprime + b : NULL);
  const int nUg = hire_oracle_union(shortlist, B, kpg, G, Ug);
  free(shortlist);
  free(Phi);

  /* exact pre-activations of every unit of every shortlisted group */
  const int nu = nUg * g;
  int32_t* units = (int32_t*)malloc((size_t)(nu > 0 ? nu : 1) * sizeof(int32_t));
  for (int t = 0; t < nUg; ++t)
    for (int l = 0; l < g; ++l) units[(size_t)t * g + l] = Ug[t] * g + l;
  double* h = (double*)malloc((size_t)B * (nu > 0 ? nu : 1) * sizeof(double));
  hire_oracle_exact_scores(w1u, x, units, nu, B, d, 1, h);

  double* E = (double*)malloc((size_t)(nUg > 0 ? nUg : 1) * sizeof(double));
  int32_t* pos = (int32_t*)malloc((size_t)kg * sizeof(int32_t));
  double* acc = (double*)malloc((size_t)d * sizeof(double));
  for (int b = 0; b < B; ++b) {
    const double* hb = h + (size_t)b * nu;
    for (int t = 0; t < nUg; ++t) {
      double sum = 0.0;
      for (int l = 0; l < g; ++l) sum += fabs(hb[(size_t)t * g + l]);
      E[t] = sum;
    }
    hire_oracle_topk(E, nUg, kg, 0, pos, margin_k ? margin_k + b : NULL);
    for (int i = 0; i < d; ++i) acc[i] = 0.0;
    for (int t = 0; t < kg; ++t) {
      if (topk_group) topk_group[(size_t)b * kg + t] = Ug[pos[t]];
      for (int l = 0; l < g; ++l) {
        const int j = units[(size_t)pos[t] * g + l];
        const double hv = hb[(size_t)pos[t] * g + l];
        if (topk_val) topk_val[(size_t)b * k + (size_t)t * g + l] = hv;
        for (int i = 0; i < d; ++i) acc[i] += hv * (double)bf16_to_float(w2u[(size_t)j * d + i]);
      }
    }
    for (int i = 0; i < d; ++i) y[(size_t)b * d + i] = acc[i];
  }
  free(acc);
  free(pos);
  free(E);
  free(h);
  free(units);
  return nUg;
}

int hire_oracle_ffn_group_step(const uint16_t* w1u, const uint16_t* w2u, int scorer_kind, const int8_t* q,
                               const float* qscale, const uint16_t* z1, const uint16_t* z2, int r, const int8_t* q1, const float* s1,
                         const uint16_t* x,
                               int B, int d, int N, int k, int kprime, int g, float* y, int32_t* topk_group,
                               double* topk_val, int32_t* Ug, int32_t* acc_out, double* margin_kprime,
                               double* margin_k) {
  double* wide = (double*)malloc((size_t)B * d * sizeof(double));
  const int n = ffn_group_step_wide(w1u, w2u, scorer_kind, q, qscale, z1, z2, r, q1, s1, x, B, d, N, k, kprime, g, wide,
                                    topk_group, topk_val, Ug, acc_out, margin_kprime, margin_k);
  if (n >= 0)
    for (size_t i = 0; i < (size_t)B * d; ++i) y[i] = (float)wide[i];
  free(wide);
  return n;
}

/* CommonPath FFN (Sec. 3.4.1, static overlap, eq. (7)): m1 hidden units (u^d, v^d) are used by every token as in
 * the dense layer of eq. (3), the other m2 = N units (u^gs, v^gs) through the group-sparse HiRE step above;
 * the two contributions are added.  dense_w1u, dense_w2u : bf16 [m1, d]; the rest as in the group step, all of
 * whose indices count inside the sparse part.  m1 = 0 is the group step itself. */
int hire_oracle_ffn_commonpath_step(const uint16_t* dense_w1u, const uint16_t* dense_w2u, int m1, const uint16_t* w1u,
                                    const uint16_t* w2u, int scorer_kind, const int8_t* q, const float* qscale,
                                    const uint16_t* z1, const uint16_t* z2, int r, const int8_t* q1, const float* s1,
                         const uint16_t* x, int B, int d,
                                    int N, int k, int kprime, int g, float* y, int32_t* topk_group, double* topk_val,
                                    int32_t* Ug, int32_t* acc_out, double* margin_kprime, double* margin_k) {
  double* sparse = (double*)malloc((size_t)B * d * sizeof(double));
  double* dense = (double*)calloc((size_t)B * d, sizeof(double));
  const int n = ffn_group_step_wide(w1u, w2u, scorer_kind, q, qscale, z1, z2, r, q1, s1, x, B, d, N, k, kprime, g, sparse,
                                    topk_group, topk_val, Ug, acc_out, margin_kprime, margin_k);
  if (n >= 0) {
    for (int b = 0; b < B; ++b)
      for (int j = 0; j < m1; ++j) {
        double pre = 0.0;
        for (int i = 0; i < d; ++i)
          pre += (double)bf16_to_float(dense_w1u[(size_t)j * d + i]) * (double)bf16_to_float(x[(size_t)b * d + i]);
        if (pre > 0.0)
          for (int i = 0; i < d; ++i)
            dense[(size_t)b * d + i] += pre * (double)bf16_to_float(dense_w2u[(size_t)j * d + i]);
      }
    for (size_t i = 0; i < (size_t)B * d; ++i) y[i] = (float)(dense[i] + sparse[i]);
  }
  free(dense);
  free(sparse);
  return n;
}

/* HiRE-FFN with the distributed approximate top-k of Algorithm 2 (DA-TOP-k), all "machines" on one device:
 * the N hidden units are split into s contiguous shards of N/s units; every shard runs Algorithm 1 on its own
 * units with the quotas k'/s and k/s - rounded up where s does not divide them (the algorithm writes the
 * fractions only): q' = ceil(k'/s), q = ceil(k/s), so s q >= k units are used in all - and the shards'
 * contributions are combined (for the FFN of eq. (4): summed).
 * With a batch, each shard unions its tokens' shortlists (Sec. 3.4.1) before the exact stage.
 *   per shard i, token b:  S'_{i,b} = TopInd_{q'}(key[b, shard i]);   U_i = union_b S'_{i,b}  (ascending)
 *                          h[b,j] = relu(<u_j, x_b>), j in U_i;       S_{i,b} = TopInd_{q}(h[b, U_i])
 *   y_b = sum_i sum_{j in S_{i,b}} h[b,j] v_j
 *   topk_idx : [B, s q]  shard after shard, ascending inside a shard (hence ascending overall)
 *   topk_val : double [B, s q] same order
 *   U        : [s, cap] padded per shard, cap = min(B*q', N/s);  nU : [s] sizes of the U_i
 * Returns 0, or -1 if s does not divide N or a quota exceeds what it is taken from (q' > N/s, q > q'). */
int hire_oracle_ffn_shard_step(const uint16_t* w1u, const uint16_t* w2u, const int8_t* q, const float* qscale,
                               const uint16_t* x, int B, int d, int N, int k, int kprime, int s, float* y,
                               int32_t* topk_idx, double* topk_val, int32_t* U, int32_t* nU, int32_t* acc_out,
                               double* margin_kprime, double* margin_k) {
  if (s < 1 || N % s || k < 1 || kprime < k) return -1;
  const int Ls = N / s, kps = (kprime + s - 1) / s, ks = (k + s - 1) / s;
  if (kps > Ls || ks > kps) return -1;
  const int kq = s * ks; /* row length of topk_idx / topk_val */
  const int cap = (long long)B * kps < Ls ? B * kps : Ls;
  int8_t* xq = (int8_t*)malloc((size_t)B * d);
  float* sx = (float*)malloc((size_t)B * sizeof(float));
  float* kf = (float*)malloc((size_t)B * N * sizeof(float));
  hire_oracle_quantize_tokens_int8(x, B, d, xq, sx);
  hire_oracle_scorer_int4(q, qscale, xq, B, N, d, 1, acc_out, kf);
  free(sx);
  free(xq);
  double* yacc = (double*)calloc((size_t)B * d, sizeof(double));
  double* key = (double*)malloc((size_t)Ls * sizeof(double));
  int32_t* shortlist = (int32_t*)malloc((size_t)B * kps * sizeof(int32_t));
  int32_t* pos = (int32_t*)malloc((size_t)ks * sizeof(int32_t));
  double* h = (double*)malloc((size_t)B * cap * sizeof(double));
  if (margin_kprime)
    for (int b = 0; b < B; ++b) margin_kprime[b] = INFINITY;
  if (margin_k)
    for (int b = 0; b < B; ++b) margin_k[b] = INFINITY;
  for (int i = 0; i < s; ++i) {
    int32_t* Ui = U + (size_t)i * cap;
    for (int b = 0; b < B; ++b) {
      double m;
      for (int j = 0; j < Ls; ++j) key[j] = (double)kf[(size_t)b * N + (size_t)i * Ls + j];
      hire_oracle_topk(key, Ls, kps, 0, shortlist + (size_t)b * kps, &m);
      if (margin_kprime && m < margin_kprime[b]) margin_kprime[b] = m;
    }
    const int n = hire_oracle_union(shortlist, B, kps, Ls, Ui); /* local indices, ascending */
    for (int t = 0; t < n; ++t) Ui[t] += i * Ls;
    nU[i] = n;
    hire_oracle_exact_scores(w1u, x, Ui, n, B, d, 1, h);
    for (int b = 0; b < B; ++b) {
      double m;
      hire_oracle_topk(h + (size_t)b * n, n, ks, 0, pos, &m);
      if (margin_k && m < margin_k[b]) margin_k[b] = m;
      for (int t = 0; t < ks; ++t) {
        const int j = Ui[pos[t]];
        const double hv = h[(size_t)b * n + pos[t]];
        if (topk_idx) topk_idx[(size_t)b * kq + (size_t)i * ks + t] = j;
        if (topk_val) topk_val[(size_t)b * kq + (size_t)i * ks + t] = hv;
        for (int c = 0; c < d; ++c) yacc[(size_t)b * d + c] += hv * (double)bf16_to_float(w2u[(size_t)j * d + c]);
      }
    }
  }
  for (size_t c = 0; c < (size_t)B * d; ++c) y[c] = (float)yacc[c];
  free(h);
  free(pos);
  free(shortlist);
  free(key);
  free(yacc);
  free(kf);
  return 0;
}

/* ---------------------------------------------------------------------- */
/* Dense definitions, written separately from the step functions above.    */

/* eq. (3): FF(x) = sum_j relu(<u_j,x>) v_j. */
void hire_oracle_dense_ffn(const uint16_t* w1u, const uint16_t* w2u, const uint16_t* x, int B, int d, int N,
                           double* y) {
  for (int b = 0; b < B; ++b) {
    for (int i = 0; i < d; ++i) y[(size_t)b * d + i] = 0.0;
    for (int j = 0; j < N; ++j) {
      double pre = 0.0;
      for (int i = 0; i < d; ++i)
        pre += (double)bf16_to_float(w1u[(size_t)j * d + i]) * (double)bf16_to_float(x[(size_t)b * d + i]);
      if (pre > 0.0)
        for (int i = 0; i < d; ++i) y[(size_t)b * d + i] += pre * (double)bf16_to_float(w2u[(size_t)j * d + i]);
    }
  }
}

/* eq. (4): FF_k(x), S(x) = TopInd_k(relu(U^T x)) over all N units. */
void hire_oracle_topk_ffn(const uint16_t* w1u, const uint16_t* w2u, const uint16_t* x, int B, int d, int N, int k,
                          double* y, int32_t* S_out) {
  double* act = (double*)malloc((size_t)N * sizeof(double));
  int32_t* S = (int32_t*)malloc((size_t)k * sizeof(int32_t));
  for (int b = 0; b < B; ++b) {
    for (int j = 0; j < N; ++j) {
      double pre = 0.0;
      for (int i = 0; i < d; ++i)
        pre += (double)bf16_to_float(w1u[(size_t)j * d + i]) * (double)bf16_to_float(x[(size_t)b * d + i]);
      act[j] = pre > 0.0 ? pre : 0.0;
    }
    hire_oracle_topk(act, N, k, 0, S, NULL);
    for (int i = 0; i < d; ++i) y[(size_t)b * d + i] = 0.0;
    for (int t = 0; t < k; ++t)
      for (int i = 0; i < d; ++i)
        y[(size_t)b * d + i] += act[S[t]] * (double)bf16_to_float(w2u[(size_t)S[t] * d + i]);
    if (S_out) memcpy(S_out + (size_t)b * k, S, (size_t)k * sizeof(int32_t));
  }
  free(S);
  free(act);
}

/* eq. (1): Softmax(x) = exp(Wx)/||exp(Wx)||_1 over all c classes. */
void hire_oracle_dense_softmax(const uint16_t* W, const uint16_t* x, int B, int d, int c, double* p) {
  for (int b = 0; b < B; ++b) {
    double* pb = p + (size_t)b * c;
    double zmax = -INFINITY, sum = 0.0;
    for (int j = 0; j < c; ++j) {
      double z = 0.0;
      for (int i = 0; i < d; ++i)
        z += (double)bf16_to_float(W[(size_t)j * d + i]) * (double)bf16_to_float(x[(size_t)b * d + i]);
      pb[j] = z;
      if (z > zmax) zmax = z;
    }
    for (int j = 0; j < c; ++j) {
      pb[j] = exp(pb[j] - zmax);
      sum += pb[j];
    }
    for (int j = 0; j < c; ++j) pb[j] /= sum;
  }
}

/* eq. (2) taken literally: Top_k of the full softmax vector (others zeroed),
 * divided by its l1 norm.  Output is the dense c-vector. */
void hire_oracle_softmax_k(const uint16_t* W, const uint16_t* x, int B, int d, int c, int k, double* pk) {
  double* p = (double*)malloc((size_t)B * c * sizeof(double));
  int32_t* S = (int32_t*)malloc((size_t)k * sizeof(int32_t));
  hire_oracle_dense_softmax(W, x, B, d, c, p);
  for (int b = 0; b < B; ++b) {
    hire_oracle_topk(p + (size_t)b * c, c, k, 0, S, NULL);
    double l1 = 0.0;
    for (int t = 0; t < k; ++t) l1 += p[(size_t)b * c + S[t]];
    for (int j = 0; j < c; ++j) pk[(size_t)b * c + j] = 0.0;
    for (int t = 0; t < k; ++t) pk[(size_t)b * c + S[t]] = p[(size_t)b * c + S[t]] / l1;
  }
  free(S);
  free(p);
}

/* Threads the row-parallel loops above will use (for the benchmark report). */
int hire_oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}
