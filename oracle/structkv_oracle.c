/*
 * StructKV CPU oracle -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, fp64 evaluation of what the scoring / selection / gather path
 * computes, written from the paper's definitions.  It shares no code with the
 * HIP library and is never on the product path: only the tests, the smoke
 * check and the bench's cpu_baseline leg may call it.
 *
 * What each routine follows (StructKV paper):
 *   skv_oracle_score_layer       Eq. 1 (window attention, softmax over keys),
 *                                Eq. 2 without its 1/w (raw in-degree D_j),
 *                                Eq. 4 (attention entropy, natural log, 0 ln 0 = 0)
 *   skv_oracle_accumulate        Alg. 1 line 6:  C <- lambda C + S,  S = D / w  (Eq. 2)
 *   skv_oracle_centrality_closed Eq. 3:  C_j = sum_l lambda^(L-1-l) S_j^(l)
 *   skv_oracle_select_topk       Eq. 10 / Eq. 13: top-k of a score vector united with
 *                                the observation window (reading: top-k over the
 *                                prefix [0, n-keep_tail), window appended, ties to the
 *                                lower index, output ascending)
 *   skv_oracle_gather_rows       Alg. 1 line 17: keep K/V rows at the selected indices; the same row copy
 *                                serves Eq. 11 (hidden states and positions kept at I_struct)
 *   skv_oracle_pivot_metrics     Eq. 5-6: sparsity (mass of the top 10 % of keys) and variance of a head's
 *                                attention, read as the head's attention pooled (mean) over the window rows
 *   skv_oracle_transition        Eq. 7-9: normalised metric gradients, transition score T_l, pivot layer L*
 *   skv_oracle_block_scores      Sec. 4.1, implementation details: a cache block's score is the sum of its
 *                                tokens' centralities
 *
 * Readings (the paper is silent or ambiguous): the window is the last w
 * positions n-w .. n-1 (the 1/w normaliser fixes w terms); by default every
 * window query sees all n keys (Eq. 1 and Eq. 4 carry no mask); causal=1 masks
 * keys j > n-w+i for window row i.
 *
 * Pins: see tests/test_oracle_pins.py (closed forms, invariants, library
 * softmax, brute force).  Parity status: pinned by invariants only -- the
 * paper prints no numeric example for this path.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

enum { SKV_F32 = 0, SKV_BF16 = 1 };

int skv_oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* exact widening of one stored element to double */
static inline double load_elem(const void* base, int64_t i, int dtype) {
  if (dtype == SKV_F32) return (double)((const float*)base)[i];
  uint32_t bits = ((uint32_t)((const uint16_t*)base)[i]) << 16;
  float f;
  memcpy(&f, &bits, 4);
  return (double)f;
}

/*
 * One layer, one sequence.
 *   q_win : [Hq][w][d]   window queries (positions n-w .. n-1), dtype as given
 *   k     : token j of KV head g at element offset g*k_stride_head + j*k_stride_tok, d contiguous
 *   indeg : [n]  out, D_j = sum over all query heads and window rows of a_{t,j}
 *   entropy          : out scalar, Eq. 4
 *   entropy_per_head : [Hq] out or NULL (Eq. 4's inner bracket per head)
 *   probs            : [Hq][w][n] out or NULL (the attention rows themselves)
 * returns 0 on success, 1 on bad arguments, 2 on allocation failure.
 */
int skv_oracle_score_layer(int dtype, const void* q_win, const void* k, int64_t k_stride_head,
                           int64_t k_stride_tok, int Hq, int G, int d, int w, int64_t n, int causal,
                           double scale, double* indeg, double* entropy, double* entropy_per_head,
                           double* probs) {
  if (Hq <= 0 || G <= 0 || Hq % G || d <= 0 || w <= 0 || n <= 0) return 1;
  if (causal && n < w) return 1;
  const int gs = Hq / G;
  const int R = gs * w; /* query rows that share one KV head */
  if (scale == 0.0) scale = 1.0 / sqrt((double)d);

  double* S = (double*)malloc(sizeof(double) * (size_t)R * (size_t)n);
  double* qd = (double*)malloc(sizeof(double) * (size_t)R * (size_t)d);
  double* row_ent = (double*)malloc(sizeof(double) * (size_t)Hq * (size_t)w);
  if (!S || !qd || !row_ent) { free(S); free(qd); free(row_ent); return 2; }

  for (int64_t j = 0; j < n; ++j) indeg[j] = 0.0;

  for (int g = 0; g < G; ++g) {
    /* the group's queries, widened: row r = (h - g*gs)*w + i */
    for (int r = 0; r < R; ++r)
      for (int c = 0; c < d; ++c)
        qd[(size_t)r * d + c] = load_elem(q_win, ((int64_t)g * R + r) * d + c, dtype);

    /* Eq. 1, the logits: s_{r,j} = (q_r . k_j) * scale */
#pragma omp parallel
    {
      double* kd = (double*)malloc(sizeof(double) * (size_t)d);
#pragma omp for schedule(static)
      for (int64_t j = 0; j < n; ++j) {
        const int64_t base = (int64_t)g * k_stride_head + j * k_stride_tok;
        for (int c = 0; c < d; ++c) kd[c] = load_elem(k, base + c, dtype);
        for (int r = 0; r < R; ++r) {
          const double* qr = qd + (size_t)r * d;
          double acc = 0.0;
#pragma omp simd reduction(+ : acc)
          for (int c = 0; c < d; ++c) acc += qr[c] * kd[c];
          S[(size_t)r * n + j] = acc * scale;
        }
      }
      free(kd);
    }

    /* Eq. 1, the softmax over keys, row by row; Eq. 4's inner sum per row */
#pragma omp parallel for schedule(static)
    for (int r = 0; r < R; ++r) {
      double* s = S + (size_t)r * n;
      const int i = r % w;
      const int64_t n_vis = causal ? (n - w + i + 1) : n; /* keys this row may see */
      double m = s[0];
      for (int64_t j = 1; j < n_vis; ++j) if (s[j] > m) m = s[j];
      double Z = 0.0;
      for (int64_t j = 0; j < n_vis; ++j) { s[j] = exp(s[j] - m); Z += s[j]; }
      double ent = 0.0;
      for (int64_t j = 0; j < n_vis; ++j) {
        const double a = s[j] / Z;
        s[j] = a;
        if (a > 0.0) ent -= a * log(a);
      }
      for (int64_t j = n_vis; j < n; ++j) s[j] = 0.0;
      row_ent[(size_t)g * R + r] = ent;
    }

    /* Eq. 2 without 1/w: column sums over the window rows and the group's heads */
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < n; ++j) {
      double acc = 0.0;
      for (int r = 0; r < R; ++r) acc += S[(size_t)r * n + j];
      indeg[j] += acc; /* groups are visited in order: the sum over g is sequential */
    }

    if (probs) memcpy(probs + (size_t)g * R * n, S, sizeof(double) * (size_t)R * (size_t)n);
  }

  /* Eq. 4: mean over window rows, then mean over heads */
  double tot = 0.0;
  for (int h = 0; h < Hq; ++h) {
    double hs = 0.0;
    for (int i = 0; i < w; ++i) hs += row_ent[(size_t)h * w + i];
    hs /= (double)w;
    if (entropy_per_head) entropy_per_head[h] = hs;
    tot += hs;
  }
  *entropy = tot / (double)Hq;

  free(S); free(qd); free(row_ent);
  return 0;
}

/* Alg. 1 line 6 with S = D * inv_w (Eq. 2's 1/w):  C <- lambda C + inv_w D */
void skv_oracle_accumulate(double* centrality, const double* indeg, int64_t n, double lambda,
                           double inv_w) {
  for (int64_t j = 0; j < n; ++j) centrality[j] = lambda * centrality[j] + inv_w * indeg[j];
}

/* Eq. 3 written out: C_j = sum_{l=0}^{L-1} lambda^(L-1-l) S_j^(l);  S is [L][n] */
void skv_oracle_centrality_closed(const double* S, int L, int64_t n, double lambda, double* C) {
  for (int64_t j = 0; j < n; ++j) {
    double acc = 0.0;
    for (int l = 0; l < L; ++l) acc += pow(lambda, (double)(L - 1 - l)) * S[(size_t)l * n + j];
    C[j] = acc;
  }
}

typedef struct { double s; int64_t j; } skv_pair;

static int cmp_score_desc_index_asc(const void* a, const void* b) {
  const skv_pair* x = (const skv_pair*)a;
  const skv_pair* y = (const skv_pair*)b;
  if (x->s > y->s) return -1;
  if (x->s < y->s) return 1;
  return (x->j < y->j) ? -1 : (x->j > y->j);
}

static int cmp_i32(const void* a, const void* b) {
  const int32_t x = *(const int32_t*)a, y = *(const int32_t*)b;
  return (x < y) ? -1 : (x > y);
}

/*
 * Eq. 10 / Eq. 13.  The k largest of scores[0 .. n-keep_tail) (ties: lower index first),
 * then the last keep_tail positions; idx_out [k + keep_tail] ascending.
 * returns 0, or 1 unless 0 <= keep_tail <= n and 0 <= k <= n - keep_tail.
 */
int skv_oracle_select_topk(const double* scores, int64_t n, int64_t k, int64_t keep_tail,
                           int32_t* idx_out) {
  if (n < 0 || keep_tail < 0 || keep_tail > n || k < 0 || k > n - keep_tail) return 1;
  const int64_t m = n - keep_tail;
  skv_pair* p = (skv_pair*)malloc(sizeof(skv_pair) * (size_t)(m > 0 ? m : 1));
  if (!p) return 2;
  for (int64_t j = 0; j < m; ++j) { p[j].s = scores[j]; p[j].j = j; }
  qsort(p, (size_t)m, sizeof(skv_pair), cmp_score_desc_index_asc);
  for (int64_t i = 0; i < k; ++i) idx_out[i] = (int32_t)p[i].j;
  qsort(idx_out, (size_t)k, sizeof(int32_t), cmp_i32);
  for (int64_t i = 0; i < keep_tail; ++i) idx_out[k + i] = (int32_t)(m + i);
  free(p);
  return 0;
}

/*
 * Alg. 1 line 17.  dst[g][i][:] = src[g][idx[i]][:], byte copy of rows of row_bytes bytes;
 * strides in bytes.
 */
void skv_oracle_gather_rows(const void* src, int64_t src_stride_head, int64_t src_stride_tok,
                            void* dst, int64_t dst_stride_head, int64_t dst_stride_tok, int G,
                            int64_t row_bytes, const int32_t* idx, int64_t n_idx, int64_t src_tok_base,
                            int64_t dst_tok_base) {
  for (int g = 0; g < G; ++g)
    for (int64_t i = 0; i < n_idx; ++i)
      memcpy((char*)dst + g * dst_stride_head + (dst_tok_base + i) * dst_stride_tok,
             (const char*)src + g * src_stride_head + (src_tok_base + idx[i]) * src_stride_tok,
             (size_t)row_bytes);
}

/* Block-level aggregation for paged caches (Sec. 4.1, implementation details): out[k] = sum of scores[k*block .. min(n,(k+1)*block)),
 * k < ceil(n / block).  Plain left-to-right fp64 sums. */
void skv_oracle_block_scores(const double* scores, int64_t n, int64_t block, double* out) {
  const int64_t nb = (n + block - 1) / block;
  for (int64_t k = 0; k < nb; ++k) {
    double s = 0.0;
    for (int64_t t = k * block; t < n && t < (k + 1) * block; ++t) s += scores[t];
    out[k] = s;
  }
}

/* Eq. 5-6.  The paper writes a^(l,h) with a free row index; reading: a^(l,h)_j = (1/w) sum_t a_{t,j}, the head's
 * attention pooled over the window rows (a probability vector over the n keys).  Per head: rho_h = sum of its
 * k = ceil(top_frac n) largest entries, var_h = (1/n) sum_j (a_j - mean)^2.  Outputs: means over the heads.
 * probs: [Hq][w][n] attention rows of ONE sequence. */
static int cmp_desc(const void* a, const void* b) {
  const double x = *(const double*)a, y = *(const double*)b;
  return x < y ? 1 : (x > y ? -1 : 0);
}
void skv_oracle_pivot_metrics(const double* probs, int Hq, int w, int64_t n, double top_frac, double* sparsity,
                              double* variance) {
  double rho = 0.0, var = 0.0;
  double* pooled = (double*)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
  int64_t k = (int64_t)ceil(top_frac * (double)n);
  if (k < 1) k = 1;
  if (k > n) k = n;
  for (int h = 0; h < Hq; ++h) {
    double mean = 0.0;
    for (int64_t j = 0; j < n; ++j) {
      double s = 0.0;
      for (int i = 0; i < w; ++i) s += probs[((int64_t)h * w + i) * n + j];
      pooled[j] = s / w;
      mean += pooled[j];
    }
    mean /= (double)n;
    double v = 0.0;
    for (int64_t j = 0; j < n; ++j) v += (pooled[j] - mean) * (pooled[j] - mean);
    var += v / (double)n;
    qsort(pooled, (size_t)n, sizeof(double), cmp_desc);
    double top = 0.0;
    for (int64_t j = 0; j < k; ++j) top += pooled[j];
    rho += top;
  }
  free(pooled);
  *sparsity = n > 0 ? rho / Hq : 0.0;
  *variance = n > 0 ? var / Hq : 0.0;
}

/* Eq. 7-9 over the layers 0..L-1 given: dM_l = M_l - M_{l-1} for l >= 1, each metric's differences scaled to
 * [0,1] over l = 1..L-1 (all equal: 0), T_l = w1 grad(-H)_l + w2 grad(rho)_l + w3 grad(V)_l, T_0 = 0 (no
 * difference exists), L* = argmax_{l>=1} T_l + 1 (lowest l on ties; L < 2: returns L).  Returns L*. */
int skv_oracle_transition(const double* H, const double* rho, const double* V, int L, double w1, double w2,
                          double w3, double* T) {
  for (int l = 0; l < L; ++l) T[l] = 0.0;
  if (L < 2) return L;
  const double* M[3] = {H, rho, V};
  const double sign[3] = {-1.0, 1.0, 1.0};
  const double wt[3] = {w1, w2, w3};
  for (int m = 0; m < 3; ++m) {
    double lo = 0.0, hi = 0.0;
    for (int l = 1; l < L; ++l) {
      const double d = sign[m] * (M[m][l] - M[m][l - 1]);
      if (l == 1 || d < lo) lo = d;
      if (l == 1 || d > hi) hi = d;
    }
    for (int l = 1; l < L; ++l) {
      const double d = sign[m] * (M[m][l] - M[m][l - 1]);
      T[l] += hi > lo ? wt[m] * (d - lo) / (hi - lo) : 0.0;
    }
  }
  int best = 1;
  for (int l = 2; l < L; ++l)
    if (T[l] > T[best]) best = l;
  return best + 1;
}
