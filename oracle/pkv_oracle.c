/*
 * pkv_oracle.c -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, step-by-step CPU statement of PyramidKV's prefill-time
 * KV-cache compression (arXiv 2406.02069), written to be checked against the
 * paper by eye.  It is the reference the GPU library is compared with; it is
 * never part of the product path, shares no code with the HIP library and is
 * never tuned.  All floating point is fp64 on the exact values of the bf16
 * inputs.  The only parallelism is OpenMP over independent query rows and
 * independent (sequence, KV head) units; nothing is blocked, fused or
 * reordered.
 *
 * Pins (tests/test_oracle_*.py): library softmax for the alpha=1 special
 * case, the harmonic closed form for identical keys (causal mask, window sum,
 * group mean), library 1-D pooling, brute-force sorting on tiny inputs,
 * planted one-hot / sink patterns, window retention, full-cache edge and the
 * closed forms of the budget sequence; for the variant with supplied softmax
 * denominators: a library log-sum-exp reproduces the plain softmax, the
 * closed form exp(-ln c) = 1/c for all-zero logits, and the exp(-delta)
 * scaling of a row whose denominator is shifted; for the paged output: a
 * hand-written pool image and the identity table; for the attention recall:
 * everything kept gives 1, identical keys give a harmonic closed form, and
 * the kept mass equals the sum of the window scores at the kept positions;
 * for the geometric schedule: its defining ratios and sum; for the decoding
 * attention over the compacted cache: a library softmax attention, the mean
 * of V for identical keys and the single-key case.  The integer rounding of the budgets,
 * the pool padding rule and the GQA mean are conventions the paper does not
 * fix ("parity unpinned" by the paper; pinned only to the stated reading).
 *
 * Notation follows the paper: m layers (here L), n tokens, d = d_k, alpha
 * instruction tokens, beta pyramid shape, k^l budget of layer l.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define PKVO_POOL_NONE 0
#define PKVO_POOL_MAX 1
#define PKVO_POOL_AVG 2

/* bf16 -> double, exact: a bf16 is the upper half of an IEEE fp32. */
static double bf16_to_f64(uint16_t h) {
  uint32_t u = ((uint32_t)h) << 16;
  float f;
  memcpy(&f, &u, sizeof f);
  return (double)f;
}

/* ------------------------------------------------------------------------
 * Budget allocation (Sec. 4.2.1, Eq. budget).
 *
 * The alpha instruction tokens are retained in every layer; the pyramid is
 * laid over the REMAINING budget A = avg - alpha per layer, k_total = L*A:
 *   top    k^{m-1} = k_total / (beta*m)           = A / beta
 *   bottom k^0     = 2*k_total/m - k^{m-1}        = 2A - A/beta
 *   k^l = k^0 - (k^0 - k^{m-1})/(m-1) * l         (arithmetic sequence)
 * which is r_l = A*[(2beta-1)(L-1) - 2(beta-1) l] / (beta (L-1)).
 * Integerisation (not fixed by the paper): floor every r_l, then hand the
 * missing units, one each, to the layers with the largest fractional part,
 * ties to the lower layer.  k_out[l] = alpha + that integer.
 * Returns 0, or 1 for invalid arguments.
 * ---------------------------------------------------------------------- */
int pkvo_budgets(int32_t L, int32_t avg, int32_t beta, int32_t alpha,
                 int32_t *k_out) {
  if (L < 1 || beta < 1 || alpha < 0 || avg < alpha || !k_out) return 1;
  int64_t A = (int64_t)avg - alpha;
  if (L == 1) {
    k_out[0] = avg;
    return 0;
  }
  int64_t den = (int64_t)beta * (L - 1);
  int64_t *rem = (int64_t *)malloc(sizeof(int64_t) * (size_t)L);
  int64_t sum_floor = 0;
  for (int32_t l = 0; l < L; ++l) {
    int64_t num = A * ((2 * (int64_t)beta - 1) * (L - 1) -
                       2 * ((int64_t)beta - 1) * l);
    int64_t f = num / den; /* num >= 0 */
    rem[l] = num % den;
    k_out[l] = (int32_t)f;
    sum_floor += f;
  }
  int64_t left = (int64_t)L * A - sum_floor;
  while (left > 0) {
    int32_t best = -1;
    for (int32_t l = 0; l < L; ++l)
      if (rem[l] >= 0 && (best < 0 || rem[l] > rem[best])) best = l;
    k_out[best] += 1;
    rem[best] = -1; /* each layer gets at most one extra unit */
    --left;
  }
  for (int32_t l = 0; l < L; ++l) k_out[l] += alpha;
  free(rem);
  return 0;
}

/* ------------------------------------------------------------------------
 * Other allocation strategies of the ablation (appendix "Allocation
 * Strategies"): the paper names a geometric and an exponential decay beside
 * the linear one and gives no formula for either.  Written in the layer
 * index both are r_l = C * q^l, so one schedule stands for the two:
 *   schedule 0: linear (pkvo_budgets above)
 *   schedule 1: geometric: r_l = C * q^l with the linear pyramid's ratio
 *               between top and bottom layer, q^(L-1) = 1/(2 beta - 1), and
 *               C such that sum_l r_l = L * A  (A = avg - alpha)
 *   schedule 2: uniform, r_l = A (what SnapKV-style selection uses)
 * Integerisation as above: floor, then one unit each to the largest
 * fractional parts (ties to the lower layer); k_out[l] = alpha + integer.
 * "Parity unpinned" by the paper (no formula, no numbers).
 * ---------------------------------------------------------------------- */
int pkvo_budgets_schedule(int32_t L, int32_t avg, int32_t beta, int32_t alpha,
                          int32_t schedule, int32_t *k_out) {
  if (schedule == 0) return pkvo_budgets(L, avg, beta, alpha, k_out);
  if (L < 1 || beta < 1 || alpha < 0 || avg < alpha || !k_out) return 1;
  if (schedule != 1 && schedule != 2) return 1;
  const int64_t A = (int64_t)avg - alpha;
  if (schedule == 2 || L == 1 || beta == 1) {
    for (int32_t l = 0; l < L; ++l) k_out[l] = avg;
    return 0;
  }
  double *r = (double *)malloc(sizeof(double) * (size_t)L);
  const double q = pow(1.0 / (2.0 * (double)beta - 1.0), 1.0 / (double)(L - 1));
  double sum = 0.0;
  for (int32_t l = 0; l < L; ++l) {
    r[l] = pow(q, (double)l);
    sum += r[l];
  }
  int64_t given = 0;
  for (int32_t l = 0; l < L; ++l) {
    r[l] = (double)L * (double)A * r[l] / sum;
    k_out[l] = (int32_t)floor(r[l]);
    given += k_out[l];
    r[l] -= floor(r[l]); /* fractional part */
  }
  for (int64_t left = (int64_t)L * A - given; left > 0; --left) {
    int32_t best = 0;
    for (int32_t l = 1; l < L; ++l)
      if (r[l] > r[best]) best = l;
    k_out[best] += 1;
    r[best] = -1.0;
  }
  for (int32_t l = 0; l < L; ++l) k_out[l] += alpha;
  free(r);
  return 0;
}

/* ------------------------------------------------------------------------
 * Window attention received by every prefix key (Sec. 4.2.2, Eq. Al and
 * Eq. att_score), for one sequence of n tokens and one KV head g whose
 * group holds G query heads.
 *
 *   q  : [G][alpha][d]  queries of the last alpha tokens (positions
 *                       n-alpha .. n-1) of the G heads of the group
 *   k  : [n][d]         keys of the KV head
 *   s_head : [G][n-alpha] out, s^h_i = sum_t A^{(h,t)}_i   (may be NULL)
 *   s_mean : [n-alpha]    out, (1/G) sum_h s^h_i
 *
 * Each window query at absolute position p attends causally to keys 0..p;
 * its softmax runs over exactly those p+1 keys (window keys included).
 * Scores are reported for prefix keys i < n-alpha only.
 *
 *   lse : [G][alpha] or NULL.  When given, lse[r] is taken as the natural
 *         log of row r's softmax denominator, ln sum_{i<=p} exp(l_ri), as
 *         the attention computation of prefill already produced it for the
 *         instruction tokens (Sec. 4.2.2 reuses that attention); then
 *         A_ri = exp(l_ri - lse[r]) and nothing is normalised here.  With
 *         the exact value this is the same softmax.
 * ---------------------------------------------------------------------- */
static void window_scores_unit(int32_t G, int32_t alpha, int32_t d, int32_t n,
                               const uint16_t *q, const uint16_t *k,
                               const double *lse, double *s_head,
                               double *s_mean) {
  const int32_t npre = n - alpha;
  const int32_t R = G * alpha;
  const double inv_sqrt_d = 1.0 / sqrt((double)d);
  /* A[r][i]: attention of query row r = h*alpha + t on key i (0 beyond p). */
  double *A = (double *)malloc(sizeof(double) * (size_t)R * (size_t)n);
#pragma omp parallel for schedule(dynamic, 1)
  for (int32_t r = 0; r < R; ++r) {
    const int32_t t = r % alpha;
    const int32_t p = npre + t; /* absolute position of this query */
    double *Ar = A + (size_t)r * n;
    const uint16_t *qr = q + (size_t)r * d;
    double mx = -INFINITY;
    for (int32_t i = 0; i <= p; ++i) {
      double dot = 0.0;
      for (int32_t c = 0; c < d; ++c)
        dot += bf16_to_f64(qr[c]) * bf16_to_f64(k[(size_t)i * d + c]);
      Ar[i] = dot * inv_sqrt_d;
      if (Ar[i] > mx) mx = Ar[i];
    }
    if (lse) {
      for (int32_t i = 0; i <= p; ++i) Ar[i] = exp(Ar[i] - lse[r]);
    } else {
      double Z = 0.0;
      for (int32_t i = 0; i <= p; ++i) {
        Ar[i] = exp(Ar[i] - mx);
        Z += Ar[i];
      }
      for (int32_t i = 0; i <= p; ++i) Ar[i] /= Z;
    }
    for (int32_t i = p + 1; i < n; ++i) Ar[i] = 0.0;
  }
  for (int32_t i = 0; i < npre; ++i) {
    double mean = 0.0;
    for (int32_t h = 0; h < G; ++h) {
      double sh = 0.0;
      for (int32_t t = 0; t < alpha; ++t)
        sh += A[(size_t)(h * alpha + t) * n + i];
      if (s_head) s_head[(size_t)h * npre + i] = sh;
      mean += sh;
    }
    s_mean[i] = mean / (double)G;
  }
  free(A);
}

/* Exported form of the above for stage-wise tests.  n > alpha >= 1. */
int pkvo_window_scores(int32_t G, int32_t alpha, int32_t d, int32_t n,
                       const uint16_t *q, const uint16_t *k, double *s_head,
                       double *s_mean) {
  if (G < 1 || alpha < 1 || d < 1 || n <= alpha || !q || !k || !s_mean)
    return 1;
  window_scores_unit(G, alpha, d, n, q, k, NULL, s_head, s_mean);
  return 0;
}

/* The same with the softmax denominators supplied: lse [G][alpha], fp64. */
int pkvo_window_scores_lse(int32_t G, int32_t alpha, int32_t d, int32_t n,
                           const uint16_t *q, const uint16_t *k,
                           const double *lse, double *s_head,
                           double *s_mean) {
  if (G < 1 || alpha < 1 || d < 1 || n <= alpha || !q || !k || !lse || !s_mean)
    return 1;
  window_scores_unit(G, alpha, d, n, q, k, lse, s_head, s_mean);
  return 0;
}

/* ------------------------------------------------------------------------
 * 1-D pooling of the prefix scores along the sequence ("a pooling layer",
 * Sec. 4.2.2): stride 1, same length, odd width w, half-width r=(w-1)/2.
 *   max: maximum over the in-range neighbours |u| <= r.
 *   avg: sum over the in-range neighbours divided by w (out-of-range
 *        neighbours count as zero).
 *   none, or w == 1: identity.
 * ---------------------------------------------------------------------- */
int pkvo_pool(int32_t pool, int32_t w, int32_t len, const double *s,
              double *p) {
  if (w < 1 || (w % 2) == 0 || len < 0) return 1;
  if (pool != PKVO_POOL_NONE && pool != PKVO_POOL_MAX && pool != PKVO_POOL_AVG)
    return 1;
  const int32_t r = (w - 1) / 2;
  for (int32_t i = 0; i < len; ++i) {
    if (pool == PKVO_POOL_NONE || w == 1) {
      p[i] = s[i];
    } else if (pool == PKVO_POOL_MAX) {
      double mx = -INFINITY;
      for (int32_t u = -r; u <= r; ++u)
        if (i + u >= 0 && i + u < len && s[i + u] > mx) mx = s[i + u];
      p[i] = mx;
    } else {
      double acc = 0.0;
      for (int32_t u = -r; u <= r; ++u)
        if (i + u >= 0 && i + u < len) acc += s[i + u];
      p[i] = acc / (double)w;
    }
  }
  return 0;
}

/* ------------------------------------------------------------------------
 * Top-kk of p[0..len) in the total order (value descending, index
 * ascending), returned sorted by ascending index (Sec. 4.2.2: "the top k^l
 * tokens with the highest scores are selected"; lower index wins ties).
 * ---------------------------------------------------------------------- */
typedef struct {
  double v;
  int32_t i;
} pkvo_pair;

static int cmp_value_desc_index_asc(const void *a, const void *b) {
  const pkvo_pair *x = (const pkvo_pair *)a, *y = (const pkvo_pair *)b;
  if (x->v > y->v) return -1;
  if (x->v < y->v) return 1;
  return (x->i > y->i) - (x->i < y->i);
}

static int cmp_int_asc(const void *a, const void *b) {
  int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
  return (x > y) - (x < y);
}

int pkvo_topk(int32_t len, const double *p, int32_t kk, int32_t *idx) {
  if (kk < 0 || kk > len) return 1;
  pkvo_pair *a = (pkvo_pair *)malloc(sizeof(pkvo_pair) * (size_t)(len + 1));
  for (int32_t i = 0; i < len; ++i) {
    a[i].v = p[i];
    a[i].i = i;
  }
  qsort(a, (size_t)len, sizeof(pkvo_pair), cmp_value_desc_index_asc);
  for (int32_t j = 0; j < kk; ++j) idx[j] = a[j].i;
  qsort(idx, (size_t)kk, sizeof(int32_t), cmp_int_asc);
  free(a);
  return 0;
}

/* ------------------------------------------------------------------------
 * One layer of compression for a (possibly ragged) batch.
 *
 * Contiguous layouts:
 *   Q_win [B][Hq][alpha][d]   bf16 bits; queries of the LAST alpha valid
 *                             tokens of each sequence
 *   K, V  [B][Hkv][N][d]      bf16 bits; rows >= seq_lens[b] are never read
 *   seq_lens [B] or NULL (all N)
 *   k_cap = min(k_l, N)
 *   K_out, V_out [B][Hkv][k_cap][d]   kept rows, bit copies; rest zero
 *   idx_out [B][Hkv][k_cap]           kept positions ascending, window
 *                                     last; rest -1
 *   count_out [B]                     min(k_l, n_b)
 *   pooled_out [B][Hkv][N] (optional) pooled scores of prefix keys; entries
 *                                     at i >= n_b - alpha, and everything
 *                                     when k_l >= n_b, are set to 0
 * Steps per sequence b (length n) and KV head g:
 *   1. k_l >= n: keep everything.
 *   2-4. window scores, sum over window, mean over group (above).
 *   5. pool.  6. top-(k_l - alpha) of the prefix, ascending, then the
 *   window positions n-alpha..n-1.  7. copy the kept K and V rows.
 * Returns 0, or 1 for invalid arguments.
 * ---------------------------------------------------------------------- */
static int compress_layer_impl(int32_t B, int32_t Hq, int32_t Hkv, int32_t d,
                               int32_t N, int32_t alpha, int32_t k_l,
                               int32_t pool, int32_t pool_w,
                               const uint16_t *Q_win, const uint16_t *K,
                               const uint16_t *V, const int32_t *seq_lens,
                               const float *lse, uint16_t *K_out,
                               uint16_t *V_out, int32_t *idx_out,
                               int32_t *count_out, double *pooled_out) {
  if (B < 1 || Hq < 1 || Hkv < 1 || Hq % Hkv || d < 1 || N < 1 || alpha < 1 ||
      k_l < alpha || pool_w < 1 || (pool_w % 2) == 0)
    return 1;
  if (pool != PKVO_POOL_NONE && pool != PKVO_POOL_MAX && pool != PKVO_POOL_AVG)
    return 1;
  const int32_t G = Hq / Hkv;
  const int32_t k_cap = k_l < N ? k_l : N;
  for (int32_t b = 0; b < B; ++b) {
    if (seq_lens && (seq_lens[b] < 0 || seq_lens[b] > N)) return 1;
  }
  for (int32_t b = 0; b < B; ++b) {
    const int32_t n = seq_lens ? seq_lens[b] : N;
    const int32_t count = k_l < n ? k_l : n;
    count_out[b] = count;
    for (int32_t g = 0; g < Hkv; ++g) {
      const size_t unit = (size_t)b * Hkv + g;
      const uint16_t *Kg = K + unit * (size_t)N * d;
      const uint16_t *Vg = V + unit * (size_t)N * d;
      int32_t *idx = idx_out + unit * (size_t)k_cap;
      uint16_t *Ko = K_out + unit * (size_t)k_cap * d;
      uint16_t *Vo = V_out + unit * (size_t)k_cap * d;
      double *po = pooled_out ? pooled_out + unit * (size_t)N : NULL;
      if (po)
        for (int32_t i = 0; i < N; ++i) po[i] = 0.0;
      if (k_l >= n) {
        for (int32_t j = 0; j < n; ++j) idx[j] = j;
      } else {
        const int32_t npre = n - alpha;
        const uint16_t *qg =
            Q_win + ((size_t)b * Hq + (size_t)g * G) * (size_t)alpha * d;
        double *s = (double *)malloc(sizeof(double) * (size_t)npre);
        double *p = (double *)malloc(sizeof(double) * (size_t)npre);
        double *lg = NULL;
        if (lse) { /* rows (b, g*G + h, t) of lse [B][Hq][alpha], fp32 */
          lg = (double *)malloc(sizeof(double) * (size_t)G * alpha);
          for (int32_t r = 0; r < G * alpha; ++r)
            lg[r] = (double)lse[((size_t)b * Hq + (size_t)g * G) * alpha + r];
        }
        window_scores_unit(G, alpha, d, n, qg, Kg, lg, NULL, s);
        free(lg);
        pkvo_pool(pool, pool_w, npre, s, p);
        pkvo_topk(npre, p, k_l - alpha, idx);
        for (int32_t t = 0; t < alpha; ++t) idx[k_l - alpha + t] = npre + t;
        if (po) memcpy(po, p, sizeof(double) * (size_t)npre);
        free(s);
        free(p);
      }
      for (int32_t j = 0; j < k_cap; ++j) {
        if (j < count) {
          memcpy(Ko + (size_t)j * d, Kg + (size_t)idx[j] * d,
                 sizeof(uint16_t) * (size_t)d);
          memcpy(Vo + (size_t)j * d, Vg + (size_t)idx[j] * d,
                 sizeof(uint16_t) * (size_t)d);
        } else {
          idx[j] = -1;
          memset(Ko + (size_t)j * d, 0, sizeof(uint16_t) * (size_t)d);
          memset(Vo + (size_t)j * d, 0, sizeof(uint16_t) * (size_t)d);
        }
      }
    }
  }
  return 0;
}

int pkvo_compress_layer(int32_t B, int32_t Hq, int32_t Hkv, int32_t d,
                        int32_t N, int32_t alpha, int32_t k_l, int32_t pool,
                        int32_t pool_w, const uint16_t *Q_win,
                        const uint16_t *K, const uint16_t *V,
                        const int32_t *seq_lens, uint16_t *K_out,
                        uint16_t *V_out, int32_t *idx_out, int32_t *count_out,
                        double *pooled_out) {
  return compress_layer_impl(B, Hq, Hkv, d, N, alpha, k_l, pool, pool_w, Q_win,
                             K, V, seq_lens, NULL, K_out, V_out, idx_out,
                             count_out, pooled_out);
}

/* The same layer with caller-supplied softmax denominators:
 *   lse : [B][Hq][alpha] fp32, lse[b][h][t] = ln sum_{i <= n_b-alpha+t}
 *         exp(q_{h,t} . k_i / sqrt(d)) of sequence b (entries of sequences
 *         that keep everything are not read). */
int pkvo_compress_layer_lse(int32_t B, int32_t Hq, int32_t Hkv, int32_t d,
                            int32_t N, int32_t alpha, int32_t k_l,
                            int32_t pool, int32_t pool_w,
                            const uint16_t *Q_win, const uint16_t *K,
                            const uint16_t *V, const int32_t *seq_lens,
                            const float *lse, uint16_t *K_out, uint16_t *V_out,
                            int32_t *idx_out, int32_t *count_out,
                            double *pooled_out) {
  if (!lse) return 1;
  return compress_layer_impl(B, Hq, Hkv, d, N, alpha, k_l, pool, pool_w, Q_win,
                             K, V, seq_lens, lse, K_out, V_out, idx_out,
                             count_out, pooled_out);
}

/* ------------------------------------------------------------------------
 * Attention recall rate (appendix, "Attention Recall Rate Experiment"): the
 * share of a query's attention over all keys that falls on the keys kept.
 * For one sequence of n tokens and one KV head with its G query heads:
 *   recall = mean over the G*alpha window queries r of
 *            sum_{i in kept, i <= p_r} A_ri ,   A = causal softmax as above
 * (the attention over all visible keys sums to 1, so the ratio is the kept
 * mass).  kept: `count` positions, any order, each < n.
 * ---------------------------------------------------------------------- */
int pkvo_attention_recall(int32_t G, int32_t alpha, int32_t d, int32_t n,
                          const uint16_t *q, const uint16_t *k,
                          const int32_t *kept, int32_t count, double *recall) {
  if (G < 1 || alpha < 1 || d < 1 || n < alpha || !q || !k || !kept ||
      count < 0 || !recall)
    return 1;
  const int32_t R = G * alpha;
  const double inv_sqrt_d = 1.0 / sqrt((double)d);
  double *l = (double *)malloc(sizeof(double) * (size_t)n);
  double total = 0.0;
  for (int32_t r = 0; r < R; ++r) {
    const int32_t p = n - alpha + r % alpha;
    double mx = -INFINITY, Z = 0.0, keptmass = 0.0;
    for (int32_t i = 0; i <= p; ++i) {
      double dot = 0.0;
      for (int32_t c = 0; c < d; ++c)
        dot += bf16_to_f64(q[(size_t)r * d + c]) *
               bf16_to_f64(k[(size_t)i * d + c]);
      l[i] = dot * inv_sqrt_d;
      if (l[i] > mx) mx = l[i];
    }
    for (int32_t i = 0; i <= p; ++i) Z += exp(l[i] - mx);
    for (int32_t j = 0; j < count; ++j) {
      if (kept[j] < 0 || kept[j] >= n) {
        free(l);
        return 1;
      }
      if (kept[j] <= p) keptmass += exp(l[kept[j]] - mx) / Z;
    }
    total += keptmass;
  }
  *recall = total / (double)R;
  free(l);
  return 0;
}

/* ------------------------------------------------------------------------
 * Per-layer paged output (appendix "PyramidKV Implementation at vLLM": every
 * layer has its own block table, because every layer keeps a different number
 * of tokens).  The kept rows of sequence b (K_out / V_out of
 * pkvo_compress_layer, rows 0 .. count_b-1) are written to the layer's page
 * pool:
 *   row j of KV head g  ->  page table[b][j / P], head g, slot j % P
 *   K_pages, V_pages : [num_pages][Hkv][P][d], only the kept rows are written
 *   table            : [B][max_pages] page numbers
 * Returns 0; 1 for invalid arguments; 2 if a needed table entry is outside
 * [0, num_pages) or the table is too short (nothing is written then).
 * ---------------------------------------------------------------------- */
int pkvo_scatter_pages(int32_t B, int32_t Hkv, int32_t d, int32_t k_cap,
                       int32_t P, int32_t num_pages, int32_t max_pages,
                       const uint16_t *K_out, const uint16_t *V_out,
                       const int32_t *count, const int32_t *table,
                       uint16_t *K_pages, uint16_t *V_pages) {
  if (B < 1 || Hkv < 1 || d < 1 || k_cap < 1 || P < 1 || num_pages < 1 ||
      max_pages < 1 || !K_out || !V_out || !count || !table || !K_pages ||
      !V_pages)
    return 1;
  for (int32_t b = 0; b < B; ++b) {
    if (count[b] < 0 || count[b] > k_cap) return 1;
    const int32_t need = (count[b] + P - 1) / P;
    if (need > max_pages) return 2;
    for (int32_t q = 0; q < need; ++q) {
      const int32_t pg = table[(size_t)b * max_pages + q];
      if (pg < 0 || pg >= num_pages) return 2;
    }
  }
  for (int32_t b = 0; b < B; ++b)
    for (int32_t g = 0; g < Hkv; ++g)
      for (int32_t j = 0; j < count[b]; ++j) {
        const int32_t pg = table[(size_t)b * max_pages + j / P];
        const size_t src = (((size_t)b * Hkv + g) * k_cap + j) * (size_t)d;
        const size_t dst =
            ((((size_t)pg * Hkv + g) * P) + (size_t)(j % P)) * (size_t)d;
        memcpy(K_pages + dst, K_out + src, sizeof(uint16_t) * (size_t)d);
        memcpy(V_pages + dst, V_out + src, sizeof(uint16_t) * (size_t)d);
      }
  return 0;
}

/* ------------------------------------------------------------------------
 * The step after the path: one decoding query per sequence attends over the
 * compacted cache of a layer (Sec. 3: after compression the model attends
 * over K_s, V_s only; the kept rows carry the rotary phases of their original
 * positions, so nothing is re-rotated).  For sequence b, query head h of KV
 * head g = h / G and the count_b kept rows:
 *   out[b][h] = sum_j softmax_j(q_bh . K_s[b][g][j] / sqrt(d)) V_s[b][g][j]
 *   lse[b][h] = ln sum_j exp(q_bh . K_s[b][g][j] / sqrt(d))   (may be NULL)
 * count_b = 0 gives a zero row and lse = -inf.
 *   q : [B][Hq][d] bf16;  K_s, V_s : [B][Hkv][k_cap][d] bf16;  out: fp64.
 * ---------------------------------------------------------------------- */
int pkvo_decode_attention(int32_t B, int32_t Hq, int32_t Hkv, int32_t d,
                          int32_t k_cap, const uint16_t *q,
                          const uint16_t *Ks, const uint16_t *Vs,
                          const int32_t *count, double *out, double *lse) {
  if (B < 1 || Hq < 1 || Hkv < 1 || Hq % Hkv || d < 1 || k_cap < 1 || !q ||
      !Ks || !Vs || !count || !out)
    return 1;
  const int32_t G = Hq / Hkv;
  const double inv_sqrt_d = 1.0 / sqrt((double)d);
  for (int32_t b = 0; b < B; ++b)
    if (count[b] < 0 || count[b] > k_cap) return 1;
  for (int32_t b = 0; b < B; ++b)
    for (int32_t h = 0; h < Hq; ++h) {
      const int32_t g = h / G, n = count[b];
      const uint16_t *qr = q + ((size_t)b * Hq + h) * d;
      const uint16_t *Kg = Ks + ((size_t)b * Hkv + g) * (size_t)k_cap * d;
      const uint16_t *Vg = Vs + ((size_t)b * Hkv + g) * (size_t)k_cap * d;
      double *o = out + ((size_t)b * Hq + h) * d;
      double *l = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
      double mx = -INFINITY, Z = 0.0;
      for (int32_t j = 0; j < n; ++j) {
        double dot = 0.0;
        for (int32_t c = 0; c < d; ++c)
          dot += bf16_to_f64(qr[c]) * bf16_to_f64(Kg[(size_t)j * d + c]);
        l[j] = dot * inv_sqrt_d;
        if (l[j] > mx) mx = l[j];
      }
      for (int32_t j = 0; j < n; ++j) Z += exp(l[j] - mx);
      for (int32_t c = 0; c < d; ++c) o[c] = 0.0;
      for (int32_t j = 0; j < n; ++j) {
        const double p = exp(l[j] - mx) / Z;
        for (int32_t c = 0; c < d; ++c)
          o[c] += p * bf16_to_f64(Vg[(size_t)j * d + c]);
      }
      if (lse) lse[(size_t)b * Hq + h] = n > 0 ? mx + log(Z) : -INFINITY;
      free(l);
    }
  return 0;
}

/* Number of OpenMP threads the scoring loop will use (for reports). */
int pkvo_num_threads(void) {
#ifdef _OPENMP
  extern int omp_get_max_threads(void);
  return omp_get_max_threads();
#else
  return 1;
#endif
}
