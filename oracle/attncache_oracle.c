/*
 * CPU oracle for the AttnCache hot path.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain definition that the GPU library is checked
 * against.  Only the test-suite, the smoke check and the benchmark's
 * cpu_baseline leg may load it; the product path never does.  It shares no
 * code, header, table or helper with the HIP sources.
 *
 * Conventions
 *   - every floating-point input arrives as IEEE binary32 (`float`) holding
 *     the exact value of the stored fp16 / bf16 / fp32 element; it is widened
 *     to `double` before any arithmetic and all sums are carried in `double`;
 *   - outputs are `double` (unrounded) unless the paper's step is itself a
 *     rounding (search scores are reported in binary32; stored maps are
 *     rounded to their storage type by oracle_round_maps);
 *   - loops are written in the order of the definitions, no blocking, no
 *     fusion; the only parallelism is an OpenMP split over independent
 *     outputs (queries, or (batch, head) tiles), which changes no sum order.
 *
 * What each routine follows in the paper (AttnCache, arXiv 2510.25979):
 *   oracle_search           Algorithm 1, the VecDB.search step and the
 *                           "similarity not less than theta" test (Sec. 3.1,
 *                           "Search Engine"); exact k-nearest search stands
 *                           in for the approximate index the paper uses.
 *   oracle_apply            Algorithm 2, reuse branch: mat_mul(attn_map, v).
 *   oracle_attention_exact  Algorithm 2, recompute branch, with
 *                           AttnMaps = softmax(Q K^T / sqrt(d_k)) from the
 *                           equation in Sec. 4 ("Applicability").
 *   oracle_round_maps       the storage step of database building (Fig. 3,
 *                           step 3): a computed map is rounded once to the
 *                           database's element type.
 *   oracle_project          Algorithm 1, the feature_projector step: the
 *                           two-layer MLP of Sec. 3.1 ("Feature Projector")
 *                           on the mean-pooled hidden states.
 *
 * Parity pins: every routine here is pinned by the CPU tests (closed forms,
 * invariants, brute force, library cross-checks).  None is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_OK 0
#define ORACLE_ERR_ARG -1
#define ORACLE_ERR_INDEX -2
#define ORACLE_ERR_NOMEM -3

#define ORACLE_METRIC_IP 0
#define ORACLE_METRIC_L2 1

#define ORACLE_ROUND_F32 0
#define ORACLE_ROUND_BF16 1

/* ------------------------------------------------------------------ search */

/* Total order used for ranking: higher score first, then lower index. */
static int ranks_before(float sa, int32_t ia, float sb, int32_t ib) {
  if (sa > sb) return 1;
  if (sa < sb) return 0;
  return ia < ib;
}

/*
 * Exact top-k similarity search with threshold routing.
 *
 *   q       [B][E]   query feature vectors
 *   emb     [N][E]   database feature vectors
 *   map_of  [N] or NULL   attention-map entry that database row n refers to
 *                         (NULL = identity: both stores share one index)
 *   metric  IP: s = <q, e>;  L2: s = -||q - e||^2
 *   idx     [B][k]   row indices, ranked (score descending, index ascending)
 *   score   [B][k]   the fp64 score rounded once to binary32
 *   hit     [B]      map entry of the best row if its similarity >= theta,
 *                    else -1.  Similarity is the score itself for IP and
 *                    1 - ||q - e|| for L2 (distance turned into a similarity).
 *
 * The comparison against theta is taken in binary32 on the rounded score,
 * the precision in which scores are reported.
 */
int32_t oracle_search(const float *q, const float *emb, const int32_t *map_of,
                      int32_t B, int32_t N, int32_t E, int32_t k, float theta,
                      int32_t metric, int32_t *idx, float *score,
                      int32_t *hit) {
  if (!q || !emb || !idx || !score || !hit) return ORACLE_ERR_ARG;
  if (B < 0 || N < 1 || E < 1 || k < 1 || k > N) return ORACLE_ERR_ARG;
  if (metric != ORACLE_METRIC_IP && metric != ORACLE_METRIC_L2)
    return ORACLE_ERR_ARG;
  int32_t status = ORACLE_OK;

#pragma omp parallel for schedule(dynamic, 1)
  for (int32_t b = 0; b < B; ++b) {
    float *s = (float *)malloc((size_t)N * sizeof(float));
    uint8_t *taken = (uint8_t *)calloc((size_t)N, 1);
    if (!s || !taken) {
      free(s);
      free(taken);
#pragma omp atomic write
      status = ORACLE_ERR_NOMEM;
      continue;
    }
    /* all N scores, each a plain left-to-right fp64 sum */
    for (int32_t n = 0; n < N; ++n) {
      double acc = 0.0;
      for (int32_t e = 0; e < E; ++e) {
        double qv = (double)q[(size_t)b * E + e];
        double ev = (double)emb[(size_t)n * E + e];
        if (metric == ORACLE_METRIC_IP) {
          acc += qv * ev;
        } else {
          double d = qv - ev;
          acc -= d * d;
        }
      }
      s[n] = (float)acc;
    }
    /* k passes of selection under the total order (brute force) */
    for (int32_t r = 0; r < k; ++r) {
      int32_t best = -1;
      for (int32_t n = 0; n < N; ++n) {
        if (taken[n]) continue;
        if (best < 0 || ranks_before(s[n], n, s[best], best)) best = n;
      }
      taken[best] = 1;
      idx[(size_t)b * k + r] = best;
      score[(size_t)b * k + r] = s[best];
    }
    /* routing: reuse only if the best similarity is not less than theta */
    {
      int32_t top = idx[(size_t)b * k];
      float sim = score[(size_t)b * k];
      if (metric == ORACLE_METRIC_L2) sim = 1.0f - sqrtf(-sim);
      hit[b] = (sim >= theta) ? (map_of ? map_of[top] : top) : -1;
    }
    free(s);
    free(taken);
  }
  return status;
}

/* ------------------------------------------------------------------- apply */

/*
 * Reuse branch: O[b][l][h] = A[hit[b]][layer_begin + l][h] . V[b][l][h / g].
 *
 *   maps  [M][L][Hq][S][S]   row-stochastic maps, one entry per database item
 *   hit   [B]                entry per query, -1 = miss (O[b] is not written)
 *   V     [B][Lc][Hkv][S][D]
 *   O     [B][Lc][Hq][S][D]  fp64, unrounded
 *   g = Hq / Hkv query heads share one value head (contiguous groups).
 *
 * The sum runs over every column j of the map, so a map with mass above the
 * diagonal is not silently treated as causal.
 */
int32_t oracle_apply(const float *maps, const int32_t *hit, const float *V,
                     double *O, int32_t B, int32_t M, int32_t L,
                     int32_t layer_begin, int32_t Lc, int32_t Hq, int32_t Hkv,
                     int32_t S, int32_t D) {
  if (!maps || !hit || !V || !O) return ORACLE_ERR_ARG;
  if (B < 0 || M < 1 || L < 1 || Lc < 0 || layer_begin < 0 ||
      layer_begin + Lc > L || Hq < 1 || Hkv < 1 || Hq % Hkv != 0 || S < 1 ||
      D < 1)
    return ORACLE_ERR_ARG;
  for (int32_t b = 0; b < B; ++b)
    if (hit[b] < -1 || hit[b] >= M) return ORACLE_ERR_INDEX;
  const int32_t g = Hq / Hkv;
  const int64_t tiles = (int64_t)B * Lc * Hq;

#pragma omp parallel for schedule(static)
  for (int64_t t = 0; t < tiles; ++t) {
    int32_t h = (int32_t)(t % Hq);
    int32_t l = (int32_t)((t / Hq) % Lc);
    int32_t b = (int32_t)(t / ((int64_t)Hq * Lc));
    if (hit[b] < 0) continue;
    const float *A = maps + ((((size_t)hit[b] * L + (size_t)(layer_begin + l)) *
                              Hq + h) * S) * S;
    const float *Vt = V + ((((size_t)b * Lc + l) * Hkv + h / g) * S) * D;
    double *Ot = O + ((((size_t)b * Lc + l) * Hq + h) * S) * D;
    for (int32_t i = 0; i < S; ++i)
      for (int32_t d = 0; d < D; ++d) {
        double acc = 0.0;
        for (int32_t j = 0; j < S; ++j)
          acc += (double)A[(size_t)i * S + j] * (double)Vt[(size_t)j * D + d];
        Ot[(size_t)i * D + d] = acc;
      }
  }
  return ORACLE_OK;
}

/* --------------------------------------------------------- exact attention */

/*
 * Recompute branch: P = softmax(scale * Q K^T) row by row (keys j > i are
 * excluded when causal, keys at or beyond the sentence's length always),
 * O = P V.
 *
 *   Q [B][Hq][S][D], K and V [B][Hkv][S][D], O [B][Hq][S][D] (fp64)
 *   P        NULL, or [B][Hq][S][S] fp64: the attention map itself, with
 *            exact zeros at excluded positions
 *   row_sel  NULL, or [B]: batch items with row_sel[b] >= 0 are skipped
 *            (they were served by the reuse branch); their O / P are not
 *            written
 *   key_len  NULL, or [B]: number of real tokens of sentence b in a batch
 *            padded on the right to S (1 <= key_len[b] <= S).  Keys
 *            j >= key_len[b] are padding and excluded for every row, the
 *            attention mask of a padded batch.  Rows i >= key_len[b] are
 *            padding themselves; they are computed by the same rule.
 *   scale    0 selects 1/sqrt(D)
 *
 * The row maximum is subtracted before exponentiation; this leaves the
 * quotient unchanged and keeps exp() in range.
 */
int32_t oracle_attention_exact(const float *Q, const float *K, const float *V,
                               double *O, double *P, const int32_t *row_sel,
                               const int32_t *key_len, int32_t B, int32_t Hq,
                               int32_t Hkv, int32_t S, int32_t D,
                               int32_t causal, double scale) {
  if (!Q || !K || !V || !O) return ORACLE_ERR_ARG;
  if (B < 0 || Hq < 1 || Hkv < 1 || Hq % Hkv != 0 || S < 1 || D < 1)
    return ORACLE_ERR_ARG;
  for (int32_t b = 0; key_len && b < B; ++b)
    if (key_len[b] < 1 || key_len[b] > S) return ORACLE_ERR_INDEX;
  if (scale == 0.0) scale = 1.0 / sqrt((double)D);
  const int32_t g = Hq / Hkv;
  const int64_t tiles = (int64_t)B * Hq;
  int32_t status = ORACLE_OK;

#pragma omp parallel for schedule(static)
  for (int64_t t = 0; t < tiles; ++t) {
    int32_t h = (int32_t)(t % Hq);
    int32_t b = (int32_t)(t / Hq);
    if (row_sel && row_sel[b] >= 0) continue;
    const float *Qt = Q + (((size_t)b * Hq + h) * S) * D;
    const float *Kt = K + (((size_t)b * Hkv + h / g) * S) * D;
    const float *Vt = V + (((size_t)b * Hkv + h / g) * S) * D;
    double *Ot = O + (((size_t)b * Hq + h) * S) * D;
    double *Pt = P ? P + (((size_t)b * Hq + h) * S) * S : NULL;
    double *p = (double *)malloc((size_t)S * sizeof(double));
    if (!p) {
#pragma omp atomic write
      status = ORACLE_ERR_NOMEM;
      continue;
    }
    for (int32_t i = 0; i < S; ++i) {
      const int32_t len = key_len ? key_len[b] : S;
      int32_t nj = causal ? i + 1 : S;
      if (nj > len) nj = len;
      double m = -INFINITY;
      for (int32_t j = 0; j < nj; ++j) {
        double acc = 0.0;
        for (int32_t d = 0; d < D; ++d)
          acc += (double)Qt[(size_t)i * D + d] * (double)Kt[(size_t)j * D + d];
        p[j] = scale * acc;
        if (p[j] > m) m = p[j];
      }
      double z = 0.0;
      for (int32_t j = 0; j < nj; ++j) {
        p[j] = exp(p[j] - m);
        z += p[j];
      }
      for (int32_t j = 0; j < nj; ++j) p[j] /= z;
      for (int32_t j = nj; j < S; ++j) p[j] = 0.0;
      if (Pt) memcpy(Pt + (size_t)i * S, p, (size_t)S * sizeof(double));
      for (int32_t d = 0; d < D; ++d) {
        double acc = 0.0;
        for (int32_t j = 0; j < nj; ++j)
          acc += p[j] * (double)Vt[(size_t)j * D + d];
        Ot[(size_t)i * D + d] = acc;
      }
    }
    free(p);
  }
  return status;
}

/* ------------------------------------------------------ map storage rounding */

/* Round-to-nearest-even of a double onto the bfloat16 grid (8-bit
 * significand, binary32 exponent range), done directly so no double
 * rounding through binary32 can occur. */
static double round_to_bf16(double x) {
  if (x == 0.0 || isnan(x) || isinf(x)) return x;
  int e = ilogb(x);
  if (e < -126) e = -126;           /* subnormal range: fixed quantum */
  double quantum = ldexp(1.0, e - 7); /* spacing of bf16 values in [2^e, 2^(e+1)) */
  double r = nearbyint(x / quantum) * quantum; /* default mode: ties to even */
  if (fabs(r) > 0x1.FEp127) r = copysign(INFINITY, x);
  return r;
}

/*
 * Storage step of database building: each map element is rounded once to the
 * database element type and handed back as binary32 (which represents every
 * bf16 and fp32 value exactly).
 */
int32_t oracle_round_maps(const double *P, float *out, int64_t count,
                          int32_t kind) {
  if (!P || !out || count < 0) return ORACLE_ERR_ARG;
  if (kind != ORACLE_ROUND_F32 && kind != ORACLE_ROUND_BF16)
    return ORACLE_ERR_ARG;
  for (int64_t i = 0; i < count; ++i)
    out[i] = (kind == ORACLE_ROUND_BF16) ? (float)round_to_bf16(P[i])
                                         : (float)P[i];
  return ORACLE_OK;
}

/* --------------------------------------------------------- feature projector */

/*
 * Algorithm 1, the feature_projector step: the input embedding h of a
 * sentence (its hidden states, one row of width dm per token) becomes the
 * feature vector that is searched for.  Sec. 3.1 ("Feature Projector") fixes
 * the network as two MLP layers that lower the dimension; it does not print
 * the pooling, the activation or the normalisation, so this oracle states the
 * reading the GPU library documents:
 *
 *   x[i]   = (1 / s) * sum_{t < s} h[t][i]                 mean over the s valid tokens
 *   u[j]   = max(0, b1[j] + sum_i W1[j][i] * x[i])         first layer, ReLU
 *   f[e]   = b2[e] + sum_j W2[e][j] * u[j]                 second layer
 *   f      = f / ||f||_2  if normalize (left as is when the norm is 0)
 *
 * h[B][S][dm], seq_len[B] (NULL: every sentence has S tokens), W1[hid][dm],
 * b1[hid] (NULL: zeros), W2[E][hid], b2[E] (NULL: zeros), out[B][E] double.
 */
int32_t oracle_project(const float *h, const int32_t *seq_len, const float *W1,
                       const float *b1, const float *W2, const float *b2,
                       double *out, int32_t B, int32_t S, int32_t dm,
                       int32_t hid, int32_t E, int32_t normalize) {
  if (!h || !W1 || !W2 || !out) return ORACLE_ERR_ARG;
  if (B < 0 || S <= 0 || dm <= 0 || hid <= 0 || E <= 0) return ORACLE_ERR_ARG;
  for (int32_t b = 0; b < B; ++b)
    if (seq_len && (seq_len[b] < 1 || seq_len[b] > S)) return ORACLE_ERR_INDEX;
  int32_t status = ORACLE_OK;
#pragma omp parallel for schedule(static)
  for (int32_t b = 0; b < B; ++b) {
    double *x = (double *)malloc(sizeof(double) * (size_t)dm);
    double *u = (double *)malloc(sizeof(double) * (size_t)hid);
    if (!x || !u) {
      status = ORACLE_ERR_NOMEM;
    } else {
      const int32_t s = seq_len ? seq_len[b] : S;
      for (int32_t i = 0; i < dm; ++i) {
        double sum = 0.0;
        for (int32_t t = 0; t < s; ++t)
          sum += (double)h[((size_t)b * S + t) * dm + i];
        x[i] = sum / (double)s;
      }
      for (int32_t j = 0; j < hid; ++j) {
        double sum = b1 ? (double)b1[j] : 0.0;
        for (int32_t i = 0; i < dm; ++i)
          sum += (double)W1[(size_t)j * dm + i] * x[i];
        u[j] = sum > 0.0 ? sum : 0.0;
      }
      double norm2 = 0.0;
      for (int32_t e = 0; e < E; ++e) {
        double sum = b2 ? (double)b2[e] : 0.0;
        for (int32_t j = 0; j < hid; ++j)
          sum += (double)W2[(size_t)e * hid + j] * u[j];
        out[(size_t)b * E + e] = sum;
        norm2 += sum * sum;
      }
      if (normalize && norm2 > 0.0) {
        const double inv = 1.0 / sqrt(norm2);
        for (int32_t e = 0; e < E; ++e) out[(size_t)b * E + e] *= inv;
      }
    }
    free(x);
    free(u);
  }
  return status;
}

/* Number of OpenMP threads a parallel region will use (1 without OpenMP);
 * the benchmark reports it next to the oracle timing. */
#ifdef _OPENMP
#include <omp.h>
int32_t oracle_threads(void) { return (int32_t)omp_get_max_threads(); }
#else
int32_t oracle_threads(void) { return 1; }
#endif
