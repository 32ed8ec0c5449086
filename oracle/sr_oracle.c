/*
 * CPU oracle for SinkRouter's routed single-token decode attention.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, fp64 statement of
 * what the hot path computes; the tests, the smoke check and the benchmark's
 * cpu_baseline leg call it.  The product library never links, loads or calls
 * anything in this directory, and this file shares no code with the HIP path.
 *
 * What is written out here, with the passage of the paper each part follows:
 *   - head update u = sum_i alpha_i v_i, alpha = softmax of the scaled
 *     query-key scores                                   (Section 3, Eq. 1)
 *   - per-head routing signal s_{g,i} = cos(q_{g,i}, K_0) (Section 4.2, Eq. 11)
 *   - group score S_g = mean over the r heads of the group (Section 4.2, Eq. 12)
 *   - Sink Group iff S_g > tau(L), strict                 (Section 4.2, Eq. 13)
 *   - tau(x) = a x^3 + b x^2 + c x + d, x = L / len_norm  (Appendix A)
 *   - Sink Groups output zero for all r heads             (Section 4.2, Eq. 14)
 *   - Active Groups: exact standard attention over the available cache
 *                                                         (Section 4.2, last paragraph)
 *   - concentration statistics alpha_0, max and mean of the other weights
 *                                                         (Section 3, Table 1)
 *   - Split-K over [chunk_start, chunk_end) with a max / sum / weighted-sum
 *     partial per chunk, merged afterwards                (Section 4.3, Split-K paragraph;
 *     the paper does not print the merge, the standard log-sum-exp merge is used)
 *
 * Readings where the paper is silent:
 *   softmax scale defaults to 1/sqrt(D); seq_lens[b] counts valid cache rows
 *   including the current token; token 0 is row 0 of the cache of that
 *   (sequence, KV group); a zero norm makes the cosine 0; a NaN score keeps
 *   the group active; seq_len 0 gives zero output and mask 0; the cached
 *   anchor norm, when supplied, replaces the recomputed one.
 *
 * Inputs are bf16 bit patterns (uint16); bf16 -> double is exact, so every
 * input value is the one the GPU sees.  All arithmetic is fp64, in the order
 * of the definitions: no blocking, no fusion, no online softmax in the
 * single-pass entry.
 *
 * Pins (tests/test_oracle_*.py): brute force against numpy/scipy library
 * softmax with explicit KV repetition, closed forms, hand-computed fixtures
 * under tests/golden/, Split-K == single pass, decision special cases,
 * invariances, and the Eq. 4 bound.  Exact values of S_g closer to tau than
 * 1e-4 are "parity unpinned" (fp32 summation order on the GPU is free).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct sr_oracle_cfg {
  int32_t batch;           /* B */
  int32_t n_q_heads;       /* H_q */
  int32_t n_kv_heads;      /* H_kv, divides H_q */
  int32_t head_dim;        /* D, any positive value */
  int32_t max_seq_len;     /* token stride of the caches */
  int32_t routing_enabled; /* 0: every group is active */
  int32_t want_dense;      /* 1: also fill dense_out/alpha0/lse for skipped groups */
  int32_t reserved;
  double sm_scale;         /* 0 => 1/sqrt(D) */
  double tau_coef[4];      /* a, b, c, d */
  double len_norm;         /* x = L / len_norm; 0 => x = 0 */
} sr_oracle_cfg;

static double bf16_to_double(uint16_t h) {
  uint32_t u = ((uint32_t)h) << 16;
  float f;
  memcpy(&f, &u, sizeof f);
  return (double)f;
}

static double scale_of(const sr_oracle_cfg* c) {
  return c->sm_scale != 0.0 ? c->sm_scale : 1.0 / sqrt((double)c->head_dim);
}

static int32_t clamp_len(int32_t L, int32_t Lmax) {
  if (L < 0) return 0;
  if (L > Lmax) return Lmax;
  return L;
}

/* tau(L) of Appendix A: cubic in the normalised length. */
static double tau_of(const sr_oracle_cfg* c, int32_t L) {
  double x = c->len_norm > 0.0 ? (double)L / c->len_norm : 0.0;
  const double* t = c->tau_coef;
  return t[0] * x * x * x + t[1] * x * x + t[2] * x + t[3];
}

/* Eq. 11: cosine between one query head and the anchor key. */
static double cosine_to_anchor(const uint16_t* q, const uint16_t* k0, int D,
                               double anchor_norm /* <0: recompute */) {
  double dot = 0.0, nq = 0.0, nk = 0.0;
  for (int d = 0; d < D; ++d) {
    double a = bf16_to_double(q[d]), b = bf16_to_double(k0[d]);
    dot += a * b;
    nq += a * a;
    nk += b * b;
  }
  nq = sqrt(nq);
  nk = anchor_norm >= 0.0 ? anchor_norm : sqrt(nk);
  double den = nq * nk;
  if (!(den > 0.0)) return 0.0;
  return dot / den;
}

/* Eq. 1 for one head over tokens [t0, t1): returns max score m, sum l of
 * exp(z - m), and o[d] = sum exp(z_t - m) v_t[d].  Empty range: m = -inf,
 * l = 0, o = 0.  z is caller scratch of at least t1 - t0 doubles. */
static void head_partial(const uint16_t* q, const uint16_t* K, const uint16_t* V,
                         int D, double scale, int32_t t0, int32_t t1,
                         double* z, double* m_out, double* l_out, double* o) {
  for (int d = 0; d < D; ++d) o[d] = 0.0;
  if (t1 <= t0) { *m_out = -INFINITY; *l_out = 0.0; return; }
  double m = -INFINITY;
  for (int32_t t = t0; t < t1; ++t) {
    const uint16_t* kr = K + (size_t)t * D;
    double s = 0.0;
    for (int d = 0; d < D; ++d) s += bf16_to_double(q[d]) * bf16_to_double(kr[d]);
    s *= scale;
    z[t - t0] = s;
    if (s > m) m = s;
  }
  double l = 0.0;
  for (int32_t t = t0; t < t1; ++t) {
    double p = exp(z[t - t0] - m);
    l += p;
    const uint16_t* vr = V + (size_t)t * D;
    for (int d = 0; d < D; ++d) o[d] += p * bf16_to_double(vr[d]);
  }
  *m_out = m;
  *l_out = l;
}

/*
 * Routing only (Eq. 11-13).  All outputs optional except mask.  k0_rows (optional) overrides
 * the anchors read from row 0 of k_cache.
 *   head_cos    [B,H_q]   s_{g,i}
 *   group_score [B,H_kv]  S_g
 *   tau_out     [B]
 *   mask        [B,H_kv]  1 = Sink Group
 */
int sr_oracle_route(const uint16_t* q, const uint16_t* k_cache, const int32_t* seq_lens,
                    const double* k0_norm, const uint16_t* k0_rows, const sr_oracle_cfg* c,
                    double* head_cos, double* group_score, double* tau_out, uint8_t* mask) {
  if (!q || !k_cache || !seq_lens || !c || !mask) return -1;
  const int B = c->batch, Hq = c->n_q_heads, Hkv = c->n_kv_heads, D = c->head_dim;
  if (B < 1 || Hq < 1 || Hkv < 1 || D < 1 || Hq % Hkv != 0 || c->max_seq_len < 1) return -2;
  const int r = Hq / Hkv;
  for (int b = 0; b < B; ++b) {
    int32_t L = clamp_len(seq_lens[b], c->max_seq_len);
    double tau = tau_of(c, L);
    if (tau_out) tau_out[b] = tau;
    for (int g = 0; g < Hkv; ++g) {
      /* the anchor: row 0 of the group's key cache, or the separately cached K_0 [B,H_kv,D] (Section 4.3) */
      const uint16_t* k0 = k0_rows ? k0_rows + ((size_t)b * Hkv + g) * D
                                   : k_cache + ((size_t)b * Hkv + g) * (size_t)c->max_seq_len * D;
      double an = k0_norm ? k0_norm[b * Hkv + g] : -1.0;
      double S = 0.0;
      for (int i = 0; i < r; ++i) {
        const uint16_t* qh = q + ((size_t)b * Hq + (size_t)g * r + i) * D;
        double s = cosine_to_anchor(qh, k0, D, an);
        if (head_cos) head_cos[b * Hq + g * r + i] = s;
        S += s;
      }
      S /= (double)r;
      if (group_score) group_score[b * Hkv + g] = S;
      mask[b * Hkv + g] = (uint8_t)((c->routing_enabled && L > 0 && S > tau) ? 1 : 0);
    }
  }
  return 0;
}

/*
 * Full routed decode step.
 *   out       [B,H_q,D]  zeros for Sink Groups, exact attention otherwise
 *   dense_out [B,H_q,D]  optional: attention of every head, routing ignored
 *   alpha0    [B,H_q]    optional: softmax mass on token 0 (the target regime's alpha_0)
 *   lse       [B,H_q]    optional: log sum exp of the scaled scores
 * dense_out/alpha0/lse of skipped heads are filled only when want_dense != 0
 * (else NaN).  Returns 0, or a negative value for bad arguments.
 */
int sr_oracle_decode(const uint16_t* q, const uint16_t* k_cache, const uint16_t* v_cache,
                     const int32_t* seq_lens, const double* k0_norm, const uint16_t* k0_rows,
                     const sr_oracle_cfg* c,
                     double* out, uint8_t* mask, double* head_cos, double* group_score,
                     double* tau_out, double* dense_out, double* alpha0, double* lse) {
  if (!v_cache || !out) return -1;
  int rc = sr_oracle_route(q, k_cache, seq_lens, k0_norm, k0_rows, c, head_cos, group_score, tau_out, mask);
  if (rc) return rc;
  const int B = c->batch, Hq = c->n_q_heads, Hkv = c->n_kv_heads, D = c->head_dim;
  const int r = Hq / Hkv;
  const double scale = scale_of(c);
  const int32_t Lmax = c->max_seq_len;
  int failed = 0;
#pragma omp parallel
  {
    double* z = (double*)malloc(sizeof(double) * (size_t)Lmax);
    double* o = (double*)malloc(sizeof(double) * (size_t)D);
    if (!z || !o) {
#pragma omp atomic write
      failed = 1;
    }
#pragma omp for schedule(dynamic, 1)
    for (int bh = 0; bh < B * Hq; ++bh) {
      if (!z || !o) continue;
      const int b = bh / Hq, h = bh % Hq, g = h / r;
      const int32_t L = clamp_len(seq_lens[b], Lmax);
      const int skip = mask[b * Hkv + g];
      double* orow = out + (size_t)bh * D;
      double* drow = dense_out ? dense_out + (size_t)bh * D : NULL;
      if (skip && !c->want_dense) {
        for (int d = 0; d < D; ++d) orow[d] = 0.0;          /* Eq. 14 */
        if (drow) for (int d = 0; d < D; ++d) drow[d] = NAN;
        if (alpha0) alpha0[bh] = NAN;
        if (lse) lse[bh] = NAN;
        continue;
      }
      const uint16_t* qh = q + (size_t)bh * D;
      const uint16_t* K = k_cache + ((size_t)b * Hkv + g) * (size_t)Lmax * D;
      const uint16_t* V = v_cache + ((size_t)b * Hkv + g) * (size_t)Lmax * D;
      double m, l;
      head_partial(qh, K, V, D, scale, 0, L, z, &m, &l, o);
      for (int d = 0; d < D; ++d) {
        double u = (L > 0) ? o[d] / l : 0.0;                 /* Eq. 1 */
        if (drow) drow[d] = u;
        orow[d] = skip ? 0.0 : u;
      }
      if (alpha0) alpha0[bh] = (L > 0) ? exp(z[0] - m) / l : NAN;
      if (lse) lse[bh] = (L > 0) ? m + log(l) : -INFINITY;
    }
    free(z);
    free(o);
  }
  return failed ? -3 : 0;
}

/*
 * Same result as sr_oracle_decode, reached through Split-K partials: tokens
 * are cut at bounds[0] = 0 <= bounds[1] <= ... <= bounds[n_splits]; chunk j
 * is [bounds[j], bounds[j+1]) intersected with [0, L_b); each chunk yields
 * (m_j, l_j, o_j) and the merge is
 *     M = max_j m_j,  out = sum_j e^{m_j - M} o_j / sum_j e^{m_j - M} l_j,
 * empty chunks (m = -inf) contributing nothing.
 * Optional outputs part_m / part_l [B,H_q,n_splits] expose the partial stats.
 */
int sr_oracle_decode_splitk(const uint16_t* q, const uint16_t* k_cache, const uint16_t* v_cache,
                            const int32_t* seq_lens, const double* k0_norm, const uint16_t* k0_rows,
                            const sr_oracle_cfg* c, const int32_t* bounds, int32_t n_splits,
                            double* out, uint8_t* mask, double* part_m, double* part_l) {
  if (!v_cache || !out || !bounds || n_splits < 1) return -1;
  int rc = sr_oracle_route(q, k_cache, seq_lens, k0_norm, k0_rows, c, NULL, NULL, NULL, mask);
  if (rc) return rc;
  for (int j = 0; j < n_splits; ++j)
    if (bounds[j] > bounds[j + 1]) return -2;
  if (bounds[0] != 0) return -2;
  const int B = c->batch, Hq = c->n_q_heads, Hkv = c->n_kv_heads, D = c->head_dim;
  const int r = Hq / Hkv;
  const double scale = scale_of(c);
  const int32_t Lmax = c->max_seq_len;
  int failed = 0;
#pragma omp parallel
  {
    double* z = (double*)malloc(sizeof(double) * (size_t)Lmax);
    double* po = (double*)malloc(sizeof(double) * (size_t)D * (size_t)n_splits);
    double* pm = (double*)malloc(sizeof(double) * (size_t)n_splits);
    double* pl = (double*)malloc(sizeof(double) * (size_t)n_splits);
    if (!z || !po || !pm || !pl) {
#pragma omp atomic write
      failed = 1;
    }
#pragma omp for schedule(dynamic, 1)
    for (int bh = 0; bh < B * Hq; ++bh) {
      if (!z || !po || !pm || !pl) continue;
      const int b = bh / Hq, h = bh % Hq, g = h / r;
      const int32_t L = clamp_len(seq_lens[b], Lmax);
      double* orow = out + (size_t)bh * D;
      for (int d = 0; d < D; ++d) orow[d] = 0.0;
      if (mask[b * Hkv + g]) {
        for (int j = 0; j < n_splits; ++j) {
          if (part_m) part_m[(size_t)bh * n_splits + j] = NAN;
          if (part_l) part_l[(size_t)bh * n_splits + j] = NAN;
        }
        continue;
      }
      const uint16_t* qh = q + (size_t)bh * D;
      const uint16_t* K = k_cache + ((size_t)b * Hkv + g) * (size_t)Lmax * D;
      const uint16_t* V = v_cache + ((size_t)b * Hkv + g) * (size_t)Lmax * D;
      double M = -INFINITY;
      for (int j = 0; j < n_splits; ++j) {
        int32_t t0 = bounds[j] < L ? bounds[j] : L;
        int32_t t1 = bounds[j + 1] < L ? bounds[j + 1] : L;
        head_partial(qh, K, V, D, scale, t0, t1, z, &pm[j], &pl[j], po + (size_t)j * D);
        if (pm[j] > M) M = pm[j];
        if (part_m) part_m[(size_t)bh * n_splits + j] = pm[j];
        if (part_l) part_l[(size_t)bh * n_splits + j] = pl[j];
      }
      /* tokens at or beyond bounds[n_splits] are not covered by any chunk: the
       * caller is expected to pass bounds[n_splits] >= L. */
      if (!(M > -INFINITY)) continue; /* no tokens at all */
      double den = 0.0;
      for (int j = 0; j < n_splits; ++j) {
        if (!(pm[j] > -INFINITY)) continue;
        double w = exp(pm[j] - M);
        den += w * pl[j];
        for (int d = 0; d < D; ++d) orow[d] += w * po[(size_t)j * D + d];
      }
      for (int d = 0; d < D; ++d) orow[d] /= den;
    }
    free(z);
    free(po);
    free(pm);
    free(pl);
  }
  return failed ? -3 : 0;
}

/*
 * Attention-concentration statistics per head, the quantities of Table 1 (Section 3):
 * with alpha = softmax of the scaled scores over the whole cache (Eq. 1),
 *   alpha0    [B,H_q]  alpha_0, the weight of token 0
 *   max_rest  [B,H_q]  max over t >= 1 of alpha_t
 *   mean_rest [B,H_q]  (sum over t >= 1 of alpha_t) / (L - 1)
 *   out_rest  [B,H_q,D] optional: the head update with token 0 left out and the remaining
 *             weights renormalised, sum_{t>=1} alpha_t v_t / sum_{t>=1} alpha_t
 * Routing plays no part.  L = 1: max_rest = mean_rest = 0 and out_rest = 0; L = 0: NaN, out_rest = 0.
 */
int sr_oracle_concentration(const uint16_t* q, const uint16_t* k_cache, const uint16_t* v_cache,
                            const int32_t* seq_lens, const sr_oracle_cfg* c,
                            double* alpha0, double* max_rest, double* mean_rest, double* out_rest) {
  if (!q || !k_cache || !seq_lens || !c || !alpha0 || !max_rest || !mean_rest) return -1;
  if (out_rest && !v_cache) return -1;
  const int B = c->batch, Hq = c->n_q_heads, Hkv = c->n_kv_heads, D = c->head_dim;
  if (B < 1 || Hq < 1 || Hkv < 1 || D < 1 || Hq % Hkv != 0 || c->max_seq_len < 1) return -2;
  const int r = Hq / Hkv;
  const double scale = scale_of(c);
  const int32_t Lmax = c->max_seq_len;
  int failed = 0;
#pragma omp parallel
  {
    double* w = (double*)malloc(sizeof(double) * (size_t)Lmax);
    if (!w) {
#pragma omp atomic write
      failed = 1;
    }
#pragma omp for schedule(dynamic, 1)
    for (int bh = 0; bh < B * Hq; ++bh) {
      if (!w) continue;
      const int b = bh / Hq, h = bh % Hq, g = h / r;
      const int32_t L = clamp_len(seq_lens[b], Lmax);
      double* orow = out_rest ? out_rest + (size_t)bh * D : NULL;
      if (orow) for (int d = 0; d < D; ++d) orow[d] = 0.0;
      if (L == 0) { alpha0[bh] = NAN; max_rest[bh] = NAN; mean_rest[bh] = NAN; continue; }
      const uint16_t* qh = q + (size_t)bh * D;
      const uint16_t* K = k_cache + ((size_t)b * Hkv + g) * (size_t)Lmax * D;
      double top = -INFINITY;
      for (int32_t t = 0; t < L; ++t) {
        double s = 0.0;
        for (int d = 0; d < D; ++d) s += bf16_to_double(qh[d]) * bf16_to_double(K[(size_t)t * D + d]);
        w[t] = s * scale;
        if (w[t] > top) top = w[t];
      }
      double total = 0.0;
      for (int32_t t = 0; t < L; ++t) { w[t] = exp(w[t] - top); total += w[t]; }
      for (int32_t t = 0; t < L; ++t) w[t] /= total;          /* alpha_t */
      double biggest = 0.0, rest = 0.0;
      for (int32_t t = 1; t < L; ++t) {
        if (w[t] > biggest) biggest = w[t];
        rest += w[t];
      }
      alpha0[bh] = w[0];
      max_rest[bh] = biggest;
      mean_rest[bh] = L > 1 ? rest / (double)(L - 1) : 0.0;
      if (orow && L > 1) {
        const uint16_t* V = v_cache + ((size_t)b * Hkv + g) * (size_t)Lmax * D;
        for (int32_t t = 1; t < L; ++t)
          for (int d = 0; d < D; ++d) orow[d] += w[t] * bf16_to_double(V[(size_t)t * D + d]);
        for (int d = 0; d < D; ++d) orow[d] /= rest;
      }
    }
    free(w);
  }
  return failed ? -3 : 0;
}

/*
 * Paged cache -> contiguous cache.  pages is [n_pages, H_kv, page_tokens, D]; logical page j of
 * sequence b is physical page table[b * pages_per_seq + j]; token t of (b, g) is therefore row
 * t % page_tokens of group g of page table[b][t / page_tokens].  Fills cache [B, H_kv, L_max, D]
 * for t < seq_lens[b] and leaves the other rows zero.  A paged decode step is, by definition, the
 * decode step on this gathered cache (the paper's kernel takes contiguous caches, Section 4.3).
 */
int sr_oracle_gather_pages(const uint16_t* pages, const int32_t* table, const int32_t* seq_lens,
                           int32_t B, int32_t Hkv, int32_t D, int32_t Lmax, int32_t page_tokens,
                           int32_t pages_per_seq, int32_t n_pages, uint16_t* cache) {
  if (!pages || !table || !seq_lens || !cache) return -1;
  if (B < 1 || Hkv < 1 || D < 1 || Lmax < 1 || page_tokens < 1 || pages_per_seq < 1 || n_pages < 1) return -2;
  memset(cache, 0, sizeof(uint16_t) * (size_t)B * Hkv * Lmax * D);
  for (int b = 0; b < B; ++b) {
    int32_t L = clamp_len(seq_lens[b], Lmax);
    for (int g = 0; g < Hkv; ++g)
      for (int32_t t = 0; t < L; ++t) {
        int32_t j = t / page_tokens;
        if (j >= pages_per_seq) return -2;
        int32_t page = table[(size_t)b * pages_per_seq + j];
        if (page < 0 || page >= n_pages) return -4;
        const uint16_t* src = pages + (((size_t)page * Hkv + g) * page_tokens + (t % page_tokens)) * D;
        memcpy(cache + (((size_t)b * Hkv + g) * Lmax + t) * D, src, sizeof(uint16_t) * D);
      }
  }
  return 0;
}

int sr_oracle_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

int sr_oracle_cfg_size(void) { return (int)sizeof(sr_oracle_cfg); }
