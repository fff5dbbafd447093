/*
 * CPU oracle for the per-layer hot path of OOMB's chunk-recurrent training:
 * page scoring + top-k page selection, paged attention forward (O + LSE) and
 * backward (dQ, dK/dV accumulated into a paged gradient pool).
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is a plain, slow, obviously-correct
 * implementation used only by the tests, the smoke check and the benchmark's
 * cpu_baseline leg.  It shares no code with the HIP path and the product never
 * calls it.
 *
 * What it follows (paper sections):
 *   - Sec. 3, Eq. 2-3: a query chunk attends to the KV cache of all preceding
 *     chunks plus itself; gradients of earlier chunks' K/V are accumulated
 *     ("+=") across later chunks' backward passes.
 *   - Sec. 4.1: K/V and their gradients live in fixed-size pages reached through
 *     a page table; the backward pass accumulates dK/dV in place.
 *   - Sec. 4.2: page-level sparse attention; each key page is represented by the
 *     mean of its keys, queries are aggregated into a score per key page, the
 *     top-K pages are kept and the same indices are reused by the backward pass.
 *     Two aggregation rules: one pooled score and one list per KV head
 *     (oomb_oracle_page_score_topk), and the section's own equation, softmax votes
 *     summed per query page, one list per query page (oomb_oracle_page_vote_topk).
 *
 * Given a selection list, forward/backward are exactly masked softmax attention
 * and its exact gradient, so they are written as that definition.  The
 * selection is a heuristic, so it is written step by step with a fixed fp32
 * operation order (see oomb_oracle_page_score_topk).
 *
 * Compile twice: -DREAL=float (the oracle proper) and -DREAL=double (used for
 * finite-difference checks and as a tighter reference).  Always compile with
 * -ffp-contract=off so that no multiply-add is fused.
 *
 * Layouts (all contiguous, row-major):
 *   Q, O, dO, dQ : [C][Hq][D]
 *   K/V pools, dK/dV pools : [n_phys][Hkv][P][D]
 *   page_table   : [n] logical page -> physical page, n = N / P
 *   LSE, Delta   : [Hq][C]
 * Token t (0 <= t < N) lives at pool[page_table[t / P]][g][t % P][:].
 * Query i of the chunk has absolute position a_i = N - C + i and sees token t
 * iff t <= a_i and page t / P is in the selection list of its KV head.
 * Query head h uses KV head g = h / (Hq / Hkv).
 *
 * Input elements (Q, K, V, dO) are either `real` or bf16 bit patterns
 * (uint16), chosen by desc->in_is_bf16; bf16 -> real conversion is exact.
 *
 * Parity pins: every function below is pinned by tests/test_oracle_*.py
 * (finite differences, library SDPA + autograd with an explicit mask, closed
 * forms, placement invariance, chunk composition, brute-force top-k).  Nothing
 * the paper prints gives an absolute value to compare with, so absolute values
 * relative to the authors' own system are "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifndef REAL
#define REAL float
#endif
typedef REAL real;

#define R_EXP(x) ((real)exp((double)(x)))
#define R_LOG(x) ((real)log((double)(x)))

typedef struct {
  int32_t n_q_heads;   /* Hq */
  int32_t n_kv_heads;  /* Hkv, divides Hq */
  int32_t head_dim;    /* D */
  int32_t page_size;   /* P */
  int32_t chunk_len;   /* C, multiple of P */
  int32_t in_is_bf16;  /* 1: Q,K,V,dO are uint16 bf16 bit patterns; 0: `real` */
  int64_t ctx_len;     /* N, includes the chunk, multiple of P */
  double sm_scale;     /* logits = sm_scale * <q, k> */
  int32_t lists_per_query_page; /* 0: one page list per KV head, sel [Hkv][stride], sel_count [Hkv];
                                   1: one list per (KV head, query page), sel [Hkv][m][stride],
                                      sel_count [Hkv][m]: chunk row i uses the list of query page i / P */
} oomb_oracle_desc;

int oomb_oracle_real_bytes(void) { return (int)sizeof(real); }

#ifdef _OPENMP
#include <omp.h>
int oomb_oracle_num_threads(void) { return omp_get_max_threads(); }
#else
int oomb_oracle_num_threads(void) { return 1; }
#endif

static inline real ld(const void *base, int64_t idx, int is_bf16) {
  if (is_bf16) {
    uint32_t bits = ((uint32_t)((const uint16_t *)base)[idx]) << 16;
    float f;
    memcpy(&f, &bits, 4);
    return (real)f;
  }
  return ((const real *)base)[idx];
}

/* Selection lists: list `lid` is that of KV head g (lid = g) or, with one list per query page
 * (Sec. 4.2: the votes are aggregated for each of the m query pages), that of KV head g and query
 * page tau (lid = g m + tau).  sel == NULL means every logical page 0..n-1 (dense). */
static inline int list_id(const oomb_oracle_desc *d, int g, int i) {
  if (!d->lists_per_query_page) return g;
  return g * (d->chunk_len / d->page_size) + i / d->page_size;
}
static inline int n_lists(const oomb_oracle_desc *d) {
  return d->lists_per_query_page ? d->n_kv_heads * (d->chunk_len / d->page_size) : d->n_kv_heads;
}
static inline int32_t sel_len(const oomb_oracle_desc *d, const int32_t *sel_count, int lid,
                              const int32_t *sel) {
  if (!sel) return (int32_t)(d->ctx_len / d->page_size);
  return sel_count[lid];
}
static inline int32_t sel_at(const int32_t *sel, int32_t sel_stride, int lid, int32_t j) {
  if (!sel) return j;
  return sel[(int64_t)lid * sel_stride + j];
}

/* ------------------------------------------------------------------------- */
/* Page scoring + top-k (Sec. 4.2; per-KV-head variant: the mean-pooled chunk
 * query against the mean-pooled key of every past page).
 *
 * All arithmetic is IEEE binary32, one rounding per operation, in this order:
 *   S1  A[h][tau][d] = sum over the P tokens j of query page tau, left to right,
 *       of Q[tau*P + j][h][d].
 *       B[g][d] = sum, left to right, over tau = 0..m-1 (outer) and the G heads
 *       of group g (inner) of A[h][tau][d].
 *       qbar[g][d] = B[g][d] * r,  r = 1.0f / (float)(C * G).
 *   S2  kbar[g][l][d] = (sum over the P tokens of logical page l, left to
 *       right, of K) * (1.0f / P).
 *   S3  x[d] = qbar[g][d] * kbar[g][l][d]; then for s = D/2, D/4, ..., 1:
 *       x[d] += x[d + s] for d < s; score[g][l] = x[0].
 *   S4  candidates are the past pages l < n_past = n - C/P, ordered by larger
 *       score first (IEEE comparison, so -0 == +0), then lower logical id.  The
 *       first k_eff = min(top_k, n_past) are kept; the C/P local pages are
 *       always appended; the list is emitted in ascending logical id.
 * Scores must be finite (NaN ordering is not defined here).
 *
 * sel       : [Hkv][top_k + C/P]  (row stride top_k + C/P)
 * sel_count : [Hkv]
 * scores    : [Hkv][n_past] or NULL
 */
typedef struct {
  float s;
  int32_t id;
} cand_t;

static int cand_cmp(const void *a, const void *b) {
  const cand_t *x = (const cand_t *)a, *y = (const cand_t *)b;
  if (x->s > y->s) return -1;
  if (x->s < y->s) return 1;
  return (x->id > y->id) - (x->id < y->id);
}

/* kbar_cache == NULL: the page means are computed from the keys (S2).  Otherwise they are read from
 * kbar_cache[l][g][d] (logical page l), as written by oomb_oracle_kv_append / oomb_oracle_page_means,
 * and Kpool / page_table are not touched. */
static void score_topk_impl(const oomb_oracle_desc *d, const void *Q, const void *Kpool,
                            const int32_t *page_table, const float *kbar_cache, int32_t top_k, int32_t *sel,
                            int32_t *sel_count, float *scores) {
  const int Hq = d->n_q_heads, Hkv = d->n_kv_heads, D = d->head_dim, P = d->page_size;
  const int C = d->chunk_len, G = Hq / Hkv, bf = d->in_is_bf16;
  const int64_t n = d->ctx_len / P;
  const int m = C / P;
  const int64_t n_past = n - m;
  const int64_t k_eff = top_k < n_past ? top_k : n_past;
  const int32_t stride = top_k + m;
  const float r = 1.0f / (float)(C * G);
  const float inv_p = 1.0f / (float)P;

  float *A = (float *)malloc(sizeof(float) * (size_t)Hq * m * D);
  float *qbar = (float *)malloc(sizeof(float) * (size_t)Hkv * D);
  float *x = (float *)malloc(sizeof(float) * (size_t)D);
  cand_t *cand = (cand_t *)malloc(sizeof(cand_t) * (size_t)(n_past > 0 ? n_past : 1));
  char *keep = (char *)malloc((size_t)(n_past > 0 ? n_past : 1));

  /* S1 */
  for (int h = 0; h < Hq; ++h)
    for (int tau = 0; tau < m; ++tau)
      for (int dd = 0; dd < D; ++dd) {
        float acc = 0.0f;
        for (int j = 0; j < P; ++j)
          acc = acc + (float)ld(Q, ((int64_t)(tau * P + j) * Hq + h) * D + dd, bf);
        A[((size_t)h * m + tau) * D + dd] = acc;
      }
  for (int g = 0; g < Hkv; ++g)
    for (int dd = 0; dd < D; ++dd) {
      float acc = 0.0f;
      for (int tau = 0; tau < m; ++tau)
        for (int h = g * G; h < g * G + G; ++h) acc = acc + A[((size_t)h * m + tau) * D + dd];
      qbar[(size_t)g * D + dd] = acc * r;
    }

  for (int g = 0; g < Hkv; ++g) {
    for (int64_t l = 0; l < n_past; ++l) {
      /* S2 + first step of S3 */
      for (int dd = 0; dd < D; ++dd) {
        float kbar;
        if (kbar_cache) {
          kbar = kbar_cache[((size_t)l * Hkv + g) * D + dd];
        } else {
          const int64_t base = ((int64_t)page_table[l] * Hkv + g) * P * D;
          float acc = 0.0f;
          for (int t = 0; t < P; ++t) acc = acc + (float)ld(Kpool, base + (int64_t)t * D + dd, bf);
          kbar = acc * inv_p;
        }
        x[dd] = qbar[(size_t)g * D + dd] * kbar;
      }
      /* S3: stride-halving tree */
      for (int s = D / 2; s >= 1; s /= 2)
        for (int dd = 0; dd < s; ++dd) x[dd] = x[dd] + x[dd + s];
      cand[l].s = x[0];
      cand[l].id = (int32_t)l;
      if (scores) scores[(int64_t)g * n_past + l] = x[0];
    }
    /* S4 */
    if (n_past > 0) {
      qsort(cand, (size_t)n_past, sizeof(cand_t), cand_cmp);
      memset(keep, 0, (size_t)n_past);
      for (int64_t j = 0; j < k_eff; ++j) keep[cand[j].id] = 1;
    }
    int32_t cnt = 0;
    for (int64_t l = 0; l < n_past; ++l)
      if (keep[l]) sel[(int64_t)g * stride + cnt++] = (int32_t)l;
    for (int64_t l = n_past; l < n; ++l) sel[(int64_t)g * stride + cnt++] = (int32_t)l;
    sel_count[g] = cnt;
    for (int32_t j = cnt; j < stride; ++j) sel[(int64_t)g * stride + j] = -1;
  }
  free(A);
  free(qbar);
  free(x);
  free(cand);
  free(keep);
}

void oomb_oracle_page_score_topk(const oomb_oracle_desc *d, const void *Q, const void *Kpool,
                                 const int32_t *page_table, int32_t top_k, int32_t *sel,
                                 int32_t *sel_count, float *scores) {
  score_topk_impl(d, Q, Kpool, page_table, NULL, top_k, sel, sel_count, scores);
}

/* The same selection with the page means read from a cache kept by the paged manager (Sec. 4.1:
 * pages are appended chunk by chunk, so the mean of a page can be taken once, when it is written). */
void oomb_oracle_page_score_topk_cached(const oomb_oracle_desc *d, const void *Q, const float *kbar_cache,
                                        int32_t top_k, int32_t *sel, int32_t *sel_count, float *scores) {
  score_topk_impl(d, Q, NULL, NULL, kbar_cache, top_k, sel, sel_count, scores);
}

/* ------------------------------------------------------------------------- */
/* Paged manager, append step (Sec. 4.1): the chunk's keys and values, Kc / Vc [C][Hkv][D] in token
 * order, become the m = C/P local pages: token i of the chunk goes to
 * pool[page_table[n_past + i / P]][g][i % P][:], bit for bit.  If kbar_cache is given, the means of
 * the new pages are written to kbar_cache[n_past + tau][g][:] in the order of step S2 above. */
void oomb_oracle_kv_append(const oomb_oracle_desc *d, const void *Kc, const void *Vc,
                           const int32_t *page_table, void *Kpool, void *Vpool, float *kbar_cache) {
  const int Hkv = d->n_kv_heads, D = d->head_dim, P = d->page_size, C = d->chunk_len, bf = d->in_is_bf16;
  const int64_t n = d->ctx_len / P, n_past = n - C / P;
  const size_t esz = bf ? 2 : sizeof(real);
  for (int i = 0; i < C; ++i)
    for (int g = 0; g < Hkv; ++g) {
      const int64_t dst = (((int64_t)page_table[n_past + i / P] * Hkv + g) * P + i % P) * D;
      const int64_t src = ((int64_t)i * Hkv + g) * D;
      memcpy((char *)Kpool + (size_t)dst * esz, (const char *)Kc + (size_t)src * esz, (size_t)D * esz);
      memcpy((char *)Vpool + (size_t)dst * esz, (const char *)Vc + (size_t)src * esz, (size_t)D * esz);
    }
  if (!kbar_cache) return;
  const float inv_p = 1.0f / (float)P;
  for (int64_t l = n_past; l < n; ++l)
    for (int g = 0; g < Hkv; ++g) {
      const int64_t base = ((int64_t)page_table[l] * Hkv + g) * P * D;
      for (int dd = 0; dd < D; ++dd) {
        float acc = 0.0f;
        for (int t = 0; t < P; ++t) acc = acc + (float)ld(Kpool, base + (int64_t)t * D + dd, bf);
        kbar_cache[((size_t)l * Hkv + g) * D + dd] = acc * inv_p;
      }
    }
}

/* Means of logical pages [first, first + count) into kbar_cache (step S2), e.g. to build the cache
 * for a pool that was filled by other means. */
void oomb_oracle_page_means(const oomb_oracle_desc *d, const void *Kpool, const int32_t *page_table,
                            int64_t first, int64_t count, float *kbar_cache) {
  const int Hkv = d->n_kv_heads, D = d->head_dim, P = d->page_size, bf = d->in_is_bf16;
  const float inv_p = 1.0f / (float)P;
  for (int64_t l = first; l < first + count; ++l)
    for (int g = 0; g < Hkv; ++g) {
      const int64_t base = ((int64_t)page_table[l] * Hkv + g) * P * D;
      for (int dd = 0; dd < D; ++dd) {
        float acc = 0.0f;
        for (int t = 0; t < P; ++t) acc = acc + (float)ld(Kpool, base + (int64_t)t * D + dd, bf);
        kbar_cache[((size_t)l * Hkv + g) * D + dd] = acc * inv_p;
      }
    }
}

/* Page list of a local-attention layer (Sec. 4.2, natively sparse models: such layers retrieve only
 * the most recent pages): for every KV head the min(window_pages, n_past) most recent past pages,
 * then the m local pages, ascending.  sel: [Hkv][window_pages + m]. */
void oomb_oracle_local_page_list(const oomb_oracle_desc *d, int32_t window_pages, int32_t *sel,
                                 int32_t *sel_count) {
  const int Hkv = d->n_kv_heads, P = d->page_size, m = d->chunk_len / P;
  const int64_t n = d->ctx_len / P, n_past = n - m;
  const int64_t w = window_pages < n_past ? window_pages : n_past;
  const int32_t stride = window_pages + m;
  for (int g = 0; g < Hkv; ++g) {
    int32_t cnt = 0;
    for (int64_t l = n_past - w; l < n; ++l) sel[(int64_t)g * stride + cnt++] = (int32_t)l;
    sel_count[g] = cnt;
    for (int32_t j = cnt; j < stride; ++j) sel[(int64_t)g * stride + j] = -1;
  }
}

/* ------------------------------------------------------------------------- */
/* Retrieval by voting (Sec. 4.2, the scoring equation): every query token scores all key pages
 * against their representative vectors, turns the scores into a distribution over the key pages
 * (softmax along the key-page index), and the distributions of the P tokens of a query page are
 * summed into one vote per key page; each query page keeps its top-K pages.
 *
 * Written out, per KV head g, query page tau, past page l < n_past (all in double):
 *   z[h][i][l]  = sm_scale * sum_d Q[i][h][d] * kbar[l][g][d]
 *   p[h][i][.]  = softmax over l of z[h][i][.]
 *   vote[g][tau][l] = sum over the G heads h of group g and the P tokens i of query page tau of p[h][i][l]
 * The candidates are the past pages only; the order is larger vote first, then lower logical id;
 * the first k_eff = min(top_k, n_past) are kept.  The list of query page tau is those pages
 * followed by the local pages n_past .. n_past + tau (the ones its rows can see), ascending.
 *
 * kbar is read from kbar_cache [>= n_past][Hkv][D] (as written by oomb_oracle_page_means); with
 * kbar_round_bf16 != 0 every element is first rounded to bf16 (nearest even), the precision in
 * which a bf16 matrix instruction takes its operands.
 *
 * sel: [Hkv][m][top_k + m] (-1 padded), sel_count: [Hkv][m], votes: [Hkv][m][n_past] or NULL. */
static double round_to_bf16(float f) {
  uint32_t u;
  memcpy(&u, &f, 4);
  u += 0x7fffu + ((u >> 16) & 1u);
  u &= 0xffff0000u;
  float r;
  memcpy(&r, &u, 4);
  return (double)r;
}

typedef struct {
  double s;
  int32_t id;
} vcand_t;

static int vcand_cmp(const void *a, const void *b) {
  const vcand_t *x = (const vcand_t *)a, *y = (const vcand_t *)b;
  if (x->s > y->s) return -1;
  if (x->s < y->s) return 1;
  return (x->id > y->id) - (x->id < y->id);
}

void oomb_oracle_page_vote_topk(const oomb_oracle_desc *d, const void *Q, const float *kbar_cache,
                                int32_t kbar_round_bf16, int32_t top_k, int32_t *sel, int32_t *sel_count,
                                double *votes) {
  const int Hq = d->n_q_heads, Hkv = d->n_kv_heads, D = d->head_dim, P = d->page_size;
  const int C = d->chunk_len, G = Hq / Hkv, bf = d->in_is_bf16, m = C / P;
  const int64_t n = d->ctx_len / P, n_past = n - m;
  const int64_t k_eff = top_k < n_past ? top_k : n_past;
  const int32_t stride = top_k + m;
  const int64_t np1 = n_past > 0 ? n_past : 1;

  double *kb = (double *)malloc(sizeof(double) * (size_t)np1 * D);
  double *vote = (double *)malloc(sizeof(double) * (size_t)np1);
  double *z = (double *)malloc(sizeof(double) * (size_t)np1);
  vcand_t *cand = (vcand_t *)malloc(sizeof(vcand_t) * (size_t)np1);
  char *keep = (char *)malloc((size_t)np1);

  for (int g = 0; g < Hkv; ++g) {
    for (int64_t l = 0; l < n_past; ++l)
      for (int dd = 0; dd < D; ++dd) {
        const float v = kbar_cache[((size_t)l * Hkv + g) * D + dd];
        kb[l * D + dd] = kbar_round_bf16 ? round_to_bf16(v) : (double)v;
      }
    for (int tau = 0; tau < m; ++tau) {
      for (int64_t l = 0; l < n_past; ++l) vote[l] = 0.0;
      for (int h = g * G; h < g * G + G; ++h)
        for (int i = tau * P; i < tau * P + P; ++i) {
          double zmax = -INFINITY;
          for (int64_t l = 0; l < n_past; ++l) {
            double dot = 0.0;
            for (int dd = 0; dd < D; ++dd)
              dot += (double)ld(Q, ((int64_t)i * Hq + h) * D + dd, bf) * kb[l * D + dd];
            z[l] = d->sm_scale * dot;
            if (z[l] > zmax) zmax = z[l];
          }
          double sum = 0.0;
          for (int64_t l = 0; l < n_past; ++l) {
            z[l] = exp(z[l] - zmax);
            sum += z[l];
          }
          for (int64_t l = 0; l < n_past; ++l) vote[l] += z[l] / sum;
        }
      for (int64_t l = 0; l < n_past; ++l) {
        cand[l].s = vote[l];
        cand[l].id = (int32_t)l;
        if (votes) votes[((int64_t)g * m + tau) * n_past + l] = vote[l];
      }
      if (n_past > 0) {
        qsort(cand, (size_t)n_past, sizeof(vcand_t), vcand_cmp);
        memset(keep, 0, (size_t)n_past);
        for (int64_t j = 0; j < k_eff; ++j) keep[cand[j].id] = 1;
      }
      int32_t *out = sel + ((int64_t)g * m + tau) * stride;
      int32_t cnt = 0;
      for (int64_t l = 0; l < n_past; ++l)
        if (keep[l]) out[cnt++] = (int32_t)l;
      for (int64_t l = n_past; l <= n_past + tau; ++l) out[cnt++] = (int32_t)l;
      sel_count[g * m + tau] = cnt;
      for (int32_t j = cnt; j < stride; ++j) out[j] = -1;
    }
  }
  free(kb);
  free(vote);
  free(z);
  free(cand);
  free(keep);
}

/* ------------------------------------------------------------------------- */
/* Logits of one query row against every visible token of the selected pages.
 * Returns the number of visible tokens; s[j] are the scaled logits, tok[j] the
 * token positions, in ascending token order. */
static int64_t row_logits(const oomb_oracle_desc *d, const void *Q, const void *Kpool,
                          const int32_t *page_table, const int32_t *sel, const int32_t *sel_count,
                          int32_t sel_stride, int h, int i, real *s, int64_t *tok) {
  const int Hq = d->n_q_heads, Hkv = d->n_kv_heads, D = d->head_dim, P = d->page_size;
  const int G = Hq / Hkv, g = h / G, bf = d->in_is_bf16;
  const int64_t a_i = d->ctx_len - d->chunk_len + i;
  const real scale = (real)d->sm_scale;
  const int lid = list_id(d, g, i);
  const int32_t cnt = sel_len(d, sel_count, lid, sel);
  int64_t nv = 0;
  for (int32_t j = 0; j < cnt; ++j) {
    const int64_t l = sel_at(sel, sel_stride, lid, j);
    const int64_t base = ((int64_t)page_table[l] * Hkv + g) * P * D;
    for (int t = 0; t < P; ++t) {
      const int64_t pos = l * P + t;
      if (pos > a_i) break;
      real dot = 0;
      for (int dd = 0; dd < D; ++dd)
        dot += ld(Q, ((int64_t)i * Hq + h) * D + dd, bf) * ld(Kpool, base + (int64_t)t * D + dd, bf);
      s[nv] = scale * dot;
      tok[nv] = pos;
      ++nv;
    }
  }
  return nv;
}

static int64_t max_visible(const oomb_oracle_desc *d, const int32_t *sel, const int32_t *sel_count) {
  int64_t mx = 0;
  for (int lid = 0; lid < n_lists(d); ++lid) {
    int64_t c = sel_len(d, sel_count, lid, sel);
    if (c > mx) mx = c;
  }
  return mx * d->page_size;
}

/* ------------------------------------------------------------------------- */
/* Forward (Sec. 4.1 operator; the softmax attention definition).
 * For query head h, row i:  s_t = sm_scale <Q[i,h], K[t,g]> over visible t;
 *   LSE = log sum_t exp(s_t)  (natural log, computed as M + log sum exp(s - M));
 *   p_t = exp(s_t - LSE);  O[i,h,:] = sum_t p_t V[t,g,:].
 * rows == NULL: all rows, O is [C][Hq][D], LSE is [Hq][C].
 * rows != NULL: rows holds n_rows (h, i) pairs; O is [n_rows][D], LSE [n_rows].
 */
void oomb_oracle_attn_fwd(const oomb_oracle_desc *d, const void *Q, const void *Kpool,
                          const void *Vpool, const int32_t *page_table, const int32_t *sel,
                          const int32_t *sel_count, int32_t sel_stride, const int32_t *rows,
                          int64_t n_rows, real *O, real *LSE) {
  const int Hq = d->n_q_heads, Hkv = d->n_kv_heads, D = d->head_dim, P = d->page_size;
  const int C = d->chunk_len, bf = d->in_is_bf16;
  const int64_t total = rows ? n_rows : (int64_t)C * Hq;
  const int64_t cap = max_visible(d, sel, sel_count);
#pragma omp parallel
  {
    real *s = (real *)malloc(sizeof(real) * (size_t)cap);
    int64_t *tok = (int64_t *)malloc(sizeof(int64_t) * (size_t)cap);
#pragma omp for schedule(dynamic, 4)
    for (int64_t r = 0; r < total; ++r) {
      const int h = rows ? rows[2 * r] : (int)(r % Hq);
      const int i = rows ? rows[2 * r + 1] : (int)(r / Hq);
      const int g = h / (Hq / Hkv);
      real *o = rows ? O + r * D : O + ((int64_t)i * Hq + h) * D;
      const int64_t nv = row_logits(d, Q, Kpool, page_table, sel, sel_count, sel_stride, h, i, s, tok);
      real M = s[0];
      for (int64_t j = 1; j < nv; ++j)
        if (s[j] > M) M = s[j];
      real sum = 0;
      for (int64_t j = 0; j < nv; ++j) sum += R_EXP(s[j] - M);
      const real lse = M + R_LOG(sum);
      for (int dd = 0; dd < D; ++dd) o[dd] = 0;
      for (int64_t j = 0; j < nv; ++j) {
        const real p = R_EXP(s[j] - lse);
        const int64_t base = ((int64_t)page_table[tok[j] / P] * Hkv + g) * P * D + (tok[j] % P) * D;
        for (int dd = 0; dd < D; ++dd) o[dd] += p * ld(Vpool, base + dd, bf);
      }
      if (rows)
        LSE[r] = lse;
      else
        LSE[(int64_t)h * C + i] = lse;
    }
    free(s);
    free(tok);
  }
}

/* Probabilities of one row (h, i): p[j] for the j-th visible token, tok[j] its
 * position.  Returns the count.  Used by tests (row sums, visible set). */
int64_t oomb_oracle_row_probs(const oomb_oracle_desc *d, const void *Q, const void *Kpool,
                              const int32_t *page_table, const int32_t *sel,
                              const int32_t *sel_count, int32_t sel_stride, int32_t h, int32_t i,
                              real *p, int64_t *tok) {
  const int64_t nv = row_logits(d, Q, Kpool, page_table, sel, sel_count, sel_stride, h, i, p, tok);
  real M = p[0];
  for (int64_t j = 1; j < nv; ++j)
    if (p[j] > M) M = p[j];
  real sum = 0;
  for (int64_t j = 0; j < nv; ++j) sum += R_EXP(p[j] - M);
  const real lse = M + R_LOG(sum);
  for (int64_t j = 0; j < nv; ++j) p[j] = R_EXP(p[j] - lse);
  return nv;
}

/* ------------------------------------------------------------------------- */
/* Delta[h][i] = sum_d dO[i,h,d] * O[i,h,d]   (O is `real`, [C][Hq][D]). */
void oomb_oracle_delta(const oomb_oracle_desc *d, const void *dO, const real *O, real *Delta) {
  const int Hq = d->n_q_heads, D = d->head_dim, C = d->chunk_len, bf = d->in_is_bf16;
  for (int i = 0; i < C; ++i)
    for (int h = 0; h < Hq; ++h) {
      real acc = 0;
      for (int dd = 0; dd < D; ++dd) {
        const int64_t idx = ((int64_t)i * Hq + h) * D + dd;
        acc += ld(dO, idx, bf) * O[idx];
      }
      Delta[(int64_t)h * C + i] = acc;
    }
}

/* ------------------------------------------------------------------------- */
/* Backward, dQ.  With p_t = exp(s_t - LSE), dp_t = <dO[i,h], V[t,g]>,
 * ds_t = p_t (dp_t - Delta):   dQ[i,h,:] = sm_scale * sum_t ds_t K[t,g,:].
 * LSE and Delta are [Hq][C].  rows as in the forward; dQ is [C][Hq][D] or
 * [n_rows][D] (overwritten). */
void oomb_oracle_attn_bwd_dq(const oomb_oracle_desc *d, const void *Q, const void *Kpool,
                             const void *Vpool, const int32_t *page_table, const int32_t *sel,
                             const int32_t *sel_count, int32_t sel_stride, const real *LSE,
                             const real *Delta, const void *dO, const int32_t *rows,
                             int64_t n_rows, real *dQ) {
  const int Hq = d->n_q_heads, Hkv = d->n_kv_heads, D = d->head_dim, P = d->page_size;
  const int C = d->chunk_len, bf = d->in_is_bf16;
  const real scale = (real)d->sm_scale;
  const int64_t total = rows ? n_rows : (int64_t)C * Hq;
  const int64_t cap = max_visible(d, sel, sel_count);
#pragma omp parallel
  {
    real *s = (real *)malloc(sizeof(real) * (size_t)cap);
    int64_t *tok = (int64_t *)malloc(sizeof(int64_t) * (size_t)cap);
#pragma omp for schedule(dynamic, 4)
    for (int64_t r = 0; r < total; ++r) {
      const int h = rows ? rows[2 * r] : (int)(r % Hq);
      const int i = rows ? rows[2 * r + 1] : (int)(r / Hq);
      const int g = h / (Hq / Hkv);
      real *dq = rows ? dQ + r * D : dQ + ((int64_t)i * Hq + h) * D;
      const real lse = LSE[(int64_t)h * C + i], delta = Delta[(int64_t)h * C + i];
      const int64_t nv = row_logits(d, Q, Kpool, page_table, sel, sel_count, sel_stride, h, i, s, tok);
      for (int dd = 0; dd < D; ++dd) dq[dd] = 0;
      for (int64_t j = 0; j < nv; ++j) {
        const int64_t base = ((int64_t)page_table[tok[j] / P] * Hkv + g) * P * D + (tok[j] % P) * D;
        const real p = R_EXP(s[j] - lse);
        real dp = 0;
        for (int dd = 0; dd < D; ++dd)
          dp += ld(dO, ((int64_t)i * Hq + h) * D + dd, bf) * ld(Vpool, base + dd, bf);
        const real ds = p * (dp - delta);
        for (int dd = 0; dd < D; ++dd) dq[dd] += ds * ld(Kpool, base + dd, bf);
      }
      for (int dd = 0; dd < D; ++dd) dq[dd] *= scale;
    }
    free(s);
    free(tok);
  }
}

/* ------------------------------------------------------------------------- */
/* Backward, dK / dV, accumulated into the gradient pools (Sec. 3 Eq. 3 and
 * Sec. 4.1: in-place accumulation).  For every token t of every selected page
 * of KV head g:
 *   dV[t,g,:] += sum_{h in g} sum_{i : t visible} p_t(h,i) dO[i,h,:]
 *   dK[t,g,:] += sm_scale * sum_{h in g} sum_{i} ds_t(h,i) Q[i,h,:]
 * written at pool[page_table[t / P]][g][t % P][:], where the sums run over the rows whose
 * list holds the page of t.  Pages outside every list are not touched.  units == NULL: every
 * (g, page in some list of g).  units != NULL: n_units pairs (g, logical page); a listed page
 * that is in no list of g contributes nothing. */
void oomb_oracle_attn_bwd_dkv(const oomb_oracle_desc *d, const void *Q, const void *Kpool,
                              const void *Vpool, const int32_t *page_table, const int32_t *sel,
                              const int32_t *sel_count, int32_t sel_stride, const real *LSE,
                              const real *Delta, const void *dO, const int32_t *units,
                              int64_t n_units, real *dKpool, real *dVpool) {
  const int Hq = d->n_q_heads, Hkv = d->n_kv_heads, D = d->head_dim, P = d->page_size;
  const int C = d->chunk_len, G = Hq / Hkv, bf = d->in_is_bf16;
  const real scale = (real)d->sm_scale;
  const int64_t N = d->ctx_len;

  /* member[(g n + l) n_tau + tau] = 1 iff logical page l is in the list that the rows of query page
   * tau use for KV head g (with one list per KV head n_tau = 1: every row uses the same list) */
  const int64_t n = N / P;
  const int n_tau = d->lists_per_query_page ? C / P : 1;
  char *member = (char *)calloc((size_t)Hkv * (size_t)n * (size_t)n_tau, 1);
  for (int g = 0; g < Hkv; ++g)
    for (int tau = 0; tau < n_tau; ++tau) {
      const int lid = d->lists_per_query_page ? g * n_tau + tau : g;
      for (int32_t j = 0; j < sel_len(d, sel_count, lid, sel); ++j)
        member[((int64_t)g * n + sel_at(sel, sel_stride, lid, j)) * n_tau + tau] = 1;
    }

  /* flatten the work list: the given units, or every (g, page) that some list of g holds */
  int64_t total = 0;
  int32_t *work = NULL;
  if (units) {
    total = n_units;
    work = (int32_t *)malloc(sizeof(int32_t) * 2 * (size_t)(total > 0 ? total : 1));
    memcpy(work, units, sizeof(int32_t) * 2 * (size_t)total);
  } else {
    work = (int32_t *)malloc(sizeof(int32_t) * 2 * (size_t)Hkv * (size_t)n);
    for (int g = 0; g < Hkv; ++g)
      for (int64_t l = 0; l < n; ++l) {
        int any = 0;
        for (int tau = 0; tau < n_tau; ++tau) any |= member[((int64_t)g * n + l) * n_tau + tau];
        if (!any) continue;
        work[2 * total] = g;
        work[2 * total + 1] = (int32_t)l;
        ++total;
      }
  }

#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t u = 0; u < total; ++u) {
    const int g = work[2 * u];
    const int64_t l = work[2 * u + 1];
    const char *mem = member + ((int64_t)g * n + l) * n_tau;
    int selected = 0;
    for (int tau = 0; tau < n_tau; ++tau) selected |= mem[tau];
    if (!selected) continue;
    const int64_t base = ((int64_t)page_table[l] * Hkv + g) * P * D;
    real *dk = (real *)malloc(sizeof(real) * (size_t)D);
    real *dv = (real *)malloc(sizeof(real) * (size_t)D);
    for (int t = 0; t < P; ++t) {
      const int64_t pos = l * P + t;
      for (int dd = 0; dd < D; ++dd) dk[dd] = dv[dd] = 0;
      for (int h = g * G; h < g * G + G; ++h)
        for (int i = 0; i < C; ++i) {
          const int64_t a_i = N - C + i;
          if (pos > a_i) continue;
          if (!mem[n_tau > 1 ? i / P : 0]) continue; /* the row's list does not hold this page */
          const int64_t qoff = ((int64_t)i * Hq + h) * D;
          real dot = 0, dp = 0;
          for (int dd = 0; dd < D; ++dd)
            dot += ld(Q, qoff + dd, bf) * ld(Kpool, base + (int64_t)t * D + dd, bf);
          for (int dd = 0; dd < D; ++dd)
            dp += ld(dO, qoff + dd, bf) * ld(Vpool, base + (int64_t)t * D + dd, bf);
          const real p = R_EXP(scale * dot - LSE[(int64_t)h * C + i]);
          const real ds = p * (dp - Delta[(int64_t)h * C + i]);
          for (int dd = 0; dd < D; ++dd) {
            dv[dd] += p * ld(dO, qoff + dd, bf);
            dk[dd] += ds * ld(Q, qoff + dd, bf);
          }
        }
      for (int dd = 0; dd < D; ++dd) {
        dKpool[base + (int64_t)t * D + dd] += scale * dk[dd];
        dVpool[base + (int64_t)t * D + dd] += dv[dd];
      }
    }
    free(dk);
    free(dv);
  }
  free(work);
  free(member);
}
