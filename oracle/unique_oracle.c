/*
 * Reference oracle for UNIQUE decode-time top-k sparse attention.
 *
 * THIS FILE IS TEST INFRASTRUCTURE. It is a plain, slow, float64 CPU
 * transcription of the definitions in the paper, used only to check the GPU
 * library and to be timed beside it as a CPU baseline. The product never
 * calls it, and it shares no code with the HIP sources.
 *
 * What it follows (paper sections / equations):
 *   - paging: Section 3.1, first paragraph (P = ceil(N/S) contiguous pages of S keys)
 *   - page mean:  Eq. 1          - page std (scalar): Eq. 2
 *   - page score: Eq. 3, and its GQA form Eq. 6 (max over the G heads of a group)
 *   - top-k page set T_k(q): Section 3.2, paragraph after Eq. 4
 *   - sparse attention: Eq. 5    - dense attention: Eq. 4
 *
 * Readings taken where the paper is silent (the same list is in the design notes):
 *   - a partial last page uses its n valid tokens with 1/n (Eq. 1-2 print 1/S);
 *   - population variance (1/n), exactly as Eq. 2 prints it;
 *   - the score carries no 1/sqrt(D) factor (Eq. 3 has none);
 *   - ties in the score are broken towards the lower logical page index;
 *   - no page is kept unconditionally: exactly min(k, P) pages, all chosen by score;
 *   - N counts the token being decoded.
 *
 *   - bf16 storage of the page means (the storage format of the paper's kernels, Appendix A "in bf16"):
 *     the float64 mean of Eq. 1 rounded once, to nearest with ties to even, by oracle_round_bf16.
 *
 * Every function has an independent pin in tests/test_oracle_pins.py
 * (brute force in pure Python, closed forms, invariants, numpy special cases).
 *
 * Inputs are the caches exactly as stored (fp32, or bf16 bit patterns), which
 * convert to double without rounding; all arithmetic is double.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
  int32_t dtype;            /* 0 = fp32, 1 = bf16 (uint16 bit patterns) : q, k_cache, v_cache */
  int32_t H, Hkv, D, S;     /* query heads, KV heads, head dim, page size */
  int32_t B;                /* sequences */
  int32_t max_pages_per_seq;/* row stride of page_table */
  int64_t num_phys_pages;
  const void* k_cache;      /* [num_phys_pages][Hkv][S][D] */
  const void* v_cache;      /* same */
  const int32_t* page_table;/* [B][max_pages_per_seq] logical -> physical */
  const int32_t* seq_lens;  /* [B] */
} oracle_cache;

static double load_elem(const void* base, int32_t dtype, int64_t idx) {
  if (dtype == 0) return (double)((const float*)base)[idx];
  uint32_t u = (uint32_t)((const uint16_t*)base)[idx] << 16;
  float f;
  memcpy(&f, &u, 4);
  return (double)f;
}

/* element offset of token slot j, dim 0 of (physical page, kv head) */
static int64_t slot_offset(const oracle_cache* c, int64_t phys, int hkv, int j) {
  return ((phys * c->Hkv + hkv) * c->S + j) * (int64_t)c->D;
}

static int num_pages(const oracle_cache* c, int b) {
  int N = c->seq_lens[b];
  return (N + c->S - 1) / c->S;
}

static int valid_tokens(const oracle_cache* c, int b, int p) {
  int N = c->seq_lens[b];
  int n = N - p * c->S;
  return n < c->S ? n : c->S;
}

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* Eq. 1 and Eq. 2 for logical pages [p0, p1) of (sequence b, kv head hkv).
 * mean: [(p1-p0)][D], std: [(p1-p0)].  Two passes: mean first, then squared
 * deviations from it. Returns 0, or -1 on a bad range. */
int oracle_page_stats(const oracle_cache* c, int b, int hkv, int p0, int p1,
                      double* mean, double* std) {
  if (b < 0 || b >= c->B || hkv < 0 || hkv >= c->Hkv) return -1;
  if (p0 < 0 || p1 > num_pages(c, b) || p0 > p1) return -1;
  const int D = c->D;
  for (int p = p0; p < p1; ++p) {
    const int n = valid_tokens(c, b, p);
    const int64_t phys = c->page_table[(int64_t)b * c->max_pages_per_seq + p];
    double* m = mean + (int64_t)(p - p0) * D;
    for (int d = 0; d < D; ++d) {
      double s = 0.0;
      for (int j = 0; j < n; ++j) s += load_elem(c->k_cache, c->dtype, slot_offset(c, phys, hkv, j) + d);
      m[d] = s / (double)n;
    }
    double norm2 = 0.0; /* sum over d of the per-dimension population variance */
    for (int d = 0; d < D; ++d) {
      double ss = 0.0;
      for (int j = 0; j < n; ++j) {
        double dev = load_elem(c->k_cache, c->dtype, slot_offset(c, phys, hkv, j) + d) - m[d];
        ss += dev * dev;
      }
      double sd = sqrt(ss / (double)n); /* per-dimension std */
      norm2 += sd * sd;                 /* l2 norm over D, squared */
    }
    std[p - p0] = sqrt(norm2);
  }
  return 0;
}

/* Eq. 6 (Eq. 3 when G == 1): scores of `npages` pages of (b, hkv) given their stats.
 * q: [B][H][D] in the cache dtype. mean: [npages][D], std: [npages]. */
int oracle_page_scores(const oracle_cache* c, const void* q, int b, int hkv, double lambda,
                       int npages, const double* mean, const double* std, double* scores) {
  if (b < 0 || b >= c->B || hkv < 0 || hkv >= c->Hkv) return -1;
  const int D = c->D, G = c->H / c->Hkv;
  for (int p = 0; p < npages; ++p) {
    double best = 0.0;
    for (int g = 0; g < G; ++g) {
      const int64_t qoff = ((int64_t)b * c->H + (int64_t)hkv * G + g) * D;
      double dot = 0.0, qq = 0.0;
      for (int d = 0; d < D; ++d) {
        double qd = load_elem(q, c->dtype, qoff + d);
        dot += qd * mean[(int64_t)p * D + d];
        qq += qd * qd;
      }
      double s = dot + lambda * sqrt(qq) * std[p];
      if (g == 0 || s > best) best = s;
    }
    scores[p] = best;
  }
  return 0;
}

typedef struct { double s; int32_t p; } scored_page;

static int cmp_scored(const void* a, const void* b) {
  const scored_page* x = (const scored_page*)a;
  const scored_page* y = (const scored_page*)b;
  if (x->s > y->s) return -1;
  if (x->s < y->s) return 1;
  return (x->p > y->p) - (x->p < y->p);
}

/* Full ranking of P pages by (score descending, page index ascending).
 * order: [P] page indices in rank order; the top-k set is order[0 .. min(k,P)).
 * Returns min(k, P). */
int oracle_topk(const double* scores, int P, int k, int32_t* order) {
  scored_page* a = (scored_page*)malloc(sizeof(scored_page) * (size_t)(P > 0 ? P : 1));
  for (int p = 0; p < P; ++p) { a[p].s = scores[p]; a[p].p = p; }
  qsort(a, (size_t)P, sizeof(scored_page), cmp_scored);
  for (int p = 0; p < P; ++p) order[p] = a[p].p;
  free(a);
  return k < P ? k : P;
}

/* Eq. 5 for query head h of sequence b over the logical pages pages[0..npages)
 * (Eq. 4 when they are all pages of the sequence). Tokens at or beyond N are
 * skipped. out: [D]; lse: natural log of sum of exp of the scaled logits.
 * sm_scale <= 0 means 1/sqrt(D). Returns 0, -1 on a bad page index, -2 when no token. */
int oracle_attention(const oracle_cache* c, const void* q, int b, int h,
                     const int32_t* pages, int npages, double sm_scale,
                     double* out, double* lse) {
  if (b < 0 || b >= c->B || h < 0 || h >= c->H) return -1;
  const int D = c->D, G = c->H / c->Hkv, hkv = h / G;
  const int P = num_pages(c, b);
  if (sm_scale <= 0.0) sm_scale = 1.0 / sqrt((double)D);
  const int64_t qoff = ((int64_t)b * c->H + h) * D;
  int64_t ntok = 0;
  for (int i = 0; i < npages; ++i) {
    if (pages[i] < 0 || pages[i] >= P) return -1;
    ntok += valid_tokens(c, b, pages[i]);
  }
  if (ntok == 0) return -2;
  double* logit = (double*)malloc(sizeof(double) * (size_t)ntok);
  /* pass 1: logits and their maximum */
  int64_t t = 0;
  double mx = -INFINITY;
  for (int i = 0; i < npages; ++i) {
    const int n = valid_tokens(c, b, pages[i]);
    const int64_t phys = c->page_table[(int64_t)b * c->max_pages_per_seq + pages[i]];
    for (int j = 0; j < n; ++j, ++t) {
      const int64_t ko = slot_offset(c, phys, hkv, j);
      double dot = 0.0;
      for (int d = 0; d < D; ++d) dot += load_elem(q, c->dtype, qoff + d) * load_elem(c->k_cache, c->dtype, ko + d);
      logit[t] = dot * sm_scale;
      if (logit[t] > mx) mx = logit[t];
    }
  }
  /* pass 2: softmax weights (max subtracted) and the weighted sum of V rows */
  double denom = 0.0;
  for (int64_t i = 0; i < ntok; ++i) denom += exp(logit[i] - mx);
  for (int d = 0; d < D; ++d) out[d] = 0.0;
  t = 0;
  for (int i = 0; i < npages; ++i) {
    const int n = valid_tokens(c, b, pages[i]);
    const int64_t phys = c->page_table[(int64_t)b * c->max_pages_per_seq + pages[i]];
    for (int j = 0; j < n; ++j, ++t) {
      const double w = exp(logit[t] - mx) / denom;
      const int64_t vo = slot_offset(c, phys, hkv, j);
      for (int d = 0; d < D; ++d) out[d] += w * load_elem(c->v_cache, c->dtype, vo + d);
    }
  }
  if (lse) *lse = mx + log(denom);
  free(logit);
  return 0;
}

/* bfloat16 (1 sign, 8 exponent, 7 fraction bits) nearest to each double, ties to the even fraction, as bit
 * patterns. The rounding is done on the double itself (never through float first, which would round twice):
 * a finite non-zero x lies in [2^e, 2^(e+1)); bf16 numbers there are multiples of ulp = 2^(e-7) (2^-133 in the
 * subnormal range e < -126); x / ulp is exact in double and rint() rounds it half-to-even. A result of 2^128 or
 * more is infinity. NaN gives a quiet NaN. */
void oracle_round_bf16(const double* x, int64_t n, uint16_t* bits) {
  for (int64_t i = 0; i < n; ++i) {
    const double v = x[i];
    const uint16_t sign = signbit(v) ? 0x8000u : 0u;
    if (isnan(v)) { bits[i] = 0x7fc0u; continue; }
    const double a = fabs(v);
    if (isinf(a)) { bits[i] = (uint16_t)(sign | 0x7f80u); continue; }
    if (a == 0.0) { bits[i] = sign; continue; }
    int ex;
    (void)frexp(a, &ex);           /* a = m * 2^ex with m in [0.5, 1) */
    int e = ex - 1;                /* a in [2^e, 2^(e+1)) */
    if (e < -126) e = -126;        /* subnormals share the spacing of the smallest normal binade */
    const double ulp = ldexp(1.0, e - 7);
    const double r = rint(a / ulp) * ulp;   /* default rounding mode: nearest, ties to even */
    if (r >= ldexp(1.0, 128)) { bits[i] = (uint16_t)(sign | 0x7f80u); continue; }
    const float f = (float)r;      /* exact: r has at most 8 significant bits and is within float range */
    uint32_t u;
    memcpy(&u, &f, 4);
    bits[i] = (uint16_t)(sign | (uint16_t)(u >> 16));
  }
}

/* ---- whole-batch drivers (the same functions, looped over rows with OpenMP) ---- */

/* Stats of every logical page of every (b, hkv) that overlaps tokens
 * [tok_begin[b], tok_end[b]) (NULL, NULL = all pages), written into the logical
 * stat cache mean_all [B][Hkv][max_pages_per_seq][D], std_all [B][Hkv][max_pages_per_seq]. */
int oracle_update_stats(const oracle_cache* c, const int32_t* tok_begin, const int32_t* tok_end,
                        double* mean_all, double* std_all) {
  const int rows = c->B * c->Hkv;
  int err = 0;
#pragma omp parallel for schedule(dynamic, 1)
  for (int r = 0; r < rows; ++r) {
    const int b = r / c->Hkv, hkv = r % c->Hkv;
    const int P = num_pages(c, b);
    int p0 = 0, p1 = P;
    if (tok_begin && tok_end) {
      int t0 = tok_begin[b], t1 = tok_end[b];
      if (t1 > c->seq_lens[b]) t1 = c->seq_lens[b];
      if (t0 < 0) t0 = 0;
      if (t0 >= t1) continue;
      p0 = t0 / c->S;
      p1 = (t1 - 1) / c->S + 1;
    }
    const int64_t base = (int64_t)r * c->max_pages_per_seq;
    if (oracle_page_stats(c, b, hkv, p0, p1, mean_all + (base + p0) * c->D, std_all + base + p0) != 0) {
#pragma omp atomic write
      err = -1;
    }
  }
  return err;
}

/* One decode step for the whole batch from cached stats: Eq. 6 scores, top-k set,
 * Eq. 5 attention over it.  sel: [B][Hkv][top_k] logical pages in ascending order
 * (-1 padded); sel_count: [B][Hkv]; scores_all (optional): [B][Hkv][max_pages_per_seq];
 * out: [B][H][D]; lse: [B][H]. */
int oracle_sparse_decode_step(const oracle_cache* c, const void* q, const double* mean_all,
                              const double* std_all, double lambda, int top_k, double sm_scale,
                              int32_t* sel, int32_t* sel_count, double* scores_all,
                              double* out, double* lse) {
  const int rows = c->B * c->Hkv, G = c->H / c->Hkv;
  int err = 0;
#pragma omp parallel for schedule(dynamic, 1)
  for (int r = 0; r < rows; ++r) {
    const int b = r / c->Hkv, hkv = r % c->Hkv;
    const int P = num_pages(c, b);
    const int64_t base = (int64_t)r * c->max_pages_per_seq;
    double* sc = (double*)malloc(sizeof(double) * (size_t)(P > 0 ? P : 1));
    int32_t* order = (int32_t*)malloc(sizeof(int32_t) * (size_t)(P > 0 ? P : 1));
    int rc = oracle_page_scores(c, q, b, hkv, lambda, P, mean_all + base * c->D, std_all + base, sc);
    const int kb = oracle_topk(sc, P, top_k, order);
    /* the set, written in ascending page order */
    int32_t* row_sel = sel + (int64_t)r * top_k;
    int cnt = 0;
    char* in = (char*)calloc((size_t)(P > 0 ? P : 1), 1);
    for (int i = 0; i < kb; ++i) in[order[i]] = 1;
    for (int p = 0; p < P; ++p) if (in[p]) row_sel[cnt++] = p;
    for (int i = cnt; i < top_k; ++i) row_sel[i] = -1;
    sel_count[r] = kb;
    if (scores_all) for (int p = 0; p < P; ++p) scores_all[base + p] = sc[p];
    for (int g = 0; g < G && rc == 0; ++g) {
      const int h = hkv * G + g;
      rc = oracle_attention(c, q, b, h, row_sel, kb, sm_scale,
                            out + ((int64_t)b * c->H + h) * c->D, lse + (int64_t)b * c->H + h);
    }
    free(in); free(order); free(sc);
    if (rc != 0) {
#pragma omp atomic write
      err = rc;
    }
  }
  return err;
}

/* Eq. 4 for every (b, h). */
int oracle_dense_decode(const oracle_cache* c, const void* q, double sm_scale, double* out, double* lse) {
  const int rows = c->B * c->H;
  int err = 0;
#pragma omp parallel for schedule(dynamic, 1)
  for (int r = 0; r < rows; ++r) {
    const int b = r / c->H, h = r % c->H;
    const int P = num_pages(c, b);
    int32_t* all = (int32_t*)malloc(sizeof(int32_t) * (size_t)(P > 0 ? P : 1));
    for (int p = 0; p < P; ++p) all[p] = p;
    int rc = oracle_attention(c, q, b, h, all, P, sm_scale, out + (int64_t)r * c->D, lse + r);
    free(all);
    if (rc != 0) {
#pragma omp atomic write
      err = rc;
    }
  }
  return err;
}

/* Eq. 5 for every (b, h) over a GIVEN page list per (b, kv head): sel [B][Hkv][sel_stride] logical pages (the first
 * sel_count[b][hkv] entries of a row are used). A row with no entries gives a zero output and lse = -inf.
 * out: [B][H][D]; lse: [B][H]. */
int oracle_attention_rows(const oracle_cache* c, const void* q, const int32_t* sel, const int32_t* sel_count,
                          int sel_stride, double sm_scale, double* out, double* lse) {
  const int rows = c->B * c->H, G = c->H / c->Hkv;
  int err = 0;
#pragma omp parallel for schedule(dynamic, 1)
  for (int r = 0; r < rows; ++r) {
    const int b = r / c->H, h = r % c->H, hkv = h / G;
    const int64_t lrow = (int64_t)b * c->Hkv + hkv;
    const int n = sel_count[lrow];
    int rc = 0;
    if (n <= 0) {
      for (int d = 0; d < c->D; ++d) out[(int64_t)r * c->D + d] = 0.0;
      lse[r] = -INFINITY;
    } else {
      rc = oracle_attention(c, q, b, h, sel + lrow * sel_stride, n, sm_scale, out + (int64_t)r * c->D, lse + r);
    }
    if (rc != 0) {
#pragma omp atomic write
      err = rc;
    }
  }
  return err;
}
