/*
 * RocketKV reference oracle -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, fp64 CPU implementation of the two RocketKV stages, written
 * from the paper (arXiv 2502.14051) so that the GPU library can be checked
 * against it.  Nothing in the product path may call into this file; it shares
 * no code, header or table with the GPU kernels.
 *
 *   Stage 2, hybrid sparse attention (HSA): Section 3.4 Steps 1-3, Algorithm 1.
 *   Stage 1, GQA-aware SnapKV with a wide pooling kernel: Section 3.3,
 *   hyper-parameters from Appendix A.3.
 *   Budget split helper: Section 3.6.
 *
 * Inputs are bf16 bit patterns (uint16_t); every value is widened to double
 * on read and all arithmetic is double.  Layouts are the oracle's own, plain
 * and contiguous (token-major K and V); they are NOT the GPU library's paged
 * layouts.  Batch-level entry points parallelise over (sequence, KV head)
 * with OpenMP and do nothing else clever.
 *
 * Readings of the paper taken where it is silent (each is listed in the
 * design notes of the repository):
 *   - score(q[i1], P) of Algorithm 1 is the raw group-summed dot product
 *     sum_c (sum_h q[h][c]) * P[c][page]; no softmax, no 1/sqrt(D).
 *   - k2 counts pages: kp = all pages if T >= n, else max(1, min(P, T/ps)).
 *   - both top-k's: larger value first, then lower index; results ascending.
 *   - a partial tail page is summarised over its valid tokens only.
 *   - sign(0) picks K_max (Algorithm 1: g >= 0 -> K_max).
 *   - SnapKV: causal softmax over the whole visible row (prefix + window),
 *     votes only on prefix columns, group-sum THEN max-pool, budget N
 *     includes the W window tokens, kept tokens in ascending position.
 *     The group-sum/pool order and the "N includes W" choice are not fixed
 *     by the paper: PARITY UNPINNED for those two readings.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static inline double bf16_val(uint16_t bits) {
  uint32_t u = ((uint32_t)bits) << 16;
  float f;
  memcpy(&f, &u, sizeof f);
  return (double)f;
}

int okv_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* ------------------------------------------------------------------ */
/* generic top-k: larger value first, ties to the lower index;         */
/* result written in ascending index order.                            */
/* ------------------------------------------------------------------ */
typedef struct { double v; int i; } okv_pair;

static int okv_pair_cmp(const void* pa, const void* pb) {
  const okv_pair* a = (const okv_pair*)pa;
  const okv_pair* b = (const okv_pair*)pb;
  if (a->v > b->v) return -1;
  if (a->v < b->v) return 1;
  return (a->i > b->i) - (a->i < b->i);
}
static int okv_int_cmp(const void* pa, const void* pb) {
  int a = *(const int*)pa, b = *(const int*)pb;
  return (a > b) - (a < b);
}

void okv_topk(const double* v, int n, int k, int* idx_out) {
  if (k > n) k = n;
  if (k <= 0) return;
  okv_pair* p = (okv_pair*)malloc(sizeof(okv_pair) * (size_t)n);
  for (int i = 0; i < n; ++i) { p[i].v = v[i]; p[i].i = i; }
  qsort(p, (size_t)n, sizeof(okv_pair), okv_pair_cmp);
  for (int i = 0; i < k; ++i) idx_out[i] = p[i].i;
  qsort(idx_out, (size_t)k, sizeof(int), okv_int_cmp);
  free(p);
}

/* ------------------------------------------------------------------ */
/* HSA Step 1 (Section 3.4): per-page element-wise max / min of K.     */
/* K: [n][D] bf16.  kmax, kmin: [D][P] double, P = ceil(n/ps),         */
/* channel-major (one row of P page values per channel).               */
/* ------------------------------------------------------------------ */
void okv_page_summaries(const uint16_t* K, int n, int D, int ps,
                        double* kmax, double* kmin) {
  int P = (n + ps - 1) / ps;
  for (int p = 0; p < P; ++p) {
    int j0 = p * ps, j1 = j0 + ps < n ? j0 + ps : n;
    for (int c = 0; c < D; ++c) {
      double mx = bf16_val(K[(size_t)j0 * D + c]), mn = mx;
      for (int j = j0 + 1; j < j1; ++j) {
        double x = bf16_val(K[(size_t)j * D + c]);
        if (x > mx) mx = x;
        if (x < mn) mn = x;
      }
      kmax[(size_t)c * P + p] = mx;
      kmin[(size_t)c * P + p] = mn;
    }
  }
}

/* ------------------------------------------------------------------ */
/* Algorithm 1, first two assignments: a = sum_group |q|, s = sum_group */
/* q, i1 = argtopk(a, k1).  q: [G][D] bf16.                            */
/* ------------------------------------------------------------------ */
void okv_channel_select(const uint16_t* q, int G, int D, int k1,
                        double* a, double* s, int* i1) {
  for (int c = 0; c < D; ++c) {
    double sa = 0.0, ss = 0.0;
    for (int h = 0; h < G; ++h) {
      double x = bf16_val(q[(size_t)h * D + c]);
      sa += fabs(x);
      ss += x;
    }
    a[c] = sa;
    s[c] = ss;
  }
  okv_topk(a, D, k1, i1);
}

/* ------------------------------------------------------------------ */
/* Algorithm 1, P and s1: for each kept channel take the K_max row if   */
/* the group-summed q is >= 0, else the K_min row; the page score is    */
/* the dot product of the group-summed q with those rows.               */
/* ------------------------------------------------------------------ */
void okv_page_scores(const double* s, const int* i1, int k1,
                     const double* kmax, const double* kmin, int P,
                     double* score) {
  for (int p = 0; p < P; ++p) {
    double acc = 0.0;
    for (int t = 0; t < k1; ++t) {
      int c = i1[t];
      double bound = (s[c] >= 0.0) ? kmax[(size_t)c * P + p] : kmin[(size_t)c * P + p];
      acc += s[c] * bound;
    }
    score[p] = acc;
  }
}

/* number of pages picked for token budget T (reading of k2, see header) */
int okv_pages_to_pick(int n, int ps, int T) {
  int P = (n + ps - 1) / ps;
  if (P == 0) return 0;
  if (T >= n) return P;
  int kp = T / ps;
  if (kp < 1) kp = 1;
  if (kp > P) kp = P;
  return kp;
}

/* Algorithm 1, i2: top-kp pages; the last n_recent pages are always in. */
void okv_page_select(const double* score, int P, int kp, int n_recent, int* i2) {
  double* sc = (double*)malloc(sizeof(double) * (size_t)(P > 0 ? P : 1));
  memcpy(sc, score, sizeof(double) * (size_t)P);
  if (n_recent > kp) n_recent = kp;
  for (int r = 0; r < n_recent; ++r) sc[P - 1 - r] = INFINITY;
  okv_topk(sc, P, kp, i2);
  free(sc);
}

/* ------------------------------------------------------------------ */
/* Algorithm 1, y = attn(q, K[i2], V[i2]) (Section 3.4 Step 3): exact   */
/* softmax attention of every head of the group over the tokens of the  */
/* picked pages.  q: [G][D]; K, V: [n][D]; pages: kp ascending ids.     */
/* y: [G][D] double; lse: [G] natural-log sum-exp of the scaled logits. */
/* ------------------------------------------------------------------ */
void okv_attend_pages(const uint16_t* q, const uint16_t* K, const uint16_t* V,
                      int G, int D, int n, int ps, const int* pages, int kp,
                      double* y, double* lse) {
  double scale = 1.0 / sqrt((double)D);
  int cap = kp * ps > 0 ? kp * ps : 1;
  int* tok = (int*)malloc(sizeof(int) * (size_t)cap);
  double* l = (double*)malloc(sizeof(double) * (size_t)cap);
  int nt = 0;
  for (int t = 0; t < kp; ++t)
    for (int j = pages[t] * ps; j < (pages[t] + 1) * ps && j < n; ++j) tok[nt++] = j;
  for (int h = 0; h < G; ++h) {
    double* yh = y + (size_t)h * D;
    for (int c = 0; c < D; ++c) yh[c] = 0.0;
    if (nt == 0) { lse[h] = -INFINITY; continue; }
    double m = -INFINITY;
    for (int t = 0; t < nt; ++t) {
      double acc = 0.0;
      const uint16_t* kr = K + (size_t)tok[t] * D;
      for (int c = 0; c < D; ++c) acc += bf16_val(q[(size_t)h * D + c]) * bf16_val(kr[c]);
      l[t] = acc * scale;
      if (l[t] > m) m = l[t];
    }
    double z = 0.0;
    for (int t = 0; t < nt; ++t) { l[t] = exp(l[t] - m); z += l[t]; }
    for (int t = 0; t < nt; ++t) {
      double w = l[t] / z;
      const uint16_t* vr = V + (size_t)tok[t] * D;
      for (int c = 0; c < D; ++c) yh[c] += w * bf16_val(vr[c]);
    }
    lse[h] = m + log(z);
  }
  free(tok);
  free(l);
}

/* ------------------------------------------------------------------ */
/* One (sequence, KV head) unit of HSA decode, Algorithm 1 end to end,  */
/* summaries rebuilt from K (Step 1) each call.                         */
/* Optional outputs may be NULL.  pages_out needs room for P entries.   */
/* ------------------------------------------------------------------ */
void okv_hsa_unit(const uint16_t* q, const uint16_t* K, const uint16_t* V,
                  int G, int D, int n, int ps, int k1, int T, int n_recent,
                  double* y, double* lse, int* pages_out, int* kp_out,
                  int* chans_out, double* score_out) {
  int P = (n + ps - 1) / ps;
  int kp = okv_pages_to_pick(n, ps, T);
  if (kp_out) *kp_out = kp;
  double* a = (double*)malloc(sizeof(double) * (size_t)D);
  double* s = (double*)malloc(sizeof(double) * (size_t)D);
  int* i1 = (int*)malloc(sizeof(int) * (size_t)k1);
  okv_channel_select(q, G, D, k1, a, s, i1);
  if (chans_out) memcpy(chans_out, i1, sizeof(int) * (size_t)k1);
  int* i2 = (int*)malloc(sizeof(int) * (size_t)(P > 0 ? P : 1));
  if (P > 0) {
    double* kmax = (double*)malloc(sizeof(double) * (size_t)D * P);
    double* kmin = (double*)malloc(sizeof(double) * (size_t)D * P);
    double* score = (double*)malloc(sizeof(double) * (size_t)P);
    okv_page_summaries(K, n, D, ps, kmax, kmin);
    okv_page_scores(s, i1, k1, kmax, kmin, P, score);
    if (score_out) memcpy(score_out, score, sizeof(double) * (size_t)P);
    okv_page_select(score, P, kp, n_recent, i2);
    free(kmax); free(kmin); free(score);
  }
  if (pages_out) memcpy(pages_out, i2, sizeof(int) * (size_t)kp);
  okv_attend_pages(q, K, V, G, D, n, ps, i2, kp, y, lse);
  free(a); free(s); free(i1); free(i2);
}

/* ------------------------------------------------------------------ */
/* Batch HSA decode.  q: [B][Hq][D]; K, V: [B][Hkv][n_cap][D];          */
/* seq_lens: [B].  y: [B][Hq][D]; lse: [B][Hq];                         */
/* pages: [B][Hkv][pages_cap] (-1 padded); chans: [B][Hkv][k1];         */
/* scores: [B][Hkv][pages_cap] (optional, untouched beyond P).          */
/* ------------------------------------------------------------------ */
void okv_hsa_decode(const uint16_t* q, const uint16_t* K, const uint16_t* V,
                    const int* seq_lens, int B, int Hq, int Hkv, int D,
                    int n_cap, int ps, int k1, int T, int n_recent,
                    double* y, double* lse, int* pages, int pages_cap,
                    int* chans, double* scores) {
  int G = Hq / Hkv;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
  for (int b = 0; b < B; ++b)
    for (int g = 0; g < Hkv; ++g) {
      size_t u = (size_t)b * Hkv + g;
      int n = seq_lens[b];
      int P = (n + ps - 1) / ps;
      int* pg = (int*)malloc(sizeof(int) * (size_t)(P > 0 ? P : 1));
      int kp = 0;
      okv_hsa_unit(q + (u * G) * D, K + u * (size_t)n_cap * D, V + u * (size_t)n_cap * D,
                   G, D, n, ps, k1, T, n_recent,
                   y + (u * G) * D, lse + u * G, pg, &kp,
                   chans ? chans + u * k1 : NULL,
                   scores ? scores + u * pages_cap : NULL);
      if (pages) {
        for (int t = 0; t < pages_cap; ++t) pages[u * pages_cap + t] = t < kp ? pg[t] : -1;
      }
      free(pg);
    }
}

/* Batch dense attention: every page picked (the Full-KV row of Table 1). */
void okv_dense_decode(const uint16_t* q, const uint16_t* K, const uint16_t* V,
                      const int* seq_lens, int B, int Hq, int Hkv, int D, int n_cap,
                      double* y, double* lse) {
  int G = Hq / Hkv;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
  for (int b = 0; b < B; ++b)
    for (int g = 0; g < Hkv; ++g) {
      size_t u = (size_t)b * Hkv + g;
      int n = seq_lens[b];
      int* pg = (int*)malloc(sizeof(int) * (size_t)(n > 0 ? n : 1));
      for (int j = 0; j < n; ++j) pg[j] = j;
      okv_attend_pages(q + (u * G) * D, K + u * (size_t)n_cap * D, V + u * (size_t)n_cap * D,
                       G, D, n, 1, pg, n, y + (u * G) * D, lse + u * G);
      free(pg);
    }
}

/* Batch attention over a GIVEN page list (used to re-evaluate Step 3 on a
 * list that came from elsewhere).  pages: [B][Hkv][pages_cap], -1 ends a row. */
void okv_attend_given(const uint16_t* q, const uint16_t* K, const uint16_t* V,
                      const int* seq_lens, int B, int Hq, int Hkv, int D, int n_cap,
                      int ps, const int* pages, int pages_cap,
                      double* y, double* lse) {
  int G = Hq / Hkv;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
  for (int b = 0; b < B; ++b)
    for (int g = 0; g < Hkv; ++g) {
      size_t u = (size_t)b * Hkv + g;
      const int* pg = pages + u * pages_cap;
      int kp = 0;
      while (kp < pages_cap && pg[kp] >= 0) ++kp;
      okv_attend_pages(q + (u * G) * D, K + u * (size_t)n_cap * D, V + u * (size_t)n_cap * D,
                       G, D, seq_lens[b], ps, pg, kp, y + (u * G) * D, lse + u * G);
    }
}

/* Batch Step 1.  K: [B][Hkv][n_cap][D]; kmax/kmin: [B][Hkv][D][pages_cap]
 * double; columns p >= P of a sequence are left untouched. */
void okv_build_summaries(const uint16_t* K, const int* seq_lens, int B, int Hkv, int D,
                         int n_cap, int ps, int pages_cap, double* kmax, double* kmin) {
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
  for (int b = 0; b < B; ++b)
    for (int g = 0; g < Hkv; ++g) {
      size_t u = (size_t)b * Hkv + g;
      int n = seq_lens[b];
      int P = (n + ps - 1) / ps;
      if (P == 0) continue;
      double* mx = (double*)malloc(sizeof(double) * (size_t)D * P);
      double* mn = (double*)malloc(sizeof(double) * (size_t)D * P);
      okv_page_summaries(K + u * (size_t)n_cap * D, n, D, ps, mx, mn);
      for (int c = 0; c < D; ++c)
        for (int p = 0; p < P; ++p) {
          kmax[(u * D + c) * pages_cap + p] = mx[(size_t)c * P + p];
          kmin[(u * D + c) * pages_cap + p] = mn[(size_t)c * P + p];
        }
      free(mx); free(mn);
    }
}

/* ------------------------------------------------------------------ */
/* Stage 1 (Section 3.3): SnapKV with per-group selection.              */
/* One (sequence, KV head) unit.                                        */
/*   qobs: [G][W][D]  queries of the last W prompt positions            */
/*   K:    [S][D]     prompt keys                                       */
/*   gv:   [S-W]      out: group-summed, window-summed attention mass   */
/*   pooled: [S-W]    out: max-pool of gv, kernel ks (odd), stride 1,   */
/*                    edges clipped to the prefix                       */
/*   kept: [min(S,N)] out: kept positions, ascending                    */
/* returns the number kept.  gv / pooled may be NULL.                   */
/* ------------------------------------------------------------------ */
int okv_snapkv_unit(const uint16_t* qobs, const uint16_t* K, int G, int W, int D,
                    int S, int ks, int N, double* gv_out, double* pooled_out, int* kept) {
  if (S <= N) {
    for (int j = 0; j < S; ++j) kept[j] = j;
    return S;
  }
  int L = S - W; /* prefix length */
  double scale = 1.0 / sqrt((double)D);
  double* gv = (double*)calloc((size_t)L, sizeof(double));
  double* l = (double*)malloc(sizeof(double) * (size_t)S);
  for (int h = 0; h < G; ++h)
    for (int w = 0; w < W; ++w) {
      int t = L + w; /* absolute position of this query: sees keys 0..t */
      const uint16_t* qr = qobs + ((size_t)h * W + w) * D;
      double m = -INFINITY;
      for (int j = 0; j <= t; ++j) {
        double acc = 0.0;
        const uint16_t* kr = K + (size_t)j * D;
        for (int c = 0; c < D; ++c) acc += bf16_val(qr[c]) * bf16_val(kr[c]);
        l[j] = acc * scale;
        if (l[j] > m) m = l[j];
      }
      double z = 0.0;
      for (int j = 0; j <= t; ++j) { l[j] = exp(l[j] - m); z += l[j]; }
      for (int j = 0; j < L; ++j) gv[j] += l[j] / z;
    }
  free(l);
  double* pooled = (double*)malloc(sizeof(double) * (size_t)L);
  int r = (ks - 1) / 2;
  for (int j = 0; j < L; ++j) {
    int lo = j - r < 0 ? 0 : j - r, hi = j + r > L - 1 ? L - 1 : j + r;
    double mx = gv[lo];
    for (int i = lo + 1; i <= hi; ++i) if (gv[i] > mx) mx = gv[i];
    pooled[j] = mx;
  }
  int keep_prefix = N - W;
  okv_topk(pooled, L, keep_prefix, kept);
  for (int w = 0; w < W; ++w) kept[keep_prefix + w] = L + w;
  if (gv_out) memcpy(gv_out, gv, sizeof(double) * (size_t)L);
  if (pooled_out) memcpy(pooled_out, pooled, sizeof(double) * (size_t)L);
  free(gv); free(pooled);
  return N;
}

/* Batch SnapKV.  qobs: [B][Hq][W][D]; K: [B][Hkv][S_cap][D]; seq_lens: [B].
 * kept: [B][Hkv][N] (-1 padded when S_b < N); n_kept: [B];
 * gv, pooled: [B][Hkv][S_cap] optional (first S_b-W entries written). */
void okv_snapkv(const uint16_t* qobs, const uint16_t* K, const int* seq_lens,
                int B, int Hq, int Hkv, int D, int S_cap, int W, int ks, int N,
                int* kept, int* n_kept, double* gv, double* pooled) {
  int G = Hq / Hkv;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
  for (int b = 0; b < B; ++b)
    for (int g = 0; g < Hkv; ++g) {
      size_t u = (size_t)b * Hkv + g;
      int S = seq_lens[b];
      int* kp = kept + u * N;
      for (int i = 0; i < N; ++i) kp[i] = -1;
      int cnt = okv_snapkv_unit(qobs + u * G * (size_t)W * D, K + u * (size_t)S_cap * D,
                                G, W, D, S, ks, N,
                                gv ? gv + u * S_cap : NULL,
                                pooled ? pooled + u * S_cap : NULL, kp);
      if (g == 0) n_kept[b] = cnt;
    }
}

/* ------------------------------------------------------------------ */
/* Section 3.6: adaptive compression decomposition.                     */
/* c = S / t; r = min(0.2 + 0.06 log2 c, 0.8); stage 1 gets c^r, stage  */
/* 2 gets c^(1-r), split into page size ceil(c^((1-r)/2)) and a head-   */
/* dimension ratio c^(1-r) / page.  out: r, c1, c2, page, head_ratio.   */
/* ------------------------------------------------------------------ */
void okv_decompose(double c, double* out) {
  double r = 0.2 + 0.06 * log2(c);
  if (r > 0.8) r = 0.8;
  double c1 = pow(c, r), c2 = pow(c, 1.0 - r);
  double page = ceil(pow(c, (1.0 - r) / 2.0));
  out[0] = r; out[1] = c1; out[2] = c2; out[3] = page; out[4] = c2 / page;
}

/* Table 1, rows RocketKV and RocketKV-MT: storage (KV cache plus the K_max / */
/* K_min tensors) and traffic relative to the full KV cache at compression   */
/* ratio c, as printed: 1/c^r + 2/c^((1+r)/2), 1 + 2/c^((1+r)/2), 1/c.       */
/* out: storage, storage_mt, traffic.                                        */
void okv_cost_model(double c, double* out) {
  double sp[5];
  okv_decompose(c, sp);
  double r = sp[0];
  double aux = 2.0 / pow(c, (1.0 + r) / 2.0);
  out[0] = 1.0 / pow(c, r) + aux;
  out[1] = 1.0 + aux;
  out[2] = 1.0 / c;
}

/* Integer operating point that follows from the split when the budget t is   */
/* shared evenly by Step 2 and Step 3 (Appendix A.3): Stage 1 keeps S / c^r   */
/* tokens, Step 2 reads D / head_ratio channels of one summary row per page,  */
/* Step 3 attends to t / 2 tokens.  c below 1 (budget above the sequence) is  */
/* taken as 1: nothing is compressed.  Rounding to nearest is this build's    */
/* reading; the paper prints only the real-valued ratios.                     */
/* out: page, keep, channels, attend_tokens.                                  */
void okv_decompose_budget(long long S, int t, int D, int* out) {
  double c = (double)S / (double)t;
  if (c < 1.0) c = 1.0;
  double sp[5];
  okv_decompose(c, sp);
  long long keep = (long long)floor((double)S / sp[1] + 0.5);
  if (keep < 1) keep = 1;
  if (keep > S) keep = S;
  int k1 = (int)floor((double)D / sp[4] + 0.5);
  if (k1 < 1) k1 = 1;
  if (k1 > D) k1 = D;
  int T = t / 2;
  if (T < 1) T = 1;
  out[0] = (int)sp[3]; out[1] = (int)keep; out[2] = k1; out[3] = T;
}
