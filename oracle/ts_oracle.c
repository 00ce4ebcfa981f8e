/*
 * CPU oracle for query-aware page selection + sparse decode attention.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference the GPU
 * library is checked against.  It shares no code with the HIP path, is never
 * called by the product path, and is written directly from the paper's
 * definitions (TinyServe, Section 3.4 "query-aware routing at page
 * granularity", Section 3.5 "Query-Aware Page Selection", Eq. 1-2, and the
 * four steps of Algorithm 1).  All arithmetic is fp64; inputs are bf16 bit
 * patterns decoded exactly to double.
 *
 * Inputs are the *logical* tensors of the paper (keys and values indexed by
 * sequence, KV head and token position); paging through a block table is a
 * storage matter of the GPU library and does not appear here.
 *
 * Logical shapes (row-major, last index fastest):
 *   K, V       bf16 bits  [B][Hkv][Lmax][d]     tokens t >= seq_lens[b] ignored
 *   q          bf16 bits  [B][Hq][d]            Hq = G * Hkv, q head g belongs
 *                                               to KV head g / G
 *   page_min,
 *   page_max   bf16 bits  [B][Hkv][Pmax][d]
 *   scores     double     [B][Hkv][Pmax]        -inf for pages j >= P_b
 *   sel        int32      [B][Hkv][Kmax]        ascending page ids, -1 padded
 *   sel_count  int32      [B]
 *   out        double     [B][Hq][d]
 * with P_b = ceil(seq_lens[b] / S)  (Section 3.5: P = ceil(t / S)).
 *
 * Pins (tests/test_oracle_pins.py): hand-worked two-page example, the bound
 * invariant r >= max q.k, K = P  ==> dense softmax attention (checked against
 * a library routine), brute force over all page subsets on tiny inputs,
 * closed forms for constant pages, append == rebuild.  The INT8 cache functions
 * at the end of the file are pinned to the bf16 ones (scales that are powers of
 * two make the two caches hold the same numbers) and by hand-worked values.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

static double bf16_to_double(uint16_t bits) {
  uint32_t w = ((uint32_t)bits) << 16;
  float f;
  memcpy(&f, &w, sizeof f);
  return (double)f;
}

/* IEEE binary16 (1 sign, 5 exponent, 10 fraction bits), decoded by its definition. */
static double half_to_double(uint16_t bits) {
  int sign = bits >> 15, e = (bits >> 10) & 31, m = bits & 1023;
  double v;
  if (e == 0) v = ldexp((double)m, -24);                 /* zero and subnormals: m * 2^-24 */
  else if (e == 31) v = m ? NAN : INFINITY;
  else v = ldexp(1.0 + (double)m / 1024.0, e - 15);
  return sign ? -v : v;
}

/* Element format of the 16-bit inputs (queries, keys, values, metadata) of the
 * functions of the paper's path: 0 = bf16 (the default), 1 = IEEE half, the
 * "FP16" the paper's experiments run in (Section 4, experimental set-up).
 * Nothing else changes with it: every value is decoded exactly to double.  The
 * INT8 cache functions at the end of this file always take bf16 queries. */
static int g_elem_half = 0;
void tso_set_element_format(int half) { g_elem_half = half ? 1 : 0; }

static double elem_to_double(uint16_t bits) {
  return g_elem_half ? half_to_double(bits) : bf16_to_double(bits);
}

void tso_decode_elements(const uint16_t* bits, int n, double* out) {
  for (int i = 0; i < n; ++i) out[i] = elem_to_double(bits[i]);
}

static int pages_of(int len, int S) { return (len + S - 1) / S; }

int tso_version(void) { return 4; }

int tso_max_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* Threads the one OpenMP loop of this file (the attention over query heads) may
 * use from now on; n <= 0 restores the default.  For timing only. */
void tso_set_num_threads(int n) {
#ifdef _OPENMP
  static int initial = 0;
  if (initial == 0) initial = omp_get_max_threads();
  omp_set_num_threads(n > 0 ? n : initial);
#else
  (void)n;
#endif
}

/* Section 3.4 / Eq. 1: phi(K_j) = (m_j, M_j), the channel-wise min and max of
 * the keys stored in page j.  Only tokens t < seq_lens[b] exist; a partly
 * filled last page is summarised over the tokens it holds.  Rows of pages
 * j >= P_b are left untouched. */
void tso_build_page_meta(const uint16_t* K, const int32_t* seq_lens, int B, int Hkv, int Lmax,
                         int d, int S, int Pmax, uint16_t* page_min, uint16_t* page_max) {
  for (int b = 0; b < B; ++b) {
    int Pb = pages_of(seq_lens[b], S);
    for (int h = 0; h < Hkv; ++h) {
      const uint16_t* Kbh = K + ((size_t)b * Hkv + h) * (size_t)Lmax * d;
      for (int j = 0; j < Pb && j < Pmax; ++j) {
        int t0 = j * S;
        int t1 = t0 + S < seq_lens[b] ? t0 + S : seq_lens[b];
        uint16_t* mrow = page_min + (((size_t)b * Hkv + h) * Pmax + j) * d;
        uint16_t* Mrow = page_max + (((size_t)b * Hkv + h) * Pmax + j) * d;
        for (int c = 0; c < d; ++c) {
          uint16_t lo = Kbh[(size_t)t0 * d + c], hi = lo;
          for (int t = t0 + 1; t < t1; ++t) {
            uint16_t x = Kbh[(size_t)t * d + c];
            if (elem_to_double(x) < elem_to_double(lo)) lo = x;
            if (elem_to_double(x) > elem_to_double(hi)) hi = x;
          }
          mrow[c] = lo;
          Mrow[c] = hi;
        }
      }
    }
  }
}

/* Section 3.4 says the metadata "is maintained" while the cache grows; the
 * reading taken here: the token appended at position p = seq_lens[b] belongs
 * to page p / S; it opens that page when p % S == 0 (m = M = k) and otherwise
 * widens the page's box.  seq_lens is NOT modified (the caller advances it). */
void tso_append_token_meta(const uint16_t* k_new /*[B][Hkv][d]*/, const int32_t* seq_lens, int B,
                           int Hkv, int d, int S, int Pmax, uint16_t* page_min,
                           uint16_t* page_max) {
  for (int b = 0; b < B; ++b) {
    int p = seq_lens[b];
    int j = p / S;
    if (j >= Pmax) continue;
    for (int h = 0; h < Hkv; ++h) {
      uint16_t* mrow = page_min + (((size_t)b * Hkv + h) * Pmax + j) * d;
      uint16_t* Mrow = page_max + (((size_t)b * Hkv + h) * Pmax + j) * d;
      const uint16_t* k = k_new + ((size_t)b * Hkv + h) * d;
      for (int c = 0; c < d; ++c) {
        if (p % S == 0) {
          mrow[c] = k[c];
          Mrow[c] = k[c];
        } else {
          if (elem_to_double(k[c]) < elem_to_double(mrow[c])) mrow[c] = k[c];
          if (elem_to_double(k[c]) > elem_to_double(Mrow[c])) Mrow[c] = k[c];
        }
      }
    }
  }
}

/* Eq. 2 (and step 1 of Algorithm 1): the directional bounding-box estimator
 *   r(q, phi_j) = sum_i  q_i * (q_i >= 0 ? M_ji : m_ji).
 * For grouped-query attention the page score of a KV head is the sum of r over
 * the G query heads that share it.  form == 1 evaluates the equivalent
 * max(q_i*m_ji, q_i*M_ji) expression instead of the sign test. */
void tso_score_pages(const uint16_t* q, const uint16_t* page_min, const uint16_t* page_max,
                     const int32_t* seq_lens, int B, int Hq, int Hkv, int d, int S, int Pmax,
                     int form, double* scores) {
  int G = Hq / Hkv;
  for (int b = 0; b < B; ++b) {
    int Pb = pages_of(seq_lens[b], S);
    for (int h = 0; h < Hkv; ++h) {
      for (int j = 0; j < Pmax; ++j) {
        double* out = scores + ((size_t)b * Hkv + h) * Pmax + j;
        if (j >= Pb) {
          *out = -INFINITY;
          continue;
        }
        const uint16_t* mrow = page_min + (((size_t)b * Hkv + h) * Pmax + j) * d;
        const uint16_t* Mrow = page_max + (((size_t)b * Hkv + h) * Pmax + j) * d;
        double s = 0.0;
        for (int g = 0; g < G; ++g) {
          const uint16_t* qg = q + ((size_t)b * Hq + (size_t)h * G + g) * d;
          for (int c = 0; c < d; ++c) {
            double qc = elem_to_double(qg[c]);
            double lo = elem_to_double(mrow[c]), hi = elem_to_double(Mrow[c]);
            if (form == 1) {
              double a = qc * lo, bb = qc * hi;
              s += a > bb ? a : bb;
            } else {
              s += qc >= 0.0 ? qc * hi : qc * lo;
            }
          }
        }
        *out = s;
      }
    }
  }
}

typedef struct {
  double score;
  int32_t id;
  int32_t forced;
} tso_cand;

static int cand_before(const void* pa, const void* pb) {
  const tso_cand* a = (const tso_cand*)pa;
  const tso_cand* b = (const tso_cand*)pb;
  if (a->forced != b->forced) return b->forced - a->forced; /* always-kept pages first */
  if (a->score > b->score) return -1;
  if (a->score < b->score) return 1;
  return (a->id > b->id) - (a->id < b->id); /* equal scores: lower page id first */
}

static int int_asc(const void* pa, const void* pb) {
  int32_t a = *(const int32_t*)pa, b = *(const int32_t*)pb;
  return (a > b) - (a < b);
}

/* Section 3.5 (S_t = TopK_j r, |S_t| = K; step 2 of Algorithm 1).  Pages are
 * ranked by (score descending, page id ascending); the first
 * K_b = min(K, P_b) are kept and reported in ascending page id.  K is
 * topk_per_seq[b] when that pointer is non-NULL, else topk.
 * gap (nullable) receives, per (b, h), the relative distance between the last
 * kept and the first dropped score, |s_K - s_{K+1}| / max(|s_K|, |s_{K+1}|),
 * or +inf when nothing is dropped or the last kept page is an always-kept one.
 *
 * The paper selects by score alone (keep_first = keep_last = 0).  As an option
 * outside the paper, the first keep_first pages of a sequence (attention sinks)
 * and its last keep_last pages (the newest tokens) can be kept whatever their
 * score: they rank ahead of every other page (among themselves by page id) and
 * count towards K_b. */
void tso_select_topk_pages(const double* scores, const int32_t* seq_lens, int B, int Hkv, int S,
                           int Pmax, int topk, const int32_t* topk_per_seq, int Kmax,
                           int keep_first, int keep_last, int32_t* sel, int32_t* sel_count,
                           double* gap) {
  tso_cand* cand = (tso_cand*)malloc(sizeof(tso_cand) * (size_t)(Pmax > 0 ? Pmax : 1));
  for (int b = 0; b < B; ++b) {
    int Pb = pages_of(seq_lens[b], S);
    if (Pb > Pmax) Pb = Pmax;
    int K = topk_per_seq ? topk_per_seq[b] : topk;
    int Kb = K < Pb ? K : Pb;
    if (Kb > Kmax) Kb = Kmax;
    if (Kb < 0) Kb = 0;
    sel_count[b] = Kb;
    for (int h = 0; h < Hkv; ++h) {
      const double* s = scores + ((size_t)b * Hkv + h) * Pmax;
      int32_t* row = sel + ((size_t)b * Hkv + h) * Kmax;
      for (int j = 0; j < Pb; ++j) {
        cand[j].score = s[j];
        cand[j].id = j;
        cand[j].forced = (j < keep_first || j >= Pb - keep_last) ? 1 : 0;
        if (cand[j].forced) cand[j].score = 0.0; /* forced pages rank by id alone */
      }
      qsort(cand, (size_t)Pb, sizeof(tso_cand), cand_before);
      for (int i = 0; i < Kmax; ++i) row[i] = i < Kb ? cand[i].id : -1;
      qsort(row, (size_t)Kb, sizeof(int32_t), int_asc);
      if (gap) {
        double g = INFINITY;
        if (Kb > 0 && Kb < Pb && !cand[Kb - 1].forced) {
          double a = cand[Kb - 1].score, c = cand[Kb].score;
          double den = fabs(a) > fabs(c) ? fabs(a) : fabs(c);
          g = den > 0.0 ? fabs(a - c) / den : 0.0;
        }
        gap[(size_t)b * Hkv + h] = g;
      }
    }
  }
  free(cand);
}

/* Section 3.5, SparseAttn, and steps 3-4 of Algorithm 1: logits
 * a_i = scale * q.k_i over the tokens of the selected pages only,
 * alpha = softmax(a) over exactly those tokens, o = sum_i alpha_i v_i.
 * (The paper writes softmax(q.k) with no scale: scale = 1 is its literal
 * form.)  A (sequence, head) with no selected token yields o = 0.
 * lse (nullable, [B][Hq]): log of the softmax denominator, log sum_i exp(a_i)
 * over the same tokens (-inf with none): the share of the dense softmax mass
 * that falls on the selected tokens is exp(lse_selected - lse_all). */
void tso_sparse_decode_attention(const uint16_t* q, const uint16_t* K, const uint16_t* V,
                                 const int32_t* sel, const int32_t* sel_count,
                                 const int32_t* seq_lens, int B, int Hq, int Hkv, int Lmax, int d,
                                 int S, int Kmax, double scale, double* out, double* lse) {
  int G = Hq / Hkv;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 1)
#endif
  for (int bh = 0; bh < B * Hq; ++bh) {
    int b = bh / Hq, g = bh % Hq, h = g / G;
    const uint16_t* qg = q + ((size_t)b * Hq + g) * d;
    const uint16_t* Kbh = K + ((size_t)b * Hkv + h) * (size_t)Lmax * d;
    const uint16_t* Vbh = V + ((size_t)b * Hkv + h) * (size_t)Lmax * d;
    const int32_t* row = sel + ((size_t)b * Hkv + h) * Kmax;
    double* o = out + ((size_t)b * Hq + g) * d;
    int n = sel_count[b];
    int L = seq_lens[b];
    double* a = (double*)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1) * S);
    int32_t* tok = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1) * S);
    int cnt = 0;
    double amax = -INFINITY;
    for (int i = 0; i < n; ++i) {
      int j = row[i];
      for (int t = j * S; t < (j + 1) * S && t < L; ++t) {
        double dot = 0.0;
        for (int c = 0; c < d; ++c)
          dot += elem_to_double(qg[c]) * elem_to_double(Kbh[(size_t)t * d + c]);
        a[cnt] = scale * dot;
        tok[cnt] = t;
        if (a[cnt] > amax) amax = a[cnt];
        ++cnt;
      }
    }
    for (int c = 0; c < d; ++c) o[c] = 0.0;
    double denom = 0.0;
    for (int i = 0; i < cnt; ++i) {
      a[i] = exp(a[i] - amax);
      denom += a[i];
    }
    for (int i = 0; i < cnt; ++i) {
      double w = a[i] / denom;
      for (int c = 0; c < d; ++c) o[c] += w * elem_to_double(Vbh[(size_t)tok[i] * d + c]);
    }
    if (lse) lse[(size_t)b * Hq + g] = cnt > 0 ? amax + log(denom) : -INFINITY;
    free(a);
    free(tok);
  }
}

/* Dense decode attention over every cached token (the "Attn(q_t, K, V)"
 * expression opening Section 3.5); used only as the K = P special case. */
void tso_dense_decode_attention(const uint16_t* q, const uint16_t* K, const uint16_t* V,
                                const int32_t* seq_lens, int B, int Hq, int Hkv, int Lmax, int d,
                                double scale, double* out, double* lse) {
  int G = Hq / Hkv;
  for (int b = 0; b < B; ++b) {
    int L = seq_lens[b];
    for (int g = 0; g < Hq; ++g) {
      int h = g / G;
      const uint16_t* qg = q + ((size_t)b * Hq + g) * d;
      const uint16_t* Kbh = K + ((size_t)b * Hkv + h) * (size_t)Lmax * d;
      const uint16_t* Vbh = V + ((size_t)b * Hkv + h) * (size_t)Lmax * d;
      double* o = out + ((size_t)b * Hq + g) * d;
      double* a = (double*)malloc(sizeof(double) * (size_t)(L > 0 ? L : 1));
      double amax = -INFINITY;
      for (int t = 0; t < L; ++t) {
        double dot = 0.0;
        for (int c = 0; c < d; ++c)
          dot += elem_to_double(qg[c]) * elem_to_double(Kbh[(size_t)t * d + c]);
        a[t] = scale * dot;
        if (a[t] > amax) amax = a[t];
      }
      double denom = 0.0;
      for (int t = 0; t < L; ++t) {
        a[t] = exp(a[t] - amax);
        denom += a[t];
      }
      for (int c = 0; c < d; ++c) o[c] = 0.0;
      for (int t = 0; t < L; ++t) {
        double w = a[t] / denom;
        for (int c = 0; c < d; ++c) o[c] += w * elem_to_double(Vbh[(size_t)t * d + c]);
      }
      if (lse) lse[(size_t)b * Hq + g] = L > 0 ? amax + log(denom) : -INFINITY;
      free(a);
    }
  }
}

/* The whole decode step of Algorithm 1 for a batch: score -> select -> attend,
 * with the metadata given.  scores / sel / sel_count / gap are outputs too so
 * a caller can inspect every stage. */
void tso_query_aware_decode(const uint16_t* q, const uint16_t* K, const uint16_t* V,
                            const uint16_t* page_min, const uint16_t* page_max,
                            const int32_t* seq_lens, int B, int Hq, int Hkv, int Lmax, int d,
                            int S, int Pmax, int topk, const int32_t* topk_per_seq, int Kmax,
                            int keep_first, int keep_last, double scale, double* scores,
                            int32_t* sel, int32_t* sel_count, double* gap, double* out) {
  tso_score_pages(q, page_min, page_max, seq_lens, B, Hq, Hkv, d, S, Pmax, 0, scores);
  tso_select_topk_pages(scores, seq_lens, B, Hkv, S, Pmax, topk, topk_per_seq, Kmax, keep_first,
                        keep_last, sel, sel_count, gap);
  tso_sparse_decode_attention(q, K, V, sel, sel_count, seq_lens, B, Hq, Hkv, Lmax, d, S, Kmax,
                              scale, out, NULL);
}

/* True per-page maximum of q.k for one query head (the quantity Eq. 2
 * bounds from above); used by the invariant pin only.
 * page_best: double [B][Hq][Pmax], -inf for pages j >= P_b. */
void tso_true_page_max(const uint16_t* q, const uint16_t* K, const int32_t* seq_lens, int B,
                       int Hq, int Hkv, int Lmax, int d, int S, int Pmax, double* page_best) {
  int G = Hq / Hkv;
  for (int b = 0; b < B; ++b) {
    int L = seq_lens[b];
    for (int g = 0; g < Hq; ++g) {
      int h = g / G;
      const uint16_t* qg = q + ((size_t)b * Hq + g) * d;
      const uint16_t* Kbh = K + ((size_t)b * Hkv + h) * (size_t)Lmax * d;
      double* row = page_best + ((size_t)b * Hq + g) * Pmax;
      for (int j = 0; j < Pmax; ++j) row[j] = -INFINITY;
      for (int t = 0; t < L; ++t) {
        double dot = 0.0;
        for (int c = 0; c < d; ++c)
          dot += elem_to_double(qg[c]) * elem_to_double(Kbh[(size_t)t * d + c]);
        if (t / S < Pmax && dot > row[t / S]) row[t / S] = dot;
      }
    }
  }
}

/* ===========================================================================
 * INT8 KV cache.  Section 3.1 names "FP16/INT8 KV formats" for the sparse
 * attention executor and gives no format; the one defined here (and in the GPU
 * library's header) is an extension of this build:
 *   - keys and values are stored as int8 with one positive fp32 scale per
 *     (token, KV head): the key of token t is  k_t[c] = Kq[t][c] * ks[t]  as a
 *     real number (no rounding), likewise v_t[c] = Vq[t][c] * vs[t];
 *   - queries and page metadata stay bf16.  A page's box must contain its
 *     dequantised keys for Eq. 2 to remain an upper bound, so the channel-wise
 *     min is rounded DOWN to bf16 and the max UP;
 *   - a bf16 vector x is quantised as  scale = max_c |x_c| / 127  (1 if x = 0),
 *     xq_c = round-half-even(x_c / scale), both in fp32 arithmetic.
 * Everything after the metadata (Eq. 2, top-K, softmax attention over the
 * selected tokens) is the paper's, applied to the dequantised keys / values.
 *
 * Logical shapes: Kq, Vq int8 [B][Hkv][Lmax][d]; ks, vs float [B][Hkv][Lmax].
 * =========================================================================== */

/* fp32 -> bf16 bits, rounded towards -inf (up == 0) or +inf (up != 0). */
static uint16_t bf16_directed(float f, int up) {
  uint32_t w;
  memcpy(&w, &f, sizeof w);
  uint16_t hi = (uint16_t)(w >> 16);
  if ((w & 0xffffu) == 0u) return hi;            /* exactly representable */
  int negative = (w >> 31) != 0;
  /* truncation moves towards zero: that is down for positive values, up for negative */
  if (negative ? !up : up) hi = (uint16_t)(hi + 1); /* one bf16 step away from zero */
  return hi;
}

void tso_quantize_rows_i8(const uint16_t* x /*bf16 [n][d]*/, int n, int d, int8_t* xq /*[n][d]*/,
                          float* scale /*[n]*/) {
  for (int i = 0; i < n; ++i) {
    float amax = 0.0f;
    for (int c = 0; c < d; ++c) {
      float v = fabsf((float)bf16_to_double(x[(size_t)i * d + c]));
      if (v > amax) amax = v;
    }
    float s = amax > 0.0f ? amax / 127.0f : 1.0f;
    scale[i] = s;
    for (int c = 0; c < d; ++c) {
      float v = (float)bf16_to_double(x[(size_t)i * d + c]);
      float r = rintf(v / s);                    /* default rounding mode: half to even */
      if (r > 127.0f) r = 127.0f;
      if (r < -127.0f) r = -127.0f;
      xq[(size_t)i * d + c] = (int8_t)r;
    }
  }
}

/* Eq. 1 on the dequantised keys, box rounded outwards to bf16. */
void tso_build_page_meta_i8(const int8_t* Kq, const float* ks, const int32_t* seq_lens, int B,
                            int Hkv, int Lmax, int d, int S, int Pmax, uint16_t* page_min,
                            uint16_t* page_max) {
  for (int b = 0; b < B; ++b) {
    int Pb = pages_of(seq_lens[b], S);
    for (int h = 0; h < Hkv; ++h) {
      const int8_t* Kbh = Kq + ((size_t)b * Hkv + h) * (size_t)Lmax * d;
      const float* sbh = ks + ((size_t)b * Hkv + h) * (size_t)Lmax;
      for (int j = 0; j < Pb && j < Pmax; ++j) {
        int t0 = j * S;
        int t1 = t0 + S < seq_lens[b] ? t0 + S : seq_lens[b];
        uint16_t* mrow = page_min + (((size_t)b * Hkv + h) * Pmax + j) * d;
        uint16_t* Mrow = page_max + (((size_t)b * Hkv + h) * Pmax + j) * d;
        for (int c = 0; c < d; ++c) {
          double lo = INFINITY, hi = -INFINITY;
          for (int t = t0; t < t1; ++t) {
            double k = (double)Kbh[(size_t)t * d + c] * (double)sbh[t];
            if (k < lo) lo = k;
            if (k > hi) hi = k;
          }
          /* int8 x fp32 has at most 31 significant bits: the fp32 product below is the
           * real product rounded once; rounding it outwards again keeps the box closed
           * only if that first rounding did not cross the value, so round from double */
          float flo = (float)lo, fhi = (float)hi;
          if ((double)flo > lo) flo = nextafterf(flo, -INFINITY);
          if ((double)fhi < hi) fhi = nextafterf(fhi, INFINITY);
          mrow[c] = bf16_directed(flo, 0);
          Mrow[c] = bf16_directed(fhi, 1);
        }
      }
    }
  }
}

/* Incremental form: the appended token (already quantised) opens or widens the
 * box of page seq_lens[b] / S.  Must equal a rebuild, bit for bit. */
void tso_append_token_meta_i8(const int8_t* kq_new /*[B][Hkv][d]*/, const float* ks_new /*[B][Hkv]*/,
                              const int32_t* seq_lens, int B, int Hkv, int d, int S, int Pmax,
                              uint16_t* page_min, uint16_t* page_max) {
  for (int b = 0; b < B; ++b) {
    int p = seq_lens[b];
    int j = p / S;
    if (j >= Pmax) continue;
    for (int h = 0; h < Hkv; ++h) {
      uint16_t* mrow = page_min + (((size_t)b * Hkv + h) * Pmax + j) * d;
      uint16_t* Mrow = page_max + (((size_t)b * Hkv + h) * Pmax + j) * d;
      for (int c = 0; c < d; ++c) {
        double k = (double)kq_new[((size_t)b * Hkv + h) * d + c] * (double)ks_new[(size_t)b * Hkv + h];
        float flo = (float)k, fhi = (float)k;
        if ((double)flo > k) flo = nextafterf(flo, -INFINITY);
        if ((double)fhi < k) fhi = nextafterf(fhi, INFINITY);
        uint16_t lo = bf16_directed(flo, 0), hi = bf16_directed(fhi, 1);
        if (p % S == 0) {
          mrow[c] = lo;
          Mrow[c] = hi;
        } else {
          if (bf16_to_double(lo) < bf16_to_double(mrow[c])) mrow[c] = lo;
          if (bf16_to_double(hi) > bf16_to_double(Mrow[c])) Mrow[c] = hi;
        }
      }
    }
  }
}

/* Section 3.5 SparseAttn on the dequantised cache.  sel == NULL: every page of
 * the sequence (the dense attention the paper compares against). */
void tso_sparse_decode_attention_i8(const uint16_t* q, const int8_t* Kq, const float* ks,
                                    const int8_t* Vq, const float* vs, const int32_t* sel,
                                    const int32_t* sel_count, const int32_t* seq_lens, int B,
                                    int Hq, int Hkv, int Lmax, int d, int S, int Kmax,
                                    double scale, double* out, double* lse) {
  int G = Hq / Hkv;
  for (int bh = 0; bh < B * Hq; ++bh) {
    int b = bh / Hq, g = bh % Hq, h = g / G;
    const uint16_t* qg = q + ((size_t)b * Hq + g) * d;
    size_t base = ((size_t)b * Hkv + h) * (size_t)Lmax;
    double* o = out + ((size_t)b * Hq + g) * d;
    int L = seq_lens[b];
    int n = sel ? sel_count[b] : pages_of(L, S);
    double* a = (double*)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1) * S);
    int32_t* tok = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1) * S);
    int cnt = 0;
    double amax = -INFINITY;
    for (int i = 0; i < n; ++i) {
      int j = sel ? sel[((size_t)b * Hkv + h) * Kmax + i] : i;
      for (int t = j * S; t < (j + 1) * S && t < L; ++t) {
        double dot = 0.0;
        for (int c = 0; c < d; ++c)
          dot += bf16_to_double(qg[c]) * ((double)Kq[(base + t) * d + c] * (double)ks[base + t]);
        a[cnt] = scale * dot;
        tok[cnt] = t;
        if (a[cnt] > amax) amax = a[cnt];
        ++cnt;
      }
    }
    for (int c = 0; c < d; ++c) o[c] = 0.0;
    double denom = 0.0;
    for (int i = 0; i < cnt; ++i) {
      a[i] = exp(a[i] - amax);
      denom += a[i];
    }
    for (int i = 0; i < cnt; ++i) {
      double w = a[i] / denom;
      for (int c = 0; c < d; ++c)
        o[c] += w * ((double)Vq[(base + tok[i]) * d + c] * (double)vs[base + tok[i]]);
    }
    if (lse) lse[(size_t)b * Hq + g] = cnt > 0 ? amax + log(denom) : -INFINITY;
    free(a);
    free(tok);
  }
}

/* Algorithm 1 with the metadata given: Eq. 2 scores, top-K, attention over the
 * dequantised selected tokens. */
void tso_query_aware_decode_i8(const uint16_t* q, const int8_t* Kq, const float* ks,
                               const int8_t* Vq, const float* vs, const uint16_t* page_min,
                               const uint16_t* page_max, const int32_t* seq_lens, int B, int Hq,
                               int Hkv, int Lmax, int d, int S, int Pmax, int topk,
                               const int32_t* topk_per_seq, int Kmax, int keep_first,
                               int keep_last, double scale, double* scores, int32_t* sel,
                               int32_t* sel_count, double* gap, double* out) {
  tso_score_pages(q, page_min, page_max, seq_lens, B, Hq, Hkv, d, S, Pmax, 0, scores);
  tso_select_topk_pages(scores, seq_lens, B, Hkv, S, Pmax, topk, topk_per_seq, Kmax, keep_first,
                        keep_last, sel, sel_count, gap);
  tso_sparse_decode_attention_i8(q, Kq, ks, Vq, vs, sel, sel_count, seq_lens, B, Hq, Hkv, Lmax, d,
                                 S, Kmax, scale, out, NULL);
}
