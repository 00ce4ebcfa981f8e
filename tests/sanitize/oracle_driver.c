/* Runs every function of the CPU oracle on small seeded inputs, with exactly-sized
 * heap buffers, and prints a checksum of every output.  Built twice by
 * tests/test_sanitizers.py: with -fsanitize=address,undefined (any out-of-bounds
 * access, signed overflow, misaligned or invalid operation aborts the run) and
 * plainly; the two must print the same text.  Shapes include empty sequences, a
 * partly filled last page, K > P, grouped-query heads, always-kept pages, both
 * 16-bit element formats and the INT8 cache. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

void tso_set_element_format(int half);
void tso_set_num_threads(int n);
void tso_build_page_meta(const uint16_t*, const int32_t*, int, int, int, int, int, int, uint16_t*, uint16_t*);
void tso_append_token_meta(const uint16_t*, const int32_t*, int, int, int, int, int, uint16_t*, uint16_t*);
void tso_score_pages(const uint16_t*, const uint16_t*, const uint16_t*, const int32_t*, int, int, int, int, int, int, int, double*);
void tso_select_topk_pages(const double*, const int32_t*, int, int, int, int, int, const int32_t*, int, int, int, int32_t*, int32_t*, double*);
void tso_sparse_decode_attention(const uint16_t*, const uint16_t*, const uint16_t*, const int32_t*, const int32_t*, const int32_t*, int, int, int, int, int, int, int, double, double*, double*);
void tso_dense_decode_attention(const uint16_t*, const uint16_t*, const uint16_t*, const int32_t*, int, int, int, int, int, double, double*, double*);
void tso_query_aware_decode(const uint16_t*, const uint16_t*, const uint16_t*, const uint16_t*, const uint16_t*, const int32_t*, int, int, int, int, int, int, int, int, const int32_t*, int, int, int, double, double*, int32_t*, int32_t*, double*, double*);
void tso_true_page_max(const uint16_t*, const uint16_t*, const int32_t*, int, int, int, int, int, int, int, double*);
void tso_quantize_rows_i8(const uint16_t*, int, int, int8_t*, float*);
void tso_build_page_meta_i8(const int8_t*, const float*, const int32_t*, int, int, int, int, int, int, uint16_t*, uint16_t*);
void tso_append_token_meta_i8(const int8_t*, const float*, const int32_t*, int, int, int, int, int, uint16_t*, uint16_t*);
void tso_sparse_decode_attention_i8(const uint16_t*, const int8_t*, const float*, const int8_t*, const float*, const int32_t*, const int32_t*, const int32_t*, int, int, int, int, int, int, int, double, double*, double*);
void tso_query_aware_decode_i8(const uint16_t*, const int8_t*, const float*, const int8_t*, const float*, const uint16_t*, const uint16_t*, const int32_t*, int, int, int, int, int, int, int, int, const int32_t*, int, int, int, double, double*, int32_t*, int32_t*, double*, double*);

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd(void) {
  rng_state = rng_state * 6364136223846793005ull + 1442695040888963407ull;
  return (uint32_t)(rng_state >> 33);
}
/* a 16-bit float of moderate size: bf16 or half of a value in (-4, 4) with 3 fraction bits */
static uint16_t rnd_elem(int half) {
  int v = (int)(rnd() % 65) - 32;          /* -32 .. 32, eighths */
  float f = (float)v / 8.0f;
  uint32_t b;
  memcpy(&b, &f, 4);
  if (!half) return (uint16_t)(b >> 16);   /* exact: few significant bits */
  if (v == 0) return 0;
  {
    int e = (int)((b >> 23) & 0xff) - 127 + 15;
    return (uint16_t)(((b >> 16) & 0x8000u) | ((uint32_t)e << 10) | ((b >> 13) & 0x3ffu));
  }
}
static double sum_d(const double* x, size_t n) {
  double s = 0;
  for (size_t i = 0; i < n; ++i) if (isfinite(x[i])) s += x[i] * (double)(1 + i % 7);
  return s;
}
static long sum_i(const int32_t* x, size_t n) {
  long s = 0;
  for (size_t i = 0; i < n; ++i) s += (long)x[i] * (long)(1 + i % 5);
  return s;
}
static long sum_u16(const uint16_t* x, size_t n) {
  long s = 0;
  for (size_t i = 0; i < n; ++i) s += (long)x[i] * (long)(1 + i % 3);
  return s;
}
#define NEW(T, n) ((T*)calloc((n) > 0 ? (size_t)(n) : 1, sizeof(T)))

static void run_case(int id, int half, int B, int Hq, int Hkv, int d, int S, const int32_t* lens,
                     int topk, int Kmax, int keep_first, int keep_last, int per_seq) {
  int Lmax = 1, Pmax, b;
  size_t nK, nq, nmeta, i;
  for (b = 0; b < B; ++b) if (lens[b] > Lmax) Lmax = lens[b];
  Pmax = (Lmax + 1 + S - 1) / S + 1;       /* room for one appended token and a spare page */
  nK = (size_t)B * Hkv * Lmax * d; nq = (size_t)B * Hq * d; nmeta = (size_t)B * Hkv * Pmax * d;
  tso_set_element_format(half);
  uint16_t* K = NEW(uint16_t, nK); uint16_t* V = NEW(uint16_t, nK); uint16_t* q = NEW(uint16_t, nq);
  uint16_t* knew = NEW(uint16_t, (size_t)B * Hkv * d);
  uint16_t* pmin = NEW(uint16_t, nmeta); uint16_t* pmax = NEW(uint16_t, nmeta);
  int32_t* L = NEW(int32_t, B); int32_t* tps = NEW(int32_t, B);
  double* scores = NEW(double, (size_t)B * Hkv * Pmax); double* scores1 = NEW(double, (size_t)B * Hkv * Pmax);
  int32_t* sel = NEW(int32_t, (size_t)B * Hkv * Kmax); int32_t* cnt = NEW(int32_t, B);
  double* gap = NEW(double, (size_t)B * Hkv); double* out = NEW(double, nq); double* lse = NEW(double, (size_t)B * Hq);
  double* best = NEW(double, (size_t)B * Hq * Pmax);
  for (i = 0; i < nK; ++i) { K[i] = rnd_elem(half); V[i] = rnd_elem(half); }
  for (i = 0; i < nq; ++i) q[i] = rnd_elem(half);
  for (i = 0; i < (size_t)B * Hkv * d; ++i) knew[i] = rnd_elem(half);
  for (b = 0; b < B; ++b) { L[b] = lens[b]; tps[b] = 1 + (int)(rnd() % (unsigned)(Kmax)); }
  tso_build_page_meta(K, L, B, Hkv, Lmax, d, S, Pmax, pmin, pmax);
  printf("case %d meta %ld %ld\n", id, sum_u16(pmin, nmeta), sum_u16(pmax, nmeta));
  tso_score_pages(q, pmin, pmax, L, B, Hq, Hkv, d, S, Pmax, 0, scores);
  tso_score_pages(q, pmin, pmax, L, B, Hq, Hkv, d, S, Pmax, 1, scores1);
  printf("case %d scores %.6f %.6f\n", id, sum_d(scores, (size_t)B * Hkv * Pmax), sum_d(scores1, (size_t)B * Hkv * Pmax));
  tso_true_page_max(q, K, L, B, Hq, Hkv, Lmax, d, S, Pmax, best);
  printf("case %d true max %.6f\n", id, sum_d(best, (size_t)B * Hq * Pmax));
  tso_query_aware_decode(q, K, V, pmin, pmax, L, B, Hq, Hkv, Lmax, d, S, Pmax, topk, per_seq ? tps : NULL,
                         Kmax, keep_first, keep_last, 0.125, scores, sel, cnt, gap, out);
  printf("case %d decode sel %ld cnt %ld out %.9f\n", id, sum_i(sel, (size_t)B * Hkv * Kmax), sum_i(cnt, B), sum_d(out, nq));
  tso_sparse_decode_attention(q, K, V, sel, cnt, L, B, Hq, Hkv, Lmax, d, S, Kmax, 1.0, out, lse);
  printf("case %d sparse out %.9f lse %.9f\n", id, sum_d(out, nq), sum_d(lse, (size_t)B * Hq));
  tso_dense_decode_attention(q, K, V, L, B, Hq, Hkv, Lmax, d, 0.125, out, lse);
  printf("case %d dense out %.9f lse %.9f\n", id, sum_d(out, nq), sum_d(lse, (size_t)B * Hq));
  tso_append_token_meta(knew, L, B, Hkv, d, S, Pmax, pmin, pmax);
  printf("case %d appended meta %ld %ld\n", id, sum_u16(pmin, nmeta), sum_u16(pmax, nmeta));
  if (!half) {   /* INT8 cache: quantise the same tensors row by row */
    size_t rows = (size_t)B * Hkv * Lmax;
    int8_t* Kq = NEW(int8_t, nK); int8_t* Vq = NEW(int8_t, nK);
    float* ks = NEW(float, rows); float* vs = NEW(float, rows);
    int8_t* kq_new = NEW(int8_t, (size_t)B * Hkv * d); float* ks_new = NEW(float, (size_t)B * Hkv);
    tso_quantize_rows_i8(K, (int)rows, d, Kq, ks);
    tso_quantize_rows_i8(V, (int)rows, d, Vq, vs);
    tso_quantize_rows_i8(knew, B * Hkv, d, kq_new, ks_new);
    tso_build_page_meta_i8(Kq, ks, L, B, Hkv, Lmax, d, S, Pmax, pmin, pmax);
    tso_query_aware_decode_i8(q, Kq, ks, Vq, vs, pmin, pmax, L, B, Hq, Hkv, Lmax, d, S, Pmax, topk,
                              per_seq ? tps : NULL, Kmax, keep_first, keep_last, 0.125, scores, sel, cnt, gap, out);
    printf("case %d int8 sel %ld out %.9f\n", id, sum_i(sel, (size_t)B * Hkv * Kmax), sum_d(out, nq));
    tso_sparse_decode_attention_i8(q, Kq, ks, Vq, vs, NULL, NULL, L, B, Hq, Hkv, Lmax, d, S, 0, 0.125, out, lse);
    printf("case %d int8 dense out %.9f lse %.9f\n", id, sum_d(out, nq), sum_d(lse, (size_t)B * Hq));
    tso_append_token_meta_i8(kq_new, ks_new, L, B, Hkv, d, S, Pmax, pmin, pmax);
    printf("case %d int8 appended meta %ld %ld\n", id, sum_u16(pmin, nmeta), sum_u16(pmax, nmeta));
    free(Kq); free(Vq); free(ks); free(vs); free(kq_new); free(ks_new);
  }
  free(K); free(V); free(q); free(knew); free(pmin); free(pmax); free(L); free(tps); free(scores);
  free(scores1); free(sel); free(cnt); free(gap); free(out); free(lse); free(best);
}

int main(void) {
  const int32_t a[3] = {37, 0, 16};         /* partly filled page, empty sequence, exactly one page */
  const int32_t c[2] = {1, 130};            /* one token; a long one */
  const int32_t e[4] = {5, 64, 63, 17};
  tso_set_num_threads(2);
  run_case(1, 0, 3, 4, 2, 8, 16, a, 2, 4, 0, 0, 0);
  run_case(2, 0, 2, 8, 1, 16, 4, c, 40, 40, 1, 2, 0);     /* K > P for the short one; always-kept pages */
  run_case(3, 1, 4, 4, 4, 8, 8, e, 3, 6, 0, 1, 1);        /* IEEE half, per-sequence budgets */
  run_case(4, 0, 4, 16, 2, 32, 32, e, 1, 2, 2, 0, 1);     /* groups of eight query heads */
  puts("ok");
  return 0;
}
