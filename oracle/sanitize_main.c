/*
 * Driver for the sanitizer build of the oracle (gcc -fsanitize=address,undefined): calls every
 * routine of the three oracle sources on small seeded inputs, edge sizes included, so that an
 * out-of-bounds access, a use after free, a signed overflow or a misaligned access in the
 * checker itself is reported.  TEST INFRASTRUCTURE, like the oracle: built and run by
 * `python -m oracle.build --sanitize` and by tests/test_sanitizers.py; prints a checksum so
 * that the calls cannot be optimised away.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

void scalekv_oracle_score(const double*, int, const double*, int, int, double, double*, double*, double*);
int scalekv_oracle_select(const double*, int, int, int32_t*);
int scalekv_oracle_compact(const double*, const int32_t*, int, const double*, int, int, double*);
void scalekv_oracle_attend(const double*, int, const double*, const double*, int, int, double, double*);
void scalekv_oracle_attend_batch(int, const double*, int, const double*, const double*, int, int, double, double*);
void scalekv_oracle_step_batch(int, const double*, const double*, const double*, int, const int32_t*, int,
                               const double*, const double*, int, int, int, double, const int32_t*, int,
                               double*, double*, int32_t*, double*, double*, double*);
int scalekv_oracle_cache_lengths(int, const int32_t*, const int32_t*, int, int32_t*, int32_t*);
int scalekv_oracle_window_centroids(int, int, int, int, int32_t*);
void scalekv_oracle_pool(const double*, int, int, double*);
void scalekv_oracle_pool_log(const double*, int, int, double*);
int scalekv_oracle_select_forced(const double*, int, int, const int32_t*, int, int32_t*);
int scalekv_oracle_step_append_first_batch(int, const double*, const double*, const double*, int, const int32_t*,
                                           int, int, const double*, const double*, int, int, int, double,
                                           const int32_t*, int, double*, double*, int32_t*, double*, double*,
                                           double*);
void scalekv_oracle_asi_terms(const double*, int, const double*, int, int, int, double, int, double*, double*);
double scalekv_oracle_asi(const double*, const double*, int);
void scalekv_oracle_zscores(const double*, int, int, double, double*);
int scalekv_oracle_drafters(const double*, int, int, int, int32_t*);
int scalekv_oracle_budgets(int, int, const int32_t*, long long, long long, long long, long long, int32_t*,
                           int32_t*, long long*);
int scalekv_oracle_positional(int, int, int, int32_t*);
void scalekv_oracle_pyramid(int, long long, long long, int32_t*);

static uint64_t rng_state = 0x243F6A8885A308D3ull;
static double rnd(void) { /* uniform in (-1, 1), xorshift */
  rng_state ^= rng_state << 13;
  rng_state ^= rng_state >> 7;
  rng_state ^= rng_state << 17;
  return (double)(rng_state >> 11) / 4503599627370496.0 - 1.0;
}
static double* vec(size_t n) {
  double* p = (double*)malloc((n ? n : 1) * sizeof(double));
  for (size_t i = 0; i < n; ++i) p[i] = rnd();
  return p;
}
static double fold(const double* p, size_t n) {
  double s = 0.0;
  for (size_t i = 0; i < n; ++i) s += p[i] * (double)(i % 7 + 1);
  return s;
}

int main(void) {
  double sum = 0.0;
  const int dims[] = {1, 8, 64};
  const int lens[] = {0, 1, 5, 33};
  for (int di = 0; di < 3; ++di)
    for (int li = 0; li < 4; ++li)
      for (int n_cur = 1; n_cur <= 9; n_cur += 4) {
        const int d = dims[di], len = lens[li], U = 3;
        const int n_win = n_cur < 4 ? n_cur : 4;
        int32_t win[4];
        for (int j = 0; j < n_win; ++j) win[j] = n_cur - 1 - j;
        double *q = vec((size_t)U * n_cur * d), *kc = vec((size_t)U * n_cur * d), *vc = vec((size_t)U * n_cur * d);
        double *ks = vec((size_t)U * len * d), *vs = vec((size_t)U * len * d);
        const int budgets[] = {0, 1, len / 2, len, len + 3};
        for (int bi = 0; bi < 5; ++bi) {
          const int budget = budgets[bi], keep = budget < len ? budget : len;
          double *kd = vec((size_t)U * (keep + n_cur) * d), *vd = vec((size_t)U * (keep + n_cur) * d);
          double *sc = vec((size_t)U * len), *lsc = vec((size_t)U * len), *out = vec((size_t)U * n_cur * d);
          int32_t* idx = (int32_t*)calloc((size_t)U * (keep ? keep : 1), sizeof(int32_t));
          scalekv_oracle_step_batch(U, q, kc, vc, n_cur, win, n_win, ks, vs, len, budget, d, 0.3, NULL, 0, kd, vd,
                                    idx, sc, lsc, out);
          sum += fold(out, (size_t)U * n_cur * d) + fold(kd, (size_t)U * (keep + n_cur) * d);
          /* the same with the selection forced to the one just made */
          scalekv_oracle_step_batch(U, q, kc, vc, n_cur, win, n_win, ks, vs, len, budget, d, 0.3, idx, keep, kd, vd,
                                    idx, sc, lsc, out);
          sum += fold(out, (size_t)U * n_cur * d);
          /* the literal order, pooled, window forced */
          const int total = len + n_cur;
          double *kn = vec((size_t)U * total * d), *vn = vec((size_t)U * total * d);
          double *sc2 = vec((size_t)U * total), *lsc2 = vec((size_t)U * total);
          int32_t* idx2 = (int32_t*)calloc((size_t)U * total, sizeof(int32_t));
          for (int pw = 1; pw <= 5; pw += 2) {
            int kept = scalekv_oracle_step_append_first_batch(U, q, kc, vc, n_cur, win, n_win, pw, ks, vs, len, budget,
                                                              d, 0.3, NULL, 0, kn, vn, idx2, sc2, lsc2, out);
            sum += kept + fold(out, (size_t)U * n_cur * d);
          }
          free(kd); free(vd); free(sc); free(lsc); free(out); free(idx); free(kn); free(vn); free(sc2); free(lsc2);
          free(idx2);
        }
        /* single stages */
        if (len > 0) {
          double *s = vec(len), *ls = vec(len), *a = vec((size_t)n_win * len);
          scalekv_oracle_score(q, n_win, ks, len, d, 0.5, s, ls, a);
          int32_t* idx = (int32_t*)calloc(len, sizeof(int32_t));
          int keep = scalekv_oracle_select(ls, len, len / 2, idx);
          double* dst = vec((size_t)(keep + n_cur) * d);
          sum += scalekv_oracle_compact(ks, idx, keep, kc, n_cur, d, dst);
          double* pooled = vec(len);
          scalekv_oracle_pool(s, len, 3, pooled);
          scalekv_oracle_pool_log(ls, len, 31, pooled);
          int32_t forced[2] = {0, len - 1};
          sum += scalekv_oracle_select_forced(pooled, len, 2, forced, len > 1 ? 2 : 1, idx);
          double* o = vec((size_t)U * n_cur * d);
          scalekv_oracle_attend(q, n_cur, ks, vs, len, d, 0.5, o);
          scalekv_oracle_attend_batch(U, q, n_cur, ks, vs, len, d, 0.5, o);
          sum += fold(o, (size_t)U * n_cur * d) + fold(s, len);
          /* Eq. 2 terms: history rows first, the rest counts as the current map */
          double *cr = vec(n_cur), *ht = vec(n_cur);
          for (int top_k = 0; top_k <= len + 1; top_k += (len / 2 > 0 ? len / 2 : 1)) {
            scalekv_oracle_asi_terms(q, n_cur, ks, len / 2, len - len / 2, d, 0.5, top_k, cr, ht);
            sum += scalekv_oracle_asi(cr, ht, n_cur);
          }
          free(s); free(ls); free(a); free(idx); free(dst); free(pooled); free(o); free(cr); free(ht);
        }
        free(q); free(kc); free(vc); free(ks); free(vs);
      }

  /* window centroids, cache lengths, Eq. 3, Eq. 4, comparison policies */
  for (int h = 1; h <= 9; h += 2)
    for (int w = 1; w <= 7; w += 3)
      for (int g = 1; g <= 5; g += 2) {
        int32_t idx[25];
        sum += scalekv_oracle_window_centroids(h, w, g, g, idx);
      }
  {
    const int32_t n_tok[4] = {1, 4, 16, 64}, budget[4] = {16, 17, 8, 0};
    int32_t len_in[4], keep[4];
    sum += scalekv_oracle_cache_lengths(16, n_tok, budget, 4, len_in, keep);
  }
  for (int L = 1; L <= 6; L += 5)
    for (int K = 1; K <= 5; K += 4) {
      double *asi = vec((size_t)L * K), *z = vec((size_t)L * K);
      int32_t* mask = (int32_t*)calloc((size_t)L * K, sizeof(int32_t));
      scalekv_oracle_zscores(asi, L, K, 1e-8, z);
      for (int n_d = 0; n_d <= L * K + 1; ++n_d) sum += scalekv_oracle_drafters(z, L, K, n_d, mask);
      int32_t *n_d = (int32_t*)calloc(K, sizeof(int32_t)), *b_r = (int32_t*)calloc(K, sizeof(int32_t)), b_d = 0;
      long long slack = 0;
      for (int k = 0; k < K; ++k) n_d[k] = (k + 1) % (L + 1);
      sum += scalekv_oracle_budgets(L, K, n_d, 650, 600, 70, 0, b_r, &b_d, &slack) + b_d + (double)slack;
      sum += scalekv_oracle_budgets(L, K, n_d, 2147483647LL, 2147483647LL, 2147483647LL, 5, b_r, &b_d, &slack);
      int32_t* pyr = (int32_t*)calloc(L, sizeof(int32_t));
      scalekv_oracle_pyramid(L, 650, 100, pyr);
      sum += pyr[0];
      free(asi); free(z); free(mask); free(n_d); free(b_r); free(pyr);
    }
  for (int len = 0; len <= 20; len += 10) {
    int32_t idx[21];
    sum += scalekv_oracle_positional(len, 3, 4, idx) + scalekv_oracle_positional(len, 0, 50, idx) +
           scalekv_oracle_positional(len, 30, 0, idx);
  }
  printf("oracle sanitizer run complete, checksum %.6e\n", sum);
  return sum != sum; /* NaN would mean a routine produced garbage */
}
