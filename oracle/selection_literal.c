/*
 * ScaleKV oracle, second reading of Sec. 3.3 (its paragraph on cache selection)
 * taken literally: the token map's K/V join the cache first, the map attends over
 * history and itself, and only then is the cache pruned, with the observation
 * window force-kept.
 *
 * THIS IS TEST INFRASTRUCTURE, like scalekv_oracle.c beside it: plain fp64
 * loops, one (sequence, head) unit at a time, no code shared with the HIP
 * library.  The single-stage routines of scalekv_oracle.c (score, attend) are
 * declared below and reused as steps.
 *
 * What Sec. 3.3 states, in its order:
 *   1. the map r_k is partitioned into N patches and the centroid token of each
 *      patch forms the observation window W;
 *   2. Eq. 5: s_i = sum_{j in W} A_ji with A = softmax(Q K^T / sqrt(d_k)); here
 *      K holds every key the map sees (history and the map itself), so each
 *      window row is normalised over all of them;
 *   3. the scores are aggregated by average pooling;
 *   4. per layer the top-k^l tokens are selected; their K/V rows and those of
 *      the observation-window tokens are what stays in the cache for the later
 *      steps.
 * Where the paper leaves a detail open the choice made here is stated at the
 * function.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

void scalekv_oracle_score(const double* qw, int n_win, const double* k, int len, int d,
                          double scale, double* s, double* log_s, double* a);
void scalekv_oracle_attend(const double* q, int n_q, const double* k, const double* v, int kv_len,
                           int d, double scale, double* out);

/* ------------------------------------------------------ window centroids --
 * Sec. 3.3: the map is cut into N patches and the token at the centre of each
 * patch is taken.  The map has h rows and w columns in raster order.  It is
 * cut into a grid of PH x PW patches, PH = min(ph, h), PW = min(pw, w) (a map
 * smaller than the grid gives one token per patch); band a of the rows covers
 * rows [floor(a*h/PH), floor((a+1)*h/PH)), likewise the columns.  The centroid
 * of a patch is the token whose centre (r + 1/2, c + 1/2) is nearest to the
 * patch's geometric centre; of equally near tokens the one with the smaller row,
 * then the smaller column, is taken (the paper does not say).  Written as a
 * search over the patch's tokens with exact integer distances.  idx receives
 * PH*PW raster indices, ascending.  Returns PH*PW.
 */
int scalekv_oracle_window_centroids(int h, int w, int ph, int pw, int32_t* idx) {
  int PH = ph < h ? ph : h, PW = pw < w ? pw : w;
  int n = 0;
  for (int a = 0; a < PH; ++a) {
    int r0 = (int)((long long)a * h / PH), r1 = (int)((long long)(a + 1) * h / PH);
    for (int b = 0; b < PW; ++b) {
      int c0 = (int)((long long)b * w / PW), c1 = (int)((long long)(b + 1) * w / PW);
      /* twice the centre: rows r0 + r1, columns c0 + c1; twice a token's centre: 2r + 1 */
      long long best = -1;
      int br = -1, bc = -1;
      for (int r = r0; r < r1; ++r)
        for (int c = c0; c < c1; ++c) {
          long long dr = 2LL * r + 1 - (r0 + r1), dc = 2LL * c + 1 - (c0 + c1);
          long long dist = dr * dr + dc * dc;
          if (best < 0 || dist < best) { /* strict <: raster order breaks ties */
            best = dist;
            br = r;
            bc = c;
          }
        }
      idx[n++] = br * w + bc;
    }
  }
  return n;
}

/* -------------------------------------------------------------- pooling --
 * Sec. 3.3 aggregates the scores by average pooling.  Kernel
 * size and padding are not given; taken as a 1-D average along the cache
 * axis, odd width pool_w, stride 1, zeros beyond both ends, divisor pool_w:
 *   out_i = (1/pool_w) * sum_{|t| <= (pool_w-1)/2} s_{i+t}.
 * pool_w = 1 is the identity.
 */
void scalekv_oracle_pool(const double* s, int len, int pool_w, double* out) {
  int r = (pool_w - 1) / 2;
  for (int i = 0; i < len; ++i) {
    double acc = 0.0;
    for (int t = -r; t <= r; ++t)
      if (i + t >= 0 && i + t < len) acc += s[i + t];
    out[i] = acc / (double)pool_w;
  }
}

/* The same average formed on log-scores: out_i = log( (1/pool_w) * sum_t exp(ls_{i+t}) ),
 * positions beyond the ends contributing zero (log-score -inf).  Written with the window's
 * largest term taken out of the sum, so that the result stays finite where exp(ls) itself
 * is not representable; it is the logarithm of what scalekv_oracle_pool returns.
 */
void scalekv_oracle_pool_log(const double* ls, int len, int pool_w, double* out) {
  int r = (pool_w - 1) / 2;
  for (int i = 0; i < len; ++i) {
    double top = -INFINITY;
    for (int t = -r; t <= r; ++t)
      if (i + t >= 0 && i + t < len && ls[i + t] > top) top = ls[i + t];
    if (!(top > -INFINITY)) {
      out[i] = -INFINITY;
      continue;
    }
    double acc = 0.0;
    for (int t = -r; t <= r; ++t)
      if (i + t >= 0 && i + t < len) acc += exp(ls[i + t] - top);
    out[i] = top + log(acc) - log((double)pool_w);
  }
}

/* ------------------------------------------------- selection with a window --
 * The forced positions (the observation window) are preserved whatever their
 * score; of the remaining len - n_forced tokens the min(budget, len - n_forced)
 * highest-scoring are selected, equal scores to the lower index.  idx receives
 * the union in ascending order.  Returns its size.
 */
int scalekv_oracle_select_forced(const double* score, int len, int budget, const int32_t* forced,
                                 int n_forced, int32_t* idx) {
  unsigned char* taken = (unsigned char*)calloc((size_t)(len > 0 ? len : 1), 1);
  unsigned char* is_forced = (unsigned char*)calloc((size_t)(len > 0 ? len : 1), 1);
  for (int j = 0; j < n_forced; ++j) is_forced[forced[j]] = 1;
  int n_f = 0;
  for (int i = 0; i < len; ++i) n_f += is_forced[i];
  int rest = len - n_f;
  int pick = budget < rest ? budget : rest;
  if (pick < 0) pick = 0;
  for (int r = 0; r < pick; ++r) {
    int best = -1;
    for (int i = 0; i < len; ++i) {
      if (taken[i] || is_forced[i]) continue;
      if (best < 0 || score[i] > score[best]) best = i;
    }
    taken[best] = 1;
  }
  int t = 0;
  for (int i = 0; i < len; ++i)
    if (taken[i] || is_forced[i]) idx[t++] = i;
  free(taken);
  free(is_forced);
  return t;
}

/* ------------------------------------------------------- the literal step --
 * One (layer, scale) call for one unit:
 *   cache <- [cache ; current K/V]            (the map's KV join the cache)
 *   out   <- attention of the map's queries over the whole cache, no mask
 *   s     <- Eq. 5 with the window rows of q against the whole cache
 *   s     <- pooled(s)                        (pool_w = 1: unchanged)
 *   keep the window tokens and the top-`budget` of the others
 *   next  <- the kept rows, ascending
 * k_cache/v_cache: cache_len rows; q/k_cur/v_cur: n_cur rows; window rows are
 * win_idx[0..n_win) of the current map, i.e. cache positions cache_len +
 * win_idx[j].  k_next/v_next and idx must hold cache_len + n_cur rows /
 * entries.  score_out / log_score_out (optional) receive the pooled scores of all
 * cache_len + n_cur positions and their logarithms.  The ranking is taken on the
 * logarithms: the order Sec. 3.3 asks for is unchanged by a strictly increasing map,
 * and the logarithm stays finite where a sharply peaked row's score underflows.
 * If force_idx is non-NULL its force_keep entries replace the oracle's own selection.
 * Returns the number of rows kept.
 */
int scalekv_oracle_step_append_first(const double* q, const double* k_cur, const double* v_cur,
                                     int n_cur, const int32_t* win_idx, int n_win, int pool_w,
                                     const double* k_cache, const double* v_cache, int cache_len,
                                     int budget, int d, double scale, const int32_t* force_idx,
                                     int force_keep, double* k_next, double* v_next, int32_t* idx,
                                     double* score_out, double* log_score_out, double* out) {
  int len = cache_len + n_cur;
  size_t row = (size_t)d * sizeof(double);
  double* k_all = (double*)malloc((size_t)(len > 0 ? len : 1) * row);
  double* v_all = (double*)malloc((size_t)(len > 0 ? len : 1) * row);
  memcpy(k_all, k_cache, (size_t)cache_len * row);
  memcpy(v_all, v_cache, (size_t)cache_len * row);
  memcpy(k_all + (size_t)cache_len * d, k_cur, (size_t)n_cur * row);
  memcpy(v_all + (size_t)cache_len * d, v_cur, (size_t)n_cur * row);

  scalekv_oracle_attend(q, n_cur, k_all, v_all, len, d, scale, out);

  double* qw = (double*)malloc((size_t)(n_win > 0 ? n_win : 1) * row);
  int32_t* forced = (int32_t*)malloc((size_t)(n_win > 0 ? n_win : 1) * sizeof(int32_t));
  for (int j = 0; j < n_win; ++j) {
    memcpy(qw + (size_t)j * d, q + (size_t)win_idx[j] * d, row);
    forced[j] = cache_len + win_idx[j];
  }
  double* s = (double*)malloc((size_t)(len > 0 ? len : 1) * sizeof(double));
  double* sp = (double*)malloc((size_t)(len > 0 ? len : 1) * sizeof(double));
  double* ls = (double*)malloc((size_t)(len > 0 ? len : 1) * sizeof(double));
  double* lsp = (double*)malloc((size_t)(len > 0 ? len : 1) * sizeof(double));
  scalekv_oracle_score(qw, n_win, k_all, len, d, scale, s, ls, NULL);
  scalekv_oracle_pool(s, len, pool_w, sp);
  scalekv_oracle_pool_log(ls, len, pool_w, lsp);
  if (score_out) memcpy(score_out, sp, (size_t)len * sizeof(double));
  if (log_score_out) memcpy(log_score_out, lsp, (size_t)len * sizeof(double));

  int keep;
  if (force_idx) {
    keep = force_keep;
    memcpy(idx, force_idx, (size_t)keep * sizeof(int32_t));
  } else {
    keep = scalekv_oracle_select_forced(lsp, len, budget, forced, n_win, idx);
  }
  for (int t = 0; t < keep; ++t) {
    memcpy(k_next + (size_t)t * d, k_all + (size_t)idx[t] * d, row);
    memcpy(v_next + (size_t)t * d, v_all + (size_t)idx[t] * d, row);
  }
  free(k_all);
  free(v_all);
  free(qw);
  free(forced);
  free(s);
  free(sp);
  free(ls);
  free(lsp);
  return keep;
}

/* Units are independent; this only spreads them over host threads.  Every unit
 * keeps the same number of rows (the window and the budget are per layer), which
 * is returned; per-unit outputs are strided by cache_len + n_cur rows. */
int scalekv_oracle_step_append_first_batch(int n_unit, const double* q, const double* k_cur,
                                           const double* v_cur, int n_cur, const int32_t* win_idx,
                                           int n_win, int pool_w, const double* k_cache,
                                           const double* v_cache, int cache_len, int budget, int d,
                                           double scale, const int32_t* force_idx, int force_keep,
                                           double* k_next, double* v_next, int32_t* idx,
                                           double* score_out, double* log_score_out,
                                           double* out) {
  size_t len = (size_t)cache_len + n_cur;
  int keep_all = 0;
#pragma omp parallel for schedule(dynamic)
  for (int u = 0; u < n_unit; ++u) {
    int kp = scalekv_oracle_step_append_first(
        q + (size_t)u * n_cur * d, k_cur + (size_t)u * n_cur * d, v_cur + (size_t)u * n_cur * d,
        n_cur, win_idx, n_win, pool_w, k_cache + (size_t)u * cache_len * d,
        v_cache + (size_t)u * cache_len * d, cache_len, budget, d, scale,
        force_idx ? force_idx + (size_t)u * force_keep : NULL, force_keep, k_next + u * len * d,
        v_next + u * len * d, idx + u * len, score_out ? score_out + u * len : NULL,
        log_score_out ? log_score_out + u * len : NULL, out + (size_t)u * n_cur * d);
    if (u == 0) keep_all = kp;
  }
  return keep_all;
}
