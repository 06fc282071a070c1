/*
 * ScaleKV oracle: a plain, slow, fp64 CPU statement of what the per-scale,
 * per-layer KV-cache step computes.
 *
 * THIS IS TEST INFRASTRUCTURE.  It exists so that the HIP kernels can be
 * checked against something written directly from the paper.  Only tests, the
 * smoke check and the bench's cpu_baseline leg may call it; the product path
 * never does, and it shares no code, header, table or helper with the HIP
 * library.
 *
 * Everything is per (sequence, head) "unit": the method treats each head of
 * each sequence independently (Sec. 3.3 states its selection per attention
 * head).  The
 * *_batch entry points only loop that per-unit code over units with OpenMP.
 *
 * Layouts: row-major doubles.  Q/K/V rows are tokens, columns are the
 * head_dim channels.
 *
 * The method is a heuristic eviction, so the functions below follow its steps
 * in the paper's order (Sec. 3.3, the paragraph on cache selection):
 *   importance score (Eq. 5)  ->  top-k under the layer budget  ->  keep the
 *   selected rows, drop the rest  ->  the current map attends over what is
 *   kept plus its own K/V (Sec. 3.1: all tokens of a scale are produced in
 *   parallel and condition on earlier scales; Sec. 3.3's attention weights
 *   range over history and current-map positions).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

int scalekv_oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* ---------------------------------------------------------------- score --
 * Eq. 5:  A = softmax(Qw K^T / sqrt(d_k)) row-wise over the cached keys,
 *         s_i = sum over window rows j of A[j][i].
 * qw: [n_win][d], k: [len][d].  Outputs (each may be NULL):
 *   s[len]      the scores,
 *   log_s[len]  log s_i formed by log-sum-exp over the window rows (the same
 *               number, kept representable when exp() would underflow),
 *   a[n_win][len] the attention rows themselves.
 * `scale` multiplies the dot products (1/sqrt(d_k) in Eq. 5).
 */
void scalekv_oracle_score(const double* qw, int n_win, const double* k, int len, int d,
                          double scale, double* s, double* log_s, double* a) {
  if (len <= 0) return;
  double* logit = (double*)malloc((size_t)n_win * len * sizeof(double));
  double* row_max = (double*)malloc((size_t)n_win * sizeof(double));
  double* row_logz = (double*)malloc((size_t)n_win * sizeof(double));
  for (int j = 0; j < n_win; ++j) {
    for (int i = 0; i < len; ++i) {
      double dot = 0.0;
      for (int c = 0; c < d; ++c) dot += qw[(size_t)j * d + c] * k[(size_t)i * d + c];
      logit[(size_t)j * len + i] = dot * scale;
    }
    double m = logit[(size_t)j * len];
    for (int i = 1; i < len; ++i)
      if (logit[(size_t)j * len + i] > m) m = logit[(size_t)j * len + i];
    double z = 0.0;
    for (int i = 0; i < len; ++i) z += exp(logit[(size_t)j * len + i] - m);
    row_max[j] = m;
    row_logz[j] = log(z);
  }
  for (int i = 0; i < len; ++i) {
    /* A[j][i] = exp(logit - max_j - logZ_j) */
    double sum = 0.0;
    double top = -INFINITY;
    for (int j = 0; j < n_win; ++j) {
      double la = logit[(size_t)j * len + i] - row_max[j] - row_logz[j];
      if (a) a[(size_t)j * len + i] = exp(la);
      sum += exp(la);
      if (la > top) top = la;
    }
    if (s) s[i] = sum;
    if (log_s) {
      if (n_win == 0) {
        log_s[i] = -INFINITY;
      } else {
        double acc = 0.0;
        for (int j = 0; j < n_win; ++j)
          acc += exp(logit[(size_t)j * len + i] - row_max[j] - row_logz[j] - top);
        log_s[i] = top + log(acc);
      }
    }
  }
  free(logit);
  free(row_max);
  free(row_logz);
}

/* --------------------------------------------------------------- select --
 * Sec. 3.3: layer l keeps the k^l tokens whose aggregated importance score is
 * highest.  keep = min(budget, len).  Order tokens by score descending,
 * equal scores by index ascending; take the first `keep`; report them in
 * ascending index order.  Written as `keep` rounds of a linear arg-max so
 * that nothing but the definition is involved.  Returns keep.
 */
int scalekv_oracle_select(const double* score, int len, int budget, int32_t* idx) {
  int keep = budget < len ? budget : len;
  if (keep <= 0) return 0;
  unsigned char* taken = (unsigned char*)calloc((size_t)len, 1);
  for (int r = 0; r < keep; ++r) {
    int best = -1;
    for (int i = 0; i < len; ++i) {
      if (taken[i]) continue;
      if (best < 0 || score[i] > score[best]) best = i; /* strict >: lower index wins ties */
    }
    taken[best] = 1;
  }
  int t = 0;
  for (int i = 0; i < len; ++i)
    if (taken[i]) idx[t++] = i;
  free(taken);
  return keep;
}

/* -------------------------------------------------------------- compact --
 * Sec. 3.3: the K/V rows of the selected tokens stay in the cache for the later
 * steps, every other row is dropped:
 *   dst[t] = src[idx[t]] for t < keep, then the current map's rows follow,
 *   dst[keep + t] = cur[t] for t < n_cur.  Returns the new length.
 */
int scalekv_oracle_compact(const double* src, const int32_t* idx, int keep, const double* cur,
                           int n_cur, int d, double* dst) {
  for (int t = 0; t < keep; ++t)
    memcpy(dst + (size_t)t * d, src + (size_t)idx[t] * d, (size_t)d * sizeof(double));
  for (int t = 0; t < n_cur; ++t)
    memcpy(dst + (size_t)(keep + t) * d, cur + (size_t)t * d, (size_t)d * sizeof(double));
  return keep + n_cur;
}

/* --------------------------------------------------------------- attend --
 * Every query of the current map attends over all kv_len rows handed in (the
 * retained history followed by the current map's own keys), no mask:
 *   p = softmax_i(scale * q_t . k_i),  out_t = sum_i p_i v_i.
 * q: [n_q][d], k, v: [kv_len][d], out: [n_q][d].
 */
void scalekv_oracle_attend(const double* q, int n_q, const double* k, const double* v, int kv_len,
                           int d, double scale, double* out) {
  double* p = (double*)malloc((size_t)(kv_len > 0 ? kv_len : 1) * sizeof(double));
  for (int t = 0; t < n_q; ++t) {
    double m = -INFINITY;
    for (int i = 0; i < kv_len; ++i) {
      double dot = 0.0;
      for (int c = 0; c < d; ++c) dot += q[(size_t)t * d + c] * k[(size_t)i * d + c];
      p[i] = dot * scale;
      if (p[i] > m) m = p[i];
    }
    double z = 0.0;
    for (int i = 0; i < kv_len; ++i) {
      p[i] = exp(p[i] - m);
      z += p[i];
    }
    for (int c = 0; c < d; ++c) out[(size_t)t * d + c] = 0.0;
    for (int i = 0; i < kv_len; ++i) {
      double w = p[i] / z;
      for (int c = 0; c < d; ++c) out[(size_t)t * d + c] += w * v[(size_t)i * d + c];
    }
  }
  free(p);
}

/* ----------------------------------------------------------------- step --
 * One (layer, scale) call for one unit, steps in the order
 *   score -> select -> compact (+ append current K/V) -> attend.
 * The window queries are rows win_idx[0..n_win) of q.  k_src/v_src hold
 * cache_len rows; k_dst/v_dst receive keep + n_cur rows; idx receives keep
 * indices; out receives n_cur rows.  budget >= cache_len keeps every row
 * (then the result is plain attention over the whole cache and the current
 * map).
 * The ranking of Sec. 3.3 (the k^l highest aggregated scores) only depends on
 * the order of the scores, and log is
 * strictly increasing, so the selection is taken on log s_i: the same order
 * wherever s_i is representable, and still an order where s_i itself would
 * underflow to zero (sharply peaked rows), where ranking on s_i would see a
 * tie that Eq. 5 does not contain.
 * score_out / log_score_out (each may be NULL) receive s_i and log s_i.
 * If force_idx is non-NULL, its force_keep entries are used in place of
 * the oracle's own selection (lets a test follow the GPU's choice at a near-tie
 * so later scales stay comparable).  Returns the new cache length.
 */
int scalekv_oracle_step(const double* q, const double* k_cur, const double* v_cur, int n_cur,
                        const int32_t* win_idx, int n_win, const double* k_src,
                        const double* v_src, int cache_len, int budget, int d, double scale,
                        const int32_t* force_idx, int force_keep, double* k_dst, double* v_dst,
                        int32_t* idx, double* score_out, double* log_score_out, double* out) {
  int keep = budget < cache_len ? budget : cache_len;
  if (keep < 0) keep = 0;
  size_t n_s = (size_t)(cache_len > 0 ? cache_len : 1);
  double* s = (double*)malloc(n_s * sizeof(double));
  double* log_s = (double*)malloc(n_s * sizeof(double));
  double* qw = (double*)malloc((size_t)(n_win > 0 ? n_win : 1) * d * sizeof(double));
  for (int j = 0; j < n_win; ++j)
    memcpy(qw + (size_t)j * d, q + (size_t)win_idx[j] * d, (size_t)d * sizeof(double));
  scalekv_oracle_score(qw, n_win, k_src, cache_len, d, scale, s, log_s, NULL);
  if (score_out) memcpy(score_out, s, (size_t)cache_len * sizeof(double));
  if (log_score_out) memcpy(log_score_out, log_s, (size_t)cache_len * sizeof(double));
  if (force_idx) {
    keep = force_keep;
    memcpy(idx, force_idx, (size_t)keep * sizeof(int32_t));
  } else {
    keep = scalekv_oracle_select(log_s, cache_len, budget, idx);
  }
  scalekv_oracle_compact(k_src, idx, keep, k_cur, n_cur, d, k_dst);
  int new_len = scalekv_oracle_compact(v_src, idx, keep, v_cur, n_cur, d, v_dst);
  scalekv_oracle_attend(q, n_cur, k_dst, v_dst, new_len, d, scale, out);
  free(s);
  free(log_s);
  free(qw);
  return new_len;
}

/* ------------------------------------------------------ batched wrappers --
 * Units are independent; these only distribute units over host threads.
 * Every per-unit tensor of unit u starts at u * (rows * d) of its array.
 */
void scalekv_oracle_attend_batch(int n_unit, const double* q, int n_q, const double* k,
                                 const double* v, int kv_len, int d, double scale, double* out) {
#pragma omp parallel for schedule(dynamic)
  for (int u = 0; u < n_unit; ++u)
    scalekv_oracle_attend(q + (size_t)u * n_q * d, n_q, k + (size_t)u * kv_len * d,
                          v + (size_t)u * kv_len * d, kv_len, d, scale, out + (size_t)u * n_q * d);
}

void scalekv_oracle_step_batch(int n_unit, const double* q, const double* k_cur,
                               const double* v_cur, int n_cur, const int32_t* win_idx, int n_win,
                               const double* k_src, const double* v_src, int cache_len, int budget,
                               int d, double scale, const int32_t* force_idx, int force_keep,
                               double* k_dst, double* v_dst, int32_t* idx, double* score_out,
                               double* log_score_out, double* out) {
  int keep = budget < cache_len ? budget : cache_len;
  if (keep < 0) keep = 0;
  if (force_idx) keep = force_keep;
  size_t new_len = (size_t)keep + n_cur;
#pragma omp parallel for schedule(dynamic)
  for (int u = 0; u < n_unit; ++u)
    scalekv_oracle_step(q + (size_t)u * n_cur * d, k_cur + (size_t)u * n_cur * d,
                        v_cur + (size_t)u * n_cur * d, n_cur, win_idx, n_win,
                        k_src + (size_t)u * cache_len * d, v_src + (size_t)u * cache_len * d,
                        cache_len, budget, d, scale,
                        force_idx ? force_idx + (size_t)u * force_keep : NULL, force_keep,
                        k_dst + u * new_len * d, v_dst + u * new_len * d,
                        idx + (size_t)u * (keep > 0 ? keep : 0),
                        score_out ? score_out + (size_t)u * cache_len : NULL,
                        log_score_out ? log_score_out + (size_t)u * cache_len : NULL,
                        out + (size_t)u * n_cur * d);
}

/* ----------------------------------------------------------- cache sizes --
 * Cache length of one layer entering each scale (Sec. 3.3; introduction:
 * scale k adds h_k*w_k entries):  len_1 = prefix,
 * len_{k+1} = min(budget_k, len_k) + n_k.   n_tok/budget: K entries;
 * len_in/keep: K entries out.  Returns the length after the last scale.
 */
int scalekv_oracle_cache_lengths(int prefix, const int32_t* n_tok, const int32_t* budget,
                                 int n_scale, int32_t* len_in, int32_t* keep) {
  int len = prefix;
  for (int k = 0; k < n_scale; ++k) {
    int kp = budget[k] < len ? budget[k] : len;
    if (kp < 0) kp = 0;
    if (len_in) len_in[k] = len;
    if (keep) keep[k] = kp;
    len = kp + n_tok[k];
  }
  return len;
}
