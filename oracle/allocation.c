/*
 * ScaleKV oracle, the offline policy that feeds the per-step budget: the
 * Attention Selectivity Index (Eq. 2), its per-scale Z-score and the drafter
 * set (Eq. 3), the budget allocation (Eq. 4), and the index / budget rules of
 * the comparison policies the paper lists in Sec. 4.1 (its paragraph on
 * compression baselines), each taken from its one-line description there.
 *
 * THIS IS TEST INFRASTRUCTURE, like scalekv_oracle.c beside it: plain fp64 /
 * integer loops, no code shared with the HIP library.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------ ASI terms --
 * Eq. 2, the two factors for one (sequence, head) unit and each sampled query:
 *   alpha_i = softmax_j(scale * q_i . k_j) over ALL keys the map sees: the
 *   hist_len history rows P_{k-1} first, then the cur_len rows of the map C_k;
 *   cur_ratio[i]  = sum_{j in C_k} alpha_ij          (current attention ratio)
 *   hist_topk[i]  = sum of the top_k largest alpha_ij, j in P_{k-1}
 *                   (history top-K ratio; all of them if hist_len < top_k).
 * (The printed equation lost the summation range of its first factor; the text
 * beside it says the factor is the share of attention that goes to the current
 * map, which fixes the range.)
 * q: [n_s][d] sampled queries of the current map, k: [hist_len + cur_len][d].
 */
void scalekv_oracle_asi_terms(const double* q, int n_s, const double* k, int hist_len, int cur_len,
                              int d, double scale, int top_k, double* cur_ratio,
                              double* hist_topk) {
  int len = hist_len + cur_len;
  double* p = (double*)malloc((size_t)(len > 0 ? len : 1) * sizeof(double));
  unsigned char* taken = (unsigned char*)malloc((size_t)(hist_len > 0 ? hist_len : 1));
  for (int i = 0; i < n_s; ++i) {
    double m = -INFINITY;
    for (int j = 0; j < len; ++j) {
      double dot = 0.0;
      for (int c = 0; c < d; ++c) dot += q[(size_t)i * d + c] * k[(size_t)j * d + c];
      p[j] = dot * scale;
      if (p[j] > m) m = p[j];
    }
    double z = 0.0;
    for (int j = 0; j < len; ++j) {
      p[j] = exp(p[j] - m);
      z += p[j];
    }
    for (int j = 0; j < len; ++j) p[j] /= z;
    double cur = 0.0;
    for (int j = hist_len; j < len; ++j) cur += p[j];
    cur_ratio[i] = cur;
    /* top_k rounds of a linear arg-max over the history weights */
    memset(taken, 0, (size_t)(hist_len > 0 ? hist_len : 1));
    double top = 0.0;
    int rounds = top_k < hist_len ? top_k : hist_len;
    for (int r = 0; r < rounds; ++r) {
      int best = -1;
      for (int j = 0; j < hist_len; ++j) {
        if (taken[j]) continue;
        if (best < 0 || p[j] > p[best]) best = j;
      }
      taken[best] = 1;
      top += p[best];
    }
    hist_topk[i] = top;
  }
  free(p);
  free(taken);
}

/* Eq. 2: ASI = E_i[cur_ratio] * E_i[hist_topk], the expectations taken over the
 * n sampled query positions handed in (of every head and sequence of the layer:
 * the paper's index (l,k) has no head, so the heads share one expectation). */
double scalekv_oracle_asi(const double* cur_ratio, const double* hist_topk, int n) {
  if (n <= 0) return 0.0;
  double a = 0.0, b = 0.0;
  for (int i = 0; i < n; ++i) {
    a += cur_ratio[i];
    b += hist_topk[i];
  }
  return (a / n) * (b / n);
}

/* -------------------------------------------------------------- Z-score --
 * Eq. 3: Z(l,k) = (ASI(l,k) - mu_k) / (sigma_k + eps), mu_k and sigma_k the mean
 * and standard deviation of ASI over the L layers at scale k (the text says the
 * normalisation is done inside each scale).  sigma_k is the population deviation
 * (divisor L); the paper does not say which.  asi, z: [L][K] row-major.
 */
void scalekv_oracle_zscores(const double* asi, int L, int K, double eps, double* z) {
  for (int k = 0; k < K; ++k) {
    double mu = 0.0;
    for (int l = 0; l < L; ++l) mu += asi[(size_t)l * K + k];
    mu /= L;
    double var = 0.0;
    for (int l = 0; l < L; ++l) {
      double t = asi[(size_t)l * K + k] - mu;
      var += t * t;
    }
    double sigma = sqrt(var / L);
    for (int l = 0; l < L; ++l) z[(size_t)l * K + k] = (asi[(size_t)l * K + k] - mu) / (sigma + eps);
  }
}

/* Eq. 3: the drafters are the n_d (layer, scale) pairs with the lowest Z over
 * all L*K pairs.  Equal Z (the printed "<= Z_(N_d)" would then admit more than
 * N_d pairs): the lower scale first, then the lower layer, so exactly n_d are
 * taken.  is_drafter: [L][K], 1 for a drafter.  Returns the number taken.
 */
int scalekv_oracle_drafters(const double* z, int L, int K, int n_d, int32_t* is_drafter) {
  int total = L * K;
  if (n_d > total) n_d = total;
  for (int i = 0; i < total; ++i) is_drafter[i] = 0;
  for (int r = 0; r < n_d; ++r) {
    int bl = -1, bk = -1;
    for (int k = 0; k < K; ++k)
      for (int l = 0; l < L; ++l) {
        if (is_drafter[(size_t)l * K + k]) continue;
        if (bl < 0 || z[(size_t)l * K + k] < z[(size_t)bl * K + bk]) { /* strict <: scan order breaks ties */
          bl = l;
          bk = k;
        }
      }
    is_drafter[(size_t)bl * K + bk] = 1;
  }
  return n_d > 0 ? n_d : 0;
}

/* -------------------------------------------------------------- budgets --
 * Eq. 4:  sum_{k=1..K} (N_d^k B_d(k) + N_r^k B_r(k)) = B_uniform * L * K,
 *         B_r(k) = B_r(0) - delta * k.
 * One equation cannot fix K drafter budgets, so B_d is taken to be the same at
 * every scale: the memory the refiners give up goes into one pool that the
 * drafter (layer, scale) pairs share equally.  k runs from 1 as in the sum.
 * With the paper's own numbers (B_r(0) = 600, delta = 70, 13 scales) the line
 * goes negative, so it is held at b_min >= 0:  B_r(k) = max(b_min, B_r(0) - delta k).
 * Integers: B_d = floor(pool / sum_k N_d^k); the left side of Eq. 4 then falls
 * short of the right by *slack, 0 <= slack < sum_k N_d^k tokens.
 * n_d: [K] drafter layers per scale (N_r^k = L - N_d^k).  b_r: [K] out.
 * Returns 0, or -1 if no drafter exists to take the pool or the refiners alone
 * already exceed the total (then nothing is written).
 */
int scalekv_oracle_budgets(int L, int K, const int32_t* n_d, long long b_uniform, long long b_r0,
                           long long delta, long long b_min, int32_t* b_r, int32_t* b_d,
                           long long* slack) {
  long long total = b_uniform * L * K;
  long long refiners = 0, drafters = 0;
  for (int k = 1; k <= K; ++k) {
    long long br = b_r0 - delta * k;
    if (br < b_min) br = b_min;
    refiners += (long long)(L - n_d[k - 1]) * br;
    drafters += n_d[k - 1];
  }
  if (drafters <= 0 || refiners > total) return -1;
  for (int k = 1; k <= K; ++k) {
    long long br = b_r0 - delta * k;
    b_r[k - 1] = (int32_t)(br < b_min ? b_min : br);
  }
  long long pool = total - refiners;
  *b_d = (int32_t)(pool / drafters);
  *slack = pool - (pool / drafters) * drafters;
  return 0;
}

/* ------------------------------------------------- comparison policies --
 * Sec. 4.1 lists them in one line each.  What is built from that line:
 *   sliding window  (keeps a local window of the newest tokens):
 *                   the last n_recent positions;
 *   sinks + recent  (keeps the initial tokens, the attention sinks, and the
 *                   newest tokens): the first n_sink positions and the last n_recent.
 * Both are the same rule (n_sink = 0 for the first).  If the two ranges meet,
 * every position is kept once.  idx receives the positions ascending; returns
 * their number, min(len, n_sink + n_recent).
 */
int scalekv_oracle_positional(int len, int n_sink, int n_recent, int32_t* idx) {
  int t = 0;
  for (int i = 0; i < len; ++i)
    if (i < n_sink || i >= len - n_recent) idx[t++] = i;
  return t;
}

/* pyramid allocation (a fixed, pyramid-shaped split of the budget over the
 * layers): the per-layer budget falls linearly from the first layer
 * to the last while the mean stays b_uniform.  b_last (<= b_uniform) is the last
 * layer's budget, the first layer gets 2 b_uniform - b_last; for the lower half
 * l < L/2:  B(l) = b_first - floor((b_first - b_last) * l / (L - 1)), the upper
 * half mirrors it, B(L-1-l) = 2 b_uniform - B(l), and the middle layer of an odd
 * L gets b_uniform; so sum_l B(l) = L * b_uniform exactly.  b: [L] out.
 */
void scalekv_oracle_pyramid(int L, long long b_uniform, long long b_last, int32_t* b) {
  long long b_first = 2 * b_uniform - b_last;
  for (int l = 0; l < L / 2; ++l) {
    long long v = L > 1 ? b_first - (b_first - b_last) * l / (L - 1) : b_uniform;
    b[l] = (int32_t)v;
    b[L - 1 - l] = (int32_t)(2 * b_uniform - v);
  }
  if (L % 2) b[L / 2] = (int32_t)b_uniform;
}
