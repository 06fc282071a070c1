/*
 * scalekv.h -- C ABI of the ScaleKV per-scale, per-layer KV-cache step for
 * AMD MI355X (gfx950).
 *
 * One call of scalekv_step does, for every (sequence, head) unit independently,
 * what the cache-selection paragraph of Sec. 3.3 of the paper describes for one layer at
 * one scale:
 *   1. score    importance of every cached token = attention mass it receives
 *               from the observation-window queries of the current token map
 *               (Eq. 5);
 *   2. select   the top-k cached tokens under the layer's budget (Sec. 3.3:
 *               the k^l highest scores of layer l; budgets come from Eq. 4);
 *   3. compact  keep the selected K/V rows, drop the rest, append the current
 *               map's K/V (Sec. 3.3, last sentence of the selection paragraph);
 *   4. attend   the current map's queries attend, unmasked, over the kept rows
 *               plus the map's own K/V (Sec. 3.1: a scale's tokens are produced
 *               in parallel, conditioned on earlier scales).
 * The four stages are also exported on their own.
 *
 * Conventions common to every entry point
 * ---------------------------------------
 * Memory.  Every pointer is DEVICE memory unless its comment says "host".  All
 *   buffers are allocated, owned and freed by the caller; the library allocates
 *   nothing and holds no device state apart from the fixed scratch array of
 *   scalekv_step_static.  Device pointers must be 16-byte aligned.
 * Layout.  Dense tensors are row-major [n_seq, n_head, rows, head_dim] with no
 *   padding.  A cache (scalekv_kv) is [n_seq, n_head, capacity, head_dim] with
 *   explicit sequence and head strides (in elements) and a contiguous row of
 *   head_dim elements; only the first `len` rows of each unit are meaningful.
 *   Element type is shape->dtype (fp32 or bf16).  Scores are fp32, indices
 *   int32.
 * Asynchrony.  Work is enqueued on `stream` (a hipStream_t passed as void*; NULL
 *   is the default stream).  No call synchronises with the host.  Integer
 *   results returned through host pointers (keep, new length) are computed on
 *   the host from the arguments and are valid on return.
 * Errors.  Each call returns a scalekv_status.  Arguments are checked on the
 *   host before anything is launched, so a failing call has no side effects.
 *   scalekv_last_error() gives a message for the calling thread's last failure.
 * Limits.  head_dim must be 64 or 128; n_win <= SCALEKV_MAX_WINDOW;
 *   n_seq * n_head <= 65535 (one grid dimension counts the units; more ->
 *   SCALEKV_ERR_UNSUPPORTED); cache lengths and row counts are int32 and each
 *   (rows * head_dim) product must fit int32.
 */
#ifndef SCALEKV_H
#define SCALEKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SCALEKV_MAX_WINDOW 16
#define SCALEKV_MAX_POOL 31
#define SCALEKV_MAX_ASI_SAMPLES 1024

typedef enum {
  SCALEKV_OK = 0,
  SCALEKV_ERR_INVALID_ARG = 1, /* null/misaligned pointer, negative size, length beyond capacity,
                                  window index out of range, overlapping source and destination */
  SCALEKV_ERR_UNSUPPORTED = 2, /* head_dim or dtype the kernels are not built for */
  SCALEKV_ERR_WORKSPACE = 3,   /* ws == NULL or ws_bytes below scalekv_workspace_bytes() */
  SCALEKV_ERR_HIP = 4          /* a kernel launch reported an error */
} scalekv_status;

typedef enum { SCALEKV_F32 = 0, SCALEKV_BF16 = 1 } scalekv_dtype;

typedef struct {
  int32_t n_seq;    /* sequences (batch rows; classifier-free-guidance rows count separately) */
  int32_t n_head;   /* attention heads; K/V have the same head count as Q */
  int32_t head_dim; /* 64 or 128 */
  int32_t dtype;    /* scalekv_dtype of Q, K, V and the attention output */
  float sm_scale;   /* multiplies q.k before the softmax; <= 0 means 1/sqrt(head_dim) (Eq. 5) */
} scalekv_shape;

typedef struct {
  void* ptr;           /* device, [n_seq, n_head, capacity, head_dim] */
  int64_t seq_stride;  /* elements between consecutive sequences */
  int64_t head_stride; /* elements between consecutive heads; >= capacity * head_dim */
  int32_t capacity;    /* rows available per (sequence, head) */
} scalekv_kv;

/* Bytes of device workspace that score/step need for caches up to max_cache_len
 * rows and up to max_q current tokens.  *out is host memory. */
scalekv_status scalekv_workspace_bytes(const scalekv_shape* shape, int32_t max_cache_len,
                                       int32_t max_q, size_t* out);

/* Eq. 5.  q_win [S,H,n_win,d]: the observation-window queries.  k: cache whose
 * first cache_len rows are scored.  log_scores [S,H,cache_len] fp32 receives
 * log s_i, where s_i = sum over window rows j of softmax_i(q_j.k_i*sm_scale);
 * the softmax runs over exactly the cache_len rows given.  The logarithm is a
 * monotone image of s_i that stays finite when exp() underflows in fp32, so the
 * ranking of Sec. 3.3 is unchanged.  cache_len == 0 is a no-op.  n_win >= 1. */
scalekv_status scalekv_score(const scalekv_shape* shape, const void* q_win, int32_t n_win,
                             const scalekv_kv* k, int32_t cache_len, float* log_scores, void* ws,
                             size_t ws_bytes, void* stream);

/* Top-k of Sec. 3.3 per (sequence, head): keep = min(budget, cache_len) indices
 * of the largest scores, equal scores resolved towards the lower index, written
 * in ascending index order to idx [S,H,keep].  *keep_out (host, may be NULL)
 * receives keep.  budget == 0 or cache_len == 0 writes nothing. */
scalekv_status scalekv_select(const scalekv_shape* shape, const float* scores, int32_t cache_len,
                              int32_t budget, int32_t* idx, int32_t* keep_out, void* stream);

/* Pruning of Sec. 3.3: for t < keep, dst row t = src row idx[t] (K and V with
 * the same idx [S,H,keep]); then rows keep .. keep+n_cur-1 = the current map's
 * k_cur / v_cur [S,H,n_cur,d].  idx == NULL means the identity (keep all of
 * the first `keep` rows, keep <= cache_len).  k_cur/v_cur may be NULL iff
 * n_cur == 0.  Copies are bit-exact.  The byte spans of the two
 * source caches and the two destination caches (first to last addressable
 * element of each) must be pairwise disjoint, except that k_src may alias
 * v_src, and k_cur / v_cur must not overlap a destination cache.  Requires keep + n_cur <= dst capacity and idx entries in
 * [0, cache_len) (entries are not checked on the device). */
scalekv_status scalekv_compact(const scalekv_shape* shape, const scalekv_kv* k_src,
                               const scalekv_kv* v_src, int32_t cache_len, const int32_t* idx,
                               int32_t keep, const void* k_cur, const void* v_cur, int32_t n_cur,
                               const scalekv_kv* k_dst, const scalekv_kv* v_dst, void* stream);

/* Unmasked attention of Sec. 3.1 / 3.3: out[t] = sum_i softmax_i(q_t.k_i *
 * sm_scale) v_i over the first kv_len rows of k and v.  q, out [S,H,n_q,d].
 * fp32 accumulation; bf16 inputs round the probabilities to bf16 before the
 * P.V product.  n_q == 0 is a no-op; kv_len must be >= 1 when n_q > 0. */
scalekv_status scalekv_attend(const scalekv_shape* shape, const void* q, int32_t n_q,
                              const scalekv_kv* k, const scalekv_kv* v, int32_t kv_len, void* out,
                              void* stream);

/* The whole step.  q, k_cur, v_cur [S,H,n_cur,d] are the current map's
 * projections; win_idx (host, n_win entries in [0, n_cur)) names the
 * observation-window rows of q.  k_src/v_src hold cache_len rows.  On return
 * (stream order) k_dst/v_dst hold keep + n_cur rows (keep = min(budget,
 * cache_len)), out [S,H,n_cur,d] holds the attention output and, if idx_out
 * (device, [S,H,keep]) is not NULL, the selected indices.  *new_len_out (host,
 * may be NULL) = keep + n_cur.  budget >= cache_len keeps everything and skips
 * scoring (the result is exact attention over cache and current map);
 * budget == 0 attends over the current map only.  n_cur >= 1.  q, k_cur, v_cur and out
 * must not overlap k_dst / v_dst (the destination is written while they are in use);
 * such an overlap -> INVALID_ARG, as for overlapping source and destination caches. */
scalekv_status scalekv_step(const scalekv_shape* shape, const void* q, const void* k_cur,
                            const void* v_cur, int32_t n_cur, const int32_t* win_idx,
                            int32_t n_win, const scalekv_kv* k_src, const scalekv_kv* v_src,
                            int32_t cache_len, int32_t budget, const scalekv_kv* k_dst,
                            const scalekv_kv* v_dst, int32_t* new_len_out, void* out,
                            int32_t* idx_out, void* ws, size_t ws_bytes, void* stream);

/* For callers that cannot allocate device memory or hand over a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  The same step as
 * scalekv_step, same arguments minus ws / ws_bytes, same kernels and bit-identical results;
 * the score / select scratch lives in an array of SCALEKV_STATIC_SCRATCH_BYTES that is part of
 * the library's device code (each GPU the library runs on holds its own copy until the
 * process ends).  The call allocates nothing and frees nothing.  The array's device address
 * is looked up on the first call on each device (a query, not an allocation); make that
 * first call outside graph capture.
 * Limit: shapes whose scalekv_workspace_bytes(shape, cache_len, n_cur) exceeds
 * SCALEKV_STATIC_SCRATCH_BYTES -> SCALEKV_ERR_WORKSPACE, nothing launched (calls that need no
 * ranking, budget >= cache_len or budget == 0, use no scratch and are never refused for size).
 * Every call on one GPU uses that GPU's one array: calls that overlap in time on the same
 * GPU (different streams or threads) race on it; serialise them or use scalekv_step with
 * separate workspaces.  Nothing in the array has to be cleared between calls.
 * Other errors as scalekv_step. */
#define SCALEKV_STATIC_SCRATCH_BYTES (64u << 20)
scalekv_status scalekv_step_static(const scalekv_shape* shape, const void* q, const void* k_cur,
                                   const void* v_cur, int32_t n_cur, const int32_t* win_idx,
                                   int32_t n_win, const scalekv_kv* k_src, const scalekv_kv* v_src,
                                   int32_t cache_len, int32_t budget, const scalekv_kv* k_dst,
                                   const scalekv_kv* v_dst, int32_t* new_len_out, void* out,
                                   int32_t* idx_out, void* stream);

/* ---- Sec. 3.3 read literally: the map's K/V join the cache, the map attends, and only
 * then is the cache pruned, with the observation window preserved. ---- */

/* Observation window of Sec. 3.3: the map is cut into N patches and the token at the
 * centre of each patch is taken.  Host only, no GPU work.  The map has map_h rows and
 * map_w columns in raster order and is cut into a grid of gr x gc patches, gr =
 * min(patch_rows, map_h), gc = min(patch_cols, map_w); band a of the rows covers rows
 * [floor(a*map_h/gr), floor((a+1)*map_h/gr)), likewise the columns.  The centroid of a
 * patch is the token nearest to the patch's centre; of equally near tokens the one with
 * the smaller row, then the smaller column.  idx_out (host, at least gr*gc entries)
 * receives the raster indices in ascending order, *n_out their number.
 * Errors: non-positive sizes or NULL outputs -> INVALID_ARG. */
scalekv_status scalekv_window_centroids(int32_t map_h, int32_t map_w, int32_t patch_rows,
                                        int32_t patch_cols, int32_t* idx_out, int32_t* n_out);

/* Selection of Sec. 3.3 with its two optional parts: average pooling of the scores
 * (the aggregation step of the selection paragraph) and positions that are preserved whatever
 * their score (the observation-window tokens, kept together with the selected ones).
 *   log_scores [S,H,cache_len] fp32 device: log of the importance scores (scalekv_score).
 *   pool_w: odd, 1..SCALEKV_MAX_POOL.  The scores are averaged along the cache axis over
 *     pool_w positions centred on each token, zeros beyond both ends, before ranking
 *     (computed on the log-scores as a log-sum-exp; 1 = no pooling).
 *   forced: host array of n_forced (0..SCALEKV_MAX_WINDOW) distinct positions in
 *     [0, cache_len), the same for every unit; they are kept whatever their score and take
 *     no part in the ranking.
 *   Of the other cache_len - n_forced tokens the min(budget, cache_len - n_forced) with
 *   the highest pooled score are selected, equal scores to the lower index.
 *   idx [S,H,keep] int32 device receives the union, ascending; *keep_out (host, may be
 *   NULL) = n_forced + min(budget, cache_len - n_forced), valid on return.
 * Errors: as scalekv_select; pool_w even or out of range, a forced position out of range
 * or repeated -> INVALID_ARG. */
scalekv_status scalekv_select_window(const scalekv_shape* shape, const float* log_scores,
                                     int32_t cache_len, int32_t budget, const int32_t* forced,
                                     int32_t n_forced, int32_t pool_w, int32_t* idx,
                                     int32_t* keep_out, void* stream);

/* One (layer, scale) call in the order of Sec. 3.3, enqueued on `stream`:
 *   1. rows [cache_len, cache_len + n_cur) of k_cache/v_cache <- k_cur/v_cur (in place;
 *      the caches must have capacity for them),
 *   2. out <- attention of q over all cache_len + n_cur rows, no mask,
 *   3. importance scores (Eq. 5) of every row from the window queries, rows win_idx[0..n_win)
 *      of q, each window row normalised over all cache_len + n_cur keys; pooled with pool_w,
 *   4. the window tokens (cache positions cache_len + win_idx[j]) and the top-`budget` of
 *      the other rows are kept,
 *   5. k_next/v_next rows [0, keep) <- the kept rows, ascending.
 * keep = n_win + min(budget, cache_len + n_cur - n_win), in *keep_out (host, may be NULL).
 * If keep == cache_len + n_cur nothing is dropped: steps 3-5 are skipped, the cache stays
 * in k_cache/v_cache (now cache_len + n_cur rows), k_next/v_next are not touched (may be
 * NULL) and *moved_out (host, may be NULL) is 0; otherwise *moved_out is 1.
 * idx_out (device, [S,H,keep], may be NULL) receives the kept positions.
 * Workspace: scalekv_workspace_bytes(shape, cache_len + n_cur, n_cur).
 * Errors: as scalekv_step, with cache_len + n_cur in place of cache_len for capacities;
 * a ranking with n_win = 0 -> INVALID_ARG. */
scalekv_status scalekv_step_append_first(const scalekv_shape* shape, const void* q,
                                         const void* k_cur, const void* v_cur, int32_t n_cur,
                                         const int32_t* win_idx, int32_t n_win, int32_t pool_w,
                                         const scalekv_kv* k_cache, const scalekv_kv* v_cache,
                                         int32_t cache_len, int32_t budget,
                                         const scalekv_kv* k_next, const scalekv_kv* v_next,
                                         int32_t* keep_out, int32_t* moved_out, void* out,
                                         int32_t* idx_out, void* ws, size_t ws_bytes,
                                         void* stream);

/* ---- The offline policy that produces the per-(layer, scale) budget. ---- */

/* Attention Selectivity Index, Eq. 2, for one layer at one scale.  q_samp [S,H,n_samp,d]:
 * queries sampled from the current map (1 <= n_samp <= SCALEKV_MAX_ASI_SAMPLES).  k: cache
 * whose rows [0, hist_len) are the history P_{k-1} and rows [hist_len, hist_len + cur_len)
 * the current map C_k; each query's softmax runs over all of them (hist_len + cur_len >= 1).
 *   terms [S,H,n_samp,2] fp32 device: per query, {attention mass on the current map,
 *     sum of its top_k largest weights on history rows (all of them if hist_len < top_k)}.
 *   asi_out (device, 3 floats, may be NULL): mean of the first term over all S*H*n_samp
 *     queries, mean of the second, and their product, the ASI of Eq. 2.  Several calls
 *     (more prompts) are combined by the caller from `terms`.
 * Workspace: scalekv_workspace_bytes(shape, hist_len + cur_len, n_samp).  All sums run in a
 * fixed order: results are reproducible bit for bit. */
scalekv_status scalekv_asi(const scalekv_shape* shape, const void* q_samp, int32_t n_samp,
                           const scalekv_kv* k, int32_t hist_len, int32_t cur_len, int32_t top_k,
                           float* terms, float* asi_out, void* ws, size_t ws_bytes, void* stream);

/* Eq. 3.  Host only, no GPU work.  asi (host, [n_layer][n_scale] row-major, finite).
 * Z = (ASI - mu_k) / (sigma_k + eps) with the mean and the population standard deviation
 * over the layers of scale k (0 where sigma_k + eps == 0); the n_drafter pairs with the
 * lowest Z over all layers and scales are the drafters, equal Z resolved towards the lower
 * scale, then the lower layer.  is_drafter (host, [n_layer][n_scale]) receives 1 / 0; z_out
 * (host, same shape, may be NULL) the Z-scores.  n_drafter beyond n_layer*n_scale takes all. */
scalekv_status scalekv_drafter_set(const double* asi, int32_t n_layer, int32_t n_scale,
                                   int32_t n_drafter, double eps, double* z_out,
                                   int32_t* is_drafter);

/* Eq. 4.  Host only.  n_drafter (host, [n_scale]): drafter layers at each scale, the other
 * n_layer - n_drafter[k] layers are refiners.  Refiner budget at scale k (k = 1..n_scale as in
 * the equation's sum): b_r[k-1] = max(b_min, b_r0 - delta * k).  The drafter budget is one
 * value for all scales, *b_d = floor((b_uniform * n_layer * n_scale - sum_k N_r^k B_r(k)) /
 * sum_k N_d^k); *slack (may be NULL) = the tokens by which the left side of Eq. 4 then falls
 * short of the right, 0 <= slack < sum_k N_d^k.  All budgets are tokens per head.
 * Errors (INVALID_ARG): no drafter at any scale; refiner budgets alone above the total;
 * negative inputs or inputs above 2^31-1. */
scalekv_status scalekv_allocate_budgets(int32_t n_layer, int32_t n_scale, const int32_t* n_drafter,
                                        int64_t b_uniform, int64_t b_r0, int64_t delta,
                                        int64_t b_min, int32_t* b_r, int32_t* b_d, int64_t* slack);

/* Eq. 3 and Eq. 4 in one call: from the measured ASI of every (layer, scale) pair to the
 * budget each scalekv_step call of that pair is given (Sec. 3.2: drafters get the large
 * budget, refiners the small, shrinking one).  Host only.  asi, n_drafter, eps as in
 * scalekv_drafter_set (n_drafter >= 1 here, at most n_layer*n_scale); b_uniform, b_r0, delta,
 * b_min as in scalekv_allocate_budgets, whose per-scale drafter counts are those of the
 * drafter set just found.  table (host, [n_layer][n_scale]) receives *b_d for a drafter pair
 * and b_r[k-1] for a refiner pair; is_drafter (host, same shape), b_r (host, [n_scale]),
 * b_d and slack (host) may each be NULL.  Errors are those of the two calls. */
scalekv_status scalekv_policy_table(const double* asi, int32_t n_layer, int32_t n_scale,
                                    int32_t n_drafter, double eps, int64_t b_uniform,
                                    int64_t b_r0, int64_t delta, int64_t b_min, int32_t* table,
                                    int32_t* is_drafter, int32_t* b_r, int32_t* b_d,
                                    int64_t* slack);

/* ---- Comparison policies of Sec. 4.1 (its paragraph on compression baselines), as index / budget
 * generators for the same compact and attend calls; each is built from the one line the
 * paper gives it. ---- */

/* Position-only retention: the first min(n_sink, cache_len) rows and the last
 * min(n_recent, rest) rows of every unit (n_sink = 0: sliding window of the most recent
 * tokens; n_sink > 0: attention sinks plus recent tokens).  idx [S,H,keep] int32 device,
 * ascending; *keep_out (host, may be NULL) = keep, valid on return. */
scalekv_status scalekv_select_positional(const scalekv_shape* shape, int32_t cache_len,
                                         int32_t n_sink, int32_t n_recent, int32_t* idx,
                                         int32_t* keep_out, void* stream);

/* Pyramid-shaped allocation across layers.  Host only.  b (host, [n_layer]) falls linearly
 * from 2*b_uniform - b_last at the first layer to b_last at the last (0 <= b_last <=
 * b_uniform): b[l] = b_first - floor((b_first - b_last) * l / (n_layer - 1)) in the lower
 * half, b[n_layer-1-l] = 2*b_uniform - b[l] in the upper, the middle layer of an odd count
 * gets b_uniform; the sum is exactly n_layer * b_uniform. */
scalekv_status scalekv_pyramid_budgets(int32_t n_layer, int64_t b_uniform, int64_t b_last,
                                       int32_t* b);

/* Benchmark aid, not part of the method.  events: host array of 5 hipEvent_t
 * (created by the caller with timing enabled), or NULL to switch off.  While
 * set, every scalekv_step call of this thread records, on its stream, events[0]
 * before the first kernel and events[1..4] after the score, select, compact and
 * attend kernels respectively (stages that are skipped record their event
 * anyway).  A NULL entry is left out, so {0,0,0,e3,e4} brackets the attend kernel
 * alone.  scalekv_step_append_first records them too: events[0] before the first
 * kernel, events[1..4] after its append, attend, score+select and compact kernels.
 * Where the attention runs in the pipelined bf16 kernel (head_dim 128, n_cur > 128) the
 * two events around it are not recorded as stream operations of their own but attached
 * to that kernel's dispatch and receive its start and end times, so timing that kernel
 * alone ({0,0,0,e3,e4}) adds nothing to the stream.
 * The array is read at each such call and must stay valid until it is replaced or
 * cleared. */
scalekv_status scalekv_step_stage_events(void** events);

/* Message for the calling thread's most recent non-OK status (static storage,
 * never NULL). */
const char* scalekv_last_error(void);

/* Library version string, e.g. "scalekv 0.1 gfx950". */
const char* scalekv_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SCALEKV_H */
