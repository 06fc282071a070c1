// C ABI of the ScaleKV step: host-side argument checks, workspace carving and
// kernel sequencing.  Nothing here touches device memory or synchronises; every
// kernel goes onto the caller's stream in order.
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <initializer_list>
#include <algorithm>
#include <cmath>
#include <vector>

#include "../../include/scalekv.h"
#include "common.h"

using namespace scalekv;

namespace {

thread_local char g_err[256] = "no error";
thread_local void** g_stage_events = nullptr;  // benchmark hook, see scalekv_step_stage_events

scalekv_status fail(scalekv_status st, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return st;
}

scalekv_status hip_fail(hipError_t e, const char* what) {
  return fail(SCALEKV_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int elem_bytes(const scalekv_shape* s) { return s->dtype == SCALEKV_F32 ? 4 : 2; }

float resolve_scale(const scalekv_shape* s) {
  return s->sm_scale > 0.f ? s->sm_scale : 1.0f / sqrtf((float)s->head_dim);
}

scalekv_status check_shape(const scalekv_shape* s) {
  if (!s) return fail(SCALEKV_ERR_INVALID_ARG, "shape is NULL");
  if (s->n_seq <= 0 || s->n_head <= 0)
    return fail(SCALEKV_ERR_INVALID_ARG, "n_seq and n_head must be positive (got %d, %d)",
                s->n_seq, s->n_head);
  if ((long long)s->n_seq * s->n_head > 65535)
    return fail(SCALEKV_ERR_UNSUPPORTED, "n_seq * n_head = %lld exceeds 65535",
                (long long)s->n_seq * s->n_head);
  if (s->dtype != SCALEKV_F32 && s->dtype != SCALEKV_BF16)
    return fail(SCALEKV_ERR_UNSUPPORTED, "dtype %d is neither SCALEKV_F32 nor SCALEKV_BF16",
                s->dtype);
  if (s->head_dim != 64 && s->head_dim != 128)
    return fail(SCALEKV_ERR_UNSUPPORTED, "head_dim %d is not 64 or 128", s->head_dim);
  if (!(s->sm_scale == s->sm_scale))
    return fail(SCALEKV_ERR_INVALID_ARG, "sm_scale is NaN");
  return SCALEKV_OK;
}

// rows * head_dim must fit int32 (kernels index a unit with 32-bit offsets in places)
scalekv_status check_rows(const scalekv_shape* s, long long rows, const char* name) {
  if (rows < 0) return fail(SCALEKV_ERR_INVALID_ARG, "%s is negative (%lld)", name, rows);
  if (rows * s->head_dim > 0x7fffffffLL)
    return fail(SCALEKV_ERR_UNSUPPORTED, "%s = %lld rows is too large", name, rows);
  return SCALEKV_OK;
}

scalekv_status check_kv(const scalekv_shape* s, const scalekv_kv* kv, int rows_needed,
                        const char* name) {
  if (!kv) return fail(SCALEKV_ERR_INVALID_ARG, "%s is NULL", name);
  if (!kv->ptr) return fail(SCALEKV_ERR_INVALID_ARG, "%s.ptr is NULL", name);
  if (!aligned16(kv->ptr)) return fail(SCALEKV_ERR_INVALID_ARG, "%s.ptr is not 16-byte aligned", name);
  if (kv->capacity < 0) return fail(SCALEKV_ERR_INVALID_ARG, "%s.capacity is negative", name);
  if (rows_needed > kv->capacity)
    return fail(SCALEKV_ERR_INVALID_ARG, "%s: %d rows needed but capacity is %d", name,
                rows_needed, kv->capacity);
  const long long unit = (long long)kv->capacity * s->head_dim;
  const int epv = 16 / elem_bytes(s);
  if (kv->head_stride < unit || kv->head_stride % epv)
    return fail(SCALEKV_ERR_INVALID_ARG,
                "%s.head_stride %lld must be >= capacity*head_dim (%lld) and a multiple of %d",
                name, (long long)kv->head_stride, unit, epv);
  if (kv->seq_stride < kv->head_stride * s->n_head || kv->seq_stride % epv)
    return fail(SCALEKV_ERR_INVALID_ARG,
                "%s.seq_stride %lld must be >= n_head*head_stride and a multiple of %d", name,
                (long long)kv->seq_stride, epv);
  return SCALEKV_OK;
}

scalekv_status check_dense(const void* p, bool required, const char* name) {
  if (!p) return required ? fail(SCALEKV_ERR_INVALID_ARG, "%s is NULL", name) : SCALEKV_OK;
  if (!aligned16(p)) return fail(SCALEKV_ERR_INVALID_ARG, "%s is not 16-byte aligned", name);
  return SCALEKV_OK;
}

// byte range [lo, hi) spanned by a cache
void kv_span(const scalekv_shape* s, const scalekv_kv* kv, uintptr_t* lo, uintptr_t* hi) {
  const long long e = elem_bytes(s);
  *lo = reinterpret_cast<uintptr_t>(kv->ptr);
  *hi = *lo + (uintptr_t)(((long long)(s->n_seq - 1) * kv->seq_stride +
                           (long long)(s->n_head - 1) * kv->head_stride +
                           (long long)kv->capacity * s->head_dim) * e);
}

bool overlaps(const scalekv_shape* s, const scalekv_kv* a, const scalekv_kv* b) {
  uintptr_t al, ah, bl, bh;
  kv_span(s, a, &al, &ah);
  kv_span(s, b, &bl, &bh);
  return al < bh && bl < ah;
}

// does the dense tensor [S, H, rows, d] at p overlap the byte span of a cache?
bool dense_overlaps(const scalekv_shape* s, const void* p, long long rows, const scalekv_kv* kv) {
  if (!p || rows <= 0) return false;
  uintptr_t kl, kh;
  kv_span(s, kv, &kl, &kh);
  const uintptr_t pl = reinterpret_cast<uintptr_t>(p);
  const uintptr_t ph = pl + (uintptr_t)((long long)s->n_seq * s->n_head * rows * s->head_dim * elem_bytes(s));
  return pl < kh && kl < ph;
}

KvView view(const scalekv_kv* kv) { return KvView{kv->ptr, kv->seq_stride, kv->head_stride}; }

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

struct WsLayout {
  size_t logits_off, partial_off, scores_off, idx_off, total;
  int len_pad, n_chunk;
};

WsLayout ws_layout(const scalekv_shape* s, int cache_len) {
  WsLayout w;
  const size_t U = (size_t)s->n_seq * s->n_head;
  const int len = cache_len > 0 ? cache_len : 1;
  w.len_pad = round_up(len, kLogitPad);
  w.n_chunk = (len + kScoreChunk - 1) / kScoreChunk;
  size_t off = 0;
  w.logits_off = off;  off += align256(U * kMaxWindow * w.len_pad * sizeof(float));
  w.partial_off = off; off += align256(U * w.n_chunk * 2 * kMaxWindow * sizeof(float));
  w.scores_off = off;  off += align256(U * w.len_pad * sizeof(float));
  w.idx_off = off;     off += align256(U * w.len_pad * sizeof(int32_t));
  w.total = off;
  return w;
}

scalekv_status check_ws(const scalekv_shape* s, int cache_len, void* ws, size_t ws_bytes) {
  const WsLayout w = ws_layout(s, cache_len);
  if (!ws) return fail(SCALEKV_ERR_WORKSPACE, "workspace is NULL (%zu bytes needed)", w.total);
  if (!aligned16(ws)) return fail(SCALEKV_ERR_INVALID_ARG, "workspace is not 16-byte aligned");
  if (ws_bytes < w.total)
    return fail(SCALEKV_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", ws_bytes, w.total);
  return SCALEKV_OK;
}

ScoreWorkspace score_ws(const WsLayout& w, void* ws) {
  ScoreWorkspace sw;
  sw.logits = reinterpret_cast<float*>(static_cast<char*>(ws) + w.logits_off);
  sw.partial = reinterpret_cast<float*>(static_cast<char*>(ws) + w.partial_off);
  sw.len_pad = w.len_pad;
  sw.n_chunk = w.n_chunk;
  return sw;
}

// forced positions and pooling width of the selection -> SelectExtras, validated
scalekv_status make_extras(const int32_t* forced, int n_forced, int pool_w, int cache_len,
                           SelectExtras* ex) {
  if (n_forced < 0 || n_forced > SCALEKV_MAX_WINDOW)
    return fail(SCALEKV_ERR_INVALID_ARG, "n_forced %d is outside 0..%d", n_forced,
                SCALEKV_MAX_WINDOW);
  if (n_forced > 0 && !forced) return fail(SCALEKV_ERR_INVALID_ARG, "forced is NULL");
  if (pool_w < 1 || pool_w % 2 == 0 || pool_w > SCALEKV_MAX_POOL)
    return fail(SCALEKV_ERR_INVALID_ARG, "pool_w %d must be odd and in 1..%d", pool_w,
                SCALEKV_MAX_POOL);
  ex->n_forced = n_forced;
  ex->pool_w = pool_w;
  for (int j = 0; j < kMaxWindow; ++j) ex->forced[j] = 0;
  for (int j = 0; j < n_forced; ++j) {
    if (forced[j] < 0 || forced[j] >= cache_len)
      return fail(SCALEKV_ERR_INVALID_ARG, "forced[%d] = %d is outside 0..cache_len-1", j,
                  forced[j]);
    for (int i = 0; i < j; ++i)
      if (forced[i] == forced[j])
        return fail(SCALEKV_ERR_INVALID_ARG, "forced[%d] repeats position %d", j, forced[j]);
    ex->forced[j] = forced[j];
  }
  return SCALEKV_OK;
}

#define SCALEKV_TRY(expr)                       \
  do {                                          \
    scalekv_status _st = (expr);                \
    if (_st != SCALEKV_OK) return _st;          \
  } while (0)

#define SCALEKV_HIP(expr, what)                 \
  do {                                          \
    hipError_t _e = (expr);                     \
    if (_e != hipSuccess) return hip_fail(_e, what); \
  } while (0)

}  // namespace

extern "C" {

const char* scalekv_last_error(void) { return g_err; }

const char* scalekv_version(void) { return "scalekv 0.1 gfx950"; }

scalekv_status scalekv_step_stage_events(void** events) {
  g_stage_events = events;
  return SCALEKV_OK;
}

scalekv_status scalekv_workspace_bytes(const scalekv_shape* shape, int32_t max_cache_len,
                                       int32_t max_q, size_t* out) {
  SCALEKV_TRY(check_shape(shape));
  if (!out) return fail(SCALEKV_ERR_INVALID_ARG, "out is NULL");
  if (max_q < 0) return fail(SCALEKV_ERR_INVALID_ARG, "max_q is negative");
  SCALEKV_TRY(check_rows(shape, max_cache_len, "max_cache_len"));
  *out = ws_layout(shape, max_cache_len).total;
  return SCALEKV_OK;
}

scalekv_status scalekv_score(const scalekv_shape* shape, const void* q_win, int32_t n_win,
                             const scalekv_kv* k, int32_t cache_len, float* log_scores, void* ws,
                             size_t ws_bytes, void* stream) {
  SCALEKV_TRY(check_shape(shape));
  if (n_win < 1 || n_win > SCALEKV_MAX_WINDOW)
    return fail(SCALEKV_ERR_INVALID_ARG, "n_win %d is outside 1..%d", n_win, SCALEKV_MAX_WINDOW);
  SCALEKV_TRY(check_rows(shape, cache_len, "cache_len"));
  SCALEKV_TRY(check_dense(q_win, true, "q_win"));
  SCALEKV_TRY(check_kv(shape, k, cache_len, "k"));
  if (!log_scores) return fail(SCALEKV_ERR_INVALID_ARG, "log_scores is NULL");
  SCALEKV_TRY(check_ws(shape, cache_len, ws, ws_bytes));
  if (cache_len == 0) return SCALEKV_OK;
  const WsLayout w = ws_layout(shape, cache_len);
  const ScoreWorkspace sw = score_ws(w, ws);
  WindowRows rows;
  for (int j = 0; j < kMaxWindow; ++j) rows.row[j] = j < n_win ? j : 0;
  hipStream_t st = static_cast<hipStream_t>(stream);
  SCALEKV_HIP(launch_score_logits(shape->dtype, shape->n_seq, shape->n_head, shape->head_dim, q_win,
                                  (long long)n_win * shape->head_dim, rows, n_win, view(k),
                                  cache_len, resolve_scale(shape), sw, st),
              "score logits launch");
  SCALEKV_HIP(launch_score_finalize(shape->n_seq * shape->n_head, n_win, cache_len, sw, log_scores,
                                    cache_len, st),
              "score finalize launch");
  return SCALEKV_OK;
}

scalekv_status scalekv_select(const scalekv_shape* shape, const float* scores, int32_t cache_len,
                              int32_t budget, int32_t* idx, int32_t* keep_out, void* stream) {
  SCALEKV_TRY(check_shape(shape));
  SCALEKV_TRY(check_rows(shape, cache_len, "cache_len"));
  if (budget < 0) return fail(SCALEKV_ERR_INVALID_ARG, "budget is negative (%d)", budget);
  const int keep = budget < cache_len ? budget : cache_len;
  if (keep > 0) {
    if (!scores) return fail(SCALEKV_ERR_INVALID_ARG, "scores is NULL");
    if (!idx) return fail(SCALEKV_ERR_INVALID_ARG, "idx is NULL");
  }
  if (keep_out) *keep_out = keep;
  SCALEKV_HIP(launch_select(shape->n_seq * shape->n_head, scores, cache_len, cache_len, keep, idx,
                            nullptr, static_cast<hipStream_t>(stream)),
              "select launch");
  return SCALEKV_OK;
}

scalekv_status scalekv_compact(const scalekv_shape* shape, const scalekv_kv* k_src,
                               const scalekv_kv* v_src, int32_t cache_len, const int32_t* idx,
                               int32_t keep, const void* k_cur, const void* v_cur, int32_t n_cur,
                               const scalekv_kv* k_dst, const scalekv_kv* v_dst, void* stream) {
  SCALEKV_TRY(check_shape(shape));
  SCALEKV_TRY(check_rows(shape, cache_len, "cache_len"));
  if (keep < 0 || keep > cache_len)
    return fail(SCALEKV_ERR_INVALID_ARG, "keep %d is outside 0..cache_len (%d)", keep, cache_len);
  if (n_cur < 0) return fail(SCALEKV_ERR_INVALID_ARG, "n_cur is negative (%d)", n_cur);
  SCALEKV_TRY(check_rows(shape, (long long)keep + n_cur, "keep + n_cur"));
  SCALEKV_TRY(check_kv(shape, k_src, cache_len, "k_src"));
  SCALEKV_TRY(check_kv(shape, v_src, cache_len, "v_src"));
  SCALEKV_TRY(check_kv(shape, k_dst, keep + n_cur, "k_dst"));
  SCALEKV_TRY(check_kv(shape, v_dst, keep + n_cur, "v_dst"));
  SCALEKV_TRY(check_dense(k_cur, n_cur > 0, "k_cur"));
  SCALEKV_TRY(check_dense(v_cur, n_cur > 0, "v_cur"));
  if (overlaps(shape, k_src, k_dst) || overlaps(shape, k_src, v_dst) ||
      overlaps(shape, v_src, k_dst) || overlaps(shape, v_src, v_dst) ||
      overlaps(shape, k_dst, v_dst))
    return fail(SCALEKV_ERR_INVALID_ARG, "source and destination caches overlap");
  if (dense_overlaps(shape, k_cur, n_cur, k_dst) || dense_overlaps(shape, k_cur, n_cur, v_dst) ||
      dense_overlaps(shape, v_cur, n_cur, k_dst) || dense_overlaps(shape, v_cur, n_cur, v_dst))
    return fail(SCALEKV_ERR_INVALID_ARG, "k_cur / v_cur overlap a destination cache");
  SCALEKV_HIP(launch_compact(shape->dtype, shape->n_seq, shape->n_head, shape->head_dim,
                             view(k_src), view(v_src), idx, keep, k_cur, v_cur, n_cur, view(k_dst),
                             view(v_dst), static_cast<hipStream_t>(stream)),
              "compact launch");
  return SCALEKV_OK;
}

scalekv_status scalekv_attend(const scalekv_shape* shape, const void* q, int32_t n_q,
                              const scalekv_kv* k, const scalekv_kv* v, int32_t kv_len, void* out,
                              void* stream) {
  SCALEKV_TRY(check_shape(shape));
  SCALEKV_TRY(check_rows(shape, n_q, "n_q"));
  SCALEKV_TRY(check_rows(shape, kv_len, "kv_len"));
  if (n_q == 0) return SCALEKV_OK;
  if (kv_len < 1) return fail(SCALEKV_ERR_INVALID_ARG, "kv_len must be >= 1 when n_q > 0");
  SCALEKV_TRY(check_dense(q, true, "q"));
  SCALEKV_TRY(check_dense(out, true, "out"));
  SCALEKV_TRY(check_kv(shape, k, kv_len, "k"));
  SCALEKV_TRY(check_kv(shape, v, kv_len, "v"));
  SCALEKV_HIP(launch_attend(shape->dtype, shape->n_seq, shape->n_head, shape->head_dim, q, n_q,
                            view(k), view(v), kv_len, resolve_scale(shape), out,
                            static_cast<hipStream_t>(stream)),
              "attend launch");
  return SCALEKV_OK;
}

}  // extern "C"

namespace {

// Library-owned scratch of scalekv_step_static: one array per GPU (every device that loads
// this code holds its own copy, at its own address, until the process ends).  Host code must
// never pass the array's name to a kernel: the name is a host-side stand-in, the device
// address comes from hipGetSymbolAddress, once per device, with that device current.
static __device__ __align__(256) unsigned char scratch[SCALEKV_STATIC_SCRATCH_BYTES];
constexpr int kMaxScratchDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxScratchDevices];

// Device address of the current device's scratch array.  Racing first calls all resolve the
// same address; nothing is allocated here.
scalekv_status static_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
  if (dev < 0 || dev >= kMaxScratchDevices)
    return fail(SCALEKV_ERR_UNSUPPORTED, "device ordinal %d is outside 0..%d", dev,
                kMaxScratchDevices - 1);
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return hip_fail(e, "hipGetSymbolAddress(scratch)");
    if (!p) return fail(SCALEKV_ERR_HIP, "hipGetSymbolAddress(scratch) returned a NULL address");
    g_scratch_ptr[dev].store(p, std::memory_order_release);
  }
  *out = p;
  return SCALEKV_OK;
}

// The step behind scalekv_step and scalekv_step_static.  `static_ws`: take the workspace from
// the library's scratch array (ws / ws_bytes ignored) instead of from the caller.
scalekv_status step_impl(const scalekv_shape* shape, const void* q, const void* k_cur,
                         const void* v_cur, int32_t n_cur, const int32_t* win_idx, int32_t n_win,
                         const scalekv_kv* k_src, const scalekv_kv* v_src, int32_t cache_len,
                         int32_t budget, const scalekv_kv* k_dst, const scalekv_kv* v_dst,
                         int32_t* new_len_out, void* out, int32_t* idx_out, void* ws,
                         size_t ws_bytes, bool static_ws, void* stream) {
  SCALEKV_TRY(check_shape(shape));
  if (n_cur < 1) return fail(SCALEKV_ERR_INVALID_ARG, "n_cur must be >= 1 (got %d)", n_cur);
  SCALEKV_TRY(check_rows(shape, n_cur, "n_cur"));
  SCALEKV_TRY(check_rows(shape, cache_len, "cache_len"));
  if (budget < 0) return fail(SCALEKV_ERR_INVALID_ARG, "budget is negative (%d)", budget);
  const int keep = budget < cache_len ? budget : cache_len;
  const bool ranks = keep > 0 && keep < cache_len;  // otherwise nothing to choose
  if (ranks) {
    if (n_win < 1 || n_win > SCALEKV_MAX_WINDOW)
      return fail(SCALEKV_ERR_INVALID_ARG, "n_win %d is outside 1..%d", n_win, SCALEKV_MAX_WINDOW);
    if (n_win > n_cur)
      return fail(SCALEKV_ERR_INVALID_ARG, "n_win %d exceeds n_cur %d", n_win, n_cur);
    if (!win_idx) return fail(SCALEKV_ERR_INVALID_ARG, "win_idx is NULL");
    for (int j = 0; j < n_win; ++j)
      if (win_idx[j] < 0 || win_idx[j] >= n_cur)
        return fail(SCALEKV_ERR_INVALID_ARG, "win_idx[%d] = %d is outside 0..n_cur-1", j,
                    win_idx[j]);
    if (static_ws) {
      const size_t need = ws_layout(shape, cache_len).total;
      if (need > (size_t)SCALEKV_STATIC_SCRATCH_BYTES)
        return fail(SCALEKV_ERR_WORKSPACE,
                    "this shape needs %zu bytes of scratch, the library's static array holds %zu "
                    "(n_seq * n_head * cache_len too large for scalekv_step_static)",
                    need, (size_t)SCALEKV_STATIC_SCRATCH_BYTES);
    } else {
      SCALEKV_TRY(check_ws(shape, cache_len, ws, ws_bytes));
    }
  }
  SCALEKV_TRY(check_rows(shape, (long long)keep + n_cur, "keep + n_cur"));
  SCALEKV_TRY(check_dense(q, true, "q"));
  SCALEKV_TRY(check_dense(k_cur, true, "k_cur"));
  SCALEKV_TRY(check_dense(v_cur, true, "v_cur"));
  SCALEKV_TRY(check_dense(out, true, "out"));
  SCALEKV_TRY(check_kv(shape, k_src, cache_len, "k_src"));
  SCALEKV_TRY(check_kv(shape, v_src, cache_len, "v_src"));
  SCALEKV_TRY(check_kv(shape, k_dst, keep + n_cur, "k_dst"));
  SCALEKV_TRY(check_kv(shape, v_dst, keep + n_cur, "v_dst"));
  if (overlaps(shape, k_src, k_dst) || overlaps(shape, k_src, v_dst) ||
      overlaps(shape, v_src, k_dst) || overlaps(shape, v_src, v_dst) ||
      overlaps(shape, k_dst, v_dst))
    return fail(SCALEKV_ERR_INVALID_ARG, "source and destination caches overlap");
  // the destination caches are written while q, k_cur, v_cur are still being read and out is written
  for (const scalekv_kv* c : {k_dst, v_dst})
    if (dense_overlaps(shape, q, n_cur, c) || dense_overlaps(shape, k_cur, n_cur, c) ||
        dense_overlaps(shape, v_cur, n_cur, c) || dense_overlaps(shape, out, n_cur, c))
      return fail(SCALEKV_ERR_INVALID_ARG, "q, k_cur, v_cur or out overlaps a destination cache");

  if (static_ws && ranks) SCALEKV_TRY(static_scratch(&ws));  // every argument check has passed
  hipStream_t st = static_cast<hipStream_t>(stream);
  void** ev = g_stage_events;
  auto mark = [&](int i) -> hipError_t {
    return ev && ev[i] ? hipEventRecord(static_cast<hipEvent_t>(ev[i]), st) : hipSuccess;
  };
  const int U = shape->n_seq * shape->n_head;
  const int32_t* idx = nullptr;  // identity unless a ranking is needed
  const bool pipe = attend_uses_pipe(shape->dtype, shape->head_dim, n_cur);
  bool pruned = false;           // the ranking kernel has already written the destination caches
  SCALEKV_HIP(mark(0), "event record");
  if (ranks) {
    const WsLayout w = ws_layout(shape, cache_len);
    const ScoreWorkspace sw = score_ws(w, ws);
    float* scores = reinterpret_cast<float*>(static_cast<char*>(ws) + w.scores_off);
    int32_t* idx_ws = idx_out ? idx_out
                              : reinterpret_cast<int32_t*>(static_cast<char*>(ws) + w.idx_off);
    WindowRows rows;
    for (int j = 0; j < kMaxWindow; ++j) rows.row[j] = j < n_win ? win_idx[j] : 0;
    // One launch for the whole ranking where it pays (enough units to fill the chip, or short
    // caches): the selection kernel streams the keys itself.  Then event 1 coincides with event 0.
    // The same workgroup then prunes its unit as well: the kept rows go to the destination
    // caches (and the map's rows behind them where the attention kernel does not append).
    const PruneTarget prune{view(v_src), view(k_dst), view(v_dst), pipe ? nullptr : k_cur,
                            pipe ? nullptr : v_cur, n_cur};
    hipError_t one = launch_score_select(shape->dtype, shape->n_seq, shape->n_head, shape->head_dim, q,
                                         (long long)n_cur * shape->head_dim, rows, n_win,
                                         view(k_src), cache_len, resolve_scale(shape), sw, keep,
                                         idx_ws, nullptr, &prune, st);
    if (one == hipErrorNotSupported) {
      SCALEKV_HIP(launch_score_logits(shape->dtype, shape->n_seq, shape->n_head, shape->head_dim, q,
                                      (long long)n_cur * shape->head_dim, rows, n_win, view(k_src),
                                      cache_len, resolve_scale(shape), sw, st),
                  "score logits launch");
      SCALEKV_HIP(mark(1), "event record");
      // the finalisation of the score is fused into the select; very long caches take the
      // three-kernel route through the scores buffer
      hipError_t fused = launch_select_from_logits(U, n_win, sw, cache_len, keep, idx_ws, nullptr, st);
      if (fused == hipErrorNotSupported) {
        SCALEKV_HIP(launch_score_finalize(U, n_win, cache_len, sw, scores, w.len_pad, st),
                    "score finalize launch");
        SCALEKV_HIP(launch_select(U, scores, w.len_pad, cache_len, keep, idx_ws, nullptr, st),
                    "select launch");
      } else {
        SCALEKV_HIP(fused, "fused select launch");
      }
    } else {
      SCALEKV_HIP(one, "score + select + prune launch");
      SCALEKV_HIP(mark(1), "event record");   // after the launch: the stages up to the pruning share it
      pruned = true;
    }
    idx = idx_ws;
  } else {
    SCALEKV_HIP(mark(1), "event record");
    if (idx_out && keep > 0)  // keep == cache_len: the selection is the identity
      SCALEKV_HIP(launch_select(U, nullptr, 0, cache_len, keep, idx_out, nullptr, st),
                  "select launch");
  }
  SCALEKV_HIP(mark(2), "event record");
  // The pipelined attention kernel reads the map's own K/V from k_cur/v_cur and copies them
  // behind the kept rows itself (it is bound by the matrix pipe, the copy by the HBM, so the
  // two overlap); for the other shapes the pruning appends them.
  const bool fused_append = pipe;
  if (!pruned)
    SCALEKV_HIP(launch_compact(shape->dtype, shape->n_seq, shape->n_head, shape->head_dim,
                               view(k_src), view(v_src), idx, keep, k_cur, v_cur,
                               fused_append ? 0 : n_cur, view(k_dst), view(v_dst), st),
                "compact launch");
  if (fused_append) {
    // events 3 and 4 ride on this kernel's dispatch: its own start and end
    SCALEKV_HIP(launch_attend_pipe(U, shape->n_head, q, n_cur, view(k_dst), view(v_dst), keep, k_cur,
                                   v_cur, n_cur, true, resolve_scale(shape), out, st,
                                   ev ? static_cast<hipEvent_t>(ev[3]) : nullptr,
                                   ev ? static_cast<hipEvent_t>(ev[4]) : nullptr),
                "attend launch");
  } else {
    SCALEKV_HIP(mark(3), "event record");
    SCALEKV_HIP(launch_attend(shape->dtype, shape->n_seq, shape->n_head, shape->head_dim, q, n_cur,
                              view(k_dst), view(v_dst), keep + n_cur, resolve_scale(shape), out, st),
                "attend launch");
    SCALEKV_HIP(mark(4), "event record");
  }
  if (new_len_out) *new_len_out = keep + n_cur;
  return SCALEKV_OK;
}

}  // namespace

extern "C" {

scalekv_status scalekv_step(const scalekv_shape* shape, const void* q, const void* k_cur,
                            const void* v_cur, int32_t n_cur, const int32_t* win_idx,
                            int32_t n_win, const scalekv_kv* k_src, const scalekv_kv* v_src,
                            int32_t cache_len, int32_t budget, const scalekv_kv* k_dst,
                            const scalekv_kv* v_dst, int32_t* new_len_out, void* out,
                            int32_t* idx_out, void* ws, size_t ws_bytes, void* stream) {
  return step_impl(shape, q, k_cur, v_cur, n_cur, win_idx, n_win, k_src, v_src, cache_len, budget,
                   k_dst, v_dst, new_len_out, out, idx_out, ws, ws_bytes, false, stream);
}

scalekv_status scalekv_step_static(const scalekv_shape* shape, const void* q, const void* k_cur,
                                   const void* v_cur, int32_t n_cur, const int32_t* win_idx,
                                   int32_t n_win, const scalekv_kv* k_src, const scalekv_kv* v_src,
                                   int32_t cache_len, int32_t budget, const scalekv_kv* k_dst,
                                   const scalekv_kv* v_dst, int32_t* new_len_out, void* out,
                                   int32_t* idx_out, void* stream) {
  return step_impl(shape, q, k_cur, v_cur, n_cur, win_idx, n_win, k_src, v_src, cache_len, budget,
                   k_dst, v_dst, new_len_out, out, idx_out, nullptr, 0, true, stream);
}

scalekv_status scalekv_window_centroids(int32_t map_h, int32_t map_w, int32_t patch_rows,
                                        int32_t patch_cols, int32_t* idx_out, int32_t* n_out) {
  if (map_h < 1 || map_w < 1 || patch_rows < 1 || patch_cols < 1)
    return fail(SCALEKV_ERR_INVALID_ARG, "map %dx%d and patch grid %dx%d must be positive", map_h,
                map_w, patch_rows, patch_cols);
  if ((long long)map_h * map_w > 0x7fffffffLL)
    return fail(SCALEKV_ERR_UNSUPPORTED, "map %dx%d has too many tokens", map_h, map_w);
  if (!idx_out || !n_out) return fail(SCALEKV_ERR_INVALID_ARG, "idx_out or n_out is NULL");
  const int gr = patch_rows < map_h ? patch_rows : map_h;
  const int gc = patch_cols < map_w ? patch_cols : map_w;
  // Band a of gr covers rows [a*h/gr, (a+1)*h/gr).  The token nearest to the middle of a band
  // [lo, hi) is row (lo + hi - 1) / 2: for an even band the two middle rows are equally near
  // and the lower one is taken.  Rows and columns are independent, so the centroid of a patch
  // is (middle row of its row band, middle column of its column band).
  int n = 0;
  for (int a = 0; a < gr; ++a) {
    const int r_lo = (int)((long long)a * map_h / gr), r_hi = (int)((long long)(a + 1) * map_h / gr);
    const int r = (r_lo + r_hi - 1) / 2;
    for (int b = 0; b < gc; ++b) {
      const int c_lo = (int)((long long)b * map_w / gc), c_hi = (int)((long long)(b + 1) * map_w / gc);
      idx_out[n++] = r * map_w + (c_lo + c_hi - 1) / 2;
    }
  }
  *n_out = n;
  return SCALEKV_OK;
}

scalekv_status scalekv_select_window(const scalekv_shape* shape, const float* log_scores,
                                     int32_t cache_len, int32_t budget, const int32_t* forced,
                                     int32_t n_forced, int32_t pool_w, int32_t* idx,
                                     int32_t* keep_out, void* stream) {
  SCALEKV_TRY(check_shape(shape));
  SCALEKV_TRY(check_rows(shape, cache_len, "cache_len"));
  if (budget < 0) return fail(SCALEKV_ERR_INVALID_ARG, "budget is negative (%d)", budget);
  SelectExtras ex;
  SCALEKV_TRY(make_extras(forced, n_forced, pool_w, cache_len, &ex));
  const int rest = cache_len - n_forced;
  const int keep = n_forced + (budget < rest ? budget : rest);
  if (keep > 0) {
    if (!log_scores) return fail(SCALEKV_ERR_INVALID_ARG, "log_scores is NULL");
    if (!idx) return fail(SCALEKV_ERR_INVALID_ARG, "idx is NULL");
  }
  if (keep_out) *keep_out = keep;
  SCALEKV_HIP(launch_select(shape->n_seq * shape->n_head, log_scores, cache_len, cache_len, keep,
                            idx, &ex, static_cast<hipStream_t>(stream)),
              "select launch");
  return SCALEKV_OK;
}

scalekv_status scalekv_step_append_first(const scalekv_shape* shape, const void* q,
                                         const void* k_cur, const void* v_cur, int32_t n_cur,
                                         const int32_t* win_idx, int32_t n_win, int32_t pool_w,
                                         const scalekv_kv* k_cache, const scalekv_kv* v_cache,
                                         int32_t cache_len, int32_t budget,
                                         const scalekv_kv* k_next, const scalekv_kv* v_next,
                                         int32_t* keep_out, int32_t* moved_out, void* out,
                                         int32_t* idx_out, void* ws, size_t ws_bytes,
                                         void* stream) {
  SCALEKV_TRY(check_shape(shape));
  if (n_cur < 1) return fail(SCALEKV_ERR_INVALID_ARG, "n_cur must be >= 1 (got %d)", n_cur);
  SCALEKV_TRY(check_rows(shape, n_cur, "n_cur"));
  SCALEKV_TRY(check_rows(shape, cache_len, "cache_len"));
  const long long len_ll = (long long)cache_len + n_cur;
  SCALEKV_TRY(check_rows(shape, len_ll, "cache_len + n_cur"));
  const int len = (int)len_ll;
  if (budget < 0) return fail(SCALEKV_ERR_INVALID_ARG, "budget is negative (%d)", budget);
  if (n_win < 0 || n_win > SCALEKV_MAX_WINDOW)
    return fail(SCALEKV_ERR_INVALID_ARG, "n_win %d is outside 0..%d", n_win, SCALEKV_MAX_WINDOW);
  if (n_win > n_cur) return fail(SCALEKV_ERR_INVALID_ARG, "n_win %d exceeds n_cur %d", n_win, n_cur);
  if (n_win > 0 && !win_idx) return fail(SCALEKV_ERR_INVALID_ARG, "win_idx is NULL");
  int32_t forced[kMaxWindow];
  for (int j = 0; j < n_win; ++j) {
    if (win_idx[j] < 0 || win_idx[j] >= n_cur)
      return fail(SCALEKV_ERR_INVALID_ARG, "win_idx[%d] = %d is outside 0..n_cur-1", j, win_idx[j]);
    forced[j] = cache_len + win_idx[j];
  }
  SelectExtras ex;
  SCALEKV_TRY(make_extras(forced, n_win, pool_w, len, &ex));
  const int rest = len - n_win;
  const int keep = n_win + (budget < rest ? budget : rest);
  const bool moves = keep < len;            // otherwise everything is kept
  const bool ranks = moves && keep > 0;
  if (ranks && n_win < 1)
    return fail(SCALEKV_ERR_INVALID_ARG, "a ranking is needed but the window is empty");
  if (ranks) SCALEKV_TRY(check_ws(shape, len, ws, ws_bytes));
  SCALEKV_TRY(check_dense(q, true, "q"));
  SCALEKV_TRY(check_dense(k_cur, true, "k_cur"));
  SCALEKV_TRY(check_dense(v_cur, true, "v_cur"));
  SCALEKV_TRY(check_dense(out, true, "out"));
  SCALEKV_TRY(check_kv(shape, k_cache, len, "k_cache"));
  SCALEKV_TRY(check_kv(shape, v_cache, len, "v_cache"));
  if (overlaps(shape, k_cache, v_cache))
    return fail(SCALEKV_ERR_INVALID_ARG, "k_cache and v_cache overlap");
  for (const scalekv_kv* c : {k_cache, v_cache})
    if (dense_overlaps(shape, q, n_cur, c) || dense_overlaps(shape, k_cur, n_cur, c) ||
        dense_overlaps(shape, v_cur, n_cur, c) || dense_overlaps(shape, out, n_cur, c))
      return fail(SCALEKV_ERR_INVALID_ARG, "q, k_cur, v_cur or out overlaps a cache that is written");
  if (moves) {
    SCALEKV_TRY(check_kv(shape, k_next, keep, "k_next"));
    SCALEKV_TRY(check_kv(shape, v_next, keep, "v_next"));
    if (overlaps(shape, k_cache, k_next) || overlaps(shape, k_cache, v_next) ||
        overlaps(shape, v_cache, k_next) || overlaps(shape, v_cache, v_next) ||
        overlaps(shape, k_next, v_next))
      return fail(SCALEKV_ERR_INVALID_ARG, "cache and next-cache buffers overlap");
    // the pruning writes k_next / v_next after the attention has stored out, while q is still in use
    for (const scalekv_kv* c : {k_next, v_next})
      if (dense_overlaps(shape, q, n_cur, c) || dense_overlaps(shape, k_cur, n_cur, c) ||
          dense_overlaps(shape, v_cur, n_cur, c) || dense_overlaps(shape, out, n_cur, c))
        return fail(SCALEKV_ERR_INVALID_ARG, "q, k_cur, v_cur or out overlaps a next-cache buffer that is written");
  }

  hipStream_t st = static_cast<hipStream_t>(stream);
  void** ev = g_stage_events;
  auto mark = [&](int i) -> hipError_t {
    return ev && ev[i] ? hipEventRecord(static_cast<hipEvent_t>(ev[i]), st) : hipSuccess;
  };
  const int U = shape->n_seq * shape->n_head;
  const int d = shape->head_dim;
  SCALEKV_HIP(mark(0), "event record");
  // 1. the map's K/V join the cache: rows [cache_len, cache_len + n_cur) of every unit (the
  //    pipelined attention kernel does this itself, overlapped with its own work)
  const bool fused_append = attend_uses_pipe(shape->dtype, d, n_cur);
  if (!fused_append) {
    const long long tail = (long long)cache_len * d * elem_bytes(shape);
    KvView kt{static_cast<const char*>(k_cache->ptr) + tail, k_cache->seq_stride,
              k_cache->head_stride};
    KvView vt{static_cast<const char*>(v_cache->ptr) + tail, v_cache->seq_stride,
              v_cache->head_stride};
    SCALEKV_HIP(launch_compact(shape->dtype, shape->n_seq, shape->n_head, d, view(k_cache),
                               view(v_cache), nullptr, 0, k_cur, v_cur, n_cur, kt, vt, st),
                "append launch");
  }
  // 2. the map attends over history and itself
  if (fused_append) {
    // events 1 and 2 ride on this kernel's dispatch: its own start and end
    SCALEKV_HIP(launch_attend_pipe(U, shape->n_head, q, n_cur, view(k_cache), view(v_cache), cache_len,
                                   k_cur, v_cur, n_cur, true, resolve_scale(shape), out, st,
                                   ev ? static_cast<hipEvent_t>(ev[1]) : nullptr,
                                   ev ? static_cast<hipEvent_t>(ev[2]) : nullptr),
                "attend launch");
  } else {
    SCALEKV_HIP(mark(1), "event record");
    SCALEKV_HIP(launch_attend(shape->dtype, shape->n_seq, shape->n_head, d, q, n_cur, view(k_cache),
                              view(v_cache), len, resolve_scale(shape), out, st),
                "attend launch");
    SCALEKV_HIP(mark(2), "event record");
  }
  if (keep_out) *keep_out = keep;
  if (moved_out) *moved_out = moves ? 1 : 0;
  if (!moves) {  // everything is kept: the cache stays where it is
    if (idx_out)
      SCALEKV_HIP(launch_select(U, nullptr, 0, len, len, idx_out, nullptr, st), "select launch");
    SCALEKV_HIP(mark(3), "event record");
    SCALEKV_HIP(mark(4), "event record");
    return SCALEKV_OK;
  }
  // 3. scores of the window rows against the whole cache, pooled; window kept + top-budget
  bool pruned = false;  // the ranking kernel has already written the next cache
  int32_t* idx_ws = idx_out;
  if (!idx_ws && ranks)
    idx_ws = reinterpret_cast<int32_t*>(static_cast<char*>(ws) + ws_layout(shape, len).idx_off);
  if (ranks) {
    const WsLayout w = ws_layout(shape, len);
    const ScoreWorkspace sw = score_ws(w, ws);
    float* scores = reinterpret_cast<float*>(static_cast<char*>(ws) + w.scores_off);
    WindowRows rows;
    for (int j = 0; j < kMaxWindow; ++j) rows.row[j] = j < n_win ? win_idx[j] : 0;
    // (the ranking workgroup also moves its unit's kept rows into the next cache)
    const PruneTarget prune{view(v_cache), view(k_next), view(v_next), nullptr, nullptr, 0};
    hipError_t one = launch_score_select(shape->dtype, shape->n_seq, shape->n_head, d, q, (long long)n_cur * d, rows,
                                         n_win, view(k_cache), len, resolve_scale(shape), sw, keep,
                                         idx_ws, &ex, &prune, st);
    if (one == hipErrorNotSupported) {
      SCALEKV_HIP(launch_score_logits(shape->dtype, shape->n_seq, shape->n_head, d, q,
                                      (long long)n_cur * d, rows, n_win, view(k_cache), len,
                                      resolve_scale(shape), sw, st),
                  "score logits launch");
      hipError_t fused = launch_select_from_logits(U, n_win, sw, len, keep, idx_ws, &ex, st);
      if (fused == hipErrorNotSupported) {
        SCALEKV_HIP(launch_score_finalize(U, n_win, len, sw, scores, w.len_pad, st),
                    "score finalize launch");
        SCALEKV_HIP(launch_select(U, scores, w.len_pad, len, keep, idx_ws, &ex, st), "select launch");
      } else {
        SCALEKV_HIP(fused, "fused select launch");
      }
    } else {
      SCALEKV_HIP(one, "score + select + prune launch");
      pruned = true;
    }
  }
  SCALEKV_HIP(mark(3), "event record");
  // 4. the kept rows become the next cache
  if (!pruned)
    SCALEKV_HIP(launch_compact(shape->dtype, shape->n_seq, shape->n_head, d, view(k_cache),
                               view(v_cache), idx_ws, keep, nullptr, nullptr, 0, view(k_next),
                               view(v_next), st),
                "compact launch");
  SCALEKV_HIP(mark(4), "event record");
  return SCALEKV_OK;
}

// ---- offline policy: ASI (Eq. 2), drafter set (Eq. 3), budgets (Eq. 4), comparison policies

scalekv_status scalekv_asi(const scalekv_shape* shape, const void* q_samp, int32_t n_samp,
                           const scalekv_kv* k, int32_t hist_len, int32_t cur_len, int32_t top_k,
                           float* terms, float* asi_out, void* ws, size_t ws_bytes, void* stream) {
  SCALEKV_TRY(check_shape(shape));
  if (n_samp < 1 || n_samp > SCALEKV_MAX_ASI_SAMPLES)
    return fail(SCALEKV_ERR_INVALID_ARG, "n_samp %d is outside 1..%d", n_samp,
                SCALEKV_MAX_ASI_SAMPLES);
  if (top_k < 0) return fail(SCALEKV_ERR_INVALID_ARG, "top_k is negative (%d)", top_k);
  SCALEKV_TRY(check_rows(shape, hist_len, "hist_len"));
  SCALEKV_TRY(check_rows(shape, cur_len, "cur_len"));
  const long long len_ll = (long long)hist_len + cur_len;
  SCALEKV_TRY(check_rows(shape, len_ll, "hist_len + cur_len"));
  if (len_ll < 1) return fail(SCALEKV_ERR_INVALID_ARG, "hist_len + cur_len must be >= 1");
  const int len = (int)len_ll;
  SCALEKV_TRY(check_dense(q_samp, true, "q_samp"));
  SCALEKV_TRY(check_kv(shape, k, len, "k"));
  if (!terms) return fail(SCALEKV_ERR_INVALID_ARG, "terms is NULL");
  SCALEKV_TRY(check_ws(shape, len, ws, ws_bytes));
  const WsLayout w = ws_layout(shape, len);
  const ScoreWorkspace sw = score_ws(w, ws);
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int U = shape->n_seq * shape->n_head;
  for (int row0 = 0; row0 < n_samp; row0 += kMaxWindow) {
    const int n_rows = std::min(kMaxWindow, n_samp - row0);
    WindowRows rows;
    for (int j = 0; j < kMaxWindow; ++j) rows.row[j] = row0 + (j < n_rows ? j : 0);
    SCALEKV_HIP(launch_score_logits(shape->dtype, shape->n_seq, shape->n_head, shape->head_dim,
                                    q_samp, (long long)n_samp * shape->head_dim, rows, n_rows,
                                    view(k), len, resolve_scale(shape), sw, st),
                "asi logits launch");
    SCALEKV_HIP(launch_asi_terms(U, sw, n_rows, hist_len, len, top_k, terms, n_samp, row0, st),
                "asi terms launch");
  }
  if (asi_out)
    SCALEKV_HIP(launch_asi_mean(terms, (long long)U * n_samp, asi_out, st), "asi mean launch");
  return SCALEKV_OK;
}

scalekv_status scalekv_drafter_set(const double* asi, int32_t n_layer, int32_t n_scale,
                                   int32_t n_drafter, double eps, double* z_out,
                                   int32_t* is_drafter) {
  if (n_layer < 1 || n_scale < 1)
    return fail(SCALEKV_ERR_INVALID_ARG, "n_layer and n_scale must be positive (got %d, %d)",
                n_layer, n_scale);
  if ((long long)n_layer * n_scale > 0x7fffffffLL)
    return fail(SCALEKV_ERR_UNSUPPORTED, "n_layer * n_scale is too large");
  if (n_drafter < 0) return fail(SCALEKV_ERR_INVALID_ARG, "n_drafter is negative (%d)", n_drafter);
  if (!(eps >= 0.0)) return fail(SCALEKV_ERR_INVALID_ARG, "eps must be >= 0");
  if (!asi || !is_drafter) return fail(SCALEKV_ERR_INVALID_ARG, "asi or is_drafter is NULL");
  const int L = n_layer, K = n_scale, total = L * K;
  for (int i = 0; i < total; ++i)
    if (!std::isfinite(asi[i])) return fail(SCALEKV_ERR_INVALID_ARG, "asi[%d] is not finite", i);
  std::vector<double> z((size_t)total);
  for (int k = 0; k < K; ++k) {
    double sum = 0.0;
    for (int l = 0; l < L; ++l) sum += asi[(size_t)l * K + k];
    const double mu = sum / L;
    double ss = 0.0;
    for (int l = 0; l < L; ++l) ss += (asi[(size_t)l * K + k] - mu) * (asi[(size_t)l * K + k] - mu);
    const double denom = std::sqrt(ss / L) + eps;  // population deviation of the scale
    for (int l = 0; l < L; ++l)
      z[(size_t)l * K + k] = denom > 0.0 ? (asi[(size_t)l * K + k] - mu) / denom : 0.0;
  }
  // rank every (layer, scale) pair by (Z, scale, layer) and take the first n_drafter
  std::vector<int> order((size_t)total);
  for (int i = 0; i < total; ++i) order[i] = i;
  std::sort(order.begin(), order.end(), [&](int a, int b) {
    if (z[a] != z[b]) return z[a] < z[b];
    const int ka = a % K, kb = b % K;
    if (ka != kb) return ka < kb;
    return a / K < b / K;
  });
  const int take = std::min(n_drafter, total);
  for (int i = 0; i < total; ++i) is_drafter[i] = 0;
  for (int i = 0; i < take; ++i) is_drafter[order[i]] = 1;
  if (z_out) std::memcpy(z_out, z.data(), (size_t)total * sizeof(double));
  return SCALEKV_OK;
}

scalekv_status scalekv_allocate_budgets(int32_t n_layer, int32_t n_scale, const int32_t* n_drafter,
                                        int64_t b_uniform, int64_t b_r0, int64_t delta,
                                        int64_t b_min, int32_t* b_r, int32_t* b_d, int64_t* slack) {
  if (n_layer < 1 || n_scale < 1)
    return fail(SCALEKV_ERR_INVALID_ARG, "n_layer and n_scale must be positive (got %d, %d)",
                n_layer, n_scale);
  if (!n_drafter || !b_r || !b_d) return fail(SCALEKV_ERR_INVALID_ARG, "n_drafter, b_r or b_d is NULL");
  constexpr int64_t kMax = 0x7fffffffLL;
  if (b_uniform < 0 || b_r0 < 0 || delta < 0 || b_min < 0 || b_uniform > kMax || b_r0 > kMax ||
      delta > kMax || b_min > kMax)
    return fail(SCALEKV_ERR_INVALID_ARG, "b_uniform, b_r0, delta and b_min must be in 0..2^31-1");
  int64_t n_d_total = 0, refiner_tokens = 0;
  for (int k = 0; k < n_scale; ++k) {
    if (n_drafter[k] < 0 || n_drafter[k] > n_layer)
      return fail(SCALEKV_ERR_INVALID_ARG, "n_drafter[%d] = %d is outside 0..n_layer", k,
                  n_drafter[k]);
    n_d_total += n_drafter[k];
    refiner_tokens += (int64_t)(n_layer - n_drafter[k]) * std::max(b_min, b_r0 - delta * (k + 1));
  }
  const int64_t target = b_uniform * n_layer * n_scale;
  if (n_d_total == 0)
    return fail(SCALEKV_ERR_INVALID_ARG, "no drafter layer at any scale: nothing can take the pool");
  if (refiner_tokens > target)
    return fail(SCALEKV_ERR_INVALID_ARG,
                "the refiner budgets alone (%lld tokens) exceed the uniform total (%lld)",
                (long long)refiner_tokens, (long long)target);
  const int64_t each = (target - refiner_tokens) / n_d_total;
  if (each > kMax) return fail(SCALEKV_ERR_UNSUPPORTED, "drafter budget does not fit int32");
  for (int k = 0; k < n_scale; ++k) b_r[k] = (int32_t)std::max(b_min, b_r0 - delta * (k + 1));
  *b_d = (int32_t)each;
  if (slack) *slack = target - refiner_tokens - each * n_d_total;
  return SCALEKV_OK;
}

scalekv_status scalekv_policy_table(const double* asi, int32_t n_layer, int32_t n_scale,
                                    int32_t n_drafter, double eps, int64_t b_uniform,
                                    int64_t b_r0, int64_t delta, int64_t b_min, int32_t* table,
                                    int32_t* is_drafter, int32_t* b_r, int32_t* b_d,
                                    int64_t* slack) {
  if (!table) return fail(SCALEKV_ERR_INVALID_ARG, "table is NULL");
  if (n_drafter < 1) return fail(SCALEKV_ERR_INVALID_ARG, "n_drafter must be >= 1 (got %d)", n_drafter);
  if (n_layer < 1 || n_scale < 1)
    return fail(SCALEKV_ERR_INVALID_ARG, "n_layer and n_scale must be positive (got %d, %d)",
                n_layer, n_scale);
  if ((long long)n_layer * n_scale > 0x7fffffffLL)
    return fail(SCALEKV_ERR_UNSUPPORTED, "n_layer * n_scale is too large");
  const size_t total = (size_t)n_layer * n_scale;
  std::vector<int32_t> role(total), per_scale((size_t)n_scale, 0), refiner((size_t)n_scale);
  SCALEKV_TRY(scalekv_drafter_set(asi, n_layer, n_scale, n_drafter, eps, nullptr, role.data()));
  for (int l = 0; l < n_layer; ++l)
    for (int k = 0; k < n_scale; ++k) per_scale[k] += role[(size_t)l * n_scale + k];
  int32_t drafter = 0;
  int64_t rest = 0;
  SCALEKV_TRY(scalekv_allocate_budgets(n_layer, n_scale, per_scale.data(), b_uniform, b_r0, delta,
                                       b_min, refiner.data(), &drafter, &rest));
  for (int l = 0; l < n_layer; ++l)
    for (int k = 0; k < n_scale; ++k)
      table[(size_t)l * n_scale + k] = role[(size_t)l * n_scale + k] ? drafter : refiner[k];
  if (is_drafter) std::memcpy(is_drafter, role.data(), total * sizeof(int32_t));
  if (b_r) std::memcpy(b_r, refiner.data(), (size_t)n_scale * sizeof(int32_t));
  if (b_d) *b_d = drafter;
  if (slack) *slack = rest;
  return SCALEKV_OK;
}

scalekv_status scalekv_pyramid_budgets(int32_t n_layer, int64_t b_uniform, int64_t b_last,
                                       int32_t* b) {
  if (n_layer < 1) return fail(SCALEKV_ERR_INVALID_ARG, "n_layer must be positive (got %d)", n_layer);
  if (!b) return fail(SCALEKV_ERR_INVALID_ARG, "b is NULL");
  if (b_uniform < 0 || b_uniform > 0x3fffffffLL || b_last < 0 || b_last > b_uniform)
    return fail(SCALEKV_ERR_INVALID_ARG, "need 0 <= b_last <= b_uniform < 2^30");
  const int64_t span = 2 * (b_uniform - b_last);  // first layer's budget minus the last layer's
  for (int l = 0; 2 * l < n_layer - 1; ++l) {
    const int64_t drop = span * l / (n_layer - 1);
    b[l] = (int32_t)(b_last + span - drop);
    b[n_layer - 1 - l] = (int32_t)(b_last + drop);
  }
  if (n_layer % 2) b[n_layer / 2] = (int32_t)b_uniform;
  return SCALEKV_OK;
}

scalekv_status scalekv_select_positional(const scalekv_shape* shape, int32_t cache_len,
                                         int32_t n_sink, int32_t n_recent, int32_t* idx,
                                         int32_t* keep_out, void* stream) {
  SCALEKV_TRY(check_shape(shape));
  SCALEKV_TRY(check_rows(shape, cache_len, "cache_len"));
  if (n_sink < 0 || n_recent < 0)
    return fail(SCALEKV_ERR_INVALID_ARG, "n_sink and n_recent must be >= 0 (got %d, %d)", n_sink,
                n_recent);
  const int sink = std::min(n_sink, cache_len);
  const int keep = sink + std::min(n_recent, cache_len - sink);
  if (keep > 0 && !idx) return fail(SCALEKV_ERR_INVALID_ARG, "idx is NULL");
  if (keep_out) *keep_out = keep;
  SCALEKV_HIP(launch_positional(shape->n_seq * shape->n_head, cache_len, sink, keep, idx,
                                static_cast<hipStream_t>(stream)),
              "positional launch");
  return SCALEKV_OK;
}

}  // extern "C"
