// Driver for the host-sanitizer build of the C ABI layer (AddressSanitizer + UBSan on the host
// code only): walks the argument checks of every entry point with fake but aligned device
// pointers (nothing is launched: every call below is rejected on the host or is host-only work)
// and runs the host-side policy routines into heap buffers of exactly the documented size, so
// that an overrun in the library's host code is reported.  Built and run by
// `python -m paper_2505_19602_amd.build --sanitize` and tests/test_sanitizers.py; needs no GPU.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <memory>
#include <vector>

#include "../../include/scalekv.h"

static int failures = 0;
#define EXPECT(cond)                                                        \
  do {                                                                      \
    if (!(cond)) {                                                          \
      std::printf("FAILED %s:%d: %s (last error: %s)\n", __FILE__, __LINE__, #cond, scalekv_last_error()); \
      ++failures;                                                           \
    }                                                                       \
  } while (0)

static void* fake(uintptr_t a) { return reinterpret_cast<void*>(a); }

int main() {
  scalekv_shape s{1, 2, 128, SCALEKV_BF16, 0.f};
  const int64_t cap = 64, d = 128, heads = 2;
  auto kv = [&](uintptr_t base, int32_t capacity = 64) {
    return scalekv_kv{fake(base), capacity * d * heads, capacity * d, capacity};
  };
  const uintptr_t span = (uintptr_t)(cap * d * heads * 2);
  scalekv_kv k = kv(0x100000), v = kv(0x100000 + span), kd = kv(0x100000 + 2 * span), vd = kv(0x100000 + 3 * span);
  size_t bytes = 0;
  EXPECT(scalekv_workspace_bytes(&s, 1000, 64, &bytes) == SCALEKV_OK && bytes > 0);
  EXPECT(scalekv_workspace_bytes(nullptr, 10, 1, &bytes) == SCALEKV_ERR_INVALID_ARG);
  EXPECT(scalekv_workspace_bytes(&s, 10, 1, nullptr) == SCALEKV_ERR_INVALID_ARG);
  scalekv_shape bad = s;
  bad.head_dim = 96;
  EXPECT(scalekv_workspace_bytes(&bad, 10, 1, &bytes) == SCALEKV_ERR_UNSUPPORTED);
  bad = s; bad.n_seq = 70000;
  EXPECT(scalekv_workspace_bytes(&bad, 10, 1, &bytes) == SCALEKV_ERR_UNSUPPORTED);

  // score / select / compact / attend: rejected before any launch
  EXPECT(scalekv_score(&s, fake(0x1000), 17, &k, 10, (float*)fake(0x2000), fake(0x8000), 1 << 30, nullptr) == SCALEKV_ERR_INVALID_ARG);
  EXPECT(scalekv_score(&s, fake(0x1004), 4, &k, 10, (float*)fake(0x2000), fake(0x8000), 1 << 30, nullptr) == SCALEKV_ERR_INVALID_ARG);
  EXPECT(scalekv_score(&s, fake(0x1000), 4, &k, 65, (float*)fake(0x2000), fake(0x8000), 1 << 30, nullptr) == SCALEKV_ERR_INVALID_ARG);
  EXPECT(scalekv_score(&s, fake(0x1000), 4, &k, 10, (float*)fake(0x2000), fake(0x8000), 8, nullptr) == SCALEKV_ERR_WORKSPACE);
  int32_t keep = -1;
  EXPECT(scalekv_select(&s, (const float*)fake(0x1000), 10, -1, (int32_t*)fake(0x2000), &keep, nullptr) == SCALEKV_ERR_INVALID_ARG);
  EXPECT(scalekv_select(&s, nullptr, 10, 3, (int32_t*)fake(0x2000), &keep, nullptr) == SCALEKV_ERR_INVALID_ARG);
  EXPECT(scalekv_compact(&s, &k, &v, 10, nullptr, 11, nullptr, nullptr, 0, &kd, &vd, nullptr) == SCALEKV_ERR_INVALID_ARG);
  EXPECT(scalekv_compact(&s, &k, &v, 10, nullptr, 5, nullptr, nullptr, 0, &k, &vd, nullptr) == SCALEKV_ERR_INVALID_ARG);
  EXPECT(scalekv_compact(&s, &k, &v, 10, nullptr, 5, fake(0x1000), nullptr, 4, &kd, &vd, nullptr) == SCALEKV_ERR_INVALID_ARG);
  EXPECT(scalekv_attend(&s, fake(0x1000), 8, &k, &v, 0, fake(0x2000), nullptr) == SCALEKV_ERR_INVALID_ARG);
  EXPECT(scalekv_attend(&s, fake(0x1000), 0, &k, &v, 10, fake(0x2000), nullptr) == SCALEKV_OK);

  // step, step_static, step_append_first
  int32_t win[4] = {0, 1, 2, 9}, new_len = -1, moved = -1;
  EXPECT(scalekv_step(&s, fake(0x1000), fake(0x2000), fake(0x3000), 8, win, 4, &k, &v, 40, 10, &kd, &vd, &new_len,
                      fake(0x4000), nullptr, fake(0x8000), 1 << 30, nullptr) == SCALEKV_ERR_INVALID_ARG);   // win 9 >= 8
  EXPECT(scalekv_step(&s, fake(0x1000), fake(0x2000), fake(0x3000), 16, win, 4, &k, &v, 40, 10, &kd, &vd, &new_len,
                      fake(0x4000), nullptr, nullptr, 0, nullptr) == SCALEKV_ERR_WORKSPACE);
  EXPECT(scalekv_step(&s, fake(0x1000), fake(0x2000), fake(0x3000), 60, win, 3, &k, &v, 40, 10, &kd, &vd, &new_len,
                      fake(0x4000), nullptr, fake(0x8000), 1 << 30, nullptr) == SCALEKV_ERR_INVALID_ARG);   // capacity
  EXPECT(scalekv_step(&s, fake(0x1000), fake(0x2000), fake(0x3000), 16, win, 3, &k, &v, 40, 10, &k, &vd, &new_len,
                      fake(0x4000), nullptr, fake(0x8000), 1 << 30, nullptr) == SCALEKV_ERR_INVALID_ARG);   // src == dst
  {
    const uintptr_t gib = (uintptr_t)1 << 30;
    scalekv_kv bk = kv(4 * gib, 600064), bv = kv(5 * gib, 600064), bkd = kv(6 * gib, 600064), bvd = kv(7 * gib, 600064);
    EXPECT(scalekv_step_static(&s, fake(0x1000), fake(0x2000), fake(0x3000), 8, win, 3, &bk, &bv, 600000, 100, &bkd,
                               &bvd, &new_len, fake(0x4000), nullptr, nullptr) == SCALEKV_ERR_WORKSPACE);
  }
  EXPECT(scalekv_step_static(&s, fake(0x1000), fake(0x2000), fake(0x3000), 0, win, 3, &k, &v, 40, 10, &kd, &vd,
                             &new_len, fake(0x4000), nullptr, nullptr) == SCALEKV_ERR_INVALID_ARG);
  EXPECT(scalekv_step_append_first(&s, fake(0x1000), fake(0x2000), fake(0x3000), 8, win, 3, 2, &k, &v, 40, 10, &kd, &vd,
                                   &keep, &moved, fake(0x4000), nullptr, fake(0x8000), 1 << 30, nullptr) ==
         SCALEKV_ERR_INVALID_ARG);   // even pooling width
  EXPECT(scalekv_step_append_first(&s, fake(0x1000), fake(0x2000), fake(0x3000), 8, win, 0, 1, &k, &v, 40, 10, &kd, &vd,
                                   &keep, &moved, fake(0x4000), nullptr, fake(0x8000), 1 << 30, nullptr) ==
         SCALEKV_ERR_INVALID_ARG);   // a ranking without a window
  // out overlapping the next cache that the final pruning writes
  EXPECT(scalekv_step_append_first(&s, fake(0x1000), fake(0x2000), fake(0x3000), 8, win, 3, 1, &k, &v, 40, 10, &kd, &vd,
                                   &keep, &moved, kd.ptr, nullptr, fake(0x8000), 1 << 30, nullptr) ==
         SCALEKV_ERR_INVALID_ARG);

  // selection with a window, positional selection: argument errors only
  int32_t forced[3] = {1, 5, 5};
  EXPECT(scalekv_select_window(&s, (const float*)fake(0x1000), 20, 4, forced, 3, 3, (int32_t*)fake(0x2000), &keep,
                               nullptr) == SCALEKV_ERR_INVALID_ARG);   // repeated position
  forced[2] = 20;
  EXPECT(scalekv_select_window(&s, (const float*)fake(0x1000), 20, 4, forced, 3, 3, (int32_t*)fake(0x2000), &keep,
                               nullptr) == SCALEKV_ERR_INVALID_ARG);   // out of range
  EXPECT(scalekv_select_positional(&s, 20, -1, 3, (int32_t*)fake(0x2000), &keep, nullptr) == SCALEKV_ERR_INVALID_ARG);
  EXPECT(scalekv_select_positional(&s, 20, 2, 3, nullptr, &keep, nullptr) == SCALEKV_ERR_INVALID_ARG);
  EXPECT(scalekv_asi(&s, fake(0x1000), 0, &k, 10, 10, 4, (float*)fake(0x2000), nullptr, fake(0x8000), 1 << 30,
                     nullptr) == SCALEKV_ERR_INVALID_ARG);

  // host-only routines into buffers of exactly the documented size
  for (int h = 1; h <= 70; h += 23)
    for (int w = 1; w <= 9; w += 4)
      for (int g = 1; g <= 5; g += 2) {
        const int n_max = (g < h ? g : h) * (g < w ? g : w);
        std::unique_ptr<int32_t[]> idx(new int32_t[n_max]);
        int32_t n = -1;
        EXPECT(scalekv_window_centroids(h, w, g, g, idx.get(), &n) == SCALEKV_OK && n == n_max);
        for (int i = 0; i < n; ++i) EXPECT(idx[i] >= 0 && idx[i] < h * w);
      }
  EXPECT(scalekv_window_centroids(0, 4, 4, 4, win, &keep) == SCALEKV_ERR_INVALID_ARG);
  for (int L = 1; L <= 7; L += 3)
    for (int K = 1; K <= 13; K += 6) {
      std::vector<double> asi((size_t)L * K), z((size_t)L * K);
      for (size_t i = 0; i < asi.size(); ++i) asi[i] = 0.01 * (double)((i * 37) % 11);
      std::unique_ptr<int32_t[]> role(new int32_t[L * K]), table(new int32_t[L * K]), b_r(new int32_t[K]), nd(new int32_t[K]);
      EXPECT(scalekv_drafter_set(asi.data(), L, K, (L * K + 1) / 2, 1e-8, z.data(), role.get()) == SCALEKV_OK);
      int32_t b_d = -1;
      int64_t slack = -1;
      for (int kk = 0; kk < K; ++kk) nd[kk] = (kk % L) + (L > 1 ? 0 : 1);
      nd[0] = 1;
      EXPECT(scalekv_allocate_budgets(L, K, nd.get(), 650, 600, 70, 0, b_r.get(), &b_d, &slack) == SCALEKV_OK);
      EXPECT(scalekv_policy_table(asi.data(), L, K, (L * K + 1) / 2, 1e-8, 650, 600, 70, 0, table.get(), role.get(),
                                  b_r.get(), &b_d, &slack) == SCALEKV_OK);
      std::unique_ptr<int32_t[]> pyr(new int32_t[L]);
      EXPECT(scalekv_pyramid_budgets(L, 650, 100, pyr.get()) == SCALEKV_OK);
    }
  EXPECT(scalekv_pyramid_budgets(4, 10, 11, win) == SCALEKV_ERR_INVALID_ARG);
  EXPECT(std::strlen(scalekv_version()) > 0);
  std::printf("ABI host sanitizer run complete, %d failed expectations\n", failures);
  return failures != 0;
}
