// Wave-level pieces of the bf16 importance-score logits (Eq. 5), shared by the score kernel
// and by the selection kernel that forms the logits itself.
//
// A wave multiplies 16 * NT cached keys by the (at most 16) window queries with MFMA 16x16x32:
// A = key rows read straight from global memory, 16 bytes per lane, every byte of every key row
// exactly once; B = window queries in registers.  All of the wave's key vectors are requested
// before the first MFMA, so that NT * D / 8 KB are in flight per wave.
//   A (16 x 32): lane holds row l%16, k-indices 8(l/16)..+7
//   B (32 x 16): lane holds column l%16, k-indices 8(l/16)..+7
//   C (16 x 16): lane holds column l%16, rows 4(l/16) + v, v = 0..3
#pragma once
#include "common.h"

namespace scalekv {

typedef __attribute__((ext_vector_type(8))) __bf16 score_bf16x8;
typedef __attribute__((ext_vector_type(4))) float score_f32x4;

// Window queries as the B operand: lane's column is window row l%16 (zero beyond n_win).
template <int D>
__device__ __forceinline__ void score_load_window(const uint16_t* qu, const WindowRows& rows, int n_win,
                                                  score_bf16x8 (&qf)[D / 32]) {
  const int lane = threadIdx.x & 63, i = lane & 15, g = lane >> 4;
#pragma unroll
  for (int sl = 0; sl < D / 32; ++sl) {
    uint4 raw = make_uint4(0, 0, 0, 0);
    if (i < n_win) raw = *(const uint4*)(qu + (long long)rows.row[i] * D + 32 * sl + 8 * g);
    qf[sl] = __builtin_bit_cast(score_bf16x8, raw);
  }
}

// Logits (scaled) of keys key0 .. key0 + 16 NT - 1 of one unit against the window rows: written
// key-major to logits_unit[key * kMaxWindow + row] for keys below cache_len.  On return every
// lane holds, for its window row l%16, m = the maximum of those logits over the wave's valid
// keys (-inf if none) and e = the sum of exp(logit - m) over them.
template <int D, int NT>
__device__ __forceinline__ void score_wave_logits(const uint16_t* ku, const score_bf16x8 (&qf)[D / 32],
                                                  int key0, int cache_len, float sm_scale,
                                                  float* logits_unit, float& m, float& e) {
  constexpr int NSL = D / 32;
  const int lane = threadIdx.x & 63, i = lane & 15, g = lane >> 4;
  score_bf16x8 kf[NT][NSL];
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    const int key = min(key0 + 16 * t + i, cache_len - 1);  // clamp: legal address, value unused
#pragma unroll
    for (int sl = 0; sl < NSL; ++sl)
      kf[t][sl] = __builtin_bit_cast(score_bf16x8, *(const uint4*)(ku + (long long)key * D + 32 * sl + 8 * g));
  }
  m = -INFINITY;
  score_f32x4 c[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    c[t] = score_f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int sl = 0; sl < NSL; ++sl)
      c[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[t][sl], qf[sl], c[t], 0, 0, 0);
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int key = key0 + 16 * t + 4 * g + v;
      c[t][v] = key < cache_len ? c[t][v] * sm_scale : -INFINITY;
      m = fmaxf(m, c[t][v]);
      if (key < cache_len) logits_unit[(long long)key * kMaxWindow + i] = c[t][v];
    }
  }
  // row statistics of window row i over this wave's keys
  m = fmaxf(m, __shfl_xor(m, 16));
  m = fmaxf(m, __shfl_xor(m, 32));
  e = 0.f;
  if (m > -INFINITY) {
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int v = 0; v < 4; ++v) e += expf(c[t][v] - m);
  }
  e += __shfl_xor(e, 16);
  e += __shfl_xor(e, 32);
}

}  // namespace scalekv
