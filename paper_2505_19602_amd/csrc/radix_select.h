// Workgroup-wide radix select over 32-bit keys, shared by the top-k selection
// (Sec. 3.3) and the history top-K' sum of the Attention Selectivity Index (Eq. 2).
#pragma once
#include "common.h"

namespace scalekv {

// Order-preserving image of a float: a > b  <=>  order_key(a) > order_key(b); -0 and +0 rank equal.
__device__ __forceinline__ uint32_t order_key(float f) {
  const uint32_t b = __float_as_uint(f + 0.0f);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float order_key_value(uint32_t k) {
  return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

// Inclusive prefix sum over the 64 lanes of a wave, all lanes active.  Within a row of 16 lanes
// four data-parallel-primitive adds (shift right by 1, 2, 4, 8; lanes shifted in from outside the
// row read zero), then the totals of rows 0..2 are added to the rows behind them.
__device__ __forceinline__ uint32_t wave_prefix_sum(uint32_t x, int lane) {
#define SCALEKV_ROW_SHR(v, n) \
  (uint32_t) __builtin_amdgcn_update_dpp(0, (int)(v), 0x110 + (n), 0xf, 0xf, true)
  x += SCALEKV_ROW_SHR(x, 1);
  x += SCALEKV_ROW_SHR(x, 2);
  x += SCALEKV_ROW_SHR(x, 4);
  x += SCALEKV_ROW_SHR(x, 8);
#undef SCALEKV_ROW_SHR
  const uint32_t t0 = __builtin_amdgcn_readlane(x, 15), t1 = __builtin_amdgcn_readlane(x, 31),
                 t2 = __builtin_amdgcn_readlane(x, 47);
  return x + (lane >= 16 ? t0 : 0u) + (lane >= 32 ? t1 : 0u) + (lane >= 48 ? t2 : 0u);
}

constexpr int kRadixHistWords = 4 * 256;  // LDS scratch of radix_kth_largest: one histogram per pass

// Among the n keys key_at(0..n-1) finds T, the key of the k-th largest (1 <= k <= n), in four
// passes of 8 bits, and need_eq >= 1, the number of keys equal to T that belong to the k
// largest.  Every thread of the workgroup (THREADS >= 256, a multiple of 64) must call it with
// the same arguments; hist (kRadixHistWords words) is LDS scratch.  Integer work only, so the
// result does not depend on the order in which threads run.
//
// One barrier per pass: each pass has a histogram of its own (all cleared up front), and after
// the barrier every wave walks the histogram by itself and arrives at the same digit, so
// nothing has to be handed from one wave to the others.  Keys of real scores share their top
// bits, which would send a whole wave's atomics to one LDS word; the lanes that hold the same
// digit as the first active lane are therefore counted with one ballot and added by that lane
// alone (twice in a row), and only the lanes left over add one by one.
template <int THREADS, typename KeyAt>
__device__ __forceinline__ void radix_kth_largest(KeyAt key_at, int n, uint32_t k, uint32_t* hist,
                                                  uint32_t& T, uint32_t& need_eq) {
  static_assert(THREADS >= 256 && THREADS % 64 == 0, "whole waves, at least four of them");
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  for (int b = tid; b < kRadixHistWords; b += THREADS) hist[b] = 0;
  __syncthreads();
  uint32_t prefix = 0, mask = 0, remaining = k;
#pragma unroll
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    uint32_t* h = hist + 256 * pass;
    for (int i = tid; i < n; i += THREADS) {
      const uint32_t kk = key_at(i);
      bool act = (kk & mask) == prefix;
      const uint32_t digit = (kk >> shift) & 255u;
#pragma unroll
      for (int round = 0; round < 2; ++round) {
        const unsigned long long am = __builtin_amdgcn_ballot_w64(act);
        if (am == 0) break;
        const int first = __builtin_ctzll(am);
        const uint32_t d0 = __builtin_amdgcn_readlane(digit, first);
        const unsigned long long same = __builtin_amdgcn_ballot_w64(act && digit == d0);
        if (lane == first) atomicAdd(&h[d0], (uint32_t)__builtin_popcountll(same));
        act = act && digit != d0;
      }
      if (act) atomicAdd(&h[digit], 1u);
    }
    __syncthreads();
    // lane L owns bins 4L..4L+3; `above` = count in all bins higher than the lane's
    const uint4 own = *reinterpret_cast<const uint4*>(h + 4 * lane);
    const uint32_t mine = own.x + own.y + own.z + own.w;
    const uint32_t upto = wave_prefix_sum(mine, lane);  // bins 0 .. 4L+3
    uint32_t above = __builtin_amdgcn_readlane(upto, 63) - upto;
    // walk the lane's bins from the top; exactly one bin of one lane holds the k-th largest
    const uint32_t hh[4] = {own.w, own.z, own.y, own.x};
    uint32_t digit_sel = 0, rem_sel = 0;
    bool found = false;
#pragma unroll
    for (int b = 0; b < 4; ++b) {
      if (above < remaining && remaining <= above + hh[b]) {
        found = true;
        digit_sel = 4 * lane + (3 - b);
        rem_sel = remaining - above;
      }
      above += hh[b];
    }
    const int owner = __builtin_ctzll(__builtin_amdgcn_ballot_w64(found));
    prefix |= (uint32_t)__builtin_amdgcn_readlane(digit_sel, owner) << shift;
    remaining = __builtin_amdgcn_readlane(rem_sel, owner);
    mask |= 255u << shift;
  }
  T = prefix;
  need_eq = remaining;
}

}  // namespace scalekv
