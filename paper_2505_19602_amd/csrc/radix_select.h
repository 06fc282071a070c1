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

// Among the n keys key_at(0..n-1) finds T, the key of the k-th largest (1 <= k <= n), in four
// passes of 8 bits, and need_eq >= 1, the number of keys equal to T that belong to the k
// largest.  Every thread of the workgroup (THREADS >= 256) must call it with the same
// arguments; hist (256 words) and sel (2 words) are LDS scratch.  Integer work only, so the
// result does not depend on the order in which threads run.
template <int THREADS, typename KeyAt>
__device__ __forceinline__ void radix_kth_largest(KeyAt key_at, int n, uint32_t k, uint32_t* hist,
                                                  uint32_t* sel, uint32_t& T, uint32_t& need_eq) {
  const int tid = threadIdx.x;
  uint32_t prefix = 0, mask = 0, remaining = k;
  for (int shift = 24; shift >= 0; shift -= 8) {
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
    for (int i = tid; i < n; i += THREADS) {
      const uint32_t kk = key_at(i);
      if ((kk & mask) == prefix) atomicAdd(&hist[(kk >> shift) & 255u], 1u);
    }
    __syncthreads();
    if (tid < 64) {
      // lane L owns bins 4L..4L+3; `above` = count in all bins higher than the lane's.
      const uint32_t h0 = hist[4 * tid], h1 = hist[4 * tid + 1], h2 = hist[4 * tid + 2],
                     h3 = hist[4 * tid + 3];
      const uint32_t mine = h0 + h1 + h2 + h3;
      uint32_t incl = mine;  // inclusive suffix sum over lanes >= tid
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const uint32_t other = __shfl_down(incl, off);
        if (tid + off < 64) incl += other;
      }
      uint32_t above = incl - mine;
      // walk the lane's bins from the top
      const uint32_t hh[4] = {h3, h2, h1, h0};
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        if (above < remaining && remaining <= above + hh[b]) {
          sel[0] = 4 * tid + (3 - b);
          sel[1] = remaining - above;
        }
        above += hh[b];
      }
    }
    __syncthreads();
    prefix |= sel[0] << shift;
    mask |= 255u << shift;
    remaining = sel[1];
    __syncthreads();
  }
  T = prefix;
  need_eq = remaining;
}

}  // namespace scalekv
