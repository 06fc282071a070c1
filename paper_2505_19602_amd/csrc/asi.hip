// Attention Selectivity Index, Eq. 2: for sampled queries of the current map, the
// attention mass that falls on the map's own keys and the sum of the K' largest
// weights on the history keys.  Calibration-time work (the paper runs it once, on
// a handful of prompts), built on the score kernels: the logits of up to 16 query
// rows against every key are already in the workspace, key-major, with the
// per-chunk softmax statistics beside them.
//
// One workgroup per (unit, query row).  The row's normaliser comes from the chunk
// statistics; the current-map mass is a plain sum; the top-K' sum needs no sort:
// a radix select over the order-preserving images of the history logits gives the
// K'-th largest value T, and the sum is (weights above T) + (copies of T that belong
// to the top K') * weight(T) -- equal logits have equal weights, so which of them are
// taken does not matter.  All float sums run in a fixed order (strided per thread,
// butterfly per wave, waves in sequence): results do not depend on scheduling.
#include "common.h"
#include "radix_select.h"

namespace scalekv {
namespace {

constexpr int kThreads = 1024;
constexpr int kWaves = kThreads / 64;
constexpr int kLdsKeys = 12288;  // history rows up to this many keep their keys in LDS

// Sum of x over the workgroup, same value in every thread.  red: kWaves floats of LDS.
__device__ __forceinline__ float block_sum(float x, float* red) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off);
  __syncthreads();  // red may still be read from a previous call
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = x;
  __syncthreads();
  float total = 0.f;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) total += red[w];
  return total;
}

template <bool IN_LDS>
__global__ __launch_bounds__(kThreads) void asi_terms_kernel(ScoreWorkspace ws, int hist_len,
                                                             int len, int top_k,
                                                             float* __restrict__ terms, int n_samp,
                                                             int row0) {
  __shared__ uint32_t keys[IN_LDS ? kLdsKeys : 1];
  __shared__ __attribute__((aligned(16))) uint32_t hist[kRadixHistWords];
  __shared__ float red[kWaves];
  __shared__ float shift_s;

  const int row = SCALEKV_WG_X, unit = SCALEKV_WG_Y;
  const int tid = threadIdx.x;
  const float* lg = ws.logits + (long long)unit * ws.len_pad * kMaxWindow + row;
  auto logit = [&](int i) -> float { return lg[(long long)i * kMaxWindow]; };
  if (tid == 0) shift_s = score_row_shift(ws, unit, row);  // max + log Z over all `len` keys
  __syncthreads();
  const float shift = shift_s;

  // attention mass on the current map: keys [hist_len, len)
  float part = 0.f;
  for (int i = hist_len + tid; i < len; i += kThreads) part += expf(logit(i) - shift);
  const float cur = block_sum(part, red);

  // sum of the K' largest history weights
  const int kk = min(top_k, hist_len);
  float top = 0.f;
  if (kk > 0) {
    if constexpr (IN_LDS) {
      for (int i = tid; i < hist_len; i += kThreads) keys[i] = order_key(logit(i));
      __syncthreads();
    }
    auto key_at = [&](int i) -> uint32_t {
      if constexpr (IN_LDS) return keys[i];
      else return order_key(logit(i));
    };
    uint32_t T = 0, need_eq = 0;
    if (kk < hist_len) radix_kth_largest<kThreads>(key_at, hist_len, (uint32_t)kk, hist, T, need_eq);
    part = 0.f;
    for (int i = tid; i < hist_len; i += kThreads) {
      const uint32_t key = key_at(i);
      if (kk == hist_len || key > T) part += expf(order_key_value(key) - shift);
    }
    top = block_sum(part, red);
    if (kk < hist_len) top += (float)need_eq * expf(order_key_value(T) - shift);
  }
  if (tid == 0) {
    float* out = terms + ((long long)unit * n_samp + row0 + row) * 2;
    out[0] = cur;
    out[1] = top;
  }
}

__global__ __launch_bounds__(kThreads) void asi_mean_kernel(const float* __restrict__ terms,
                                                            long long n, float* __restrict__ out) {
  __shared__ float red[kWaves];
  float a = 0.f, b = 0.f;
  for (long long i = threadIdx.x; i < n; i += kThreads) {
    a += terms[2 * i];
    b += terms[2 * i + 1];
  }
  const float sa = block_sum(a, red), sb = block_sum(b, red);
  if (threadIdx.x == 0) {
    const float ma = sa / (float)n, mb = sb / (float)n;
    out[0] = ma;
    out[1] = mb;
    out[2] = ma * mb;
  }
}

}  // namespace

hipError_t launch_asi_terms(int n_unit, ScoreWorkspace ws, int n_rows, int hist_len, int len,
                            int top_k, float* terms, int n_samp, int row0, hipStream_t stream) {
  if (n_unit <= 0 || n_rows <= 0 || len <= 0) return hipSuccess;
  dim3 grid(n_rows, n_unit);
  if (hist_len <= kLdsKeys)
    hipLaunchKernelGGL((asi_terms_kernel<true>), grid, dim3(kThreads), 0, stream, ws, hist_len, len,
                       top_k, terms, n_samp, row0);
  else
    hipLaunchKernelGGL((asi_terms_kernel<false>), grid, dim3(kThreads), 0, stream, ws, hist_len, len,
                       top_k, terms, n_samp, row0);
  return hipGetLastError();
}

hipError_t launch_asi_mean(const float* terms, long long n, float* out, hipStream_t stream) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(asi_mean_kernel, dim3(1), dim3(kThreads), 0, stream, terms, n, out);
  return hipGetLastError();
}

}  // namespace scalekv
