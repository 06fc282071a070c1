// Importance score of Eq. 5: for every cached key i of a unit,
//   s_i = sum over window rows j of softmax_i(q_j . k_i * sm_scale),
// reported as log s_i.
//
// Two kernels.  `logits` streams the cached keys once (the HBM-bound part),
// writes the fp32 logits of the <=16 window rows (key-major, 64 B per key) and, per
// 256-key chunk, each
// row's running max and sum of exp.  `finalize` merges the chunk statistics
// into the row normalisers and folds the rows with a log-sum-exp, so no
// probability is ever rounded below fp32 and nothing underflows.
#include "common.h"
#include "score_mfma.h"

namespace scalekv {
namespace {

constexpr int kThreads = kScoreChunk;  // one key per thread

// Generic logits kernel (fp32 or bf16 storage, plain FMA).  Window queries sit
// in LDS as fp32 and are broadcast to every thread; each thread walks its own
// key row in 16-byte vectors.
template <typename T, int D>
__global__ __launch_bounds__(kThreads) void score_logits_kernel(
    const T* __restrict__ q, long long q_unit_stride, WindowRows rows, int n_win,
    const T* __restrict__ k, long long k_seq_stride, long long k_head_stride, int n_head,
    int cache_len, float sm_scale, ScoreWorkspace ws) {
  constexpr int EPV = Elem<T>::kPerVec;
  __shared__ float qs[kMaxWindow][D];
  __shared__ float red_max[kThreads / 64][kMaxWindow];
  __shared__ float red_sum[kThreads / 64][kMaxWindow];

  const int unit = SCALEKV_WG_Y;
  const int seq = unit / n_head, head = unit - seq * n_head;
  const int tid = threadIdx.x;
  const T* qu = q + unit * q_unit_stride;
  for (int e = tid; e < kMaxWindow * D; e += kThreads) {
    const int j = e / D, c = e - j * D;
    float val = 0.f;
    if (j < n_win) {
      if constexpr (sizeof(T) == 4) val = ((const float*)qu)[(long long)rows.row[j] * D + c];
      else val = bf16_bits_to_float(((const uint16_t*)qu)[(long long)rows.row[j] * D + c]);
    }
    qs[j][c] = val;
  }
  __syncthreads();

  const int key = SCALEKV_WG_X * kThreads + tid;
  const bool valid = key < cache_len;
  const int krow = valid ? key : cache_len - 1;  // clamp: load something legal, ignore it later
  const uint4* kv = (const uint4*)(k + seq * k_seq_stride + head * k_head_stride +
                                   (long long)krow * D);
  float acc[kMaxWindow];
#pragma unroll
  for (int j = 0; j < kMaxWindow; ++j) acc[j] = 0.f;
#pragma unroll 4
  for (int c0 = 0; c0 < D / EPV; ++c0) {
    float kf[EPV];
    Elem<T>::unpack(kv[c0], kf);
#pragma unroll
    for (int e = 0; e < EPV; ++e) {
#pragma unroll
      for (int j = 0; j < kMaxWindow; ++j) acc[j] = fmaf(qs[j][c0 * EPV + e], kf[e], acc[j]);
    }
  }

  float* lg = ws.logits + ((long long)unit * ws.len_pad + key) * kMaxWindow;
  const int lane = tid & 63, wave = tid >> 6;
  if (valid) {
#pragma unroll
    for (int j4 = 0; j4 < kMaxWindow; j4 += 4)
      *(float4*)(lg + j4) = make_float4(acc[j4] * sm_scale, acc[j4 + 1] * sm_scale,
                                        acc[j4 + 2] * sm_scale, acc[j4 + 3] * sm_scale);
  }
#pragma unroll
  for (int j = 0; j < kMaxWindow; ++j) {
    const float x = valid ? acc[j] * sm_scale : -INFINITY;
    float m = x;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
    float e = valid ? expf(x - m) : 0.f;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) e += __shfl_xor(e, off);
    if (lane == 0) { red_max[wave][j] = m; red_sum[wave][j] = e; }
  }
  __syncthreads();
  if (tid < kMaxWindow) {
    float m = -INFINITY;
    for (int w = 0; w < kThreads / 64; ++w) m = fmaxf(m, red_max[w][tid]);
    float ssum = 0.f;
    for (int w = 0; w < kThreads / 64; ++w)
      if (red_max[w][tid] > -INFINITY) ssum += red_sum[w][tid] * expf(red_max[w][tid] - m);
    float* part = ws.partial + ((long long)unit * ws.n_chunk + SCALEKV_WG_X) * 2 * kMaxWindow;
    part[tid] = m;
    part[kMaxWindow + tid] = ssum;
  }
}

// bf16 logits kernel: the HBM-bound part of the score.  Each wave handles 64 keys of the
// workgroup's 256-key chunk (see score_mfma.h) and the workgroup leaves the chunk's row maximum
// and sum of exponentials for the finalisation.
template <int D>
__global__ __launch_bounds__(kThreads) void score_logits_mfma_kernel(
    const uint16_t* __restrict__ q, long long q_unit_stride, WindowRows rows, int n_win,
    const uint16_t* __restrict__ k, long long k_seq_stride, long long k_head_stride, int n_head,
    int cache_len, float sm_scale, ScoreWorkspace ws) {
  constexpr int NT = 4;  // 16-key tiles per wave
  __shared__ float red_max[kThreads / 64][kMaxWindow];
  __shared__ float red_sum[kThreads / 64][kMaxWindow];
  const int unit = SCALEKV_WG_Y;
  const int seq = unit / n_head, head = unit - seq * n_head;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const uint16_t* ku = k + seq * k_seq_stride + head * k_head_stride;
  score_bf16x8 qf[D / 32];
  score_load_window<D>(q + unit * q_unit_stride, rows, n_win, qf);
  float m, e;
  score_wave_logits<D, NT>(ku, qf, SCALEKV_WG_X * kScoreChunk + wave * (16 * NT), cache_len, sm_scale,
                           ws.logits + (long long)unit * ws.len_pad * kMaxWindow, m, e);
  if (lane < kMaxWindow) { red_max[wave][lane] = m; red_sum[wave][lane] = e; }
  __syncthreads();
  if (tid < kMaxWindow) {
    float mm = -INFINITY;
    for (int w = 0; w < kThreads / 64; ++w) mm = fmaxf(mm, red_max[w][tid]);
    float ssum = 0.f;
    for (int w = 0; w < kThreads / 64; ++w)
      if (red_max[w][tid] > -INFINITY) ssum += red_sum[w][tid] * expf(red_max[w][tid] - mm);
    float* part = ws.partial + ((long long)unit * ws.n_chunk + SCALEKV_WG_X) * 2 * kMaxWindow;
    part[tid] = mm;
    part[kMaxWindow + tid] = ssum;
  }
}

// log s_i = logsumexp_j( logit[j][i] - max_j - log Z_j ).
__global__ __launch_bounds__(256) void score_finalize_kernel(int n_win, int cache_len,
                                                             ScoreWorkspace ws,
                                                             float* __restrict__ log_scores,
                                                             long long score_unit_stride) {
  __shared__ float row_shift[kMaxWindow];  // max_j + log Z_j
  const int unit = SCALEKV_WG_Y;
  const int tid = threadIdx.x;
  if (tid < kMaxWindow) row_shift[tid] = tid < n_win ? score_row_shift(ws, unit, tid) : 0.f;
  __syncthreads();
  const int key = SCALEKV_WG_X * 256 + tid;
  if (key >= cache_len) return;
  log_scores[unit * score_unit_stride + key] = score_log_sum(ws, unit, key, n_win, row_shift);
}

template <typename T>
hipError_t launch_logits_t(int n_seq, int n_head, int d, const void* q, long long q_unit_stride,
                           WindowRows rows, int n_win, KvView k, int cache_len, float sm_scale,
                           ScoreWorkspace ws, hipStream_t stream) {
  dim3 grid(ws.n_chunk, n_seq * n_head);
  if (d == 128)
    hipLaunchKernelGGL((score_logits_kernel<T, 128>), grid, dim3(kThreads), 0, stream,
                       (const T*)q, q_unit_stride, rows, n_win, (const T*)k.ptr, k.seq_stride,
                       k.head_stride, n_head, cache_len, sm_scale, ws);
  else
    hipLaunchKernelGGL((score_logits_kernel<T, 64>), grid, dim3(kThreads), 0, stream, (const T*)q,
                       q_unit_stride, rows, n_win, (const T*)k.ptr, k.seq_stride, k.head_stride,
                       n_head, cache_len, sm_scale, ws);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_score_logits(int dtype, int n_seq, int n_head, int d, const void* q,
                               long long q_unit_stride, WindowRows rows, int n_win, KvView k,
                               int cache_len, float sm_scale, ScoreWorkspace ws,
                               hipStream_t stream) {
  if (cache_len <= 0 || n_seq * n_head <= 0) return hipSuccess;
  if (dtype == 0)
    return launch_logits_t<float>(n_seq, n_head, d, q, q_unit_stride, rows, n_win, k, cache_len,
                                  sm_scale, ws, stream);
  dim3 grid(ws.n_chunk, n_seq * n_head);
  if (d == 128)
    hipLaunchKernelGGL((score_logits_mfma_kernel<128>), grid, dim3(kThreads), 0, stream,
                       (const uint16_t*)q, q_unit_stride, rows, n_win, (const uint16_t*)k.ptr,
                       k.seq_stride, k.head_stride, n_head, cache_len, sm_scale, ws);
  else
    hipLaunchKernelGGL((score_logits_mfma_kernel<64>), grid, dim3(kThreads), 0, stream,
                       (const uint16_t*)q, q_unit_stride, rows, n_win, (const uint16_t*)k.ptr,
                       k.seq_stride, k.head_stride, n_head, cache_len, sm_scale, ws);
  return hipGetLastError();
}

hipError_t launch_score_finalize(int n_unit, int n_win, int cache_len, ScoreWorkspace ws,
                                 float* log_scores, long long score_unit_stride,
                                 hipStream_t stream) {
  if (cache_len <= 0 || n_unit <= 0) return hipSuccess;
  dim3 grid((cache_len + 255) / 256, n_unit);
  hipLaunchKernelGGL(score_finalize_kernel, grid, dim3(256), 0, stream, n_win, cache_len, ws,
                     log_scores, score_unit_stride);
  return hipGetLastError();
}

}  // namespace scalekv
