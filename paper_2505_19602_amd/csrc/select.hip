// Top-k of Sec. 3.3 for one (sequence, head) unit per workgroup.
//
// Scores are mapped to order-preserving unsigned keys; a 4-pass, 8-bit radix
// select finds the key T of the keep-th largest score; one stable pass then
// emits, in ascending index order, every index with key > T and the first
// (keep - #greater) indices with key == T.  Only integer compares are involved,
// so the result is deterministic and ties always go to the lower index.
//
// Two optional parts of the paper's selection are folded into the key set-up:
// average pooling of the scores along the cache axis (odd width, zeros beyond the
// ends; done on log-scores as a log-sum-exp, which ranks the same), and positions
// that are preserved whatever their score (the observation window): those get the
// largest key, and `keep` counts them.
#include "common.h"
#include "radix_select.h"
#include "score_mfma.h"

namespace scalekv {
namespace {

constexpr int kThreads = 1024;
constexpr int kWaves = kThreads / 64;
constexpr int kLdsKeys = 12288;  // units up to this many scores keep their keys in LDS
static_assert(kLdsKeys == 12288, "score_select_fits() in common.h states the same limit");

// FUSED: the scores are not read but formed here from the logits workspace (the score
// finalisation), so the fused step neither writes nor re-reads them.
// log of the average of exp(v[i + t]), |t| <= r, positions outside [0, len) counting as zero
template <typename Load>
__device__ __forceinline__ float pooled_log(Load v, int i, int len, int r) {
  const int a = max(i - r, 0), b = min(i + r, len - 1);
  float m = -INFINITY;
  for (int t = a; t <= b; ++t) m = fmaxf(m, v(t));
  if (!(m > -INFINITY)) return -INFINITY;
  float acc = 0.f;
  for (int t = a; t <= b; ++t) acc += expf(v(t) - m);
  return m + logf(acc) - logf((float)(2 * r + 1));
}

// What the kernel needs to form the logits itself (SCORE_D != 0): bf16 storage only.
struct ScoreInputs {
  const uint16_t* q;        // [U, *, D]; window queries are rows `rows` of every unit
  long long q_unit_stride;
  WindowRows rows;
  const uint16_t* k;        // cache
  long long k_seq_stride, k_head_stride;
  int n_head;
  float sm_scale;
  // Pruning by the same workgroup (Sec. 3.3: the selected rows are preserved): after the
  // selection, row idx[t] of the source caches is copied to row t of the destination caches, and
  // n_app rows of k_cur / v_cur ([U, n_app, D]) are appended behind the kept ones.  Off if
  // k_dst == NULL.  v_src may differ from the key cache in base and strides; strides in elements.
  const uint16_t* v_src;
  long long v_seq_stride, v_head_stride;
  uint16_t* k_dst;
  uint16_t* v_dst;
  long long kd_seq_stride, kd_head_stride, vd_seq_stride, vd_head_stride;
  const uint16_t* k_cur;
  const uint16_t* v_cur;
  int n_app;
};

// SCORE_D = 64 / 128: the whole ranking step of Sec. 3.3 in one kernel.  The workgroup first
// streams the unit's cached keys itself (16 waves x 32 keys per round, logits to the workspace,
// running row maximum and sum of exponentials per wave), so that neither a second launch nor the
// per-chunk statistics are needed; then it ranks as in the FUSED form.
// MIN_WAVES = 8 holds the kernel to 64 registers so that two workgroups share a compute unit (one
// streams keys while the other ranks): for launches with more units than compute units.  With
// one workgroup per compute unit the unconstrained form (MIN_WAVES = 4) is a little faster.
template <bool IN_LDS, bool FUSED, int SCORE_D, int MIN_WAVES = 4>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(MIN_WAVES, 8))) void select_kernel(const float* __restrict__ scores,
                                                          long long score_unit_stride,
                                                          int cache_len, int keep,
                                                          int32_t* __restrict__ idx,
                                                          ScoreWorkspace ws, int n_win,
                                                          SelectExtras ex, ScoreInputs si) {
  static_assert(IN_LDS || !FUSED, "the fused form keeps its keys in LDS");
  static_assert(FUSED || SCORE_D == 0, "forming the logits here implies the fused form");
  constexpr int kPerThread = IN_LDS ? kLdsKeys / kThreads : 1;
  __shared__ uint32_t keys[IN_LDS ? kLdsKeys : 1];
  __shared__ float row_shift[kMaxWindow];
  __shared__ __attribute__((aligned(16))) uint32_t hist[kRadixHistWords];
  __shared__ uint32_t wave_gt[kWaves], wave_eq[kWaves];
  __shared__ float red_max[SCORE_D ? kWaves : 1][kMaxWindow], red_sum[SCORE_D ? kWaves : 1][kMaxWindow];

  const int unit = SCALEKV_WG_X;
  const int tid = threadIdx.x;
  const float* s = scores + unit * score_unit_stride;
  const int pool_r = (ex.pool_w - 1) / 2;
  auto key_at = [&](int i) -> uint32_t {
    if constexpr (IN_LDS) {
      return keys[i];
    } else {
      for (int j = 0; j < ex.n_forced; ++j)
        if (ex.forced[j] == i) return 0xffffffffu;
      if (pool_r > 0) return order_key(pooled_log([&](int t) { return s[t]; }, i, cache_len, pool_r));
      return order_key(s[i]);
    }
  };
  if constexpr (IN_LDS) {
    // log-scores into LDS (formed from the logits workspace when FUSED), pooled in place if
    // asked for, then turned into keys
    if constexpr (SCORE_D != 0) {
      // Eq. 5, logits and row normalisers: every wave walks its share of the keys, 32 per round
      constexpr int NT = 2;
      const int lane = tid & 63, wave = tid >> 6;
      const int seq = unit / si.n_head, head = unit - seq * si.n_head;
      const uint16_t* ku = si.k + seq * si.k_seq_stride + head * si.k_head_stride;
      float* logits_unit = ws.logits + (long long)unit * ws.len_pad * kMaxWindow;
      score_bf16x8 qf[SCORE_D / 32];
      score_load_window<SCORE_D>(si.q + unit * si.q_unit_stride, si.rows, n_win, qf);
      float m_run = -INFINITY, e_run = 0.f;
      for (int key0 = wave * (16 * NT); key0 < cache_len; key0 += kWaves * 16 * NT) {
        float m, e;
        score_wave_logits<SCORE_D, NT>(ku, qf, key0, cache_len, si.sm_scale, logits_unit, m, e);
        const float m_new = fmaxf(m_run, m);   // m is finite: the round has at least one valid key
        e_run = e_run * expf(m_run - m_new) + e * expf(m - m_new);
        m_run = m_new;
      }
      if (lane < kMaxWindow) { red_max[wave][lane] = m_run; red_sum[wave][lane] = e_run; }
      __syncthreads();   // also makes the logits visible to the whole workgroup
      if (tid < kMaxWindow) {
        float mm = -INFINITY;
        for (int w = 0; w < kWaves; ++w) mm = fmaxf(mm, red_max[w][tid]);
        float z = 0.f;
        for (int w = 0; w < kWaves; ++w)
          if (red_max[w][tid] > -INFINITY) z += red_sum[w][tid] * expf(red_max[w][tid] - mm);
        row_shift[tid] = tid < n_win ? mm + logf(z) : 0.f;
      }
      __syncthreads();
    } else if constexpr (FUSED) {
      if (tid < kMaxWindow) row_shift[tid] = tid < n_win ? score_row_shift(ws, unit, tid) : 0.f;
      __syncthreads();
    }
    float* raw = reinterpret_cast<float*>(keys);
    for (int i = tid; i < cache_len; i += kThreads) {
      if constexpr (FUSED) raw[i] = score_log_sum(ws, unit, i, n_win, row_shift);
      else raw[i] = s[i];
    }
    __syncthreads();
    float mine[kPerThread];
#pragma unroll
    for (int c = 0; c < kPerThread; ++c) {
      const int i = tid + c * kThreads;
      if (i < cache_len)
        mine[c] = pool_r > 0 ? pooled_log([&](int t) { return raw[t]; }, i, cache_len, pool_r) : raw[i];
    }
    __syncthreads();
#pragma unroll
    for (int c = 0; c < kPerThread; ++c) {
      const int i = tid + c * kThreads;
      if (i < cache_len) keys[i] = order_key(mine[c]);
    }
    if (ex.n_forced > 0) {
      __syncthreads();
      if (tid < ex.n_forced) keys[ex.forced[tid]] = 0xffffffffu;
    }
  }

  // ---- radix select: T = key of the keep-th largest ----
  uint32_t T, need_eq;  // need_eq: how many keys equal to T are taken (>= 1)
  radix_kth_largest<kThreads>(key_at, cache_len, (uint32_t)keep, hist, T, need_eq);

  // ---- stable emission ----
  const int per = (cache_len + kThreads - 1) / kThreads;
  const int lo = min(tid * per, cache_len), hi = min(lo + per, cache_len);
  uint32_t n_gt = 0, n_eq = 0;
  for (int i = lo; i < hi; ++i) {
    const uint32_t kk = key_at(i);
    n_gt += kk > T;
    n_eq += kk == T;
  }
  // exclusive block scan of (n_gt, n_eq)
  const int lane = tid & 63, wave = tid >> 6;
  const uint32_t sg = wave_prefix_sum(n_gt, lane), se = wave_prefix_sum(n_eq, lane);
  if (lane == 63) { wave_gt[wave] = sg; wave_eq[wave] = se; }
  __syncthreads();
  uint32_t base_g = 0, base_e = 0;
  for (int w = 0; w < wave; ++w) { base_g += wave_gt[w]; base_e += wave_eq[w]; }
  const uint32_t ex_g = base_g + sg - n_gt, ex_e = base_e + se - n_eq;
  uint32_t pos = ex_g + min(ex_e, need_eq);
  uint32_t eq_seen = ex_e;
  int32_t* out = idx + (long long)unit * keep;
  for (int i = lo; i < hi; ++i) {
    const uint32_t kk = key_at(i);
    if (kk > T) {
      out[pos++] = i;
    } else if (kk == T) {
      if (eq_seen < need_eq) out[pos++] = i;
      ++eq_seen;
    }
  }

  // ---- pruning: the kept rows (and, if asked, the map's rows behind them) into the destination
  if constexpr (SCORE_D != 0) {
    if (si.k_dst != nullptr) {
      typedef unsigned int vec4 __attribute__((ext_vector_type(4)));
      constexpr int VPR = SCORE_D * 2 / 16;  // 16-byte vectors per row
      constexpr int kFly = 4;                // vectors in flight per thread and tensor
      __syncthreads();  // the unit's index list is complete (written by this workgroup)
      const int seq = unit / si.n_head, head = unit - seq * si.n_head;
      const vec4* ksrc = (const vec4*)(si.k + seq * si.k_seq_stride + head * si.k_head_stride);
      const vec4* vsrc = (const vec4*)(si.v_src + seq * si.v_seq_stride + head * si.v_head_stride);
      vec4* kdst = (vec4*)(si.k_dst + seq * si.kd_seq_stride + head * si.kd_head_stride);
      vec4* vdst = (vec4*)(si.v_dst + seq * si.vd_seq_stride + head * si.vd_head_stride);
      const vec4* kcur = (const vec4*)(si.k_cur + (long long)unit * si.n_app * SCORE_D);
      const vec4* vcur = (const vec4*)(si.v_cur + (long long)unit * si.n_app * SCORE_D);
      const int total = (keep + si.n_app) * VPR;
      for (int f0 = tid; f0 < total; f0 += kThreads * kFly) {
        vec4 a[kFly], b[kFly];
#pragma unroll
        for (int u = 0; u < kFly; ++u) {
          const int f = f0 + u * kThreads;
          if (f < total) {
            const int row = f / VPR, c = f % VPR;
            if (row < keep) {
              const long long o = (long long)out[row] * VPR + c;
              a[u] = __builtin_nontemporal_load(ksrc + o);
              b[u] = __builtin_nontemporal_load(vsrc + o);
            } else {
              const long long o = (long long)(row - keep) * VPR + c;
              a[u] = __builtin_nontemporal_load(kcur + o);
              b[u] = __builtin_nontemporal_load(vcur + o);
            }
          }
        }
#pragma unroll
        for (int u = 0; u < kFly; ++u) {
          const int f = f0 + u * kThreads;
          if (f < total) {
            __builtin_nontemporal_store(a[u], kdst + f);
            __builtin_nontemporal_store(b[u], vdst + f);
          }
        }
      }
    }
  }
}

__global__ void iota_kernel(int32_t* __restrict__ idx, int keep, long long total) {
  const long long e = (long long)SCALEKV_WG_X * blockDim.x + threadIdx.x;
  if (e < total) idx[e] = (int32_t)(e % keep);
}

// Position-only retention (the sliding-window and sinks-plus-recent policies the paper
// compares against in Sec. 4.1): every unit keeps the first n_sink and the last
// keep - n_sink positions of its cache_len rows.
__global__ void positional_kernel(int32_t* __restrict__ idx, int keep, int n_sink, int cache_len,
                                  long long total) {
  const long long e = (long long)SCALEKV_WG_X * blockDim.x + threadIdx.x;
  if (e >= total) return;
  const int t = (int)(e % keep);
  idx[e] = t < n_sink ? t : cache_len - keep + t;
}

}  // namespace

hipError_t launch_positional(int n_unit, int cache_len, int n_sink, int keep, int32_t* idx,
                             hipStream_t stream) {
  if (n_unit <= 0 || keep <= 0) return hipSuccess;
  const long long total = (long long)n_unit * keep;
  hipLaunchKernelGGL(positional_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0,
                     stream, idx, keep, n_sink, cache_len, total);
  return hipGetLastError();
}

hipError_t launch_select(int n_unit, const float* scores, long long score_unit_stride,
                         int cache_len, int keep, int32_t* idx, const SelectExtras* extras,
                         hipStream_t stream) {
  SelectExtras ex{};
  ex.pool_w = 1;
  if (extras) ex = *extras;
  if (n_unit <= 0 || keep <= 0 || cache_len <= 0) return hipSuccess;
  if (keep >= cache_len) {  // keep everything: identity, no ranking needed
    const long long total = (long long)n_unit * keep;
    hipLaunchKernelGGL(iota_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream,
                       idx, keep, total);
    return hipGetLastError();
  }
  const ScoreWorkspace none{nullptr, nullptr, 0, 0};
  const ScoreInputs no_score{};
  if (cache_len <= kLdsKeys)
    hipLaunchKernelGGL((select_kernel<true, false, 0>), dim3(n_unit), dim3(kThreads), 0, stream,
                       scores, score_unit_stride, cache_len, keep, idx, none, 0, ex, no_score);
  else
    hipLaunchKernelGGL((select_kernel<false, false, 0>), dim3(n_unit), dim3(kThreads), 0, stream,
                       scores, score_unit_stride, cache_len, keep, idx, none, 0, ex, no_score);
  return hipGetLastError();
}

hipError_t launch_select_from_logits(int n_unit, int n_win, ScoreWorkspace ws, int cache_len,
                                     int keep, int32_t* idx, const SelectExtras* extras,
                                     hipStream_t stream) {
  SelectExtras ex{};
  ex.pool_w = 1;
  if (extras) ex = *extras;
  if (cache_len > kLdsKeys) return hipErrorNotSupported;
  if (n_unit <= 0 || keep <= 0 || cache_len <= 0) return hipSuccess;
  hipLaunchKernelGGL((select_kernel<true, true, 0>), dim3(n_unit), dim3(kThreads), 0, stream, nullptr,
                     0, cache_len, keep, idx, ws, n_win, ex, ScoreInputs{});
  return hipGetLastError();
}

hipError_t launch_score_select(int dtype, int n_seq, int n_head, int d, const void* q, long long q_unit_stride,
                               WindowRows rows, int n_win, KvView k, int cache_len, float sm_scale,
                               ScoreWorkspace ws, int keep, int32_t* idx, const SelectExtras* extras,
                               const PruneTarget* prune, hipStream_t stream) {
  SelectExtras ex{};
  ex.pool_w = 1;
  if (extras) ex = *extras;
  const int n_unit = n_seq * n_head;
  if (!score_select_fits(dtype, d, n_unit, cache_len)) return hipErrorNotSupported;
  if (n_unit <= 0 || keep <= 0 || cache_len <= 0) return hipSuccess;
  ScoreInputs si{};
  si.q = (const uint16_t*)q; si.q_unit_stride = q_unit_stride; si.rows = rows;
  si.k = (const uint16_t*)k.ptr; si.k_seq_stride = k.seq_stride; si.k_head_stride = k.head_stride;
  si.n_head = n_head; si.sm_scale = sm_scale;
  if (prune) {
    si.v_src = (const uint16_t*)prune->v_src.ptr;
    si.v_seq_stride = prune->v_src.seq_stride; si.v_head_stride = prune->v_src.head_stride;
    si.k_dst = (uint16_t*)const_cast<void*>(prune->k_dst.ptr); si.v_dst = (uint16_t*)const_cast<void*>(prune->v_dst.ptr);
    si.kd_seq_stride = prune->k_dst.seq_stride; si.kd_head_stride = prune->k_dst.head_stride;
    si.vd_seq_stride = prune->v_dst.seq_stride; si.vd_head_stride = prune->v_dst.head_stride;
    si.k_cur = (const uint16_t*)prune->k_cur; si.v_cur = (const uint16_t*)prune->v_cur;
    si.n_app = prune->k_cur ? prune->n_app : 0;
  }
  constexpr int kComputeUnits = 256;  // MI355X
  if (d == 128 && n_unit > kComputeUnits)
    hipLaunchKernelGGL((select_kernel<true, true, 128, 8>), dim3(n_unit), dim3(kThreads), 0, stream, nullptr,
                       0, cache_len, keep, idx, ws, n_win, ex, si);
  else if (d == 128)
    hipLaunchKernelGGL((select_kernel<true, true, 128>), dim3(n_unit), dim3(kThreads), 0, stream, nullptr,
                       0, cache_len, keep, idx, ws, n_win, ex, si);
  else
    hipLaunchKernelGGL((select_kernel<true, true, 64>), dim3(n_unit), dim3(kThreads), 0, stream, nullptr,
                       0, cache_len, keep, idx, ws, n_win, ex, si);
  return hipGetLastError();
}

}  // namespace scalekv
