// Internal declarations shared by the ScaleKV HIP translation units (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

namespace scalekv {

constexpr int kMaxWindow = 16;     // window rows held per unit by the score kernels
constexpr int kScoreChunk = 256;   // cached keys handled per workgroup in the score kernels
constexpr int kLogitPad = 64;      // logits row stride is the cache length rounded up to this

// A cache viewed by kernels: base pointer plus strides in elements.
struct KvView {
  const void* ptr;
  long long seq_stride;
  long long head_stride;
};

struct WindowRows {
  int row[kMaxWindow];
};

struct ScoreWorkspace {
  float* logits;    // [U][len_pad][kMaxWindow]  (key-major: the 16 window logits of a key are 64 B)
  float* partial;   // [U][n_chunk][2][kMaxWindow]  (row max, row sum of exp(logit - max))
  int len_pad;
  int n_chunk;
};

// Optional parts of the selection (Sec. 3.3): positions preserved whatever their score
// (the observation window) and average pooling of the scores along the cache axis.
struct SelectExtras {
  int n_forced;             // 0..kMaxWindow
  int forced[kMaxWindow];   // distinct positions in [0, cache_len)
  int pool_w;               // odd, 1 = no pooling
};

inline int round_up(int x, int m) { return (x + m - 1) / m * m; }

// Raises a kernel's dynamic-LDS limit, once per device: the attribute belongs to the current
// device's copy of the code, so a second GPU needs its own call.  `done` holds one bit per
// device (devices 64 and up are simply set every time); any number of host threads may race
// here, the call is idempotent.
inline hipError_t allow_dynamic_lds(const void* kernel, int bytes, std::atomic<uint64_t>& done) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const uint64_t bit = dev >= 0 && dev < 64 ? (uint64_t)1 << dev : 0;
  if (bit && (done.load(std::memory_order_acquire) & bit)) return hipSuccess;
  e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess && bit) done.fetch_or(bit, std::memory_order_release);
  return e;
}

// ---- launchers (each enqueues on `stream` and returns hipGetLastError()) ----

hipError_t launch_score_logits(int dtype, int n_seq, int n_head, int d, const void* q,
                               long long q_unit_stride, WindowRows rows, int n_win, KvView k,
                               int cache_len, float sm_scale, ScoreWorkspace ws,
                               hipStream_t stream);
hipError_t launch_score_finalize(int n_unit, int n_win, int cache_len, ScoreWorkspace ws,
                                 float* log_scores, long long score_unit_stride,
                                 hipStream_t stream);
// `keep` counts the forced positions of `extras` (NULL: none, no pooling) as well.
hipError_t launch_select(int n_unit, const float* scores, long long score_unit_stride,
                         int cache_len, int keep, int32_t* idx, const SelectExtras* extras,
                         hipStream_t stream);
// select straight from the logits workspace (score finalisation fused in); returns
// hipErrorNotSupported when the unit is too long for the fused kernel
hipError_t launch_select_from_logits(int n_unit, int n_win, ScoreWorkspace ws, int cache_len,
                                     int keep, int32_t* idx, const SelectExtras* extras,
                                     hipStream_t stream);
// The whole ranking step in one launch (bf16 only): one workgroup per unit forms the logits of
// the window rows against the unit's cached keys, the row normalisers and the log-scores
// (Eq. 5) and selects.  Worth it when there are enough units to fill the chip or the caches are
// short; returns hipErrorNotSupported otherwise (and for fp32 or very long caches), and the
// caller takes the two launches.  The logits part of `ws` is used, the chunk statistics are not.
inline bool score_select_fits(int dtype, int d, int n_unit, int cache_len) {
  return dtype == 1 && (d == 64 || d == 128) && cache_len <= 12288 && (n_unit >= 64 || cache_len <= 4096);
}
// With `prune` the same workgroup then also prunes its unit (Sec. 3.3): source row idx[t] of k
// (keys) / prune->v_src (values) goes to row t of the destination caches, and the n_app rows of
// k_cur / v_cur ([U, n_app, d], NULL: none) are appended behind the keep rows.
struct PruneTarget {
  KvView v_src, k_dst, v_dst;
  const void* k_cur;
  const void* v_cur;
  int n_app;
};
hipError_t launch_score_select(int dtype, int n_seq, int n_head, int d, const void* q, long long q_unit_stride,
                               WindowRows rows, int n_win, KvView k, int cache_len, float sm_scale,
                               ScoreWorkspace ws, int keep, int32_t* idx, const SelectExtras* extras,
                               const PruneTarget* prune, hipStream_t stream);
// first n_sink and last keep - n_sink positions of every unit (n_sink <= keep <= cache_len)
hipError_t launch_positional(int n_unit, int cache_len, int n_sink, int keep, int32_t* idx,
                             hipStream_t stream);
// Eq. 2 for the n_rows (<= kMaxWindow) query rows whose logits sit in `ws`: per row the
// attention mass on keys [hist_len, len) and the sum of its top_k largest weights on keys
// [0, hist_len), written to terms[((unit * n_samp) + row0 + row) * 2 + {0, 1}]
hipError_t launch_asi_terms(int n_unit, ScoreWorkspace ws, int n_rows, int hist_len, int len,
                            int top_k, float* terms, int n_samp, int row0, hipStream_t stream);
// out[0], out[1] = means of the two columns of terms [n][2]; out[2] = their product
hipError_t launch_asi_mean(const float* terms, long long n, float* out, hipStream_t stream);
hipError_t launch_compact(int dtype, int n_seq, int n_head, int d, KvView k_src, KvView v_src,
                          const int32_t* idx, int keep, const void* k_cur, const void* v_cur,
                          int n_cur, KvView k_dst, KvView v_dst, hipStream_t stream);
hipError_t launch_attend(int dtype, int n_seq, int n_head, int d, const void* q, int n_q, KvView k,
                         KvView v, int kv_len, float sm_scale, void* out, hipStream_t stream);

// bf16, head_dim 128 only: the pipelined kernel used when n_q is large.  Keys and values are the
// first len1 rows of the caches k, v followed by the len2 rows of the dense tensors k2, v2
// ([U, len2, d]; may be NULL when len2 == 0).  With `append` the kernel also copies k2, v2 into
// rows [len1, len1 + len2) of the caches, which must have room for them.  `start` / `stop`
// (either may be NULL): events that receive the kernel's own start and end times; they ride on
// the kernel's dispatch, so unlike hipEventRecord they put no operation of their own on the stream.
hipError_t launch_attend_pipe(int n_unit, int n_head, const void* q, int n_q, KvView k, KvView v,
                              int len1, const void* k2, const void* v2, int len2, bool append,
                              float sm_scale, void* out, hipStream_t stream,
                              hipEvent_t start = nullptr, hipEvent_t stop = nullptr);
// whether launch_attend would take the pipelined kernel for this shape
inline bool attend_uses_pipe(int dtype, int d, int n_q) { return dtype == 1 && d == 128 && n_q > 128; }

// ---- device helpers ----
// Workgroup coordinates as the kernels read them.  A build with SCALEKV_REVERSE_WG
// (python -m paper_2505_19602_amd.build --variant reversed_order) walks every grid backwards:
// workgroup i does the work that workgroup n-1-i does in the plain build.  No result may depend
// on which workgroup runs first; a test compares the two builds bit for bit.
#if defined(SCALEKV_REVERSE_WG)
#define SCALEKV_WG_X ((int)(gridDim.x - 1 - blockIdx.x))
#define SCALEKV_WG_Y ((int)(gridDim.y - 1 - blockIdx.y))
#define SCALEKV_WG_Z ((int)(gridDim.z - 1 - blockIdx.z))
#else
#define SCALEKV_WG_X ((int)blockIdx.x)
#define SCALEKV_WG_Y ((int)blockIdx.y)
#define SCALEKV_WG_Z ((int)blockIdx.z)
#endif
// Shared by the two MFMA attention kernels: the key row fed to MFMA row i of the first product
// is row pi32(i) of the 32-key block (bits 2 and 3 swapped), which makes the registers of an
// S^T block the B operand of the second product; and the number of log2 units a row maximum may
// grow before the running offset is moved and the accumulators are rescaled.
__device__ __forceinline__ int pi32(int i) { return (i & ~12) | ((i & 4) << 1) | ((i & 8) >> 1); }
constexpr float kRescaleThreshold = 8.f;

__device__ __forceinline__ float bf16_bits_to_float(uint32_t bits16) {
  return __uint_as_float(bits16 << 16);
}

template <typename T>
struct Elem;
template <>
struct Elem<float> {
  static constexpr int kPerVec = 4;  // elements per 16-byte vector
  __device__ static void unpack(const uint4& v, float* f) {
    f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y);
    f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
  }
};
struct bf16_t { uint16_t bits; };
template <>
struct Elem<bf16_t> {
  static constexpr int kPerVec = 8;
  __device__ static void unpack(const uint4& v, float* f) {
    f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xffff0000u);
    f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xffff0000u);
    f[4] = __uint_as_float(v.z << 16); f[5] = __uint_as_float(v.z & 0xffff0000u);
    f[6] = __uint_as_float(v.w << 16); f[7] = __uint_as_float(v.w & 0xffff0000u);
  }
};

// ---- shared between the score finalisation and the fused select ----
// Row normaliser of window row j: max_j + log Z_j from the per-chunk (max, sum exp) pairs.
__device__ __forceinline__ float score_row_shift(const ScoreWorkspace& ws, int unit, int j) {
  const float* part = ws.partial + (long long)unit * ws.n_chunk * 2 * kMaxWindow;
  float m = -INFINITY;
  for (int c = 0; c < ws.n_chunk; ++c) m = fmaxf(m, part[c * 2 * kMaxWindow + j]);
  float z = 0.f;
  for (int c = 0; c < ws.n_chunk; ++c)
    z += part[c * 2 * kMaxWindow + kMaxWindow + j] * expf(part[c * 2 * kMaxWindow + j] - m);
  return m + logf(z);
}
// log s_i = logsumexp_j(logit[i][j] - shift_j) for one key; row_shift lives in LDS.
__device__ __forceinline__ float score_log_sum(const ScoreWorkspace& ws, int unit, int key, int n_win,
                                               const float* row_shift) {
  const float* lg = ws.logits + ((long long)unit * ws.len_pad + key) * kMaxWindow;
  float la[kMaxWindow];
#pragma unroll
  for (int j4 = 0; j4 < kMaxWindow; j4 += 4) {
    const float4 x = *(const float4*)(lg + j4);
    la[j4] = x.x; la[j4 + 1] = x.y; la[j4 + 2] = x.z; la[j4 + 3] = x.w;
  }
  float top = -INFINITY;
#pragma unroll
  for (int j = 0; j < kMaxWindow; ++j) {
    la[j] = j < n_win ? la[j] - row_shift[j] : -INFINITY;
    top = fmaxf(top, la[j]);
  }
  float acc = 0.f;
#pragma unroll
  for (int j = 0; j < kMaxWindow; ++j) acc += j < n_win ? expf(la[j] - top) : 0.f;
  return top + logf(acc);
}

// round-to-nearest-even float -> bf16 bits (NaN kept quiet)
__device__ __forceinline__ uint32_t float_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

}  // namespace scalekv
