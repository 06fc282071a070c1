// Pruning step of Sec. 3.3: gather the selected K/V rows of every (sequence,
// head) unit into the front of the destination cache and append the current
// map's rows behind them.  Pure HBM streaming: every lane moves 16-byte vectors,
// a row (head_dim elements, 128..512 bytes) is covered by consecutive lanes, and
// each thread keeps several independent loads in flight before storing.
#include "common.h"

namespace scalekv {
namespace {

constexpr int kThreads = 256;
constexpr int kUnroll = 4;  // 16-byte vectors in flight per thread per tensor pass

// 16-byte vector in the compiler's native form, so that the streaming (non-temporal)
// load and store builtins accept it.  Every byte is read once and written once per
// call, so neither side should displace cache lines that other kernels still want.
typedef unsigned int vec4 __attribute__((ext_vector_type(4)));

// One workgroup copies a contiguous range of destination vectors of one unit,
// for K (blockIdx.z == 0) or V (blockIdx.z == 1).
//   vec_per_row = head_dim * elem_bytes / 16.
struct Side {
  const vec4* src;  // cache base, strides below in 16-byte vectors
  const vec4* cur;  // dense [U, n_cur, row]
  vec4* dst;
  long long src_seq_stride, src_head_stride, dst_seq_stride, dst_head_stride;
};

__global__ __launch_bounds__(kThreads) void compact_kernel(Side k_side, Side v_side,
                                                           const int32_t* __restrict__ idx,
                                                           int keep, int n_cur, int n_head,
                                                           int vec_per_row_log2) {
  const int unit = SCALEKV_WG_Y;
  const int seq = unit / n_head, head = unit - seq * n_head;
  const Side side = SCALEKV_WG_Z != 0 ? v_side : k_side;
  const vec4* __restrict__ src = side.src + seq * side.src_seq_stride + head * side.src_head_stride;
  const vec4* __restrict__ cur = side.cur;
  vec4* __restrict__ dst = side.dst + seq * side.dst_seq_stride + head * side.dst_head_stride;
  const int vpr_mask = (1 << vec_per_row_log2) - 1;
  const long long cur_base = (long long)unit * n_cur << vec_per_row_log2;
  const int32_t* uidx = idx ? idx + (long long)unit * keep : nullptr;
  const int total = (keep + n_cur) << vec_per_row_log2;

  int f0 = (SCALEKV_WG_X * kThreads * kUnroll) + threadIdx.x;
  vec4 val[kUnroll];
  bool ok[kUnroll];
#pragma unroll
  for (int u = 0; u < kUnroll; ++u) {
    const int f = f0 + u * kThreads;
    ok[u] = f < total;
    if (ok[u]) {
      const int row = f >> vec_per_row_log2, c = f & vpr_mask;
      if (row < keep) {
        const int srow = uidx ? uidx[row] : row;
        val[u] = __builtin_nontemporal_load(src + ((long long)srow << vec_per_row_log2) + c);
      } else {
        val[u] = __builtin_nontemporal_load(cur + cur_base + ((long long)(row - keep) << vec_per_row_log2) + c);
      }
    }
  }
#pragma unroll
  for (int u = 0; u < kUnroll; ++u) {
    const int f = f0 + u * kThreads;
    if (ok[u]) __builtin_nontemporal_store(val[u], dst + f);
  }
}

}  // namespace

hipError_t launch_compact(int dtype, int n_seq, int n_head, int d, KvView k_src, KvView v_src,
                          const int32_t* idx, int keep, const void* k_cur, const void* v_cur,
                          int n_cur, KvView k_dst, KvView v_dst, hipStream_t stream) {
  const int elem = dtype == 0 ? 4 : 2;
  const int vpr = d * elem / 16;  // 8, 16 or 32
  int vlog = 0;
  while ((1 << vlog) < vpr) ++vlog;
  const int total = (keep + n_cur) * vpr;
  if (total <= 0 || n_seq * n_head <= 0) return hipSuccess;
  const int per_block = kThreads * kUnroll;
  dim3 grid((total + per_block - 1) / per_block, n_seq * n_head, 2);
  const int epv = 16 / elem;  // elements per vector: strides arrive in elements
  Side ks{(const vec4*)k_src.ptr, (const vec4*)k_cur, (vec4*)k_dst.ptr, k_src.seq_stride / epv,
          k_src.head_stride / epv, k_dst.seq_stride / epv, k_dst.head_stride / epv};
  Side vs{(const vec4*)v_src.ptr, (const vec4*)v_cur, (vec4*)v_dst.ptr, v_src.seq_stride / epv,
          v_src.head_stride / epv, v_dst.seq_stride / epv, v_dst.head_stride / epv};
  hipLaunchKernelGGL(compact_kernel, grid, dim3(kThreads), 0, stream, ks, vs, idx, keep, n_cur,
                     n_head, vlog);
  return hipGetLastError();
}

}  // namespace scalekv
