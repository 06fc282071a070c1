// Unmasked attention of the current token map over [retained cache ; current
// map] (Sec. 3.1 / 3.3): out[t] = sum_i softmax_i(q_t . k_i * sm_scale) v_i.
//
// Two kernels:
//  * attend_mfma_kernel   bf16, flash-style: K/V tiles staged through LDS, bf16
//    MFMA 32x32x16 for both products, fp32 online softmax.  The products are
//    formed transposed (S^T = K Q^T, O^T = V^T P^T) so that one lane owns one
//    query column: the softmax statistics are per-lane scalars and P^T leaves
//    the first product already in the register layout the second one consumes.
//  * attend_simple_kernel fp32 (and any case the MFMA kernel is not built for):
//    plain FMA, fp32 throughout.
#include "common.h"

namespace scalekv {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

// =====================================================================
// fp32 / generic kernel.  256 threads: 32 query rows x 8 lanes per row.
// =====================================================================
template <typename T, int D>
__global__ __launch_bounds__(256) void attend_simple_kernel(
    const T* __restrict__ q, int n_q, const T* __restrict__ k, long long k_seq_stride,
    long long k_head_stride, const T* __restrict__ v, long long v_seq_stride,
    long long v_head_stride, int kv_len, int n_head, float sm_scale, T* __restrict__ out) {
  constexpr int BQ = 32, BK = 32, G = 8, CPT = D / G;  // CPT output columns per thread
  __shared__ float qs[BQ][D + 1];
  __shared__ float ks[BK][D + 1];
  __shared__ float vs[BK][D];
  __shared__ float ps[BQ][BK + 1];

  const int unit = SCALEKV_WG_Y;
  const int seq = unit / n_head, head = unit - seq * n_head;
  const int tid = threadIdx.x, r = tid / G, g = tid % G;
  const int q0 = SCALEKV_WG_X * BQ;
  const T* qu = q + (long long)unit * n_q * D;
  const T* ku = k + seq * k_seq_stride + head * k_head_stride;
  const T* vu = v + seq * v_seq_stride + head * v_head_stride;

  auto ld = [](const T* p) -> float {
    if constexpr (sizeof(T) == 4) return *(const float*)p;
    else return bf16_bits_to_float(*(const uint16_t*)p);
  };

  for (int e = tid; e < BQ * D; e += 256) {
    const int rr = e / D, c = e - rr * D;
    qs[rr][c] = (q0 + rr < n_q) ? ld(qu + (long long)(q0 + rr) * D + c) : 0.f;
  }
  float acc[CPT];
#pragma unroll
  for (int c = 0; c < CPT; ++c) acc[c] = 0.f;
  float m = -INFINITY, l = 0.f;

  for (int t0 = 0; t0 < kv_len; t0 += BK) {
    __syncthreads();
    for (int e = tid; e < BK * D; e += 256) {
      const int rr = e / D, c = e - rr * D;
      const bool ok = t0 + rr < kv_len;
      ks[rr][c] = ok ? ld(ku + (long long)(t0 + rr) * D + c) : 0.f;
      vs[rr][c] = ok ? ld(vu + (long long)(t0 + rr) * D + c) : 0.f;
    }
    __syncthreads();
    float s[BK / G];
    float mx = m;
#pragma unroll
    for (int jj = 0; jj < BK / G; ++jj) {
      const int j = g + G * jj;
      float dot = 0.f;
      for (int c = 0; c < D; ++c) dot = fmaf(qs[r][c], ks[j][c], dot);
      s[jj] = (t0 + j < kv_len) ? dot * sm_scale : -INFINITY;
      mx = fmaxf(mx, s[jj]);
    }
#pragma unroll
    for (int off = 1; off < G; off <<= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
    const float alpha = expf(m - mx);  // m == -inf on the first tile -> 0
    float rs = 0.f;
#pragma unroll
    for (int jj = 0; jj < BK / G; ++jj) {
      const float p = expf(s[jj] - mx);
      ps[r][g + G * jj] = p;
      rs += p;
    }
#pragma unroll
    for (int off = 1; off < G; off <<= 1) rs += __shfl_xor(rs, off);
    l = l * alpha + rs;
    m = mx;
    __syncthreads();
#pragma unroll
    for (int c = 0; c < CPT; ++c) acc[c] *= alpha;
    for (int j = 0; j < BK; ++j) {
      const float p = ps[r][j];
#pragma unroll
      for (int c = 0; c < CPT; ++c) acc[c] = fmaf(p, vs[j][g + G * c], acc[c]);
    }
  }
  if (q0 + r < n_q) {
    const float inv = 1.f / l;
    T* o = out + ((long long)unit * n_q + q0 + r) * D;
#pragma unroll
    for (int c = 0; c < CPT; ++c) {
      const float val = acc[c] * inv;
      if constexpr (sizeof(T) == 4) ((float*)o)[g + G * c] = val;
      else ((uint16_t*)o)[g + G * c] = (uint16_t)float_to_bf16_bits(val);
    }
  }
}

// =====================================================================
// bf16 MFMA kernel.
//
// Workgroup = 4 waves; wave w owns QB blocks of 32 query rows; one iteration
// consumes BN = 64 keys.
//
// MFMA 32x32x16 operand layout (lane = 32*h + j):
//   A (32 x 16): lane holds row j, k-indices 8h..8h+7
//   B (16 x 32): lane holds column j, k-indices 8h..8h+7
//   C (32 x 32): lane holds column j, rows 8*(r/4) + 4h + (r%4) for r = 0..15
// First product  S^T[key][query]: A = K rows (k-index = channel), B = Q.
// Second product O^T[chan][query]: A = V^T (k-index = key), B = P^T.
// The C rows a lane owns in S^T are not 8 consecutive keys, so the key row fed to
// MFMA row i is taken from LDS row pi(i), pi swapping bits 2 and 3 of i.  Then
// registers r = 8m..8m+7 of an S^T block are exactly keys 16m + 8h + (0..7) of
// that block: the B operand of the second product with no data movement, and the
// matching V^T operand is one contiguous 16-byte LDS read.
// =====================================================================
constexpr int BN = 64;

template <int D>
struct AttendLds {
  static constexpr int KS = D + 8;    // LDS row stride of a K tile (elements)
  static constexpr int VS = BN + 8;   // LDS row stride of a V^T tile
  static constexpr int kTileK = BN * KS;
  static constexpr int kTileV = D * VS;
  static constexpr int kBytes = 2 * (kTileK + kTileV) * 2;  // two stages
};

template <int D, int QB>
__global__ __launch_bounds__(256) void attend_mfma_kernel(
    const uint16_t* __restrict__ q, int n_q, const uint16_t* __restrict__ k,
    long long k_seq_stride, long long k_head_stride, const uint16_t* __restrict__ v,
    long long v_seq_stride, long long v_head_stride, int kv_len, int n_head, float scale_log2e,
    uint16_t* __restrict__ out) {
  using L = AttendLds<D>;
  constexpr int KS = L::KS, VS = L::VS;
  constexpr int NSL = D / 16;  // k-slabs of the first product
  constexpr int NDB = D / 32;  // 32-channel blocks of the output
  constexpr int KV_LOADS = BN * D / 8 / 256;  // 16-byte vectors per thread per tile
  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
  uint16_t* const k_lds0 = smem;
  uint16_t* const vt_lds0 = smem + 2 * L::kTileK;

  const int unit = SCALEKV_WG_Y;
  const int seq = unit / n_head, head = unit - seq * n_head;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int j = lane & 31, h = lane >> 5;
  const int q_base = SCALEKV_WG_X * (128 * QB) + wave * (32 * QB);
  const uint16_t* qu = q + (long long)unit * n_q * D;
  const uint16_t* ku = k + seq * k_seq_stride + head * k_head_stride;
  const uint16_t* vu = v + seq * v_seq_stride + head * v_head_stride;

  // ---- Q fragments (B operand of the first product), kept for the whole kernel
  bf16x8 qf[QB][NSL];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int row = q_base + qb * 32 + j;
#pragma unroll
    for (int s = 0; s < NSL; ++s) {
      uint4 raw = make_uint4(0, 0, 0, 0);
      if (row < n_q) raw = *(const uint4*)(qu + (long long)row * D + 16 * s + 8 * h);
      qf[qb][s] = __builtin_bit_cast(bf16x8, raw);
    }
  }

  f32x16 o[NDB][QB];
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[db][qb][r] = 0.f;
  // m_run: the (possibly stale, see below) row max used as the exponent offset;
  // l_run: this lane's share of the row sum (the two half-waves are added at the end).
  float m_run[QB], l_run[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) { m_run[qb] = -INFINITY; l_run[qb] = 0.f; }

  // ---- staging maps
  // K tile: vector f = tid + 256*p covers row f/(D/8), 16-byte column f%(D/8).
  // V tile: thread owns 4 consecutive keys x 8 consecutive channels and writes them transposed.
  constexpr int CPR = D / 8;           // 16-byte vectors per row
  const int v_cg = tid % CPR;          // channel group: channels 8*v_cg .. +7
  const int v_rg = tid / CPR;          // key group (4 keys each), 256/CPR groups per pass
  constexpr int V_GROUPS = BN / 4;
  constexpr int V_PASSES = (V_GROUPS + 256 / CPR - 1) / (256 / CPR);
  uint4 k_stage[KV_LOADS];
  uint4 v_stage[V_PASSES][4];

  auto issue_loads = [&](int t0) {
#pragma unroll
    for (int p = 0; p < KV_LOADS; ++p) {
      const int f = tid + 256 * p;
      const int row = f / CPR, c = f % CPR;
      const int g = t0 + row;
      k_stage[p] = make_uint4(0, 0, 0, 0);
      if (g < kv_len) k_stage[p] = *(const uint4*)(ku + (long long)g * D + 8 * c);
    }
#pragma unroll
    for (int p = 0; p < V_PASSES; ++p) {
      const int key0 = 4 * (v_rg + p * (256 / CPR));
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int g = t0 + key0 + r;
        v_stage[p][r] = make_uint4(0, 0, 0, 0);  // zero rows: 0 * garbage must not reach the MFMA
        if (g < kv_len && key0 < BN) v_stage[p][r] = *(const uint4*)(vu + (long long)g * D + 8 * v_cg);
      }
    }
  };
  auto store_lds = [&](int stage) {
    uint16_t* k_lds = k_lds0 + stage * L::kTileK;
    uint16_t* vt_lds = vt_lds0 + stage * L::kTileV;
#pragma unroll
    for (int p = 0; p < KV_LOADS; ++p) {
      const int f = tid + 256 * p;
      const int row = f / CPR, c = f % CPR;
      *(uint4*)(k_lds + row * KS + 8 * c) = k_stage[p];
    }
#pragma unroll
    for (int p = 0; p < V_PASSES; ++p) {
      const int key0 = 4 * (v_rg + p * (256 / CPR));
      if (key0 >= BN) continue;  // head_dim 64: only half of the threads carry V
      const uint32_t* a = (const uint32_t*)&v_stage[p][0];
      const uint32_t* b = (const uint32_t*)&v_stage[p][1];
      const uint32_t* c = (const uint32_t*)&v_stage[p][2];
      const uint32_t* d = (const uint32_t*)&v_stage[p][3];
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        // channels 2w (low halves) and 2w+1 (high halves) of the four keys
        uint2 lo, hi;
        lo.x = __builtin_amdgcn_perm(b[w], a[w], 0x05040100u);  // (a.lo, b.lo)
        lo.y = __builtin_amdgcn_perm(d[w], c[w], 0x05040100u);
        hi.x = __builtin_amdgcn_perm(b[w], a[w], 0x07060302u);  // (a.hi, b.hi)
        hi.y = __builtin_amdgcn_perm(d[w], c[w], 0x07060302u);
        *(uint2*)(vt_lds + (8 * v_cg + 2 * w) * VS + key0) = lo;
        *(uint2*)(vt_lds + (8 * v_cg + 2 * w + 1) * VS + key0) = hi;
      }
    }
  };

  const int n_tile = (kv_len + BN - 1) / BN;
  issue_loads(0);
  store_lds(0);
  __syncthreads();
  for (int t = 0; t < n_tile; ++t) {
    const int stage = t & 1;
    const uint16_t* k_lds = k_lds0 + stage * L::kTileK;
    const uint16_t* vt_lds = vt_lds0 + stage * L::kTileV;
    const bool more = t + 1 < n_tile;
    if (more) issue_loads((t + 1) * BN);  // lands in registers while this tile is computed

    // ---- S^T = K Q^T for two 32-key blocks
    f32x16 s[2][QB];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int qb = 0; qb < QB; ++qb)
#pragma unroll
        for (int r = 0; r < 16; ++r) s[kb][qb][r] = 0.f;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      const uint16_t* krow = k_lds + (32 * kb + pi32(j)) * KS + 8 * h;
#pragma unroll
      for (int sl = 0; sl < NSL; ++sl) {
        const bf16x8 a = *(const bf16x8*)(krow + 16 * sl);
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
          s[kb][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[qb][sl], s[kb][qb], 0, 0, 0);
      }
    }

    // ---- online softmax; register r of block kb is key 32kb + 16(r/8) + 8h + r%8
    const int tile0 = t * BN;
    if (tile0 + BN > kv_len) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = tile0 + 32 * kb + 16 * (r / 8) + 8 * h + (r % 8);
          if (key >= kv_len) {
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) s[kb][qb][r] = -INFINITY;
          }
        }
    }
    // Row max of this tile.  The running offset m_run is only moved (and O, l
    // rescaled) when some row's max grew by more than kRescaleThreshold in log2
    // units; otherwise exp2 arguments stay <= the threshold, which fp32 and bf16
    // hold without loss, and the accumulators are left alone.
    float mx[QB];
    bool grow = false;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      float m = s[0][qb][0];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) m = fmaxf(m, s[kb][qb][r]);
      m = fmaxf(m, __shfl_xor(m, 32));
      mx[qb] = m;
      grow |= (m - m_run[qb]) * scale_log2e > kRescaleThreshold;
    }
    if (__builtin_amdgcn_ballot_w64(grow) != 0) {
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        const float m_new = fmaxf(m_run[qb], mx[qb]);
        const float alpha = __builtin_amdgcn_exp2f((m_run[qb] - m_new) * scale_log2e);
        m_run[qb] = m_new;
        l_run[qb] *= alpha;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[db][qb][r] *= alpha;
      }
    }
    bf16x8 pf[QB][4];
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      const float off = m_run[qb] * scale_log2e;
      float rs = 0.f;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
          const float p0 = __builtin_amdgcn_exp2f(fmaf(s[kb][qb][r], scale_log2e, -off));
          const float p1 = __builtin_amdgcn_exp2f(fmaf(s[kb][qb][r + 1], scale_log2e, -off));
          const bf16x2 pr = {(__bf16)p0, (__bf16)p1};
          pf[qb][2 * kb + r / 8][r % 8] = pr[0];
          pf[qb][2 * kb + r / 8][r % 8 + 1] = pr[1];
          // the row sum adds the rounded probabilities, the very numbers the MFMA multiplies by
          rs = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, rs, false);
        }
      l_run[qb] += rs;
    }

    // ---- O^T += V^T P^T
#pragma unroll
    for (int sl = 0; sl < 4; ++sl) {
#pragma unroll
      for (int db = 0; db < NDB; ++db) {
        const bf16x8 a = *(const bf16x8*)(vt_lds + (32 * db + j) * VS + 16 * sl + 8 * h);
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
          o[db][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[qb][sl], o[db][qb], 0, 0, 0);
      }
    }

    // the other stage was last read one iteration ago, before the barrier below
    if (more) store_lds(stage ^ 1);
    __syncthreads();
  }

  // ---- normalise and write: lane owns query column j, channels 32db + 8(r/4) + 4h + r%4
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int row = q_base + qb * 32 + j;
    const float l_tot = l_run[qb] + __shfl_xor(l_run[qb], 32);
    if (row >= n_q) continue;
    const float inv = 1.f / l_tot;
    uint16_t* orow = out + ((long long)unit * n_q + row) * D;
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        uint2 pk;
        pk.x = float_to_bf16_bits(o[db][qb][4 * g] * inv) |
               (float_to_bf16_bits(o[db][qb][4 * g + 1] * inv) << 16);
        pk.y = float_to_bf16_bits(o[db][qb][4 * g + 2] * inv) |
               (float_to_bf16_bits(o[db][qb][4 * g + 3] * inv) << 16);
        *(uint2*)(orow + 32 * db + 8 * g + 4 * h) = pk;
      }
  }
}

template <int D, int QB>
hipError_t launch_mfma(dim3 grid, hipStream_t stream, const uint16_t* q, int n_q, const uint16_t* k,
                       KvView kv, const uint16_t* v, KvView vv, int kv_len, int n_head,
                       float scale_log2e, uint16_t* out) {
  static std::atomic<uint64_t> configured{0};  // LDS above 64 KB per workgroup has to be asked for
  const hipError_t e = allow_dynamic_lds((const void*)attend_mfma_kernel<D, QB>,
                                         AttendLds<D>::kBytes, configured);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((attend_mfma_kernel<D, QB>), grid, dim3(256), AttendLds<D>::kBytes, stream, q,
                     n_q, k, kv.seq_stride, kv.head_stride, v, vv.seq_stride, vv.head_stride,
                     kv_len, n_head, scale_log2e, out);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_attend(int dtype, int n_seq, int n_head, int d, const void* q, int n_q, KvView k,
                         KvView v, int kv_len, float sm_scale, void* out, hipStream_t stream) {
  const int n_unit = n_seq * n_head;
  if (n_q <= 0 || n_unit <= 0) return hipSuccess;
  if (dtype == 0) {
    dim3 grid((n_q + 31) / 32, n_unit);
    if (d == 128)
      hipLaunchKernelGGL((attend_simple_kernel<float, 128>), grid, dim3(256), 0, stream,
                         (const float*)q, n_q, (const float*)k.ptr, k.seq_stride, k.head_stride,
                         (const float*)v.ptr, v.seq_stride, v.head_stride, kv_len, n_head,
                         sm_scale, (float*)out);
    else
      hipLaunchKernelGGL((attend_simple_kernel<float, 64>), grid, dim3(256), 0, stream,
                         (const float*)q, n_q, (const float*)k.ptr, k.seq_stride, k.head_stride,
                         (const float*)v.ptr, v.seq_stride, v.head_stride, kv_len, n_head,
                         sm_scale, (float*)out);
    return hipGetLastError();
  }
  const float scale_log2e = sm_scale * 1.4426950408889634f;
  const uint16_t* qp = (const uint16_t*)q;
  const uint16_t* kp = (const uint16_t*)k.ptr;
  const uint16_t* vp = (const uint16_t*)v.ptr;
  uint16_t* op = (uint16_t*)out;
  if (d == 128) {
    if (attend_uses_pipe(dtype, d, n_q))
      return launch_attend_pipe(n_unit, n_head, q, n_q, k, v, kv_len, nullptr, nullptr, 0, false,
                                sm_scale, out, stream);
    return launch_mfma<128, 1>(dim3((n_q + 127) / 128, n_unit), stream, qp, n_q, kp, k, vp, v,
                               kv_len, n_head, scale_log2e, op);
  }
  return launch_mfma<64, 1>(dim3((n_q + 127) / 128, n_unit), stream, qp, n_q, kp, k, vp, v, kv_len,
                            n_head, scale_log2e, op);
}

}  // namespace scalekv
