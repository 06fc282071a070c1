// Software-pipelined bf16 MFMA attention for head_dim 128 and large query
// counts: the kernel that carries almost all of the flops of the ScaleKV step
// (Sec. 3.1 / 3.3: the current token map attends, unmasked, over the retained
// cache followed by its own keys).
//
// Shape of the computation (transposed formulation):
//   S^T[key][query] = K Q^T          A = K rows from LDS,  B = Q held in registers
//   O^T[chan][query] += V^T P^T      A = V^T from LDS,     B = P^T straight from the
//                                    registers the first product left it in.
// A workgroup is 4 waves; each wave owns 64 query rows (two 32-row blocks), so an
// LDS operand fetched once feeds two MFMAs.  Keys are consumed in blocks of 32.
//
// MFMA 32x32x16 operand layout (lane = 32h + j):
//   A (32 x 16): lane holds row j, k-indices 8h..8h+7
//   B (16 x 32): lane holds column j, k-indices 8h..8h+7
//   C (32 x 32): lane holds column j, rows 8(r/4) + 4h + r%4 for r = 0..15
// MFMA row i of the first product is fed key row pi(i) (pi swaps bits 2 and 3),
// so registers r = 8m..8m+7 of an S^T block are keys 16m + 8h + (0..7) of the
// block: already the B operand of the second product.
//
// Data movement.  K and V tiles (64 keys x 256 B) go from HBM straight into LDS
// (global_load_lds, 16 B per lane, no registers), row-major, with the 16-byte
// chunks of each row XOR-swizzled so that operand reads are bank-conflict free.
// The V^T operand is read with the transposing LDS load (ds_read_b64_tr_b16):
// inside a group of 16 lanes, lane i supplies the address of 4 elements and
// receives element (i & 3) of the data addressed by lanes (i >> 2) + 4r, r = 0..3.
//
// Pipeline.  With one wave per SIMD nothing hides the softmax VALU work unless it
// is interleaved with MFMAs of the same wave, so the region of block b issues
//     MFMA:  S(b+1) and P(b-1) V(b-1)        VALU:  softmax of S(b).
// The exponentials of block b are taken against the running offset m_run as it
// stood after block b-1; only if some row max grew by more than kRescaleThreshold
// (log2 units) does a cold path rescale O and l and redo the block.  This is the
// usual online softmax with another, still safe, choice of offsets.
//
// LDS holds three stages of K and V tiles; tile t+2 is requested once every wave
// has left tile t-1 behind, which costs one barrier per 64 keys.
#include <type_traits>

#include "common.h"

namespace scalekv {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) const void glb_void;

constexpr int D = 128;
constexpr int QB = 2;                // 32-row query blocks per wave
constexpr int BM = 4 * 32 * QB;      // query rows per workgroup
constexpr int TN = 64;               // keys per staged tile (two blocks of 32)
constexpr int kRowBytes = D * 2;     // 256
constexpr int kTileBytes = TN * kRowBytes;  // 16 KB
constexpr int kStages = 3;
constexpr int kLdsBytes = 2 * kStages * kTileBytes;  // K stages then V stages
constexpr float kRescaleThreshold = 8.f;
constexpr int kSchedMfma = 0x008, kSchedValu = 0x002, kSchedDsRead = 0x100;
constexpr int kValuPerMfma = 6;

__device__ __forceinline__ int pi32(int i) {  // swap bits 2 and 3
  return (i & ~12) | ((i & 4) << 1) | ((i & 8) >> 1);
}

// Three-input max as one instruction and without the NaN-quieting pre-pass the compiler
// puts in front of fmaxf on values it has not produced itself.
__device__ __forceinline__ float max3(float a, float b, float c) {
  float r;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}

// Lanes l and l^32 hold the two halves of one query row's statistics.  The swap
// hands every lane {own value, partner's value} in some order; max and sum do not
// care which is which.
__device__ __forceinline__ float both_halves_max(float x) {
  const uint32_t u = __float_as_uint(x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float both_halves_sum(float x) {
  const uint32_t u = __float_as_uint(x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

__global__ __launch_bounds__(256) void attend_pipe_kernel(
    const uint16_t* __restrict__ q, int n_q, const uint16_t* __restrict__ k,
    long long k_seq_stride, long long k_head_stride, const uint16_t* __restrict__ v,
    long long v_seq_stride, long long v_head_stride, int kv_len, int n_head, float scale_log2e,
    uint16_t* __restrict__ out) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  unsigned char* const k_lds = smem;
  unsigned char* const v_lds = smem + kStages * kTileBytes;

  const int unit = blockIdx.y;
  const int seq = unit / n_head, head = unit - seq * n_head;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int j = lane & 31, h = lane >> 5;
  const int q_base = blockIdx.x * BM + wave * (32 * QB);
  const uint16_t* qu = q + (long long)unit * n_q * D;
  const unsigned char* ku = (const unsigned char*)(k + seq * k_seq_stride + head * k_head_stride);
  const unsigned char* vu = (const unsigned char*)(v + seq * v_seq_stride + head * v_head_stride);

  // ---- tile loader: per thread 4 K vectors and 4 V vectors of 16 bytes.
  // Instruction p of wave w fills LDS rows 16w + 4p .. +3 (64 lanes x 16 B = 4 rows);
  // the lane that lands in chunk slot s of row r fetches global chunk s ^ f(r).
  int ld_row[4];
  unsigned ld_kofs[4], ld_vofs[4];  // byte offset of this lane's vector inside a full tile
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    const int r = 16 * wave + 4 * p + (lane >> 4);
    ld_row[p] = r;
    ld_kofs[p] = r * kRowBytes + 16 * ((lane & 15) ^ (r & 15));
    ld_vofs[p] = r * kRowBytes + 16 * ((lane & 15) ^ ((r & 3) << 2));
  }
  auto issue_tile = [&](int tile) {
    unsigned char* ks = k_lds + (tile % kStages) * kTileBytes + (16 * wave) * kRowBytes;
    unsigned char* vs = v_lds + (tile % kStages) * kTileBytes + (16 * wave) * kRowBytes;
    const unsigned char* kt = ku + (long long)tile * kTileBytes;  // wave-uniform tile base
    const unsigned char* vt = vu + (long long)tile * kTileBytes;
    if ((tile + 1) * TN <= kv_len) {
#pragma unroll
      for (int p = 0; p < 4; ++p) {
        __builtin_amdgcn_global_load_lds((glb_void*)(kt + ld_kofs[p]), (lds_void*)(ks + 4 * p * kRowBytes), 16, 0, 0);
        __builtin_amdgcn_global_load_lds((glb_void*)(vt + ld_vofs[p]), (lds_void*)(vs + 4 * p * kRowBytes), 16, 0, 0);
      }
    } else {
      // ragged last tile: rows past the end re-read the last valid row (finite data that
      // the mask turns into zero weight)
      const int last_row = kv_len - 1 - tile * TN;
#pragma unroll
      for (int p = 0; p < 4; ++p) {
        const int back = max(ld_row[p] - last_row, 0) * kRowBytes;
        __builtin_amdgcn_global_load_lds((glb_void*)(kt + (ld_kofs[p] - back)), (lds_void*)(ks + 4 * p * kRowBytes), 16, 0, 0);
        __builtin_amdgcn_global_load_lds((glb_void*)(vt + (ld_vofs[p] - back)), (lds_void*)(vs + 4 * p * kRowBytes), 16, 0, 0);
      }
    }
  };

  // ---- per-lane operand offsets inside a 32-key block (bytes)
  int k_ofs[8];  // K operand, slab sl: row pi(j), chunk (2sl + h) ^ (row & 15)
  {
    const int row = pi32(j);
#pragma unroll
    for (int sl = 0; sl < 8; ++sl) k_ofs[sl] = row * kRowBytes + 16 * ((2 * sl + h) ^ (row & 15));
  }
  int v_ofs[4];  // V^T operand, channel block db: this lane's address role in the transposing load
  {
    const int i = j & 15, g = i >> 2;
#pragma unroll
    for (int db = 0; db < 4; ++db)
      v_ofs[db] = (8 * h + g) * kRowBytes + 64 * (db ^ g) + 32 * (j >> 4) + 8 * (i & 3);
  }

  // ---- Q fragments: B operand of the first product, resident for the whole kernel
  bf16x8 qf[QB][8];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int row = q_base + qb * 32 + j;
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      uint4 raw = make_uint4(0, 0, 0, 0);
      if (row < n_q) raw = *(const uint4*)(qu + (long long)row * D + 16 * s + 8 * h);
      qf[qb][s] = __builtin_bit_cast(bf16x8, raw);
    }
  }

  f32x16 o[4][QB];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[db][qb][r] = 0.f;
  float m_run[QB], l_run[QB];  // exponent offset; this lane's share of the row sum
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) { m_run[qb] = -INFINITY; l_run[qb] = 0.f; }

  // S(blk) = K Q^T for the 32 keys of block `blk`.
  // Operand fetches.  `ofs` = byte offset of the block inside the stage array (a constant
  // in the main loop, where it folds into the instruction's offset field).
  auto load_k = [&](int ofs, int sl) -> bf16x8 {  // K rows of the block, channels of slab sl
    return *(const bf16x8*)(k_lds + ofs + k_ofs[sl]);
  };
  auto load_vt = [&](int ofs, int sl, int db) -> bf16x8 {  // V^T: channels of block db, keys of slab sl
    const unsigned char* p = v_lds + ofs + sl * 16 * kRowBytes + v_ofs[db];
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)p);
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (__attribute__((address_space(3))) s16x4*)(p + 4 * kRowBytes));
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
  };
  auto mfma_s_step = [&](const bf16x8& a, int sl, f32x16 (&s_out)[QB]) {
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      f32x16 c = s_out[qb];
      if (sl == 0) {
#pragma unroll
        for (int r = 0; r < 16; ++r) c[r] = 0.f;
      }
      s_out[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[qb][sl], c, 0, 0, 0);
    }
  };
  auto mfma_pv_step = [&](const bf16x8& a, int sl, int db, const bf16x8 (&p_in)[QB][2]) {
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
      o[db][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, p_in[qb][sl], o[db][qb], 0, 0, 0);
  };
  // whole-block forms, used outside the pipelined regions
  auto mfma_s = [&](int ofs, f32x16 (&s_out)[QB]) {
#pragma unroll
    for (int sl = 0; sl < 8; ++sl) mfma_s_step(load_k(ofs, sl), sl, s_out);
  };
  auto mfma_pv = [&](int ofs, const bf16x8 (&p_in)[QB][2]) {
#pragma unroll
    for (int sl = 0; sl < 2; ++sl)
#pragma unroll
      for (int db = 0; db < 4; ++db) mfma_pv_step(load_vt(ofs, sl, db), sl, db, p_in);
  };
  // two scores -> two probabilities (bf16) against exponent offset `off`; the row-sum share
  // adds the rounded values, the very numbers the MFMA multiplies by
  auto exp_pair = [&](const f32x16& s, int r, float off, bf16x8 (&p)[2], float& rs) {
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
    const float p0 = __builtin_amdgcn_exp2f(fmaf(s[r], scale_log2e, -off));
    const float p1 = __builtin_amdgcn_exp2f(fmaf(s[r + 1], scale_log2e, -off));
    const bf16x2 pr = {(__bf16)p0, (__bf16)p1};
    p[r / 8][r % 8] = pr[0];
    p[r / 8][r % 8 + 1] = pr[1];
    rs = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, rs, false);
  };
  auto exp_pair2 = [&](float x0, float x1, int r, float off, bf16x8 (&p)[2], float& rs) {
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
    const float p0 = __builtin_amdgcn_exp2f(fmaf(x0, scale_log2e, -off));
    const float p1 = __builtin_amdgcn_exp2f(fmaf(x1, scale_log2e, -off));
    const bf16x2 pr = {(__bf16)p0, (__bf16)p1};
    p[r / 8][r % 8] = pr[0];
    p[r / 8][r % 8 + 1] = pr[1];
    rs = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, rs, false);
  };
  auto exps = [&](const f32x16& s, float off, bf16x8 (&p)[2]) -> float {
    float rs = 0.f;
#pragma unroll
    for (int r = 0; r < 16; r += 2) exp_pair(s, r, off, p, rs);
    return rs;
  };

  // One region: softmax of block `blk` (scores in s_in; register r = key 16(r/8) + 8h + r%8
  // of the block) together with S(blk+1) -> s_out (K block at k_next_ofs) and
  // P(blk-1) V(blk-1) from p_in (V block at v_prev_ofs).  `mask` (only looked at when
  // may_mask) hides keys at or beyond kv_len.
  //
  // The body is 16 steps.  Step i issues one MFMA pair (first the 8 slabs of S, then the 8
  // (slab, channel block) pieces of PV), fetches the operand two steps ahead, and then does
  // 1/16 of the softmax VALU work, which executes while the pair is in the matrix pipe.
  // Scheduling fences keep the compiler from regrouping the steps.
  auto region = [&](auto has_prev, auto has_next, auto may_mask, bool mask, int blk, int k_next_ofs,
                    int v_prev_ofs, f32x16 (&s_in)[QB], f32x16 (&s_out)[QB],
                    const bf16x8 (&p_in)[QB][2], bf16x8 (&p_out)[QB][2]) {
    constexpr bool kPrev = decltype(has_prev)::value, kNext = decltype(has_next)::value;
    if constexpr (decltype(may_mask)::value) {
      if (mask) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = 32 * blk + 16 * (r / 8) + 8 * h + (r % 8);
          if (key >= kv_len) {
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) s_in[qb][r] = -INFINITY;
          }
        }
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    auto fetch = [&](int i) -> bf16x8 {  // operand of step i
      if (i < 8) return load_k(k_next_ofs, i);
      return load_vt(v_prev_ofs, (i - 8) >> 2, (i - 8) & 3);
    };
    auto wanted = [&](int i) { return i < 8 ? kNext : (i < 16 ? kPrev : false); };
    bf16x8 frag[3];
    if (wanted(0)) frag[0] = fetch(0);
    if (wanted(1)) frag[1] = fetch(1);
    float mx[QB], rs[QB], off[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) { rs[qb] = 0.f; off[qb] = m_run[qb] * scale_log2e; }
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      if (wanted(i + 2)) frag[(i + 2) % 3] = fetch(i + 2);
      if (wanted(i)) {
        if (i < 8) mfma_s_step(frag[i % 3], i, s_out);
        else mfma_pv_step(frag[i % 3], (i - 8) >> 2, (i - 8) & 3, p_in);
      }
      __builtin_amdgcn_sched_barrier(0);
      {  // VALU share of this step: one pair of exponentials and one piece of the row max.
        // The scores sit in accumulation registers (where the MFMAs of the previous region
        // left them, long enough ago for any wait state) and are fetched here, two at a
        // time, rather than all at once behind the MFMA that produced them.
        const int qb = i & 1, pair = i >> 1;
        float x0, x1;
        asm volatile("v_accvgpr_read_b32 %0, %2\n\tv_accvgpr_read_b32 %1, %3"
                     : "=v"(x0), "=v"(x1)
                     : "a"(s_in[qb][2 * pair]), "a"(s_in[qb][2 * pair + 1]));
        exp_pair2(x0, x1, 2 * pair, off[qb], p_out[qb], rs[qb]);
        mx[qb] = pair == 0 ? fmaxf(x0, x1) : max3(mx[qb], x0, x1);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    bool grow = false;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      mx[qb] = both_halves_max(mx[qb]);
      grow |= (mx[qb] - m_run[qb]) * scale_log2e > kRescaleThreshold;
    }
    // Pin the speculative results before the branch: without this the compiler may move
    // the exponentials onto the common path after it.
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      asm volatile("" : "+v"(rs[qb]), "+v"(p_out[qb][0]), "+v"(p_out[qb][1]));
    }
    if (__builtin_amdgcn_ballot_w64(grow) != 0) {  // cold: some row max moved a lot
      // O lives in accumulation registers, which only MFMA and the accvgpr moves can
      // touch; scale it through one scratch VGPR.  The leading no-ops cover the wait
      // states between an MFMA writing O and a move reading it.
      asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        const float m_new = fmaxf(m_run[qb], mx[qb]);
        const float alpha = __builtin_amdgcn_exp2f((m_run[qb] - m_new) * scale_log2e);
        m_run[qb] = m_new;
        l_run[qb] *= alpha;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            float x = o[db][qb][r], tmp;
            asm volatile(
                "v_accvgpr_read_b32 %1, %0\n\t"
                "s_nop 1\n\t"
                "v_mul_f32 %1, %1, %2\n\t"
                "s_nop 1\n\t"
                "v_accvgpr_write_b32 %0, %1"
                : "+a"(x), "=&v"(tmp)
                : "v"(alpha));
            o[db][qb][r] = x;
          }
        rs[qb] = exps(s_in[qb], m_new * scale_log2e, p_out[qb]);
      }
      asm volatile("s_nop 7" ::: "memory");
    }
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) l_run[qb] += rs[qb];
  };

  const int n_tile = (kv_len + TN - 1) / TN;
  const bool ragged = (kv_len % TN) != 0;
  std::true_type yes;
  std::false_type no;

  // Even blocks read their scores from s_a and leave the next block's in s_b; odd blocks
  // the other way round.  P of an even block goes to p_a, of an odd block to p_b.
  f32x16 s_a[QB], s_b[QB];
  bf16x8 p_a[QB][2], p_b[QB][2];

  auto blk_ofs = [](int blk) { return ((blk >> 1) % kStages) * kTileBytes + (blk & 1) * 32 * kRowBytes; };

  issue_tile(0);
  if (n_tile > 1) issue_tile(1);
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();
  mfma_s(0, s_a);
  region(no, yes, yes, ragged && n_tile == 1, 0, blk_ofs(1), 0, s_a, s_b, p_b, p_a);

  // Crossing from tile t to tile t+1: tile t+1 was requested a whole tile ago; once every
  // wave is past tile t-1 its stage is free for tile t+2.
  auto next_tile = [&](int t) {
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (t + 2 < n_tile) issue_tile(t + 2);
  };
  int t = 0;
  if (n_tile > 1) next_tile(0);
  // Main loop, three tiles per trip so that every LDS stage offset is a constant.  Tile
  // t+u sits in stage u; all blocks touched lie in full, interior tiles.
  for (; t + 4 < n_tile; t += 3) {
#pragma unroll
    for (int u = 0; u < 3; ++u) {
      constexpr int kHalf = 32 * kRowBytes;
      const int un = (u + 1) % 3;
      region(yes, yes, no, false, 0, un * kTileBytes, u * kTileBytes, s_b, s_a, p_a, p_b);
      region(yes, yes, no, false, 0, un * kTileBytes + kHalf, u * kTileBytes + kHalf, s_a, s_b, p_b, p_a);
      next_tile(t + u + 1);
    }
  }
  for (; t + 2 < n_tile; ++t) {  // left-over interior tiles, offsets computed at run time
    region(yes, yes, no, false, 0, blk_ofs(2 * t + 2), blk_ofs(2 * t), s_b, s_a, p_a, p_b);
    region(yes, yes, no, false, 0, blk_ofs(2 * t + 3), blk_ofs(2 * t + 1), s_a, s_b, p_b, p_a);
    next_tile(t + 1);
  }
  if (t + 1 < n_tile) {  // into the last tile, which may be ragged
    region(yes, yes, no, false, 0, blk_ofs(2 * t + 2), blk_ofs(2 * t), s_b, s_a, p_a, p_b);
    region(yes, yes, yes, ragged, 2 * t + 2, blk_ofs(2 * t + 3), blk_ofs(2 * t + 1), s_a, s_b, p_b, p_a);
  }
  region(yes, no, yes, ragged, 2 * n_tile - 1, 0, blk_ofs(2 * n_tile - 2), s_b, s_a, p_a, p_b);
  mfma_pv(blk_ofs(2 * n_tile - 1), p_b);

  // ---- normalise and write: lane owns query column j, channels 32db + 8(r/4) + 4h + r%4
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int row = q_base + qb * 32 + j;
    const float l_tot = both_halves_sum(l_run[qb]);
    if (row >= n_q) continue;
    const float inv = 1.f / l_tot;
    uint16_t* orow = out + ((long long)unit * n_q + row) * D;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const bf16x2 lo = {(__bf16)(o[db][qb][4 * g] * inv), (__bf16)(o[db][qb][4 * g + 1] * inv)};
        const bf16x2 hi = {(__bf16)(o[db][qb][4 * g + 2] * inv), (__bf16)(o[db][qb][4 * g + 3] * inv)};
        uint2 pk;
        pk.x = __builtin_bit_cast(uint32_t, lo);
        pk.y = __builtin_bit_cast(uint32_t, hi);
        *(uint2*)(orow + 32 * db + 8 * g + 4 * h) = pk;
      }
  }
}

}  // namespace

hipError_t launch_attend_pipe(int n_unit, int n_head, const void* q, int n_q, KvView k, KvView v,
                              int kv_len, float sm_scale, void* out, hipStream_t stream) {
  static bool configured = false;  // more than 64 KB of LDS per workgroup has to be requested
  if (!configured) {
    hipError_t e = hipFuncSetAttribute((const void*)attend_pipe_kernel,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (e != hipSuccess) return e;
    configured = true;
  }
  const float scale_log2e = sm_scale * 1.4426950408889634f;
  dim3 grid((n_q + BM - 1) / BM, n_unit);
  hipLaunchKernelGGL(attend_pipe_kernel, grid, dim3(256), kLdsBytes, stream, (const uint16_t*)q,
                     n_q, (const uint16_t*)k.ptr, k.seq_stride, k.head_stride,
                     (const uint16_t*)v.ptr, v.seq_stride, v.head_stride, kv_len, n_head,
                     scale_log2e, (uint16_t*)out);
  return hipGetLastError();
}

}  // namespace scalekv
