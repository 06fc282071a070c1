// bf16 MFMA attention for head_dim 128 and large query counts: the kernel that
// carries almost all of the flops of the ScaleKV step (Sec. 3.1 / 3.3: the current
// token map attends, unmasked, over the retained cache followed by its own keys).
//
// Shape of the computation (transposed formulation):
//   S^T[key][query] = K Q^T          A = K rows from LDS,  B = Q held in registers
//   O^T[chan][query] += V^T P^T      A = V^T from LDS,     B = P^T straight from the
//                                    registers the first product left it in.
// so one lane owns one query column: the softmax statistics are per-lane scalars.
//
// MFMA 32x32x16 operand layout (lane = 32h + j):
//   A (32 x 16): lane holds row j, k-indices 8h..8h+7
//   B (16 x 32): lane holds column j, k-indices 8h..8h+7
//   C (32 x 32): lane holds column j, rows 8(r/4) + 4h + r%4 for r = 0..15
// MFMA row i of the first product is fed key row pi(i) (pi swaps bits 2 and 3),
// so registers r = 8m..8m+7 of an S^T block are keys 16m + 8h + (0..7) of the
// block: already the B operand of the second product.
//
// Occupancy.  Vector instructions that follow a run of a wave's own MFMAs wait for the
// run (the wave issues in order and stalls at each MFMA until the pipe takes it), so
// the softmax of a block hides behind the matrix pipe only if a second wave shares
// the SIMD, or if it is cut up and spread between the MFMAs of another product.  The
// second form was built as well (blocks skewed by one, PV(b-1) interleaved with the
// softmax of block b) and measured 2-3 % slower than this one.  The kernel is written
// for two workgroups of 4 waves per CU: every wave owns 32 query rows, stays under
// 256 registers, and runs plain in-order code (S, softmax, PV per block of 32 keys);
// the two workgroups drift apart and fill each other's gaps.  LDS operand traffic is
// 16 KB per wave and block, half of what the LDS delivers at full MFMA rate.
//
// Data movement.  K and V tiles (64 keys x 256 B) go from HBM/L2 straight into LDS
// (global_load_lds, 16 B per lane, no registers), row-major, with the 16-byte
// chunks of each row XOR-swizzled so that operand reads are bank-conflict free.
// The V^T operand is read with the transposing LDS load (ds_read_b64_tr_b16):
// inside a group of 16 lanes, lane i supplies the address of 4 elements and
// receives element (i & 3) of the data addressed by lanes (i >> 2) + 4r, r = 0..3.
// Two stages per workgroup; tile t+2 is requested right after the barrier in the
// middle of tile t's second block, which is also the point from which tile t+1 may
// be read.  LDS operands are requested one phase ahead of the MFMAs that use them.
//
// Softmax.  The exponent offset m_run of a query row is taken from the row's maximum
// over the first tile and then left alone: every later probability is exp2 of
// (score - m_run), whatever its size, and the row sum adds the bf16-rounded
// probabilities, the very numbers the MFMA multiplies by.  No running maximum is
// formed (it costs a sixth of the vector instructions of a block).  This is exact as
// long as nothing overflows, and fp32 / bf16 carry 2^127: a lane only checks that its
// share of a block's row sum stays below 2^100 (scores up to 69 natural units above the
// first tile's maximum: heavy-tailed keys reach 35) and records a failure in a scalar
// mask; row sums then stay below 2^114.  The accumulators could still overflow if the
// values themselves are huge (2^100 times 2^14 keys leaves room for |v| up to 2^13), so
// at the end of the pass every lane also checks that its accumulators are finite.
// If any wave of the workgroup recorded a failure (forced by the tests), the workgroup
// discards its result and repeats the whole pass with the classical scheme: running
// maximum per block, offsets moved (and O, l rescaled) when some row maximum grew by
// more than kRescaleThreshold in log2 units.
//
// Workgroups of one (sequence, head) unit are numbered so that they land on the
// same XCD and share its L2 while they stream the same K/V.
//
// Two key segments.  The keys are the first len1 rows of a cache followed by len2
// rows of a dense tensor (the current map's own K/V); each segment is walked in tiles
// of its own, so at most one ragged tile per segment is masked.  When asked to, every
// workgroup also copies its share of the second segment behind the first in the cache
// (rows len1 .. len1+len2-1): the append of the pruning step, done here because this
// kernel is bound by the matrix pipe and leaves the HBM idle, while a separate copy
// kernel would be bound by the HBM and leave the matrix pipe idle.
#include <hip/hip_ext.h>

#include <type_traits>

#include "common.h"

namespace scalekv {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) const void glb_void;

constexpr int D = 128;
constexpr int BM = 128;              // query rows per workgroup: 4 waves x 32
constexpr int TN = 64;               // keys per staged tile (two blocks of 32)
constexpr int kRowBytes = D * 2;     // 256
constexpr int kTileBytes = TN * kRowBytes;  // 16 KB
constexpr int kStages = 2;
// Measurement-only builds (python -m paper_2505_19602_amd.build --variant ...; never the library
// the tests or the bench's headline load): each takes one ingredient out of the kernel so that
// its share of the running time can be read off a timing.  Their results are wrong on purpose.
//   SCALEKV_ABLATE_SOFTMAX    probabilities are the raw scores converted to bf16: no exp2, no
//                             row sums, no overflow watch
//   SCALEKV_ABLATE_TRANSFER   only the first two key tiles are fetched; later tiles re-use them
//   SCALEKV_ONE_WG_PER_CU     the workgroup claims more than half of the LDS, so that one
//                             workgroup runs per compute unit (results stay correct)
//   SCALEKV_TIMELINE          every workgroup records when it started, when its first tile had
//                             arrived, when it left the tile loop and when it ended (results stay
//                             correct); scalekv_timeline_read() hands the records to the host
#if defined(SCALEKV_ONE_WG_PER_CU)
constexpr int kLdsBytes = 96 * 1024;
#else
constexpr int kLdsBytes = 2 * kStages * kTileBytes;  // K stages then V stages: 64 KB
#endif
#if defined(SCALEKV_TIMELINE)
constexpr int kTimelineMaxWg = 8192;
constexpr int kTimelineWords = 7;  // four readings of the 100 MHz counter, the hardware id register, the shader clock counter at start and end
__device__ unsigned long long g_timeline[kTimelineMaxWg * kTimelineWords];
#define SCALEKV_STAMP(name) const unsigned long long name = __builtin_amdgcn_s_memrealtime()
#else
#define SCALEKV_STAMP(name)
#endif
constexpr float kBlockSumLimit = 0x1p100f;  // largest row-sum share a block may add unchecked
constexpr int kXcds = 8;

// Three-input max as one instruction and without the NaN-quieting pre-pass the
// compiler puts in front of fmaxf on values it has not produced itself.
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

// One 16-byte-per-lane transfer from global memory straight into LDS: lane l's vector comes
// from base + voff + IMM and lands at LDS byte lds_addr + IMM + 16 l (the instruction's
// immediate offset applies to both addresses).  The request is written in
// assembly on purpose: the compiler, when it knows about a global->LDS transfer, waits for
// it before the next LDS read of the same array, which would serialise the transfer of tile
// t+1 with the consumption of tile t.  Here the only wait is the explicit one in front of the
// barrier that publishes the tile.
template <int IMM>
__device__ __forceinline__ void dma16(const unsigned char* base_uniform, unsigned voff,
                                      unsigned lds_addr_uniform) {
  asm volatile(
      "s_mov_b32 m0, %0\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %1, %2 offset:%3"
      :
      : "s"(lds_addr_uniform), "v"(voff), "s"(base_uniform), "n"(IMM)
      : "m0", "memory");
}

// The same with the lane's offset formed on the spot as (chunk ^ flip) + row: the K tile's
// chunk swizzle differs between a lane's four transfers by an XOR, and forming it here keeps
// the compiler from holding four precomputed offsets in registers through the main loop.
template <int IMM>
__device__ __forceinline__ void dma16_xor(const unsigned char* base_uniform, unsigned row_part,
                                          unsigned chunk_part, unsigned flip_uniform,
                                          unsigned lds_addr_uniform) {
  unsigned voff;
  asm volatile(
      "v_xad_u32 %0, %2, %3, %1\n\t"
      "s_mov_b32 m0, %4\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %0, %5 offset:%6"
      : "=&v"(voff)
      : "v"(row_part), "v"(chunk_part), "s"(flip_uniform), "s"(lds_addr_uniform),
        "s"(base_uniform), "n"(IMM)
      : "m0", "memory");
}

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
void attend_pipe_kernel(const uint16_t* __restrict__ q, int n_q, uint16_t* k, long long k_seq_stride,
                        long long k_head_stride, uint16_t* v, long long v_seq_stride,
                        long long v_head_stride, int len1, const uint16_t* __restrict__ k2,
                        const uint16_t* __restrict__ v2, int len2, int append, int n_head,
                        int n_qtile, int n_wg, float scale_log2e, uint16_t* __restrict__ out) {
  SCALEKV_STAMP(t_start);
#if defined(SCALEKV_TIMELINE)
  unsigned long long t_first_tile = 0;
  const unsigned long long c_start = __builtin_readcyclecounter();
#endif
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  unsigned char* const k_lds = smem;
  unsigned char* const v_lds = smem + kStages * kTileBytes;

  // Consecutive workgroup ids go round-robin over the XCDs.  Renumber so that the ids an
  // XCD receives are consecutive: all query tiles of a unit then share one L2.
  int wg = SCALEKV_WG_X;
  {
    const int per = n_wg / kXcds, full = per * kXcds;  // the tail (< 8 groups) keeps its ids
    if (wg < full) wg = (wg % kXcds) * per + wg / kXcds;
  }
  const int unit = wg / n_qtile, qtile = wg - unit * n_qtile;
  const int seq = unit / n_head, head = unit - seq * n_head;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int j = lane & 31, h = lane >> 5;
  const int q_base = qtile * BM + wave * 32;
  const uint16_t* qu = q + (long long)unit * n_q * D;
  const unsigned char* ku = (const unsigned char*)(k + seq * k_seq_stride + head * k_head_stride);
  const unsigned char* vu = (const unsigned char*)(v + seq * v_seq_stride + head * v_head_stride);
  const unsigned char* k2u = (const unsigned char*)(k2 + (long long)unit * len2 * D);
  const unsigned char* v2u = (const unsigned char*)(v2 + (long long)unit * len2 * D);
  const int n_tile1 = (len1 + TN - 1) / TN;
  const int n_tile = n_tile1 + (len2 + TN - 1) / TN;

  // ---- tile loader: per thread 4 K vectors and 4 V vectors of 16 bytes.
  // Instruction p of wave w fills LDS rows 16w + 4p .. +3 (64 lanes x 16 B = 4 rows);
  // the lane that lands in chunk slot s of row r fetches global chunk s ^ f(r), with
  // f(r) = r & 15 for K and (r & 3) << 2 for V.  For this lane r = r0 + 4p with r0 & 15 =
  // lane >> 4 < 4, so its K chunk is c0 ^ 4p with c0 = (lane & 15) ^ (lane >> 4) and its V
  // chunk does not depend on p: one register pair serves all four instructions, the rest
  // (1024 p bytes) rides in the instruction's immediate offset.
  const int ld_row0 = 16 * wave + (lane >> 4);
  const unsigned ld_krow = ld_row0 * kRowBytes;                          // K: row part
  const unsigned ld_kchunk = 16 * ((lane & 15) ^ (lane >> 4));           // K: chunk part for p = 0
  const unsigned ld_vofs = ld_row0 * kRowBytes + 16 * ((lane & 15) ^ ((lane >> 4) << 2));
  auto lds_addr = [](const unsigned char* p) -> unsigned {
    return (unsigned)(size_t)(const __attribute__((address_space(3))) unsigned char*)p;
  };
  // LDS byte addresses of this wave's 16 rows in stage 0 (wave-uniform, kept in scalar registers)
  const unsigned k_lds_wave = __builtin_amdgcn_readfirstlane(lds_addr(k_lds + (16 * wave) * kRowBytes));
  const unsigned v_lds_wave = __builtin_amdgcn_readfirstlane(lds_addr(v_lds + (16 * wave) * kRowBytes));
  auto issue_tile = [&](int tile) __attribute__((always_inline)) {
    const unsigned ks = k_lds_wave + (tile % kStages) * kTileBytes;
    const unsigned vs = v_lds_wave + (tile % kStages) * kTileBytes;
    // wave-uniform tile base and number of valid rows, in whichever segment the tile lies
    const bool second = tile >= n_tile1;
    const int lt = second ? tile - n_tile1 : tile;
    const unsigned char* kt = (second ? k2u : ku) + (long long)lt * kTileBytes;
    const unsigned char* vt = (second ? v2u : vu) + (long long)lt * kTileBytes;
    const int valid = (second ? len2 : len1) - lt * TN;
    if (valid >= TN) {
      // the immediate offset moves the LDS destination along with the global source, which
      // is exactly the 4 rows between a lane's consecutive transfers
      dma16_xor<0>(kt, ld_krow, ld_kchunk, 0u, ks);
      dma16<0>(vt, ld_vofs, vs);
      dma16_xor<1024>(kt, ld_krow, ld_kchunk, 64u, ks);
      dma16<1024>(vt, ld_vofs, vs);
      dma16_xor<2048>(kt, ld_krow, ld_kchunk, 128u, ks);
      dma16<2048>(vt, ld_vofs, vs);
      dma16_xor<3072>(kt, ld_krow, ld_kchunk, 192u, ks);
      dma16<3072>(vt, ld_vofs, vs);
    } else {
      // ragged last tile: rows past the end re-read the last valid row (finite data that
      // the mask turns into zero weight)
      const int last_row = valid - 1;
#pragma unroll
      for (int p = 0; p < 4; ++p) {
        const int back = max(ld_row0 + 4 * p - last_row, 0) * kRowBytes;
        dma16<0>(kt, ld_krow + (ld_kchunk ^ (64 * p)) + 1024 * p - back, ks + 4 * p * kRowBytes);
        dma16<0>(vt, ld_vofs + 1024 * p - back, vs + 4 * p * kRowBytes);
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

  // ---- Q fragments: B operand of the first product, resident for the whole kernel.  A lane's
  // fragments are eight 16-byte pieces of its query row, 32 bytes apart: fetched as such, every
  // instruction of the wave would touch 32 rows with 32 bytes each.  Instead the wave's 32 rows
  // go, whole and 16 bytes per lane, straight into LDS and are read from there once the first
  // tile has arrived.  They wait in the second stage, which is not in use before the first
  // barrier, each wave's rows exactly where the same wave will later put its share of the second
  // tile (16 K rows and 16 V rows, 4 KB each): nobody else writes there, so no barrier is needed
  // before that tile is requested, only the wave's own reads must have returned.  Chunk c of row
  // r sits in slot c ^ (r & 15), so that the fragment reads are free of bank conflicts.  Rows
  // past the end of the map repeat its last row; nothing is stored for them.
  bf16x8 qf[8];
  unsigned char* const q_stage_k = k_lds + kTileBytes + (16 * wave) * kRowBytes;  // query rows 0-15 of the wave
  unsigned char* const q_stage_v = v_lds + kTileBytes + (16 * wave) * kRowBytes;  // query rows 16-31
  {
    const unsigned qk = __builtin_amdgcn_readfirstlane(lds_addr(q_stage_k));
    const unsigned qv = __builtin_amdgcn_readfirstlane(lds_addr(q_stage_v));
#pragma unroll
    for (int p = 0; p < 8; ++p) {
      const int r = 4 * p + (lane >> 4);
      const unsigned row = (unsigned)min(q_base + r, n_q - 1);
      dma16<0>((const unsigned char*)qu, row * kRowBytes + 16 * ((lane & 15) ^ (r & 15)),
               (p < 4 ? qk : qv) + 4 * (p & 3) * kRowBytes);
    }
  }
  auto read_q = [&]() __attribute__((always_inline)) {
    const unsigned char* row = (j < 16 ? q_stage_k : q_stage_v) + (j & 15) * kRowBytes;
#pragma unroll
    for (int s = 0; s < 8; ++s) qf[s] = *(const bf16x8*)(row + 16 * ((2 * s + h) ^ (j & 15)));
  };

  f32x16 o[4];
  float m_run;  // exponent offset
  float l_run;  // this lane's share of the row sum
  unsigned long long overflowed = 0;  // lanes whose block sum left the unchecked range

  auto load_k = [&](int ofs, int sl) -> bf16x8 { return *(const bf16x8*)(k_lds + ofs + k_ofs[sl]); };
  auto load_vt = [&](int ofs, int sl, int db) -> bf16x8 {
    const unsigned char* p = v_lds + ofs + sl * 16 * kRowBytes + v_ofs[db];
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)p);
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (__attribute__((address_space(3))) s16x4*)(p + 4 * kRowBytes));
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
  };
  auto exps = [&](const f32x16& s, float off, bf16x8 (&p)[2]) -> float {
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
    float rs = 0.f;
#pragma unroll
    for (int r = 0; r < 16; r += 2) {
#if defined(SCALEKV_ABLATE_SOFTMAX)
      const float p0 = s[r], p1 = s[r + 1];
#else
      const float p0 = __builtin_amdgcn_exp2f(fmaf(s[r], scale_log2e, -off));
      const float p1 = __builtin_amdgcn_exp2f(fmaf(s[r + 1], scale_log2e, -off));
#endif
      const bf16x2 pr = {(__bf16)p0, (__bf16)p1};
      p[r / 8][r % 8] = pr[0];
      p[r / 8][r % 8 + 1] = pr[1];
#if !defined(SCALEKV_ABLATE_SOFTMAX)
      rs = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, rs, false);
#endif
    }
#if defined(SCALEKV_ABLATE_SOFTMAX)
    rs = 1.f;
#endif
    return rs;
  };

  // ---- the phases of one block of 32 keys
  auto fetch_k = [&](bf16x8 (&kf)[8], int ofs) {
#pragma unroll
    for (int sl = 0; sl < 8; ++sl) kf[sl] = load_k(ofs, sl);
  };
  auto fetch_vt = [&](bf16x8 (&vf)[2][4], int ofs) {
#pragma unroll
    for (int sl = 0; sl < 2; ++sl)
#pragma unroll
      for (int db = 0; db < 4; ++db) vf[sl][db] = load_vt(ofs, sl, db);
  };
  auto scores = [&](const bf16x8 (&kf)[8]) -> f32x16 {
    f32x16 s;
#pragma unroll
    for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
    for (int sl = 0; sl < 8; ++sl) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[sl], qf[sl], s, 0, 0, 0);
    return s;
  };
  // softmax of the block's scores (register r = key 16(r/8) + 8h + r%8 of the block, which
  // starts at row first_key of its tile; `mask` hides rows at or beyond `valid`) followed by
  // O^T += V^T P^T
  // `tracked` (a std::bool_constant): follow the running maximum; otherwise keep m_run and
  // only watch for overflow.
  auto softmax_pv = [&](auto tracked, f32x16& s, const bf16x8 (&vf)[2][4], bool mask, int first_key,
                        int valid) __attribute__((always_inline)) {
    if (mask) {
      // (the lane half is taken from the lane number on the spot, so that the sixteen key
      // indices of this rarely taken branch are not kept in registers through the main loop)
      const int half = __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u)) >> 5;
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (first_key + 16 * (r / 8) + 8 * half + (r % 8) >= valid) s[r] = -INFINITY;
    }
    if constexpr (decltype(tracked)::value) {
      float mx = max3(s[0], s[1], s[2]);
#pragma unroll
      for (int r = 3; r < 15; r += 2) mx = max3(mx, s[r], s[r + 1]);
      mx = both_halves_max(fmaxf(mx, s[15]));
      if (__builtin_amdgcn_ballot_w64((mx - m_run) * scale_log2e > kRescaleThreshold) != 0) {
        const float m_new = fmaxf(m_run, mx);
        const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * scale_log2e);
        m_run = m_new;
        l_run *= alpha;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[db][r] *= alpha;
      }
    }
    bf16x8 pf[2];
    const float rs = exps(s, m_run * scale_log2e, pf);
    if constexpr (!decltype(tracked)::value)
      overflowed |= __builtin_amdgcn_ballot_w64(!(rs <= kBlockSumLimit));  // catches NaN too
    l_run += rs;
#pragma unroll
    for (int sl = 0; sl < 2; ++sl)
#pragma unroll
      for (int db = 0; db < 4; ++db)
        o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[sl][db], pf[sl], o[db], 0, 0, 0);
  };

  // Schedule.  LDS operands are always requested one phase before the MFMAs that use
  // them: V^T of a block ahead of its S MFMAs, K of the next block ahead of the softmax.
  // One barrier per tile, in the middle of the tile's second block: by then a wave has
  // finished every LDS read of the tile (so its stage may be refilled) and has waited for
  // its share of the next tile (so that tile may be read).  The fences stop the compiler
  // from sinking the requests back next to their uses.
  constexpr int kHalf = 32 * kRowBytes;
  bf16x8 kf[8], vf[2][4];
  // One tile (two blocks).  `ofs` / `next_ofs` are the byte offsets of this tile's and the
  // next tile's stage; in the main loop they are constants and fold into the LDS
  // instructions' offset fields.
  auto tile = [&](auto tracked, int t, int ofs, int next_ofs) __attribute__((always_inline)) {
    const int valid = t < n_tile1 ? len1 - t * TN : len2 - (t - n_tile1) * TN;
    const bool mask = valid < TN;
    // ---- first block of the tile
    fetch_vt(vf, ofs);
    __builtin_amdgcn_sched_barrier(0);
    f32x16 s = scores(kf);
    __builtin_amdgcn_sched_barrier(0);
    fetch_k(kf, ofs + kHalf);
    __builtin_amdgcn_sched_barrier(0);
    softmax_pv(tracked, s, vf, mask, 0, valid);
    // ---- second block
    __builtin_amdgcn_sched_barrier(0);
    fetch_vt(vf, ofs + kHalf);
    __builtin_amdgcn_sched_barrier(0);
    s = scores(kf);
    __builtin_amdgcn_sched_barrier(0);
    if (t + 1 < n_tile) {
      __builtin_amdgcn_s_waitcnt(0);
      __syncthreads();
#if !defined(SCALEKV_ABLATE_TRANSFER)
      if (t + 2 < n_tile) issue_tile(t + 2);
#endif
      fetch_k(kf, next_ofs);
    }
    __builtin_amdgcn_sched_barrier(0);
    softmax_pv(tracked, s, vf, mask, 32, valid);
  };
  // One pass over all tiles.  The first tile always follows its maxima: that is where
  // m_run comes from.
  // `first` (a std::bool_constant): the query rows are waiting in LDS and are taken into registers
  // before the second tile may overwrite them.
  auto pass = [&](auto tracked, auto first) __attribute__((always_inline)) {
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[db][r] = 0.f;
    m_run = -INFINITY;
    l_run = 0.f;
    issue_tile(0);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if constexpr (decltype(first)::value) {
#if defined(SCALEKV_TIMELINE)
      t_first_tile = __builtin_amdgcn_s_memrealtime();
#endif
      read_q();
      __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): the fragments are in registers, their space may be refilled
    }
    if (n_tile > 1) issue_tile(1);
    fetch_k(kf, 0);
    tile(std::true_type{}, 0, 0, kTileBytes);
    int t = 1;
    for (; t + 1 < n_tile; t += 2) {  // t odd: stage 1 then stage 0
      tile(tracked, t, kTileBytes, 0);
      tile(tracked, t + 1, 0, kTileBytes);
    }
    if (t < n_tile) tile(tracked, t, kTileBytes, 0);
    if constexpr (!decltype(tracked)::value) {
      // inf or NaN in an accumulator (huge values times large unchecked weights): repeat tracked
      bool bad = false;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) bad |= !(fabsf(o[db][r]) < INFINITY);
      overflowed |= __builtin_amdgcn_ballot_w64(bad);
    }
  };
  pass(std::false_type{}, std::true_type{});
  // every wave has left its last tile when the votes are in, so the stages may be refilled
  if (__syncthreads_or(overflowed != 0)) pass(std::true_type{}, std::false_type{});
  SCALEKV_STAMP(t_loop_end);

  // ---- append, first half: this workgroup's share of the second segment goes behind the first,
  // as 16-byte vectors.  The vectors of the first round (the whole share when it is at most 128
  // rows) are requested here, before the output is normalised and stored, so that their latency
  // hides behind that work; the registers of the operand fragments are free by now.
  const int ap_per = append ? (len2 + n_qtile - 1) / n_qtile : 0;
  const int ap_row0 = min(qtile * ap_per, len2);
  const int ap_vec = min(ap_per, len2 - ap_row0) * (kRowBytes / 16);  // per tensor
  const u32x4* ap_ks = (const u32x4*)(k2u + (long long)ap_row0 * kRowBytes);
  const u32x4* ap_vs = (const u32x4*)(v2u + (long long)ap_row0 * kRowBytes);
  u32x4 ap_a[8], ap_b[8];
  int ap_tid = tid;
  asm volatile("" : "+v"(ap_tid));  // keeps the requests below the tile loop: they must not be hoisted into it
  if (ap_vec > 0) {
    // (lanes past the end of the share re-read its last vector and store nothing)
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int i = min(u * 256 + ap_tid, ap_vec - 1);
      ap_a[u] = ap_ks[i];
      ap_b[u] = ap_vs[i];
    }
  }
  __builtin_amdgcn_sched_barrier(0);

  // ---- normalise and write.  A lane owns query column j, channels 32db + 8(r/4) + 4h + r%4:
  // sixteen 8-byte pieces of its output row.  Stored from there, every instruction of the wave
  // would touch 32 rows with 16 bytes each; instead the wave turns its 32 x 128 block round in
  // LDS (the tile stages are free: every wave has left its last tile; each wave uses a region of
  // its own, rows padded to 272 bytes against bank conflicts) and writes whole 256-byte rows,
  // 16 bytes per lane.
  {
    constexpr int kOutRowStride = kRowBytes + 16;
    unsigned char* const ostage = smem + wave * (32 * kOutRowStride);
    const float l_tot = both_halves_sum(l_run);
    const float inv = 1.f / l_tot;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const bf16x2 lo = {(__bf16)(o[db][4 * g] * inv), (__bf16)(o[db][4 * g + 1] * inv)};
        const bf16x2 hi = {(__bf16)(o[db][4 * g + 2] * inv), (__bf16)(o[db][4 * g + 3] * inv)};
        uint2 pk;
        pk.x = __builtin_bit_cast(uint32_t, lo);
        pk.y = __builtin_bit_cast(uint32_t, hi);
        *(uint2*)(ostage + j * kOutRowStride + 64 * db + 16 * g + 8 * h) = pk;
      }
    // the wave's own LDS writes have landed before it reads them back (same wave: no barrier)
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0)
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    unsigned char* const obase = (unsigned char*)(out + ((long long)unit * n_q + q_base) * D);
#pragma unroll
    for (int p = 0; p < 8; ++p) {
      const int r = 4 * p + (lane >> 4);
      const u32x4 val = *(const u32x4*)(ostage + r * kOutRowStride + 16 * (lane & 15));
      if (q_base + r < n_q) *(u32x4*)(obase + (long long)r * kRowBytes + 16 * (lane & 15)) = val;
    }
  }
  __builtin_amdgcn_sched_barrier(0);

  // ---- append, second half: store the first round, then whatever is left of a larger share.
  // The other workgroup on the compute unit keeps the matrix pipe busy meanwhile.
  if (ap_vec > 0) {
    u32x4* kd = (u32x4*)(const_cast<unsigned char*>(ku) + (long long)(len1 + ap_row0) * kRowBytes);
    u32x4* vd = (u32x4*)(const_cast<unsigned char*>(vu) + (long long)(len1 + ap_row0) * kRowBytes);
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int i = u * 256 + tid;
      if (i < ap_vec) {
        __builtin_nontemporal_store(ap_a[u], kd + i);
        __builtin_nontemporal_store(ap_b[u], vd + i);
      }
    }
    for (int i0 = 8 * 256; i0 < ap_vec; i0 += 8 * 256) {
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int i = i0 + u * 256 + tid;
        if (i < ap_vec) { ap_a[u] = ap_ks[i]; ap_b[u] = ap_vs[i]; }
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int i = i0 + u * 256 + tid;
        if (i < ap_vec) {
          __builtin_nontemporal_store(ap_a[u], kd + i);
          __builtin_nontemporal_store(ap_b[u], vd + i);
        }
      }
    }
  }
#if defined(SCALEKV_TIMELINE)
  __builtin_amdgcn_s_waitcnt(0);  // the workgroup's stores have been issued and acknowledged
  if (tid == 0 && blockIdx.x < kTimelineMaxWg) {
    unsigned long long* rec = g_timeline + (long long)blockIdx.x * kTimelineWords;
    rec[0] = t_start;
    rec[1] = t_first_tile;
    rec[2] = t_loop_end;
    rec[3] = __builtin_amdgcn_s_memrealtime();
    rec[4] = __builtin_amdgcn_s_getreg((31 << 11) | 4);  // HW_ID: compute unit, shader array, shader engine
    rec[5] = c_start;
    rec[6] = __builtin_readcyclecounter();
  }
#endif
}

}  // namespace

hipError_t launch_attend_pipe(int n_unit, int n_head, const void* q, int n_q, KvView k, KvView v,
                              int len1, const void* k2, const void* v2, int len2, bool append,
                              float sm_scale, void* out, hipStream_t stream, hipEvent_t start,
                              hipEvent_t stop) {
  static std::atomic<uint64_t> configured{0};
  const hipError_t e = allow_dynamic_lds((const void*)attend_pipe_kernel, kLdsBytes, configured);
  if (e != hipSuccess) return e;
  const float scale_log2e = sm_scale * 1.4426950408889634f;
  const int n_qtile = (n_q + BM - 1) / BM;
  const int n_wg = n_qtile * n_unit;
  if (start || stop)
    hipExtLaunchKernelGGL(attend_pipe_kernel, dim3(n_wg), dim3(256), kLdsBytes, stream, start, stop, 0,
                          (const uint16_t*)q, n_q, (uint16_t*)const_cast<void*>(k.ptr), k.seq_stride,
                          k.head_stride, (uint16_t*)const_cast<void*>(v.ptr), v.seq_stride,
                          v.head_stride, len1, (const uint16_t*)k2, (const uint16_t*)v2, len2,
                          append ? 1 : 0, n_head, n_qtile, n_wg, scale_log2e, (uint16_t*)out);
  else
    hipLaunchKernelGGL(attend_pipe_kernel, dim3(n_wg), dim3(256), kLdsBytes, stream,
                       (const uint16_t*)q, n_q, (uint16_t*)const_cast<void*>(k.ptr), k.seq_stride,
                       k.head_stride, (uint16_t*)const_cast<void*>(v.ptr), v.seq_stride,
                       v.head_stride, len1, (const uint16_t*)k2, (const uint16_t*)v2, len2,
                       append ? 1 : 0, n_head, n_qtile, n_wg, scale_log2e, (uint16_t*)out);
  return hipGetLastError();
}

}  // namespace scalekv

#if defined(SCALEKV_TIMELINE)
// Measurement-only builds: copies the records of workgroups 0 .. n_wg-1 of the most recent
// attend_pipe_kernel launch (kTimelineWords words each) to host memory.  Synchronises the device.
extern "C" int scalekv_timeline_read(unsigned long long* dst, int n_wg) {
  if (!dst || n_wg < 0 || n_wg > scalekv::kTimelineMaxWg) return -1;
  if (hipDeviceSynchronize() != hipSuccess) return -2;
  return hipMemcpyFromSymbol(dst, HIP_SYMBOL(scalekv::g_timeline),
                             sizeof(unsigned long long) * scalekv::kTimelineWords * n_wg) == hipSuccess ? 0 : -2;
}
#endif
