// Row-tile partial attention (paper Section 4, first paragraph: query rows attend to cache
// segments independently and emit a partial output plus normalizer; Section 2.1: the new
// tokens' self-attention is one more such partial).
//
// One workgroup = 8 wavefronts = 256 query rows of one kv head (row = (token, head in the
// GQA group)); wave w owns rows 32w..32w+31 (two waves per SIMD).  The workgroup walks the work
// item's kv tokens in tiles of 64, brought into LDS by direct global->LDS loads (16 bytes per
// lane, whole 256-byte rows, three tile buffers each for K and V).
//
// With 32x32x16 bf16 MFMA, per 32-token block and wave:
//   S^T[kv, row] = K[kv, :] . Q[row, :]      A = K block from LDS, B = Q (registers)
//   softmax numerators down the kv axis       lane l holds row l%32; its partner l^32 holds
//                                             the other half of that row's kv values
//   O^T[d, row] += V^T[d, kv] . P^T[kv, row]  A = V block read transposed from LDS, B = P
// Scores never leave registers between the two products.
//
// Fast path (completely filled tiles): the stream of 32-token blocks is software-pipelined
// inside each wave.  While the vector ALU turns the scores of block i into probabilities, the
// matrix unit computes the scores of block i+1 and accumulates block i-1; the three touch
// different registers, so neither unit waits for the other.  (Measured on gfx950: MFMA and
// vector-ALU instructions of the SAME wave overlap, those of two waves of a SIMD hardly do, and
// both kinds leave through one issue port, so the vector-ALU instruction count per MFMA is what
// the loop is trimmed for: LDS addresses are loop-invariant registers plus immediates -- the
// loop is unrolled over the three tile buffers -- and LDS operands are fetched three operand
// groups ahead of their MFMA.)  The exponent's reference point is fixed from the first block
// (any reference gives the same normalised result), which leaves the loop free of branches and
// of rescaling; if a row sum ends up above 2^60 or not finite -- scores far above the reference
// -- the workgroup discards the result and redoes the full tiles on the careful path.
// Careful path (tiles cut short by a slot's fill, tiles on the causal diagonal, and the
// redo): one tile at a time, masked, running maximum raised (and O rescaled) when a block
// exceeds it by more than 2^8.
// Repeated slots: a work item's list may name a slot several times (a multiset); the plan's tile
// lists hold each distinct slot once with log2 of its multiplicity, which is added to the exponent
// of the tile's probabilities (m equal keys weigh m exp(s) in numerator and denominator alike).
//
// Normalisation.  The probabilities enter the second product rounded to bf16, so O should be
// divided by the sum of the ROUNDED values -- it is then a convex combination of V rows whatever
// the rounding did to the weights -- while the normalizer that leaves the kernel (LSE) needs the
// sum of the unrounded fp32 values.  The kernel keeps the fp32 sum l and, beside it, a
// correction d ~= sum(rounded) - sum(unrounded); O is divided by l + d, LSE = m + ln l.
//  * careful path: d is exact (v_dot2c_f32_bf16 sums each packed pair as the matrix unit sees it);
//  * fast path: a second exact sum of every tile would cost 7 % of the kernel's time (the dot
//    instructions share the matrix pipeline), so a tile gets its exact d only if it raised some
//    lane's row sum by more than a sixteenth (one compare per tile; both blocks' packed
//    probabilities are still in registers then).  That is every tile at the start of a phase and
//    hardly any later on, unless a row is peaked: with a fixed exponent reference a dominant
//    probability is a rounded number like any other (with a running maximum it would be exactly
//    1), and its rounding is what the error of a peaked row consists of.  What remains is the
//    error of terms from tiles that added little, sum_j w_j e_j (v_j - O) with |e_j| <= 2^-8 over
//    those terms: no more than in a kernel that keeps a running maximum.
#include <type_traits>

#include "attn_common.h"

namespace tl {

namespace {

constexpr int kRG = 1;                                    // 32-row groups per wave
constexpr int kWaves = kRowTile / (32 * kRG);             // 8
constexpr int kThreads = 64 * kWaves;                     // 512
constexpr int kChunks = kKvTile * 16 / kThreads;          // 16-byte chunks per thread per K (or V) tile: 2
constexpr int kChunkRows = kThreads / 16;                 // rows covered by one chunk index: 32
constexpr int kKS = kHeadDim;        // K row stride in LDS (bf16): unpadded, 16-byte chunks swizzled
constexpr int kVS = kHeadDim;        // V row stride in LDS (bf16): unpadded, 16-byte chunks swizzled
constexpr int kKTile = kKvTile * kKS;
constexpr int kVTile = kKvTile * kVS;
constexpr int kIdxRing = 512;        // tile-base entries kept in LDS (ring over the work item's tile list)
constexpr int kBufs = 3;             // LDS tile buffers: K(t+2) and V(t+1) stream in while tile t is computed
constexpr size_t kLdsBytes = (size_t)kBufs * (kKTile + kVTile) * sizeof(uint16_t) + (2 * kIdxRing + 4) * sizeof(int32_t);
constexpr float kRescaleLog2 = 8.0f;             // careful path: raise the maximum when exceeded by 2^8
constexpr float kFastPathLimit = 1.152921504606846976e18f;  // 2^60
constexpr int kDmaPerWave = 16 / kWaves;                  // direct-load instructions per wave per K (or V) tile
constexpr float kExactCorrectionGrowth = 1.0625f;   // fast path: growth of a lane's row sum over one tile from which the tile's correction is exact
constexpr int kDepth = 3;            // LDS operands in flight ahead of the MFMA that uses them (ring of kDepth + 1)

// Lanes l and l^32 exchange x: returns {own, partner} in some order.  The swap instruction
// exchanges the upper half of its first operand with the lower half of its second; the second
// copy of x is laundered through an empty asm so that the compiler treats the two operands
// (and hence the two results) as unrelated values.
__device__ __forceinline__ void xor32_pair(float x, float& r0, float& r1) {
  unsigned a = __builtin_bit_cast(unsigned, x), b = a;
  asm volatile("" : "+v"(b));
  auto r = __builtin_amdgcn_permlane32_swap(a, b, false, false);
  unsigned u0 = r[0], u1 = r[1];
  asm volatile("" : "+v"(u0), "+v"(u1));
  r0 = __builtin_bit_cast(float, u0);
  r1 = __builtin_bit_cast(float, u1);
}

__device__ __forceinline__ float xor32_max(float x) {
  float r0, r1;
  xor32_pair(x, r0, r1);
  return fmaxf(r0, r1);
}

__device__ __forceinline__ float xor32_sum(float x) {
  float r0, r1;
  xor32_pair(x, r0, r1);
  return r0 + r1;
}

// a packed bf16 operand held as four 32-bit words, so that a pair of elements is one register write
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
// word `pair` (0..3) of a packed operand := (a, b) rounded to bf16
__device__ __forceinline__ void set_pair(u32x4& p, int pair, float a, float b) {
  typedef float f32x2_t __attribute__((ext_vector_type(2)));
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  p[pair] = __builtin_bit_cast(unsigned, __builtin_convertvector(f32x2_t{a, b}, bf16x2_t));
}

__device__ __forceinline__ float max16(const f32x16& s) {
  float a = fmaxf(fmaxf(s[0], s[1]), s[2]);
  float b = fmaxf(fmaxf(s[3], s[4]), s[5]);
  float c = fmaxf(fmaxf(s[6], s[7]), s[8]);
  float d = fmaxf(fmaxf(s[9], s[10]), s[11]);
  float e = fmaxf(fmaxf(s[12], s[13]), s[14]);
  return fmaxf(fmaxf(fmaxf(a, b), fmaxf(c, d)), fmaxf(e, s[15]));
}

// MODE 0: pool work item (tile lists) -> partial.  MODE 1: causal block of the new tokens ->
// partial.  MODE 2: both in one pass -- the row tile walks its request's pool tiles, then the
// new tokens up to its own rows -- and writes the final, normalised output: such rows have one
// partial, so they need no merge.
template <int MODE, int VREAD>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2 / kRG, 2 / kRG))) void row_tile_attn_kernel(const AttnArgs a) {
  extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
  uint16_t* lds_k = lds;                 // [kBufs][64][kKS]
  uint16_t* lds_v = lds + kBufs * kKTile;    // [kBufs][64][kVS]
  int32_t* lds_idx = (int32_t*)(lds + kBufs * (kKTile + kVTile));   // [kIdxRing]
  float* lds_lm = (float*)(lds_idx + kIdxRing);   // [kIdxRing] log2(multiplicity) of the same tiles
  int32_t* lds_flag = lds_idx + 2 * kIdxRing;

  const int g = blockIdx.x % a.kv_heads;
  const Work wk = a.work[blockIdx.x / a.kv_heads];
  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63, l32 = lane & 31, h = lane >> 5;
  const int G = a.group;
  const int first_token = a.tok[wk.tok_off];   // causal work: tokens of a tile are consecutive
  constexpr bool kHasPool = MODE != 1, kHasSelf = MODE != 0;
  // K/V of the new tokens: the launch's main K/V for the causal block alone, the second pair when fused
  const uint16_t* self_k = MODE == 2 ? a.k2 : a.k;
  const uint16_t* self_v = MODE == 2 ? a.v2 : a.v;

  // per row group: this lane's row, its token and head
  int tok_local[kRG], head_j[kRG], token[kRG];
  bool row_ok[kRG];
#pragma unroll
  for (int rg = 0; rg < kRG; ++rg) {
    const int row = wave * (32 * kRG) + 32 * rg + l32;
    tok_local[rg] = row / G;                    // any group size: the last 256 % G rows of a tile are idle
    head_j[rg] = row - tok_local[rg] * G;
    row_ok[rg] = tok_local[rg] < wk.n_tok;
    token[rg] = row_ok[rg] ? a.tok[wk.tok_off + tok_local[rg]] : -1;
  }

  // Q as the B operand: lane holds its row, head-dim elements 16 s + 8 h .. +7 of step s
  bf16x8 qreg[kRG][8];
#pragma unroll
  for (int rg = 0; rg < kRG; ++rg) {
    const uint4* qp =
        (const uint4*)(a.q + ((size_t)(row_ok[rg] ? token[rg] : 0) * a.q_heads + g * G + head_j[rg]) * kHeadDim);
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      uint4 u = make_uint4(0, 0, 0, 0);
      if (row_ok[rg]) u = qp[2 * s + h];
      qreg[rg][s] = as_bf16x8(u);
    }
  }

  // O^T accumulators: o[rg][d][r] = channel 32 d + 8 (r/4) + 4 h + r%4 of the lane's row in group rg
  f32x16 o[kRG][4];
  float m_ref[kRG];   // reference point of the exponent (raw score units), -inf before any key
  float l_run[kRG];   // this lane's share of sum exp(s - m_ref), unrounded (-> LSE)
  float lr_run[kRG];  // correction: (sum of the values as rounded to bf16 for the second product) - (unrounded sum)
  auto reset_state = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int rg = 0; rg < kRG; ++rg) {
#pragma unroll
      for (int d = 0; d < 4; ++d)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[rg][d][r] = 0.f;
      m_ref[rg] = -INFINITY;
      l_run[rg] = 0.f;
      lr_run[rg] = 0.f;
    }
  };
  reset_state();
  const float c = a.scale_log2e;

  // which tiles are full (no masking needed for any row of this workgroup)
  const int nf_pool = kHasPool ? wk.n_full : 0, np_pool = kHasPool ? wk.n_part : 0;
  int nf_self = 0, np_self = 0;
  if (kHasSelf) {
    nf_self = (first_token - wk.kv_off + 1) / kKvTile;
    np_self = (wk.kv_len + kKvTile - 1) / kKvTile - nf_self;
  }
  // first kv row of a full pool tile comes from the item's tile list, kept in an LDS ring (a
  // dependent global load per iteration would stall the wave); that of a full tile of new tokens
  // is arithmetic
  auto ring_fill = [&](int first, int count) __attribute__((always_inline)) {   // entries [first, first+count) of the list, clipped
    for (int i = first + tid; i < first + count && i < nf_pool; i += kThreads)
    {
      lds_idx[i & (kIdxRing - 1)] = a.tile_base[wk.full_off + i];
      if (a.tile_lm) lds_lm[i & (kIdxRing - 1)] = a.tile_lm[wk.full_off + i];
    }
  };

  // ---- careful path staging (global -> registers -> LDS): kChunks chunks of 16 B per thread per
  // tile, for K and for V; chunk i of a thread: tile row (tid >> 4) + kChunkRows i, 16-byte column tid & 15
  const size_t kv_row = (size_t)a.kv_heads * kHeadDim;
  const int c_tr = tid >> 4, c_part = tid & 15;
  // address = (tile's first row: workgroup-uniform, 64-bit, scalar registers) + (this thread's
  // constant 32-bit offset inside a tile), so that a tile costs no per-lane 64-bit arithmetic
  const unsigned lane_off0 = (unsigned)((c_tr * kv_row + (size_t)g * kHeadDim) * 2 + c_part * 16);
  const unsigned chunk_step = (unsigned)(kChunkRows * kv_row * 2);
  auto chunk_ptr = [&](const uint16_t* src, int base, int i) __attribute__((always_inline)) -> const uint4* {
    const char* tile = (const char*)src + (size_t)__builtin_amdgcn_readfirstlane(base) * (kv_row * 2);
    return (const uint4*)(tile + (lane_off0 + chunk_step * i));
  };
  auto lds_chunk_k = [&](uint16_t* tile, int i) __attribute__((always_inline)) -> uint4* {
    const int r_ = c_tr + kChunkRows * i;
    return (uint4*)&tile[r_ * kKS + 8 * (c_part ^ (r_ & 15))];
  };
  auto lds_chunk_v = [&](uint16_t* tile, int i) __attribute__((always_inline)) -> uint4* {
    const int r_ = c_tr + kChunkRows * i;
    return (uint4*)&tile[r_ * kVS + 8 * (c_part ^ (4 * (r_ & 3)))];
  };
  // ---- fast path staging: direct global -> LDS load of a whole tile.  A tile is 16 wave
  // instructions; wave w issues instructions w + kWaves u, instruction i filling rows 4 i .. 4 i + 3;
  // lane L lands at row 4 i + L / 16, position L % 16, so it fetches the logical chunk that belongs there
  unsigned dma_off_k[kDmaPerWave], dma_off_v[kDmaPerWave];
#pragma unroll
  for (int u = 0; u < kDmaPerWave; ++u) {
    const int r_ = 4 * (wave + kWaves * u) + (lane >> 4), pos = lane & 15;
    dma_off_k[u] = (unsigned)((r_ * kv_row + (size_t)g * kHeadDim) * 2 + 16 * (pos ^ (r_ & 15)));
    dma_off_v[u] = (unsigned)((r_ * kv_row + (size_t)g * kHeadDim) * 2 + 16 * (pos ^ (4 * (r_ & 3))));
  }
  // (issued as inline assembly: the compiler does not see these loads, so it puts no wait for them
  // in front of the LDS reads that follow; dma_wait() before the iteration's barrier is the wait)
  const unsigned lds_base_addr = __builtin_amdgcn_readfirstlane((unsigned)(size_t)(__attribute__((address_space(3))) void*)lds);
  const unsigned dma_wave_off = __builtin_amdgcn_readfirstlane(wave) * (4 * kHeadDim * 2);
  static_assert(kDmaPerWave == 2, "dma_tile issues exactly two direct loads per wave");
  auto dma_tile = [&](const uint16_t* src, int base, uint16_t* tile, const unsigned (&off)[kDmaPerWave]) {
    const char* trow = (const char*)src + (size_t)__builtin_amdgcn_readfirstlane(base) * (kv_row * 2);
    const unsigned dst0 = lds_base_addr + (unsigned)(tile - lds) * 2u + dma_wave_off;
    const unsigned dst1 = dst0 + (unsigned)(kWaves * 4 * kHeadDim) * 2u;
    // address = wave-uniform 64-bit tile base (scalar registers) + this lane's constant 32-bit offset;
    // the LDS destination travels in M0, which the compiler does not accept as a clobber: its value
    // is put back before the statement ends
    unsigned saved_m0;
    asm volatile(
        "s_mov_b32 %[sv], m0\n\t"
        "s_mov_b32 m0, %[d0]\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %[o0], %[b]\n\t"
        "s_mov_b32 m0, %[d1]\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %[o1], %[b]\n\t"
        "s_mov_b32 m0, %[sv]"
        : [sv] "=&s"(saved_m0)
        : [o0] "v"(off[0]), [o1] "v"(off[1]), [d0] "s"(dst0), [d1] "s"(dst1), [b] "s"(trow)
        : "memory");
  };
  // wait for all of this wave's direct loads (vmcnt(0); the other counters are left alone so that
  // LDS operand reads already in flight stay in flight)
  auto dma_wait = [&]() __attribute__((always_inline)) { __builtin_amdgcn_s_waitcnt(0x0F70); };

  // ---- building blocks ----
  // LDS tiles are unpadded rows of 256 B = 16 chunks of 16 B, written by direct global->LDS
  // loads (one wave instruction fills 4 rows contiguously).  Bank conflicts are avoided by
  // storing logical chunk c of row r at position c ^ swz(r):
  //   K: swz(r) = r & 15      -> the 16 rows that 16 lanes read at one logical chunk hit 16 positions
  //   V: swz(r) = 4 (r & 3)   -> the 4 rows x 4 chunks of one transposing read hit 16 positions
  auto k_operand = [&](const uint16_t* kt, int hb, int s8) __attribute__((always_inline)) -> bf16x8 {
    return *(const bf16x8*)&kt[(32 * hb + l32) * kKS + 8 * ((2 * s8 + h) ^ (l32 & 15))];
  };
  // V^T operand of accumulation step (sp, d) of block hb: channels 32 d .. 32 d + 31, block
  // tokens 16 sp + {4h..4h+3, 8+4h..8+4h+3} -- the order in which the score registers hold them
  auto v_operand = [&](const uint16_t* vt, int hb, int sp, int d) __attribute__((always_inline)) -> bf16x8 {
    const int kvb = 32 * hb + 16 * sp;
    if (VREAD == 0) {
      const int blk = lane >> 4, jj = lane & 15;
      // logical chunk 4 d + 2 (blk & 1) + (jj & 3) / 2 of row kvb + 4 (blk >> 1) + jj / 4 (row & 3 = jj / 4)
      const int chunk = (4 * d + 2 * (blk & 1) + ((jj & 3) >> 1)) ^ (4 * (jj >> 2));
      const uint16_t* p = vt + (kvb + 4 * (blk >> 1) + (jj >> 2)) * kVS + 8 * chunk + 4 * (jj & 1);
      return join_tr(lds_read_tr(p), lds_read_tr(p + 8 * kVS));
    } else {
      s16x8 t;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int r_ = kvb + 8 * (e >> 2) + 4 * h + (e & 3), col = 32 * d + l32;
        t[e] = (short)vt[r_ * kVS + 8 * ((col >> 3) ^ (4 * (r_ & 3))) + (col & 7)];
      }
      return __builtin_bit_cast(bf16x8, t);
    }
  };
  // scores of block hb of the K tile at kt, for every row group of the wave
  auto qk_block = [&](const uint16_t* kt, int hb, f32x16 (&s)[kRG]) {
    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s8 = 0; s8 < 8; ++s8) {
      const bf16x8 ak = k_operand(kt, hb, s8);
#pragma unroll
      for (int rg = 0; rg < kRG; ++rg)
        s[rg] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ak, qreg[rg][s8], s8 == 0 ? zero : s[rg], 0, 0, 0);
    }
  };
  // probabilities of a block against the reference: p = 2^(c (s - m_ref)); B operands pb[sp]
  // hold registers 8 sp .. 8 sp + 7
  auto exp_block = [&](int rg, f32x16& s, bf16x8 (&pb)[2], float lm) {
    const float mc = m_ref[rg] * c - lm;   // lm = log2(times the tile's slot is listed): p = m 2^(c (s - m_ref))
#pragma unroll
    for (int r = 0; r < 16; ++r) s[r] = fast_exp2(fmaf(s[r], c, -mc));
    pb[0] = pack_bf16x8(s[0], s[1], s[2], s[3], s[4], s[5], s[6], s[7]);
    pb[1] = pack_bf16x8(s[8], s[9], s[10], s[11], s[12], s[13], s[14], s[15]);
    // the normalizer (LSE) sums the probabilities before their rounding to bf16, in fp32 ...
    float lsum = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) lsum += s[r];
    l_run[rg] += lsum;
    // ... and O is divided by the sum of what the matrix unit is given: lr = that sum, exactly
    float lr = 0.f;
#pragma unroll
    for (int sp = 0; sp < 2; ++sp) {
      const u32x4 w = __builtin_bit_cast(u32x4, pb[sp]);
#pragma unroll
      for (int i = 0; i < 4; ++i) lr = add_bf16_pair(lr, w[i]);
    }
    lr_run[rg] += lr - lsum;
  };
  auto pv_block = [&](const uint16_t* vt, int hb, const bf16x8 (&pb)[kRG][2]) {
#pragma unroll
    for (int sp = 0; sp < 2; ++sp)
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        const bf16x8 av = v_operand(vt, hb, sp, d);
#pragma unroll
        for (int rg = 0; rg < kRG; ++rg)
          o[rg][d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, pb[rg][sp], o[rg][d], 0, 0, 0);
      }
  };
  // careful path: raise the reference maximum if the block's scores exceed it by too much
  auto maybe_rescale = [&](int rg, const f32x16& s) __attribute__((always_inline)) {
    const float mx = xor32_max(max16(s));
    const bool need = (mx - m_ref[rg]) * c > kRescaleLog2 || m_ref[rg] == -INFINITY;
    if (__builtin_amdgcn_ballot_w64(need) != 0) {
      const float m_new = fmaxf(m_ref[rg], mx);
      const float alpha = (m_new == -INFINITY) ? 1.f : fast_exp2((m_ref[rg] - m_new) * c);
      m_ref[rg] = m_new;
      l_run[rg] *= alpha;
      lr_run[rg] *= alpha;
#pragma unroll
      for (int d = 0; d < 4; ++d)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[rg][d][r] *= alpha;
    }
  };
  // careful path: one tile (rows beyond `valid` hidden; causal work also hides later tokens)
  auto careful_tile = [&](auto SELF, const uint16_t* src_k, const uint16_t* src_v, int base, int valid, float lm) __attribute__((always_inline)) {
    constexpr bool CAUSAL = decltype(SELF)::value;
    {
      // rows beyond `valid` are written as zero: 0 * garbage cannot make NaN
      const uint4 z = make_uint4(0, 0, 0, 0);
#pragma unroll
      for (int i = 0; i < kChunks; ++i) {
        const bool in = c_tr + kChunkRows * i < valid;
        const uint4 kk = in ? *chunk_ptr(src_k, base, i) : z;
        const uint4 vv = in ? *chunk_ptr(src_v, base, i) : z;
        *lds_chunk_k(lds_k, i) = kk;
        *lds_chunk_v(lds_v, i) = vv;
      }
    }
    __syncthreads();
#pragma unroll 1
    for (int hb = 0; hb < 2; ++hb) {
      if (32 * hb >= valid) break;              // uniform
      f32x16 s[kRG];
      qk_block(lds_k, hb, s);
      bf16x8 pb[kRG][2];
#pragma unroll
      for (int rg = 0; rg < kRG; ++rg) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int kv = 32 * hb + 8 * (r >> 2) + 4 * h + (r & 3);
          bool hide = kv >= valid;
          if (CAUSAL) hide = hide || (base + kv > token[rg]);
          if (hide) s[rg][r] = -INFINITY;
        }
        maybe_rescale(rg, s[rg]);
        if (m_ref[rg] == -INFINITY) {
          // every key so far is hidden from this row: probabilities are zero
          pb[rg][0] = pack_bf16x8(0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f);
          pb[rg][1] = pb[rg][0];
        } else {
          exp_block(rg, s[rg], pb[rg], lm);
        }
      }
      pv_block(lds_v, hb, pb);
    }
    __syncthreads();
  };

  // ======================= fast path: full tiles, software-pipelined by 32-token block =======================
  // Steady state, per block i of the tile stream (two blocks per tile = two steps per iteration):
  //   MFMA:  scores(block i+1)  and  accumulate(block i-1)      16 kRG MFMA each
  //   VALU:  probabilities(block i)
  // An iteration is 32 operand groups: one LDS operand (a K fragment, or a transposed V fragment)
  // and the kRG MFMAs that use it, plus a slice of the probabilities; the operand is fetched
  // kDepth groups earlier.  sched_barrier(0) after every group keeps the compiler to this order.
  // Runs the n_full (> 0) full tiles of one phase; have_ref says whether the exponent's reference
  // point exists already.  Returns false if the result overflowed and has to be discarded.
  auto fast_phase = [&](auto SELF, const uint16_t* src_k, const uint16_t* src_v, const int n_full, const bool have_ref) __attribute__((always_inline)) -> bool {
    constexpr bool CAUSAL = decltype(SELF)::value;
    auto full_base = [&](int t) __attribute__((always_inline)) -> int { return CAUSAL ? wk.kv_off + kKvTile * t : lds_idx[t & (kIdxRing - 1)]; };
    if (tid == 0) *lds_flag = 0;
    if (!CAUSAL) ring_fill(0, kIdxRing);
    {
      // "tile -1" (V buffer kBufs-1) is multiplied by zero probabilities in the first iteration
      const uint4 z = make_uint4(0, 0, 0, 0);
      for (int i = tid; i < kVTile / 8; i += kThreads) ((uint4*)(lds_v + (kBufs - 1) * kVTile))[i] = z;
    }
    __syncthreads();
    dma_tile(src_k, full_base(0), lds_k, dma_off_k);
    dma_tile(src_v, full_base(0), lds_v, dma_off_v);
    if (n_full > 1) dma_tile(src_k, full_base(1), lds_k + kKTile, dma_off_k);
    dma_wait();
    __syncthreads();

    float l_prev[kRG];                  // the lane's row sum before the current tile
#pragma unroll
    for (int rg = 0; rg < kRG; ++rg) l_prev[rg] = l_run[rg];
    f32x16 s0[kRG], s1[kRG];            // scores of block 0 / block 1 of a tile (then their probabilities)
    u32x4 p0[kRG][2], p1[kRG][2];       // packed probabilities (bf16 pairs)
    qk_block(lds_k, 0, s0);
    float mc[kRG];
#pragma unroll
    for (int rg = 0; rg < kRG; ++rg) {
      if (!have_ref) m_ref[rg] = xor32_max(max16(s0[rg]));   // reference: the first block's row maximum
      mc[rg] = m_ref[rg] * c;
      p1[rg][0] = u32x4{0u, 0u, 0u, 0u};
      p1[rg][1] = p1[rg][0];
      p0[rg][0] = p0[rg][1] = p1[rg][0];
    }

    // operand group g of an iteration (0..31): step g / 16; even = K operand (head-dim step g%16 / 2),
    // odd = V operand ((sp, d) = g%16 / 2).  Step 0: K(t, block 1), V(t-1, block 1); step 1:
    // K(t+1, block 0), V(t, block 0).
    auto operand = [&](int gq, const uint16_t* k_t, const uint16_t* k_n, const uint16_t* v_p, const uint16_t* v_t) __attribute__((always_inline)) -> bf16x8 {
      const int step = gq >> 4, idx = (gq & 15) >> 1;
      if ((gq & 1) == 0) return k_operand(step == 0 ? k_t : k_n, step == 0 ? 1 : 0, idx);
      return v_operand(step == 0 ? v_p : v_t, step == 0 ? 1 : 0, idx >> 2, idx & 3);
    };
    bf16x8 ring[kDepth + 1];
    {
      const uint16_t* k_t = lds_k;
      const uint16_t* k_n = lds_k + kKTile;
      const uint16_t* v_p = lds_v + (kBufs - 1) * kVTile;
      const uint16_t* v_t = lds_v;
#pragma unroll
      for (int gq = 0; gq < kDepth; ++gq) ring[gq] = operand(gq, k_t, k_n, v_p, v_t);
    }
    __builtin_amdgcn_sched_barrier(0);

    // first rows of the tiles that the coming iteration streams in, K(t+2) and V(t+1) (indices past
    // the end are clamped: such a value is never used for a load)
    int base_k = full_base(min(2, n_full - 1)), base_v = full_base(min(1, n_full - 1));
    // log2 of the multiplicity of the tile whose probabilities the coming iteration forms
    // (a.tile_lm is null when no list of the plan names a slot twice: then nothing is read)
    auto tile_lm = [&](int t) __attribute__((always_inline)) -> float { return CAUSAL || !a.tile_lm ? 0.f : lds_lm[t & (kIdxRing - 1)]; };
    float lm_cur = tile_lm(0);
    // one tile; kb = t % kBufs is a compile-time constant (the loop below is unrolled kBufs times),
    // so that every LDS address is a loop-invariant per-lane register plus an immediate offset
    auto tile_iteration = [&](auto KB, int t) __attribute__((always_inline)) {
      constexpr int kb = decltype(KB)::value;
      constexpr int kb1 = kb + 1 == kBufs ? 0 : kb + 1;
      constexpr int km1 = kb == 0 ? kBufs - 1 : kb - 1;
      constexpr int km2 = km1 == 0 ? kBufs - 1 : km1 - 1;
      const uint16_t* k_t = lds_k + kb * kKTile;     // K(t), V(t)
      const uint16_t* v_t = lds_v + kb * kVTile;
      const uint16_t* k_n = lds_k + kb1 * kKTile;    // K(t+1), V(t+1)
      const uint16_t* v_n = lds_v + kb1 * kVTile;
      const uint16_t* v_p = lds_v + km1 * kVTile;    // V(t-1)
      if (!CAUSAL && t > 0 && (t & (kIdxRing / 2 - 1)) == 0) ring_fill(t + kIdxRing / 2, kIdxRing / 2);
      // K(t+2) replaces K(t-1), V(t+1) replaces V(t-2): both were last read before the previous barrier
      if (t + 2 < n_full) dma_tile(src_k, base_k, lds_k + km1 * kKTile, dma_off_k);
      if (t + 1 < n_full) dma_tile(src_v, base_v, lds_v + km2 * kVTile, dma_off_v);
      int base_k_next = 0, base_k_next_v = 0;
      float lm_next = 0.f;
      float nmc[kRG];               // exponent offset of this tile's probabilities: p = m 2^(c (s - m_ref))
#pragma unroll
      for (int rg = 0; rg < kRG; ++rg) nmc[rg] = lm_cur - mc[rg];
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int gq = 0; gq < 32; ++gq) {
        const int step = gq >> 4, gi = gq & 15, idx = gi >> 1;
        // read early and made wave-uniform well before the next iteration's start needs it
        if (gq == 6) {
          base_k_next_v = full_base(min(t + 3, n_full - 1));
          lm_next = tile_lm(min(t + 1, n_full - 1));
        }
        if (gq == 20) {
          base_k_next = __builtin_amdgcn_readfirstlane(base_k_next_v);
        }
        // fetch ahead (the first groups of the next iteration read tiles that are already resident)
        {
          const int gp = gq + kDepth;
          ring[gp % (kDepth + 1)] = gp < 32 ? operand(gp, k_t, k_n, v_p, v_t) : operand(gp - 32, k_n, k_n, v_t, v_n);
        }
        const bf16x8 x = ring[gq % (kDepth + 1)];
        // kRG MFMAs share the operand; each is followed by its own slice of the probabilities of
        // the block whose scores are complete (one element), so that matrix and vector
        // instructions alternate in the wave's instruction stream
#pragma unroll
        for (int j = 0; j < kRG; ++j) {
          if ((gi & 1) == 0) {
            const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            if (step == 0) s1[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, qreg[j][idx], idx == 0 ? zero : s1[j], 0, 0, 0);
            else s0[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, qreg[j][idx], idx == 0 ? zero : s0[j], 0, 0, 0);
          } else {
            const int sp = idx >> 2, d = idx & 3;
            o[j][d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, __builtin_bit_cast(bf16x8, step == 0 ? p1[j][sp] : p0[j][sp]), o[j][d], 0, 0, 0);
          }
          __builtin_amdgcn_sched_barrier(0);   // the MFMA first, then its slice (+0.8 % over leaving the order to the compiler)
          const int e = gi * kRG + j, rg = e >> 4, r = e & 15;
          f32x16& s = step == 0 ? s0[rg] : s1[rg];
          s[r] = fast_exp2(fmaf(s[r], c, nmc[rg]));
          // The row sum and the packing to bf16 trail the exponentials by one element / one pair, so
          // that every slice carries the same few vector instructions (a burst of eight adds and
          // four converts in one place would hold up the MFMA behind it) and none of them waits
          // for the exponential issued just before it.
          u32x4 (&pp)[2] = step == 0 ? p0[rg] : p1[rg];
          if (r >= 1) l_run[rg] += s[r - 1];
          if (r >= 2 && (r & 1) == 0) set_pair(pp[(r - 2) >> 3], ((r - 2) & 7) >> 1, s[r - 2], s[r - 1]);
          if (r == 15) {
            l_run[rg] += s[15];
            set_pair(pp[1], 3, s[14], s[15]);
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      // A tile that raised some lane's row sum by more than a sixteenth gets its exact correction: the sum
      // of its 32 probabilities per lane as rounded (both blocks' packed values are still in registers)
      // minus what they added to the row sum.  Rare after the first few tiles of a phase.
      {
        bool big = false;
#pragma unroll
        for (int rg = 0; rg < kRG; ++rg) big = big || l_run[rg] > kExactCorrectionGrowth * l_prev[rg];
        if (__builtin_amdgcn_ballot_w64(big) != 0) {
#pragma unroll
          for (int rg = 0; rg < kRG; ++rg) {
            float lr = 0.f;
#pragma unroll
            for (int sp = 0; sp < 2; ++sp)
#pragma unroll
              for (int i = 0; i < 4; ++i) {
                lr = add_bf16_pair(lr, p0[rg][sp][i]);
                lr = add_bf16_pair(lr, p1[rg][sp][i]);
              }
            lr_run[rg] += lr - (l_run[rg] - l_prev[rg]);
          }
        }
#pragma unroll
        for (int rg = 0; rg < kRG; ++rg) l_prev[rg] = l_run[rg];
      }
      // this wave's share of K(t+2) / V(t+1) has landed; after the barrier everybody's has, and
      // everybody is done reading K(t) block 1 and V(t-1), the buffers the next loads overwrite
      dma_wait();
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");   // no memory access moves across the barrier at compile time
      __builtin_amdgcn_sched_barrier(0);
      base_v = base_k;
      base_k = base_k_next;
      lm_cur = lm_next;
    };
    {
      int t = 0;
      while (true) {
        tile_iteration(std::integral_constant<int, 0>{}, t);
        if (++t == n_full) break;
        tile_iteration(std::integral_constant<int, 1>{}, t);
        if (++t == n_full) break;
        tile_iteration(std::integral_constant<int, 2>{}, t);
        if (++t == n_full) break;
      }
    }
    // drain: accumulate block 1 of the last tile
    {
      bf16x8 pl[kRG][2];
#pragma unroll
      for (int rg = 0; rg < kRG; ++rg) {
        pl[rg][0] = __builtin_bit_cast(bf16x8, p1[rg][0]);
        pl[rg][1] = __builtin_bit_cast(bf16x8, p1[rg][1]);
      }
      pv_block(lds_v + ((n_full - 1) % kBufs) * kVTile, 1, pl);
    }

    // did the fixed reference hold?  (row sums are sums of positive terms: one huge term shows)
    bool bad = false;
#pragma unroll
    for (int rg = 0; rg < kRG; ++rg) bad = bad || !(l_run[rg] < kFastPathLimit);
    if (__builtin_amdgcn_ballot_w64(bad) != 0 && lane == 0) *lds_flag = 1;
    __syncthreads();
    const bool redo = *lds_flag != 0;
    __syncthreads();
    return !redo;
  };

  // ======================= the same tiles on the careful path =======================
  const std::false_type kPoolPhase{};
  const std::true_type kSelfPhase{};
  auto careful_pool_full = [&]() __attribute__((always_inline)) {
    ring_fill(0, kIdxRing);
    __syncthreads();
    for (int t = 0; t < nf_pool; ++t) {
      if (t > 0 && (t & (kIdxRing / 2 - 1)) == 0) {
        __syncthreads();
        ring_fill(t + kIdxRing / 2, kIdxRing / 2);
        __syncthreads();
      }
      careful_tile(kPoolPhase, a.k, a.v, lds_idx[t & (kIdxRing - 1)], kKvTile, a.tile_lm ? lds_lm[t & (kIdxRing - 1)] : 0.f);
    }
  };
  auto careful_pool_part = [&]() __attribute__((always_inline)) {   // tiles cut short by a slot's fill
    for (int pt = 0; pt < np_pool; ++pt)
      careful_tile(kPoolPhase, a.k, a.v, a.part_tile[2 * (wk.part_off + pt)], a.part_tile[2 * (wk.part_off + pt) + 1],
                   a.part_lm ? a.part_lm[wk.part_off + pt] : 0.f);
  };
  auto careful_self = [&](int first_tile, int n_tiles) __attribute__((always_inline)) {
    for (int t = first_tile; t < first_tile + n_tiles; ++t)
      careful_tile(kSelfPhase, self_k, self_v, wk.kv_off + kKvTile * t, min(kKvTile, wk.kv_len - kKvTile * t), 0.f);
  };

  // ======================= the phases =======================
  if constexpr (kHasPool) {
    const bool ok = nf_pool > 0 ? fast_phase(kPoolPhase, a.k, a.v, nf_pool, false) : true;
    if (!ok) {
      reset_state();
      careful_pool_full();
    }
    careful_pool_part();
  }
  if constexpr (kHasSelf) {
    const bool have_ref = kHasPool && nf_pool + np_pool > 0;
    const bool ok = nf_self > 0 ? fast_phase(kSelfPhase, self_k, self_v, nf_self, have_ref) : true;
    if (!ok) {   // everything so far is spoilt: start again, carefully
      reset_state();
      if constexpr (kHasPool) {
        careful_pool_full();
        careful_pool_part();
      }
      careful_self(0, nf_self);
    }
    careful_self(nf_self, np_self);   // tiles on the diagonal
  }

  // ---- epilogue: normalise, LSE, store ----
#pragma unroll
  for (int rg = 0; rg < kRG; ++rg) {
    const float l_tot = xor32_sum(l_run[rg]);
    const float lr_tot = l_tot + xor32_sum(lr_run[rg]);
    if (row_ok[rg]) {
      float inv = lr_tot > 0.f ? 1.f / lr_tot : 0.f;
      const int head = g * G + head_j[rg];
      float lse_val = l_tot > 0.f ? m_ref[rg] * a.scale + __logf(l_tot) : -INFINITY;
      if (MODE == 2 && wk.n_prior > 0) {
        // One-pass tail: the row's partials in the work items above it (shared runs, computed by an
        // earlier launch) are merged in with the rule of the merge kernel,
        //   M = max LSE_j, w_j = exp(LSE_j - M), O = sum w_j O_j / sum w_j, LSE = M + ln sum w_j,
        // taken one partial at a time: (M, W, acc) <- (max(M, L), W e^(M-M') + e^(L-M'), acc e^(M-M') + O_j e^(L-M')).
        // The accumulators are brought to their normalised values first.
#pragma unroll
        for (int d = 0; d < 4; ++d)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[rg][d][r] *= inv;
        float M = lse_val, W = lse_val > -INFINITY ? 1.f : 0.f;
        const int tok_in_req = wk.out_row - wk.kv_off + tok_local[rg];
        for (int j = 0; j < wk.n_prior; ++j) {
          const size_t prow = (size_t)(a.prior_rows[wk.prior_off + j] + tok_in_req) * a.q_heads + head;
          const float L = a.prior_lse[prow];
          if (!(L > -INFINITY)) continue;              // a partial without keys has weight 0
          const float Mn = fmaxf(M, L);
          const float ea = M > -INFINITY ? __expf(M - Mn) : 0.f, eb = __expf(L - Mn);
          const float* pp = a.prior_out + prow * kHeadDim;
#pragma unroll
          for (int d = 0; d < 4; ++d)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
              const float4 x = *(const float4*)&pp[32 * d + 8 * q4 + 4 * h];
              o[rg][d][4 * q4 + 0] = o[rg][d][4 * q4 + 0] * ea + x.x * eb;
              o[rg][d][4 * q4 + 1] = o[rg][d][4 * q4 + 1] * ea + x.y * eb;
              o[rg][d][4 * q4 + 2] = o[rg][d][4 * q4 + 2] * ea + x.z * eb;
              o[rg][d][4 * q4 + 3] = o[rg][d][4 * q4 + 3] * ea + x.w * eb;
            }
          W = W * ea + eb;
          M = Mn;
        }
        inv = W > 0.f ? 1.f / W : 0.f;
        lse_val = W > 0.f ? M + __logf(W) : -INFINITY;
      }
      if (MODE == 2) {
        // final output of the token, in the caller's layout and type
        const size_t orow = (size_t)token[rg] * a.q_heads + head;
        if (a.final_is_bf16) {
          uint16_t* op = (uint16_t*)a.final_out + orow * kHeadDim;
#pragma unroll
          for (int d = 0; d < 4; ++d)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
              const bf16x4 b = __builtin_convertvector(
                  f32x4{o[rg][d][4 * q4 + 0] * inv, o[rg][d][4 * q4 + 1] * inv, o[rg][d][4 * q4 + 2] * inv, o[rg][d][4 * q4 + 3] * inv}, bf16x4);
              *(uint2*)&op[32 * d + 8 * q4 + 4 * h] = __builtin_bit_cast(uint2, b);
            }
        } else {
          float* op = (float*)a.final_out + orow * kHeadDim;
#pragma unroll
          for (int d = 0; d < 4; ++d)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4)
              *(float4*)&op[32 * d + 8 * q4 + 4 * h] = make_float4(o[rg][d][4 * q4 + 0] * inv, o[rg][d][4 * q4 + 1] * inv,
                                                                    o[rg][d][4 * q4 + 2] * inv, o[rg][d][4 * q4 + 3] * inv);
        }
        if (h == 0 && a.final_lse) a.final_lse[orow] = lse_val;
      } else {
        const size_t orow = (size_t)(wk.out_row + tok_local[rg]) * a.q_heads + head;
        float* op = a.out + orow * kHeadDim;
#pragma unroll
        for (int d = 0; d < 4; ++d)
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4) {
            float4 val = make_float4(o[rg][d][4 * q4 + 0] * inv, o[rg][d][4 * q4 + 1] * inv, o[rg][d][4 * q4 + 2] * inv,
                                     o[rg][d][4 * q4 + 3] * inv);
            *(float4*)&op[32 * d + 8 * q4 + 4 * h] = val;
          }
        if (h == 0) a.lse[orow] = lse_val;
      }
    }
  }
}

template <int MODE>
tl_status launch_row_tiles(const AttnArgs& a, int n_work, hipStream_t st) {
  if (n_work == 0) return TL_OK;
  const dim3 grid((unsigned)n_work * a.kv_heads), block(kThreads);
  if (get_option_vread() == 0) {
    auto kern = row_tile_attn_kernel<MODE, 0>;
    TL_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBytes));
    hipLaunchKernelGGL(kern, grid, block, kLdsBytes, st, a);
  } else {
    auto kern = row_tile_attn_kernel<MODE, 1>;
    TL_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBytes));
    hipLaunchKernelGGL(kern, grid, block, kLdsBytes, st, a);
  }
  TL_HIP(hipGetLastError());
  return TL_OK;
}

}  // namespace

tl_status launch_pool_row_tiles(const AttnArgs& a, int n_work, hipStream_t st) { return launch_row_tiles<0>(a, n_work, st); }
tl_status launch_causal_row_tiles(const AttnArgs& a, int n_work, hipStream_t st) { return launch_row_tiles<1>(a, n_work, st); }
tl_status launch_fused_row_tiles(const AttnArgs& a, int n_work, hipStream_t st) { return launch_row_tiles<2>(a, n_work, st); }

}  // namespace tl
