// Row-tile partial attention (paper Section 4, first paragraph: query rows attend to cache
// segments independently and emit a partial output plus normalizer; Section 2.1: the new
// tokens' self-attention is one more such partial).
//
// One workgroup = 8 wavefronts = 256 query rows of one kv head (row = (token, head in the
// GQA group)); wave w owns rows 32w..32w+31.  The workgroup walks the work item's kv tokens
// in tiles of 64, staged through LDS with 16-byte coalesced loads.
//
// With 32x32x16 bf16 MFMA, per 32-token block and wave:
//   S^T[kv, row] = K[kv, :] . Q[row, :]      A = K block from LDS, B = Q (registers)
//   softmax numerators down the kv axis       lane l holds row l%32; its partner l^32 holds
//                                             the other half of that row's kv values
//   O^T[d, row] += V^T[d, kv] . P^T[kv, row]  A = V block read transposed from LDS, B = P
// Scores never leave registers between the two products.
//
// Completely filled tiles run in a ping-pong between the two wavefronts that share a SIMD
// (waves w and w+4): waves 0-3 go scores -> softmax -> accumulate within an iteration, waves 4-7
// accumulate the previous tile first and then do scores -> softmax, so that one wave's MFMA
// phase lines up with the other's vector-ALU phase.  V is triple buffered for that reason.
// The running maximum is only a reference point for the exponent (any reference gives the
// same normalised result), so it is raised -- and O rescaled -- only when a tile maximum
// exceeds it by more than 2^8.  Tiles cut short by a slot's fill, and the tiles on the causal
// diagonal, are masked and go through a plain path afterwards.
#include "attn_common.h"

#ifndef TL_STAGE_POS
#define TL_STAGE_POS 0
#endif
#ifdef TL_NO_SETPRIO
#define TL_SETPRIO(x)
#else
#define TL_SETPRIO(x) __builtin_amdgcn_s_setprio(x)
#endif

namespace tl {

namespace {

constexpr int kThreads = 512;
constexpr int kKS = kLdsStride;      // K row stride in LDS (bf16)
constexpr int kVS = kVStrideTile;    // V row stride in LDS (bf16)
constexpr int kKTile = kKvTile * kKS;
constexpr int kVTile = kKvTile * kVS;
constexpr size_t kLdsBytes = (size_t)(2 * kKTile + 3 * kVTile) * sizeof(uint16_t);
constexpr float kRescaleLog2 = 8.0f;  // raise the reference maximum when exceeded by 2^8
constexpr float kOptimisticLimit = 4294967296.0f;  // 2^32

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

__device__ __forceinline__ float max16(const f32x16& s) {
  float a = fmaxf(fmaxf(s[0], s[1]), s[2]);
  float b = fmaxf(fmaxf(s[3], s[4]), s[5]);
  float c = fmaxf(fmaxf(s[6], s[7]), s[8]);
  float d = fmaxf(fmaxf(s[9], s[10]), s[11]);
  float e = fmaxf(fmaxf(s[12], s[13]), s[14]);
  return fmaxf(fmaxf(fmaxf(a, b), fmaxf(c, d)), fmaxf(e, s[15]));
}

// Instruction order for one tile's MFMA phase: LDS reads run two groups of four MFMAs ahead
// of their use, so that the matrix unit is not left waiting on LDS latency.
// (mask 0x008 = MFMA, 0x100 = LDS read)
__device__ __forceinline__ void sched_qk_tile() {
  __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
  __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
  __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
  __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
  __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
  __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
}
__device__ __forceinline__ void sched_pv_tile() {
  __builtin_amdgcn_sched_group_barrier(0x100, 16, 0);
  __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
  __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
  __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
  __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
  __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
}

struct RowState {
  f32x16 o[4];     // O^T accumulators: o[d][r] = channel 32 d + 8 (r/4) + 4 h + r%4 of row l32
  float m_ref;     // reference maximum of the exponent (raw score units), -inf before any key
  float l_run;     // this lane's share of sum exp(s - m_ref)
};

template <bool CAUSAL, int VREAD>
__global__ __launch_bounds__(kThreads) void row_tile_attn_kernel(const AttnArgs a) {
  extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
  uint16_t* lds_k = lds;                 // [2][64][kKS]
  uint16_t* lds_v = lds + 2 * kKTile;    // [3][64][kVS]

  const int g = blockIdx.x % a.kv_heads;
  const Work wk = a.work[blockIdx.x / a.kv_heads];
  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63, l32 = lane & 31, h = lane >> 5;
  const int G = 1 << a.log2g;

  const int row = wave * 32 + l32;
  const int tok_local = row >> a.log2g;
  const int j = row & (G - 1);
  const bool row_ok = tok_local < wk.n_tok;
  const int token = row_ok ? a.tok[wk.tok_off + tok_local] : -1;
  const int first_token = a.tok[wk.tok_off];   // causal work: tokens of a tile are consecutive

  // Q as the B operand: lane holds row l32, head-dim elements 16 s + 8 h .. +7 of step s
  bf16x8 qreg[8];
  {
    const uint4* qp = (const uint4*)(a.q + ((size_t)(row_ok ? token : 0) * a.q_heads + g * G + j) * kHeadDim);
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      uint4 u = make_uint4(0, 0, 0, 0);
      if (row_ok) u = qp[2 * s + h];
      qreg[s] = as_bf16x8(u);
    }
  }

  RowState st;
#pragma unroll
  for (int d = 0; d < 4; ++d)
#pragma unroll
    for (int r = 0; r < 16; ++r) st.o[d][r] = 0.f;
  st.m_ref = -INFINITY;
  st.l_run = 0.f;
  const float c = a.scale_log2e;

  // which tiles are full (no masking needed for any row of this workgroup)
  int n_full, n_part;
  if (CAUSAL) {
    n_full = (first_token - wk.kv_off + 1) / kKvTile;
    n_part = (wk.kv_len + kKvTile - 1) / kKvTile - n_full;
  } else {
    n_full = wk.n_full;
    n_part = wk.n_part;
  }
  auto full_base = [&](int t) -> int { return CAUSAL ? wk.kv_off + kKvTile * t : a.tile_base[wk.full_off + t]; };

  // ---- global <-> LDS staging: 2 chunks of 16 B per thread per tile, for K and for V ----
  const size_t kv_row = (size_t)a.kv_heads * kHeadDim;
  const int c_tr = tid >> 4, c_part = tid & 15;          // chunk 0: token c_tr, chunk 1: token c_tr + 32
  // (plain scalars, not arrays: the staged chunks must live in registers across iterations)
  auto chunk_ptr = [&](const uint16_t* src, int base, int i) -> const uint4* {
    return (const uint4*)src + ((size_t)(base + c_tr + 32 * i) * kv_row + (size_t)g * kHeadDim) / 8 + c_part;
  };
  auto lds_chunk = [&](uint16_t* tile, int stride, int i) -> uint4* {
    return (uint4*)&tile[(c_tr + 32 * i) * stride + c_part * 8];
  };

  // ---- the three stages of a block ----
  // scores of one 32-token block (half hb of the K tile at `kt`)
  auto qk_block = [&](const uint16_t* kt, int hb, f32x16& s) {
#pragma unroll
    for (int r = 0; r < 16; ++r) s[r] = 0.f;
    const uint16_t* p = kt + (32 * hb + l32) * kKS + 8 * h;
#pragma unroll
    for (int s8 = 0; s8 < 8; ++s8) {
      const bf16x8 ak = *(const bf16x8*)&p[16 * s8];
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ak, qreg[s8], s, 0, 0, 0);
    }
  };
  // scores of both blocks of a tile, the two accumulation chains interleaved so that
  // consecutive MFMAs are independent
  auto qk_tile = [&](const uint16_t* kt, f32x16& sa, f32x16& sb) {
#pragma unroll
    for (int r = 0; r < 16; ++r) { sa[r] = 0.f; sb[r] = 0.f; }
    const uint16_t* p = kt + l32 * kKS + 8 * h;
#pragma unroll
    for (int s8 = 0; s8 < 8; ++s8) {
      const bf16x8 ak0 = *(const bf16x8*)&p[16 * s8];
      const bf16x8 ak1 = *(const bf16x8*)&p[32 * kKS + 16 * s8];
      sa = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ak0, qreg[s8], sa, 0, 0, 0);
      sb = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ak1, qreg[s8], sb, 0, 0, 0);
    }
  };
  // probabilities of a block against the current reference: p = 2^(c (s - m_ref)); B operands
  // pb[sp] cover registers 8 sp .. 8 sp + 7, i.e. block tokens 16 sp + {4h..4h+3, 8+4h..8+4h+3}
  auto exp_block = [&](f32x16& s, bf16x8 (&pb)[2]) {
    const float mc = st.m_ref * c;
    float lsum = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      s[r] = fast_exp2(fmaf(s[r], c, -mc));
      lsum += s[r];
    }
    st.l_run += lsum;
    pb[0] = pack_bf16x8(s[0], s[1], s[2], s[3], s[4], s[5], s[6], s[7]);
    pb[1] = pack_bf16x8(s[8], s[9], s[10], s[11], s[12], s[13], s[14], s[15]);
  };
  // O^T += V^T P^T for one block (half hb of the V tile at `vt`)
  auto pv_block = [&](const uint16_t* vt, int hb, const bf16x8 (&pb)[2]) {
#pragma unroll
    for (int sp = 0; sp < 2; ++sp) {
      const int kvb = 32 * hb + 16 * sp;
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        bf16x8 av;
        if (VREAD == 0) {
          const int blk = lane >> 4, jj = lane & 15;
          const uint16_t* p = vt + (kvb + 4 * (blk >> 1) + (jj >> 2)) * kVS + 32 * d + 16 * (blk & 1) + 4 * (jj & 3);
          av = join_tr(lds_read_tr(p), lds_read_tr(p + 8 * kVS));
        } else {
          s16x8 t;
#pragma unroll
          for (int e = 0; e < 8; ++e) t[e] = (short)vt[(kvb + 8 * (e >> 2) + 4 * h + (e & 3)) * kVS + 32 * d + l32];
          av = __builtin_bit_cast(bf16x8, t);
        }
        st.o[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, pb[sp], st.o[d], 0, 0, 0);
      }
    }
  };
  // raise the reference maximum if the scores of a tile (two blocks) exceed it by too much
  auto maybe_rescale = [&](const f32x16& sa, const f32x16& sb) {
    const float mx = xor32_max(fmaxf(max16(sa), max16(sb)));
    const bool need = (mx - st.m_ref) * c > kRescaleLog2 || st.m_ref == -INFINITY;
    if (__builtin_amdgcn_ballot_w64(need) != 0) {
      const float m_new = fmaxf(st.m_ref, mx);
      const float alpha = (m_new == -INFINITY) ? 1.f : fast_exp2((st.m_ref - m_new) * c);
      st.m_ref = m_new;
      st.l_run *= alpha;
#pragma unroll
      for (int d = 0; d < 4; ++d)
#pragma unroll
        for (int r = 0; r < 16; ++r) st.o[d][r] *= alpha;
    }
  };

  // ======================= pass 1: full tiles, ping-pong =======================
  if (n_full > 0) {
#ifdef TL_PINGPONG
    const bool group_b = wave >= 4;
#else
    const bool group_b = false;
#endif
    uint4 k0, k1, v0, v1;
    {
      const int b0 = full_base(0);
      k0 = *chunk_ptr(a.k, b0, 0); k1 = *chunk_ptr(a.k, b0, 1);
      v0 = *chunk_ptr(a.v, b0, 0); v1 = *chunk_ptr(a.v, b0, 1);
      *lds_chunk(lds_k, kKS, 0) = k0; *lds_chunk(lds_k, kKS, 1) = k1;
      *lds_chunk(lds_v, kVS, 0) = v0; *lds_chunk(lds_v, kVS, 1) = v1;
    }
    if (n_full > 1) {
      const int b1 = full_base(1);
      k0 = *chunk_ptr(a.k, b1, 0); k1 = *chunk_ptr(a.k, b1, 1);
      v0 = *chunk_ptr(a.v, b1, 0); v1 = *chunk_ptr(a.v, b1, 1);
    }
    int base_t2 = n_full > 2 ? full_base(2) : 0;   // first kv row of tile t+2, fetched one iteration early
    __syncthreads();

    f32x16 s0, s1;
    bf16x8 pa[2], pb[2];      // probabilities of the two 32-token halves of a tile
    int vprev = 0;            // V buffer of the previous tile
    int vcur = 0;
    for (int t = 0; t < n_full; ++t) {
      const uint16_t* kt = lds_k + (t & 1) * kKTile;
      const uint16_t* vt = lds_v + vcur * kVTile;
      const int vnext = vcur == 2 ? 0 : vcur + 1;
      // tile t+1 (fetched during the previous iteration) goes to the free buffers; fetch t+2
      auto stage_next = [&]() {
        if (t + 1 < n_full) {
          uint16_t* kn = lds_k + ((t + 1) & 1) * kKTile;
          uint16_t* vn = lds_v + vnext * kVTile;
          *lds_chunk(kn, kKS, 0) = k0; *lds_chunk(kn, kKS, 1) = k1;
          *lds_chunk(vn, kVS, 0) = v0; *lds_chunk(vn, kVS, 1) = v1;
        }
        if (t + 2 < n_full) {
          k0 = *chunk_ptr(a.k, base_t2, 0); k1 = *chunk_ptr(a.k, base_t2, 1);
          v0 = *chunk_ptr(a.v, base_t2, 0); v1 = *chunk_ptr(a.v, base_t2, 1);
        }
        if (t + 3 < n_full) base_t2 = full_base(t + 3);
      };
#if TL_STAGE_POS == 0
      stage_next();
#endif
      if (group_b && t > 0) {
        const uint16_t* vp = lds_v + vprev * kVTile;
        TL_SETPRIO(1);
        pv_block(vp, 0, pa);
        pv_block(vp, 1, pb);
        sched_pv_tile();
        TL_SETPRIO(0);
      }
      TL_SETPRIO(1);
      qk_tile(kt, s0, s1);
      sched_qk_tile();
      TL_SETPRIO(0);
#if TL_STAGE_POS == 1
      stage_next();
#endif
      // The exponent's reference point is set from the first tile; afterwards probabilities are
      // computed optimistically against it and the (rare) tile whose row sum comes out above
      // 2^32 -- scores far above the reference -- is redone with the reference raised first.
      if (t == 0) maybe_rescale(s0, s1);
      const float l_before = st.l_run;
      exp_block(s0, pa);
      exp_block(s1, pb);
      if (__builtin_amdgcn_ballot_w64(!(st.l_run - l_before < kOptimisticLimit)) != 0) {
        st.l_run = l_before;
        qk_tile(kt, s0, s1);
        maybe_rescale(s0, s1);
        exp_block(s0, pa);
        exp_block(s1, pb);
      }
#if TL_STAGE_POS == 2
      stage_next();
#endif
      if (!group_b) {
        TL_SETPRIO(1);
        pv_block(vt, 0, pa);
        pv_block(vt, 1, pb);
        sched_pv_tile();
        TL_SETPRIO(0);
      }
#if TL_STAGE_POS == 3
      stage_next();
#endif
      __syncthreads();
      vprev = vcur;
      vcur = vnext;
    }
    if (group_b) {
      const uint16_t* vp = lds_v + vprev * kVTile;
      pv_block(vp, 0, pa);
      pv_block(vp, 1, pb);
    }
    __syncthreads();
  }

  // ======================= pass 2: masked tiles, one at a time =======================
  for (int pt = 0; pt < n_part; ++pt) {
    int base, valid;
    if (CAUSAL) {
      const int off = kKvTile * (n_full + pt);
      base = wk.kv_off + off;
      valid = min(kKvTile, wk.kv_len - off);
    } else {
      base = a.part_tile[2 * (wk.part_off + pt)];
      valid = a.part_tile[2 * (wk.part_off + pt) + 1];
    }
    {
      // rows beyond `valid` are written as zero: 0 * garbage cannot make NaN
      const uint4 z = make_uint4(0, 0, 0, 0);
      const uint4 k0 = c_tr < valid ? *chunk_ptr(a.k, base, 0) : z;
      const uint4 k1 = c_tr + 32 < valid ? *chunk_ptr(a.k, base, 1) : z;
      const uint4 v0 = c_tr < valid ? *chunk_ptr(a.v, base, 0) : z;
      const uint4 v1 = c_tr + 32 < valid ? *chunk_ptr(a.v, base, 1) : z;
      *lds_chunk(lds_k, kKS, 0) = k0; *lds_chunk(lds_k, kKS, 1) = k1;
      *lds_chunk(lds_v, kVS, 0) = v0; *lds_chunk(lds_v, kVS, 1) = v1;
    }
    __syncthreads();
#pragma unroll 1
    for (int hb = 0; hb < 2; ++hb) {
      if (32 * hb >= valid) break;              // uniform
      f32x16 s;
      qk_block(lds_k, hb, s);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int kv = 32 * hb + 8 * (r >> 2) + 4 * h + (r & 3);
        bool hide = kv >= valid;
        if (CAUSAL) hide = hide || (base + kv > token);
        if (hide) s[r] = -INFINITY;
      }
      maybe_rescale(s, s);
      bf16x8 pb[2];
      if (st.m_ref == -INFINITY) {
        // every key so far is hidden from this row: probabilities are zero
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = 0.f;
        pb[0] = pack_bf16x8(0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f);
        pb[1] = pb[0];
      } else {
        exp_block(s, pb);
      }
      pv_block(lds_v, hb, pb);
    }
    __syncthreads();
  }

  // ---- epilogue: normalise, LSE, store ----
  const float l_tot = xor32_sum(st.l_run);
  if (row_ok) {
    const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
    const int head = g * G + j;
    const size_t orow = (size_t)(wk.out_row + tok_local) * a.q_heads + head;
    float* op = a.out + orow * kHeadDim;
#pragma unroll
    for (int d = 0; d < 4; ++d)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        float4 val = make_float4(st.o[d][4 * q4 + 0] * inv, st.o[d][4 * q4 + 1] * inv, st.o[d][4 * q4 + 2] * inv,
                                 st.o[d][4 * q4 + 3] * inv);
        *(float4*)&op[32 * d + 8 * q4 + 4 * h] = val;
      }
    if (h == 0) a.lse[orow] = l_tot > 0.f ? st.m_ref * a.scale + __logf(l_tot) : -INFINITY;
  }
}

template <bool CAUSAL>
tl_status launch_row_tiles(const AttnArgs& a, int n_work, hipStream_t st) {
  if (n_work == 0) return TL_OK;
  const dim3 grid((unsigned)n_work * a.kv_heads), block(kThreads);
  if (get_option_vread() == 0) {
    auto kern = row_tile_attn_kernel<CAUSAL, 0>;
    TL_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBytes));
    hipLaunchKernelGGL(kern, grid, block, kLdsBytes, st, a);
  } else {
    auto kern = row_tile_attn_kernel<CAUSAL, 1>;
    TL_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBytes));
    hipLaunchKernelGGL(kern, grid, block, kLdsBytes, st, a);
  }
  TL_HIP(hipGetLastError());
  return TL_OK;
}

}  // namespace

tl_status launch_pool_row_tiles(const AttnArgs& a, int n_work, hipStream_t st) { return launch_row_tiles<false>(a, n_work, st); }
tl_status launch_causal_row_tiles(const AttnArgs& a, int n_work, hipStream_t st) { return launch_row_tiles<true>(a, n_work, st); }

}  // namespace tl
