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
// Completely filled tiles run through a software pipeline three blocks deep: while the MFMA
// unit computes the scores of block j+1 and accumulates block j-1 into O, the vector ALU turns
// the scores of block j into probabilities.  The running maximum is only a reference point
// for the exponent (any reference gives the same normalised result), so it is raised -- and O
// rescaled -- only when a block maximum exceeds it by more than 2^8; that test is the single
// branch of a pipeline step.  Tiles cut short by a slot's fill, and the tiles on the causal
// diagonal, are masked and go through a plain (unpipelined) path afterwards.
#include "attn_common.h"

namespace tl {

namespace {

constexpr int kThreads = 512;
constexpr int kKS = kLdsStride;      // K row stride in LDS (bf16)
constexpr int kVS = kVStrideTile;    // V row stride in LDS (bf16)
constexpr int kKTile = kKvTile * kKS;
constexpr int kVTile = kKvTile * kVS;
constexpr size_t kLdsBytes = (size_t)2 * (kKTile + kVTile) * sizeof(uint16_t);
constexpr float kRescaleLog2 = 8.0f;  // raise the reference maximum when exceeded by 2^8

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

struct RowState {
  f32x16 o[4];     // O^T accumulators: o[d][r] = channel 32 d + 8 (r/4) + 4 h + r%4 of row l32
  float m_ref;     // reference maximum of the exponent (raw score units), -inf before any key
  float l_run;     // this lane's share of sum exp(s - m_ref)
};

template <bool CAUSAL, int VREAD>
__global__ __launch_bounds__(kThreads) void row_tile_attn_kernel(const AttnArgs a) {
  extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
  uint16_t* lds_k = lds;                 // [2][64][kKS]
  uint16_t* lds_v = lds + 2 * kKTile;    // [2][64][kVS]

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
  auto gload_tile = [&](const uint16_t* src, int base, uint4 (&dst)[2]) {
#pragma unroll
    for (int i = 0; i < 2; ++i)
      dst[i] = ((const uint4*)src)[((size_t)(base + c_tr + 32 * i) * kv_row + (size_t)g * kHeadDim) / 8 + c_part];
  };
  auto gload_tile_masked = [&](const uint16_t* src, int base, int valid, uint4 (&dst)[2]) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      dst[i] = make_uint4(0, 0, 0, 0);
      if (c_tr + 32 * i < valid)
        dst[i] = ((const uint4*)src)[((size_t)(base + c_tr + 32 * i) * kv_row + (size_t)g * kHeadDim) / 8 + c_part];
    }
  };
  auto lwrite_tile = [&](uint16_t* tile, int stride, const uint4 (&srcv)[2]) {
#pragma unroll
    for (int i = 0; i < 2; ++i) *(uint4*)&tile[(c_tr + 32 * i) * stride + c_part * 8] = srcv[i];
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
  // raise the reference maximum to cover block scores `s` if they exceed it by too much;
  // `pend` holds probabilities computed against the old reference and not yet accumulated
  auto maybe_rescale = [&](const f32x16& s, bf16x8 (*pend)[2]) {
    const float mx = xor32_max(max16(s));
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
      if (pend) {
#pragma unroll
        for (int sp = 0; sp < 2; ++sp) {
          f32x8 f = __builtin_convertvector((*pend)[sp], f32x8);
#pragma unroll
          for (int e = 0; e < 8; ++e) f[e] *= alpha;
          (*pend)[sp] = __builtin_convertvector(f, bf16x8);
        }
      }
    }
  };

  // ======================= pass 1: full tiles, pipelined =======================
  if (n_full > 0) {
    uint4 kst[2], vst[2];
    // prologue: K(0), V(0), K(1) into LDS; K(2), V(1) into the staging registers
    gload_tile(a.k, full_base(0), kst);
    gload_tile(a.v, full_base(0), vst);
    lwrite_tile(lds_k, kKS, kst);
    lwrite_tile(lds_v, kVS, vst);
    if (n_full > 1) {
      gload_tile(a.k, full_base(1), kst);
      gload_tile(a.v, full_base(1), vst);
      lwrite_tile(lds_k + kKTile, kKS, kst);
    }
    if (n_full > 2) gload_tile(a.k, full_base(2), kst);
    __syncthreads();

    f32x16 s0, s1;
    bf16x8 p0[2], p1[2];
    qk_block(lds_k, 0, s0);

    for (int t = 0; t < n_full; ++t) {
      const uint16_t* k_cur = lds_k + (t & 1) * kKTile;
      const uint16_t* k_nxt = lds_k + ((t + 1) & 1) * kKTile;
      const uint16_t* v_cur = lds_v + (t & 1) * kVTile;
      const uint16_t* v_prv = lds_v + ((t + 1) & 1) * kVTile;

      // ---- step A: scores of block 2t+1 | probabilities of block 2t | accumulate block 2t-1
      if (t > 0) {
        maybe_rescale(s0, &p1);
        qk_block(k_cur, 1, s1);
        exp_block(s0, p0);
        pv_block(v_prv, 1, p1);
      } else {
        maybe_rescale(s0, nullptr);
        qk_block(k_cur, 1, s1);
        exp_block(s0, p0);
      }

      // K(t) and V(t-1) are dead now: refill their buffers with K(t+2) and V(t+1)
      __syncthreads();
      if (t + 2 < n_full) lwrite_tile(lds_k + (t & 1) * kKTile, kKS, kst);
      if (t + 1 < n_full) lwrite_tile(lds_v + ((t + 1) & 1) * kVTile, kVS, vst);
      if (t + 3 < n_full) gload_tile(a.k, full_base(t + 3), kst);
      if (t + 2 < n_full) gload_tile(a.v, full_base(t + 2), vst);

      // ---- step B: scores of block 2t+2 | probabilities of block 2t+1 | accumulate block 2t
      maybe_rescale(s1, &p0);
      if (t + 1 < n_full) {
        qk_block(k_nxt, 0, s0);
        exp_block(s1, p1);
        pv_block(v_cur, 0, p0);
      } else {
        exp_block(s1, p1);
        pv_block(v_cur, 0, p0);
      }
    }
    // the last block is still pending
    pv_block(lds_v + ((n_full - 1) & 1) * kVTile, 1, p1);
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
    uint4 kst[2], vst[2];
    gload_tile_masked(a.k, base, valid, kst);
    gload_tile_masked(a.v, base, valid, vst);   // rows beyond `valid` are zero: 0 * garbage cannot make NaN
    lwrite_tile(lds_k, kKS, kst);
    lwrite_tile(lds_v, kVS, vst);
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
      maybe_rescale(s, nullptr);
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
