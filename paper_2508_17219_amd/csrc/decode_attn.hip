// Split-K partial attention for work with at most 16 query rows per kv head (decode: one
// token x the GQA group).  Bandwidth-bound: every K/V byte is used once (paper Section 4.2:
// the memory-bound side of max(4Cd/F, 4Cd/B_mem)).
//
// One workgroup = one unit (a few query tokens x a chunk of the slot list) for ALL kv heads:
// wave w handles kv head 8*blockIdx.y + w, so that the workgroup as a whole reads whole
// token rows of the slot (kv_heads * 256 B contiguous).  Each wave streams its head's K and
// V in tiles of 32 tokens: global -> registers (prefetched one tile ahead) -> wave-private
// LDS -> MFMA 16x16x32 operands.  The 8 (or fewer) GQA rows ride in a 16-row MFMA tile.
#include "attn_common.h"

// Each wave stages its kv head's tiles in an LDS region of its own, and a wave's LDS
// operations execute in program order, so no workgroup barrier is needed between the
// wave's writes and its reads: a compiler-level ordering point is enough.
#define TL_UNIT_SYNC() do { __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront"); __builtin_amdgcn_wave_barrier(); } while (0)

namespace tl {

namespace {

constexpr int kThreads = 512;
constexpr int kWaves = 8;
constexpr int kTok = 32;                                   // kv tokens per wave tile
constexpr int kWaveElems = kTok * (kLdsStride + kVStrideUnit);   // K tile + V tile, bf16 elements
constexpr size_t kLdsBytes = (size_t)kWaves * kWaveElems * sizeof(uint16_t);

template <int VREAD>
__global__ __launch_bounds__(kThreads) void splitk_unit_attn_kernel(const AttnArgs a) {
  extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
  const Work wk = a.work[blockIdx.x];
  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63, l16 = lane & 15, c4 = lane >> 4;
  const int g = blockIdx.y * kWaves + wave;
  const bool active = g < a.kv_heads;
  const int G = a.group;
  uint16_t* kt = lds + wave * kWaveElems;
  uint16_t* vt = kt + kTok * kLdsStride;

  const int tok_local = l16 / G;
  const int j = l16 - tok_local * G;
  const bool row_ok = active && tok_local < wk.n_tok;
  const int token = row_ok ? a.tok[wk.tok_off + tok_local] : 0;

  // Q as B operand of 16x16x32: lane holds row l16, head-dim 32 s + 8 c4 .. +7
  bf16x8 qreg[4];
  {
    const uint4* qp = (const uint4*)(a.q + ((size_t)token * a.q_heads + (active ? g : 0) * G + j) * kHeadDim);
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      uint4 u = make_uint4(0, 0, 0, 0);
      if (row_ok) u = qp[4 * s + c4];
      qreg[s] = as_bf16x8(u);
    }
  }

  f32x4 o[8];
#pragma unroll
  for (int d = 0; d < 8; ++d) o[d] = f32x4{0.f, 0.f, 0.f, 0.f};
  // two row sums: the unrounded fp32 one gives the LSE, the one over the probabilities as rounded
  // to bf16 for the second product normalises O (a convex combination of V rows whatever the rounding)
  float m_run = -INFINITY, l_run = 0.f, lr_run = 0.f;
  const float c = a.scale_log2e;
  const size_t kv_row = (size_t)a.kv_heads * kHeadDim;

  uint4 kst[8], vst[8];
  auto gload = [&](int base, int valid) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int cidx = lane + 64 * i;
      const int tr = cidx >> 4, part = cidx & 15;
      kst[i] = make_uint4(0, 0, 0, 0);
      vst[i] = make_uint4(0, 0, 0, 0);
      if (active && tr < valid) {
        const size_t off = ((size_t)(base + tr) * kv_row + (size_t)g * kHeadDim) / 8 + part;
        kst[i] = ((const uint4*)a.k)[off];
        vst[i] = ((const uint4*)a.v)[off];
      }
    }
  };
  auto lstore = [&]() {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int cidx = lane + 64 * i;
      const int tr = cidx >> 4, part = cidx & 15;
      *(uint4*)&kt[tr * kLdsStride + part * 8] = kst[i];
      *(uint4*)&vt[tr * kVStrideUnit + part * 8] = vst[i];
    }
  };

  // tile cursor over the unit's slots (uniform across the workgroup)
  // (a slot that the unit's run lists m times is walked once; its keys weigh m: lm = log2 m is
  // added to the exponent of the tile's probabilities)
  int li = 0, kk = 0;
  auto next_tile = [&](int& base, int& valid, float& lm) -> bool {
    while (li < wk.kv_len) {
      const int slot = a.slots[wk.kv_off + li];
      const int f = a.fill[slot];
      const int off = kk * kTok;
      if (off < f) {
        base = slot * a.seg_len + off;
        valid = min(kTok, f - off);
        lm = a.slot_lm ? a.slot_lm[wk.kv_off + li] : 0.f;
        kk++;
        if (kk * kTok >= f) { li++; kk = 0; }
        return true;
      }
      li++;
      kk = 0;
    }
    return false;
  };

  int base = 0, valid = 0;
  float lm = 0.f;
  bool have = next_tile(base, valid, lm);
  if (have) gload(base, valid);

  while (have) {
    lstore();
    int nbase = 0, nvalid = 0;
    float nlm = 0.f;
    const bool have_next = next_tile(nbase, nvalid, nlm);
    if (have_next) gload(nbase, nvalid);
    TL_UNIT_SYNC();

    if (active) {
      // S^T = K Q^T : two blocks of 16 tokens
      f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const bf16x8 a0 = *(const bf16x8*)&kt[l16 * kLdsStride + 32 * s + 8 * c4];
        const bf16x8 a1 = *(const bf16x8*)&kt[(16 + l16) * kLdsStride + 32 * s + 8 * c4];
        s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, qreg[s], s0, 0, 0, 0);
        s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, qreg[s], s1, 0, 0, 0);
      }
      if (valid < kTok) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          if (4 * c4 + r >= valid) s0[r] = -INFINITY;
          if (16 + 4 * c4 + r >= valid) s1[r] = -INFINITY;
        }
      }
      float mx = fmaxf(fmaxf(fmaxf(s0[0], s0[1]), fmaxf(s0[2], s0[3])), fmaxf(fmaxf(s1[0], s1[1]), fmaxf(s1[2], s1[3])));
      mx = fmaxf(mx, __shfl_xor(mx, 16));
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float m_new = fmaxf(m_run, mx);
      const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
      const float alpha = fast_exp2((m_run - m_use) * c);
      m_run = m_new;
      const float mc = m_use * c - lm;
      float lsum = 0.f;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        s0[r] = fast_exp2(fmaf(s0[r], c, -mc));
        s1[r] = fast_exp2(fmaf(s1[r], c, -mc));
        lsum += s0[r] + s1[r];
      }
      l_run = l_run * alpha + lsum;
      // P^T operand: elements 0..3 = block 0 (tokens 4 c4 + r), 4..7 = block 1 (16 + 4 c4 + r)
      const bf16x8 pb = pack_bf16x8(s0[0], s0[1], s0[2], s0[3], s1[0], s1[1], s1[2], s1[3]);
      {
        typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
        const u32x4 w = __builtin_bit_cast(u32x4, pb);
        float lr = lr_run * alpha;
#pragma unroll
        for (int i = 0; i < 4; ++i) lr = add_bf16_pair(lr, w[i]);
        lr_run = lr;
      }
#pragma unroll
      for (int d = 0; d < 8; ++d) {
        bf16x8 av;
        if (VREAD == 0) {
          const uint16_t* p = vt + (4 * c4 + (l16 >> 2)) * kVStrideUnit + 16 * d + 4 * (l16 & 3);
          av = join_tr(lds_read_tr(p), lds_read_tr(p + 16 * kVStrideUnit));
        } else {
          s16x8 t;
#pragma unroll
          for (int e = 0; e < 8; ++e) t[e] = (short)vt[(16 * (e >> 2) + 4 * c4 + (e & 3)) * kVStrideUnit + 16 * d + l16];
          av = __builtin_bit_cast(bf16x8, t);
        }
        f32x4 acc = o[d];
        acc[0] *= alpha; acc[1] *= alpha; acc[2] *= alpha; acc[3] *= alpha;
        o[d] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, pb, acc, 0, 0, 0);
      }
    }
    TL_UNIT_SYNC();
    have = have_next;
    base = nbase;
    valid = nvalid;
    lm = nlm;
  }

  float l_tot = l_run + __shfl_xor(l_run, 16);
  l_tot += __shfl_xor(l_tot, 32);
  float lr_tot = lr_run + __shfl_xor(lr_run, 16);
  lr_tot += __shfl_xor(lr_tot, 32);
  if (row_ok) {
    const float inv = lr_tot > 0.f ? 1.f / lr_tot : 0.f;
    const size_t orow = (size_t)(wk.out_row + tok_local) * a.q_heads + g * G + j;
    float* op = a.out + orow * kHeadDim;
#pragma unroll
    for (int d = 0; d < 8; ++d)
      *(float4*)&op[16 * d + 4 * c4] = make_float4(o[d][0] * inv, o[d][1] * inv, o[d][2] * inv, o[d][3] * inv);
    if (c4 == 0) a.lse[orow] = l_tot > 0.f ? m_run * a.scale + __logf(l_tot) : -INFINITY;
  }
}

}  // namespace

tl_status launch_splitk_units(const AttnArgs& a, int n_work, hipStream_t st) {
  if (n_work == 0) return TL_OK;
  const dim3 grid((unsigned)n_work, (unsigned)((a.kv_heads + kWaves - 1) / kWaves)), block(kThreads);
  if (get_option_vread() == 0) {
    auto kern = splitk_unit_attn_kernel<0>;
    TL_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBytes));
    hipLaunchKernelGGL(kern, grid, block, kLdsBytes, st, a);
  } else {
    auto kern = splitk_unit_attn_kernel<1>;
    TL_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBytes));
    hipLaunchKernelGGL(kern, grid, block, kLdsBytes, st, a);
  }
  TL_HIP(hipGetLastError());
  return TL_OK;
}

}  // namespace tl
