// Row-tile partial attention (paper Section 4, first paragraph: query rows attend to cache
// segments independently and emit a partial output plus normalizer; Section 2.1: the new
// tokens' self-attention is one more such partial).
//
// One workgroup = 8 wavefronts = 256 query rows of one kv head (row = (token, head in the
// GQA group)); wave w owns rows 32w..32w+31.  The workgroup walks the work item's slot list
// (or, for the causal block, the request's new tokens) in tiles of 64 kv tokens, staged
// through LDS with 16-byte coalesced loads, double buffered.
//
// Per tile and wave, with 32x32x16 bf16 MFMA:
//   S^T[kv, row] = K[kv, :] . Q[row, :]      A = K tile from LDS, B = Q (registers)
//   online softmax down the kv axis           lane l holds row l%32; its partner l^32 holds
//                                             the other half of that row's kv values
//   O^T[d, row] += V^T[d, kv] . P^T[kv, row]  A = V tile read transposed from LDS, B = P
// Scores never leave registers between the two products.
#include "attn_common.h"

namespace tl {

namespace {

constexpr int kThreads = 512;
constexpr int kTileElems = kKvTile * kLdsStride;                       // bf16 per K (or V) tile
constexpr size_t kLdsBytes = (size_t)4 * kTileElems * sizeof(uint16_t);  // K,V x 2 buffers

struct KvCursor {
  int i;    // position in the slot list / tile index for causal work
  int kt;   // tile inside the slot
};

// Next tile of kv tokens for this work: first token (in units of kv rows of a.k / a.v) and
// number of valid tokens (1..64).  Returns false at the end.  Uniform across the workgroup.
template <bool CAUSAL>
__device__ __forceinline__ bool next_tile(const AttnArgs& a, const Work& wk, KvCursor& c, int& base, int& valid) {
  if (CAUSAL) {
    const int off = c.i * kKvTile;
    if (off >= wk.kv_len) return false;
    base = wk.kv_off + off;
    valid = min(kKvTile, wk.kv_len - off);
    c.i++;
    return true;
  } else {
    while (c.i < wk.kv_len) {
      const int slot = a.slots[wk.kv_off + c.i];
      const int f = a.fill[slot];
      const int off = c.kt * kKvTile;
      if (off < f) {
        base = slot * a.seg_len + off;
        valid = min(kKvTile, f - off);
        c.kt++;
        if (c.kt * kKvTile >= f) { c.i++; c.kt = 0; }
        return true;
      }
      c.i++;
      c.kt = 0;
    }
    return false;
  }
}

template <bool CAUSAL, int VREAD>
__global__ __launch_bounds__(kThreads) void row_tile_attn_kernel(const AttnArgs a) {
  extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
  uint16_t* lds_k = lds;                    // [2][64][136]
  uint16_t* lds_v = lds + 2 * kTileElems;   // [2][64][136]

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

  f32x16 o[4];
#pragma unroll
  for (int d = 0; d < 4; ++d)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[d][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  const float c = a.scale_log2e;

  // global -> register staging: 2 K chunks + 2 V chunks of 16 B per thread per tile
  const size_t kv_row = (size_t)a.kv_heads * kHeadDim;
  uint4 kst[2], vst[2];
  auto gload = [&](int base, int valid) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int cidx = tid + kThreads * i;
      const int tr = cidx >> 4, part = cidx & 15;
      kst[i] = make_uint4(0, 0, 0, 0);
      vst[i] = make_uint4(0, 0, 0, 0);
      if (tr < valid) {
        const size_t off = ((size_t)(base + tr) * kv_row + (size_t)g * kHeadDim) / 8 + part;
        kst[i] = ((const uint4*)a.k)[off];
        vst[i] = ((const uint4*)a.v)[off];
      }
    }
  };
  auto lstore = [&](int buf) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int cidx = tid + kThreads * i;
      const int tr = cidx >> 4, part = cidx & 15;
      *(uint4*)&lds_k[buf * kTileElems + tr * kLdsStride + part * 8] = kst[i];
      *(uint4*)&lds_v[buf * kTileElems + tr * kLdsStride + part * 8] = vst[i];
    }
  };

  KvCursor cur{0, 0};
  int base = 0, valid = 0;
  bool have = next_tile<CAUSAL>(a, wk, cur, base, valid);
  if (have) {
    gload(base, valid);
    lstore(0);
  }
  __syncthreads();

  int buf = 0;
  while (have) {
    int nbase = 0, nvalid = 0;
    const bool have_next = next_tile<CAUSAL>(a, wk, cur, nbase, nvalid);
    if (have_next) gload(nbase, nvalid);

    const uint16_t* kt = lds_k + buf * kTileElems;
    const uint16_t* vt = lds_v + buf * kTileElems;

    // ---- S^T = K Q^T : two 32-token blocks ----
    f32x16 s0, s1;
#pragma unroll
    for (int r = 0; r < 16; ++r) { s0[r] = 0.f; s1[r] = 0.f; }
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      const bf16x8 a0 = *(const bf16x8*)&kt[l32 * kLdsStride + 16 * s + 8 * h];
      const bf16x8 a1 = *(const bf16x8*)&kt[(32 + l32) * kLdsStride + 16 * s + 8 * h];
      s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, qreg[s], s0, 0, 0, 0);
      s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, qreg[s], s1, 0, 0, 0);
    }

    // ---- mask: tokens beyond the slot's fill; causal diagonal ----
    const bool need_mask = valid < kKvTile || (CAUSAL && base + kKvTile - 1 > first_token);
    if (need_mask) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int kv0 = 8 * (r >> 2) + 4 * h + (r & 3);
        const int kv1 = 32 + kv0;
        bool hide0 = kv0 >= valid, hide1 = kv1 >= valid;
        if (CAUSAL) {
          hide0 = hide0 || (base + kv0 > token);
          hide1 = hide1 || (base + kv1 > token);
        }
        if (hide0) s0[r] = -INFINITY;
        if (hide1) s1[r] = -INFINITY;
      }
    }

    // ---- online softmax (per lane: one row, 32 of its 64 scores) ----
    float mx = s0[0];
#pragma unroll
    for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s0[r]);
#pragma unroll
    for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s1[r]);
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(m_run, mx);
    const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
    const float alpha = fast_exp2((m_run - m_use) * c);
    m_run = m_new;
    const float mc = m_use * c;
    float lsum = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      s0[r] = fast_exp2(fmaf(s0[r], c, -mc));
      s1[r] = fast_exp2(fmaf(s1[r], c, -mc));
      lsum += s0[r] + s1[r];
    }
    l_run = l_run * alpha + lsum;
#pragma unroll
    for (int d = 0; d < 4; ++d)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[d][r] *= alpha;

    // P^T as B operands: step (b, sp) covers registers 8 sp .. 8 sp + 7 of block b, i.e. kv
    // tokens 32 b + 16 sp + {4h..4h+3, 8+4h..8+4h+3}
    bf16x8 pb[2][2];
    pb[0][0] = pack_bf16x8(s0[0], s0[1], s0[2], s0[3], s0[4], s0[5], s0[6], s0[7]);
    pb[0][1] = pack_bf16x8(s0[8], s0[9], s0[10], s0[11], s0[12], s0[13], s0[14], s0[15]);
    pb[1][0] = pack_bf16x8(s1[0], s1[1], s1[2], s1[3], s1[4], s1[5], s1[6], s1[7]);
    pb[1][1] = pack_bf16x8(s1[8], s1[9], s1[10], s1[11], s1[12], s1[13], s1[14], s1[15]);

    // ---- O^T += V^T P^T ----
#pragma unroll
    for (int b = 0; b < 2; ++b) {
#pragma unroll
      for (int sp = 0; sp < 2; ++sp) {
        const int kvb = 32 * b + 16 * sp;
#pragma unroll
        for (int d = 0; d < 4; ++d) {
          bf16x8 av;
          if (VREAD == 0) {
            const int blk = lane >> 4, jj = lane & 15;
            const uint16_t* p = vt + (kvb + 4 * (blk >> 1) + (jj >> 2)) * kLdsStride + 32 * d + 16 * (blk & 1) + 4 * (jj & 3);
            av = join_tr(lds_read_tr(p), lds_read_tr(p + 8 * kLdsStride));
          } else {
            s16x8 t;
#pragma unroll
            for (int e = 0; e < 8; ++e)
              t[e] = (short)vt[(kvb + 8 * (e >> 2) + 4 * h + (e & 3)) * kLdsStride + 32 * d + l32];
            av = __builtin_bit_cast(bf16x8, t);
          }
          o[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, pb[b][sp], o[d], 0, 0, 0);
        }
      }
    }

    if (have_next) lstore(buf ^ 1);
    __syncthreads();
    buf ^= 1;
    have = have_next;
    base = nbase;
    valid = nvalid;
  }

  // ---- epilogue: normalise, LSE, store ----
  const float l_tot = l_run + __shfl_xor(l_run, 32);
  if (row_ok) {
    const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
    const int head = g * G + j;
    const size_t orow = (size_t)(wk.out_row + tok_local) * a.q_heads + head;
    float* op = a.out + orow * kHeadDim;
#pragma unroll
    for (int d = 0; d < 4; ++d)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        float4 val = make_float4(o[d][4 * q4 + 0] * inv, o[d][4 * q4 + 1] * inv, o[d][4 * q4 + 2] * inv,
                                 o[d][4 * q4 + 3] * inv);
        *(float4*)&op[32 * d + 8 * q4 + 4 * h] = val;
      }
    if (h == 0) a.lse[orow] = l_tot > 0.f ? m_run * a.scale + __logf(l_tot) : -INFINITY;
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
