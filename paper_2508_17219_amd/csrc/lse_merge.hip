// Exact recombination of partial outputs by their log-sum-exp (paper Section 2.1: partial
// outputs and normalizers are reduced into the final output; Section 4, first paragraph),
// the self block of single-token requests, and the four compute entry points of the ABI
// (tl_segment_attn, tl_causal_block, tl_fused_attn, tl_merge).
#include <cmath>
#include <mutex>

#include "attn_common.h"

namespace tl {

tl_status launch_pool_row_tiles(const AttnArgs& a, int n_work, hipStream_t st);
tl_status launch_causal_row_tiles(const AttnArgs& a, int n_work, hipStream_t st);
tl_status launch_splitk_units(const AttnArgs& a, int n_work, hipStream_t st);
tl_status launch_fused_row_tiles(const AttnArgs& a, int n_work, hipStream_t st);

namespace {

// blockIdx.x = position in the list of tokens to merge, blockIdx.y = chunk of 256 (head, channel-quad) positions; a thread owns
// 4 consecutive channels of one head.
//   M = max_j LSE_j;  w_j = exp(LSE_j - M);  O = sum w_j O_j / sum w_j;  LSE = M + ln sum w_j
template <bool OUT_BF16>
__global__ __launch_bounds__(256) void lse_merge_kernel(const float* __restrict__ part, const float* __restrict__ lse,
                                                        const int32_t* __restrict__ mfix, void* __restrict__ out,
                                                        float* __restrict__ lse_out, int q_heads) {
  // the token's record: {token, partial rows..., -1 ...}; the same for every lane, one load
  int32_t rec[kMergeFixInts];
#pragma unroll
  for (int u = 0; u < kMergeFixInts; ++u) rec[u] = mfix[(size_t)blockIdx.x * kMergeFixInts + u];
  const int t = rec[0];
  const int idx = blockIdx.y * blockDim.x + threadIdx.x;
  if (idx < q_heads * 32) {
    const int hd = idx >> 5, c4 = idx & 31;
    // LSEs and partial rows of the whole list are fetched at once, neither waiting for the other:
    // one memory latency after the record's
    constexpr int kList = kMergeFixInts - 1;
    float l[kList];
    float4 v[kList];
#pragma unroll
    for (int u = 0; u < kList; ++u) {
      l[u] = -INFINITY;
      v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (rec[1 + u] >= 0) {
        const size_t row = (size_t)rec[1 + u] * q_heads + hd;
        l[u] = lse[row];
        v[u] = ((const float4*)part)[row * 32 + c4];
      }
    }
    float M = -INFINITY;
#pragma unroll
    for (int u = 0; u < kList; ++u) M = fmaxf(M, l[u]);
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    float wsum = 0.f;
    if (M > -INFINITY) {
#pragma unroll
      for (int u = 0; u < kList; ++u) {
        if (rec[1 + u] >= 0) {
          const float w = expf(l[u] - M);
          acc.x += w * v[u].x; acc.y += w * v[u].y; acc.z += w * v[u].z; acc.w += w * v[u].w;
          wsum += w;
        }
      }
      const float inv = 1.f / wsum;
      acc.x *= inv; acc.y *= inv; acc.z *= inv; acc.w *= inv;
    }
    const size_t orow = (size_t)t * q_heads + hd;
    if (OUT_BF16) {
      typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
      f32x4 f = {acc.x, acc.y, acc.z, acc.w};
      ((bf16x4_t*)out)[orow * 32 + c4] = __builtin_convertvector(f, bf16x4_t);
    } else {
      ((float4*)out)[orow * 32 + c4] = acc;
    }
    if (lse_out && c4 == 0) lse_out[orow] = M > -INFINITY ? M + logf(wsum) : -INFINITY;
  }
}

// The same recombination for tokens with many partials (split-K decode: tens to hundreds per
// token, and few tokens): one workgroup per (token, head), the partials dealt round-robin to
// kMergeSlices slices of 32 lanes (a lane owns 4 channels), so that a long list is walked
// kMergeSlices entries at a time.  The maximum is agreed on first, then every slice
// accumulates with the same weights w_j = exp(LSE_j - M) as the kernel above, and slice 0 adds
// the slices up in a fixed order.
constexpr int kMergeSlices = 8;
template <bool OUT_BF16>
__global__ __launch_bounds__(32 * kMergeSlices) void lse_merge_sliced_kernel(
    const float* __restrict__ part, const float* __restrict__ lse, const int32_t* __restrict__ mptr,
    const int32_t* __restrict__ mrows, const int32_t* __restrict__ mtok, void* __restrict__ out,
    float* __restrict__ lse_out, int q_heads) {
  __shared__ float sh_m[kMergeSlices];
  __shared__ float sh_w[kMergeSlices];
  __shared__ float4 sh_acc[kMergeSlices][32];
  const int t = mtok[blockIdx.x], hd = blockIdx.y;
  const int b = mptr[t], e = mptr[t + 1];
  const int sl = threadIdx.x >> 5, c4 = threadIdx.x & 31;
  // (both walks take four entries at a time so that their loads are in flight together)
  constexpr int kStep = 4 * kMergeSlices;
  float m = -INFINITY;
  int j0 = b + sl;
  for (; j0 + 3 * kMergeSlices < e; j0 += kStep) {
    const float l0 = lse[(size_t)mrows[j0] * q_heads + hd], l1 = lse[(size_t)mrows[j0 + kMergeSlices] * q_heads + hd];
    const float l2 = lse[(size_t)mrows[j0 + 2 * kMergeSlices] * q_heads + hd], l3 = lse[(size_t)mrows[j0 + 3 * kMergeSlices] * q_heads + hd];
    m = fmaxf(fmaxf(m, fmaxf(l0, l1)), fmaxf(l2, l3));
  }
  for (; j0 < e; j0 += kMergeSlices) m = fmaxf(m, lse[(size_t)mrows[j0] * q_heads + hd]);
  if (c4 == 0) sh_m[sl] = m;
  __syncthreads();
  float M = sh_m[0];
#pragma unroll
  for (int i = 1; i < kMergeSlices; ++i) M = fmaxf(M, sh_m[i]);
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  float wsum = 0.f;
  if (M > -INFINITY) {
    auto add = [&](float l, const float4& v) {
      const float w = expf(l - M);
      acc.x += w * v.x; acc.y += w * v.y; acc.z += w * v.z; acc.w += w * v.w;
      wsum += w;
    };
    int jj = b + sl;
    for (; jj + 3 * kMergeSlices < e; jj += kStep) {
      size_t row[4];
      float l[4];
      float4 v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) row[u] = (size_t)mrows[jj + u * kMergeSlices] * q_heads + hd;
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        l[u] = lse[row[u]];
        v[u] = ((const float4*)part)[row[u] * 32 + c4];
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) add(l[u], v[u]);       // same order as one by one
    }
    for (; jj < e; jj += kMergeSlices) {
      const size_t row = (size_t)mrows[jj] * q_heads + hd;
      add(lse[row], ((const float4*)part)[row * 32 + c4]);
    }
  }
  sh_acc[sl][c4] = acc;
  if (c4 == 0) sh_w[sl] = wsum;
  __syncthreads();
  if (sl == 0) {
    acc = sh_acc[0][c4];
    wsum = sh_w[0];
#pragma unroll
    for (int i = 1; i < kMergeSlices; ++i) {
      const float4 v = sh_acc[i][c4];
      acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
      wsum += sh_w[i];
    }
    if (M > -INFINITY) {
      const float inv = 1.f / wsum;
      acc.x *= inv; acc.y *= inv; acc.z *= inv; acc.w *= inv;
    }
    const size_t orow = (size_t)t * q_heads + hd;
    if (OUT_BF16) {
      typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
      f32x4 f = {acc.x, acc.y, acc.z, acc.w};
      ((bf16x4_t*)out)[orow * 32 + c4] = __builtin_convertvector(f, bf16x4_t);
    } else {
      ((float4*)out)[orow * 32 + c4] = acc;
    }
    if (lse_out && c4 == 0) lse_out[orow] = M > -INFINITY ? M + logf(wsum) : -INFINITY;
  }
}

// Self block of a request with one new token (decode): the token sees itself only, so its
// partial is O = v, LSE = scale * <q, k>.  32 lanes per (token, head), 4 channels each.
__global__ __launch_bounds__(256) void single_token_self_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
                                                                const uint16_t* __restrict__ v,
                                                                const int32_t* __restrict__ stok, int n_pairs,
                                                                float* __restrict__ part, float* __restrict__ lse,
                                                                int self_base, int q_heads, int group, float scale) {
  const int pair = blockIdx.x * 8 + (threadIdx.x >> 5), c4 = threadIdx.x & 31;
  if (pair >= n_pairs) return;              // whole 32-lane groups leave together
  const int t = stok[pair / q_heads], hd = pair % q_heads, g = hd / group, kv_heads = q_heads / group;
  const uint2 qb = ((const uint2*)(q + ((size_t)t * q_heads + hd) * kHeadDim))[c4];
  const uint2 kb = ((const uint2*)(k + ((size_t)t * kv_heads + g) * kHeadDim))[c4];
  const uint2 vb = ((const uint2*)(v + ((size_t)t * kv_heads + g) * kHeadDim))[c4];
  auto lo = [](uint32_t w) { return __uint_as_float(w << 16); };
  auto hi = [](uint32_t w) { return __uint_as_float(w & 0xffff0000u); };
  float s = lo(qb.x) * lo(kb.x) + hi(qb.x) * hi(kb.x) + lo(qb.y) * lo(kb.y) + hi(qb.y) * hi(kb.y);
#pragma unroll
  for (int off = 16; off >= 1; off >>= 1) s += __shfl_xor(s, off, 32);
  const size_t row = (size_t)(self_base + t) * q_heads + hd;
  ((float4*)part)[row * 32 + c4] = make_float4(lo(vb.x), hi(vb.x), lo(vb.y), hi(vb.y));
  if (c4 == 0) lse[row] = s * scale;
}

void fill_args(AttnArgs& a, const tl_plan* plan, const PlanDev& d, const void* q, float scale, float* out, float* lse) {
  a.q = (const uint16_t*)q;
  a.tok = d.tok;
  a.slots = d.slots;
  a.slot_lm = plan->any_unit_repeat ? d.unit_lm : nullptr;
  a.tile_base = d.tile_base;
  a.part_tile = d.part_tile;
  a.tile_lm = plan->any_repeat ? d.tile_lm : nullptr;   // null: every tile has multiplicity 1
  a.part_lm = plan->any_repeat ? d.part_lm : nullptr;
  a.out = out;
  a.lse = lse;
  a.q_heads = plan->q_heads;
  a.kv_heads = plan->kv_heads;
  a.group = plan->group;
  a.scale = scale;
  a.scale_log2e = scale * 1.4426950408889634f;
  a.k2 = a.v2 = nullptr;
  a.prior_rows = d.prior_rows;
  a.prior_out = nullptr;
  a.prior_lse = nullptr;
  a.final_out = nullptr;
  a.final_lse = nullptr;
  a.final_is_bf16 = 0;
}

}  // namespace
}  // namespace tl

using namespace tl;

namespace {

// one-pass rows of a plan whose block sits at `base` on the device
tl_status fused_rows(const tl_pool* pool, const tl_plan* plan, const void* base, const void* q_dev, const void* k_new_dev,
                     const void* v_new_dev, float scale, const float* prior_partial, const float* prior_lse, void* out_dev,
                     int32_t out_is_bf16, float* lse_out, hipStream_t st) {
  const PlanDev d = plan_dev(plan, base);
  AttnArgs a;
  fill_args(a, plan, d, q_dev, scale, nullptr, nullptr);
  a.prior_out = prior_partial;
  a.prior_lse = prior_lse;
  a.k = (const uint16_t*)pool->k_dev;
  a.v = (const uint16_t*)pool->v_dev;
  a.k2 = (const uint16_t*)k_new_dev;
  a.v2 = (const uint16_t*)v_new_dev;
  a.final_out = out_dev;
  a.final_lse = lse_out;
  a.final_is_bf16 = out_is_bf16 ? 1 : 0;
  a.fill = nullptr;            // the row-tile kernel reads the fills that the plan baked into its tile lists
  a.seg_len = pool->seg_len;
  a.work = d.ftiles;
  a.n_work = (int)plan->ftiles.size();
  return launch_fused_row_tiles(a, a.n_work, st);
}

// ---- for callers that cannot allocate ---------------------------------------------------------
// tl_fused_attn_static stages the plan's work lists in this array instead of hipMalloc'd memory.
// Every GPU the library runs on holds its own copy of the array, at its own address, until the
// process ends.  In host code the array's name is only a handle for hipGetSymbolAddress: the
// device address is looked up once per device, with that device current, and kept.
constexpr size_t kStaticScratchBytes = (size_t)4 << 20;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mu;

tl_status static_scratch(void** out) {
  int dev = -1;
  TL_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) TL_FAIL(TL_EINVAL, "tl_fused_attn_static: device index %d not supported", dev);
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    TL_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) TL_FAIL(TL_EHIP, "tl_fused_attn_static: no device address for the static buffer");
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return TL_OK;
}

}  // namespace

extern "C" {

tl_status tl_fused_attn_static(const tl_pool* pool, tl_plan* plan, const void* q_dev, const void* k_new_dev,
                               const void* v_new_dev, float scale, const float* prior_partial, const float* prior_lse,
                               void* out_dev, int32_t out_is_bf16, float* lse_out, void* stream) {
  if (plan && plan->n_tokens == 0) return TL_OK;
  if (!pool || !plan || !q_dev || !k_new_dev || !v_new_dev || !out_dev) TL_FAIL(TL_EINVAL, "tl_fused_attn_static: null argument");
  tl_status rc = plan_is_current(plan, pool, "tl_fused_attn_static");
  if (rc != TL_OK) return rc;
  if (!(scale > 0.f) || !std::isfinite(scale)) TL_FAIL(TL_EINVAL, "tl_fused_attn_static: scale must be positive and finite");
  if (plan->ftiles.empty()) return TL_OK;
  if (!plan->prior_rows.empty() && (!prior_partial || !prior_lse))
    TL_FAIL(TL_EINVAL, "tl_fused_attn_static: the plan has one-pass tails: the partials of tl_segment_attn are needed");
  if (plan->blob_host.size() > kStaticScratchBytes)
    TL_FAIL(TL_EINVAL, "tl_fused_attn_static: the plan's work lists take %zu bytes, the static buffer holds %zu",
            plan->blob_host.size(), kStaticScratchBytes);
  void* base = nullptr;
  rc = static_scratch(&base);
  if (rc != TL_OK) return rc;
  hipStream_t st = (hipStream_t)stream;
  // the buffer keeps the last call's lists: this call's are copied over them, in stream order
  // (nothing in the buffer has to start at zero)
  TL_HIP(hipMemcpyAsync(base, plan->blob_host.data(), plan->blob_host.size(), hipMemcpyHostToDevice, st));
  return fused_rows(pool, plan, base, q_dev, k_new_dev, v_new_dev, scale, prior_partial, prior_lse, out_dev, out_is_bf16, lse_out, st);
}

tl_status tl_segment_attn(const tl_pool* pool, tl_plan* plan, const void* q_dev, float scale, float* out_partial,
                          float* lse, void* stream) {
  if (plan && plan->n_tokens == 0) return TL_OK;   // a batch without new tokens: nothing to do, buffers may be empty
  if (!pool || !plan || !q_dev || !out_partial || !lse) TL_FAIL(TL_EINVAL, "tl_segment_attn: null argument");
  tl_status rc = plan_is_current(plan, pool, "tl_segment_attn");
  if (rc != TL_OK) return rc;
  if (!(scale > 0.f) || !std::isfinite(scale)) TL_FAIL(TL_EINVAL, "tl_segment_attn: scale must be positive and finite");
  hipStream_t st = (hipStream_t)stream;
  rc = pool_device_ready(pool, st);
  if (rc != TL_OK) return rc;
  rc = plan_device_ready(plan, st);
  if (rc != TL_OK) return rc;
  const PlanDev d = plan_dev(plan, plan->blob_dev);
  AttnArgs a;
  fill_args(a, plan, d, q_dev, scale, out_partial, lse);
  a.k = (const uint16_t*)pool->k_dev;
  a.v = (const uint16_t*)pool->v_dev;
  a.fill = pool->fill_dev;
  a.seg_len = pool->seg_len;
  a.work = d.tiles;
  a.n_work = (int)plan->tiles.size();
  rc = launch_pool_row_tiles(a, a.n_work, st);
  if (rc != TL_OK) return rc;
  a.work = d.units;
  a.n_work = (int)plan->units.size();
  return launch_splitk_units(a, a.n_work, st);
}

tl_status tl_causal_block(tl_plan* plan, const void* q_dev, const void* k_new_dev, const void* v_new_dev, float scale,
                          float* out_partial, float* lse, void* stream) {
  if (plan && plan->n_tokens == 0) return TL_OK;   // a batch without new tokens: nothing to do, buffers may be empty
  if (!plan || !q_dev || !k_new_dev || !v_new_dev || !out_partial || !lse) TL_FAIL(TL_EINVAL, "tl_causal_block: null argument");
  if (!(plan->flags & TL_PLAN_SELF_BLOCK)) TL_FAIL(TL_EINVAL, "tl_causal_block: plan has no self block");
  if (!(scale > 0.f) || !std::isfinite(scale)) TL_FAIL(TL_EINVAL, "tl_causal_block: scale must be positive and finite");
  hipStream_t st = (hipStream_t)stream;
  tl_status rc = plan_device_ready(plan, st);
  if (rc != TL_OK) return rc;
  const PlanDev d = plan_dev(plan, plan->blob_dev);
  AttnArgs a;
  fill_args(a, plan, d, q_dev, scale, out_partial, lse);
  a.k = (const uint16_t*)k_new_dev;
  a.v = (const uint16_t*)v_new_dev;
  a.fill = nullptr;
  a.seg_len = 0;
  a.work = d.ctiles;
  a.n_work = (int)plan->ctiles.size();
  if (!plan->single_tok.empty()) {
    const int n_pairs = (int)plan->single_tok.size() * plan->q_heads;
    hipLaunchKernelGGL(single_token_self_kernel, dim3((unsigned)((n_pairs + 7) / 8)), dim3(256), 0, st,
                       (const uint16_t*)q_dev, (const uint16_t*)k_new_dev, (const uint16_t*)v_new_dev, d.single_tok,
                       n_pairs, out_partial, lse, plan->info.self_row_base, plan->q_heads, plan->group, scale);
    TL_HIP(hipGetLastError());
  }
  return launch_causal_row_tiles(a, a.n_work, st);
}

tl_status tl_fused_attn(const tl_pool* pool, tl_plan* plan, const void* q_dev, const void* k_new_dev,
                        const void* v_new_dev, float scale, const float* prior_partial, const float* prior_lse,
                        void* out_dev, int32_t out_is_bf16, float* lse_out, void* stream) {
  if (plan && plan->n_tokens == 0) return TL_OK;   // a batch without new tokens: nothing to do, buffers may be empty
  if (!pool || !plan || !q_dev || !k_new_dev || !v_new_dev || !out_dev) TL_FAIL(TL_EINVAL, "tl_fused_attn: null argument");
  tl_status rc = plan_is_current(plan, pool, "tl_fused_attn");
  if (rc != TL_OK) return rc;
  if (!(scale > 0.f) || !std::isfinite(scale)) TL_FAIL(TL_EINVAL, "tl_fused_attn: scale must be positive and finite");
  if (plan->ftiles.empty()) return TL_OK;
  if (!plan->prior_rows.empty() && (!prior_partial || !prior_lse))
    TL_FAIL(TL_EINVAL, "tl_fused_attn: the plan has one-pass tails: the partials of tl_segment_attn are needed");
  hipStream_t st = (hipStream_t)stream;
  rc = plan_device_ready(plan, st);
  if (rc != TL_OK) return rc;
  return fused_rows(pool, plan, plan->blob_dev, q_dev, k_new_dev, v_new_dev, scale, prior_partial, prior_lse, out_dev,
                    out_is_bf16, lse_out, st);
}

tl_status tl_merge(tl_plan* plan, const float* out_partial, const float* lse, void* out_dev, int32_t out_is_bf16,
                   float* lse_out, void* stream) {
  if (plan && plan->n_tokens == 0) return TL_OK;   // a batch without new tokens: nothing to do, buffers may be empty
  if (!plan || !out_partial || !lse || !out_dev) TL_FAIL(TL_EINVAL, "tl_merge: null argument");
  hipStream_t st = (hipStream_t)stream;
  tl_status rc = plan_device_ready(plan, st);
  if (rc != TL_OK) return rc;
  if (plan->merge_tok.empty()) return TL_OK;
  const PlanDev d = plan_dev(plan, plan->blob_dev);
  const int n_short = plan->n_merge_short, n_long = (int)plan->merge_tok.size() - n_short;
  if (n_short > 0) {
    const dim3 grid((unsigned)n_short, (unsigned)((plan->q_heads * 32 + 255) / 256)), block(256);
    if (out_is_bf16)
      hipLaunchKernelGGL(lse_merge_kernel<true>, grid, block, 0, st, out_partial, lse, d.merge_fix, out_dev, lse_out,
                         plan->q_heads);
    else
      hipLaunchKernelGGL(lse_merge_kernel<false>, grid, block, 0, st, out_partial, lse, d.merge_fix, out_dev, lse_out,
                         plan->q_heads);
  }
  if (n_long > 0) {
    // long merge lists (split-K): the sliced kernel, one workgroup per (token, head)
    const dim3 grid((unsigned)n_long, (unsigned)plan->q_heads), block(32 * kMergeSlices);
    if (out_is_bf16)
      hipLaunchKernelGGL(lse_merge_sliced_kernel<true>, grid, block, 0, st, out_partial, lse, d.merge_ptr, d.merge_rows,
                         d.merge_tok + n_short, out_dev, lse_out, plan->q_heads);
    else
      hipLaunchKernelGGL(lse_merge_sliced_kernel<false>, grid, block, 0, st, out_partial, lse, d.merge_ptr, d.merge_rows,
                         d.merge_tok + n_short, out_dev, lse_out, plan->q_heads);
  }
  TL_HIP(hipGetLastError());
  return TL_OK;
}

}  // extern "C"
