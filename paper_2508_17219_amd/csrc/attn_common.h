// Device-side helpers shared by the attention kernels (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>

#include "tl_internal.h"

namespace tl {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// LDS rows of the split-K unit kernel are padded from 128 bf16.  K rows: 136 (272 B), so that the
// 16-byte reads of 16 consecutive rows fall in different banks; V rows: 144 (288 B = 32 mod 256)
// for the 8 rows x 32 B of its transposing reads.  (The row-tile kernel keeps unpadded rows and
// swizzles 16-byte chunks instead, because direct global->LDS loads write contiguously.)
constexpr int kLdsStride = 136;
constexpr int kVStrideUnit = 144;

struct AttnArgs {
  const uint16_t* q;      // [n_tokens, q_heads, 128] bf16
  const uint16_t* k;      // pool K base, or new-token K [n_tokens, kv_heads, 128]
  const uint16_t* v;
  const uint16_t* k2;     // fused rows only: the new tokens' K/V [n_tokens, kv_heads, 128]
  const uint16_t* v2;
  void* final_out;        // fused rows only: [n_tokens, q_heads, 128] fp32 or bf16
  float* final_lse;       // fused rows only: [n_tokens, q_heads] or null
  int32_t final_is_bf16;
  const int32_t* fill;    // per-slot valid tokens (pool work)
  const Work* work;
  const int32_t* tok;     // token index lists
  const int32_t* slots;   // slot lists of the split-K units
  const float* slot_lm;   // log2(times the unit's run lists the slot), parallel to slots; null = all once
  const int32_t* tile_base;  // first kv row of each full 64-token tile (pool row tiles)
  const int32_t* part_tile;  // (first kv row, valid tokens) of each cut-short tile
  const float* tile_lm;      // log2(times the tile's slot is listed), parallel to tile_base
  const float* part_lm;      // the same for the cut-short tiles
  const int32_t* prior_rows;  // one-pass tails: partial rows to merge in (see Work::prior_off)
  const float* prior_out;     // [rows, q_heads, 128] partials written by an earlier launch
  const float* prior_lse;     // [rows, q_heads]
  float* out;             // [rows, q_heads, 128]
  float* lse;             // [rows, q_heads]
  int32_t q_heads, kv_heads, group, seg_len, n_work;   // group = q_heads / kv_heads
  float scale;            // softmax scale
  float scale_log2e;      // scale * log2(e)
};

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ bf16x8 pack_bf16x8(float a0, float a1, float a2, float a3, float a4, float a5, float a6,
                                              float a7) {
  f32x8 f = {a0, a1, a2, a3, a4, a5, a6, a7};
  return __builtin_convertvector(f, bf16x8);
}

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 u) { return __builtin_bit_cast(bf16x8, u); }

// acc + lo + hi of a packed pair of bf16 values (one v_dot2c_f32_bf16 against the pair (1, 1)):
// the running sum of the probabilities as the matrix unit sees them, after rounding
__device__ __forceinline__ float add_bf16_pair(float acc, unsigned pair) {
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, pair), __builtin_bit_cast(bf16x2_t, 0x3f803f80u), acc,
                                         false);
}

typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

// Transposing LDS read: within each group of 16 lanes, lane j supplies the address of 4
// consecutive bf16 (row j/4, columns 4*(j%4)..+3 of a 4 x 16 block); lane i receives column
// i of that block, rows 0..3.
__device__ __forceinline__ s16x4 lds_read_tr(const uint16_t* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)p);
}

__device__ __forceinline__ bf16x8 join_tr(s16x4 lo, s16x4 hi) {
  s16x8 r = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return __builtin_bit_cast(bf16x8, r);
}

}  // namespace tl
