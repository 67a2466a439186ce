// Device probe: what the matrix unit sustains by itself.  A loop of nothing but
// v_mfma_f32_32x32x16_bf16 (4 independent accumulators per wave, 8 waves per workgroup, 4
// workgroups per CU's worth of grid), either with constant operands or with operands that
// change with every instruction (pseudo-random signs and mantissas, magnitudes 2^-3..2^1, like
// the N(0,1) inputs of the attention workloads).  The second draws far more power and the GPU
// lowers its clock under it: the roofline discussion needs both numbers.
//
// A measurement aid for the benchmark, no part of the method and no part of libtokenlake.so: it
// is built into a small library of its own (libtlprobe.so) that only bench.py loads.
#include <hip/hip_runtime.h>

#include <cstdint>

namespace {

typedef __bf16 probe_bf16x8 __attribute__((ext_vector_type(8)));
typedef float probe_f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned probe_u32x4 __attribute__((ext_vector_type(4)));

__device__ inline unsigned probe_mix(unsigned x) {
  x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
  return x;
}
// two bf16 values with random sign and mantissa, exponent 2^-3 .. 2^0
__device__ inline unsigned probe_pair(unsigned seed) {
  const unsigned r = probe_mix(seed);
  const unsigned lo = (r & 0x807f) | ((124 + ((r >> 8) & 3)) << 7);
  const unsigned hi = ((r >> 16) & 0x807f) | ((124 + ((r >> 24) & 3)) << 7);
  return lo | (hi << 16);
}

template <int RANDOM>
__global__ __launch_bounds__(512) void mfma_probe_kernel(float* out, int iters) {
  probe_u32x4 a[8], b[8];
  for (int i = 0; i < 8; ++i)
    for (int e = 0; e < 4; ++e) {
      a[i][e] = RANDOM ? probe_pair(threadIdx.x * 64 + i * 4 + e + 1) : 0x3f803f80u;
      b[i][e] = RANDOM ? probe_pair(threadIdx.x * 64 + i * 4 + e + 77777) : 0x3f803f80u;
    }
  probe_f32x16 acc[4];
  for (int i = 0; i < 4; ++i)
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 8; ++u)
#pragma unroll
      for (int i = 0; i < 4; ++i)
        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(probe_bf16x8, a[(u + i) & 7]),
                                                         __builtin_bit_cast(probe_bf16x8, b[(u + 3 * i) & 7]), acc[i], 0, 0, 0);
  }
  float s = 0;
  for (int i = 0; i < 4; ++i)
    for (int r = 0; r < 16; ++r) s += acc[i][r];
  if (s == 1.2345f) out[0] = s;     // keeps the loop alive; practically never true
}


// Variants for the question of what the matrix unit's power depends on.
//   KIND 0: both operands random (sign, mantissa, exponent 2^-3..2^0), fixed for the whole loop
//        1: +-1.0 with random signs, changing          2: random mantissas at one exponent, positive, changing
//        3: A changing as in the kernel above, B = 1.0  4: A = 1.0, B changing
//        5: both changing, and IDLE > 0: after every IDLE-th MFMA the wave idles (s_nop), so that the
//           same instructions on the same operands take more cycles (one wave per SIMD: the launch
//           asks for enough LDS that a workgroup of 4 waves has a CU to itself)
template <int KIND> __device__ inline unsigned probe_pair_kind(unsigned seed) {
  const unsigned r = probe_mix(seed);
  if (KIND == 1) return (r & 0x8000) | 0x3f80 | ((((r >> 16) & 0x8000) | 0x3f80) << 16);
  if (KIND == 2) return (r & 0x7f) | (127 << 7) | ((((r >> 16) & 0x7f) | (127 << 7)) << 16);
  return probe_pair(seed);
}
template <int KIND, int IDLE>
__global__ __launch_bounds__(256) void mfma_probe_kind_kernel(float* out, int iters) {
  extern __shared__ char probe_lds[];
  probe_u32x4 a[8], b[8];
  for (int i = 0; i < 8; ++i)
    for (int e = 0; e < 4; ++e) {
      a[i][e] = KIND == 4 ? 0x3f803f80u : probe_pair_kind<KIND>(threadIdx.x * 64 + i * 4 + e + 1);
      b[i][e] = KIND == 3 ? 0x3f803f80u : probe_pair_kind<KIND>(threadIdx.x * 64 + i * 4 + e + 77777);
    }
  probe_f32x16 acc[4];
  for (int i = 0; i < 4; ++i)
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 8; ++u)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int ia = KIND == 0 ? 0 : (u + i) & 7, ib = KIND == 0 ? 0 : (u + 3 * i) & 7;
        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(probe_bf16x8, a[ia]),
                                                         __builtin_bit_cast(probe_bf16x8, b[ib]), acc[i], 0, 0, 0);
        if (IDLE > 0 && (u * 4 + i) % IDLE == 0) asm volatile("s_nop 7");
      }
  }
  float s = 0;
  for (int i = 0; i < 4; ++i)
    for (int r = 0; r < 16; ++r) s += acc[i][r];
  if (s == 1.2345f) { out[0] = s; probe_lds[threadIdx.x] = 1; }
}

template <int KIND, int IDLE>
int launch_kind(float* out, int iters, hipStream_t st) {
  const int lds = IDLE > 0 ? 100 * 1024 : 0;
  if (lds && hipFuncSetAttribute((const void*)mfma_probe_kind_kernel<KIND, IDLE>, hipFuncAttributeMaxDynamicSharedMemorySize, lds) != hipSuccess)
    return -5;
  hipLaunchKernelGGL((mfma_probe_kind_kernel<KIND, IDLE>), dim3(IDLE > 0 ? 1024 : 2048), dim3(256), lds, st, out, iters);
  return hipGetLastError() == hipSuccess ? 0 : -5;
}

}  // namespace

// Enqueues the probe on `stream`: 1024 workgroups of 8 waves, iters x 32 MFMAs per wave, with constant
// operands (random_operands = 0) or operands that differ from instruction to instruction.
// scratch_dev: device, at least 4 bytes (practically never written).  *flops_out = floating-point
// operations of the launch; the caller times it.  Returns 0, -1 for a bad argument, -5 for a HIP error.
extern "C" int32_t tlprobe_mfma(int32_t random_operands, int32_t iters, void* scratch_dev, double* flops_out, void* stream) {
  if (iters <= 0 || iters > (1 << 20) || !scratch_dev || !flops_out) return -1;
  const int wgs = 1024, threads = 512;
  hipStream_t st = (hipStream_t)stream;
  if (random_operands)
    hipLaunchKernelGGL(mfma_probe_kernel<1>, dim3(wgs), dim3(threads), 0, st, (float*)scratch_dev, iters);
  else
    hipLaunchKernelGGL(mfma_probe_kernel<0>, dim3(wgs), dim3(threads), 0, st, (float*)scratch_dev, iters);
  if (hipGetLastError() != hipSuccess) return -5;
  *flops_out = (double)wgs * (threads / 64) * (double)iters * 32.0 * 32768.0;
  return 0;
}

// The variants above: kind 0..5 as listed at mfma_probe_kind_kernel; idle_every (kind 5 only) = 0, 32, 16, 8, 4 or 2:
// the wave idles after every idle_every-th MFMA.  Same arguments and return values as tlprobe_mfma.
extern "C" int32_t tlprobe_mfma_kind(int32_t kind, int32_t idle_every, int32_t iters, void* scratch_dev, double* flops_out, void* stream) {
  if (iters <= 0 || iters > (1 << 20) || !scratch_dev || !flops_out) return -1;
  hipStream_t st = (hipStream_t)stream;
  float* o = (float*)scratch_dev;
  int rc = -1;
  if (kind == 0 && idle_every == 0) rc = launch_kind<0, 0>(o, iters, st);
  else if (kind == 1 && idle_every == 0) rc = launch_kind<1, 0>(o, iters, st);
  else if (kind == 2 && idle_every == 0) rc = launch_kind<2, 0>(o, iters, st);
  else if (kind == 3 && idle_every == 0) rc = launch_kind<3, 0>(o, iters, st);
  else if (kind == 4 && idle_every == 0) rc = launch_kind<4, 0>(o, iters, st);
  else if (kind == 5 && idle_every == 0) rc = launch_kind<5, 0>(o, iters, st);
  else if (kind == 5 && idle_every == 32) rc = launch_kind<5, 32>(o, iters, st);
  else if (kind == 5 && idle_every == 16) rc = launch_kind<5, 16>(o, iters, st);
  else if (kind == 5 && idle_every == 8) rc = launch_kind<5, 8>(o, iters, st);
  else if (kind == 5 && idle_every == 4) rc = launch_kind<5, 4>(o, iters, st);
  else if (kind == 5 && idle_every == 2) rc = launch_kind<5, 2>(o, iters, st);
  if (rc != 0) return rc;
  const int wgs = idle_every > 0 ? 1024 : 2048;
  *flops_out = (double)wgs * 4 * (double)iters * 32.0 * 32768.0;
  return 0;
}
