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
