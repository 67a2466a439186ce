// Device probe: what an MFMA and the vector instructions of a softmax cost in issue cycles on
// one SIMD, alone and together, with one or two waves per SIMD.  Fixed-count loops on registers
// only; every wave stamps the cycle counter before and after its loop.  A measurement aid for the
// benchmark (built into libtlprobe.so, which only bench.py loads), no part of the method.
#include <hip/hip_runtime.h>

#include <cstdint>

namespace {

typedef __bf16 iprobe_bf16x8 __attribute__((ext_vector_type(8)));
typedef float iprobe_f32x16 __attribute__((ext_vector_type(16)));

#define IP_FMA(x) asm volatile("v_fma_f32 %0, %0, %1, %2" : "+v"(x) : "v"(ca), "v"(cb))
#define IP_ADD(x) asm volatile("v_add_f32 %0, %0, %1" : "+v"(x) : "v"(cb))
#define IP_EXP(x) asm volatile("v_exp_f32 %0, %0" : "+v"(x))
#define IP_CVT(u, x, y) asm volatile("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(u) : "v"(x), "v"(y))
#define IP_MAX3(x, y, z) asm volatile("v_max3_f32 %0, %0, %1, %2" : "+v"(x) : "v"(y), "v"(z))
#define IP_PERM(u, x, y) asm volatile("v_perm_b32 %0, %1, %2, %3" : "=v"(u) : "v"(x), "v"(y), "s"(0x07060302u))

// One loop iteration = 4 groups.  MODE:
//   0..5  eight instructions of one kind per group: v_fma, v_add, v_exp, v_cvt_pk_bf16_f32, v_max3, v_perm_b32
//   10    one MFMA per group
//   11    one MFMA + one element's softmax (fma, exp, add, a convert in every other group)
//   12    one MFMA + two elements' softmax
//   20    waves 0-3: one MFMA per group; waves 4-7: eight v_fma per group
template <int MODE>
__global__ __launch_bounds__(512) void issue_probe_kernel(unsigned long long* out, int iters) {
  extern __shared__ char iprobe_lds[];      // only there to keep one workgroup per CU
  const int wave = threadIdx.x >> 6;
  float x[8];
  for (int i = 0; i < 8; ++i) x[i] = 0.001f * (threadIdx.x + i);
  const float ca = 0.999f, cb = 0.0001f;
  unsigned u[4] = {0, 0, 0, 0};
  iprobe_bf16x8 a, b;
  for (int i = 0; i < 8; ++i) {
    a[i] = (__bf16)(0.01f * (threadIdx.x % 7 + i));
    b[i] = (__bf16)(0.02f * (threadIdx.x % 5 + i));
  }
  iprobe_f32x16 acc[4];
  for (int i = 0; i < 4; ++i)
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  const bool do_m = MODE >= 10 && (MODE != 20 || wave < 4), do_v = MODE != 20 || wave >= 4;
  __syncthreads();
  const unsigned long long t0 = clock64();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      if (do_m) {
        acc[g] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[g], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
      if (do_v) {
        if (MODE == 0 || MODE == 20) { IP_FMA(x[0]); IP_FMA(x[1]); IP_FMA(x[2]); IP_FMA(x[3]); IP_FMA(x[4]); IP_FMA(x[5]); IP_FMA(x[6]); IP_FMA(x[7]); }
        if (MODE == 1) { IP_ADD(x[0]); IP_ADD(x[1]); IP_ADD(x[2]); IP_ADD(x[3]); IP_ADD(x[4]); IP_ADD(x[5]); IP_ADD(x[6]); IP_ADD(x[7]); }
        if (MODE == 2) { IP_EXP(x[0]); IP_EXP(x[1]); IP_EXP(x[2]); IP_EXP(x[3]); IP_EXP(x[4]); IP_EXP(x[5]); IP_EXP(x[6]); IP_EXP(x[7]); }
        if (MODE == 3) { IP_CVT(u[0], x[0], x[1]); IP_CVT(u[1], x[2], x[3]); IP_CVT(u[2], x[4], x[5]); IP_CVT(u[3], x[6], x[7]); IP_CVT(u[0], x[1], x[2]); IP_CVT(u[1], x[3], x[4]); IP_CVT(u[2], x[5], x[6]); IP_CVT(u[3], x[7], x[0]); }
        if (MODE == 4) { IP_MAX3(x[0], x[1], x[2]); IP_MAX3(x[3], x[4], x[5]); IP_MAX3(x[6], x[7], x[1]); IP_MAX3(x[2], x[4], x[6]); IP_MAX3(x[0], x[3], x[5]); IP_MAX3(x[1], x[2], x[7]); IP_MAX3(x[4], x[0], x[6]); IP_MAX3(x[5], x[3], x[1]); }
        if (MODE == 5) { IP_PERM(u[0], x[0], x[1]); IP_PERM(u[1], x[2], x[3]); IP_PERM(u[2], x[4], x[5]); IP_PERM(u[3], x[6], x[7]); IP_PERM(u[0], x[1], x[2]); IP_PERM(u[1], x[3], x[4]); IP_PERM(u[2], x[5], x[6]); IP_PERM(u[3], x[7], x[0]); }
        if (MODE == 11 || MODE == 12) {
#pragma unroll
          for (int j = 0; j < MODE - 10; ++j) {
            IP_FMA(x[(g + j) & 7]); IP_EXP(x[(g + j + 3) & 7]); IP_ADD(x[(g + j + 5) & 7]);
            if ((g + j) & 1) IP_CVT(u[g & 3], x[g & 7], x[(g + 1) & 7]);
          }
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  const unsigned long long t1 = clock64();
  float s = 0;
  for (int i = 0; i < 8; ++i) s += x[i];
  for (int i = 0; i < 4; ++i) s += acc[i][0] + (float)u[i];
  if ((threadIdx.x & 63) == 0) out[blockIdx.x * 8 + wave] = t1 - t0;
  if (s == 1.2345f) { out[0] = 0; iprobe_lds[threadIdx.x] = 1; }     // keeps the loop alive; practically never true
}

template <int MODE>
int launch_issue(unsigned long long* out, int waves_per_simd, int iters, hipStream_t st) {
  const int lds = 100 * 1024;
  if (hipFuncSetAttribute((const void*)issue_probe_kernel<MODE>, hipFuncAttributeMaxDynamicSharedMemorySize, lds) != hipSuccess) return -5;
  hipLaunchKernelGGL((issue_probe_kernel<MODE>), dim3(256), dim3(256 * waves_per_simd), lds, st, out, iters);
  return hipGetLastError() == hipSuccess ? 0 : -5;
}

}  // namespace

// Runs one variant (mode as listed at issue_probe_kernel) with 1 or 2 waves per SIMD on 256 workgroups and returns, for
// workgroup 5, the cycles per group (a quarter of a loop iteration) of waves 0-3 and of waves 4-7 (0 with one wave per
// SIMD), averaged over the four waves.  Allocates and frees a small device buffer and waits for the kernel.
// Returns 0, -1 for a bad argument, -5 for a HIP error.
extern "C" int32_t tlprobe_issue(int32_t mode, int32_t waves_per_simd, int32_t iters, double* cycles_first, double* cycles_second) {
  if (iters <= 0 || iters > (1 << 20) || (waves_per_simd != 1 && waves_per_simd != 2) || !cycles_first || !cycles_second) return -1;
  if (mode == 20 && waves_per_simd != 2) return -1;
  unsigned long long* d = nullptr;
  if (hipMalloc((void**)&d, 256 * 8 * sizeof(unsigned long long)) != hipSuccess) return -5;
  int rc = -1;
  for (int rep = 0; rep < 2 && (rep == 0 || rc == 0); ++rep) {     // the second launch is the one that is read
    switch (mode) {
      case 0: rc = launch_issue<0>(d, waves_per_simd, iters, 0); break;
      case 1: rc = launch_issue<1>(d, waves_per_simd, iters, 0); break;
      case 2: rc = launch_issue<2>(d, waves_per_simd, iters, 0); break;
      case 3: rc = launch_issue<3>(d, waves_per_simd, iters, 0); break;
      case 4: rc = launch_issue<4>(d, waves_per_simd, iters, 0); break;
      case 5: rc = launch_issue<5>(d, waves_per_simd, iters, 0); break;
      case 10: rc = launch_issue<10>(d, waves_per_simd, iters, 0); break;
      case 11: rc = launch_issue<11>(d, waves_per_simd, iters, 0); break;
      case 12: rc = launch_issue<12>(d, waves_per_simd, iters, 0); break;
      case 20: rc = launch_issue<20>(d, waves_per_simd, iters, 0); break;
      default: rc = -1;
    }
    if (rc == 0 && hipDeviceSynchronize() != hipSuccess) rc = -5;
  }
  unsigned long long h[16] = {0};
  if (rc == 0 && hipMemcpy(h, d + 5 * 8, sizeof(unsigned long long) * 8, hipMemcpyDeviceToHost) != hipSuccess) rc = -5;
  (void)hipFree(d);
  if (rc != 0) return rc;
  double lo = 0, hi = 0;
  for (int w = 0; w < 4; ++w) lo += (double)h[w];
  for (int w = 4; w < 4 * waves_per_simd; ++w) hi += (double)h[w];
  *cycles_first = lo / 4 / iters / 4;
  *cycles_second = waves_per_simd == 2 ? hi / 4 / iters / 4 : 0.0;
  return 0;
}
