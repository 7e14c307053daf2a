// libdsk_diag: measurements of the device itself, kept out of the product library (libdsk.so).
// Matrix-core peak: a register-only loop of v_mfma_f32_32x32x16_bf16 on independent accumulators, two waves per
// SIMD on every CU.  bench.py quotes utilisation against this figure next to the one against the spec-sheet peak.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dsk_diag.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kProbeThreads = 512;     // 8 waves per workgroup: 2 per SIMD
constexpr int kMfmaPerIter = 8;

__global__ void __launch_bounds__(kProbeThreads) mfma_peak_kernel(float* __restrict__ out, int iters) {
  f32x16 acc[4];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[a][r] = 0.f;
  bf16x8 x, y;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    x[e] = (__bf16)(0.001f * (float)(threadIdx.x & 63));
    y[e] = (__bf16)(0.01f * (float)e);
  }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < kMfmaPerIter; ++j) acc[j & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, y, acc[j & 3], 0, 0, 0);
  }
  float sum = 0.f;
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int r = 0; r < 16; ++r) sum += acc[a][r];
  out[(int64_t)blockIdx.x * kProbeThreads + threadIdx.x] = sum;
}

}  // namespace

extern "C" int dsk_diag_mfma_peak(double* tflops, void* stream) {
  if (!tflops) return -1;
  hipStream_t s = (hipStream_t)stream;
  int dev = 0, n_cu = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e == hipSuccess) e = hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev);
  float* out = nullptr;
  hipEvent_t t0 = nullptr, t1 = nullptr;
  const int blocks = n_cu > 0 ? n_cu : 256;
  const int iters = 20000;
  if (e == hipSuccess) e = hipMalloc(&out, (size_t)blocks * kProbeThreads * sizeof(float));
  if (e == hipSuccess) e = hipEventCreate(&t0);
  if (e == hipSuccess) e = hipEventCreate(&t1);
  float ms = 0.f;
  if (e == hipSuccess) {
    hipLaunchKernelGGL(mfma_peak_kernel, dim3(blocks), dim3(kProbeThreads), 0, s, out, 100);  // warm-up
    e = hipEventRecord(t0, s);
    hipLaunchKernelGGL(mfma_peak_kernel, dim3(blocks), dim3(kProbeThreads), 0, s, out, iters);
    if (e == hipSuccess) e = hipEventRecord(t1, s);
    if (e == hipSuccess) e = hipEventSynchronize(t1);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, t0, t1);
  }
  if (t0) (void)hipEventDestroy(t0);
  if (t1) (void)hipEventDestroy(t1);
  if (out) (void)hipFree(out);
  if (e != hipSuccess) return -5;
  const double flops = (double)blocks * (kProbeThreads / 64) * (double)iters * kMfmaPerIter * 2.0 * 32 * 32 * 16;
  *tflops = flops / ((double)ms * 1e-3) / 1e12;
  return 0;
}
