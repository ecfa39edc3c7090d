// Measurement aid for bench.py, not part of the attention path: register-resident back-to-back
// v_mfma_f32_32x32x16_bf16 on every SIMD of the chip, to quote the kernels' rate against a measured matrix
// peak next to the vendor figure.  Built into its own small library.
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

namespace {
constexpr int kChains = 4;   // independent accumulators per wave

__global__ void __launch_bounds__(256, 2) mfma_peak_kernel(float *sink, int iters) {
  const int tid = threadIdx.x;
  bf16x8 a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = (__bf16)(0.001f * (float)((tid + i) & 7));
    b[i] = (__bf16)(0.002f * (float)((tid + 3 * i) & 7));
  }
  f32x16 c[kChains];
#pragma unroll
  for (int j = 0; j < kChains; ++j)
#pragma unroll
    for (int v = 0; v < 16; ++v) c[j][v] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
      for (int j = 0; j < kChains; ++j) c[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c[j], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < kChains; ++j)
#pragma unroll
    for (int v = 0; v < 16; ++v) s += c[j][v];
  if (s == 12345.678f) sink[blockIdx.x * 256 + tid] = s;   // keeps the products alive; never true in practice
}
}  // namespace

// Launches the probe on `hip_stream`: `workgroups` x 256 threads, each wave issuing 16 * iters matrix
// instructions (32768 flops per instruction and wave).  `sink` is device memory of at least
// workgroups * 256 floats.  Returns 0, or 1 on a bad argument or a launch failure.
extern "C" int s1f_probe_mfma_bf16(int workgroups, int iters, float *sink, void *hip_stream) {
  if (workgroups < 1 || iters < 1 || !sink) return 1;
  hipLaunchKernelGGL(mfma_peak_kernel, dim3((unsigned)workgroups), dim3(256), 0, reinterpret_cast<hipStream_t>(hip_stream),
                     sink, iters);
  return hipGetLastError() == hipSuccess ? 0 : 1;
}
