// Measurement aid for bench.py, not part of the attention path: register-resident back-to-back
// v_mfma_f32_32x32x16_bf16 on every SIMD of the chip, to quote the kernels' rate against a measured matrix
// peak next to the vendor figure: once with operands that never change and once with operands that toggle the
// datapath like real activations (the chip clocks lower then).  Built into its own small library.
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

namespace {
constexpr int kChains = 4;   // independent accumulators per wave
constexpr int kFrags = 8;    // operand fragments a wave rotates through when the data varies

__device__ __forceinline__ float hashed(unsigned x) {   // deterministic value in [-2, 2)
  x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
  return (float)(x & 0xffff) * (4.f / 65536.f) - 2.f;
}

// VARIED = false: every instruction multiplies the same two fragments of small values, so hardly a bit changes
// between instructions and the chip draws little power.  VARIED = true: the wave rotates through kFrags
// fragments of pseudo-random values per operand, the way real activations toggle the datapath.
template <bool VARIED>
__global__ void __launch_bounds__(256, 2) mfma_peak_kernel(float *sink, int iters) {
  const int tid = threadIdx.x;
  bf16x8 a[kFrags], b[kFrags];
#pragma unroll
  for (int f = 0; f < kFrags; ++f)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if (VARIED) {
        a[f][i] = (__bf16)hashed((unsigned)((blockIdx.x * 256 + tid) * 64 + f * 8 + i));
        b[f][i] = (__bf16)hashed(0x9e3779b9U + (unsigned)((blockIdx.x * 256 + tid) * 64 + f * 8 + i));
      } else {
        a[f][i] = (__bf16)(0.001f * (float)((tid + i) & 7));
        b[f][i] = (__bf16)(0.002f * (float)((tid + 3 * i) & 7));
      }
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
      for (int j = 0; j < kChains; ++j) {
        const int f = VARIED ? (4 * r + j) % kFrags : 0, h = VARIED ? (4 * r + j + 3 * r) % kFrags : 0;
        c[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[f], b[h], c[j], 0, 0, 0);
      }
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
// instructions (32768 flops per instruction and wave).  `varied_data` != 0 feeds pseudo-random operands that
// change from instruction to instruction, 0 the same small constants every time.  `sink` is device memory of at
// least workgroups * 256 floats.  Returns 0, or 1 on a bad argument or a launch failure.
extern "C" int s1f_probe_mfma_bf16(int workgroups, int iters, int varied_data, float *sink, void *hip_stream) {
  if (workgroups < 1 || iters < 1 || !sink) return 1;
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  if (varied_data) hipLaunchKernelGGL(mfma_peak_kernel<true>, dim3((unsigned)workgroups), dim3(256), 0, st, sink, iters);
  else hipLaunchKernelGGL(mfma_peak_kernel<false>, dim3((unsigned)workgroups), dim3(256), 0, st, sink, iters);
  return hipGetLastError() == hipSuccess ? 0 : 1;
}
