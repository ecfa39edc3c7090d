// Measurement aids for bench.py, not part of the attention path.
// (1) Register-resident back-to-back
// v_mfma_f32_32x32x16_bf16 on every SIMD of the chip, to quote the kernels' rate against a measured matrix
// peak next to the vendor figure: once with operands that never change and once with operands that toggle the
// datapath like real activations (the chip clocks lower then).
// (2) The rate of fp32 global atomic adds in the access shape a dK/dV kernel would need to accumulate dQ as well
// (the measurement behind keeping dQ in a kernel of its own).  Built into their own small library.
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

namespace {
// Each wave adds (mode 0: atomically; mode 1: plain stores, for comparison) 32 rows x 32 floats per step, rows
// 512 bytes apart, walking over a [rows x 128] fp32 array shared by the workgroups of one head; heads are spread
// over the XCDs the way the attention kernels spread them (workgroup id modulo 8).
__global__ void __launch_bounds__(256) dq_atomics_kernel(float *acc, int rows, int n_heads, int steps, int mode) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, ln = lane & 31, g = lane >> 5;
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int wg_per_head = gridDim.x / n_heads;
  const int head = xcd + 8 * (slot / wg_per_head), wg = slot % wg_per_head;
  float *base = acc + (size_t)head * rows * 128 + 32 * wave + ln;
  int r0 = (wg * 97) % (rows / 32) * 32;   // workgroups of a head start at different tiles
  for (int s = 0; s < steps; ++s) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int row = r0 + 8 * (v >> 2) + 4 * g + (v & 3);
      float *p = base + (size_t)row * 128;
      if (mode == 0) __builtin_amdgcn_global_atomic_fadd_f32(p, 1.0f);
      else *p = 1.0f;
    }
    r0 += 32;
    if (r0 >= rows) r0 = 0;
  }
}
}  // namespace

// `acc`: device memory of n_heads * rows * 128 floats.  workgroups and n_heads must be multiples of 8, workgroups a
// multiple of n_heads, rows a multiple of 32.  Moves workgroups * 4 * steps * 16 * 64 * 4 bytes of updates.
// Returns 0, or 1 on a bad argument or a launch failure.
extern "C" int s1f_probe_dq_atomics(int workgroups, int rows, int n_heads, int steps, int mode, float *acc,
                                    void *hip_stream) {
  if (workgroups < 8 || n_heads < 8 || workgroups % 8 || n_heads % 8 || workgroups % n_heads || rows < 32 ||
      rows % 32 || steps < 1 || (mode != 0 && mode != 1) || !acc)
    return 1;
  hipLaunchKernelGGL(dq_atomics_kernel, dim3((unsigned)workgroups), dim3(256), 0,
                     reinterpret_cast<hipStream_t>(hip_stream), acc, rows, n_heads, steps, mode);
  return hipGetLastError() == hipSuccess ? 0 : 1;
}
