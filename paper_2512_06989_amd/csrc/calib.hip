// Calibration kernels for the bench (libmhffn_calib.so, not part of the operation's library):
// what rate does the MFMA pipe of this machine sustain when nothing else runs?
//
// The published dense bf16 peak (2.5 PFLOP/s) is the product of the unit count and the maximum
// clock.  Under sustained matrix work the clock is set by power management, and how far it
// drops depends on how much the operands toggle: a loop of v_mfma_f32_32x32x16_bf16 on constant
// operands runs at the maximum clock, the same loop on fresh random operands noticeably below
// it.  The bench reports both beside the fused kernels' figures, so that their distance from
// the published peak can be split into "what no kernel on this machine reaches with such data"
// and "what this kernel loses".
//
//   mode 0: every operand element 1.0
//   mode 1: 24 A x 8 B register sets of pseudo-random values (A scaled like weights, 0.02;
//           B like activations, 1.0), cycling, so that consecutive products see new operands
// Two waves per SIMD on every CU, four independent accumulators per wave, no memory traffic.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kProductsPerIter = 96;

__device__ unsigned mix(unsigned x) {
  x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
  return x;
}
// roughly normal (sum of four uniform bytes), standard deviation `scale`
__device__ float pseudo_normal(unsigned s, float scale) {
  const unsigned h = mix(s);
  const float u = ((h & 255) + ((h >> 8) & 255) + ((h >> 16) & 255) + (h >> 24)) * (1.0f / 256.0f) - 2.0f;
  return u * 1.7f * scale;
}

template <int MODE>
__global__ __launch_bounds__(512) void mfma_rate_kernel(float* sink, long long* clocks, int iters) {
  constexpr int NA = MODE ? 24 : 1, NB = MODE ? 8 : 1;
  bf16x8 A[NA], B[NB];
  const unsigned tid = blockIdx.x * 512 + threadIdx.x;
  for (int a = 0; a < NA; ++a)
    for (int i = 0; i < 8; ++i) A[a][i] = (__bf16)(MODE ? pseudo_normal(tid * 977u + a * 131u + i, 0.02f) : 1.0f);
  for (int b = 0; b < NB; ++b)
    for (int i = 0; i < 8; ++i) B[b][i] = (__bf16)(MODE ? pseudo_normal(tid * 7919u + b * 17u + i + 12345u, 1.0f) : 1.0f);
  f32x16 acc[4] = {f32x16{0}, f32x16{0}, f32x16{0}, f32x16{0}};
  const long long c0 = clock64(), w0 = wall_clock64();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < kProductsPerIter; ++j)
      acc[j & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[j % NA], B[(j / 3) % NB], acc[j & 3], 0, 0, 0);
  }
  const long long c1 = clock64(), w1 = wall_clock64();
  float s = 0.f;
  for (int i = 0; i < 16; ++i) s += acc[0][i] + acc[1][i] + acc[2][i] + acc[3][i];
  sink[tid] = s;
  if ((threadIdx.x & 63) == 0) {
    const int w = blockIdx.x * 8 + (threadIdx.x >> 6);
    clocks[2 * w] = c1 - c0;        // shader clock cycles
    clocks[2 * w + 1] = w1 - w0;    // constant 100 MHz clock
  }
}

}  // namespace

extern "C" {

// Device scratch the caller provides: `sink` n_workgroups * 512 floats, `clocks` n_workgroups * 16 int64.
// Enqueues one launch of `iters` x 96 products per wave on `n_workgroups` workgroups of 8 waves.
// Returns the hipError_t of the launch.
int mhffn_calib_mfma_launch(int mode, int n_workgroups, int iters, void* sink, void* clocks, void* stream) {
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (mode)
    hipLaunchKernelGGL(mfma_rate_kernel<1>, dim3(n_workgroups), dim3(512), 0, st, static_cast<float*>(sink),
                       static_cast<long long*>(clocks), iters);
  else
    hipLaunchKernelGGL(mfma_rate_kernel<0>, dim3(n_workgroups), dim3(512), 0, st, static_cast<float*>(sink),
                       static_cast<long long*>(clocks), iters);
  return (int)hipGetLastError();
}

// flops of one launch
double mhffn_calib_mfma_flops(int n_workgroups, int iters) {
  return (double)n_workgroups * 8.0 * iters * kProductsPerIter * 32768.0;
}

}  // extern "C"
