// Measurement aid: the rate the chip sustains on the MFMA instruction the attention kernels
// use, with all operands in registers. The datasheet peak assumes the nominal clock; under a
// power limit the clock depends on what the operands look like, so the loop runs either on
// constant operands or on pseudo-random bf16 bit patterns.
#include "fa_common.h"
#include "fa_kernels.h"

namespace fa {

__device__ __forceinline__ unsigned mix32(unsigned x) {
  x ^= x >> 16;
  x *= 0x7feb352dU;
  x ^= x >> 15;
  x *= 0x846ca68bU;
  x ^= x >> 16;
  return x;
}

// Every wavefront issues iters * 32 MFMAs (4 accumulators, 8 operand pairs in rotation). With
// random operands the accumulators are scaled down once per 32 MFMAs so they stay finite.
template <bool RANDOM>
__global__ __launch_bounds__(512) void mfma_probe_kernel(float* sink, long long* clocks, int iters) {
  bf16x8 a[8], b[8];
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    u32x4 ua, ub;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      if (!RANDOM) {
        ua[t] = ub[t] = 0x3f803f80u;  // 1.0, 1.0
      } else {
        // random sign and mantissa, exponents 2^-2 .. 2^0
        const unsigned h1 = mix32(threadIdx.x * 131 + q * 17 + t), h2 = mix32(threadIdx.x * 257 + q * 29 + t + 1000);
        ua[t] = (h1 & 0x807f807fu) | 0x3e803e80u | ((h1 >> 3) & 0x01000100u);
        ub[t] = (h2 & 0x807f807fu) | 0x3e803e80u | ((h2 >> 3) & 0x01000100u);
      }
    }
    a[q] = __builtin_bit_cast(bf16x8, ua);
    b[q] = __builtin_bit_cast(bf16x8, ub);
  }
  f32x16 acc[4];
#pragma unroll
  for (int n = 0; n < 4; ++n) acc[n] = (f32x16){0};
  const long long t0 = clock64(), w0 = wall_clock64();
  for (int i = 0; i < iters; ++i) {
#pragma unroll
    for (int r = 0; r < 8; ++r)
#pragma unroll
      for (int n = 0; n < 4; ++n) acc[n] = mfma32(a[(r + n) & 7], b[(r + 3 * n) & 7], acc[n]);
    if (RANDOM) {
#pragma unroll
      for (int n = 0; n < 4; ++n)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[n][r] *= 0.03125f;
    }
  }
  const long long t1 = clock64(), w1 = wall_clock64();
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    clocks[0] = t1 - t0;  // shader clock cycles
    clocks[1] = w1 - w0;  // ticks of the constant 100 MHz counter
  }
  float s = 0.f;
#pragma unroll
  for (int n = 0; n < 4; ++n)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[n][r];
  sink[blockIdx.x * 512 + threadIdx.x] = s;
}

hipError_t launch_mfma_probe(float* sink, long long* clocks, int workgroups, int iters, int random_operands,
                             hipStream_t st) {
  if (random_operands) hipLaunchKernelGGL((mfma_probe_kernel<true>), dim3(workgroups), dim3(512), 0, st, sink, clocks, iters);
  else hipLaunchKernelGGL((mfma_probe_kernel<false>), dim3(workgroups), dim3(512), 0, st, sink, clocks, iters);
  return hipGetLastError();
}

}  // namespace fa
