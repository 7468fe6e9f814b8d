// Two yardstick kernels for the measurement harness: what this very part sustains
// when it does nothing but bf16 matrix instructions, and nothing but streaming
// reads.  They put the attention kernels' figures beside the achievable rate of the
// same device in the same run (clocks under load differ from the data sheet's).
#pragma once

#include "common.h"

namespace medha {

// Each wavefront chains `iters` rounds of 4 independent 32x32x16 bf16 MFMAs
// (4 accumulators, 4 distinct A operands, one B operand) on operands read from
// `operands` (the caller fills it, so the data -- and with it the switching
// power -- is the caller's choice).  Launch: any grid, 512 threads per block so
// that two wavefronts share a SIMD as in the prefill kernel.  Flops per
// wavefront: iters * 4 * 2*32*32*16.  `sink` receives one float per lane.
__global__ void __launch_bounds__(512)
mfma_ceiling_kernel(const uint4* __restrict__ operands, int iters, float* __restrict__ sink) {
  const int lane = threadIdx.x & 63;
  bf16x8 a[4], b;
#pragma unroll
  for (int i = 0; i < 4; ++i) a[i] = __builtin_bit_cast(bf16x8, operands[i * 64 + lane]);
  b = __builtin_bit_cast(bf16x8, operands[4 * 64 + lane]);
  f32x16 acc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b, acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) s += acc[i][e];
  sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// Grid-stride read of `n16` 16-byte words, 4 loads in flight per lane per step; the
// words are XOR-folded so nothing can be dropped.  `sink` receives one word per thread.
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
__global__ void __launch_bounds__(256)
read_ceiling_kernel(const u32x4* __restrict__ src, size_t n16, u32x4* __restrict__ sink) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  u32x4 acc = {0u, 0u, 0u, 0u};
  for (; i + 3 * stride < n16; i += 4 * stride) {
    const u32x4 v0 = __builtin_nontemporal_load(src + i);
    const u32x4 v1 = __builtin_nontemporal_load(src + i + stride);
    const u32x4 v2 = __builtin_nontemporal_load(src + i + 2 * stride);
    const u32x4 v3 = __builtin_nontemporal_load(src + i + 3 * stride);
    acc ^= v0 ^ v1 ^ v2 ^ v3;
  }
  for (; i < n16; i += stride) acc ^= __builtin_nontemporal_load(src + i);
  sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = acc;
}

}  // namespace medha
