// Yardstick kernels of the measurement harness (their own shared library, see
// include/medha_yardstick.h): the rate of nothing but bf16 matrix instructions and
// of nothing but HBM -> LDS streaming on the device at hand.
#include "medha_yardstick.h"

#include <hip/hip_runtime.h>

#include "common.h"
#include "prefill_kernel.h"  // async_load16, lds_address

namespace medha {
namespace {

// Each wavefront chains `iters` rounds of 4 independent 32x32x16 bf16 MFMAs
// (4 accumulators, 4 distinct A operands, one B operand).
__global__ void __launch_bounds__(512)
mfma_yardstick_kernel(const uint4* __restrict__ operands, int iters, float* __restrict__ sink) {
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

constexpr int kPieceBytes = 16384;               // one ring stage
constexpr int kLoadsPerPiece = kPieceBytes / 1024;  // 1 KiB per wave-wide load

// Wavefront w of the grid streams pieces w, w + W, w + 2W, ... (W = wavefronts of the grid)
// through a private two-stage ring, two pieces in flight.
__global__ void __launch_bounds__(256)
stream_yardstick_kernel(const char* __restrict__ src, size_t n_pieces, uint32_t* __restrict__ sink) {
  __shared__ __attribute__((aligned(1024))) char lds[4 * 2 * kPieceBytes];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  const size_t n_waves = (size_t)gridDim.x * 4;
  const size_t w0 = (size_t)blockIdx.x * 4 + wave;
  const uint32_t ring = lds_address(lds) + wave * (2 * kPieceBytes);
  const char* ring_ptr = lds + wave * (2 * kPieceBytes);
  auto issue = [&](size_t piece, int st) {
    const char* p = src + piece * kPieceBytes;
#pragma unroll
    for (int j = 0; j < kLoadsPerPiece; ++j)
      async_load16(p + j * 1024, (uint32_t)(lane * 16), ring + st * kPieceBytes + j * 1024);
  };
  uint32_t acc = 0;
  if (w0 < n_pieces) issue(w0, 0);
  if (w0 + n_waves < n_pieces) issue(w0 + n_waves, 1);
  int st = 0;
  for (size_t p = w0; p < n_pieces; p += n_waves, st ^= 1) {
    if (p + n_waves < n_pieces)
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kLoadsPerPiece) : "memory");
    else
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    acc ^= *reinterpret_cast<const uint32_t*>(ring_ptr + st * kPieceBytes + lane * 4);
    // the read has returned before the stage is refilled
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    if (p + 2 * n_waves < n_pieces) issue(p + 2 * n_waves, st);
  }
  sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = acc;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

}  // namespace
}  // namespace medha

using namespace medha;

extern "C" {

int medha_yardstick_mfma_bf16(const void* operands, size_t operand_bytes, int32_t blocks,
                              int32_t iters, float* sink, size_t sink_floats, void* hip_stream) {
  if (operands == nullptr || sink == nullptr || blocks <= 0 || iters <= 0) return -1;
  if (!aligned16(operands) || operand_bytes < 5 * 64 * 16) return -1;
  if (sink_floats < (size_t)blocks * 512) return -3;
  hipLaunchKernelGGL(mfma_yardstick_kernel, dim3(blocks), dim3(512), 0,
                     static_cast<hipStream_t>(hip_stream), static_cast<const uint4*>(operands),
                     iters, sink);
  return hipGetLastError() == hipSuccess ? 0 : -4;
}

int medha_yardstick_stream_lds(const void* src, size_t bytes, int32_t blocks, uint32_t* sink,
                               size_t sink_words, void* hip_stream) {
  if (src == nullptr || sink == nullptr || blocks <= 0 || bytes == 0 || bytes % 65536 != 0)
    return -1;
  if (!aligned16(src)) return -1;
  if (sink_words < (size_t)blocks * 256) return -3;
  hipLaunchKernelGGL(stream_yardstick_kernel, dim3(blocks), dim3(256), 0,
                     static_cast<hipStream_t>(hip_stream), static_cast<const char*>(src),
                     bytes / kPieceBytes, sink);
  return hipGetLastError() == hipSuccess ? 0 : -4;
}

}  // extern "C"
