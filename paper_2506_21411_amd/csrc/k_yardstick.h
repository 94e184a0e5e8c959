// Two yardstick kernels for benchmarks (not part of the paper's method): what this chip reaches on a loop of nothing
// but bf16 MFMAs, and on a plain device-to-device stream copy.  bench.py quotes the library's kernels against these
// achievable rates next to the nominal peaks.
#pragma once
#include "dchag_dev.h"

namespace dchag {

// Every wavefront issues `iters` rounds of eight independent 32x32x16 bf16 MFMAs on registers (no memory traffic in
// the loop): 8 * 32768 flops per round and wavefront.  sink[blockIdx.x * blockDim.x + threadIdx.x] takes one value so
// that the loop is kept.
__global__ __launch_bounds__(256) void k_yardstick_mfma(int iters, float* __restrict__ sink) {
  const int lane = threadIdx.x & 63;
  bf16x8 a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = (bf16)(0.001f * (float)(lane + i));
    b[i] = (bf16)(0.002f * (float)(lane - i));
  }
  f32x16 acc[8];
#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[j], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < 8; ++j) s += acc[j][0] + acc[j][15];
  sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// dst[i] = src[i] for n 16-byte pieces, grid-stride: reads 16 n bytes, writes 16 n bytes.
__global__ __launch_bounds__(256) void k_yardstick_copy(size_t n, const f32x4* __restrict__ src, f32x4* __restrict__ dst) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

}  // namespace dchag
