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

// dst[i] = src[i] for n 16-byte pieces: reads 16 n bytes, writes 16 n bytes.  A block of 256 threads copies 1024
// consecutive pieces, a thread four of them 256 pieces apart (four independent 16-byte loads in flight per lane).
__global__ __launch_bounds__(256) void k_yardstick_copy(size_t n, const f32x4* __restrict__ src, f32x4* __restrict__ dst) {
  const size_t base = (size_t)blockIdx.x * 1024 + threadIdx.x;
  f32x4 v[4];
#pragma unroll
  for (int t = 0; t < 4; ++t)
    if (base + 256 * t < n) v[t] = src[base + 256 * t];
#pragma unroll
  for (int t = 0; t < 4; ++t)
    if (base + 256 * t < n) dst[base + 256 * t] = v[t];
}

// Reads n 16-byte pieces and writes (next to) nothing: the streaming-read rate.  The sum keeps the loads alive; a
// thread stores it only if it equals a value it cannot take.
__global__ __launch_bounds__(256) void k_yardstick_read(size_t n, const f32x4* __restrict__ src, float* __restrict__ sink) {
  const size_t base = (size_t)blockIdx.x * 1024 + threadIdx.x;
  f32x4 v[4];
#pragma unroll
  for (int t = 0; t < 4; ++t) v[t] = base + 256 * t < n ? src[base + 256 * t] : f32x4{0.f, 0.f, 0.f, 0.f};
  const f32x4 s4 = (v[0] + v[1]) + (v[2] + v[3]);
  const float s = (s4[0] + s4[1]) + (s4[2] + s4[3]);
  if (s == -1.2345e38f) sink[threadIdx.x] = s;
}

}  // namespace dchag
