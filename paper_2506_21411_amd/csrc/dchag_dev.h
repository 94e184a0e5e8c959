// Device-side basics shared by every kernel of the library: element types, conversions,
// wavefront reductions.  gfx950 only (64-wide wavefronts).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dchag {

typedef __bf16 bf16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kWave = 64;

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16 v) { return (float)v; }

template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16 from_f32<bf16>(float v) { return (bf16)v; }  // round to nearest even

// Butterfly reductions over the 64 lanes of a wavefront (every lane ends with the result).
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, kWave));
  return v;
}

// Batched row-block addressing used by the projection kernels.  A batch item zb = b * G + k
// (batch element b, group k) owns `rows` consecutive rows of a [.., D] matrix:
//   first row  = b * rows_per_b + k * rows_per_group
//   rows       = min(rows_per_group, rows_per_b - k * rows_per_group)
struct RowBlocks {
  int G;               // groups per batch element
  int rows_per_b;      // rows of one batch element (all groups)
  int rows_per_group;  // nominal rows of one group
  __host__ __device__ int rows_of(int k) const {
    int left = rows_per_b - k * rows_per_group;
    return left < rows_per_group ? left : rows_per_group;
  }
  __host__ __device__ long first_row(int b, int k) const {
    return (long)b * rows_per_b + (long)k * rows_per_group;
  }
};

}  // namespace dchag
