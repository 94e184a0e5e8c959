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

// Reductions over the 64 lanes of a wavefront (every lane ends with the result).  Inside a row of 16 lanes the partial
// results travel by DPP (two quad permutes, then rotations of the row by 4 and by 8 lanes: no LDS crossbar, one VALU
// instruction per step); the four row results are then read out of lanes 0, 16, 32, 48 and combined in a fixed order.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}
constexpr int kDppSwapPairs = 0xB1;    // quad_perm [1, 0, 3, 2]
constexpr int kDppSwapHalves = 0x4E;   // quad_perm [2, 3, 0, 1]
constexpr int kDppRowRor4 = 0x124;     // rotate the row of 16 lanes by 4
constexpr int kDppRowRor8 = 0x128;     // ... by 8
__device__ __forceinline__ float lane_value(float v, int lane) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}
__device__ __forceinline__ float wave_sum(float v) {
  v += dpp_move<kDppSwapPairs>(v);
  v += dpp_move<kDppSwapHalves>(v);
  v += dpp_move<kDppRowRor4>(v);
  v += dpp_move<kDppRowRor8>(v);
  return (lane_value(v, 0) + lane_value(v, 16)) + (lane_value(v, 32) + lane_value(v, 48));
}
__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, dpp_move<kDppSwapPairs>(v));
  v = fmaxf(v, dpp_move<kDppSwapHalves>(v));
  v = fmaxf(v, dpp_move<kDppRowRor4>(v));
  v = fmaxf(v, dpp_move<kDppRowRor8>(v));
  return fmaxf(fmaxf(lane_value(v, 0), lane_value(v, 16)), fmaxf(lane_value(v, 32), lane_value(v, 48)));
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
