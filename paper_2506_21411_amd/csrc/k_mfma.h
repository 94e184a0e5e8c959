// bf16 MFMA kernels for gfx950 (CDNA4): the per-group projections  Y = A W^T + b  of the
// aggregation layers (paper Section 2.1: the cross-attention layer's value and output
// projections), as an NT GEMM with both operands K-contiguous, fp32 accumulation in
// v_mfma_f32_32x32x16_bf16, operand tiles staged through XOR-swizzled LDS.
#pragma once
#include "dchag_dev.h"

namespace dchag {

constexpr int kBK = 64;       // K extent of one LDS stage (bf16 elements) = 8 chunks of 16 bytes
constexpr int kXcds = 8;      // accelerator complex dies; workgroup ids go to them round-robin

// LDS tiles are [rows][8 chunks] of 16-byte chunks (8 bf16).  The chunk index is XOR-ed with
// low row bits so that the 32 rows a wavefront reads at one logical chunk spread over banks.
template <int SH>
__device__ __forceinline__ int lds_slot(int row, int chunk) { return row * 8 + (chunk ^ ((row >> SH) & 7)); }

// Work decode shared by the MFMA kernels: linear workgroup id -> (group k, batch b, m-tile, n-tile).
// Each XCD (id % 8) receives a contiguous range of the (k, b, m, n) order, n fastest, so that the
// n-tiles sharing an A tile and the m-tiles/batches sharing a group's weights meet in one L2.
struct TileWork {
  int total, n_tiles, m_tiles, nb;
  // position w of the (k, b, m, n) order, n fastest
  __device__ __forceinline__ void decode_linear(int w, int& k, int& b, int& mt, int& nt) const {
    nt = w % n_tiles;
    int rest = w / n_tiles;
    mt = rest % m_tiles;
    rest /= m_tiles;
    b = rest % nb;
    k = rest / nb;
  }
  __device__ __forceinline__ bool decode(int L, int& k, int& b, int& mt, int& nt) const {
    const int per = (total + kXcds - 1) / kXcds;
    const int w = (L % kXcds) * per + L / kXcds;
    if (L / kXcds >= per || w >= total) return false;
    nt = w % n_tiles;
    int rest = w / n_tiles;
    mt = rest % m_tiles;
    rest /= m_tiles;
    b = rest % nb;
    k = rest / nb;
    return true;
  }
};

// ---------------------------------------------------------------------------------------
// Y[r][o] = sum_j A[r][j] * Wt[k][o][j] + bias[k][o] (+ rowadd[r][o], r inside the row block)   bf16, fp32 accumulate
//   BM x BN block tile, WM x WN wavefronts, each a (BM/WM) x (BN/WN) tile of 32x32 MFMA blocks.
//   Requires D % 64 == 0 and D % BN == 0 (checked on the host); rows are ragged (clamped loads,
//   masked stores).  Dynamic LDS: 2 stages x (BM + BN) x 128 bytes.
// ---------------------------------------------------------------------------------------
template <int BM, int BN, int WM, int WN, int SH>
__global__ __launch_bounds__(WM * WN * 64) void k_linear_mfma(int D, RowBlocks rb, TileWork tw,
                                                              const bf16* __restrict__ A,
                                                              const bf16* __restrict__ Wt,
                                                              const bf16* __restrict__ bias,
                                                              bf16* __restrict__ Y,
                                                              const bf16* __restrict__ rowadd) {
  constexpr int NT = WM * WN * 64;
  constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
  constexpr int A_CH = BM * 8 / NT, B_CH = BN * 8 / NT;   // 16-byte chunks per thread per stage
  static_assert(BM * 8 % NT == 0 && BN * 8 % NT == 0, "tile does not split over the threads");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16x8* As = reinterpret_cast<bf16x8*>(smem);           // [2][BM * 8]
  bf16x8* Bs = As + 2 * BM * 8;                           // [2][BN * 8]

  int k, b, mt, nt;
  if (!tw.decode(blockIdx.x, k, b, mt, nt)) return;
  const int rows = rb.rows_of(k);
  const int r0 = mt * BM, o0 = nt * BN;
  if (r0 >= rows) return;
  const bf16* Ab = A + (size_t)rb.first_row(b, k) * D;
  bf16* Yb = Y + (size_t)rb.first_row(b, k) * D;
  const bf16* Wb = Wt + (size_t)k * D * D;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const int l32 = lane & 31, lhi = lane >> 5;

  // global source pointers of this thread's chunks (row clamped into the matrix)
  const bf16x8* a_src[A_CH];
  const bf16x8* b_src[B_CH];
  int a_dst[A_CH], b_dst[B_CH];
#pragma unroll
  for (int i = 0; i < A_CH; ++i) {
    const int idx = tid + i * NT, row = idx >> 3, ch = idx & 7;
    const int gr = min(r0 + row, rows - 1);
    a_src[i] = reinterpret_cast<const bf16x8*>(Ab + (size_t)gr * D) + ch;
    a_dst[i] = lds_slot<SH>(row, ch);
  }
#pragma unroll
  for (int i = 0; i < B_CH; ++i) {
    const int idx = tid + i * NT, row = idx >> 3, ch = idx & 7;
    b_src[i] = reinterpret_cast<const bf16x8*>(Wb + (size_t)(o0 + row) * D) + ch;
    b_dst[i] = lds_slot<SH>(row, ch);
  }

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  bf16x8 a_reg[A_CH], b_reg[B_CH];
  const int KT = D / kBK;
#pragma unroll
  for (int i = 0; i < A_CH; ++i) a_reg[i] = a_src[i][0];
#pragma unroll
  for (int i = 0; i < B_CH; ++i) b_reg[i] = b_src[i][0];
#pragma unroll
  for (int i = 0; i < A_CH; ++i) As[a_dst[i]] = a_reg[i];
#pragma unroll
  for (int i = 0; i < B_CH; ++i) Bs[b_dst[i]] = b_reg[i];
  __syncthreads();

  for (int kt = 0; kt < KT; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < KT) {
#pragma unroll
      for (int i = 0; i < A_CH; ++i) a_reg[i] = a_src[i][(kt + 1) * 8];
#pragma unroll
      for (int i = 0; i < B_CH; ++i) b_reg[i] = b_src[i][(kt + 1) * 8];
    }
    const bf16x8* Ac = As + cur * BM * 8;
    const bf16x8* Bc = Bs + cur * BN * 8;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      bf16x8 af[TM], bfr[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) af[i] = Ac[lds_slot<SH>(wm * (BM / WM) + i * 32 + l32, kk * 2 + lhi)];
#pragma unroll
      for (int j = 0; j < TN; ++j) bfr[j] = Bc[lds_slot<SH>(wn * (BN / WN) + j * 32 + l32, kk * 2 + lhi)];
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < KT) {
      bf16x8* An = As + (cur ^ 1) * BM * 8;
      bf16x8* Bn = Bs + (cur ^ 1) * BN * 8;
#pragma unroll
      for (int i = 0; i < A_CH; ++i) An[a_dst[i]] = a_reg[i];
#pragma unroll
      for (int i = 0; i < B_CH; ++i) Bn[b_dst[i]] = b_reg[i];
    }
    __syncthreads();
  }

  // 32x32 accumulator block: lane holds column (lane % 32); register r holds row
  // 8 * (r / 4) + 4 * (lane / 32) + (r % 4).
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int o = o0 + wn * (BN / WN) + j * 32 + l32;
    const float bv = bias ? (float)bias[(size_t)k * D + o] : 0.f;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = r0 + wm * (BM / WM) + i * 32 + 8 * (r >> 2) + 4 * lhi + (r & 3);
        if (row < rows)
          Yb[(size_t)row * D + o] = (bf16)(acc[i][j][r] + bv + (rowadd ? (float)rowadd[(size_t)row * D + o] : 0.f));
      }
    }
  }
}

}  // namespace dchag
