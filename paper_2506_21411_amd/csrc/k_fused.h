// bf16 fast path of one aggregation level on gfx950 (paper Section 2.1: a cross-attention layer
// reduces the channel tokens of a patch to one token; Section 3.2: one layer per channel group).
//
//   k_scores_mfma     raw scores of every token against the query-folded key weights (MFMA)
//   k_softmax_alpha   softmax of the scores over the members of each group
//   k_vagg_mfma       value projection GEMM whose epilogue takes the softmax-weighted sum over
//                     the channels of the group, so that the projected values never leave the CU
//   k_linear_dl       plain per-group projection GEMM (output projection)
//   k_fold_value_dl   weight-only product Wv We[c] (value projection folded into the tokenizer weights)
//   k_scores_pixels*, k_compose_score_weights*   first-level scores straight from the pixels
//   k_tokenize_ws, k_tokenize_mfma               the per-channel tokenizer (paper Section 2.1)
//   k_tokenize_reduce_ring, k_tokenize_mix_*, k_tokenize_attend_wide   tokenizer fused with the first level
//                     (linear level of D-CHAG-L, or attention level with folded value weights): no tokens in HBM
//
// The two GEMM kernels share one core: 256x256 block tile, 8 wavefronts (2 x 4), 32x32x16 bf16
// MFMA, K staged in 64-element slices through two LDS stages that are filled by direct-to-LDS
// global loads of 128-byte row segments (no register staging; L2 delivers 128-byte segments at
// about twice the rate of 64-byte ones) and read with conflict-free swizzled ds_read_b128.
//
// Softmax weights are exchanged between the kernels in the layout
//   alpha[b][k][cl][head][n]   (n fastest, pitch Np = N rounded up to 32; cl < gpad = g rounded up to 8)
// with zeros for the padding members cl >= size of group k.
#pragma once
#include "dchag_dev.h"
#include "k_mfma.h"

namespace dchag {

typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

// Wait until at most N vector-memory operations of this wavefront are outstanding
// (gfx9 s_waitcnt immediate: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[5:4] at [15:14]).
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

// Each lane's 16 bytes of a wave-wide direct-to-LDS load land at lds_base + 16 * lane (lds_base is wave-uniform).
// Written as an asm statement on purpose: the compiler files the builtin under "flat access that may touch LDS and
// global memory", and while one is pending it turns every counted wait of the wavefront into a wait for zero, which
// serialises the LDS fragment reads of the GEMM loops.  The kernels order these loads themselves (wait_vmcnt + barrier
// before the stage is read; nothing outstanding when the block retires), so the compiler need not know them; the
// memory clobber keeps it from moving LDS or global accesses across the statement.
__device__ __forceinline__ void load16_to_lds(const void* src, void* lds_base) {
  const unsigned lds_off = __builtin_amdgcn_readfirstlane((unsigned)(size_t)(lptr_t)lds_base);
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(lds_off), "v"(src) : "memory", "m0");
}

// LDS stages hold rows of 64 bf16 (128 bytes = 8 chunks of 16 bytes).  Chunk c of row r sits at chunk
// position c ^ ((r >> 1) & 7): the 16 consecutive rows a quarter-wavefront reads at one logical chunk
// then fall into 16 different 16-byte bank groups (64 banks x 4 bytes), so ds_read_b128 is conflict-free.
__device__ __forceinline__ int swz_chunk(int row) { return (row >> 1) & 7; }

constexpr int kGemmBM = 256, kGemmBN = 256, kGemmBK = 64, kGemmWM = 2, kGemmWN = 4, kGemmStages = 2;
constexpr int kGemmStageBytes = (kGemmBM + kGemmBN) * kGemmBK * 2;             // 64 KiB
constexpr int kGemmRingBytes = kGemmStages * kGemmStageBytes;                  // 128 KiB

// ---------------------------------------------------------------------------------------------
// Weight-only prep of attention levels (paper Section 2.1's cross-attention layer; the learned query is fixed, so its
// projection and its product with the key weights depend on the weights alone), one launch for any number of levels:
//   Q[k][i]    = sum_j Wq[k][i][j] query[k][j] + bq[k][i]
//   M[k][a][d] = (1 / sqrt(dh)) sum_{i in head a} Wk[k][i][d] Q[k][i]      (the key bias shifts every score of a softmax
//                                                                          equally and is dropped)
// so that the score of token z for head a is z . M[k][a][:].  grid (heads, all groups of all levels, column shares),
// block 256: a block of (head a, group k) first forms the dh entries of Q of its head (a wavefront per row of Wq, the
// rows dealt round-robin), leaves them in LDS (and, the first share, in Qp), then sums the dh rows of Wk of that head
// into its share of M's columns (fixed summation order).  Writes M as fp32 (Mf), bf16 (Mb) and, where asked,
// transposed fp32 MfT[G][D][heads].  Requires dh % 4 == 0 and (D / shares) % 8 == 0.  Dynamic LDS: dh + 1536 floats.
// ---------------------------------------------------------------------------------------------
struct KeyPrepLevel {
  const bf16 *query, *Wq, *bq, *Wk;
  float *Qp, *Mf, *MfT;
  bf16* Mb;
  int g_first;                     // index of this level's first group in the launch's group axis
};
constexpr int kKeyPrepMaxLevels = 16;
struct KeyPrepArgs {
  int n_levels;
  KeyPrepLevel lv[kKeyPrepMaxLevels];
};

__global__ __launch_bounds__(256) void k_query_keys(int D, int heads, KeyPrepArgs args) {
  extern __shared__ float qs[];                          // [dh] projected query of the head, then [3][512] partial sums
  const int a = blockIdx.x;
  int l = 0;
  while (l + 1 < args.n_levels && (int)blockIdx.y >= args.lv[l + 1].g_first) ++l;     // uniform over the block
  const KeyPrepLevel& P = args.lv[l];
  const int k = blockIdx.y - P.g_first;
  const int dh = D / heads;
  float* part = qs + dh;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const bf16* q = P.query + (size_t)k * D;
  const size_t row0 = (size_t)k * D + (size_t)a * dh;
  // Q of this head: wavefront w takes rows w, w + 4, ..., eight of them at a time so that their loads are in flight
  // together (every block of a head computes all of Q_a: the second block's reads come out of L2)
  for (int r0 = wave; r0 < dh; r0 += 32) {
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int j = lane * 8; j < D; j += kWave * 8) {
      const bf16x8 qv = *reinterpret_cast<const bf16x8*>(q + j);
      bf16x8 wv[8];
#pragma unroll
      for (int t = 0; t < 8; ++t)
        wv[t] = *reinterpret_cast<const bf16x8*>(P.Wq + (row0 + min(r0 + 4 * t, dh - 1)) * D + j);
#pragma unroll
      for (int t = 0; t < 8; ++t)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[t] += (float)wv[t][e] * (float)qv[e];
    }
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      const float v = wave_sum(acc[t]);
      const int r = r0 + 4 * t;
      if (lane == 0 && r < dh) {
        const float qv = v + (P.bq ? (float)P.bq[row0 + r] : 0.f);
        if (blockIdx.z == 0) P.Qp[row0 + r] = qv;
        qs[r] = qv;
      }
    }
  }
  __syncthreads();
  // M of this head, this block's share of the columns: a lane takes eight adjacent columns (16-byte loads, eight rows
  // in flight), wavefront w the w-th quarter of the head's rows; the four partial sums meet in LDS in that order
  const float scale = rsqrtf((float)dh);
  const int qrows = dh / 4;
  const int cper = D / gridDim.z, cbeg = blockIdx.z * cper, cend = cbeg + cper;
  for (int c0 = cbeg; c0 < cend; c0 += 512) {
    const int d0 = c0 + lane * 8;
    const bool live = d0 < cend;
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (live) {
      const bf16* w = P.Wk + (row0 + (size_t)wave * qrows) * D + d0;
      const float* qh = qs + wave * qrows;
#pragma unroll 8
      for (int r = 0; r < qrows; ++r) {
        const bf16x8 v = *reinterpret_cast<const bf16x8*>(w + (size_t)r * D);
        const float qr = qh[r];
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] += (float)v[e] * qr;
      }
    }
    if (wave > 0) {
#pragma unroll
      for (int e = 0; e < 8; ++e) part[(wave - 1) * 512 + lane * 8 + e] = acc[e];
    }
    __syncthreads();
    if (wave == 0 && live) {
      const size_t o = ((size_t)k * heads + a) * D + d0;
      bf16x8 b8;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        acc[e] = (((acc[e] + part[lane * 8 + e]) + part[512 + lane * 8 + e]) + part[1024 + lane * 8 + e]) * scale;
        b8[e] = (bf16)acc[e];
      }
      *reinterpret_cast<f32x4*>(P.Mf + o) = f32x4{acc[0], acc[1], acc[2], acc[3]};
      *reinterpret_cast<f32x4*>(P.Mf + o + 4) = f32x4{acc[4], acc[5], acc[6], acc[7]};
      *reinterpret_cast<bf16x8*>(P.Mb + o) = b8;
      if (P.MfT) {
#pragma unroll
        for (int e = 0; e < 8; ++e) P.MfT[((size_t)k * D + d0 + e) * heads + a] = acc[e];
      }
    }
    __syncthreads();
  }
}

// ---------------------------------------------------------------------------------------------
// Scores.  S[b][k][cl][head][n] = z[b, c, n, :] . Mb[k][head][:]   (c = k*g + cl)
// grid (ceil(N/16), G * ceil(g/4), B), block 256: a block takes 16 patches x 4 channels of one group; its
// four wavefronts each take a quarter of D (operands straight from global memory: 16 rows x 64 bytes per
// load for the tokens, the folded keys come from L2), and the partial 16x16 blocks meet in LDS in a
// fixed order.  The kernel is bound by the HBM read of the tokens (2*D bytes per token).
// Requires D % 128 == 0.
// ---------------------------------------------------------------------------------------------
template <int NB>   // head blocks of 16 (heads padded to 16 * NB)
__global__ __launch_bounds__(256) void k_scores_mfma(int Cin, int N, int D, int heads, int g, int gpad, int Np,
                                                     const bf16* __restrict__ z, const bf16* __restrict__ Mb,
                                                     float* __restrict__ S) {
  __shared__ float part[3][4 * NB * 4][64];
  const int qch = (g + 3) / 4;                         // channel quads per group
  const int k = blockIdx.y / qch, cq = blockIdx.y % qch;
  const int G = gridDim.y / qch;
  const int b = blockIdx.z, n0 = blockIdx.x * 16;
  const int c0 = k * g;
  const int gk = min(g, Cin - c0);                     // members of this group
  if (cq * 4 >= gk) return;                            // uniform: nothing in this quad
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l16 = lane & 15, lq = lane >> 4;
  const int kq = D / 4, kbeg = wave * kq;
  const int n = min(n0 + l16, N - 1);

  const bf16* zrow[4];
  const bf16* mrow[NB];
#pragma unroll
  for (int i = 0; i < 4; ++i)
    zrow[i] = z + (((size_t)b * Cin + c0 + min(cq * 4 + i, gk - 1)) * N + n) * D + kbeg + lq * 8;
#pragma unroll
  for (int nb = 0; nb < NB; ++nb)
    mrow[nb] = Mb + ((size_t)k * heads + min(nb * 16 + l16, heads - 1)) * D + kbeg + lq * 8;

  f32x4 acc[4][NB];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) acc[i][nb] = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int ks = 0; ks < kq; ks += 32) {
    bf16x8 bfr[NB], af[4];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      bfr[nb] = *reinterpret_cast<const bf16x8*>(mrow[nb] + ks);
      if (nb * 16 + l16 >= heads) bfr[nb] = bf16x8{};
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) af[i] = *reinterpret_cast<const bf16x8*>(zrow[i] + ks);
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
        acc[i][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[i], bfr[nb], acc[i][nb], 0, 0, 0);
  }
  if (wave > 0) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int e = 0; e < 4; ++e) part[wave - 1][(i * NB + nb) * 4 + e][lane] = acc[i][nb][e];
  }
  __syncthreads();
  if (wave == 0) {
    // 16x16 accumulator block: lane holds head (lane % 16), patches 4 * (lane / 16) + 0..3
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int cl = cq * 4 + i;
      if (cl >= gk) continue;
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        const int head = nb * 16 + l16;
        f32x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int slot = (i * NB + nb) * 4 + e;
          v[e] = acc[i][nb][e] + part[0][slot][lane] + part[1][slot][lane] + part[2][slot][lane];
        }
        if (head < heads) {
          float* dst = S + ((((size_t)b * G + k) * gpad + cl) * heads + head) * Np + n0 + lq * 4;
          *reinterpret_cast<f32x4*>(dst) = v;
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Scores, group-resident form of the kernel above for D = 128 * KI (KI even): a block takes 16 patches and a
// run of whole channel quads of ONE group, so each wavefront loads its quarter of the folded keys once into
// registers (KI * NB operand fragments) and then only streams tokens; the token loads of the next 32-feature
// step are in flight while the current one is multiplied.  The four partial 16x16 blocks of a quad meet in
// LDS (two buffers, one barrier per quad) and wavefront w adds up and stores channel w of the quad, always in
// the order of the wavefronts.  grid (ceil(N/16), G * qsplit, B), block 256; part = blockIdx.y % qsplit takes
// quads [part * qper, (part + 1) * qper) of its group.  Bound by the HBM read of the tokens.
// ---------------------------------------------------------------------------------------------
template <int NB, int KI>
__global__ __launch_bounds__(256) void k_scores_group(int Cin, int N, int heads, int g, int gpad, int Np, int qsplit,
                                                      int qper, const bf16* __restrict__ z,
                                                      const bf16* __restrict__ Mb, float* __restrict__ S) {
  // one step = one 16-byte load per lane = 32 features of one channel; a quad takes 4 * KI steps, channel after
  // channel, so that a wavefront streams 16 rows x (D / 4) contiguous bytes of one channel before it moves on
  constexpr int STEPS = 4 * KI;
  constexpr int NBUF = STEPS < 8 ? STEPS : 8;            // NBUF - 1 loads in flight per lane
  constexpr int PD = NBUF - 1;
  static_assert(STEPS % NBUF == 0, "the fragment buffers rotate with the step index");
  constexpr int D = KI * 128;
  __shared__ float part[2][4][4][NB * 4][64];           // [buffer][source wavefront][channel of the quad]
  const int k = blockIdx.y / qsplit, prt = blockIdx.y % qsplit;
  const int G = gridDim.y / qsplit;
  const int b = blockIdx.z, n0 = blockIdx.x * 16;
  const int c0 = k * g;
  const int gk = min(g, Cin - c0);
  const int q_end = min((gk + 3) / 4, (prt + 1) * qper);
  const int q_begin = prt * qper;
  if (q_begin >= q_end) return;                          // uniform over the block
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l16 = lane & 15, lq = lane >> 4;
  const int n = min(n0 + l16, N - 1);
  const int koff = wave * (D / 4) + lq * 16;
  // features of step ks (same for tokens and keys): the two steps of a pair read the two 16-byte halves of a
  // lane's 32 bytes, so that the four lanes of a row cover one 128-byte line with two back-to-back loads
  auto kstep = [](int ks) { return (ks >> 1) * 64 + (ks & 1) * 8; };

  bf16x8 bfr[KI][NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    const bf16* mrow = Mb + ((size_t)k * heads + min(nb * 16 + l16, heads - 1)) * D + koff;
#pragma unroll
    for (int ks = 0; ks < KI; ++ks) {
      bfr[ks][nb] = *reinterpret_cast<const bf16x8*>(mrow + kstep(ks));
      if (nb * 16 + l16 >= heads) bfr[ks][nb] = bf16x8{};
    }
  }
  // tokens of channel cl of this group, this lane's patch and feature offset; members past the end of a
  // short group re-read the last member (their scores are never stored)
  const bf16* zb = z + (((size_t)b * Cin + c0) * N + n) * D + koff;
  const size_t cstride = (size_t)N * D;
  auto zptr = [&](int cl) { return zb + (size_t)min(cl, gk - 1) * cstride; };

  bf16x8 af[NBUF];
#pragma unroll
  for (int t = 0; t < PD; ++t) af[t] = *reinterpret_cast<const bf16x8*>(zptr(q_begin * 4 + t / KI) + kstep(t % KI));
  for (int q = q_begin; q < q_end; ++q) {
    const bf16* cur[4];
    const bf16* nxt[4];
    const int qn = min(q + 1, q_end - 1);                // past the last quad: re-read it (in bounds, unused)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      cur[i] = zptr(q * 4 + i);
      nxt[i] = zptr(qn * 4 + i);
    }
    f32x4 acc[4][NB];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) acc[i][nb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int t = 0; t < STEPS; ++t) {
      const int tp = t + PD;                             // the step whose load is issued now
      af[tp % NBUF] = (tp < STEPS) ? *reinterpret_cast<const bf16x8*>(cur[tp / KI] + kstep(tp % KI))
                                   : *reinterpret_cast<const bf16x8*>(nxt[(tp - STEPS) / KI] + kstep((tp - STEPS) % KI));
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
        acc[t / KI][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[t % NBUF], bfr[t % KI][nb], acc[t / KI][nb], 0, 0, 0);
    }
    const int pb = (q - q_begin) & 1;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int e = 0; e < 4; ++e) part[pb][wave][i][nb * 4 + e][lane] = acc[i][nb][e];
    __syncthreads();
    // 16x16 accumulator block: lane holds head (lane % 16), patches 4 * (lane / 16) + 0..3
    const int cl = q * 4 + wave;
    if (cl < gk) {
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        const int head = nb * 16 + l16;
        f32x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e)
          v[e] = ((part[pb][0][wave][nb * 4 + e][lane] + part[pb][1][wave][nb * 4 + e][lane]) +
                  part[pb][2][wave][nb * 4 + e][lane]) + part[pb][3][wave][nb * 4 + e][lane];
        if (head < heads) {
          float* dst = S + ((((size_t)b * G + k) * gpad + cl) * heads + head) * Np + n0 + lq * 4;
          *reinterpret_cast<f32x4*>(dst) = v;
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Scores and softmax in one kernel, for heads <= 16 and D % 256 == 0: a block takes 32 patches and ALL members
// of one group, so the raw scores stay in LDS and only the softmax weights are written (128-byte runs).
// The folded keys of the group sit in LDS (rows padded by 16 bytes: conflict-free ds_read_b128).  Wavefront w
// streams whole token rows of members w, w + 8, ...: per step two 16-row fragments (patches 0..15 and 16..31,
// 64 contiguous bytes per row and load) that share one key fragment, with the loads of the next seven steps in
// flight; no cross-wavefront reduction is needed.  After one barrier thread (head, patch) takes the softmax
// over the members and writes alpha, zeros for padding members and padding patches.
// grid (Np / 32, G, B), block 512, dynamic LDS 16 * (2 D + 16) + gpad * 2048 bytes.
// Bound by the HBM read of the tokens.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(512) void k_scores_softmax(int Cin, int N, int D, int heads, int g, int gpad, int Np,
                                                        const bf16* __restrict__ z, const bf16* __restrict__ Mb,
                                                        float* __restrict__ alpha) {
  constexpr int NBUF = 8, PD = NBUF - 1;                 // PD steps of loads in flight per lane and fragment
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int krow = D * 2 + 16;                           // bytes of one padded key row
  float* sc = reinterpret_cast<float*>(smem + 16 * krow);   // [gpad][16 heads][32 patches]
  const int k = blockIdx.y, G = gridDim.y, b = blockIdx.z, n0 = blockIdx.x * 32;
  const int c0 = k * g;
  const int gk = min(g, Cin - c0);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l16 = lane & 15, lq = lane >> 4;
  const int KF = D / 32;

  for (int idx = threadIdx.x; idx < 16 * (D / 8); idx += 512) {
    const int head = idx / (D / 8), c = idx % (D / 8);
    bf16x8 v = {};
    if (head < heads) v = *reinterpret_cast<const bf16x8*>(Mb + ((size_t)k * heads + head) * D + c * 8);
    *reinterpret_cast<bf16x8*>(smem + head * krow + c * 16) = v;
  }
  __syncthreads();

  if (wave < gk) {
    const bf16* zb0 = z + (((size_t)b * Cin + c0) * N + min(n0 + l16, N - 1)) * D + lq * 8;
    const bf16* zb1 = z + (((size_t)b * Cin + c0) * N + min(n0 + 16 + l16, N - 1)) * D + lq * 8;
    const size_t cstride = (size_t)N * D;
    const unsigned char* kfrag = smem + l16 * krow + lq * 16;
    const int last = wave + ((gk - 1 - wave) / 8) * 8;     // this wavefront's last member
    bf16x8 a0[NBUF], a1[NBUF];
#pragma unroll
    for (int t = 0; t < PD; ++t) {
      a0[t] = *reinterpret_cast<const bf16x8*>(zb0 + (size_t)wave * cstride + t * 32);
      a1[t] = *reinterpret_cast<const bf16x8*>(zb1 + (size_t)wave * cstride + t * 32);
    }
    for (int cl = wave; cl < gk; cl += 8) {
      const size_t co = (size_t)cl * cstride;
      const size_t no = (size_t)min(cl + 8, last) * cstride - (size_t)KF * 32;   // past the end: re-read (unused)
      f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
      for (int tb = 0; tb < KF; tb += NBUF) {
#pragma unroll
        for (int u = 0; u < NBUF; ++u) {
          const int t = tb + u, tp = t + PD;               // tp: the step whose loads are issued now
          const size_t off = (tp < KF ? co : no) + (size_t)tp * 32;
          a0[(u + PD) % NBUF] = *reinterpret_cast<const bf16x8*>(zb0 + off);
          a1[(u + PD) % NBUF] = *reinterpret_cast<const bf16x8*>(zb1 + off);
          const bf16x8 kf = *reinterpret_cast<const bf16x8*>(kfrag + t * 64);
          acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0[u], kf, acc0, 0, 0, 0);
          acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1[u], kf, acc1, 0, 0, 0);
        }
      }
      // 16x16 accumulator block: lane holds head (lane % 16), patches 4 * (lane / 16) + 0..3
      *reinterpret_cast<f32x4*>(&sc[(cl * 16 + l16) * 32 + lq * 4]) = acc0;
      *reinterpret_cast<f32x4*>(&sc[(cl * 16 + l16) * 32 + 16 + lq * 4]) = acc1;
    }
  }
  __syncthreads();
  const int head = threadIdx.x >> 5, patch = threadIdx.x & 31;
  if (head >= heads) return;
  const int n = n0 + patch;
  const size_t stride = (size_t)heads * Np;
  float* p = alpha + ((((size_t)b * G + k) * gpad) * heads + head) * Np + n;
  if (n >= N) {                                            // pitch padding: never scored, weight zero
    for (int cl = 0; cl < gpad; ++cl) p[cl * stride] = 0.f;
    return;
  }
  const float* s = sc + head * 32 + patch;
  float mx = -INFINITY;
  for (int cl = 0; cl < gk; ++cl) mx = fmaxf(mx, s[cl * 512]);
  float den = 0.f;
  for (int cl = 0; cl < gk; ++cl) den += __expf(s[cl * 512] - mx);
  const float inv = 1.f / den;
  for (int cl = 0; cl < gk; ++cl) p[cl * stride] = __expf(s[cl * 512] - mx) * inv;
  for (int cl = gk; cl < gpad; ++cl) p[cl * stride] = 0.f;
}

// ---------------------------------------------------------------------------------------------
// In-place softmax over the members of a group: S[b][k][0..gk)[head][n] -> alpha, zeros for cl >= gk.
// grid (ceil(Np/256), heads, B*G), block 256; one thread per (b, k, head, n).
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_softmax_alpha(int Cin, int N, int heads, int g, int gpad, int G, int Np,
                                                       float* __restrict__ S) {
  const int n = blockIdx.x * 256 + threadIdx.x;
  if (n >= Np) return;
  const int head = blockIdx.y;
  const int k = blockIdx.z % G;
  const int gk = min(g, Cin - k * g);
  const size_t stride = (size_t)heads * Np;
  float* p = S + ((size_t)blockIdx.z * gpad * heads + head) * Np + n;
  if (n >= N) {                                          // pitch padding: never scored, weight zero
    for (int cl = 0; cl < gpad; ++cl) p[cl * stride] = 0.f;
    return;
  }
  if (gk <= 32) {
    // the whole group in registers: all loads of the thread are in flight together, one pass over memory each way
    // (same arithmetic and order as the loop below)
    float v[32];
#pragma unroll
    for (int cl = 0; cl < 32; ++cl) v[cl] = cl < gk ? p[cl * stride] : -INFINITY;
    float mx = -INFINITY;
#pragma unroll
    for (int cl = 0; cl < 32; ++cl) mx = fmaxf(mx, v[cl]);
    float den = 0.f;
#pragma unroll
    for (int cl = 0; cl < 32; ++cl)
      if (cl < gk) den += __expf(v[cl] - mx);
    const float inv = 1.f / den;
#pragma unroll
    for (int cl = 0; cl < 32; ++cl)
      if (cl < gk) p[cl * stride] = __expf(v[cl] - mx) * inv;
    for (int cl = gk; cl < gpad; ++cl) p[cl * stride] = 0.f;
    return;
  }
  float mx = -INFINITY;
  for (int cl = 0; cl < gk; ++cl) mx = fmaxf(mx, p[cl * stride]);
  float den = 0.f;
  for (int cl = 0; cl < gk; ++cl) den += __expf(p[cl * stride] - mx);
  const float inv = 1.f / den;
  for (int cl = 0; cl < gk; ++cl) p[cl * stride] = __expf(p[cl * stride] - mx) * inv;
  for (int cl = gk; cl < gpad; ++cl) p[cl * stride] = 0.f;
}

// ---------------------------------------------------------------------------------------------
// GEMM core pieces shared by k_vagg_mfma and k_linear_dl.
//   Block tile 256 x 256 x 64, wavefront (wm, wn) of 2 x 4 owns rows [128 wm, +128) x cols [64 wn, +64):
//   TM = 4 by TN = 2 MFMA blocks of 32 x 32.  One stage = A rows 0..255 then B rows 0..255, 128 bytes each;
//   two stages: while one is multiplied the other is filled by direct-to-LDS loads of 128-byte row
//   segments (8 lanes per row), issued a whole slice ahead.
//   Global -> LDS: wavefront w issues 4 A loads and 4 B loads per slice; load i covers tile rows
//   w*32 + i*8 + lane/8, i.e. the A rows of wavefront w are the 32 patches of ONE channel of the chunk.
// ---------------------------------------------------------------------------------------------
struct GemmLane {
  int lane, wave, wm, wn, l32, lhi;
  int a_base, b_base;             // byte offsets of this lane's first A / B fragment row inside a stage
  int ck[4];                      // swizzled chunk byte offset of k-step kk
  __device__ __forceinline__ void init() {
    lane = threadIdx.x & 63;
    wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform: lives in a scalar register
    wm = wave / kGemmWN;
    wn = wave % kGemmWN;
    l32 = lane & 31;
    lhi = lane >> 5;
    a_base = (wm * 128 + l32) * 128;
    b_base = kGemmBM * 128 + (wn * 64 + l32) * 128;
    const int sw = swz_chunk(l32);               // row offsets of the other fragments are multiples of 32
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) ck[kk] = ((kk * 2 + lhi) ^ sw) * 16;
  }
  // load i of this wavefront covers tile row wave*32 + i*8 + lane/8, logical chunk (lane%8) ^ swz(row)
  __device__ __forceinline__ int load_row(int i) const { return wave * 32 + i * 8 + (lane >> 3); }
  __device__ __forceinline__ int load_chunk(int row) const { return (lane & 7) ^ swz_chunk(row); }
};

struct Frags {
  bf16x8 a[4], b[2];
};

// Timing probes of the GEMM core (compile-time; 0 in the product build).  `python -m paper_2506_21411_amd.build
// --define DCHAG_GEMM_PROBE=n --out <file>` builds a library whose RESULTS ARE MEANINGLESS and whose timing tells what
// each part of k_vagg_mfma costs: bit 1 = no MFMAs (the fragments are still read), 2 = no fragment reads, 4 = no
// barrier per slice, 8 = no global -> LDS loads (32 = none of the A operand, 64 = none of the B operand, k_vagg_mfma only),
// 16 = k_linear_dl stores (next to) nothing.  Every access stays in bounds
// and every loop keeps its trip count.
#ifndef DCHAG_GEMM_PROBE
#define DCHAG_GEMM_PROBE 0
#endif

__device__ __forceinline__ void read_frags(Frags& f, const unsigned char* stage, const GemmLane& L, int kk) {
  if (DCHAG_GEMM_PROBE & 2) {                            // keep the registers opaque, read nothing
#pragma unroll
    for (int i = 0; i < 4; ++i) asm volatile("" : "+v"(f.a[i]));
#pragma unroll
    for (int j = 0; j < 2; ++j) asm volatile("" : "+v"(f.b[j]));
    return;
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) f.a[i] = *reinterpret_cast<const bf16x8*>(stage + L.a_base + i * 4096 + L.ck[kk]);
#pragma unroll
  for (int j = 0; j < 2; ++j) f.b[j] = *reinterpret_cast<const bf16x8*>(stage + L.b_base + j * 4096 + L.ck[kk]);
}

__device__ __forceinline__ void mfma_step(f32x16 (&acc)[4][2], const Frags& f) {
  if (DCHAG_GEMM_PROBE & 1) {                            // the fragments count as used, nothing is multiplied
#pragma unroll
    for (int i = 0; i < 4; ++i) asm volatile("" : : "v"(f.a[i]));
#pragma unroll
    for (int j = 0; j < 2; ++j) asm volatile("" : : "v"(f.b[j]));
    return;
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[i], f.b[j], acc[i][j], 0, 0, 0);
}

// First k-step of an accumulation: C = 0 is an inline operand of the MFMA, the accumulators need no clearing.
__device__ __forceinline__ void mfma_step_first(f32x16 (&acc)[4][2], const Frags& f) {
  if (DCHAG_GEMM_PROBE & 1) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    mfma_step(acc, f);
    return;
  }
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[i], f.b[j], zero, 0, 0, 0);
}

// Scheduling of one k-step of the GEMM loops: the six fragment reads of step kk + 1 and the eight products of step kk
// that were written since the last scheduling barrier are issued as product, read, product, read, ... (a read behind
// each of the first six products), and nothing moves across the end of the step.  Left alone, the compiler sinks the
// reads next to their use to save registers and then waits for each of them in turn; in this order every wait is a
// counted one for fragments that were requested a whole step earlier.
__device__ __forceinline__ void pin_step_schedule() {
#pragma unroll
  for (int t = 0; t < 6; ++t) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // one MFMA
    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // one LDS read
  }
  __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
  __builtin_amdgcn_sched_barrier(0);
}

// One 64-deep slice: four k-steps with the fragments of step kk+1 read while step kk multiplies.
__device__ __forceinline__ void mfma_slice(f32x16 (&acc)[4][2], const unsigned char* stage, const GemmLane& L) {
  Frags f0, f1;
  read_frags(f0, stage, L, 0);
  read_frags(f1, stage, L, 1);
  mfma_step(acc, f0);
  read_frags(f0, stage, L, 2);
  mfma_step(acc, f1);
  read_frags(f1, stage, L, 3);
  mfma_step(acc, f0);
  mfma_step(acc, f1);
}

// ---------------------------------------------------------------------------------------------
// Value projection with the channel aggregation in its epilogue:
//   O[b,k,n,o] = sum_{cl < gk} alpha[b][k][cl][head(o)][n] * (z[b, k*g + cl, n, :] . Wv[k][o][:]) + bv[k][o]
// Work item (decoded by TileWork with m = patch tile): group k, batch b, 32 patches, 256 columns; the group
// is walked in chunks of 8 channels.  LDS tile row (wm*128 + i*32 + l) holds channel 2i + l/16 of the chunk,
// patch 16*wm + l%16, so wavefront (wm, wn) sees all 8 channels of ITS 16 patches: the weighted sum over
// the channels stays inside the wavefront's registers (rows q = 0,1 of an accumulator block belong to
// channel 2i, rows q = 2,3 to channel 2i+1) and no cross-wavefront merge is needed.
// The kernel is persistent: workgroup L takes items L/8, L/8 + slots, ... of its XCD's contiguous
// range, and the two-stage ring keeps prefetching across chunk and item boundaries (one slice ahead).
// Requires D % 256 == 0, dh = D / heads a multiple of 32, and 256 % dh == 0 or dh % 256 == 0.
// Dynamic LDS: ring (128 KiB) + 3 alpha tiles of 8 * NHS * 32 floats, used round-robin by chunk.
// ---------------------------------------------------------------------------------------------
struct VaggItem {
  int k, b, n0, o0, c0, gk, nch, h0, ch0, split;
};

__global__ __launch_bounds__(512) void k_vagg_mfma(int Cin, int N, int D, int heads, int g, int gpad, int G, int Np,
                                                   TileWork tw, int slots, const bf16* __restrict__ z,
                                                   const bf16* __restrict__ Wv, const bf16* __restrict__ bv,
                                                   const float* __restrict__ alpha, bf16* __restrict__ O, int S,
                                                   float* __restrict__ Opart) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  const int KT = D / kGemmBK;
  const int dh = D / heads;
  const int NHS = dh >= kGemmBN ? 1 : kGemmBN / dh;      // heads inside a 256-column slice
  unsigned char* alds = smem + kGemmRingBytes;           // 3 tiles of [8][NHS][32] floats
  const int atile = 8 * NHS * 32 * 4;

  // this workgroup's items: w = xcd * per + t * slots + slot, t = 0, 1, ...
  const int xcd = blockIdx.x % kXcds, slot = blockIdx.x / kXcds;
  const int per = (tw.total + kXcds - 1) / kXcds;
  const int xcd_end = min((xcd + 1) * per, tw.total);
  auto item_of = [&](int t, VaggItem& it) -> bool {
    const int w = xcd * per + t * slots + slot;
    if (w >= xcd_end) return false;
    int pt, nt;
    it.split = w % S;                                    // the group's chunks are dealt to S items (S <= chunks of any group)
    tw.decode_linear(w / S, it.k, it.b, pt, nt);
    it.n0 = pt * 32;
    it.o0 = nt * kGemmBN;
    it.c0 = it.k * g;
    it.gk = min(g, Cin - it.c0);
    const int nch = (it.gk + 7) / 8;
    it.ch0 = it.split * nch / S;
    it.nch = (it.split + 1) * nch / S - it.ch0;
    it.h0 = it.o0 / dh;
    return true;
  };

  GemmLane L;
  L.init();
  // A loads of wavefront w fill LDS rows w*32 + i*8 + lane/8: channel 2*(w%4) + (l>>4), patch 16*(w/4) + (l&15)
  int a_ch[4], a_patch[4], ld_chunk[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int l = i * 8 + (L.lane >> 3);
    a_ch[i] = 2 * (L.wave & 3) + (l >> 4);
    a_patch[i] = 16 * (L.wave >> 2) + (l & 15);
    ld_chunk[i] = L.load_chunk(L.load_row(i)) * 8;
  }

  // ---- issue side ----
  VaggItem ii;
  int ti = 0;
  bool live = item_of(0, ii);
  if (!live) return;                                     // uniform: the whole workgroup has nothing to do
  size_t a_rowoff[4];
  const bf16* b_src[4];
  const bf16* zb;
  const bf16* a_cur[4];                                  // running source pointers: advance 64 elements per slice
  const bf16* b_cur[4];
  int ci = 0, ki = 0, si = 0, gci = 0;                   // chunk, k-slice, stage, running chunk count (alpha buffer)
  auto setup_chunk = [&]() {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int c = ii.c0 + min((ii.ch0 + ci) * 8 + a_ch[i], ii.gk - 1);
      a_cur[i] = zb + (size_t)c * N * D + a_rowoff[i];
      b_cur[i] = b_src[i];
    }
  };
  auto setup_issue = [&]() {
    zb = z + (size_t)ii.b * Cin * N * D;
    const bf16* Wb = Wv + (size_t)ii.k * D * D;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      a_rowoff[i] = (size_t)min(ii.n0 + a_patch[i], N - 1) * D + ld_chunk[i];
      b_src[i] = Wb + (size_t)(ii.o0 + L.load_row(i)) * D + ld_chunk[i];
    }
  };
  setup_issue();
  setup_chunk();
  auto issue = [&]() {
    if (live) {
      if (ki == 0 && L.wave < NHS) {                     // entering a chunk: fetch its softmax weights
        const int sgm = L.wave * 8 + (L.lane >> 3);      // segment = (channel of the chunk, head of the slice)
        const int cl = (ii.ch0 + ci) * 8 + sgm / NHS, hd = sgm % NHS;
        const float* src = alpha + ((((size_t)ii.b * G + ii.k) * gpad + cl) * heads + ii.h0 + hd) * Np + ii.n0 +
                           (L.lane & 7) * 4;
        load16_to_lds(src, alds + (gci % 3) * atile + L.wave * 1024);
      }
      unsigned char* st = smem + si * kGemmStageBytes + L.wave * 4096;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if (!(DCHAG_GEMM_PROBE & (8 | 32))) load16_to_lds(a_cur[i], st + i * 1024);
        a_cur[i] += kGemmBK;
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if (!(DCHAG_GEMM_PROBE & (8 | 64))) load16_to_lds(b_cur[i], st + kGemmBM * 128 + i * 1024);
        b_cur[i] += kGemmBK;
      }
      if (++ki == KT) {
        ki = 0;
        ++gci;
        if (++ci == ii.nch) {
          ci = 0;
          live = item_of(++ti, ii);
          if (live) setup_issue();
        }
        if (live) setup_chunk();
      }
    }
    si ^= 1;
  };

  // ---- compute side ----
  issue();                                               // first slice -> stage 0
  int sc = 0, gcc = 0;
  Frags f0, f1;
  wait_vmcnt<0>();
  __builtin_amdgcn_s_barrier();
  if (L.wm == 0) issue();                                // second slice -> stage 1 (wm = 1 issues inside the loop)
  read_frags(f0, smem, L, 0);
  VaggItem ic;
  for (int tc = 0; item_of(tc, ic); ++tc) {
    f32x16 o[2];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[j][r] = 0.f;      // only entries 0..7 are used
    for (int chunk = 0; chunk < ic.nch; ++chunk, ++gcc) {
      f32x16 acc[4][2];
      for (int kt = 0; kt < KT; ++kt) {
        // k-steps 0..2 of the current slice; the fragments of step 0 were read across the last barrier.  Each step's
        // products are issued with the reads of the step after it between them (pin_step_schedule).
        const unsigned char* st = smem + sc * kGemmStageBytes;
        __builtin_amdgcn_sched_barrier(0);
        read_frags(f1, st, L, 1);
        if (kt == 0) mfma_step_first(acc, f0);           // a chunk starts from C = 0
        else mfma_step(acc, f0);
        pin_step_schedule();
        if (L.wm == 1) issue();                          // slice after next -> the stage released at the last barrier
        __builtin_amdgcn_sched_barrier(0);
        read_frags(f0, st, L, 2);
        mfma_step(acc, f1);
        pin_step_schedule();
        read_frags(f1, st, L, 3);
        mfma_step(acc, f0);
        pin_step_schedule();
        // every read of this stage is in registers and the next slice has landed: swap stages
        __builtin_amdgcn_s_waitcnt(0);                   // vmcnt(0) and lgkmcnt(0)
        if (!(DCHAG_GEMM_PROBE & 4)) __builtin_amdgcn_s_barrier();
        if (L.wm == 0) issue();                          // slice after next -> the stage just released
        sc ^= 1;
        __builtin_amdgcn_sched_barrier(0);
        read_frags(f0, smem + sc * kGemmStageBytes, L, 0);
        mfma_step(acc, f1);
        pin_step_schedule();
      }
      // o += alpha * acc over the 8 channels of the chunk (channel 2i in rows q = 0,1; 2i+1 in rows q = 2,3)
      const float* al = reinterpret_cast<const float*>(alds + (gcc % 3) * atile);
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int hrel = (ic.o0 + L.wn * 64 + j * 32) / dh - ic.h0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
#pragma unroll
          for (int half = 0; half < 2; ++half) {
            const float* ap = al + ((2 * i + half) * NHS + hrel) * 32 + 16 * L.wm + 4 * L.lhi;
#pragma unroll
            for (int q = 0; q < 2; ++q) {
              const f32x4 a4 = *reinterpret_cast<const f32x4*>(ap + 8 * q);
#pragma unroll
              for (int e = 0; e < 4; ++e) o[j][4 * q + e] += a4[e] * acc[i][j][8 * half + 4 * q + e];
            }
          }
        }
      }
    }
    if (S == 1) {
      bf16* Ob = O + (((size_t)ic.b * G + ic.k) * N) * D;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int col = ic.o0 + L.wn * 64 + j * 32 + L.l32;
        const float bias = bv ? (float)bv[(size_t)ic.k * D + col] : 0.f;
#pragma unroll
        for (int r = 0; r < 8; ++r) {
          const int nrow = ic.n0 + 16 * L.wm + 8 * (r >> 2) + 4 * L.lhi + (r & 3);
          if (nrow < N) Ob[(size_t)nrow * D + col] = (bf16)(o[j][r] + bias);
        }
      }
    } else {                                             // partial sum over this item's chunks; k_vagg_merge adds them up
      float* Pb = Opart + ((((size_t)ic.split * tw.nb + ic.b) * G + ic.k) * N) * D;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int col = ic.o0 + L.wn * 64 + j * 32 + L.l32;
#pragma unroll
        for (int r = 0; r < 8; ++r) {
          const int nrow = ic.n0 + 16 * L.wm + 8 * (r >> 2) + 4 * L.lhi + (r & 3);
          if (nrow < N) Pb[(size_t)nrow * D + col] = o[j][r];
        }
      }
    }
  }
  wait_vmcnt<0>();                                       // nothing may still target LDS when the block retires
}

// O[b,k,n,:] = sum over the S partial sums of k_vagg_mfma + bv[k][:], in a fixed order.  One thread per 4 columns.
__global__ __launch_bounds__(256) void k_vagg_merge(long quads, int S, int G, int N, int D, long per_split,
                                                    const float* __restrict__ Opart, const bf16* __restrict__ bv,
                                                    bf16* __restrict__ O) {
  const long q = (long)blockIdx.x * 256 + threadIdx.x;
  if (q >= quads) return;
  const long i = q * 4;                                  // ((b * G + k) * N + n) * D + col
  const int col = (int)(i % D);
  const int k = (int)((i / ((long)N * D)) % G);
  f32x4 acc = *reinterpret_cast<const f32x4*>(Opart + i);
  for (int sidx = 1; sidx < S; ++sidx) acc += *reinterpret_cast<const f32x4*>(Opart + sidx * per_split + i);
  bf16x4 out;
#pragma unroll
  for (int e = 0; e < 4; ++e) out[e] = (bf16)(acc[e] + (bv ? (float)bv[(size_t)k * D + col + e] : 0.f));
  *reinterpret_cast<bf16x4*>(O + i) = out;
}

// ---------------------------------------------------------------------------------------------
// Plain per-group projection  Y[r][o] = sum_j A[r][j] * Wt[k][o][j] + bias[k][o] (+ rowadd[r][o])  on the same core.
// Requires D % 256 == 0.  Dynamic LDS: the ring (128 KiB).
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(512) void k_linear_dl(int D, RowBlocks rb, TileWork tw, const bf16* __restrict__ A,
                                                   const bf16* __restrict__ Wt, const bf16* __restrict__ bias,
                                                   bf16* __restrict__ Y, const bf16* __restrict__ rowadd) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  int k, b, mt, nt;
  if (!tw.decode(blockIdx.x, k, b, mt, nt)) return;
  const int rows = rb.rows_of(k);
  const int r0 = mt * kGemmBM, o0 = nt * kGemmBN;
  if (r0 >= rows) return;
  const int KT = D / kGemmBK;
  GemmLane L;
  L.init();
  const bf16* Ab = A + (size_t)rb.first_row(b, k) * D;
  bf16* Yb = Y + (size_t)rb.first_row(b, k) * D;
  const bf16* Wb = Wt + (size_t)k * D * D;
  const bf16* a_src[4];
  const bf16* b_src[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = L.load_row(i);
    a_src[i] = Ab + (size_t)min(r0 + row, rows - 1) * D + L.load_chunk(row) * 8;
    b_src[i] = Wb + (size_t)(o0 + row) * D + L.load_chunk(row) * 8;
  }
  int ki = 0, si = 0;
  auto issue = [&]() {
    unsigned char* st = smem + si * kGemmStageBytes;
#pragma unroll
    for (int i = 0; i < 4; ++i) load16_to_lds(a_src[i] + ki * kGemmBK, st + (L.wave * 4 + i) * 1024);
#pragma unroll
    for (int i = 0; i < 4; ++i)
      load16_to_lds(b_src[i] + ki * kGemmBK, st + kGemmBM * 128 + (L.wave * 4 + i) * 1024);
    si ^= 1;
    ki = (ki + 1 < KT) ? ki + 1 : ki;                    // past the end: harmless re-load of the last slice
  };
  // The pipeline of k_vagg_mfma: the fragments of a slice's first k-step are read across the barrier that hands the
  // slice over, the products of its last k-step are issued behind that barrier, and the two wavefronts of a SIMD
  // (wm = 0 and 1) issue their loads at different points of the slice.
  f32x16 acc[4][2];
  Frags f0, f1;
  issue();                                               // slice 0 -> stage 0
  wait_vmcnt<0>();
  __builtin_amdgcn_s_barrier();
  if (L.wm == 0) issue();                                // slice 1 -> stage 1 (wm = 1 issues inside the loop)
  read_frags(f0, smem, L, 0);
  int sc = 0;
  for (int kt = 0; kt < KT; ++kt) {
    const unsigned char* st = smem + sc * kGemmStageBytes;
    __builtin_amdgcn_sched_barrier(0);
    read_frags(f1, st, L, 1);
    if (kt == 0) mfma_step_first(acc, f0);
    else mfma_step(acc, f0);
    pin_step_schedule();
    if (L.wm == 1) issue();                              // slice kt + 1 -> the stage released at the last barrier
    __builtin_amdgcn_sched_barrier(0);
    read_frags(f0, st, L, 2);
    mfma_step(acc, f1);
    pin_step_schedule();
    read_frags(f1, st, L, 3);
    mfma_step(acc, f0);
    pin_step_schedule();
    __builtin_amdgcn_s_waitcnt(0);                       // vmcnt(0) and lgkmcnt(0): slice kt + 1 has landed
    __builtin_amdgcn_s_barrier();
    if (L.wm == 0) issue();                              // slice kt + 2 -> the stage just released
    sc ^= 1;
    __builtin_amdgcn_sched_barrier(0);
    read_frags(f0, smem + sc * kGemmStageBytes, L, 0);   // past the last slice: a re-load of it, read and not used
    mfma_step(acc, f1);
    pin_step_schedule();
  }
  wait_vmcnt<0>();                                       // no load may still target LDS when the block retires
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int col = o0 + L.wn * 64 + j * 32 + L.l32;
    const float bvv = bias ? (float)bias[(size_t)k * D + col] : 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = r0 + L.wm * 128 + i * 32 + 8 * (r >> 2) + 4 * L.lhi + (r & 3);
        if (row < rows && !((DCHAG_GEMM_PROBE & 16) && acc[i][j][r] != 12345.f))
          Yb[(size_t)row * D + col] = (bf16)(acc[i][j][r] + bvv + (rowadd ? (float)rowadd[(size_t)row * D + col] : 0.f));
      }
  }
}

// ---------------------------------------------------------------------------------------------
// The same projection for a problem of FEW tiles (the output projection of an upper level: 64 tiles of 128 x 128 at the
// headline shape).  With less than one 256 x 256 tile per compute unit the run time is the depth of the contraction times
// the round trip of one slice's loads, so this form trades tile size for depth of prefetch: 128 x 128 tiles, four
// wavefronts (2 x 2) of 64 x 64, FOUR 32-KiB stages filled by direct-to-LDS loads issued three slices ahead; a slice
// then costs its transfer and its 16 MFMAs per wavefront, not a round trip.  One barrier per slice; the fragments of a
// slice are read behind it.  Requires D % 128 == 0.  Dynamic LDS: 128 KiB.
// ---------------------------------------------------------------------------------------------
constexpr int kSmallStageBytes = 256 * 128, kSmallStages = 4, kSmallRingBytes = kSmallStages * kSmallStageBytes;

__global__ __launch_bounds__(256) void k_linear_ring(int D, RowBlocks rb, TileWork tw, const bf16* __restrict__ A,
                                                     const bf16* __restrict__ Wt, const bf16* __restrict__ bias,
                                                     bf16* __restrict__ Y, const bf16* __restrict__ rowadd) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  int k, b, mt, nt;
  if (!tw.decode(blockIdx.x, k, b, mt, nt)) return;
  const int rows = rb.rows_of(k);
  const int r0 = mt * 128, o0 = nt * 128;
  if (r0 >= rows) return;
  const int KT = D / kGemmBK;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wave >> 1, wn = wave & 1, l32 = lane & 31, lhi = lane >> 5;
  const bf16* Ab = A + (size_t)rb.first_row(b, k) * D;
  bf16* Yb = Y + (size_t)rb.first_row(b, k) * D;
  const bf16* Wb = Wt + (size_t)k * D * D;
  // a stage: A rows 0..127, then B rows 0..127, 128 bytes each, chunks swizzled as in the large core; wavefront w loads
  // rows 32 w .. 32 w + 31 of both (four loads each per slice)
  const bf16* a_src[4];
  const bf16* b_src[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = wave * 32 + i * 8 + (lane >> 3);
    const int ch = ((lane & 7) ^ swz_chunk(row)) * 8;
    a_src[i] = Ab + (size_t)min(r0 + row, rows - 1) * D + ch;
    b_src[i] = Wb + (size_t)(o0 + row) * D + ch;
  }
  int issued = 0;
  auto issue = [&]() {                                   // slice `issued` -> stage issued % 4
    unsigned char* st = smem + (issued & 3) * kSmallStageBytes + wave * 4096;
#pragma unroll
    for (int i = 0; i < 4; ++i) load16_to_lds(a_src[i] + issued * kGemmBK, st + i * 1024);
#pragma unroll
    for (int i = 0; i < 4; ++i) load16_to_lds(b_src[i] + issued * kGemmBK, st + 128 * 128 + i * 1024);
    ++issued;
  };
  const int a_base = (wm * 64 + l32) * 128, b_base = 128 * 128 + (wn * 64 + l32) * 128;
  int ck[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) ck[kk] = ((kk * 2 + lhi) ^ swz_chunk(l32)) * 16;

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  for (int s0 = 0; s0 < 3 && s0 < KT; ++s0) issue();
  for (int kt = 0; kt < KT; ++kt) {
    // slice kt has landed (this wavefront's share; the slices behind it may stay in flight: 8 loads each) ...
    const int behind = issued - 1 - kt;                  // uniform
    if (behind >= 2) wait_vmcnt<16>();
    else if (behind == 1) wait_vmcnt<8>();
    else wait_vmcnt<0>();
    // ... and for everyone; all wavefronts are done with slice kt - 1, whose stage takes slice kt + 3
    __builtin_amdgcn_s_barrier();
    if (issued < KT) issue();
    const unsigned char* st = smem + (kt & 3) * kSmallStageBytes;
    bf16x8 af[4][2], bfr[4][2];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        af[kk][i] = *reinterpret_cast<const bf16x8*>(st + a_base + i * 4096 + ck[kk]);
        bfr[kk][i] = *reinterpret_cast<const bf16x8*>(st + b_base + i * 4096 + ck[kk]);
      }
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[kk][i], bfr[kk][j], acc[i][j], 0, 0, 0);
  }
  wait_vmcnt<0>();                                       // nothing may still target LDS when the block retires
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int col = o0 + wn * 64 + j * 32 + l32;
    const float bvv = bias ? (float)bias[(size_t)k * D + col] : 0.f;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = r0 + wm * 64 + i * 32 + 8 * (r >> 2) + 4 * lhi + (r & 3);
        if (row < rows)
          Yb[(size_t)row * D + col] = (bf16)(acc[i][j][r] + bvv + (rowadd ? (float)rowadd[(size_t)row * D + col] : 0.f));
      }
  }
}

// ---------------------------------------------------------------------------------------------
// Value projection folded into the tokenizer weights (weight-only; 64 pixels per patch), on the same core:
//   Wf[c][o][kk] = sum_d Wv[k][o][d] * We[c][d][kk],   k = c / g.
// Work item: group k, 256 rows o, four channels of the group (one per wavefront column wn).  The A operand (rows of
// Wv, contraction index contiguous) goes through the ring as in k_linear_dl; the B stage holds, per channel, the 64
// rows d of the slice as they lie in memory (128 bytes of kk each), so a B fragment (8 consecutive d of one column
// kk) is put together from eight 2-byte LDS reads -- the operand is small, the A tile is shared by the four channels,
// which is what the product's L2 traffic hinges on.  Requires D % 256 == 0.  Dynamic LDS: the ring (128 KiB).
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(512) void k_fold_value_dl(int C, int D, int g, TileWork tw, const bf16* __restrict__ Wv,
                                                       const bf16* __restrict__ We, bf16* __restrict__ Wf) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  int k, b, mt, nt;
  if (!tw.decode(blockIdx.x, k, b, mt, nt)) return;
  const int c0 = k * g, gk = min(g, C - c0), q0 = nt * 4;
  if (q0 >= gk) return;                                  // uniform: a short last group has fewer quads
  const int r0 = mt * kGemmBM;
  const int KT = D / kGemmBK;
  GemmLane L;
  L.init();
  const bf16* a_src[4];
  const bf16* b_src[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = L.load_row(i);
    a_src[i] = Wv + ((size_t)k * D + r0 + row) * D + L.load_chunk(row) * 8;
    const int c = c0 + min(q0 + (row >> 6), gk - 1);     // a missing channel of the quad repeats the last one; not stored
    b_src[i] = We + ((size_t)c * D + (row & 63)) * 64 + L.load_chunk(row) * 8;
  }
  int ki = 0, si = 0;
  auto issue = [&]() {
    unsigned char* st = smem + si * kGemmStageBytes;
#pragma unroll
    for (int i = 0; i < 4; ++i) load16_to_lds(a_src[i] + ki * kGemmBK, st + (L.wave * 4 + i) * 1024);
#pragma unroll
    for (int i = 0; i < 4; ++i)
      load16_to_lds(b_src[i] + (size_t)ki * 64 * 64, st + kGemmBM * 128 + (L.wave * 4 + i) * 1024);
    si ^= 1;
    ki = (ki + 1 < KT) ? ki + 1 : ki;                    // past the end: harmless re-load of the last slice
  };
  // byte offset, inside a stage's B half, of element (d = 8 lhi + i of a 16-deep k-step, column kk = 32 j + l32) of this
  // wavefront's channel; the k-step adds 16 rows (2048 bytes, no change of the row's chunk swizzle)
  int boff[2][8];
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int row = L.wn * 64 + L.lhi * 8 + i, col = j * 32 + L.l32;
      boff[j][i] = kGemmBM * 128 + row * 128 + (((col >> 3) ^ swz_chunk(row)) * 16) + (col & 7) * 2;
    }
  f32x16 acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  issue();
  int sc = 0;
  for (int kt = 0; kt < KT; ++kt) {
    wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();
    issue();
    const unsigned char* st = smem + sc * kGemmStageBytes;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      Frags f;
#pragma unroll
      for (int i = 0; i < 4; ++i) f.a[i] = *reinterpret_cast<const bf16x8*>(st + L.a_base + i * 4096 + L.ck[kk]);
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int i = 0; i < 8; ++i) f.b[j][i] = *reinterpret_cast<const bf16*>(st + boff[j][i] + kk * 2048);
      mfma_step(acc, f);
    }
    sc ^= 1;
  }
  wait_vmcnt<0>();                                       // no load may still target LDS when the block retires
  if (q0 + L.wn >= gk) return;
  bf16* out = Wf + ((size_t)(c0 + q0 + L.wn) * D + r0 + L.wm * 128 + 4 * L.lhi) * 64 + L.l32;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) out[(size_t)(i * 32 + 8 * (r >> 2) + (r & 3)) * 64 + j * 32] = (bf16)acc[i][j][r];
}

// The token biases under the same fold (weight-only):  fb[c][o] = sum_d (be[c][d] + ce[c][d]) * Wv[k][o][d],  k = c / g;
// either vector may be absent.  grid (D / 32, G), block 256: 32 rows o of Wv against the group's members, 32 per pass
// (one 32 x 32 MFMA block: rows o, columns members, operands straight from memory), the four wavefronts a quarter of d
// each, their partial blocks merged in LDS in a fixed order.  Requires D % 64 == 0 and 16-byte aligned rows.
__global__ __launch_bounds__(256) void k_fold_token_bias(int C, int D, int g, const bf16* __restrict__ Wv,
                                                         const bf16* __restrict__ be, const bf16* __restrict__ ce,
                                                         bf16* __restrict__ fb) {
  __shared__ float part[4][32][33];
  const int k = blockIdx.y, o0 = blockIdx.x * 32;
  const int c0 = k * g, gk = min(g, C - c0);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, lhi = lane >> 5;
  const int dq = D / 4;
  const bf16* arow = Wv + ((size_t)k * D + o0 + l32) * D + wave * dq + lhi * 8;
  for (int cb = 0; cb < gk; cb += 32) {
    const size_t coff = (size_t)(c0 + min(cb + l32, gk - 1)) * D + wave * dq + lhi * 8;
    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    for (int ks = 0; ks < dq; ks += 16) {
      const bf16x8 a = *reinterpret_cast<const bf16x8*>(arow + ks);
      if (be) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, *reinterpret_cast<const bf16x8*>(be + coff + ks), acc, 0, 0, 0);
      if (ce) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, *reinterpret_cast<const bf16x8*>(ce + coff + ks), acc, 0, 0, 0);
    }
    // accumulator register r of lane (member l32, half lhi): row o = 8 (r / 4) + 4 lhi + r % 4
#pragma unroll
    for (int r = 0; r < 16; ++r) part[wave][8 * (r >> 2) + 4 * lhi + (r & 3)][l32] = acc[r];
    __syncthreads();
    {
      const int mm = tid >> 3, r0 = 4 * (tid & 7);       // member of the pass, four adjacent rows o
      if (cb + mm < gk) {
        typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4_t;
        bf16x4_t out;
#pragma unroll
        for (int e = 0; e < 4; ++e)
          out[e] = (bf16)(part[0][r0 + e][mm] + part[1][r0 + e][mm] + part[2][r0 + e][mm] + part[3][r0 + e][mm]);
        *reinterpret_cast<bf16x4_t*>(fb + (size_t)(c0 + cb + mm) * D + o0 + r0) = out;
      }
    }
    __syncthreads();
  }
}

// ---------------------------------------------------------------------------------------------
// Level-1 scores straight from the pixels.  The tokenizer is linear, so the score of token
// t = We[c] u + be[c] + ce[c] against the folded key M[k][a] is
//   t . M[k][a] = u . (We[c]^T M[k][a]) + (be[c] + ce[c]) . M[k][a]
// k_compose_score_weights builds the weight-only pieces  Ms[c][a][kk] = sum_d M[k][a][d] We[c][d][kk]
// and cs[c][a] = sum_d M[k][a][d] (be[c][d] + ce[c][d]) in fp32 (k = c / g);
// k_scores_pixels then scores every (channel, patch) with a p*p-long dot product per head.
// ---------------------------------------------------------------------------------------------
// grid (C), block 256.  The channel's tokenizer weights and the transposed folded key MfT[G][D][heads]
// stream through LDS in blocks of DQ rows of d (full-width 16-byte loads); outputs are tiled 4 heads x 4
// pixels, lane l of every wavefront owns tiles l, l+64, ... (TPL of them) and wavefront w sums the
// rows d = w (mod 4) of a block; the four partial sums meet in LDS in a fixed order.  Writes fp32 Ms,
// its bf16 copy Msb (the MFMA operand of k_scores_pixels) and cs.
// Requires heads % 4 == 0, pp % 8 == 0, DQ % 4 == 0, D % DQ == 0.
// Dynamic LDS: DQ * (pp * 2 + heads * 4 + 4) bytes, then 3 * TPL * 64 * 20 floats.
template <int TPL>
__global__ __launch_bounds__(256) void k_compose_score_weights(int D, int heads, int pp, int g, int DQ,
                                                               const float* __restrict__ MfT,
                                                               const bf16* __restrict__ We, const bf16* __restrict__ be,
                                                               const bf16* __restrict__ ce, float* __restrict__ Ms,
                                                               bf16* __restrict__ Msb, float* __restrict__ cs) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16* w_s = reinterpret_cast<bf16*>(smem);                                   // [DQ][pp]
  float* m_s = reinterpret_cast<float*>(smem + (size_t)DQ * pp * 2);           // [DQ][heads]
  float* b_s = m_s + (size_t)DQ * heads;                                       // [DQ]
  float* part = b_s + DQ;                                                      // [3][TPL*20][64]
  const int c = blockIdx.x, k = c / g;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int kq_n = pp / 4, aq_n = heads / 4, ntiles = kq_n * aq_n;
  const float* M = MfT + (size_t)k * D * heads;
  const bf16* Wc = We + (size_t)c * D * pp;
  float acc[TPL][16], cacc[TPL][4];
  int kq[TPL], aq[TPL];
#pragma unroll
  for (int t = 0; t < TPL; ++t) {
    const int tile = lane + t * 64;
    kq[t] = tile < ntiles ? tile % kq_n : -1;
    aq[t] = tile < ntiles ? tile / kq_n : 0;
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;
#pragma unroll
    for (int e = 0; e < 4; ++e) cacc[t][e] = 0.f;
  }
  for (int d0 = 0; d0 < D; d0 += DQ) {
    __syncthreads();
    for (int idx = tid; idx < DQ * pp / 8; idx += 256)
      reinterpret_cast<bf16x8*>(w_s)[idx] = reinterpret_cast<const bf16x8*>(Wc + (size_t)d0 * pp)[idx];
    for (int idx = tid; idx < DQ * heads / 4; idx += 256)
      reinterpret_cast<f32x4*>(m_s)[idx] = reinterpret_cast<const f32x4*>(M + (size_t)d0 * heads)[idx];
    for (int idx = tid; idx < DQ; idx += 256) {
      float bsum = 0.f;
      if (be) bsum += (float)be[(size_t)c * D + d0 + idx];
      if (ce) bsum += (float)ce[(size_t)c * D + d0 + idx];
      b_s[idx] = bsum;
    }
    __syncthreads();
#pragma unroll 4
    for (int d = wave; d < DQ; d += 4) {
      const float bsum = b_s[d];
#pragma unroll
      for (int t = 0; t < TPL; ++t) {
        if (kq[t] < 0) continue;
        const f32x4 m4 = *reinterpret_cast<const f32x4*>(m_s + (size_t)d * heads + aq[t] * 4);
        const bf16x4 w4 = *reinterpret_cast<const bf16x4*>(w_s + (size_t)d * pp + kq[t] * 4);
#pragma unroll
        for (int a = 0; a < 4; ++a) {
#pragma unroll
          for (int q = 0; q < 4; ++q) acc[t][a * 4 + q] += m4[a] * (float)w4[q];
          cacc[t][a] += m4[a] * bsum;
        }
      }
    }
  }
  if (wave > 0) {
#pragma unroll
    for (int t = 0; t < TPL; ++t) {
#pragma unroll
      for (int e = 0; e < 16; ++e) part[((wave - 1) * TPL * 20 + t * 20 + e) * 64 + lane] = acc[t][e];
#pragma unroll
      for (int e = 0; e < 4; ++e) part[((wave - 1) * TPL * 20 + t * 20 + 16 + e) * 64 + lane] = cacc[t][e];
    }
  }
  __syncthreads();
  if (wave == 0) {
    float* Mo = Ms + (size_t)c * heads * pp;
    bf16* Mbo = Msb + (size_t)c * heads * pp;
#pragma unroll
    for (int t = 0; t < TPL; ++t) {
      if (kq[t] < 0) continue;
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        const int head = aq[t] * 4 + a;
        f32x4 v4;
        bf16x4 b4;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int e = a * 4 + q;
          v4[q] = acc[t][e] + part[((0 * TPL + t) * 20 + e) * 64 + lane] + part[((1 * TPL + t) * 20 + e) * 64 + lane] +
                  part[((2 * TPL + t) * 20 + e) * 64 + lane];
          b4[q] = (bf16)v4[q];
        }
        *reinterpret_cast<f32x4*>(Mo + (size_t)head * pp + kq[t] * 4) = v4;
        *reinterpret_cast<bf16x4*>(Mbo + (size_t)head * pp + kq[t] * 4) = b4;
        if (kq[t] == 0) {
          const int e = 16 + a;
          cs[(size_t)c * heads + head] = cacc[t][a] + part[((0 * TPL + t) * 20 + e) * 64 + lane] +
                                         part[((1 * TPL + t) * 20 + e) * 64 + lane] +
                                         part[((2 * TPL + t) * 20 + e) * 64 + lane];
        }
      }
    }
  }
}

// The same weights on 16x16x32 MFMA for pp = 16, 32, 64 or 128 (NKB = pp / 8 blocks of 8 pixels) and group sizes that
// are multiples of CPB = 16 / NKB: a block takes CPB channels of one group, its four wavefronts a quarter of D each.
// A fragments: the fp32 folded key rows Mf[k][head][d] split in two bf16 parts (nothing of them is lost); B fragments:
// a lane reads 8 rows d x 8 adjacent pixels of We[c] (16 bytes per row) and transposes them in registers, which gives
// it the fragments (column = channel l16 / NKB, pixel 8 (l16 % NKB) + j; d = 8 (lane / 16) ..) of eight products
// j = 0..7.  The bias part takes two more products per step (be and ce as they are: column = channel).  The partial
// blocks of the wavefronts meet in LDS in a fixed order.  grid (ceil(C / CPB)), block 256.  D % 128 == 0.
__device__ __forceinline__ void split_hi_lo(const f32x4& x0, const f32x4& x1, bf16x8& hi, bf16x8& lo) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    hi[i] = (bf16)x0[i];
    lo[i] = (bf16)(x0[i] - (float)hi[i]);
    hi[4 + i] = (bf16)x1[i];
    lo[4 + i] = (bf16)(x1[i] - (float)hi[4 + i]);
  }
}

template <int HB>   // blocks of 16 heads (heads <= 16 HB)
__global__ __launch_bounds__(256) void k_compose_score_weights_mfma(int C, int D, int heads, int pp, int g,
                                                                    const float* __restrict__ Mf,
                                                                    const bf16* __restrict__ We,
                                                                    const bf16* __restrict__ be,
                                                                    const bf16* __restrict__ ce, float* __restrict__ Ms,
                                                                    bf16* __restrict__ Msb, float* __restrict__ cs) {
  __shared__ f32x4 part[3][HB][9][64];
  const int nkb = pp / 8, cpb = 16 / nkb;
  const int c0 = blockIdx.x * cpb, k = c0 / g;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, l16 = lane & 15, lq = lane >> 4;
  const int csub = l16 / nkb, kkb = l16 % nkb;
  const int c = min(c0 + csub, C - 1);                   // a short last block: its repeats are not written
  const int cbias = min(c0 + l16, C - 1);                // the channel this lane supplies in the bias products
  const bf16* wsrc = We + (size_t)c * D * pp + kkb * 8;
  const int dq = D / 4;
  f32x4 acc[HB][8], bacc[HB];
#pragma unroll
  for (int hb = 0; hb < HB; ++hb) {
    bacc[hb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[hb][j] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  for (int d0 = wave * dq; d0 < (wave + 1) * dq; d0 += 32) {
    const int d = d0 + 8 * lq;                           // this lane's 8 steps of the contraction
    bf16x8 mhi[HB], mlo[HB];
#pragma unroll
    for (int hb = 0; hb < HB; ++hb) {
      const float* mp = Mf + ((size_t)k * heads + min(16 * hb + l16, heads - 1)) * D + d;
      split_hi_lo(*reinterpret_cast<const f32x4*>(mp), *reinterpret_cast<const f32x4*>(mp + 4), mhi[hb], mlo[hb]);
    }
    bf16x8 rows[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) rows[i] = *reinterpret_cast<const bf16x8*>(wsrc + (size_t)(d + i) * pp);
    bf16x8 bev = {}, cev = {};
    if (l16 < cpb) {
      if (be) bev = *reinterpret_cast<const bf16x8*>(be + (size_t)cbias * D + d);
      if (ce) cev = *reinterpret_cast<const bf16x8*>(ce + (size_t)cbias * D + d);
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      bf16x8 col;
#pragma unroll
      for (int i = 0; i < 8; ++i) col[i] = rows[i][j];
#pragma unroll
      for (int hb = 0; hb < HB; ++hb) {
        acc[hb][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(mhi[hb], col, acc[hb][j], 0, 0, 0);
        acc[hb][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(mlo[hb], col, acc[hb][j], 0, 0, 0);
      }
    }
#pragma unroll
    for (int hb = 0; hb < HB; ++hb) {
      bacc[hb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(mhi[hb], bev, bacc[hb], 0, 0, 0);
      bacc[hb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(mlo[hb], bev, bacc[hb], 0, 0, 0);
      bacc[hb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(mhi[hb], cev, bacc[hb], 0, 0, 0);
      bacc[hb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(mlo[hb], cev, bacc[hb], 0, 0, 0);
    }
  }
  if (wave > 0) {
#pragma unroll
    for (int hb = 0; hb < HB; ++hb) {
#pragma unroll
      for (int j = 0; j < 8; ++j) part[wave - 1][hb][j][lane] = acc[hb][j];
      part[wave - 1][hb][8][lane] = bacc[hb];
    }
  }
  __syncthreads();
  if (wave != 0) return;
  // accumulator block: lane holds column l16, rows (heads) 4 lq + r
#pragma unroll
  for (int hb = 0; hb < HB; ++hb) {
    f32x4 tot[9];
#pragma unroll
    for (int j = 0; j < 8; ++j) tot[j] = acc[hb][j] + part[0][hb][j][lane] + part[1][hb][j][lane] + part[2][hb][j][lane];
    tot[8] = bacc[hb] + part[0][hb][8][lane] + part[1][hb][8][lane] + part[2][hb][8][lane];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int head = 16 * hb + 4 * lq + r;
      if (head >= heads) continue;
      if (c0 + csub < C) {
        const size_t o = ((size_t)(c0 + csub) * heads + head) * pp + kkb * 8;
        *reinterpret_cast<f32x4*>(Ms + o) = f32x4{tot[0][r], tot[1][r], tot[2][r], tot[3][r]};
        *reinterpret_cast<f32x4*>(Ms + o + 4) = f32x4{tot[4][r], tot[5][r], tot[6][r], tot[7][r]};
        bf16x8 b8;
#pragma unroll
        for (int j = 0; j < 8; ++j) b8[j] = (bf16)tot[j][r];
        *reinterpret_cast<bf16x8*>(Msb + o) = b8;
      }
      if (l16 < cpb && c0 + l16 < C) cs[(size_t)(c0 + l16) * heads + head] = tot[8][r];
    }
  }
}

// Level-1 scores on MFMA: S[b][k][cl][head][n] = u[b,c,n][:] . Msb[c][head][:] + cs[c][head].
// grid (ceil(N/128), C, B), block 256: wavefront w scores 32 patches of channel c against up to 32 heads
// with one 32x32x16 MFMA per 16 pixels.  A lane's operand (8 consecutive pixels of a patch) is one
// 16-byte load when p % 8 == 0, two 8-byte loads when p == 4.  Requires heads <= 32, pp % 16 == 0.
__global__ __launch_bounds__(256) void k_scores_pixels(int C, int H, int W, int p, int heads, int g, int gpad, int G,
                                                       int Np, const bf16* __restrict__ x,
                                                       const bf16* __restrict__ Msb, const float* __restrict__ cs,
                                                       float* __restrict__ S) {
  const int pp = p * p, pw = W / p, N = (H / p) * pw;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, l32 = lane & 31, lhi = lane >> 5;
  const int c = blockIdx.y, b = blockIdx.z, k = c / g, cl = c % g;
  const int n0 = blockIdx.x * 128 + wave * 32;
  if (n0 >= N) return;
  const int n = min(n0 + l32, N - 1);
  const int pi = n / pw, pj = n % pw;
  const bf16* img = x + ((size_t)b * C + c) * H * W + (size_t)(pi * p) * W + pj * p;
  const bf16* mrow = Msb + ((size_t)c * heads + min(l32, heads - 1)) * pp;
  f32x16 acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;
  for (int kc = lhi; kc < pp / 8; kc += 2) {            // 8-pixel chunk of the patch
    bf16x8 a;
    if (p == 4) {
      const bf16x4 lo = *reinterpret_cast<const bf16x4*>(img + (size_t)(2 * kc) * W);
      const bf16x4 hi = *reinterpret_cast<const bf16x4*>(img + (size_t)(2 * kc + 1) * W);
#pragma unroll
      for (int e = 0; e < 4; ++e) { a[e] = lo[e]; a[4 + e] = hi[e]; }
    } else {
      const int r = (kc * 8) / p, s0 = (kc * 8) % p;
      a = *reinterpret_cast<const bf16x8*>(img + (size_t)r * W + s0);
    }
    bf16x8 m = *reinterpret_cast<const bf16x8*>(mrow + kc * 8);
    if (l32 >= heads) m = bf16x8{};
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, m, acc, 0, 0, 0);
  }
  if (l32 < heads) {
    const float add = cs[(size_t)c * heads + l32];
    float* dst = S + ((((size_t)b * G + k) * gpad + cl) * heads + l32) * Np + n0 + 4 * lhi;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      f32x4 v;
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = acc[4 * q + e] + add;
      *reinterpret_cast<f32x4*>(dst + 8 * q) = v;
    }
  }
}

// The same scores with the softmax over the group in the same kernel, for groups whose scores of 32 patches fit LDS
// (size of the group x heads x 33 floats): grid (ceil(N/32), G, B), block 256.  The wavefronts take the group's
// channels in turn (the products of k_scores_pixels) and leave the scores in LDS as [member][head][patch, pitch 33];
// then every (head, patch) is normalised over the members in the order and with the arithmetic of k_softmax_alpha,
// and the weights are written in the layout of the forward kernels (alpha_f[b][k][cl][head][n], zeros for padding
// members and the pitch) and / or token-major (alpha_tm[b,c,n,head]), whichever pointer is given.
// PP: pixels per patch when known at compile time (16 or 64: a channel's operand loads are then issued together, and
// those of the wavefront's next channel while the current one is multiplied), 0 for any other patch size.
template <int PP>
__global__ __launch_bounds__(256) void k_scores_pixels_softmax(int C, int H, int W, int p, int heads, int g, int gpad,
                                                               int G, int Np, const bf16* __restrict__ x,
                                                               const bf16* __restrict__ Msb,
                                                               const float* __restrict__ cs,
                                                               float* __restrict__ alpha_f,
                                                               float* __restrict__ alpha_tm) {
  extern __shared__ __attribute__((aligned(16))) float sc[];       // [gk][heads][33]
  const int pp = PP ? PP : p * p, pw = W / p, N = (H / p) * pw;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, l32 = lane & 31, lhi = lane >> 5;
  const int k = blockIdx.y, b = blockIdx.z;
  const int c0 = k * g, gk = min(g, C - c0);
  const int n0 = blockIdx.x * 32;
  const int n = min(n0 + l32, N - 1);
  const int pi = n / pw, pj = n % pw;
  const size_t img_off = (size_t)(pi * p) * W + pj * p;
  // one 8-pixel chunk of this lane's patch of channel c, and the matching chunk of the composed score weights
  auto load_a = [&](int c, int kc) -> bf16x8 {
    const bf16* img = x + ((size_t)b * C + c) * H * W + img_off;
    bf16x8 a;
    if (p == 4) {
      const bf16x4 lo = *reinterpret_cast<const bf16x4*>(img + (size_t)(2 * kc) * W);
      const bf16x4 hi = *reinterpret_cast<const bf16x4*>(img + (size_t)(2 * kc + 1) * W);
#pragma unroll
      for (int e = 0; e < 4; ++e) { a[e] = lo[e]; a[4 + e] = hi[e]; }
    } else {
      const int r = (kc * 8) / p, s0 = (kc * 8) % p;
      a = *reinterpret_cast<const bf16x8*>(img + (size_t)r * W + s0);
    }
    return a;
  };
  auto load_m = [&](int c, int kc) -> bf16x8 {
    bf16x8 m = *reinterpret_cast<const bf16x8*>(Msb + ((size_t)c * heads + min(l32, heads - 1)) * pp + kc * 8);
    if (l32 >= heads) m = bf16x8{};
    return m;
  };
  auto leave = [&](int cl, const f32x16& acc) {          // lane: head l32, patches 8 (r / 4) + 4 lhi + r % 4
    if (l32 < heads) {
      const float add = cs[(size_t)(c0 + cl) * heads + l32];
      float* dst = sc + ((size_t)cl * heads + l32) * 33 + 4 * lhi;
#pragma unroll
      for (int r = 0; r < 16; ++r) dst[8 * (r >> 2) + (r & 3)] = acc[r] + add;
    }
  };
  if constexpr (PP > 0) {
    constexpr int NIT = PP / 16;                         // chunks per lane half
    bf16x8 a0[NIT], m0[NIT], a1[NIT], m1[NIT];
    auto fetch = [&](int cl, bf16x8 (&a)[NIT], bf16x8 (&m)[NIT]) {
#pragma unroll
      for (int t = 0; t < NIT; ++t) {
        a[t] = load_a(c0 + cl, lhi + 2 * t);
        m[t] = load_m(c0 + cl, lhi + 2 * t);
      }
    };
    auto product = [&](int cl, const bf16x8 (&a)[NIT], const bf16x8 (&m)[NIT]) {
      f32x16 acc;
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
      for (int t = 0; t < NIT; ++t) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[t], m[t], acc, 0, 0, 0);
      leave(cl, acc);
    };
    int cl = wave;
    if (cl < gk) fetch(cl, a0, m0);
    while (cl < gk) {
      if (cl + 4 < gk) fetch(cl + 4, a1, m1);
      product(cl, a0, m0);
      cl += 4;
      if (cl >= gk) break;
      if (cl + 4 < gk) fetch(cl + 4, a0, m0);
      product(cl, a1, m1);
      cl += 4;
    }
  } else {
    for (int cl = wave; cl < gk; cl += 4) {
      f32x16 acc;
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[r] = 0.f;
      for (int kc = lhi; kc < pp / 8; kc += 2)           // 8-pixel chunk of the patch
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(load_a(c0 + cl, kc), load_m(c0 + cl, kc), acc, 0, 0, 0);
      leave(cl, acc);
    }
  }
  __syncthreads();
  for (int pr = threadIdx.x; pr < heads * 32; pr += 256) {         // (head, patch), patch fastest
    float* col = sc + (size_t)(pr >> 5) * 33 + (pr & 31);
    const int stride = heads * 33;
    float mx = -INFINITY;
    for (int cl = 0; cl < gk; ++cl) mx = fmaxf(mx, col[cl * stride]);
    float den = 0.f;
    for (int cl = 0; cl < gk; ++cl) den += __expf(col[cl * stride] - mx);
    const float inv = 1.f / den;
    for (int cl = 0; cl < gk; ++cl) col[cl * stride] = __expf(col[cl * stride] - mx) * inv;
  }
  __syncthreads();
  if (alpha_f) {
    for (int idx = threadIdx.x; idx < gpad * heads * 8; idx += 256) {       // four patches per thread: 16-byte stores
      const int quad = idx & 7, head = (idx >> 3) % heads, cl = (idx >> 3) / heads;
      f32x4 v;
#pragma unroll
      for (int e = 0; e < 4; ++e)
        v[e] = (cl < gk && n0 + 4 * quad + e < N) ? sc[((size_t)cl * heads + head) * 33 + 4 * quad + e] : 0.f;
      *reinterpret_cast<f32x4*>(alpha_f + ((((size_t)b * G + k) * gpad + cl) * heads + head) * Np + n0 + 4 * quad) = v;
    }
  }
  if (alpha_tm) {
    const int hq = heads / 4;                            // heads % 4 == 0: four heads per thread, 16-byte stores
    for (int idx = threadIdx.x; idx < gk * 32 * hq; idx += 256) {
      const int h4 = idx % hq, patch = (idx / hq) & 31, cl = idx / (hq * 32);
      if (n0 + patch < N) {
        f32x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = sc[((size_t)cl * heads + 4 * h4 + e) * 33 + patch];
        *reinterpret_cast<f32x4*>(alpha_tm + (((size_t)b * C + c0 + cl) * N + n0 + patch) * heads + 4 * h4) = v;
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Tokenizer on MFMA (paper Section 2.1: every patch of every channel is embedded on its own by
// that channel's convolution, kernel = stride = patch):
//   tokens[b,c,n,d] = sum_k u[b,c,n][k] * We[c][d][k] + be[c][d] + ce[c][d],   k = p*p pixels of the patch
// grid (ceil(N/128), C, B), block 256.  The block gathers its 128 patches into LDS (rows of p*p bf16,
// padded by 16 bytes), then every wavefront sweeps 64-column slices: 4 x 2 MFMA blocks whose two
// column blocks interleave (block j holds columns 2*lane+j), so that a lane owns two adjacent
// outputs per row and half a wavefront stores 128 contiguous bytes.
// Requires p*p % 16 == 0, p*p <= 256, D % 64 == 0.  The kernel is HBM-write bound.
// ---------------------------------------------------------------------------------------------
// KSS = p*p / 16 when that is 1, 2 or 4 (the weight fragments of the next column slice are then fetched while
// the current slice is multiplied and stored), 0 for any other patch size (fragments fetched step by step).
template <int KSS>
__global__ __launch_bounds__(256, 2) void k_tokenize_mfma(int C, int H, int W, int p, int D, const bf16* __restrict__ x,
                                                       const bf16* __restrict__ We, const bf16* __restrict__ be,
                                                       const bf16* __restrict__ ce, bf16* __restrict__ tokens) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
  const int pp = p * p, pw = W / p, N = (H / p) * pw;
  const int KS = KSS ? KSS : pp / 16;
  const int rbp = pp * 2 + 16;                           // padded bytes per patch row
  const int n0 = blockIdx.x * 128, c = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, lhi = lane >> 5;
  const bf16* img = x + ((size_t)b * C + c) * H * W;

  // gather: 4 pixels (8 bytes) at a time; p % 4 == 0 keeps every piece inside one patch row
  const int pieces = pp / 4;
  for (int idx = tid; idx < 128 * pieces; idx += 256) {
    const int t = idx / pieces, q = idx % pieces;
    const int r = (q * 4) / p, s0 = (q * 4) % p;
    const int n = n0 + t;
    bf16x4 v = {};
    if (n < N) {
      const int pi = n / pw, pj = n % pw;
      v = *reinterpret_cast<const bf16x4*>(img + (size_t)(pi * p + r) * W + pj * p + s0);
    }
    *reinterpret_cast<bf16x4*>(smem + t * rbp + q * 8) = v;
  }
  __syncthreads();

  const bf16* Wc = We + (size_t)c * D * pp;
  // uniform tile base + per-lane byte offset (the two half-wavefronts sit 4 rows apart); a tile spans at most
  // 128 rows of 2 D bytes, so 32-bit offsets do
  typedef __attribute__((address_space(1))) unsigned char gbyte_t;
  typedef __attribute__((address_space(1))) bf16x2 gbf16x2_t;
  gbyte_t* tbase = (gbyte_t*)(tokens + (((size_t)b * C + c) * N + n0) * D);
  const unsigned rowb = (unsigned)D * 2;
  const int nlim = N - n0 - 4 * lhi;                     // rows of this lane's half that are inside the image
  const bool full = n0 + 128 <= N;                       // uniform: no row of the tile is outside

  constexpr int NF = KSS ? KSS : 1;
  bf16x8 bfrag[NF][2];                                   // weight fragments of the slice about to be multiplied
  if (KSS) {
    // a wavefront whose first slice lies past D (D < 256) never enters the loop below: it preloads slice 0 instead,
    // so that no read leaves We
    const int colp = wave * 64 < D ? wave * 64 : 0;
    const bf16* wrow = Wc + (size_t)(colp + 2 * l32) * pp + lhi * 8;
#pragma unroll
    for (int kk = 0; kk < NF; ++kk)
#pragma unroll
      for (int j = 0; j < 2; ++j) bfrag[kk][j] = *reinterpret_cast<const bf16x8*>(wrow + (size_t)j * pp + kk * 16);
  }
  const unsigned rowb5 = 5 * rowb;
  for (int col0 = wave * 64; col0 < D; col0 += 256) {
    f32x16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    const int d0 = col0 + 2 * l32;
    if (KSS) {
#pragma unroll
      for (int kk = 0; kk < NF; ++kk) {
        bf16x8 af[4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
          af[i] = *reinterpret_cast<const bf16x8*>(smem + (i * 32 + l32) * rbp + (kk * 2 + lhi) * 16);
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfrag[kk][j], acc[i][j], 0, 0, 0);
      }
      // fetch the slice after this one while this one is stored (the last slice fetches itself again:
      // in bounds, unused)
      const int coln = col0 + 256 < D ? col0 + 256 : col0;
      const bf16* wrow = Wc + (size_t)(coln + 2 * l32) * pp + lhi * 8;
#pragma unroll
      for (int kk = 0; kk < NF; ++kk)
#pragma unroll
        for (int j = 0; j < 2; ++j) bfrag[kk][j] = *reinterpret_cast<const bf16x8*>(wrow + (size_t)j * pp + kk * 16);
    } else {
      const bf16* wrow = Wc + (size_t)d0 * pp + lhi * 8;
      for (int kk = 0; kk < KS; ++kk) {
        bf16x8 bfr[2], af[4];
#pragma unroll
        for (int j = 0; j < 2; ++j) bfr[j] = *reinterpret_cast<const bf16x8*>(wrow + (size_t)j * pp + kk * 16);
#pragma unroll
        for (int i = 0; i < 4; ++i)
          af[i] = *reinterpret_cast<const bf16x8*>(smem + (i * 32 + l32) * rbp + (kk * 2 + lhi) * 16);
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
      }
    }
    float add0 = 0.f, add1 = 0.f;
    if (be) { add0 += (float)be[(size_t)c * D + d0]; add1 += (float)be[(size_t)c * D + d0 + 1]; }
    if (ce) { add0 += (float)ce[(size_t)c * D + d0]; add1 += (float)ce[(size_t)c * D + d0 + 1]; }
    // rows of a lane in register order: 0 1 2 3 8 9 10 11 16 ... (steps of 1, 1, 1, 5 rows).  The row pointer
    // is uniform and walks in scalar registers; the asm keeps the compiler from precomputing all 64 of them
    // outside the slice loop (which costs more registers than there are).
    const unsigned lane_off = (unsigned)(4 * lhi * D + d0) * 2;
    gbyte_t* rowp = tbase;
    asm volatile("" : "+s"(rowp));
    if (full) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          bf16x2 pk;
          pk[0] = (bf16)(acc[i][0][r] + add0);
          pk[1] = (bf16)(acc[i][1][r] + add1);
          *(gbf16x2_t*)(rowp + lane_off) = pk;
          rowp += (r & 3) == 3 ? rowb5 : rowb;
        }
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int rr = i * 32 + 8 * (r >> 2) + (r & 3);  // uniform row index inside the tile
          if (rr < nlim) {
            bf16x2 pk;
            pk[0] = (bf16)(acc[i][0][r] + add0);
            pk[1] = (bf16)(acc[i][1][r] + add1);
            *(gbf16x2_t*)(rowp + lane_off) = pk;
          }
          rowp += (r & 3) == 3 ? rowb5 : rowb;
        }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Tokenizer on MFMA, weight-stationary form for p*p = 16 * KSS, KSS in {1, 2, 4}, D % 256 == 0 (same result
// as k_tokenize_mfma).  grid (D / 256, C, TS), block 256: wavefront w of block (x, c, z) owns the 64 columns
// 256 x + 64 w .. + 63 of channel c, loads their weight fragments ONCE and then walks the 128-patch tiles
// [z * per, (z + 1) * per) of the B * ceil(N / 128) tiles of its channel.  The patches of the next tile are
// fetched into registers while the current tile is multiplied and stored, and handed over through one of two
// LDS buffers (one barrier per tile).  Dynamic LDS: 2 * 128 * (p*p*2 + 16) bytes.  HBM-write bound.
// ---------------------------------------------------------------------------------------------
template <int KSS>
__global__ __launch_bounds__(256, 2) void k_tokenize_ws(int B, int C, int H, int W, int p, int D, int per,
                                                        const bf16* __restrict__ x, const bf16* __restrict__ We,
                                                        const bf16* __restrict__ be, const bf16* __restrict__ ce,
                                                        bf16* __restrict__ tokens) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
  typedef __attribute__((address_space(1))) unsigned char gbyte_t;
  typedef __attribute__((address_space(1))) bf16x2 gbf16x2_t;
  constexpr int pp = 16 * KSS, pieces = pp / 4;          // 8-byte pieces per patch
  constexpr int rbp = pp * 2 + 16;                       // padded bytes per patch row
  constexpr int NG = 128 * pieces / 256;                 // pieces a thread gathers per tile
  const int pw = W / p, N = (H / p) * pw;
  const int ntile = (N + 127) / 128, T = B * ntile;
  const int c = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, lhi = lane >> 5;
  const int d0 = blockIdx.x * 256 + wave * 64 + 2 * l32;   // this lane's two adjacent columns
  const int t_begin = blockIdx.z * per, t_end = min(T, t_begin + per);
  if (t_begin >= t_end) return;                          // uniform over the block

  bf16x8 bfrag[KSS][2];
  {
    const bf16* wrow = We + ((size_t)c * D + d0) * pp + lhi * 8;
#pragma unroll
    for (int kk = 0; kk < KSS; ++kk)
#pragma unroll
      for (int j = 0; j < 2; ++j) bfrag[kk][j] = *reinterpret_cast<const bf16x8*>(wrow + (size_t)j * pp + kk * 16);
  }
  float add0 = 0.f, add1 = 0.f;
  if (be) { add0 += (float)be[(size_t)c * D + d0]; add1 += (float)be[(size_t)c * D + d0 + 1]; }
  if (ce) { add0 += (float)ce[(size_t)c * D + d0]; add1 += (float)ce[(size_t)c * D + d0 + 1]; }

  // gather of tile t: piece idx = tid + 256 * i covers patch idx / pieces, pixels 4 * (idx % pieces) .. + 3
  bf16x4 gv[NG];
  auto fetch = [&](int t) {
    const int b = t / ntile, n0 = (t % ntile) * 128;
    const bf16* img = x + ((size_t)b * C + c) * H * W;
#pragma unroll
    for (int i = 0; i < NG; ++i) {
      const int idx = tid + 256 * i;
      const int tp = idx / pieces, q = idx % pieces;
      const int r = (q * 4) / p, s0 = (q * 4) % p;
      const int n = n0 + tp;
      gv[i] = bf16x4{};
      if (n < N) {
        const int pi = n / pw, pj = n % pw;
        gv[i] = *reinterpret_cast<const bf16x4*>(img + (size_t)(pi * p + r) * W + pj * p + s0);
      }
    }
  };
  auto stash = [&](int buf) {
    unsigned char* u = smem + buf * 128 * rbp;
#pragma unroll
    for (int i = 0; i < NG; ++i) {
      const int idx = tid + 256 * i;
      *reinterpret_cast<bf16x4*>(u + (idx / pieces) * rbp + (idx % pieces) * 8) = gv[i];
    }
  };
  fetch(t_begin);
  stash(0);
  __syncthreads();

  const unsigned rowb = (unsigned)D * 2, rowb5 = 5 * rowb;
  const unsigned lane_off = (unsigned)(4 * lhi * D + d0) * 2;
  for (int t = t_begin; t < t_end; ++t) {
    const int cur = (t - t_begin) & 1;
    if (t + 1 < t_end) fetch(t + 1);
    const unsigned char* u = smem + cur * 128 * rbp;
    f32x16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
#pragma unroll
    for (int kk = 0; kk < KSS; ++kk) {
      bf16x8 af[4];
#pragma unroll
      for (int i = 0; i < 4; ++i)
        af[i] = *reinterpret_cast<const bf16x8*>(u + (i * 32 + l32) * rbp + (kk * 2 + lhi) * 16);
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfrag[kk][j], acc[i][j], 0, 0, 0);
    }
    // rows of a lane in register order: 0 1 2 3 8 9 10 11 16 ... (steps of 1, 1, 1, 5 rows); the row pointer
    // is uniform and walks in scalar registers (the asm keeps it from being expanded into 64 precomputed ones)
    const int b = t / ntile, n0 = (t % ntile) * 128;
    gbyte_t* rowp = (gbyte_t*)(tokens + (((size_t)b * C + c) * N + n0) * D);
    asm volatile("" : "+s"(rowp));
    if (n0 + 128 <= N) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          bf16x2 pk;
          pk[0] = (bf16)(acc[i][0][r] + add0);
          pk[1] = (bf16)(acc[i][1][r] + add1);
          *(gbf16x2_t*)(rowp + lane_off) = pk;
          rowp += (r & 3) == 3 ? rowb5 : rowb;
        }
    } else {
      const int nlim = N - n0 - 4 * lhi;                 // rows of this lane's half that are inside the image
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int rr = i * 32 + 8 * (r >> 2) + (r & 3);
          if (rr < nlim) {
            bf16x2 pk;
            pk[0] = (bf16)(acc[i][0][r] + add0);
            pk[1] = (bf16)(acc[i][1][r] + add1);
            *(gbf16x2_t*)(rowp + lane_off) = pk;
          }
          rowp += (r & 3) == 3 ? rowb5 : rowb;
        }
    }
    if (t + 1 < t_end) stash(cur ^ 1);
    __syncthreads();
  }
}

// ---------------------------------------------------------------------------------------------
// Tokenizer fused with a linear first level (D-CHAG-L: paper Section 2.1 tokenization, Sections 3.2/3.3
// linear partial aggregation): the tokens of a group are mixed as they are produced and never reach HBM,
//   y[b,k,n,d] = sum_{cl < gk} w[k][cl][d] * (We[c] u[b,c,n] + be[c] + ce[c])[d] + bias[k][d],   c = k*g + cl.
// grid (ceil(N/64) * (D/256), G, B), block 256: 64 patches x 256 columns x all members of one group.
// Wavefront w owns columns 64 w .. 64 w + 63 of the block's slice as 2 x 2 MFMA blocks (the two column
// blocks interleave as in k_tokenize_mfma).  Members are pipelined: while member cl is multiplied, scaled by
// its weight of the lane's column and added up in registers, the 64 patches and the weight fragments of member
// cl + 1 are already on their way (patches through registers into the other of two LDS buffers, one barrier
// per member).  p*p = 16 * KSS, KSS in {1, 4}; D % 256 == 0.  Dynamic LDS: 2 * 64 * (p*p*2 + 16) bytes.
// ---------------------------------------------------------------------------------------------
template <int KSS>
__global__ __launch_bounds__(256, 2) void k_tokenize_mix_mfma(int C, int H, int W, int p, int D, int g,
                                                              const bf16* __restrict__ x, const bf16* __restrict__ We,
                                                              const bf16* __restrict__ be, const bf16* __restrict__ ce,
                                                              const bf16* __restrict__ wmix,
                                                              const bf16* __restrict__ bias, bf16* __restrict__ y) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
  constexpr int pp = 16 * KSS, pieces = pp / 4;
  constexpr int rbp = pp * 2 + 16;
  constexpr int NG = (64 * pieces + 255) / 256;          // 8-byte pieces a thread gathers per member
  const int pw = W / p, N = (H / p) * pw;
  const int ns_n = D / 256;
  const int n0 = (blockIdx.x / ns_n) * 64, col_base = (blockIdx.x % ns_n) * 256;
  const int k = blockIdx.y, b = blockIdx.z, G = gridDim.y;
  const int c0 = k * g, gk = min(g, C - c0);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, lhi = lane >> 5;
  const int d0 = col_base + wave * 64 + 2 * l32;         // this lane's two adjacent columns

  // what member cl needs: its patches (gv), its weight fragments (bfrag) and four per-column scalars
  bf16x4 gv[NG];
  bf16x8 bfrag[KSS][2];
  float w0, w1, a0, a1;
  // source offsets of this thread's pieces inside a channel image (-1: patch outside the image)
  int goff[NG];
#pragma unroll
  for (int i = 0; i < NG; ++i) {
    const int idx = tid + 256 * i;
    const int t = idx / pieces, q = idx % pieces;
    const int r = (q * 4) / p, s0 = (q * 4) % p;
    const int n = n0 + t;
    goff[i] = (idx < 64 * pieces && n < N) ? ((n / pw) * p + r) * W + (n % pw) * p + s0 : -1;
  }
  auto fetch = [&](int cl) {
    const int c = c0 + cl;
    const bf16* img = x + ((size_t)b * C + c) * H * W;
#pragma unroll
    for (int i = 0; i < NG; ++i) {
      gv[i] = bf16x4{};
      if (goff[i] >= 0) gv[i] = *reinterpret_cast<const bf16x4*>(img + goff[i]);
    }
    const bf16* wrow = We + ((size_t)c * D + d0) * pp + lhi * 8;
#pragma unroll
    for (int kk = 0; kk < KSS; ++kk)
#pragma unroll
      for (int j = 0; j < 2; ++j) bfrag[kk][j] = *reinterpret_cast<const bf16x8*>(wrow + (size_t)j * pp + kk * 16);
    w0 = (float)wmix[((size_t)k * g + cl) * D + d0];
    w1 = (float)wmix[((size_t)k * g + cl) * D + d0 + 1];
    a0 = 0.f;
    a1 = 0.f;
    if (be) { a0 += (float)be[(size_t)c * D + d0]; a1 += (float)be[(size_t)c * D + d0 + 1]; }
    if (ce) { a0 += (float)ce[(size_t)c * D + d0]; a1 += (float)ce[(size_t)c * D + d0 + 1]; }
  };
  auto stash = [&](int buf) {
    unsigned char* u = smem + buf * 64 * rbp;
#pragma unroll
    for (int i = 0; i < NG; ++i) {
      const int idx = tid + 256 * i;
      if (idx < 64 * pieces) *reinterpret_cast<bf16x4*>(u + (idx / pieces) * rbp + (idx % pieces) * 8) = gv[i];
    }
  };

  f32x16 o[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[i][j][r] = 0.f;
  float cst0 = 0.f, cst1 = 0.f;                          // patch-independent part: sum_c w * (be + ce) + bias

  fetch(0);
  stash(0);
  __syncthreads();
  for (int cl = 0; cl < gk; ++cl) {
    const unsigned char* u = smem + (cl & 1) * 64 * rbp;
    // this member's operands move to their own registers; the next member's loads start right away
    bf16x8 bcur[KSS][2];
#pragma unroll
    for (int kk = 0; kk < KSS; ++kk)
#pragma unroll
      for (int j = 0; j < 2; ++j) bcur[kk][j] = bfrag[kk][j];
    const float cw0 = w0, cw1 = w1;
    cst0 += w0 * a0;
    cst1 += w1 * a1;
    if (cl + 1 < gk) fetch(cl + 1);
    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      f32x16 acc0 = zero, acc1 = zero;                   // two independent chains: row block i, both column blocks
#pragma unroll
      for (int kk = 0; kk < KSS; ++kk) {
        const bf16x8 af = *reinterpret_cast<const bf16x8*>(u + (i * 32 + l32) * rbp + (kk * 2 + lhi) * 16);
        acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, bcur[kk][0], acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, bcur[kk][1], acc1, 0, 0, 0);
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        o[i][0][r] += cw0 * acc0[r];
        o[i][1][r] += cw1 * acc1[r];
      }
    }
    if (cl + 1 < gk) stash((cl + 1) & 1);
    __syncthreads();
  }
  if (bias) { cst0 += (float)bias[(size_t)k * D + d0]; cst1 += (float)bias[(size_t)k * D + d0 + 1]; }
  bf16* ybase = y + (((size_t)b * G + k) * N + n0) * D;
  const int lane_off = 4 * lhi * D + d0;
  const int nlim = N - n0 - 4 * lhi;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int rr = i * 32 + 8 * (r >> 2) + (r & 3);
      if (rr < nlim) {
        bf16x2 pk;
        pk[0] = (bf16)(o[i][0][r] + cst0);
        pk[1] = (bf16)(o[i][1][r] + cst1);
        *reinterpret_cast<bf16x2*>(ybase + (size_t)rr * D + lane_off) = pk;
      }
    }
}

// The same with 128 patches x 256 columns per workgroup of eight wavefronts (wavefront w: columns 32 w .. 32 w + 31,
// 4 row blocks): every workgroup re-reads the tokenizer weights of its members and gathers their pixels once per column
// slice, so the larger patch tile halves the weight traffic at the same pixel traffic.  grid (ceil(N/128) * (D/256), G, B),
// block 512.  Dynamic LDS: 2 * 128 * (p*p*2 + 16) bytes.
template <int KSS>
__global__ __launch_bounds__(512) void k_tokenize_mix_wide(int C, int H, int W, int p, int D, int g,
                                                              const bf16* __restrict__ x, const bf16* __restrict__ We,
                                                              const bf16* __restrict__ be, const bf16* __restrict__ ce,
                                                              const bf16* __restrict__ wmix,
                                                              const bf16* __restrict__ bias, bf16* __restrict__ y) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
  constexpr int pp = 16 * KSS, pieces = pp / 4;
  constexpr int rbp = pp * 2 + 16;
  constexpr int PB = 128;                                // patches per workgroup
  constexpr int NG = (PB * pieces + 511) / 512;          // 8-byte pieces a thread gathers per member
  const int pw = W / p, N = (H / p) * pw;
  const int ns_n = D / 256;
  const int n0 = (blockIdx.x / ns_n) * PB, col_base = (blockIdx.x % ns_n) * 256;
  const int k = blockIdx.y, b = blockIdx.z, G = gridDim.y;
  const int c0 = k * g, gk = min(g, C - c0);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, lhi = lane >> 5;
  const int d0 = col_base + wave * 32 + l32;             // this lane's column

  // what member cl needs: its patches (gv), its weight fragments (bfrag) and four per-column scalars
  bf16x4 gv[NG];
  bf16x8 bfrag[KSS];
  float w0, a0;
  // source offsets of this thread's pieces inside a channel image (-1: patch outside the image)
  int goff[NG];
#pragma unroll
  for (int i = 0; i < NG; ++i) {
    const int idx = tid + 512 * i;
    const int t = idx / pieces, q = idx % pieces;
    const int r = (q * 4) / p, s0 = (q * 4) % p;
    const int n = n0 + t;
    goff[i] = (idx < PB * pieces && n < N) ? ((n / pw) * p + r) * W + (n % pw) * p + s0 : -1;
  }
  auto fetch = [&](int cl) {
    const int c = c0 + cl;
    const bf16* img = x + ((size_t)b * C + c) * H * W;
#pragma unroll
    for (int i = 0; i < NG; ++i) {
      gv[i] = bf16x4{};
      if (goff[i] >= 0) gv[i] = *reinterpret_cast<const bf16x4*>(img + goff[i]);
    }
    const bf16* wrow = We + ((size_t)c * D + d0) * pp + lhi * 8;
#pragma unroll
    for (int kk = 0; kk < KSS; ++kk) bfrag[kk] = *reinterpret_cast<const bf16x8*>(wrow + kk * 16);
    w0 = (float)wmix[((size_t)k * g + cl) * D + d0];
    a0 = 0.f;
    if (be) a0 += (float)be[(size_t)c * D + d0];
    if (ce) a0 += (float)ce[(size_t)c * D + d0];
  };
  auto stash = [&](int buf) {
    unsigned char* u = smem + buf * PB * rbp;
#pragma unroll
    for (int i = 0; i < NG; ++i) {
      const int idx = tid + 512 * i;
      if (idx < PB * pieces) *reinterpret_cast<bf16x4*>(u + (idx / pieces) * rbp + (idx % pieces) * 8) = gv[i];
    }
  };

  f32x16 o[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[i][r] = 0.f;
  float cst0 = 0.f;                                      // patch-independent part: sum_c w * (be + ce) + bias

  fetch(0);
  stash(0);
  __syncthreads();
  for (int cl = 0; cl < gk; ++cl) {
    const unsigned char* u = smem + (cl & 1) * PB * rbp;
    // this member's operands move to their own registers; the next member's loads start right away
    bf16x8 bcur[KSS];
#pragma unroll
    for (int kk = 0; kk < KSS; ++kk) bcur[kk] = bfrag[kk];
    const float cw0 = w0;
    cst0 += w0 * a0;
    if (cl + 1 < gk) fetch(cl + 1);
    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < 4; i += 2) {
      f32x16 acc0 = zero, acc1 = zero;                   // two independent chains: row blocks i and i + 1
#pragma unroll
      for (int kk = 0; kk < KSS; ++kk) {
        const bf16x8 af0 = *reinterpret_cast<const bf16x8*>(u + (i * 32 + l32) * rbp + (kk * 2 + lhi) * 16);
        const bf16x8 af1 = *reinterpret_cast<const bf16x8*>(u + ((i + 1) * 32 + l32) * rbp + (kk * 2 + lhi) * 16);
        acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af0, bcur[kk], acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af1, bcur[kk], acc1, 0, 0, 0);
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        o[i][r] += cw0 * acc0[r];
        o[i + 1][r] += cw0 * acc1[r];
      }
    }
    if (cl + 1 < gk) stash((cl + 1) & 1);
    __syncthreads();
  }
  if (bias) cst0 += (float)bias[(size_t)k * D + d0];
  bf16* ybase = y + (((size_t)b * G + k) * N + n0) * D;
  const int lane_off = 4 * lhi * D + d0;
  const int nlim = N - n0 - 4 * lhi;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int rr = i * 32 + 8 * (r >> 2) + (r & 3);
      if (rr < nlim) ybase[(size_t)rr * D + lane_off] = (bf16)(o[i][r] + cst0);
    }
}

// The attention form of k_tokenize_mix_wide (cross-attention first level with the value projection folded into the
// tokenizer weights: Wf[c] = Wv[k] We[c], v1 = Wv be, v2 = Wv ce), for the shapes the ring kernel below does not take
// (16 pixels per patch, heads of 32 columns, unaligned images):
//   y[b,k,n,d] = sum_{cl < gk} alpha[b][k][cl][head(d)][n] * (Wf[c] u[b,c,n] + v1[c] + v2[c])[d] + bias[k][d].
// The member's constant enters as the MFMA's C operand; its softmax weights (NHS heads x 128 patches, fp32) travel with
// the patches through registers into LDS.  Requires (D / heads) % 32 == 0 and 256 % dh == 0 or dh % 256 == 0.
// Dynamic LDS: 2 * 128 * (p*p*2 + 16) + 2 * NHS * 512 bytes.
template <int KSS>
__global__ __launch_bounds__(512) void k_tokenize_attend_wide(int C, int H, int W, int p, int D, int g, int heads,
                                                              int gpad, int Np, const bf16* __restrict__ x,
                                                              const bf16* __restrict__ Wf, const bf16* __restrict__ v1,
                                                              const bf16* __restrict__ v2,
                                                              const float* __restrict__ alpha,
                                                              const bf16* __restrict__ bias, bf16* __restrict__ y) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int pp = 16 * KSS, pieces = pp / 4;
  constexpr int rbp = pp * 2 + 16;
  constexpr int PB = 128;                                // patches per workgroup
  constexpr int NG = (PB * pieces + 511) / 512;          // 8-byte pieces a thread gathers per member
  const int pw = W / p, N = (H / p) * pw;
  const int ns_n = D / 256;
  const int n0 = (blockIdx.x / ns_n) * PB, col_base = (blockIdx.x % ns_n) * 256;
  const int k = blockIdx.y, b = blockIdx.z, G = gridDim.y;
  const int c0 = k * g, gk = min(g, C - c0);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, lhi = lane >> 5;
  const int d0 = col_base + wave * 32 + l32;             // this lane's column
  const int dh = D / heads, nhs = dh >= 256 ? 1 : 256 / dh, h0 = col_base / dh;
  const int hrel = (col_base + wave * 32) / dh - h0;     // the wavefront's 32 columns lie in one head
  unsigned char* alds = smem + 2 * PB * rbp;             // [2][nhs][128] floats

  bf16x4 gv[NG];
  bf16x8 bfrag[KSS];
  f32x4 av = {0.f, 0.f, 0.f, 0.f};
  float a0;
  int goff[NG];
#pragma unroll
  for (int i = 0; i < NG; ++i) {
    const int idx = tid + 512 * i;
    const int t = idx / pieces, q = idx % pieces;
    const int r = (q * 4) / p, s0 = (q * 4) % p;
    const int n = n0 + t;
    goff[i] = (idx < PB * pieces && n < N) ? ((n / pw) * p + r) * W + (n % pw) * p + s0 : -1;
  }
  // thread t < 32 nhs fetches the weights of head h0 + t / 32 for patches n0 + 4 (t % 32) .. + 3
  const float* asrc = alpha + ((((size_t)b * G + k) * gpad) * heads + h0 + min(tid >> 5, nhs - 1)) * Np +
                      min(n0 + 4 * (tid & 31), Np - 4);
  auto fetch = [&](int cl) {
    const int c = c0 + cl;
    const bf16* img = x + ((size_t)b * C + c) * H * W;
#pragma unroll
    for (int i = 0; i < NG; ++i) {
      gv[i] = bf16x4{};
      if (goff[i] >= 0) gv[i] = *reinterpret_cast<const bf16x4*>(img + goff[i]);
    }
    const bf16* wrow = Wf + ((size_t)c * D + d0) * pp + lhi * 8;
#pragma unroll
    for (int kk = 0; kk < KSS; ++kk) bfrag[kk] = *reinterpret_cast<const bf16x8*>(wrow + kk * 16);
    a0 = 0.f;
    if (v1) a0 += (float)v1[(size_t)c * D + d0];
    if (v2) a0 += (float)v2[(size_t)c * D + d0];
    if (tid < 32 * nhs) av = *reinterpret_cast<const f32x4*>(asrc + (size_t)cl * heads * Np);
  };
  auto stash = [&](int buf) {
    unsigned char* u = smem + buf * PB * rbp;
#pragma unroll
    for (int i = 0; i < NG; ++i) {
      const int idx = tid + 512 * i;
      if (idx < PB * pieces) *reinterpret_cast<bf16x4*>(u + (idx / pieces) * rbp + (idx % pieces) * 8) = gv[i];
    }
    if (tid < 32 * nhs) *reinterpret_cast<f32x4*>(alds + buf * nhs * 512 + tid * 16) = av;
  };

  f32x16 o[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[i][r] = 0.f;

  fetch(0);
  stash(0);
  __syncthreads();
  for (int cl = 0; cl < gk; ++cl) {
    const unsigned char* u = smem + (cl & 1) * PB * rbp;
    const float* al = reinterpret_cast<const float*>(alds + (cl & 1) * nhs * 512 + hrel * 512) + 4 * lhi;
    bf16x8 bcur[KSS];
#pragma unroll
    for (int kk = 0; kk < KSS; ++kk) bcur[kk] = bfrag[kk];
    const float cb = a0;
    if (cl + 1 < gk) fetch(cl + 1);
    const f32x16 init = {cb, cb, cb, cb, cb, cb, cb, cb, cb, cb, cb, cb, cb, cb, cb, cb};
#pragma unroll
    for (int i = 0; i < 4; i += 2) {
      f32x16 acc0 = init, acc1 = init;                   // two independent chains: row blocks i and i + 1
#pragma unroll
      for (int kk = 0; kk < KSS; ++kk) {
        const bf16x8 af0 = *reinterpret_cast<const bf16x8*>(u + (i * 32 + l32) * rbp + (kk * 2 + lhi) * 16);
        const bf16x8 af1 = *reinterpret_cast<const bf16x8*>(u + ((i + 1) * 32 + l32) * rbp + (kk * 2 + lhi) * 16);
        acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af0, bcur[kk], acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af1, bcur[kk], acc1, 0, 0, 0);
      }
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const f32x4 w0 = *reinterpret_cast<const f32x4*>(al + i * 32 + 8 * q);
        const f32x4 w1 = *reinterpret_cast<const f32x4*>(al + (i + 1) * 32 + 8 * q);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          o[i][4 * q + e] += w0[e] * acc0[4 * q + e];
          o[i + 1][4 * q + e] += w1[e] * acc1[4 * q + e];
        }
      }
    }
    if (cl + 1 < gk) stash((cl + 1) & 1);
    __syncthreads();
  }
  const float add = bias ? (float)bias[(size_t)k * D + d0] : 0.f;
  bf16* ybase = y + (((size_t)b * G + k) * N + n0) * D;
  const int lane_off = 4 * lhi * D + d0;
  const int nlim = N - n0 - 4 * lhi;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int rr = i * 32 + 8 * (r >> 2) + (r & 3);
      if (rr < nlim) ybase[(size_t)rr * D + lane_off] = (bf16)(o[i][r] + add);
    }
}

// ---------------------------------------------------------------------------------------------
// Tokenizer fused with the first aggregation level, operands streamed through a three-stage LDS ring
// (8 x 8 patches only: a patch and a weight row are both one 128-byte LDS row).  Two forms:
//   ATT = false (D-CHAG-L, paper Sections 3.2/3.3: linear partial aggregation)
//     y[b,k,n,d] = sum_cl wmix[k][cl][d] * (Wt[c] u[b,c,n] + v1[c] + v2[c])[d] + bias[k][d]
//   ATT = true (cross-attention level, paper Section 2.1, with the value projection folded into the tokenizer
//     weights: Wt[c] = Wv[k] We[c], v1 = Wv be, v2 = Wv ce; exact because the softmax weights sum to one)
//     y[b,k,n,d] = sum_cl alpha[b][k][cl][head(d)][n] * (Wt[c] u[b,c,n] + v1[c] + v2[c])[d] + bias[k][d]
// c = k*g + cl; u = the 64 pixels of patch n; alpha laid out [B][G][gpad][heads][Np] (fp32).
// Workgroup = 128 patches x 256 columns x all members of one group; wavefront (wm, wn) of 2 x 4 owns 64 patches x
// 64 columns as 2 x 2 MFMA blocks.  One ring stage = one member: its 128 patches (16 KiB, gathered from the image
// 16 bytes per lane), its 256 weight rows (32 KiB) and 4 KiB of per-member vectors (per-column scalars, softmax
// weights of the slice's heads), all by direct-to-LDS loads issued two members ahead; one barrier per member.
// Workgroups are dealt to the XCDs in contiguous ranges of the (k, b, patch tile, column slice) order, so the
// workgroups that share a member's weights or a patch tile meet in one L2.
// With S > 1 the members of a group are dealt to S workgroups per tile (few groups: not enough tiles to fill the
// chip otherwise); each writes its fp32 partial sums to ypart [S][B][G][N][D] and k_vagg_merge adds them and the bias.
// Requires D % 256 == 0, W % 8 == 0, 16-byte aligned x; ATT: (D / heads) % 64 == 0 and 256 % dh == 0 or dh % 256 == 0.
// Dynamic LDS: kRedLdsBytes.
// ---------------------------------------------------------------------------------------------
// Workgroup shapes of k_tokenize_reduce_ring.  CFG 0: 128 patches x 256 columns, 8 wavefronts (2 x 4) of 64 x 64, three
// stages, one workgroup per compute unit.  CFG 1: 128 x 128, 4 wavefronts (2 x 2) of 64 x 64, two stages, two workgroups
// per compute unit (the one taken: 0.107 against 0.114 ms at the headline shape; 64 x 128 with wavefronts of 64 x 32,
// three workgroups per compute unit, was slower than both: 0.127 ms).
// Timing probes of k_tokenize_reduce_ring's three-stage form (compile-time; 0 in the product build; results
// meaningless, every access in bounds, every loop keeps its trip count): bit 1 = a member costs only its waits, its
// barrier and its loads (no fragment reads, products or scaling), 2 = no global -> LDS loads.
#ifndef DCHAG_RING_PROBE
#define DCHAG_RING_PROBE 0
#endif

template <int CFG>
struct RedCfg {
  static constexpr int kPatches = 128;
  static constexpr int WM = kPatches / 64, WN = CFG == 1 ? 2 : 4, TN = 2;
  static constexpr int kWaves = WM * WN, kThreads = kWaves * 64, kCols = WN * TN * 32;
  static constexpr int kABytes = kPatches * 128, kBBytes = kCols * 128, kXBytes = 4096;
  static constexpr int kStageBytes = kABytes + kBBytes + kXBytes;           // 52 or 36 KiB
  static constexpr int kStages = CFG == 0 ? 3 : 2;
  static constexpr int kPerCu = CFG + 1;                                    // workgroups per compute unit
  static constexpr int kLdsBytes = kStages * kStageBytes;                   // 156 or 72 KiB
};

template <bool ATT, int CFG>
__global__ __launch_bounds__(RedCfg<CFG>::kThreads, RedCfg<CFG>::kPerCu) void k_tokenize_reduce_ring(
    int C, int H, int W, int D, int g, int G, int heads, int gpad, int Np, TileWork tw, const bf16* __restrict__ x,
    const bf16* __restrict__ Wt, const bf16* __restrict__ wmix, const bf16* __restrict__ v1,
    const bf16* __restrict__ v2, const float* __restrict__ alpha, const bf16* __restrict__ bias, bf16* __restrict__ y,
    int S, float* __restrict__ ypart) {
  typedef RedCfg<CFG> Cfg;
  constexpr int WN = Cfg::WN, TN = Cfg::TN, kRedPatches = Cfg::kPatches;
  constexpr int kRedCols = Cfg::kCols, kRedABytes = Cfg::kABytes, kRedBBytes = Cfg::kBBytes;
  constexpr int kRedStageBytes = Cfg::kStageBytes, NS = Cfg::kStages;
  constexpr int AL = kRedPatches / 8 / Cfg::kWaves;      // A loads per wavefront and member
  constexpr int BL = kRedCols / 8 / Cfg::kWaves;         // B loads per wavefront and member
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  int k, b, pt, cs, split;
  {
    // position w of the (k, b, patch tile, column slice, split) order; each XCD takes a contiguous range of it
    const int total = tw.total * S, per = (total + kXcds - 1) / kXcds;
    const int w = (blockIdx.x % kXcds) * per + blockIdx.x / kXcds;
    if ((int)(blockIdx.x / kXcds) >= per || w >= total) return;   // uniform: the whole workgroup leaves
    split = w % S;
    tw.decode_linear(w / S, k, b, pt, cs);
  }
  const int pw = W / 8, N = (H / 8) * pw;
  const size_t HW = (size_t)H * W;
  const int n0 = pt * kRedPatches, col_base = cs * kRedCols;
  // this workgroup's members of the group: the S workgroups of a tile share them out evenly
  const int gfull = min(g, C - k * g);
  const int m_lo = split * gfull / S, gk = (split + 1) * gfull / S - m_lo;
  const int c0 = k * g + m_lo;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wave / WN, wn = wave % WN, l32 = lane & 31, lhi = lane >> 5;
  const int wcol = wn * TN * 32;                         // first column of this wavefront inside the slice
  const int dh = D / heads;

  // ---- issue side: per-lane sources of this wavefront's loads of one member ----
  const bf16* a_src[AL];
  const bf16* b_src[BL];
#pragma unroll
  for (int i = 0; i < AL; ++i) {
    const int row = wave * (AL * 8) + i * 8 + (lane >> 3);
    const int n = min(n0 + row, N - 1);                  // rows past the image repeat its last patch; never stored
    const int q = (lane & 7) ^ swz_chunk(row);           // logical chunk = pixel row of the patch
    a_src[i] = x + ((size_t)b * C + c0) * HW + (size_t)((n / pw) * 8 + q) * W + (n % pw) * 8;
  }
#pragma unroll
  for (int i = 0; i < BL; ++i) {
    const int row = wave * (BL * 8) + i * 8 + (lane >> 3);
    const int q = (lane & 7) ^ swz_chunk(row);
    b_src[i] = Wt + ((size_t)c0 * D + col_base + row) * 64 + q * 8;
  }
  // The stage's vectors: four per-column vectors of kCols bf16 each (ATT: v1, v2, -, -; else wmix, v1, v2, -) in the
  // first half, filled by the first wavefront(s), 64 / (kCols / 8) vectors per load; in the second half the softmax
  // weights of the slice's heads (kPatches floats each), 64 / (kPatches / 4) heads per load of the next wavefront(s).
  constexpr int LPV = kRedCols / 8, VPI = 64 / LPV, NVW = 4 / VPI;
  constexpr int AOFF = Cfg::kXBytes / 2, LPH = kRedPatches / 4, HPI = 64 / LPH, HB = kRedPatches * 4;
  constexpr int NAW = (kRedCols / 64 + HPI - 1) / HPI;   // heads are at least 64 columns wide
  const unsigned char* e_src = reinterpret_cast<const unsigned char*>(Wt);   // absent vector: any valid 16 bytes
  size_t e_step = 0;
  bool extra = false;
  int e_slot = 0;
  if (wave < NVW && (!ATT || wave == 0)) {
    extra = true;
    e_slot = wave * 1024;
    const int vi = wave * VPI + lane / LPV, lv = lane % LPV;
    const bf16* v = ATT ? (vi == 0 ? v1 : (vi == 1 ? v2 : nullptr)) : (vi == 0 ? wmix : (vi == 1 ? v1 : (vi == 2 ? v2 : nullptr)));
    if (v) {
      const size_t row0 = (!ATT && vi == 0) ? (size_t)k * g + m_lo : (size_t)c0;
      e_src = reinterpret_cast<const unsigned char*>(v + row0 * D + col_base + 8 * lv);
      e_step = (size_t)D * 2;
    }
  } else if (ATT && wave >= NVW && wave < NVW + NAW) {
    extra = true;
    e_slot = AOFF + (wave - NVW) * 1024;
    const int nhs = dh >= kRedCols ? 1 : kRedCols / dh;
    const int head = col_base / dh + min(HPI * (wave - NVW) + lane / LPH, nhs - 1);
    e_src = reinterpret_cast<const unsigned char*>(alpha + ((((size_t)b * G + k) * gpad + m_lo) * heads + head) * Np +
                                                   min(n0 + 4 * (lane % LPH), Np - 4));
    e_step = (size_t)heads * Np * 4;
  }
  extra = __builtin_amdgcn_readfirstlane(extra);
  e_slot = __builtin_amdgcn_readfirstlane(e_slot);
  const size_t b_step = (size_t)D * 64;
  auto issue = [&](int stage) {
    unsigned char* st = smem + stage * kRedStageBytes;
    if (DCHAG_RING_PROBE & 2) return;
#pragma unroll
    for (int i = 0; i < AL; ++i) {
      load16_to_lds(a_src[i], st + (wave * AL + i) * 1024);
      a_src[i] += HW;
    }
#pragma unroll
    for (int i = 0; i < BL; ++i) {
      load16_to_lds(b_src[i], st + kRedABytes + (wave * BL + i) * 1024);
      b_src[i] += b_step;
    }
    if (extra) {
      load16_to_lds(e_src, st + kRedABytes + kRedBBytes + e_slot);
      e_src += e_step;
    }
  };

  // ---- compute side ----
  const int a_base = (wm * 64 + l32) * 128, b_base = kRedABytes + (wcol + l32) * 128;
  int ck[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) ck[kk] = ((kk * 2 + lhi) ^ swz_chunk(l32)) * 16;
  const int xoff = kRedABytes + kRedBBytes;
  constexpr int VB = kRedCols * 2;                       // bytes of one per-column vector
  const int colj = (wcol + l32) * 2;                     // byte offset of this lane's first column in a vector
  const int hrel = ATT ? (col_base + wcol) / dh - col_base / dh : 0;

  const unsigned short mask1 = v1 ? 0xFFFF : 0, mask2 = v2 ? 0xFFFF : 0;
  f32x16 o[2][TN];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[i][j][r] = 0.f;
  float cst[TN];                                         // ATT = false: patch-independent part sum_c w * (v1 + v2)
#pragma unroll
  for (int j = 0; j < TN; ++j) cst[j] = 0.f;

  if constexpr (NS == 3) {
    // Three stages: the pipeline of k_vagg_mfma with a member in the place of a slice.  The barrier sits behind the
    // member's third k-step: by then every fragment of the member is in registers (its last k-step's, its softmax
    // weights / mixing weights too), so the barrier hands its stage to member m + 3 and the next member over to
    // everyone; the fragments of the next member's first k-step are read right behind the barrier and the member's last
    // four products and its scaling into the running sum cover their latency.  Loads run two members ahead.
    struct F2 {
      bf16x8 a[2], b[TN];
    };
    auto read2 = [&](F2& f, const unsigned char* st, int kk) {
#pragma unroll
      for (int i = 0; i < 2; ++i) f.a[i] = *reinterpret_cast<const bf16x8*>(st + a_base + i * 4096 + ck[kk]);
#pragma unroll
      for (int j = 0; j < TN; ++j) f.b[j] = *reinterpret_cast<const bf16x8*>(st + b_base + j * 4096 + ck[kk]);
    };
    f32x16 acc[2][TN];
    auto mfma2 = [&](const F2& f) {
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[i], f.b[j], acc[i][j], 0, 0, 0);
    };
    auto mfma2_from = [&](const F2& f, const float (&c)[TN]) {       // a member starts from its per-column constant
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const f32x16 init = {c[j], c[j], c[j], c[j], c[j], c[j], c[j], c[j], c[j], c[j], c[j], c[j], c[j], c[j], c[j], c[j]};
#pragma unroll
        for (int i = 0; i < 2; ++i) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[i], f.b[j], init, 0, 0, 0);
      }
    };
    auto pin = [&]() {                                     // a fragment read behind each of the step's four products
#pragma unroll
      for (int t = 0; t < 2 + TN; ++t) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
    };
    auto vectors_of = [&](const unsigned char* st, float (&vb)[TN], float (&wj)[TN]) {
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const unsigned char* xs = st + xoff + colj + j * 64;
        auto column_value = [&](int slot, unsigned short mask) {
          const unsigned short raw = *reinterpret_cast<const unsigned short*>(xs + slot * VB) & mask;
          return (float)__builtin_bit_cast(bf16, raw);
        };
        if (ATT) {
          wj[j] = 1.f;
          vb[j] = column_value(0, mask1) + column_value(1, mask2);
        } else {
          wj[j] = column_value(0, 0xFFFF);
          vb[j] = column_value(1, mask1) + column_value(2, mask2);
        }
      }
    };
    if (gk == 0) return;                                   // uniform (the host never deals more shares than members)
    issue(0);
    if (gk > 1) issue(1);
    if (gk > 1) {
      if (extra) wait_vmcnt<AL + BL + 1>();
      else wait_vmcnt<AL + BL>();
    } else {
      wait_vmcnt<0>();
    }
    __builtin_amdgcn_s_barrier();
    if (gk > 2) issue(2);
    F2 f0, f1;
    float vb[TN], wj[TN], vbn[TN], wjn[TN];
    f32x4 areg[2][4];                                      // softmax weights of the member's rows (ATT)
    read2(f0, smem, 0);
    vectors_of(smem, vb, wj);
    int sc = 0;
    for (int m = 0; m < gk; ++m) {
      const unsigned char* st = smem + sc * kRedStageBytes;
      if (DCHAG_RING_PROBE & 1) {                          // waits, barrier and loads of a member, nothing else
        if (m + 2 < gk) {
          if (extra) wait_vmcnt<AL + BL + 1>();
          else wait_vmcnt<AL + BL>();
        } else {
          __builtin_amdgcn_s_waitcnt(0);
        }
        __builtin_amdgcn_s_barrier();
        if (m + 3 < gk) issue(sc);
        sc = sc == 2 ? 0 : sc + 1;
        continue;
      }
      __builtin_amdgcn_sched_barrier(0);
      read2(f1, st, 1);
      if (ATT) mfma2_from(f0, vb);
      else {
        const float zero[TN] = {};
        mfma2_from(f0, zero);
      }
      pin();
      read2(f0, st, 2);
      mfma2(f1);
      pin();
      read2(f1, st, 3);
      mfma2(f0);
      pin();
      if (ATT) {
        const float* al = reinterpret_cast<const float*>(st + xoff + AOFF + hrel * HB) + wm * 64 + 4 * lhi;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int q = 0; q < 4; ++q) areg[i][q] = *reinterpret_cast<const f32x4*>(al + i * 32 + 8 * q);
      }
      // member m + 1 has landed (this wavefront's share; member m + 2's loads may stay in flight) and every read of
      // member m's stage is in registers
      if (m + 2 < gk) {
        if (extra) wait_vmcnt<AL + BL + 1>();
        else wait_vmcnt<AL + BL>();
        __builtin_amdgcn_s_waitcnt((7 << 4) | (63 & 15) | ((63 >> 4) << 14));   // lgkmcnt(0), vmcnt untouched
      } else {
        __builtin_amdgcn_s_waitcnt(0);
      }
      __builtin_amdgcn_s_barrier();
      if (m + 3 < gk) issue(sc);                           // member m + 3 -> the stage just released
      sc = sc == 2 ? 0 : sc + 1;
      const unsigned char* sn = smem + sc * kRedStageBytes;
      __builtin_amdgcn_sched_barrier(0);
      read2(f0, sn, 0);                                    // past the last member: a stale stage, read and not used
      vectors_of(sn, vbn, wjn);
      mfma2(f1);
      __builtin_amdgcn_sched_barrier(0);
      if (ATT) {
        // rows of accumulator register r: 8 (r / 4) + 4 lhi + r % 4 of the block
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
              for (int e = 0; e < 4; ++e) o[i][j][4 * q + e] += areg[i][q][e] * acc[i][j][4 * q + e];
      } else {
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[i][j][r] += wj[j] * acc[i][j][r];
#pragma unroll
        for (int j = 0; j < TN; ++j) cst[j] += wj[j] * vb[j];
      }
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        vb[j] = vbn[j];
        wj[j] = wjn[j];
      }
    }
    wait_vmcnt<0>();
  } else {
#pragma unroll
  for (int s0 = 0; s0 < NS - 1; ++s0)
    if (gk > s0) issue(s0);
  int sc = 0, si = NS - 1;
  for (int m = 0; m < gk; ++m) {
    // member m has landed (this wavefront's share: with three stages the loads of member m + 1 may stay in flight) ...
    if (NS == 3 && m + 1 < gk) {
      if (extra) wait_vmcnt<AL + BL + 1>();
      else wait_vmcnt<AL + BL>();
    } else {
      wait_vmcnt<0>();
    }
    // ... and for everyone; all wavefronts are done with member m - 1, whose stage takes member m + NS - 1
    __builtin_amdgcn_s_barrier();
    if (m + NS - 1 < gk) issue(si);
    si = si == NS - 1 ? 0 : si + 1;
    const unsigned char* st = smem + sc * kRedStageBytes;
    sc = sc == NS - 1 ? 0 : sc + 1;

    // per-column vectors of this member, read without a branch: an absent vector's slot holds arbitrary bytes, which the
    // mask turns into +0 (a branch per vector would put one LDS round trip after the other in front of the products)
    float vb[TN];                                        // per-column constant of this member: v1 + v2
    float wj[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const unsigned char* xs = st + xoff + colj + j * 64;
      auto column_value = [&](int slot, unsigned short mask) {
        const unsigned short raw = *reinterpret_cast<const unsigned short*>(xs + slot * VB) & mask;
        return (float)__builtin_bit_cast(bf16, raw);
      };
      if (ATT) {
        wj[j] = 1.f;
        vb[j] = column_value(0, mask1) + column_value(1, mask2);
      } else {
        wj[j] = column_value(0, 0xFFFF);
        vb[j] = column_value(1, mask1) + column_value(2, mask2);
      }
    }
    // Row block i = 0 first, then i = 1: while the matrix pipe works on the second block the vector ALUs scale the
    // first into the running sum (the two instruction streams are interleaved below, one MFMA per four FMAs).
    f32x16 acc[2][TN];
    bf16x8 bfr[4][TN], af[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      af[kk] = *reinterpret_cast<const bf16x8*>(st + a_base + ck[kk]);
#pragma unroll
      for (int j = 0; j < TN; ++j) bfr[kk][j] = *reinterpret_cast<const bf16x8*>(st + b_base + j * 4096 + ck[kk]);
    }
    const float* al = reinterpret_cast<const float*>(st + xoff + AOFF + hrel * HB) + wm * 64 + 4 * lhi;
    auto product = [&](int i) {
#pragma unroll
      for (int kk = 0; kk < 4; ++kk)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          if (kk == 0) {
            // the accumulation starts from the member's per-column constant (ATT) or from zero
            const float c = ATT ? vb[j] : 0.f;
            const f32x16 init = {c, c, c, c, c, c, c, c, c, c, c, c, c, c, c, c};
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[kk], bfr[kk][j], init, 0, 0, 0);
          } else {
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[kk], bfr[kk][j], acc[i][j], 0, 0, 0);
          }
        }
    };
    auto scale_in = [&](int i) {
      if (ATT) {
        // rows of accumulator register r: 8 (r / 4) + 4 lhi + r % 4 of the block
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const f32x4 a4 = *reinterpret_cast<const f32x4*>(al + i * 32 + 8 * q);
#pragma unroll
          for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) o[i][j][4 * q + e] += a4[e] * acc[i][j][4 * q + e];
        }
      } else {
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[i][j][r] += wj[j] * acc[i][j][r];
      }
    };
    product(0);
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) af[kk] = *reinterpret_cast<const bf16x8*>(st + a_base + 4096 + ck[kk]);
    __builtin_amdgcn_sched_barrier(0);
    product(1);
    scale_in(0);
#pragma unroll
    for (int t = 0; t < 4 * TN; ++t) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // one MFMA
      __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);   // four vector-ALU instructions
    }
    __builtin_amdgcn_sched_barrier(0);
    scale_in(1);
    if (!ATT) {
#pragma unroll
      for (int j = 0; j < TN; ++j) cst[j] += wj[j] * vb[j];
    }
  }
  }

  const size_t yoff = (((size_t)b * G + k) * N + n0 + wm * 64) * D + col_base + wcol + l32;
  const int nlim = N - n0 - wm * 64 - 4 * lhi;           // rows of this lane's half that are inside the image
  if (S > 1) {                                           // partial sum over this workgroup's members; k_vagg_merge adds them up
    float* pbase = ypart + (size_t)split * tw.nb * G * N * D + yoff;
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int rr = i * 32 + 8 * (r >> 2) + (r & 3);
          if (rr < nlim) pbase[(size_t)(rr + 4 * lhi) * D + j * 32] = o[i][j][r] + cst[j];
        }
    return;
  }
  bf16* ybase = y + yoff;
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int col = col_base + wcol + j * 32 + l32;
    const float add = cst[j] + (bias ? (float)bias[(size_t)k * D + col] : 0.f);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int rr = i * 32 + 8 * (r >> 2) + (r & 3);
        if (rr < nlim) ybase[(size_t)(rr + 4 * lhi) * D + j * 32] = (bf16)(o[i][j][r] + add);
      }
  }
}

}  // namespace dchag
