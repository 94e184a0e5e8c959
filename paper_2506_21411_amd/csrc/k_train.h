// Shape-generic kernels of the weight-folded forward and of the backward pass (any D, any group
// size, fp32 or bf16 storage, fp32 arithmetic).  Paper Section 2.1 (cross-attention aggregation),
// Section 3.3 (the module is trained through; its backward is the reverse of its forward).
//
// Notation: z[b,c,n,:] input tokens of a level, alpha[b,c,n,a] softmax weight of member c for head a,
// u[b,k,n,a,:] = sum_c alpha[b,c,n,a] z[b,c,n,:] (the group's tokens averaged per head),
// o = concatenated heads before the output projection, M[k][a][:] the query folded into the key
// weights.  Since the weights of a softmax sum to one,
//   o_a = sum_c alpha[c,a] (Wv z[c] + bv)_a = (Wv_a u_a) + bv_a ,
// so the value projection can run once per (group, patch, head) on u instead of once per member.
#pragma once
#include "dchag_dev.h"
#include "k_mfma.h"

namespace dchag {

// ---------------------------------------------------------------------------------------
// Strided batched matrix product, fp32 FMA, 64x64 tiles:
//   C(m,n) = scale * sum_kk A(m,kk) * B(kk,n) (+ bias[n])
// over a batch (b, k, a) = (batch element, group, head); with reduce_b the sum also runs over b
// (a contraction over token rows that are split in one block per batch element).
// ragged = 1: M of group k is rows_of(k); ragged = 2: K of group k is rows_of(k).
// grid (ceil(N/64), ceil(M/64), batch), block 256.
// ---------------------------------------------------------------------------------------
struct GemmOperand {
  long sb, sk, sa;   // offset per batch element, group, head
  long s0, s1;       // strides of the operand's two indices: A(m,kk), B(kk,n), C(m,n)
};
struct GemmDesc {
  int M, N, K;
  int nb, nk, na;
  int reduce_b;
  int ragged, ragged_total, ragged_nominal;
  GemmOperand A, Bm, C;
  long bias_sk, bias_sa;
  float scale;
  long rs_sk, rs_sa;   // k_gemm_mfma with a transposed A: optional row sums of A over the contraction, per (k, a)
  int c_vec;           // k_gemm_mfma: C rows are contiguous and 16-byte aligned, N % 8 == 0: store whole 16-byte chunks
};

template <typename TA, typename TB, typename TC>
__global__ __launch_bounds__(256) void k_gemm_generic(GemmDesc d, const TA* __restrict__ A, const TB* __restrict__ Bm,
                                                      const TB* __restrict__ bias, TC* __restrict__ C) {
  __shared__ float As[16][64 + 1];
  __shared__ float Bs[16][64 + 1];
  int z = blockIdx.z;
  const int a = z % d.na;
  z /= d.na;
  const int k = z % d.nk;
  const int b0 = d.reduce_b ? 0 : z / d.nk;
  const int b1 = d.reduce_b ? d.nb : b0 + 1;
  int M = d.M, K = d.K;
  if (d.ragged) {
    int left = d.ragged_total - k * d.ragged_nominal;
    left = left < d.ragged_nominal ? left : d.ragged_nominal;
    if (d.ragged == 1) M = left; else K = left;
  }
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  if (m0 >= M) return;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;
  const bool a_kfast = d.A.s1 == 1, b_kfast = d.Bm.s0 == 1;
  for (int b = b0; b < b1; ++b) {
    const TA* Ab = A + d.A.sb * b + d.A.sk * k + d.A.sa * a;
    const TB* Bb = Bm + d.Bm.sb * b + d.Bm.sk * k + d.Bm.sa * a;
    for (int k0 = 0; k0 < K; k0 += 16) {
      for (int idx = threadIdx.x; idx < 64 * 16; idx += 256) {
        const int mm = a_kfast ? idx >> 4 : idx & 63, kk = a_kfast ? idx & 15 : idx >> 6;
        As[kk][mm] = (m0 + mm < M && k0 + kk < K) ? to_f32(Ab[d.A.s0 * (m0 + mm) + d.A.s1 * (k0 + kk)]) : 0.f;
        const int nn = b_kfast ? idx >> 4 : idx & 63, kb = b_kfast ? idx & 15 : idx >> 6;
        Bs[kb][nn] = (n0 + nn < d.N && k0 + kb < K) ? to_f32(Bb[d.Bm.s0 * (k0 + kb) + d.Bm.s1 * (n0 + nn)]) : 0.f;
      }
      __syncthreads();
#pragma unroll
      for (int kk = 0; kk < 16; ++kk) {
        float av[4], bv[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) av[i] = As[kk][ty * 4 + i];
#pragma unroll
        for (int j = 0; j < 4; ++j) bv[j] = Bs[kk][tx * 4 + j];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[i][j] += av[i] * bv[j];
      }
      __syncthreads();
    }
  }
  TC* Cb = C + d.C.sb * b0 + d.C.sk * k + d.C.sa * a;
  const TB* bs = bias ? bias + d.bias_sk * k + d.bias_sa * a : nullptr;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + ty * 4 + i;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx * 4 + j;
      if (n < d.N) Cb[d.C.s0 * m + d.C.s1 * n] = from_f32<TC>(acc[i][j] * d.scale + (bs ? to_f32(bs[n]) : 0.f));
    }
  }
}

// ---------------------------------------------------------------------------------------
// Softmax over the members of a group, in place on the scores S[B,Cin,N,heads] (fp32).
// One thread per (b, k, n, head).
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_softmax_group(int Cin, int N, int heads, int g, int G, long total,
                                                       float* __restrict__ S) {
  const long idx = (long)blockIdx.x * 256 + threadIdx.x;     // ((b * G + k) * N + n) * heads + a
  if (idx >= total) return;
  const int a = (int)(idx % heads);
  long t = idx / heads;
  const int n = (int)(t % N);
  t /= N;
  const int k = (int)(t % G), b = (int)(t / G);
  const int c0 = k * g, c1 = min(c0 + g, Cin);
  float* s = S + (((size_t)b * Cin) * N + n) * heads + a;
  const size_t cs = (size_t)N * heads;
  float mx = -INFINITY;
  for (int c = c0; c < c1; ++c) mx = fmaxf(mx, s[c * cs]);
  float den = 0.f;
  for (int c = c0; c < c1; ++c) den += __expf(s[c * cs] - mx);
  const float inv = 1.f / den;
  for (int c = c0; c < c1; ++c) s[c * cs] = __expf(s[c * cs] - mx) * inv;
}

// Reverse of the softmax, in place on dalpha:  ds[c] = alpha[c] * (dalpha[c] - sum_c' alpha[c'] dalpha[c']).
__global__ __launch_bounds__(256) void k_softmax_group_backward(int Cin, int N, int heads, int g, int G, long total,
                                                                const float* __restrict__ alpha,
                                                                float* __restrict__ dalpha) {
  const long idx = (long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  const int a = (int)(idx % heads);
  long t = idx / heads;
  const int n = (int)(t % N);
  t /= N;
  const int k = (int)(t % G), b = (int)(t / G);
  const int c0 = k * g, c1 = min(c0 + g, Cin);
  const size_t base = (((size_t)b * Cin) * N + n) * heads + a, cs = (size_t)N * heads;
  float dot = 0.f;
  for (int c = c0; c < c1; ++c) dot += alpha[base + c * cs] * dalpha[base + c * cs];
  for (int c = c0; c < c1; ++c) dalpha[base + c * cs] = alpha[base + c * cs] * (dalpha[base + c * cs] - dot);
}

// ---------------------------------------------------------------------------------------
// Per-head weighted token sums:  u[b,k,n,a,:] = sum_{c in group k} alpha[b,c,n,a] * z[b,c,n,:]
// grid (N, G, B), block 256; a thread owns columns d = tid, tid + 256, .. and HMAX heads at a time.
// ---------------------------------------------------------------------------------------
template <typename T, int HMAX>
__global__ __launch_bounds__(256) void k_head_sums(int Cin, int N, int D, int heads, int g,
                                                   const float* __restrict__ alpha, const T* __restrict__ z,
                                                   T* __restrict__ u) {
  __shared__ float al[32][HMAX];
  const int n = blockIdx.x, k = blockIdx.y, b = blockIdx.z, G = gridDim.y;
  const int c0 = k * g, c1 = min(c0 + g, Cin);
  for (int a0 = 0; a0 < heads; a0 += HMAX) {
    for (int d0 = 0; d0 < D; d0 += 256) {
      const int dcol = d0 + threadIdx.x;
      float acc[HMAX];
#pragma unroll
      for (int a = 0; a < HMAX; ++a) acc[a] = 0.f;
      for (int cb = c0; cb < c1; cb += 32) {
        __syncthreads();
        for (int idx = threadIdx.x; idx < 32 * HMAX; idx += 256) {
          const int cc = idx / HMAX, a = idx % HMAX;
          al[cc][a] = (cb + cc < c1 && a0 + a < heads)
                          ? alpha[(((size_t)b * Cin + cb + cc) * N + n) * heads + a0 + a] : 0.f;
        }
        __syncthreads();
        if (dcol < D) {
          const int cn = min(32, c1 - cb);
          for (int cc = 0; cc < cn; ++cc) {
            const float zv = to_f32(z[(((size_t)b * Cin + cb + cc) * N + n) * D + dcol]);
#pragma unroll
            for (int a = 0; a < HMAX; ++a) acc[a] += al[cc][a] * zv;
          }
        }
      }
      if (dcol < D) {
#pragma unroll
        for (int a = 0; a < HMAX; ++a)
          if (a0 + a < heads) u[((((size_t)b * G + k) * N + n) * heads + a0 + a) * D + dcol] = from_f32<T>(acc[a]);
      }
    }
  }
}

// ---------------------------------------------------------------------------------------
// dalpha[b,c,n,a] = w[b,k,n,a,:] . z[b,c,n,:]      (w = Wv_a^T do_a, the gradient at u_a)
// The value bias adds the same amount to every member of a group and cancels in the softmax
// Jacobian, so it is left out.  One wave per token; grid ceil(T/4), block 256.
// ---------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void k_dalpha(long T_total, int Cin, int N, int D, int heads, int g, int G,
                                                const T* __restrict__ z, const T* __restrict__ w,
                                                float* __restrict__ dalpha) {
  const long tok = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (tok >= T_total) return;
  const int n = (int)(tok % N);
  const int c = (int)((tok / N) % Cin);
  const int b = (int)(tok / ((long)N * Cin));
  const int k = c / g;
  const T* zr = z + (size_t)tok * D;
  const T* wr = w + (((size_t)b * G + k) * N + n) * heads * D;
  for (int a = 0; a < heads; ++a) {
    float acc = 0.f;
    for (int j = lane; j < D; j += kWave) acc += to_f32(zr[j]) * to_f32(wr[(size_t)a * D + j]);
    acc = wave_sum(acc);
    if (lane == 0) dalpha[(size_t)tok * heads + a] = acc;
  }
}

// ---------------------------------------------------------------------------------------
// Gradient at the input tokens of an attention level:
//   dz[b,c,n,:] = sum_a alpha[b,c,n,a] * w[b,k,n,a,:]  +  ds[b,c,n,a] * M[k][a][:]
// (value path and key path).  grid (Cin, N, B), block 256.
// ---------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void k_dz_attention(int Cin, int N, int D, int heads, int g, int G,
                                                      const float* __restrict__ alpha, const float* __restrict__ ds,
                                                      const T* __restrict__ w, const float* __restrict__ Mf,
                                                      T* __restrict__ dz) {
  const int c = blockIdx.x, n = blockIdx.y, b = blockIdx.z;
  const int k = c / g;
  const size_t tok = ((size_t)b * Cin + c) * N + n;
  const float* al = alpha + tok * heads;
  const float* dsr = ds + tok * heads;
  const T* wr = w + (((size_t)b * G + k) * N + n) * heads * D;
  const float* mr = Mf + (size_t)k * heads * D;
  for (int j = threadIdx.x; j < D; j += 256) {
    float acc = 0.f;
    for (int a = 0; a < heads; ++a) acc += al[a] * to_f32(wr[(size_t)a * D + j]) + dsr[a] * mr[(size_t)a * D + j];
    dz[tok * D + j] = from_f32<T>(acc);
  }
}

// ---------------------------------------------------------------------------------------
// Column sums over the rows of every group:  out[k][i] = sum_b sum_{r < rows_of(k)} X[first_row(b,k) + r][i]
// grid (ceil(D/64), G), block 1024: a block owns 64 columns; lane l of a wavefront takes the 4 columns 4 (l % 16) .. of
// row 4 wave + l / 16 and every 64th row after it (one 8- or 16-byte load per row); the four row groups of a
// wavefront meet by lane exchange, the 16 wavefronts in LDS, both in a fixed order.  D % 4 == 0.
template <typename T, typename TO>
__global__ __launch_bounds__(1024) void k_colsum(int B, int D, RowBlocks rb, const T* __restrict__ X,
                                                 TO* __restrict__ out) {
  typedef __attribute__((ext_vector_type(4))) T vec4;
  __shared__ float part[16][64];
  const int k = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int cg = lane & 15, rs = lane >> 4;               // 4 columns of the block's 64; row wave * 4 + rs, then every 64th
  const int i = blockIdx.x * 64 + cg * 4;
  const int rows = rb.rows_of(k);
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  if (i < D)
    for (int b = 0; b < B; ++b) {
      const T* xb = X + (size_t)rb.first_row(b, k) * D + i;
      for (int r = wave * 4 + rs; r < rows; r += 64) {
        const vec4 v = *reinterpret_cast<const vec4*>(xb + (size_t)r * D);
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[e] += to_f32(v[e]);
      }
    }
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    acc[e] += __shfl_xor(acc[e], 16, kWave);
    acc[e] += __shfl_xor(acc[e], 32, kWave);
  }
  if (rs == 0) {
#pragma unroll
    for (int e = 0; e < 4; ++e) part[wave][cg * 4 + e] = acc[e];
  }
  __syncthreads();
  if (threadIdx.x < 64) {
    const int ii = blockIdx.x * 64 + threadIdx.x;
    float sum = 0.f;
#pragma unroll
    for (int w16 = 0; w16 < 16; ++w16) sum += part[w16][threadIdx.x];
    if (ii < D) out[(size_t)k * D + ii] = from_f32<TO>(sum);
  }
}

// ---------------------------------------------------------------------------------------
// dQ[k][i] = (1/sqrt(dh)) * sum_j Wk[k][i][j] * r[k][a(i)][j]   with  r[k][a][:] = sum over the group's tokens
// of ds[.,a] * z  (one wave per row).  Also writes the query-bias gradient, which equals dQ.
// grid (ceil(D/4), G), block 256.
// ---------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void k_query_grad(int D, int heads, const T* __restrict__ Wk,
                                                    const float* __restrict__ r, float* __restrict__ dQ,
                                                    T* __restrict__ dbq) {
  const int k = blockIdx.y;
  const int i = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (i >= D) return;
  const int dh = D / heads;
  const T* w = Wk + ((size_t)k * D + i) * D;
  const float* rv = r + ((size_t)k * heads + i / dh) * D;
  float acc = 0.f;
  for (int j = lane; j < D; j += kWave) acc += to_f32(w[j]) * rv[j];
  acc = wave_sum(acc) * rsqrtf((float)dh);
  if (lane == 0) {
    dQ[(size_t)k * D + i] = acc;
    if (dbq) dbq[(size_t)k * D + i] = from_f32<T>(acc);
  }
}

// dquery[k][j] = sum_i Wq[k][i][j] * dQ[k][i].  grid (ceil(D/64), G), block 1024: a block owns 64 columns; lane l of a
// wavefront takes the 4 columns 4 (l % 16) .. of row 4 wave + l / 16 and every 64th row after it; the four row groups
// of a wavefront meet by lane exchange, the 16 wavefronts in LDS, both in a fixed order.  Requires D % 4 == 0.
template <typename T>
__global__ __launch_bounds__(1024) void k_query_input_grad(int D, const T* __restrict__ Wq,
                                                           const float* __restrict__ dQ, T* __restrict__ dquery) {
  __shared__ float part[16][64];
  const int k = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int cg = lane & 15, rs = lane >> 4;
  const int j = blockIdx.x * 64 + cg * 4;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  if (j < D) {
    const T* w = Wq + (size_t)k * D * D + j;
    const float* dq = dQ + (size_t)k * D;
    for (int i = wave * 4 + rs; i < D; i += 64) {
      const float q = dq[i];
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[e] += to_f32(w[(size_t)i * D + e]) * q;
    }
  }
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    acc[e] += __shfl_xor(acc[e], 16, kWave);
    acc[e] += __shfl_xor(acc[e], 32, kWave);
  }
  if (rs == 0) {
#pragma unroll
    for (int e = 0; e < 4; ++e) part[wave][cg * 4 + e] = acc[e];
  }
  __syncthreads();
  if (threadIdx.x < 64) {
    const int jj = blockIdx.x * 64 + threadIdx.x;
    float sum = 0.f;
#pragma unroll
    for (int w16 = 0; w16 < 16; ++w16) sum += part[w16][threadIdx.x];
    if (jj < D) dquery[(size_t)k * D + jj] = from_f32<T>(sum);
  }
}

// ---------------------------------------------------------------------------------------
// Rank-one weight gradients:  out[k][i][j] = scale * rowv[k][i] * colv[k][i / rows_per_vec][j]
//   key weights:   rowv = projected query, colv = r[k][a][:], rows_per_vec = dh, scale = 1/sqrt(dh)
//   query weights: rowv = dQ, colv = the learned query, rows_per_vec = D
// grid (ceil(D/256), D, G), block 256.
// ---------------------------------------------------------------------------------------
// The same for D % 8 == 0 and 16-byte aligned tensors: a thread writes 8 adjacent columns at once and takes 8 such
// chunks, 256 * 8 chunks per block.  grid (ceil(D * D / 8 / 2048), G), block 256.
template <typename TV, typename T>
__global__ __launch_bounds__(256) void k_outer_rows_vec(int D, int rows_per_vec, float scale,
                                                        const float* __restrict__ rowv, const TV* __restrict__ colv,
                                                        T* __restrict__ out) {
  const int k = blockIdx.y;
  const int cpr = D / 8;                                           // chunks per row
  const long chunks = (long)D * cpr;
  const int nvec = D / rows_per_vec;
#pragma unroll
  for (int u = 0; u < 8; ++u) {
    const long idx = ((long)blockIdx.x * 8 + u) * 256 + threadIdx.x;
    if (idx >= chunks) return;
    const int i = (int)(idx / cpr), j = (int)(idx % cpr) * 8;
    const float rv = rowv[(size_t)k * D + i] * scale;
    const TV* cv = colv + ((size_t)k * nvec + i / rows_per_vec) * D + j;
    T* o = out + ((size_t)k * D + i) * D + j;
    float c[8];
    if constexpr (sizeof(TV) == 2) {
      const bf16x8 v = *reinterpret_cast<const bf16x8*>(cv);
#pragma unroll
      for (int e = 0; e < 8; ++e) c[e] = (float)v[e];
    } else {
      const f32x4 v0 = *reinterpret_cast<const f32x4*>(cv), v1 = *reinterpret_cast<const f32x4*>(cv + 4);
#pragma unroll
      for (int e = 0; e < 4; ++e) { c[e] = v0[e]; c[4 + e] = v1[e]; }
    }
    if constexpr (sizeof(T) == 2) {
      bf16x8 r;
#pragma unroll
      for (int e = 0; e < 8; ++e) r[e] = (bf16)(rv * c[e]);
      *reinterpret_cast<bf16x8*>(o) = r;
    } else {
      *reinterpret_cast<f32x4*>(o) = f32x4{rv * c[0], rv * c[1], rv * c[2], rv * c[3]};
      *reinterpret_cast<f32x4*>(o + 4) = f32x4{rv * c[4], rv * c[5], rv * c[6], rv * c[7]};
    }
  }
}

template <typename TV, typename T>
__global__ __launch_bounds__(256) void k_outer_rows(int D, int rows_per_vec, float scale,
                                                    const float* __restrict__ rowv, const TV* __restrict__ colv,
                                                    T* __restrict__ out) {
  const int k = blockIdx.z, i = blockIdx.y;
  const int j = blockIdx.x * 256 + threadIdx.x;
  if (j >= D) return;
  const int nvec = D / rows_per_vec;
  const float rv = rowv[(size_t)k * D + i] * scale;
  out[((size_t)k * D + i) * D + j] = from_f32<T>(rv * to_f32(colv[((size_t)k * nvec + i / rows_per_vec) * D + j]));
}

template <typename T>
__global__ __launch_bounds__(256) void k_fill_zero(long n, T* __restrict__ out) {
  const long i = (long)blockIdx.x * 256 + threadIdx.x;
  if (i < n) out[i] = from_f32<T>(0.f);
}

// ---------------------------------------------------------------------------------------
// Patches as rows:  patches[b,c,n,kk] = pixel kk (row by row) of patch n of x[b,c]   and the reverse
// scatter of patch rows back into an image.  One thread per run of V adjacent pixels of one patch row
// (V divides p: both sides of the copy are V contiguous elements).  `total` counts runs.
// ---------------------------------------------------------------------------------------
template <typename T, int V, bool TO_IMAGE>
__global__ __launch_bounds__(256) void k_patch_rows(long total, int H, int W, int p, T* __restrict__ img,
                                                    T* __restrict__ patches) {
  typedef __attribute__((ext_vector_type(V))) T vec;
  const long idx = (long)blockIdx.x * 256 + threadIdx.x;      // run index in [B*C, H, W / V]
  if (idx >= total) return;
  const int wv = W / V;
  const int wx = (int)(idx % wv) * V;
  long t = idx / wv;
  const int hy = (int)(t % H);
  const long bc = t / H;
  const int pw = W / p, pp = p * p;
  const int n = (hy / p) * pw + wx / p, kk = (hy % p) * p + wx % p;
  const size_t pi = ((size_t)bc * (H / p) * pw + n) * pp + kk;
  const size_t ii = ((size_t)bc * H + hy) * W + wx;
  if (V == 1) {
    if (TO_IMAGE) img[ii] = patches[pi];
    else patches[pi] = img[ii];
  } else {
    if (TO_IMAGE) *reinterpret_cast<vec*>(img + ii) = *reinterpret_cast<const vec*>(patches + pi);
    else *reinterpret_cast<vec*>(patches + pi) = *reinterpret_cast<const vec*>(img + ii);
  }
}

// ---------------------------------------------------------------------------------------
// Linear (D-CHAG-L) level, backward:   y[b,k,n,d] = sum_cl w[k][cl][d] z[b,k*g+cl,n,d] + bias[k][d]
//   dz[b,c,n,d] = w[k][cl][d] * dy[b,k,n,d]                       grid ceil(total/256), one thread per element
//   dw[k][cl][d] = sum_{b,n} dy[b,k,n,d] * z[b,k*g+cl,n,d]        grid (ceil(D/64), G*g), block 256 (waves split rows)
// Members a short last group does not have get a zero weight gradient.
// ---------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void k_channel_mix_dz(long total, int Cin, int N, int D, int g, int G,
                                                        const T* __restrict__ w, const T* __restrict__ dy,
                                                        T* __restrict__ dz) {
  const long idx = (long)blockIdx.x * 256 + threadIdx.x;      // ((b * Cin + c) * N + n) * D + d
  if (idx >= total) return;
  const int d = (int)(idx % D);
  long t = idx / D;
  const int n = (int)(t % N);
  t /= N;
  const int c = (int)(t % Cin), b = (int)(t / Cin);
  const int k = c / g, cl = c % g;
  dz[idx] = from_f32<T>(to_f32(w[((size_t)k * g + cl) * D + d]) * to_f32(dy[(((size_t)b * G + k) * N + n) * D + d]));
}

template <typename T>
__global__ __launch_bounds__(256) void k_channel_mix_dw(int B, int Cin, int N, int D, int g, int G,
                                                        const T* __restrict__ z, const T* __restrict__ dy,
                                                        T* __restrict__ dw) {
  __shared__ float part[3][64];
  const int kc = blockIdx.y;
  const int k = kc / g, cl = kc % g, c = k * g + cl;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int d = blockIdx.x * 64 + lane;
  float acc = 0.f;
  if (d < D && c < Cin)
    for (int b = 0; b < B; ++b) {
      const T* zb = z + (((size_t)b * Cin + c) * N) * D + d;
      const T* yb = dy + (((size_t)b * G + k) * N) * D + d;
      for (int n = wave; n < N; n += 4) acc += to_f32(zb[(size_t)n * D]) * to_f32(yb[(size_t)n * D]);
    }
  if (wave > 0) part[wave - 1][lane] = acc;
  __syncthreads();
  if (wave == 0 && d < D) dw[(size_t)kc * D + d] = from_f32<T>(acc + part[0][lane] + part[1][lane] + part[2][lane]);
}

// The same two kernels for D % 8 == 0 and 16-byte aligned tensors, 8 adjacent columns per thread.
template <typename T>
__device__ __forceinline__ void load8(const T* p, float (&v)[8]) {
  if constexpr (sizeof(T) == 2) {
    const bf16x8 x = *reinterpret_cast<const bf16x8*>(p);
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = (float)x[e];
  } else {
    const f32x4 x0 = *reinterpret_cast<const f32x4*>(p), x1 = *reinterpret_cast<const f32x4*>(p + 4);
#pragma unroll
    for (int e = 0; e < 4; ++e) { v[e] = x0[e]; v[4 + e] = x1[e]; }
  }
}
template <typename T>
__device__ __forceinline__ void store8(T* p, const float (&v)[8]) {
  if constexpr (sizeof(T) == 2) {
    bf16x8 x;
#pragma unroll
    for (int e = 0; e < 8; ++e) x[e] = (bf16)v[e];
    *reinterpret_cast<bf16x8*>(p) = x;
  } else {
    *reinterpret_cast<f32x4*>(p) = f32x4{v[0], v[1], v[2], v[3]};
    *reinterpret_cast<f32x4*>(p + 4) = f32x4{v[4], v[5], v[6], v[7]};
  }
}

// dz: grid (ceil(N / 16), Cin, B), block 256: thread t takes the columns 8 (t % (D/8)) .. of every (256 / (D/8))-th
// patch of the block's 16 when D <= 2048, and walks the columns otherwise; the mixing weights stay in registers.
template <typename T>
__global__ __launch_bounds__(256) void k_channel_mix_dz_vec(int Cin, int N, int D, int g, int G,
                                                            const T* __restrict__ w, const T* __restrict__ dy,
                                                            T* __restrict__ dz) {
  const int c = blockIdx.y, b = blockIdx.z, k = c / g, cl = c % g;
  const int n0 = blockIdx.x * 16, n1 = min(n0 + 16, N);
  const int d8 = D / 8;
  const T* wr = w + ((size_t)k * g + cl) * D;
  const T* yb = dy + (((size_t)b * G + k) * N) * D;
  T* zb = dz + (((size_t)b * Cin + c) * N) * D;
  for (int ch = threadIdx.x; ch < 16 * d8; ch += 256) {            // chunk: (patch of the tile, 8 columns)
    const int n = n0 + ch / d8, d = (ch % d8) * 8;
    if (n >= n1) break;
    float wv[8], yv[8];
    load8(wr + d, wv);
    load8(yb + (size_t)n * D + d, yv);
#pragma unroll
    for (int e = 0; e < 8; ++e) yv[e] *= wv[e];
    store8(zb + (size_t)n * D + d, yv);
  }
}

// dw: grid (ceil(D / 1024), G * g), block 256: 128 threads cover 1024 columns, the two halves of the block take the
// even and the odd rows (b, n) and meet in LDS.
template <typename T>
__global__ __launch_bounds__(256) void k_channel_mix_dw_vec(int B, int Cin, int N, int D, int g, int G,
                                                            const T* __restrict__ z, const T* __restrict__ dy,
                                                            T* __restrict__ dw) {
  __shared__ float part[128][9];
  const int kc = blockIdx.y;
  const int k = kc / g, cl = kc % g, c = k * g + cl;
  const int t = threadIdx.x & 127, half = threadIdx.x >> 7;
  const int d = blockIdx.x * 1024 + t * 8;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  const bool live = d < D && c < Cin;
  if (live) {
    const long rows = (long)B * N;
#pragma unroll 4
    for (long r = half; r < rows; r += 2) {
      const int b = (int)(r / N), n = (int)(r % N);
      float zv[8], yv[8];
      load8(z + (((size_t)b * Cin + c) * N + n) * D + d, zv);
      load8(dy + (((size_t)b * G + k) * N + n) * D + d, yv);
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] += zv[e] * yv[e];
    }
  }
  if (half == 1) {
#pragma unroll
    for (int e = 0; e < 8; ++e) part[t][e] = acc[e];
  }
  __syncthreads();
  if (half == 0 && d < D) {                                        // members a short last group lacks: zero
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] += part[t][e];
    store8(dw + (size_t)kc * D + d, acc);
  }
}

// ---------------------------------------------------------------------------------------
// Gradients of a linear first level and of the tokenizer below it without the tokens (bf16).  With
//   P[c][d][kk] = sum_{b,n} dy[b,k(c),n,d] * patch[b,c,n,kk]   (one product per channel)   and   S[k][d] = sum_{b,n} dy
// the token t[c] = We[c] patch + be[c] + ce[c] and the mixing weight s[c] give
//   dmix[c][d]      = sum_{b,n} t[c][d] dy[d]  = sum_kk We[c][d][kk] P[c][d][kk] + (be + ce)[c][d] S[k][d]
//   dWe[c][d][kk]   = s[c][d] P[c][d][kk]          dtok_bias[c][d] = s[c][d] S[k][d]
// and the pixel gradient is dy times the scaled weights  Ws[c][d][kk] = We[c][d][kk] s[c][d], which this kernel also
// writes.  One thread per 8 pixels of a (c, d) row, pp / 8 threads per row (a power of two <= 64), rows summed by
// lane exchange.  grid ceil(C D (pp/8) / 256), block 256.  Any output pointer may be NULL.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_linear_first_grads(long chunks, int C, int D, int pp, int g,
                                                            const float* __restrict__ P, const float* __restrict__ S,
                                                            const bf16* __restrict__ We, const bf16* __restrict__ be,
                                                            const bf16* __restrict__ ce, const bf16* __restrict__ mix,
                                                            bf16* __restrict__ dWe, bf16* __restrict__ dtok_bias,
                                                            bf16* __restrict__ dmix, bf16* __restrict__ Ws) {
  const long idx = (long)blockIdx.x * 256 + threadIdx.x;           // ((c * D + d) * (pp / 8) + chunk)
  const int cpr = pp / 8;
  const bool live = idx < chunks;
  const long row = (live ? idx : chunks - 1) / cpr;                // c * D + d
  const int ch = (int)((live ? idx : chunks - 1) % cpr);
  const int c = (int)(row / D), d = (int)(row % D);
  const int k = c / g;
  const float s = (float)mix[(size_t)c * D + d];                   // mixing weights are [G * g][D], member c = k g + cl
  const size_t o = (size_t)row * pp + ch * 8;
  const bf16x8 w8 = *reinterpret_cast<const bf16x8*>(We + o);
  float dot = 0.f;
  if (P) {
    const f32x4 p0 = *reinterpret_cast<const f32x4*>(P + o), p1 = *reinterpret_cast<const f32x4*>(P + o + 4);
    bf16x8 g8;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      dot += (float)w8[e] * p0[e] + (float)w8[4 + e] * p1[e];
      g8[e] = (bf16)(s * p0[e]);
      g8[4 + e] = (bf16)(s * p1[e]);
    }
    if (dWe && live) *reinterpret_cast<bf16x8*>(dWe + o) = g8;
  }
  if (Ws && live) {
    bf16x8 v;
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = (bf16)((float)w8[e] * s);
    *reinterpret_cast<bf16x8*>(Ws + o) = v;
  }
  for (int off = 1; off < cpr; off <<= 1) dot += __shfl_xor(dot, off, kWave);     // the cpr threads of a row are adjacent lanes
  if (live && ch == 0) {
    const float sv = S[(size_t)k * D + d];
    if (dmix) {
      float bias = 0.f;
      if (be) bias += (float)be[(size_t)c * D + d];
      if (ce) bias += (float)ce[(size_t)c * D + d];
      dmix[(size_t)c * D + d] = (bf16)(dot + bias * sv);
    }
    if (dtok_bias) dtok_bias[(size_t)c * D + d] = (bf16)(s * sv);
  }
}

}  // namespace dchag

// =======================================================================================
// bf16 MFMA kernels of the folded forward and of the backward
// =======================================================================================
namespace dchag {

// ---------------------------------------------------------------------------------------
// Strided batched matrix product on bf16 MFMA (32x32x16, fp32 accumulation), BM x BN x 64 tiles,
// four wavefronts (WM x WN), operands staged through XOR-swizzled LDS rows of 64 contraction elements.
// Same contract as k_gemm_generic (GemmDesc), restricted to:
//   K % 64 == 0 (no ragged K), every operand has one unit stride, 16-byte aligned rows.
// An operand whose unit stride is the contraction index is copied chunk by chunk (AT / BT = false);
// one whose unit stride is its row index m (or n) is read as 8 x 8 blocks (8 contraction steps x 8
// rows), transposed in registers and written as whole 16-byte LDS chunks (AT / BT = true; threads
// 0 .. BM-1 take A's blocks, the last BN threads B's).
// With a transposed A the kernel can also write the sums of A's rows over the whole contraction (all batch
// elements when reduce_b is set): the bias gradients that go with a weight gradient, at no extra pass over A.
// grid (ceil(N/BN), ceil(M/BM), batch), block 256, dynamic LDS 2 x (BM + BN) x 128 bytes.
// ---------------------------------------------------------------------------------------
template <int BM, int BN, int WM, int WN, bool AT, bool BT, typename TC>
__global__ __launch_bounds__(256) void k_gemm_mfma(GemmDesc d, const bf16* __restrict__ A, const bf16* __restrict__ Bm,
                                                   const bf16* __restrict__ bias, TC* __restrict__ C,
                                                   TC* __restrict__ rowsum) {
  static_assert(WM * WN == 4 && BM % (WM * 32) == 0 && BN % (WN * 32) == 0 && BM <= 128 && BN <= 128, "tile");
  constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
  constexpr int A_CH = BM * 8 / 256, B_CH = BN * 8 / 256;          // 16-byte chunks per thread and stage (copied)
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16x8* As = reinterpret_cast<bf16x8*>(smem);           // [2][BM * 8]
  bf16x8* Bs = As + 2 * BM * 8;                           // [2][BN * 8]
  int z = blockIdx.z;
  const int a = z % d.na;
  z /= d.na;
  const int k = z % d.nk;
  const int b0 = d.reduce_b ? 0 : z / d.nk;
  const int b1 = d.reduce_b ? d.nb : b0 + 1;
  int M = d.M;
  if (d.ragged == 1) {
    const int left = d.ragged_total - k * d.ragged_nominal;
    M = left < d.ragged_nominal ? left : d.ragged_nominal;
  }
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  if (m0 >= M) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const int l32 = lane & 31, lhi = lane >> 5;

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  bf16x8 a_reg[AT ? 8 : A_CH], b_reg[BT ? 8 : B_CH];
  const int KT = d.K / 64;
  const int steps = (b1 - b0) * KT;
  const int tb = tid - (256 - BN);                          // B's transposing threads: tb >= 0

  // optional by-product with a transposed A: rsum[r] collects sum over the contraction of A(row 8 mc + r, .)
  // for this thread's share of the contraction steps (only the blocks of the first column tile do it)
  const bool want_rs = AT && rowsum != nullptr && blockIdx.x == 0;
  float rsum[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

  auto load = [&](int s) {
    const int b = b0 + s / KT, k0 = (s % KT) * 64;
    const bf16* Ab = A + d.A.sb * b + d.A.sk * k + d.A.sa * a;
    const bf16* Bb = Bm + d.Bm.sb * b + d.Bm.sk * k + d.Bm.sa * a;
    if (!AT) {
#pragma unroll
      for (int i = 0; i < A_CH; ++i) {
        const int idx = tid + i * 256, row = idx >> 3, ch = idx & 7;
        const int gr = min(m0 + row, M - 1);
        a_reg[i] = *reinterpret_cast<const bf16x8*>(Ab + d.A.s0 * gr + k0 + ch * 8);
      }
    } else if (tid < BM) {
      const int mc = tid % (BM / 8), kc = tid / (BM / 8);  // 8 rows m0 + 8 mc .., contraction steps k0 + 8 kc ..
      const int gm = min(m0 + mc * 8, M - 8);
#pragma unroll
      for (int i = 0; i < 8; ++i) a_reg[i] = *reinterpret_cast<const bf16x8*>(Ab + d.A.s1 * (k0 + kc * 8 + i) + gm);
    }
    if (!BT) {
#pragma unroll
      for (int i = 0; i < B_CH; ++i) {
        const int idx = tid + i * 256, row = idx >> 3, ch = idx & 7;
        const int gr = min(n0 + row, d.N - 1);
        b_reg[i] = *reinterpret_cast<const bf16x8*>(Bb + d.Bm.s1 * gr + k0 + ch * 8);
      }
    } else if (tb >= 0) {
      const int nc = tb % (BN / 8), kc = tb / (BN / 8);
      const int gn = min(n0 + nc * 8, d.N - 8);
#pragma unroll
      for (int i = 0; i < 8; ++i) b_reg[i] = *reinterpret_cast<const bf16x8*>(Bb + d.Bm.s0 * (k0 + kc * 8 + i) + gn);
    }
  };
  auto store = [&](int buf) {
    bf16x8* Ad = As + buf * BM * 8;
    bf16x8* Bd = Bs + buf * BN * 8;
    if (!AT) {
#pragma unroll
      for (int i = 0; i < A_CH; ++i) {
        const int idx = tid + i * 256, row = idx >> 3, ch = idx & 7;
        Ad[lds_slot<1>(row, ch)] = a_reg[i];
      }
    } else if (tid < BM) {
      const int mc = tid % (BM / 8), kc = tid / (BM / 8);
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        bf16x8 v;
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = a_reg[i][r];
        Ad[lds_slot<1>(mc * 8 + r, kc)] = v;
        if (want_rs) {
#pragma unroll
          for (int i = 0; i < 8; ++i) rsum[r] += (float)a_reg[i][r];
        }
      }
    }
    if (!BT) {
#pragma unroll
      for (int i = 0; i < B_CH; ++i) {
        const int idx = tid + i * 256, row = idx >> 3, ch = idx & 7;
        Bd[lds_slot<1>(row, ch)] = b_reg[i];
      }
    } else if (tb >= 0) {
      const int nc = tb % (BN / 8), kc = tb / (BN / 8);
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        bf16x8 v;
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = b_reg[i][r];
        Bd[lds_slot<1>(nc * 8 + r, kc)] = v;
      }
    }
  };

  load(0);
  store(0);
  __syncthreads();
  for (int s = 0; s < steps; ++s) {
    const int cur = s & 1;
    if (s + 1 < steps) load(s + 1);
    const bf16x8* Ac = As + cur * BM * 8;
    const bf16x8* Bc = Bs + cur * BN * 8;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      bf16x8 af[TM], bfr[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) af[i] = Ac[lds_slot<1>(wm * (BM / WM) + i * 32 + l32, kk * 2 + lhi)];
#pragma unroll
      for (int j = 0; j < TN; ++j) bfr[j] = Bc[lds_slot<1>(wn * (BN / WN) + j * 32 + l32, kk * 2 + lhi)];
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    if (s + 1 < steps) store(cur ^ 1);
    __syncthreads();
  }

  if (AT && rowsum != nullptr && blockIdx.x == 0) {       // block-uniform: the eight shares of a row meet in LDS
    float* part = reinterpret_cast<float*>(smem);         // [8 shares][BM rows]; the stages are no longer read
    if (tid < BM) {
      const int mc = tid % (BM / 8), kc = tid / (BM / 8);
#pragma unroll
      for (int r = 0; r < 8; ++r) part[kc * BM + mc * 8 + r] = rsum[r];
    }
    __syncthreads();
    if (tid < BM && m0 + tid < M) {
      float sum = 0.f;
#pragma unroll
      for (int kc = 0; kc < 8; ++kc) sum += part[kc * BM + tid];
      rowsum[d.rs_sk * k + d.rs_sa * a + m0 + tid] = from_f32<TC>(sum);
    }
  }

  // 32x32 accumulator block: lane holds column (lane % 32); register r holds row 8 (r / 4) + 4 (lane / 32) + r % 4
  TC* Cb = C + d.C.sb * b0 + d.C.sk * k + d.C.sa * a;
  const bf16* bs = bias ? bias + d.bias_sk * k + d.bias_sa * a : nullptr;
  if (sizeof(TC) == 2 && d.c_vec) {
    // the tile goes through LDS (the stages are no longer read) so that rows leave in 16-byte chunks:
    // a lane's accumulator column is 2 bytes wide, a row of the tile up to 256 bytes
    constexpr int PITCH = BN + 8;                          // bf16 elements; 16 extra bytes keep the row starts apart
    bf16* tile = reinterpret_cast<bf16*>(smem);
    __syncthreads();                                      // (also orders the row-sum scratch before this reuse)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int nl = wn * (BN / WN) + j * 32 + l32;
      const float bv = (bs && n0 + nl < d.N) ? (float)bs[n0 + nl] : 0.f;
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int ml = wm * (BM / WM) + i * 32 + 8 * (r >> 2) + 4 * lhi + (r & 3);
          tile[ml * PITCH + nl] = (bf16)(acc[i][j][r] * d.scale + bv);
        }
    }
    __syncthreads();
    for (int idx = tid; idx < BM * (BN / 8); idx += 256) {
      const int ml = idx / (BN / 8), ch = idx % (BN / 8);
      const int m = m0 + ml, n = n0 + ch * 8;
      if (m < M && n < d.N)
        *reinterpret_cast<bf16x8*>(reinterpret_cast<bf16*>(Cb) + d.C.s0 * m + n) =
            *reinterpret_cast<const bf16x8*>(tile + ml * PITCH + ch * 8);
    }
    return;
  }
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int n = n0 + wn * (BN / WN) + j * 32 + l32;
    if (n >= d.N) continue;
    const float bv = bs ? (float)bs[n] : 0.f;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = m0 + wm * (BM / WM) + i * 32 + 8 * (r >> 2) + 4 * lhi + (r & 3);
        if (m < M) Cb[d.C.s0 * m + d.C.s1 * n] = from_f32<TC>(acc[i][j][r] * d.scale + bv);
      }
  }
}

// ---------------------------------------------------------------------------------------
// Softmax weights from the layout of the forward kernels, alpha_f[b][k][cl][head][n] (pitch Np, gpad
// members per group), to token-major alpha[b,c,n,head].  One thread per output element.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_alpha_token_major(long total, int Cin, int N, int heads, int g, int gpad,
                                                           int G, int Np, const float* __restrict__ alpha_f,
                                                           float* __restrict__ alpha) {
  const long idx = (long)blockIdx.x * 256 + threadIdx.x;      // ((b * Cin + c) * N + n) * heads + a
  if (idx >= total) return;
  const int a = (int)(idx % heads);
  long t = idx / heads;
  const int n = (int)(t % N);
  t /= N;
  const int c = (int)(t % Cin), b = (int)(t / Cin);
  const int k = c / g, cl = c % g;
  alpha[idx] = alpha_f[((((size_t)b * G + k) * gpad + cl) * heads + a) * Np + n];
}

// ---------------------------------------------------------------------------------------
// Per-head weighted token sums, bf16, D % 4 == 0:
//   u[b,k,n,a,:] = sum_{c in group k} alpha[b,c,n,a] * z[b,c,n,:]
// grid (N, G, B), block 256: a thread owns 4 adjacent columns (and every 1024th after them) and
// keeps one fp32 sum per head; the group's weights for this patch sit in LDS.  Bound by the read
// of z (2 D bytes per token) and the write of u.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_head_sums_bf16(int Cin, int N, int D, int heads, int g,
                                                        const float* __restrict__ alpha, const bf16* __restrict__ z,
                                                        bf16* __restrict__ u) {
  extern __shared__ __attribute__((aligned(16))) float al[];      // [gk][16]: the weights of one block of 16 heads
  const int n = blockIdx.x, k = blockIdx.y, b = blockIdx.z, G = gridDim.y;
  const int c0 = k * g, gk = min(g, Cin - c0);
  const size_t cstride = (size_t)N * D;
  for (int a0 = 0; a0 < heads; a0 += 16) {                        // more than 16 heads: z is walked once per block
    __syncthreads();
    for (int idx = threadIdx.x; idx < gk * 16; idx += 256) {
      const int cl = idx >> 4, a = a0 + (idx & 15);
      al[idx] = a < heads ? alpha[(((size_t)b * Cin + c0 + cl) * N + n) * heads + a] : 0.f;
    }
    __syncthreads();
    for (int d0 = threadIdx.x * 4; d0 < D; d0 += 1024) {
      const bf16* zp = z + (((size_t)b * Cin + c0) * N + n) * D + d0;
      float acc[16][4];
#pragma unroll
      for (int a = 0; a < 16; ++a)
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[a][e] = 0.f;
      int cl = 0;
      for (; cl + 4 <= gk; cl += 4) {
        bf16x4 zv[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) zv[i] = *reinterpret_cast<const bf16x4*>(zp + (size_t)(cl + i) * cstride);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const f32x4* ar = reinterpret_cast<const f32x4*>(al + (cl + i) * 16);
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const f32x4 av = ar[q];
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
              for (int e = 0; e < 4; ++e) acc[q * 4 + a][e] += av[a] * (float)zv[i][e];
          }
        }
      }
      for (; cl < gk; ++cl) {
        const bf16x4 zv = *reinterpret_cast<const bf16x4*>(zp + (size_t)cl * cstride);
#pragma unroll
        for (int a = 0; a < 16; ++a)
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[a][e] += al[cl * 16 + a] * (float)zv[e];
      }
      bf16* up = u + ((((size_t)b * G + k) * N + n) * heads + a0) * D + d0;
#pragma unroll
      for (int a = 0; a < 16; ++a)
        if (a0 + a < heads) {
          bf16x4 o;
#pragma unroll
          for (int e = 0; e < 4; ++e) o[e] = (bf16)acc[a][e];
          *reinterpret_cast<bf16x4*>(up + (size_t)a * D) = o;
        }
    }
  }
}

// ---------------------------------------------------------------------------------------
// d alpha and the softmax Jacobian in one kernel (bf16, D % 32 == 0, group size <= 16 MT):
//   dalpha[c,a] = w[b,k,n,a,:] . z[b,c,n,:]            (16x16x32 MFMA: 16 members x 16 heads per block)
//   ds[c,a]     = alpha[c,a] * (dalpha[c,a] - sum_c' alpha[c',a] dalpha[c',a])
// One wavefront per (b, k, n): its A fragments are 16 member rows of z (64 contiguous bytes per row and
// step), its B fragments the head rows of w at this patch.  Accumulator block: lane holds head lane % 16,
// members 4 (lane / 16) + 0..3 of the tile.  grid ceil(B G N / 4), block 256.  Heads beyond 16 take
// further passes.  ds is written token-major [B,Cin,N,heads] like alpha.
// ---------------------------------------------------------------------------------------
template <int MT>
__global__ __launch_bounds__(256) void k_dalpha_softmax_mfma(long items, int Cin, int N, int D, int heads, int g,
                                                             int G, const bf16* __restrict__ z,
                                                             const bf16* __restrict__ w,
                                                             const float* __restrict__ alpha,
                                                             float* __restrict__ ds) {
  const long item = (long)blockIdx.x * 4 + (threadIdx.x >> 6);     // (b * G + k) * N + n
  if (item >= items) return;
  const int lane = threadIdx.x & 63, l16 = lane & 15, lq = lane >> 4;
  const int n = (int)(item % N);
  const int k = (int)((item / N) % G), b = (int)(item / ((long)N * G));
  const int c0 = k * g, gk = min(g, Cin - c0);
  const size_t cstride = (size_t)N * D;
  const bf16* zb = z + (((size_t)b * Cin + c0) * N + n) * D + lq * 8;
  for (int a0 = 0; a0 < heads; a0 += 16) {
    const int head = min(a0 + l16, heads - 1);
    const bf16* wr = w + ((size_t)item * heads + head) * D + lq * 8;
    const bf16* zr[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) zr[mt] = zb + (size_t)min(mt * 16 + l16, gk - 1) * cstride;
    f32x4 acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int t = 0; t < D; t += 128) {                             // four steps of 32 per trip, loads first
      bf16x8 wf[4], zf[MT][4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int tt = min(t + q * 32, D - 32);
        wf[q] = *reinterpret_cast<const bf16x8*>(wr + tt);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) zf[mt][q] = *reinterpret_cast<const bf16x8*>(zr[mt] + tt);
      }
#pragma unroll
      for (int q = 0; q < 4; ++q)
        if (t + q * 32 < D) {
#pragma unroll
          for (int mt = 0; mt < MT; ++mt)
            acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(zf[mt][q], wf[q], acc[mt], 0, 0, 0);
        }
    }
    // softmax Jacobian over the members (registers and the four lane groups of a head)
    float al[MT][4];
    float dot = 0.f;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int cl = mt * 16 + lq * 4 + r;
        al[mt][r] = (cl < gk && a0 + l16 < heads)
                        ? alpha[(((size_t)b * Cin + c0 + cl) * N + n) * heads + a0 + l16] : 0.f;
        dot += al[mt][r] * acc[mt][r];
      }
    dot += __shfl_xor(dot, 16, kWave);
    dot += __shfl_xor(dot, 32, kWave);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int cl = mt * 16 + lq * 4 + r;
        if (cl < gk && a0 + l16 < heads)
          ds[(((size_t)b * Cin + c0 + cl) * N + n) * heads + a0 + l16] = al[mt][r] * (acc[mt][r] - dot);
      }
  }
}

// ---------------------------------------------------------------------------------------
// The same for groups of any size (the flat single-layer baseline has one group of all channels), bf16, D % 32 == 0:
// one block of four wavefronts per (b, k, n).  The wavefronts take the tiles of 16 members in turn (16x16x32 MFMA as
// above, the head rows of w re-read from L1 per tile) and leave d alpha of the whole group in LDS; then the sums
// sum_c alpha dalpha per head are formed in a fixed order and ds is written.  grid B G N, block 256, dynamic LDS
// (16 ceil(g/16) + 17) * 16 floats.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_dalpha_softmax_group(int Cin, int N, int D, int heads, int g, int G,
                                                              const bf16* __restrict__ z, const bf16* __restrict__ w,
                                                              const float* __restrict__ alpha, float* __restrict__ ds) {
  extern __shared__ __attribute__((aligned(16))) float sm[];       // da[16 ntile][16], red[16][16], dot[16]
  const long item = blockIdx.x;                                    // (b * G + k) * N + n
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, l16 = lane & 15, lq = lane >> 4;
  const int n = (int)(item % N);
  const int k = (int)((item / N) % G), b = (int)(item / ((long)N * G));
  const int c0 = k * g, gk = min(g, Cin - c0);
  const int ntile = (gk + 15) / 16;
  float* da = sm;
  float* red = sm + ntile * 256;
  float* dot = red + 256;
  const size_t cstride = (size_t)N * D;
  const bf16* zb = z + (((size_t)b * Cin + c0) * N + n) * D + lq * 8;
  const float* ab = alpha + (((size_t)b * Cin + c0) * N + n) * heads;   // member cl: + cl * N * heads
  float* dsb = ds + (((size_t)b * Cin + c0) * N + n) * heads;
  const size_t astride = (size_t)N * heads;
  for (int a0 = 0; a0 < heads; a0 += 16) {
    const int head = min(a0 + l16, heads - 1);
    const bf16* wr = w + ((size_t)item * heads + head) * D + lq * 8;
    for (int tile = wave; tile < ntile; tile += 4) {
      const bf16* zr = zb + (size_t)min(tile * 16 + l16, gk - 1) * cstride;
      f32x4 acc = {0.f, 0.f, 0.f, 0.f};
      for (int t = 0; t < D; t += 128) {                           // four steps of 32 per trip, loads first
        bf16x8 wf[4], zf[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int tt = min(t + q * 32, D - 32);
          wf[q] = *reinterpret_cast<const bf16x8*>(wr + tt);
          zf[q] = *reinterpret_cast<const bf16x8*>(zr + tt);
        }
#pragma unroll
        for (int q = 0; q < 4; ++q)
          if (t + q * 32 < D) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(zf[q], wf[q], acc, 0, 0, 0);
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) da[(tile * 16 + lq * 4 + r) * 16 + l16] = acc[r];   // lane: head l16, members 4 lq + r
    }
    __syncthreads();
    {
      const int hd = threadIdx.x & 15, part = threadIdx.x >> 4;
      float p = 0.f;
      if (a0 + hd < heads)
        for (int cl = part; cl < gk; cl += 16) p += ab[(size_t)cl * astride + a0 + hd] * da[cl * 16 + hd];
      red[part * 16 + hd] = p;
    }
    __syncthreads();
    if (threadIdx.x < 16) {
      float sum = 0.f;
#pragma unroll
      for (int part = 0; part < 16; ++part) sum += red[part * 16 + threadIdx.x];
      dot[threadIdx.x] = sum;
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < gk * 16; idx += 256) {
      const int cl = idx >> 4, hd = idx & 15;
      if (a0 + hd < heads)
        dsb[(size_t)cl * astride + a0 + hd] = ab[(size_t)cl * astride + a0 + hd] * (da[idx] - dot[hd]);
    }
    __syncthreads();                                               // the next block of heads overwrites da
  }
}

// ---------------------------------------------------------------------------------------
// Gradient at the input tokens and the key-path sums, bf16, heads <= 16, D % 4 == 0:
//   dz[b,c,n,:]   = sum_a alpha[b,c,n,a] * w[b,k,n,a,:] + ds[b,c,n,a] * M[k][a][:]
//   rpart[b,k,t][a][:] = sum over the PT patches of tile t and the members c of  ds[b,c,n,a] * z[b,c,n,:]
// grid (n_tiles * ceil(D/1024), G, B), n_tiles = ceil(N/PT), block 256: a thread owns 4 adjacent columns, keeps the 16 rows
// of M and (per patch) of w for them in registers, and walks the members.  The softmax weights and ds of
// the whole tile of PT patches sit in LDS (dynamic, 2 * PT * g * 16 floats).  The partial sums are added up in a fixed
// order by k_sum_partials.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_dz_rpart_bf16(int Cin, int N, int D, int heads, int g, int n_tiles, int PT,
                                                       const float* __restrict__ alpha, const float* __restrict__ ds,
                                                       const bf16* __restrict__ z, const bf16* __restrict__ w,
                                                       const bf16* __restrict__ Mb, bf16* __restrict__ dz,
                                                       float* __restrict__ rpart) {
  extern __shared__ __attribute__((aligned(16))) float sm[];       // al[PT][g][16], then dsv[PT][g][16]
  const int tile = blockIdx.x % n_tiles, cb = blockIdx.x / n_tiles;
  const int k = blockIdx.y, b = blockIdx.z, G = gridDim.y;
  const int c0 = k * g, gk = min(g, Cin - c0);
  const int n0 = tile * PT, np = min(PT, N - n0);
  float* al = sm;
  float* dsv = sm + PT * g * 16;
  for (int idx = threadIdx.x; idx < np * gk * 16; idx += 256) {
    const int a = idx & 15, cl = (idx >> 4) % gk, pi = (idx >> 4) / gk;
    const size_t src = (((size_t)b * Cin + c0 + cl) * N + n0 + pi) * heads + a;
    al[(pi * g + cl) * 16 + a] = a < heads ? alpha[src] : 0.f;
    dsv[(pi * g + cl) * 16 + a] = a < heads ? ds[src] : 0.f;
  }
  __syncthreads();
  const int d0 = cb * 1024 + threadIdx.x * 4;
  if (d0 >= D) return;
  float mr[16][4], racc[16][4];
#pragma unroll
  for (int a = 0; a < 16; ++a) {
    bf16x4 mv = {};
    if (a < heads) mv = *reinterpret_cast<const bf16x4*>(Mb + ((size_t)k * heads + a) * D + d0);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      mr[a][e] = (float)mv[e];
      racc[a][e] = 0.f;
    }
  }
  const size_t cstride = (size_t)N * D;
  for (int pi = 0; pi < np; ++pi) {
    const int n = n0 + pi;
    float wr[16][4];
    const bf16* wp = w + ((((size_t)b * G + k) * N + n) * heads) * D + d0;
#pragma unroll
    for (int a = 0; a < 16; ++a) {
      bf16x4 wv = {};
      if (a < heads) wv = *reinterpret_cast<const bf16x4*>(wp + (size_t)a * D);
#pragma unroll
      for (int e = 0; e < 4; ++e) wr[a][e] = (float)wv[e];
    }
    const bf16* zp = z + (((size_t)b * Cin + c0) * N + n) * D + d0;
    bf16* dzp = dz + (((size_t)b * Cin + c0) * N + n) * D + d0;
    bf16x4 znext = *reinterpret_cast<const bf16x4*>(zp);
    for (int cl = 0; cl < gk; ++cl) {
      const bf16x4 zv = znext;
      if (cl + 1 < gk) znext = *reinterpret_cast<const bf16x4*>(zp + (size_t)(cl + 1) * cstride);
      const f32x4* ar = reinterpret_cast<const f32x4*>(al + (pi * g + cl) * 16);
      const f32x4* dr = reinterpret_cast<const f32x4*>(dsv + (pi * g + cl) * 16);
      float acc[4] = {0.f, 0.f, 0.f, 0.f};
      float zf[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) zf[e] = (float)zv[e];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const f32x4 av = ar[q], dv = dr[q];
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            acc[e] += av[a] * wr[q * 4 + a][e] + dv[a] * mr[q * 4 + a][e];
            racc[q * 4 + a][e] += dv[a] * zf[e];
          }
      }
      bf16x4 o;
#pragma unroll
      for (int e = 0; e < 4; ++e) o[e] = (bf16)acc[e];
      *reinterpret_cast<bf16x4*>(dzp + (size_t)cl * cstride) = o;
    }
  }
  float* rp = rpart + ((((size_t)b * G + k) * n_tiles + tile) * heads) * D + d0;
#pragma unroll
  for (int a = 0; a < 16; ++a)
    if (a < heads) *reinterpret_cast<f32x4*>(rp + (size_t)a * D) = f32x4{racc[a][0], racc[a][1], racc[a][2], racc[a][3]};
}

// ---------------------------------------------------------------------------------------
// The same two results as two kernels for D % 256 == 0 (bf16, heads <= 32): the token gradients on MFMA
// (reads w, writes dz) and the key-path sums on the vector ALUs (reads z); neither needs the other's stream.
//
// k_dz_mfma:  dz[b, c0 + m, n, :] = [alpha | ds](m, 0..31) . [w ; M](0..31, :)   one 32x32x16 product per 32
// columns, alpha and ds split in two bf16 parts each (hi + lo) so that the fp32 softmax weights lose nothing.
// A wavefront owns 256 columns, lane l the four columns 4 l .. 4 l + 3 of them: it loads the 16 head rows of
// w (per patch) and of M (once) for its columns, packs them into 8-head chunks and swaps one chunk per column
// with lane l ^ 32, which gives both half-wavefronts the B fragments (column, heads 8 (l / 32) ..) of the eight
// 32-column tiles {4 (j + 32 half) + e : j < 32}.  Accumulator block (half, e): lane holds column
// 4 (l % 32 + 32 half) + e, register r member 8 (r / 4) + 4 (l / 32) + r % 4: four blocks give a lane four
// adjacent columns of a member row (one 8-byte store).  The A fragments (member row, 8 heads) come straight
// from the token-major alpha / ds.  grid (n_tiles * ceil(D/1024), G, B), block 256, pt patches per block.
// ---------------------------------------------------------------------------------------
typedef __attribute__((ext_vector_type(4))) int i32x4;

// B fragments of the eight column tiles from 16 rows (heads) of a [heads][D] bf16 matrix at this lane's 4 columns.
template <bool LAST_USE = false>   // LAST_USE: streaming loads (the rows are not needed in the caches afterwards)
__device__ __forceinline__ void head_row_frags(const bf16* __restrict__ base, int D, int heads, int lhi,
                                               bf16x8 (&frag)[2][4]) {
  bf16x4 rows[16];
#pragma unroll
  for (int a = 0; a < 16; ++a) {
    rows[a] = bf16x4{};
    if (a < heads) {                                               // heads: rows that exist from base on
      const bf16x4* src = reinterpret_cast<const bf16x4*>(base + (size_t)a * D);
      rows[a] = LAST_USE ? __builtin_nontemporal_load(src) : *src;
    }
  }
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    bf16x8 c0, c1;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      c0[i] = rows[i][e];
      c1[i] = rows[8 + i][e];
    }
    const i32x4 v0 = __builtin_bit_cast(i32x4, c0), v1 = __builtin_bit_cast(i32x4, c1);
    i32x4 own, snd, rcv;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      own[q] = lhi ? v1[q] : v0[q];                      // the chunk this half-wavefront multiplies for its own columns
      snd[q] = lhi ? v0[q] : v1[q];                      // the chunk the other half needs for these columns
      rcv[q] = __shfl_xor(snd[q], 32, kWave);
    }
    const bf16x8 o8 = __builtin_bit_cast(bf16x8, own), r8 = __builtin_bit_cast(bf16x8, rcv);
    frag[0][e] = lhi ? r8 : o8;                          // tile of the lower half's columns
    frag[1][e] = lhi ? o8 : r8;                          // tile of the upper half's columns
  }
}

__device__ __forceinline__ void split_bf16(const f32x4& x0, const f32x4& x1, bf16x8& hi, bf16x8& lo) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    hi[i] = (bf16)x0[i];
    lo[i] = (bf16)(x0[i] - (float)hi[i]);
    hi[4 + i] = (bf16)x1[i];
    lo[4 + i] = (bf16)(x1[i] - (float)hi[4 + i]);
  }
}

template <int HB>   // blocks of 16 heads (heads <= 16 HB): the contraction runs over 2 HB steps of 16
__global__ __launch_bounds__(256, 3 - HB) void k_dz_mfma(int Cin, int N, int D, int heads, int g, int n_tiles, int pt,
                                                         const float* __restrict__ alpha, const float* __restrict__ ds,
                                                         const bf16* __restrict__ w, const bf16* __restrict__ Mb,
                                                         bf16* __restrict__ dz) {
  const int tile = blockIdx.x % n_tiles, cb = blockIdx.x / n_tiles;
  const int k = blockIdx.y, b = blockIdx.z, G = gridDim.y;
  const int c0 = k * g, gk = min(g, Cin - c0);
  const int n0 = tile * pt, np = min(pt, N - n0);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, l32 = lane & 31, lhi = lane >> 5;
  const int col0 = cb * 1024 + wave * 256;
  if (col0 >= D) return;
  const int d0 = col0 + 4 * lane;
  bf16x8 mfrag[HB][2][4];
#pragma unroll
  for (int hb = 0; hb < HB; ++hb)
    head_row_frags(Mb + ((size_t)k * heads + 16 * hb) * D + d0, D, heads - 16 * hb, lhi, mfrag[hb]);
  const size_t cstride = (size_t)N * D;
  const f32x4 z4 = {0.f, 0.f, 0.f, 0.f};
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  const bool h8 = heads % 8 == 0;                        // then a lane's 8 heads are two aligned 16-byte loads
  for (int pi = 0; pi < np; ++pi) {
    const int n = n0 + pi;
    bf16x8 wfrag[HB][2][4];
#pragma unroll
    for (int hb = 0; hb < HB; ++hb)
      head_row_frags(w + ((((size_t)b * G + k) * N + n) * heads + 16 * hb) * D + d0, D, heads - 16 * hb, lhi, wfrag[hb]);
    for (int m0 = 0; m0 < gk; m0 += 32) {
      const int row = m0 + l32;
      bf16x8 ahi[HB], alo[HB], dhi[HB], dlo[HB];
#pragma unroll
      for (int hb = 0; hb < HB; ++hb) {
        const int h0 = 16 * hb + 8 * lhi;                // this lane's 8 heads of the block
        const size_t src = (((size_t)b * Cin + c0 + min(row, gk - 1)) * N + n) * heads + h0;
        f32x4 a0 = z4, a1 = z4, e0 = z4, e1 = z4;
        if (row < gk) {
          if (h8) {
            if (h0 < heads) {
              a0 = *reinterpret_cast<const f32x4*>(alpha + src);
              a1 = *reinterpret_cast<const f32x4*>(alpha + src + 4);
              e0 = *reinterpret_cast<const f32x4*>(ds + src);
              e1 = *reinterpret_cast<const f32x4*>(ds + src + 4);
            }
          } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              if (h0 + i < heads) { a0[i] = alpha[src + i]; e0[i] = ds[src + i]; }
              if (h0 + 4 + i < heads) { a1[i] = alpha[src + 4 + i]; e1[i] = ds[src + 4 + i]; }
            }
          }
        }
        split_bf16(a0, a1, ahi[hb], alo[hb]);
        split_bf16(e0, e1, dhi[hb], dlo[hb]);
      }
      auto tiles_of_half = [&](int half) {
        f32x16 acc[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          acc[e] = zero;
#pragma unroll
          for (int hb = 0; hb < HB; ++hb) {
            acc[e] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ahi[hb], wfrag[hb][half][e], acc[e], 0, 0, 0);
            acc[e] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(alo[hb], wfrag[hb][half][e], acc[e], 0, 0, 0);
            acc[e] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dhi[hb], mfrag[hb][half][e], acc[e], 0, 0, 0);
            acc[e] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dlo[hb], mfrag[hb][half][e], acc[e], 0, 0, 0);
          }
        }
        bf16* dzp = dz + (((size_t)b * Cin + c0) * N + n) * D + col0 + 4 * (l32 + 32 * half);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int m = m0 + 8 * (r >> 2) + 4 * lhi + (r & 3);
          if (m < gk) {
            bf16x4 o;
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] = (bf16)acc[e][r];
            *reinterpret_cast<bf16x4*>(dzp + (size_t)m * cstride) = o;
          }
        }
      };
      tiles_of_half(0);
      tiles_of_half(1);
    }
  }
}

// ---------------------------------------------------------------------------------------
// The whole reverse step at the tokens of one level in one kernel (bf16, heads <= 16, D % 256 == 0, D <= 1024 CB,
// group size <= 16 MT <= 32), so that a patch's token rows and its w rows are fetched from HBM once (their second
// use, a few microseconds later in the same workgroup, finds them in L2) and ds never leaves the compute unit:
//   ds as in k_dalpha_softmax_mfma;  rpart[b,k,t][a][:] = sum over the pt patches of tile t and the members c of
//   ds[b,c,n,a] * z[b,c,n,:]  (the partial sums k_sum_partials adds up);  dz as in k_dz_mfma.
// grid (n_tiles, G, B), block 512, PP patches (one) per round of barriers:
//   d alpha   all eight wavefronts, each an eighth of D; the partial 16x16 blocks meet in LDS in a fixed order, the
//             first PP wavefronts apply the Jacobian (one patch each) and leave the softmax weights and ds in LDS;
//   sums      wavefronts 0..3, wavefront w columns 256 w .. 256 w + 255 (of each block of 1024 columns): ds^T (heads x 32 members, split in two
//             bf16 parts) times the 32 member rows on 16x16x32 MFMA; a lane reads 8 members x 8 adjacent columns
//             (16 bytes per row) and transposes them in registers, which gives it the B fragments (column
//             8 (lane % 16) + j, members 8 (lane / 16) ..) of eight products j = 0..7; accumulator (half, j): lane
//             holds column 128 half + 8 (lane % 16) + j, heads 4 (lane / 16) + r;
//   dz        wavefronts 4..7, wavefront 4 + w the same columns: the body of k_dz_mfma, A fragments from LDS.
// The two roles are separate loops (same barriers), so neither carries the other's accumulators.
// ---------------------------------------------------------------------------------------
template <int MT, int CB>   // CB: blocks of 1024 columns (D <= 1024 CB)
__global__ __launch_bounds__(512) void k_tokens_backward_fused(int Cin, int N, int D, int heads, int g, int pt,
                                                               const bf16* __restrict__ z, const bf16* __restrict__ w,
                                                               const float* __restrict__ alpha,
                                                               const bf16* __restrict__ Mb, bf16* __restrict__ dz,
                                                               float* __restrict__ rpart) {
  constexpr int PP = 1;                                            // patches per round of barriers (2: no faster)
  __shared__ f32x4 part[8][PP][MT][64];
  __shared__ float dsv[2][PP][32][17];                             // [round parity][patch][member][head], padded rows
  __shared__ float alv[2][PP][32][17];                             // the softmax weights, same layout
  const int tile = blockIdx.x, n_tiles = gridDim.x, k = blockIdx.y, b = blockIdx.z, G = gridDim.y;
  const int c0 = k * g, gk = min(g, Cin - c0);
  const int n0 = tile * pt, np = min(pt, N - n0);
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int l16 = lane & 15, lq = lane >> 4, l32 = lane & 31, lhi = lane >> 5;
  const size_t cstride = (size_t)N * D;
  const int kq = D / 8;                                            // this wavefront's share of the contraction
  const int col0 = (wave & 3) * 256;                               // this wavefront's columns of the sums / of dz
  const int head = min(l16, heads - 1);
  const bf16* zg = z + (((size_t)b * Cin + c0) * N + n0) * D;      // member 0 of the group at the tile's first patch
  const size_t item0 = ((size_t)b * G + k) * N + n0;
  for (int i = threadIdx.x; i < 2 * PP * 32 * 17; i += 512) {      // members beyond 16 MT stay zero
    (&dsv[0][0][0][0])[i] = 0.f;
    (&alv[0][0][0][0])[i] = 0.f;
  }
  __syncthreads();

  // partial d alpha of patches pi .. pi + PP - 1 (past the tile's end: its last patch again, never used)
  auto dalpha_partial = [&](int pi) {
    const bf16* wr[PP];
    const bf16* zr[PP][MT];
    f32x4 acc[PP][MT];
#pragma unroll
    for (int q = 0; q < PP; ++q) {
      const int pq = min(pi + q, np - 1);
      wr[q] = w + ((item0 + pq) * heads + head) * D + wave * kq + lq * 8;
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        zr[q][mt] = zg + (size_t)pq * D + (size_t)min(mt * 16 + l16, gk - 1) * cstride + wave * kq + lq * 8;
        acc[q][mt] = f32x4{0.f, 0.f, 0.f, 0.f};
      }
    }
    for (int t = 0; t < kq; t += 128) {                            // four steps of 32 per trip, loads first
      bf16x8 wf[PP][4], zf[PP][MT][4];
#pragma unroll
      for (int q = 0; q < PP; ++q)
#pragma unroll
        for (int s4 = 0; s4 < 4; ++s4) {
          const int tt = min(t + s4 * 32, kq - 32);
          wf[q][s4] = *reinterpret_cast<const bf16x8*>(wr[q] + tt);
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) zf[q][mt][s4] = *reinterpret_cast<const bf16x8*>(zr[q][mt] + tt);
        }
#pragma unroll
      for (int q = 0; q < PP; ++q)
#pragma unroll
        for (int s4 = 0; s4 < 4; ++s4)
          if (t + s4 * 32 < kq) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
              acc[q][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(zf[q][mt][s4], wf[q][s4], acc[q][mt], 0, 0, 0);
          }
    }
#pragma unroll
    for (int q = 0; q < PP; ++q)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) part[wave][q][mt][lane] = acc[q][mt];
  };
  // Wavefront q < PP applies the Jacobian of patch pi + q.  It fetches the softmax weights of that patch before its
  // share of d alpha, so that they have arrived when the others wait (lane: head l16, members 4 lq + r of each tile).
  auto fetch_alpha = [&](int pi, float (&al)[MT][4]) {
    const int n = n0 + min(pi + wave, np - 1);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int cl = mt * 16 + lq * 4 + r;
        al[mt][r] = (cl < gk && l16 < heads) ? alpha[(((size_t)b * Cin + c0 + cl) * N + n) * heads + l16] : 0.f;
      }
  };
  auto jacobian = [&](int par, const float (&al)[MT][4]) {
    float da[MT][4];
    float dot = 0.f;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      f32x4 tot = part[0][wave][mt][lane];
#pragma unroll
      for (int v = 1; v < 8; ++v) tot += part[v][wave][mt][lane];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        da[mt][r] = tot[r];
        dot += al[mt][r] * tot[r];
      }
    }
    dot += __shfl_xor(dot, 16, kWave);
    dot += __shfl_xor(dot, 32, kWave);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int cl = mt * 16 + lq * 4 + r;
        dsv[par][wave][cl][l16] = al[mt][r] * (da[mt][r] - dot);   // 0 for padding members and heads
        alv[par][wave][cl][l16] = al[mt][r];
      }
  };
  // Per round of PP patches: every wavefront writes its partial blocks, barrier, wavefronts 0 .. PP-1 fill the tables
  // of the round's parity, barrier, the roles read them.  The next round writes the other parity, and `part` only
  // after every wavefront has passed the second barrier of this one.
  if (wave < 4) {
    f32x4 racc[CB][2][8];
#pragma unroll
    for (int cbk = 0; cbk < CB; ++cbk)
#pragma unroll
      for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int j = 0; j < 8; ++j) racc[cbk][h][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int pi = 0, par = 0; pi < np; pi += PP, par ^= 1) {
      float al[MT][4];
      if (wave < PP) fetch_alpha(pi, al);
      dalpha_partial(pi);
      __syncthreads();
      if (wave < PP) jacobian(par, al);
      __syncthreads();
      for (int q = 0; q < PP && pi + q < np; ++q) {
        f32x4 v0, v1;                                              // ds of head l16 at members 8 lq .. 8 lq + 7
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          v0[i] = dsv[par][q][8 * lq + i][l16];
          v1[i] = dsv[par][q][8 * lq + 4 + i][l16];
        }
        bf16x8 dhi, dlo;
        split_bf16(v0, v1, dhi, dlo);
#pragma unroll
        for (int cbk = 0; cbk < CB; ++cbk) {
          const int colc = col0 + 1024 * cbk;
          if (colc >= D) continue;
          const bf16* zc = zg + (size_t)(pi + q) * D + colc + 8 * l16;
          constexpr int HL = CB == 1 ? 2 : 1;                      // halves of 128 columns fetched together
#pragma unroll
          for (int h0 = 0; h0 < 2; h0 += HL) {
            bf16x8 rows[HL][8];
#pragma unroll
            for (int h = 0; h < HL; ++h)
#pragma unroll
              for (int i = 0; i < 8; ++i)
                rows[h][i] = __builtin_nontemporal_load(            // second and last use of the row
                    reinterpret_cast<const bf16x8*>(zc + (size_t)min(8 * lq + i, gk - 1) * cstride + 128 * (h0 + h)));
#pragma unroll
            for (int h = 0; h < HL; ++h)
#pragma unroll
              for (int j = 0; j < 8; ++j) {
                bf16x8 col;
#pragma unroll
                for (int i = 0; i < 8; ++i) col[i] = rows[h][i][j];
                racc[cbk][h0 + h][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(dhi, col, racc[cbk][h0 + h][j], 0, 0, 0);
                racc[cbk][h0 + h][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(dlo, col, racc[cbk][h0 + h][j], 0, 0, 0);
              }
          }
        }
      }
    }
#pragma unroll
    for (int cbk = 0; cbk < CB; ++cbk) {
      const int colc = col0 + 1024 * cbk;
      if (colc >= D) continue;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int a = 4 * lq + r;
        if (a < heads) {
          float* rp = rpart + ((((size_t)b * G + k) * n_tiles + tile) * heads + a) * D + colc + 8 * l16;
#pragma unroll
          for (int h = 0; h < 2; ++h) {
            *reinterpret_cast<f32x4*>(rp + 128 * h) =
                f32x4{racc[cbk][h][0][r], racc[cbk][h][1][r], racc[cbk][h][2][r], racc[cbk][h][3][r]};
            *reinterpret_cast<f32x4*>(rp + 128 * h + 4) =
                f32x4{racc[cbk][h][4][r], racc[cbk][h][5][r], racc[cbk][h][6][r], racc[cbk][h][7][r]};
          }
        }
      }
    }
  } else {
    const int d0c = col0 + 4 * lane;                               // this lane's 4 columns (of each column block)
    bf16x8 mfrag[CB][2][4];
#pragma unroll
    for (int cbk = 0; cbk < CB; ++cbk)
      if (col0 + 1024 * cbk < D)
        head_row_frags(Mb + ((size_t)k * heads) * D + d0c + 1024 * cbk, D, heads, lhi, mfrag[cbk]);
    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int pi = 0, par = 0; pi < np; pi += PP, par ^= 1) {
      dalpha_partial(pi);
      __syncthreads();
      __syncthreads();
      for (int q = 0; q < PP && pi + q < np; ++q) {
        f32x4 a0, a1, e0, e1;                                      // member row l32, heads 8 lhi .. 8 lhi + 7
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          a0[i] = alv[par][q][l32][8 * lhi + i];
          a1[i] = alv[par][q][l32][8 * lhi + 4 + i];
          e0[i] = dsv[par][q][l32][8 * lhi + i];
          e1[i] = dsv[par][q][l32][8 * lhi + 4 + i];
        }
        bf16x8 ahi, alo, ehi, elo;
        split_bf16(a0, a1, ahi, alo);
        split_bf16(e0, e1, ehi, elo);
#pragma unroll
        for (int cbk = 0; cbk < CB; ++cbk) {
          const int colc = col0 + 1024 * cbk;
          if (colc >= D) continue;
          bf16x8 wfrag[2][4];
          head_row_frags<true>(w + ((item0 + pi + q) * heads) * D + d0c + 1024 * cbk, D, heads, lhi, wfrag);
          auto tiles_of_half = [&](int half) {
            f32x16 acc[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              acc[e] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ahi, wfrag[half][e], zero, 0, 0, 0);
              acc[e] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(alo, wfrag[half][e], acc[e], 0, 0, 0);
              acc[e] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ehi, mfrag[cbk][half][e], acc[e], 0, 0, 0);
              acc[e] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(elo, mfrag[cbk][half][e], acc[e], 0, 0, 0);
            }
            bf16* dzp = dz + (((size_t)b * Cin + c0) * N + n0 + pi + q) * D + colc + 4 * (l32 + 32 * half);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const int m = 8 * (r >> 2) + 4 * lhi + (r & 3);
              if (m < gk) {
                bf16x4 o;
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = (bf16)acc[e][r];
                // streaming store: dz is not read again here, and the rows to come back from L2 are z's and w's
                __builtin_nontemporal_store(o, reinterpret_cast<bf16x4*>(dzp + (size_t)m * cstride));
              }
            }
          };
          tiles_of_half(0);
          tiles_of_half(1);
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------------------
// k_rpart_bf16:  rpart[b,k,t][a][:] = sum over the pt patches of tile t and the members c of ds[b,c,n,a] * z[b,c,n,:]
// grid (n_tiles * ceil(D/1024), G, B), block 256: a thread owns 4 adjacent columns and one fp32 sum per head;
// ds of the whole tile sits in LDS (dynamic, pt * g * 16 floats).
// ---------------------------------------------------------------------------------------
template <int HB>   // blocks of 16 heads, heads <= 16 HB
__global__ __launch_bounds__(256) void k_rpart_bf16(int Cin, int N, int D, int heads, int g, int n_tiles, int pt,
                                                    const float* __restrict__ ds, const bf16* __restrict__ z,
                                                    float* __restrict__ rpart) {
  extern __shared__ __attribute__((aligned(16))) float dsv[];      // [np * gk rows in (patch, member) order][16 heads]
  const int tile = blockIdx.x % n_tiles, cb = blockIdx.x / n_tiles;
  const int k = blockIdx.y, b = blockIdx.z, G = gridDim.y;
  const int c0 = k * g, gk = min(g, Cin - c0);
  const int n0 = tile * pt, np = min(pt, N - n0);
  const int rows = np * gk;
  const int d0 = cb * 1024 + threadIdx.x * 4;
#pragma unroll
  for (int hb = 0; hb < HB; ++hb) {                                // more than 16 heads: one pass over z per block of 16
    const int a0 = 16 * hb;
    if (HB > 1) __syncthreads();
    for (int idx = threadIdx.x; idx < rows * 16; idx += 256) {
      const int a = a0 + (idx & 15), cl = (idx >> 4) % gk, pi = (idx >> 4) / gk;
      dsv[idx] = a < heads ? ds[(((size_t)b * Cin + c0 + cl) * N + n0 + pi) * heads + a] : 0.f;
    }
    __syncthreads();
    if (d0 >= D) continue;
    float racc[16][4];
  #pragma unroll
    for (int a = 0; a < 16; ++a)
  #pragma unroll
      for (int e = 0; e < 4; ++e) racc[a][e] = 0.f;
    const size_t cstride = (size_t)N * D;
    const bf16* zb = z + (((size_t)b * Cin + c0) * N + n0) * D + d0;
    // the rows of the tile are walked eight at a time, the next eight already in flight while these are summed
    int pcl = 0, ppi = 0;                                  // (member, patch) of the next row to fetch
    bf16x4 cur[8], nxt[8];
    auto fetch = [&](bf16x4 (&buf)[8]) {
  #pragma unroll
      for (int i = 0; i < 8; ++i) {
        buf[i] = bf16x4{};
        if (ppi < np) buf[i] = *reinterpret_cast<const bf16x4*>(zb + (size_t)ppi * D + (size_t)pcl * cstride);
        if (++pcl == gk) { pcl = 0; ++ppi; }
      }
    };
    fetch(cur);
    for (int base = 0; base < rows; base += 8) {
      fetch(nxt);                                          // past the end: nothing is loaded
  #pragma unroll
      for (int i = 0; i < 8; ++i) {
        if (base + i < rows) {
          const f32x4* dr = reinterpret_cast<const f32x4*>(dsv + (base + i) * 16);
  #pragma unroll
          for (int q = 0; q < 4; ++q) {
            const f32x4 dv = dr[q];
  #pragma unroll
            for (int a = 0; a < 4; ++a)
  #pragma unroll
              for (int e = 0; e < 4; ++e) racc[q * 4 + a][e] += dv[a] * (float)cur[i][e];
          }
        }
      }
  #pragma unroll
      for (int i = 0; i < 8; ++i) cur[i] = nxt[i];
    }
    float* rp = rpart + ((((size_t)b * G + k) * n_tiles + tile) * heads + a0) * D + d0;
  #pragma unroll
    for (int a = 0; a < 16; ++a)
      if (a0 + a < heads) *reinterpret_cast<f32x4*>(rp + (size_t)a * D) = f32x4{racc[a][0], racc[a][1], racc[a][2], racc[a][3]};
  }
}

// ---------------------------------------------------------------------------------------
// k_rpart_mfma: the same partial sums on 16x16x32 MFMA for D % 256 == 0 (bf16, heads <= 16 HB), as in
// k_tokens_backward_fused: per patch and block of 32 members, ds^T (16 heads x 32 members, hi + lo bf16 parts) times
// the 32 member rows; a lane reads 8 members x 8 adjacent columns and transposes them in registers.
// grid (n_tiles * ceil(D/1024), G, B), block 256: wavefront w owns columns 1024 cb + 256 w .. + 255.  ds of the whole
// tile sits in LDS (dynamic, pt * g * 16 HB floats, rows in (patch, member) order).
// ---------------------------------------------------------------------------------------
template <int HB>
__global__ __launch_bounds__(256, 2) void k_rpart_mfma(int Cin, int N, int D, int heads, int g, int n_tiles, int pt,
                                                       const float* __restrict__ ds, const bf16* __restrict__ z,
                                                       float* __restrict__ rpart) {
  extern __shared__ __attribute__((aligned(16))) float dsv[];      // [np * gk rows][16 HB heads]
  constexpr int HP = 16 * HB;
  const int tile = blockIdx.x % n_tiles, cb = blockIdx.x / n_tiles;
  const int k = blockIdx.y, b = blockIdx.z, G = gridDim.y;
  const int c0 = k * g, gk = min(g, Cin - c0);
  const int n0 = tile * pt, np = min(pt, N - n0);
  const int rows = np * gk;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, l16 = lane & 15, lq = lane >> 4;
  const int col0 = cb * 1024 + wave * 256;
  for (int idx = threadIdx.x; idx < rows * HP; idx += 256) {
    const int a = idx % HP, cl = (idx / HP) % gk, pi = (idx / HP) / gk;
    dsv[idx] = a < heads ? ds[(((size_t)b * Cin + c0 + cl) * N + n0 + pi) * heads + a] : 0.f;
  }
  __syncthreads();
  if (col0 >= D) return;
  f32x4 racc[HB][2][8];
#pragma unroll
  for (int hb = 0; hb < HB; ++hb)
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int j = 0; j < 8; ++j) racc[hb][h][j] = f32x4{0.f, 0.f, 0.f, 0.f};
  const size_t cstride = (size_t)N * D;
  const bf16* zb = z + (((size_t)b * Cin + c0) * N + n0) * D + col0 + 8 * l16;
  for (int pi = 0; pi < np; ++pi)
    for (int m0 = 0; m0 < gk; m0 += 32) {                          // members m0 + 8 lq .. + 7 are this lane's
      bf16x8 dhi[HB], dlo[HB];
#pragma unroll
      for (int hb = 0; hb < HB; ++hb) {
        f32x4 v0, v1;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const int cl = m0 + 8 * lq + i;
          const float v = cl < gk ? dsv[(pi * gk + cl) * HP + 16 * hb + l16] : 0.f;
          if (i < 4) v0[i] = v; else v1[i - 4] = v;
        }
        split_bf16(v0, v1, dhi[hb], dlo[hb]);
      }
      bf16x8 zr[2][8];
#pragma unroll
      for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int i = 0; i < 8; ++i)
          zr[h][i] = *reinterpret_cast<const bf16x8*>(zb + (size_t)pi * D + (size_t)min(m0 + 8 * lq + i, gk - 1) * cstride +
                                                     128 * h);
#pragma unroll
      for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          bf16x8 col;
#pragma unroll
          for (int i = 0; i < 8; ++i) col[i] = zr[h][i][j];
#pragma unroll
          for (int hb = 0; hb < HB; ++hb) {
            racc[hb][h][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(dhi[hb], col, racc[hb][h][j], 0, 0, 0);
            racc[hb][h][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(dlo[hb], col, racc[hb][h][j], 0, 0, 0);
          }
        }
    }
#pragma unroll
  for (int hb = 0; hb < HB; ++hb)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int a = 16 * hb + 4 * lq + r;
      if (a < heads) {
        float* rp = rpart + ((((size_t)b * G + k) * n_tiles + tile) * heads + a) * D + col0 + 8 * l16;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          *reinterpret_cast<f32x4*>(rp + 128 * h) =
              f32x4{racc[hb][h][0][r], racc[hb][h][1][r], racc[hb][h][2][r], racc[hb][h][3][r]};
          *reinterpret_cast<f32x4*>(rp + 128 * h + 4) =
              f32x4{racc[hb][h][4][r], racc[hb][h][5][r], racc[hb][h][6][r], racc[hb][h][7][r]};
        }
      }
    }
}

// r[k][i] = sum_b sum_t rpart[b][k][t][i]   (i over heads * D), fixed order.  grid (ceil(per/64), G), block 1024:
// 64 adjacent i per block, the sixteen wavefronts take every sixteenth partial (four in flight each) and meet in LDS.
__global__ __launch_bounds__(1024) void k_sum_partials(int B, int G, int n_tiles, long per, const float* __restrict__ rpart,
                                                       float* __restrict__ r) {
  __shared__ float part[15][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const long i = (long)blockIdx.x * 64 + lane;
  const int k = blockIdx.y;
  float acc = 0.f;
  if (i < per)
    for (int b = 0; b < B; ++b) {
      const float* src = rpart + (((size_t)b * G + k) * n_tiles) * per + i;
      int t = wave;
      for (; t + 48 < n_tiles; t += 64) {
        const float v0 = src[(size_t)t * per], v1 = src[(size_t)(t + 16) * per], v2 = src[(size_t)(t + 32) * per],
                    v3 = src[(size_t)(t + 48) * per];
        acc += v0;
        acc += v1;
        acc += v2;
        acc += v3;
      }
      for (; t < n_tiles; t += 16) acc += src[(size_t)t * per];
    }
  if (wave > 0) part[wave - 1][lane] = acc;
  __syncthreads();
  if (wave == 0 && i < per) {
#pragma unroll
    for (int w = 0; w < 15; ++w) acc += part[w][lane];
    r[(size_t)k * per + i] = acc;
  }
}

}  // namespace dchag
