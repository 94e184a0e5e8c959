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
// grid (ceil(D/64), G), block 256: the four waves take every fourth row and meet in LDS in a fixed order.
// ---------------------------------------------------------------------------------------
template <typename T, typename TO>
__global__ __launch_bounds__(256) void k_colsum(int B, int D, RowBlocks rb, const T* __restrict__ X,
                                                TO* __restrict__ out) {
  __shared__ float part[3][64];
  const int k = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int i = blockIdx.x * 64 + lane;
  const int rows = rb.rows_of(k);
  float acc = 0.f;
  if (i < D)
    for (int b = 0; b < B; ++b) {
      const T* xb = X + (size_t)rb.first_row(b, k) * D + i;
      for (int r = wave; r < rows; r += 4) acc += to_f32(xb[(size_t)r * D]);
    }
  if (wave > 0) part[wave - 1][lane] = acc;
  __syncthreads();
  if (wave == 0 && i < D) out[(size_t)k * D + i] = from_f32<TO>(acc + part[0][lane] + part[1][lane] + part[2][lane]);
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

// dquery[k][j] = sum_i Wq[k][i][j] * dQ[k][i];  grid (ceil(D/256), G), block 256.
template <typename T>
__global__ __launch_bounds__(256) void k_query_input_grad(int D, const T* __restrict__ Wq,
                                                          const float* __restrict__ dQ, T* __restrict__ dquery) {
  const int k = blockIdx.y;
  const int j = blockIdx.x * 256 + threadIdx.x;
  if (j >= D) return;
  const T* w = Wq + (size_t)k * D * D + j;
  const float* dq = dQ + (size_t)k * D;
  float acc = 0.f;
  for (int i = 0; i < D; ++i) acc += to_f32(w[(size_t)i * D]) * dq[i];
  dquery[(size_t)k * D + j] = from_f32<T>(acc);
}

// ---------------------------------------------------------------------------------------
// Rank-one weight gradients:  out[k][i][j] = scale * rowv[k][i] * colv[k][i / rows_per_vec][j]
//   key weights:   rowv = projected query, colv = r[k][a][:], rows_per_vec = dh, scale = 1/sqrt(dh)
//   query weights: rowv = dQ, colv = the learned query, rows_per_vec = D
// grid (ceil(D/256), D, G), block 256.
// ---------------------------------------------------------------------------------------
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
// scatter of patch rows back into an image.  One thread per pixel.
// ---------------------------------------------------------------------------------------
template <typename T, bool TO_IMAGE>
__global__ __launch_bounds__(256) void k_patch_rows(long total, int H, int W, int p, T* __restrict__ img,
                                                    T* __restrict__ patches) {
  const long idx = (long)blockIdx.x * 256 + threadIdx.x;      // pixel index in [B*C, H, W]
  if (idx >= total) return;
  const int wx = (int)(idx % W);
  long t = idx / W;
  const int hy = (int)(t % H);
  const long bc = t / H;
  const int pw = W / p, pp = p * p;
  const int n = (hy / p) * pw + wx / p, kk = (hy % p) * p + wx % p;
  const size_t pi = ((size_t)bc * (H / p) * pw + n) * pp + kk;
  if (TO_IMAGE) img[idx] = patches[pi];
  else patches[pi] = img[idx];
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

}  // namespace dchag
