// Shape-generic kernels (any D, any group size, fp32 or bf16 storage, fp32 arithmetic).
// They are the whole fp32 path and the bf16 path's fallback for shapes the MFMA kernels
// do not tile.  Paper Section 2.1 (tokenization, cross-attention aggregation).
#pragma once
#include "dchag_dev.h"

namespace dchag {

// ---------------------------------------------------------------------------------------
// Q[k][i] = sum_j Wq[k][i][j] q[k][j] + bq[k][i]          (weight-only; one wave per row)
// grid (ceil(D/4), G), block 256
// ---------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void k_project_query(int D, const T* __restrict__ query,
                                                       const T* __restrict__ Wq, const T* __restrict__ bq,
                                                       float* __restrict__ Qp) {
  const int k = blockIdx.y;
  const int i = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (i >= D) return;
  const T* w = Wq + ((size_t)k * D + i) * D;
  const T* q = query + (size_t)k * D;
  float acc = 0.f;
  constexpr int V = 16 / sizeof(T);                       // elements per 16-byte load
  if (D % (kWave * V) == 0) {
    typedef __attribute__((ext_vector_type(V))) T vec;
    for (int j = lane * V; j < D; j += kWave * V) {
      const vec wv = *reinterpret_cast<const vec*>(w + j);
      const vec qv = *reinterpret_cast<const vec*>(q + j);
#pragma unroll
      for (int e = 0; e < V; ++e) acc += to_f32(wv[e]) * to_f32(qv[e]);
    }
  } else {
    for (int j = lane; j < D; j += kWave) acc += to_f32(w[j]) * to_f32(q[j]);
  }
  acc = wave_sum(acc);
  if (lane == 0) Qp[(size_t)k * D + i] = acc + (bq ? to_f32(bq[(size_t)k * D + i]) : 0.f);
}

// ---------------------------------------------------------------------------------------
// Query folded into the key weights (the key bias shifts every score of a softmax by the
// same amount and is dropped):
//   M[k][a][j] = (1/sqrt(dh)) * sum_{i in head a} Wk[k][i][j] * Q[k][i]
// so that the score of token z for head a is  z . M[k][a][:].
// grid (ceil(D/64), heads, G), block 256: 64 columns per block, the four wavefronts each sum a
// quarter of the head's rows and meet in LDS in a fixed order.  Writes fp32 and, when asked, a
// bf16 copy and a transposed fp32 copy [G][D][heads].
// ---------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void k_fold_query_into_key(int D, int heads, const T* __restrict__ Wk,
                                                             const float* __restrict__ Qp,
                                                             float* __restrict__ Mf, bf16* __restrict__ Mb,
                                                             float* __restrict__ MfT) {
  __shared__ float part[3][64];
  const int k = blockIdx.z, a = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int j = blockIdx.x * 64 + lane;
  const int dh = D / heads;
  const int i0 = (dh * wave) / 4, i1 = (dh * (wave + 1)) / 4;
  float acc = 0.f;
  if (j < D) {
    const T* w = Wk + ((size_t)k * D + (size_t)a * dh) * D + j;
    const float* q = Qp + (size_t)k * D + (size_t)a * dh;
#pragma unroll 8
    for (int i = i0; i < i1; ++i) acc += to_f32(w[(size_t)i * D]) * q[i];
  }
  if (wave > 0) part[wave - 1][lane] = acc;
  __syncthreads();
  if (wave == 0 && j < D) {
    acc = (acc + part[0][lane] + part[1][lane] + part[2][lane]) * rsqrtf((float)dh);
    const size_t o = ((size_t)k * heads + a) * D + j;
    Mf[o] = acc;
    if (Mb) Mb[o] = (bf16)acc;
    if (MfT) MfT[((size_t)k * D + j) * heads + a] = acc;   // transposed copy [G][D][heads]
  }
}

// ---------------------------------------------------------------------------------------
// Tokenizer: tokens[b,c,n,d] = sum_kk We[c][d][kk] * u[b,c,n][kk] + be[c][d] + ce[c][d]
// grid (ceil(N/TP), C, B), block 256; TP patches per block staged in LDS as fp32.
// ---------------------------------------------------------------------------------------
template <typename T, int TP>
__global__ __launch_bounds__(256) void k_tokenize_generic(int C, int H, int W, int p, int D,
                                                          const T* __restrict__ x, const T* __restrict__ We,
                                                          const T* __restrict__ be, const T* __restrict__ ce,
                                                          T* __restrict__ tokens) {
  extern __shared__ float u_lds[];  // [TP][pp]
  const int pp = p * p, pw = W / p, N = (H / p) * pw;
  const int n0 = blockIdx.x * TP, c = blockIdx.y, b = blockIdx.z;
  const T* img = x + ((size_t)b * C + c) * H * W;
  for (int idx = threadIdx.x; idx < TP * pp; idx += 256) {
    const int t = idx / pp, kk = idx % pp;
    const int n = n0 + t;
    float v = 0.f;
    if (n < N) {
      const int pi = n / pw, pj = n % pw, r = kk / p, s = kk % p;
      v = to_f32(img[(size_t)(pi * p + r) * W + pj * p + s]);
    }
    u_lds[idx] = v;
  }
  __syncthreads();
  for (int d = threadIdx.x; d < D; d += 256) {
    const T* w = We + ((size_t)c * D + d) * pp;
    float acc[TP];
#pragma unroll
    for (int t = 0; t < TP; ++t) acc[t] = 0.f;
    for (int kk = 0; kk < pp; ++kk) {
      const float wv = to_f32(w[kk]);
#pragma unroll
      for (int t = 0; t < TP; ++t) acc[t] += wv * u_lds[t * pp + kk];
    }
    float add = 0.f;
    if (be) add += to_f32(be[(size_t)c * D + d]);
    if (ce) add += to_f32(ce[(size_t)c * D + d]);
#pragma unroll
    for (int t = 0; t < TP; ++t)
      if (n0 + t < N) tokens[(((size_t)b * C + c) * N + n0 + t) * D + d] = from_f32<T>(acc[t] + add);
  }
}

// ---------------------------------------------------------------------------------------
// Batched projection  Y[r][o] = sum_j A[r][j] * Wt[k][o][j] + bias[k][o] (+ rowadd[r][o], r counted inside the
// batch item's row block: a per-row addend such as a positional embedding)   (64x64 tile, fp32 FMA)
// grid (ceil(D/64), ceil(max rows/64), B*G), block 256 (16x16 threads, 4x4 outputs each)
// ---------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void k_linear_generic(int D, RowBlocks rb, const T* __restrict__ A,
                                                        const T* __restrict__ Wt, const T* __restrict__ bias,
                                                        T* __restrict__ Y, const T* __restrict__ rowadd) {
  __shared__ float As[16][64 + 1];
  __shared__ float Ws[16][64 + 1];
  const int b = blockIdx.z / rb.G, k = blockIdx.z % rb.G;
  const int rows = rb.rows_of(k);
  const int r0 = blockIdx.y * 64, o0 = blockIdx.x * 64;
  if (r0 >= rows) return;
  const T* Ab = A + (size_t)rb.first_row(b, k) * D;
  T* Yb = Y + (size_t)rb.first_row(b, k) * D;
  const T* Wb = Wt + (size_t)k * D * D;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;
  for (int j0 = 0; j0 < D; j0 += 16) {
    for (int idx = threadIdx.x; idx < 64 * 16; idx += 256) {
      const int rr = idx >> 4, jj = idx & 15;
      const bool kin = (j0 + jj) < D;
      As[jj][rr] = (kin && r0 + rr < rows) ? to_f32(Ab[(size_t)(r0 + rr) * D + j0 + jj]) : 0.f;
      Ws[jj][rr] = (kin && o0 + rr < D) ? to_f32(Wb[(size_t)(o0 + rr) * D + j0 + jj]) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int jj = 0; jj < 16; ++jj) {
      float av[4], wv[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) av[i] = As[jj][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) wv[j] = Ws[jj][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += av[i] * wv[j];
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = r0 + ty * 4 + i;
    if (r >= rows) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int o = o0 + tx * 4 + j;
      if (o < D)
        Yb[(size_t)r * D + o] = from_f32<T>(acc[i][j] + (bias ? to_f32(bias[(size_t)k * D + o]) : 0.f) +
                                            (rowadd ? to_f32(rowadd[(size_t)r * D + o]) : 0.f));
    }
  }
}

// ---------------------------------------------------------------------------------------
// Scores through the folded key weights:  S[b,c,n,a] = z[b,c,n,:] . M[c / g][a][:]
// One wave per token; grid ceil(T/4), block 256.  HMAX bounds the heads a wave keeps in registers.
// ---------------------------------------------------------------------------------------
template <typename T, int HMAX>
__global__ __launch_bounds__(256) void k_scores_generic(long T_total, int Cin, int N, int D, int heads, int g,
                                                        const T* __restrict__ z, const float* __restrict__ Mf,
                                                        float* __restrict__ S) {
  const long tok = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (tok >= T_total) return;
  const int c = (int)((tok / N) % Cin);
  const int k = c / g;
  const T* zr = z + (size_t)tok * D;
  for (int a0 = 0; a0 < heads; a0 += HMAX) {
    float acc[HMAX];
#pragma unroll
    for (int a = 0; a < HMAX; ++a) acc[a] = 0.f;
    const float* m = Mf + ((size_t)k * heads + a0) * D;
    for (int j = lane; j < D; j += kWave) {
      const float zv = to_f32(zr[j]);
#pragma unroll
      for (int a = 0; a < HMAX; ++a)
        if (a0 + a < heads) acc[a] += zv * m[(size_t)a * D + j];
    }
#pragma unroll
    for (int a = 0; a < HMAX; ++a) {
      const float v = wave_sum(acc[a]);
      if (lane == 0 && a0 + a < heads) S[(size_t)tok * heads + a0 + a] = v;
    }
  }
}

// ---------------------------------------------------------------------------------------
// Softmax over the members of a group and the weighted sum of their values:
//   O[b,k,n,d] = sum_{c in S_k} softmax_c(S[b,c,n,a(d)]) * V[b,c,n,d]
// grid (N, G, B), block 256; one thread per output element (loop over D).
// ---------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void k_softmax_aggregate_generic(int Cin, int N, int D, int heads, int g,
                                                                   const float* __restrict__ S,
                                                                   const T* __restrict__ V, T* __restrict__ O) {
  const int n = blockIdx.x, k = blockIdx.y, b = blockIdx.z;
  const int G = gridDim.y;
  const int c0 = k * g;
  const int c1 = min(c0 + g, Cin);
  const int dh = D / heads;
  for (int d = threadIdx.x; d < D; d += 256) {
    const int a = d / dh;
    float mx = -INFINITY;
    for (int c = c0; c < c1; ++c) mx = fmaxf(mx, S[(((size_t)b * Cin + c) * N + n) * heads + a]);
    float den = 0.f, acc = 0.f;
    for (int c = c0; c < c1; ++c) {
      const size_t tok = ((size_t)b * Cin + c) * N + n;
      const float e = __expf(S[tok * heads + a] - mx);
      den += e;
      acc += e * to_f32(V[tok * D + d]);
    }
    O[(((size_t)b * G + k) * N + n) * D + d] = from_f32<T>(acc / den);
  }
}

// ---------------------------------------------------------------------------------------
// Linear partial-aggregation level (D-CHAG-L, paper Sections 3.2 and 3.3):
//   y[b,k,n,d] = sum_{cl < gk} w[k][cl][d] * z[b, k*g + cl, n, d] + bias[k][d]
// grid (ceil(N * D / V / 256), G, B), block 256; a thread owns V = 16 bytes of adjacent features of
// one (b, k, n) and walks the members of the group.  Bound by the HBM read of z.  Requires D % V == 0.
// ---------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void k_channel_mix(int Cin, int N, int D, int g, const T* __restrict__ z,
                                                     const T* __restrict__ w, const T* __restrict__ bias,
                                                     T* __restrict__ y) {
  constexpr int V = 16 / sizeof(T);
  typedef __attribute__((ext_vector_type(V))) T vec;
  const int dv_n = D / V;
  const long idx = (long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (long)N * dv_n) return;
  const int n = (int)(idx / dv_n), d0 = (int)(idx % dv_n) * V;
  const int k = blockIdx.y, b = blockIdx.z, G = gridDim.y;
  const int c0 = k * g, gk = min(g, Cin - c0);
  float acc[V];
#pragma unroll
  for (int e = 0; e < V; ++e) acc[e] = 0.f;
  const T* zp = z + (((size_t)b * Cin + c0) * N + n) * D + d0;
  const T* wp = w + (size_t)k * g * D + d0;
#pragma unroll 4
  for (int cl = 0; cl < gk; ++cl) {
    const vec zv = *reinterpret_cast<const vec*>(zp + (size_t)cl * N * D);
    const vec wv = *reinterpret_cast<const vec*>(wp + (size_t)cl * D);
#pragma unroll
    for (int e = 0; e < V; ++e) acc[e] += to_f32(wv[e]) * to_f32(zv[e]);
  }
  vec out;
  if (bias) {
    const vec bv = *reinterpret_cast<const vec*>(bias + (size_t)k * D + d0);
#pragma unroll
    for (int e = 0; e < V; ++e) acc[e] += to_f32(bv[e]);
  }
#pragma unroll
  for (int e = 0; e < V; ++e) out[e] = from_f32<T>(acc[e]);
  *reinterpret_cast<vec*>(y + (((size_t)b * G + k) * N + n) * D + d0) = out;
}

}  // namespace dchag
