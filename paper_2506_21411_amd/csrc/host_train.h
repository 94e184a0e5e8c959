// Host side of dchag_forward_folded and dchag_backward: workspace layout, level scheduler, launches.
// Included by dchag_api.hip inside its anonymous namespace (it uses that file's helpers).
//
// Both calls evaluate an attention level with the value projection behind the weighted sum:
//   alpha = softmax over the group of (z . M),  u_a = sum_c alpha[c,a] z[c],  o_a = Wv_a u_a + bv_a,
//   y = Wo o + bo.
// The backward call keeps alpha, u and o of every level in its workspace and then walks the levels
// in reverse (paper Section 3.3: the backward pass is local, the plain reverse of the forward).

// Per-level pieces that a forward sweep leaves behind for the reverse sweep.
struct KeptLevel {
  size_t qp, mf, alpha, u, o, y, total;
};

inline KeptLevel kept_level(dchag_dtype dt, int B, int Cin, int N, int D, int heads, int g, bool linear,
                            bool keep_y) {
  const int G = groups_of(Cin, g);
  const size_t es = elem_size(dt);
  KeptLevel w{};
  size_t off = 0;
  if (!linear) {
    w.qp = off; off += align_up((size_t)G * D * 4);
    w.mf = off; off += align_up((size_t)G * heads * D * 4);
    w.alpha = off; off += align_up((size_t)B * Cin * N * heads * 4);
    w.u = off; off += align_up((size_t)B * G * N * heads * D * es);
    w.o = off; off += align_up((size_t)B * G * N * D * es);
  }
  w.y = off;
  if (keep_y) off += align_up((size_t)B * G * N * D * es);
  w.total = off;
  return w;
}

struct FoldedWs {
  size_t tokens, ping, pong, level, total;
};

inline FoldedWs folded_ws(dchag_dtype dt, int B, int C, int N, int D, int heads, int n_levels,
                          const int32_t* group_sizes) {
  FoldedWs w{};
  const size_t es = elem_size(dt);
  size_t off = 0;
  w.tokens = off; off += align_up((size_t)B * C * N * D * es);
  int c_in = C;
  size_t lvl_max = 0, inter_max = 0;
  for (int l = 0; l < n_levels; ++l) {
    const int g = group_sizes[l];
    if (g < 1) return FoldedWs{};
    const size_t t = kept_level(dt, B, c_in, N, D, heads, g, false, false).total;
    if (t > lvl_max) lvl_max = t;
    c_in = groups_of(c_in, g);
    if (l + 1 < n_levels) {
      const size_t it = align_up((size_t)B * c_in * N * D * es);
      if (it > inter_max) inter_max = it;
    }
  }
  if (c_in != 1) return FoldedWs{};
  w.ping = off; off += inter_max;
  w.pong = off; off += inter_max;
  w.level = off; off += lvl_max;
  w.total = off;
  return w;
}

struct BackwardWs {
  size_t tokens, patches, kept[16], dz[2], dalpha, w, d_o, r, dq, total;
};

inline BackwardWs backward_ws(dchag_dtype dt, int B, int C, int N, int pp, int D, int heads, int n_levels,
                              const int32_t* group_sizes, const int32_t* kinds) {
  BackwardWs w{};
  const size_t es = elem_size(dt);
  size_t off = 0;
  w.tokens = off; off += align_up((size_t)B * C * N * D * es);
  w.patches = off; off += align_up((size_t)B * C * N * pp * es);
  int c_in = C;
  size_t dal = 0, wv = 0, dov = 0, rv = 0, dqv = 0, dz0 = 0, dz1 = 0;
  for (int l = 0; l < n_levels; ++l) {
    const int g = group_sizes[l];
    if (g < 1) return BackwardWs{};
    const int G = groups_of(c_in, g);
    const bool linear = kinds && kinds[l] == DCHAG_LEVEL_LINEAR;
    w.kept[l] = off;
    off += kept_level(dt, B, c_in, N, D, heads, g, linear, l + 1 < n_levels).total;
    const size_t dzb = align_up((size_t)B * c_in * N * D * es);
    if (l & 1) { if (dzb > dz1) dz1 = dzb; } else { if (dzb > dz0) dz0 = dzb; }
    if (!linear) {
      dal = std::max(dal, align_up((size_t)B * c_in * N * heads * 4));
      wv = std::max(wv, align_up((size_t)B * G * N * heads * D * es));
      dov = std::max(dov, align_up((size_t)B * G * N * D * es));
      rv = std::max(rv, align_up((size_t)G * heads * D * 4));
      dqv = std::max(dqv, align_up((size_t)G * D * 4));
    }
    c_in = G;
  }
  if (c_in != 1) return BackwardWs{};
  w.dz[0] = off; off += dz0;
  w.dz[1] = off; off += dz1;
  w.dalpha = off; off += dal;
  w.w = off; off += wv;
  w.d_o = off; off += dov;
  w.r = off; off += rv;
  w.dq = off; off += dqv;
  w.total = off;
  return w;
}

template <typename TA, typename TB, typename TC>
int launch_gemm(const GemmDesc& d, const TA* A, const TB* Bm, const TB* bias, TC* C, hipStream_t st) {
  const long batch = (long)(d.reduce_b ? 1 : d.nb) * d.nk * d.na;
  const long mt = (d.M + 63) / 64;
  if (batch > 65535 || mt > 65535 || d.M < 1 || d.N < 1) return DCHAG_ERR_SHAPE;
  k_gemm_generic<TA, TB, TC><<<dim3((d.N + 63) / 64, (unsigned)mt, (unsigned)batch), 256, 0, st>>>(d, A, Bm, bias, C);
  return launch_status();
}

// One attention level evaluated as  alpha -> u -> o -> y  (y skipped when zout is NULL).
template <typename T>
int folded_level_forward(int B, int Cin, int N, int D, int heads, const dchag_level* lv, const T* zin, T* zout,
                         float* Qp, float* Mf, float* alpha, T* u, T* o, hipStream_t st) {
  const int g = lv->group_size, G = groups_of(Cin, g), dh = D / heads;
  const T* Wv = static_cast<const T*>(lv->Wv);
  int rc;
  {
    StageTimer tm(DCHAG_STAGE_QUERY, st);
    k_project_query<T><<<dim3((D + 3) / 4, G), 256, 0, st>>>(D, static_cast<const T*>(lv->query),
                                                             static_cast<const T*>(lv->Wq),
                                                             static_cast<const T*>(lv->bq), Qp);
    if ((rc = launch_status())) return rc;
  }
  {
    StageTimer tm(DCHAG_STAGE_FOLD, st);
    k_fold_query_into_key<T><<<dim3((D + 63) / 64, heads, G), 256, 0, st>>>(D, heads, static_cast<const T*>(lv->Wk),
                                                                            Qp, Mf, nullptr, nullptr);
    if ((rc = launch_status())) return rc;
  }
  {
    StageTimer tm(DCHAG_STAGE_SCORES, st);
    const long T_total = (long)B * Cin * N;
    k_scores_generic<T, 8><<<dim3((unsigned)((T_total + 3) / 4)), 256, 0, st>>>(T_total, Cin, N, D, heads, g, zin,
                                                                               Mf, alpha);
    if ((rc = launch_status())) return rc;
    const long total = (long)B * G * N * heads;
    k_softmax_group<<<dim3((unsigned)((total + 255) / 256)), 256, 0, st>>>(Cin, N, heads, g, G, total, alpha);
    if ((rc = launch_status())) return rc;
  }
  {
    StageTimer tm(DCHAG_STAGE_HEAD_SUMS, st);
    k_head_sums<T, 16><<<dim3(N, G, B), 256, 0, st>>>(Cin, N, D, heads, g, alpha, zin, u);
    if ((rc = launch_status())) return rc;
  }
  {
    StageTimer tm(DCHAG_STAGE_HEAD_VPROJ, st);
    GemmDesc d{};
    d.M = N; d.N = dh; d.K = D;
    d.nb = B; d.nk = G; d.na = heads;
    d.A = {(long)G * N * heads * D, (long)N * heads * D, (long)D, (long)heads * D, 1};
    d.Bm = {0, (long)D * D, (long)dh * D, 1, (long)D};
    d.C = {(long)G * N * D, (long)N * D, (long)dh, (long)D, 1};
    d.bias_sk = D; d.bias_sa = dh;
    d.scale = 1.f;
    if ((rc = launch_gemm<T, T, T>(d, u, Wv, static_cast<const T*>(lv->bv), o, st))) return rc;
  }
  if (!zout) return DCHAG_OK;
  StageTimer tm(DCHAG_STAGE_OPROJ, st);
  RowBlocks rbo{G, G * N, N};
  return launch_linear<T>(B, D, rbo, o, static_cast<const T*>(lv->Wo), static_cast<const T*>(lv->bo), zout, st);
}

template <typename T>
int forward_folded_impl(dchag_dtype dt, int B, int C, int H, int W, int p, int D, int heads, const void* x,
                        const void* We, const void* be, const void* ce, int n_levels, const dchag_level* levels,
                        const int32_t* gs, void* out, unsigned char* ws, const FoldedWs& w, hipStream_t st) {
  const int N = (H / p) * (W / p);
  g_level = 0;
  int rc = dchag_tokenize(dt, B, C, H, W, p, D, x, We, be, ce, ws + w.tokens, st);
  if (rc) return rc;
  const T* zin = reinterpret_cast<const T*>(ws + w.tokens);
  int c_in = C;
  for (int l = 0; l < n_levels; ++l) {
    g_level = l + 1;
    T* zout = (l + 1 == n_levels) ? static_cast<T*>(out) : reinterpret_cast<T*>(ws + ((l & 1) ? w.pong : w.ping));
    if (levels[l].kind == DCHAG_LEVEL_LINEAR)
      rc = run_level_linear<T>(B, c_in, N, D, &levels[l], zin, zout, st);
    else {
      const KeptLevel kl = kept_level(dt, B, c_in, N, D, heads, gs[l], false, false);
      unsigned char* lw = ws + w.level;
      rc = folded_level_forward<T>(B, c_in, N, D, heads, &levels[l], zin, zout, reinterpret_cast<float*>(lw + kl.qp),
                                   reinterpret_cast<float*>(lw + kl.mf), reinterpret_cast<float*>(lw + kl.alpha),
                                   reinterpret_cast<T*>(lw + kl.u), reinterpret_cast<T*>(lw + kl.o), st);
    }
    if (rc) return rc;
    zin = zout;
    c_in = groups_of(c_in, gs[l]);
  }
  return DCHAG_OK;
}

template <typename T>
int colsum(int B, int D, RowBlocks rb, const T* X, T* out, hipStream_t st) {
  k_colsum<T, T><<<dim3((D + 63) / 64, rb.G), 256, 0, st>>>(B, D, rb, X, out);
  return launch_status();
}

// Reverse of one attention level.  dy is the gradient at the level's output [B,G,N,D]; dz receives the
// gradient at its input [B,Cin,N,D].
template <typename T>
int attention_level_backward(int B, int Cin, int N, int D, int heads, const dchag_level* lv,
                             const dchag_level_grads* gr, const T* zin, const T* dy, T* dz, const float* Qp,
                             const float* Mf, const float* alpha, const T* u, const T* o, float* dalpha, T* w,
                             T* d_o, float* r, float* dQ, hipStream_t st) {
  const int g = lv->group_size, G = groups_of(Cin, g), dh = D / heads;
  const T* Wv = static_cast<const T*>(lv->Wv);
  const T* Wo = static_cast<const T*>(lv->Wo);
  const RowBlocks rbo{G, G * N, N};
  const long sBG = (long)G * N * D, sG = (long)N * D;          // strides of a [B,G,N,D] tensor
  const long uB = (long)G * N * heads * D, uG = (long)N * heads * D;
  int rc;
  {
    StageTimer tm(DCHAG_STAGE_BWD_OPROJ, st);
    if (gr->dbo && (rc = colsum<T>(B, D, rbo, dy, static_cast<T*>(gr->dbo), st))) return rc;
    if (gr->dWo) {                                              // dWo[k][i][j] = sum_{b,n} dy[..,i] o[..,j]
      GemmDesc d{};
      d.M = D; d.N = D; d.K = N; d.nb = B; d.nk = G; d.na = 1; d.reduce_b = 1;
      d.A = {sBG, sG, 0, 1, (long)D};
      d.Bm = {sBG, sG, 0, (long)D, 1};
      d.C = {0, (long)D * D, 0, (long)D, 1};
      d.scale = 1.f;
      if ((rc = launch_gemm<T, T, T>(d, dy, o, nullptr, static_cast<T*>(gr->dWo), st))) return rc;
    }
    GemmDesc d{};                                               // d_o[.., j] = sum_i dy[.., i] Wo[k][i][j]
    d.M = N; d.N = D; d.K = D; d.nb = B; d.nk = G; d.na = 1;
    d.A = {sBG, sG, 0, (long)D, 1};
    d.Bm = {0, (long)D * D, 0, (long)D, 1};
    d.C = {sBG, sG, 0, (long)D, 1};
    d.scale = 1.f;
    if ((rc = launch_gemm<T, T, T>(d, dy, Wo, nullptr, d_o, st))) return rc;
  }
  {
    StageTimer tm(DCHAG_STAGE_BWD_VALUE, st);
    if (gr->dbv && (rc = colsum<T>(B, D, rbo, d_o, static_cast<T*>(gr->dbv), st))) return rc;
    if (gr->dWv) {                                              // dWv[k][a*dh+i][j] = sum_{b,n} d_o[.., a*dh+i] u[.., a, j]
      GemmDesc d{};
      d.M = dh; d.N = D; d.K = N; d.nb = B; d.nk = G; d.na = heads; d.reduce_b = 1;
      d.A = {sBG, sG, (long)dh, 1, (long)D};
      d.Bm = {uB, uG, (long)D, (long)heads * D, 1};
      d.C = {0, (long)D * D, (long)dh * D, (long)D, 1};
      d.scale = 1.f;
      if ((rc = launch_gemm<T, T, T>(d, d_o, u, nullptr, static_cast<T*>(gr->dWv), st))) return rc;
    }
    GemmDesc d{};                                               // w[.., a, j] = sum_i d_o[.., a*dh+i] Wv[k][a*dh+i][j]
    d.M = N; d.N = D; d.K = dh; d.nb = B; d.nk = G; d.na = heads;
    d.A = {sBG, sG, (long)dh, (long)D, 1};
    d.Bm = {0, (long)D * D, (long)dh * D, (long)D, 1};
    d.C = {uB, uG, (long)D, (long)heads * D, 1};
    d.scale = 1.f;
    if ((rc = launch_gemm<T, T, T>(d, d_o, Wv, nullptr, w, st))) return rc;
  }
  {
    StageTimer tm(DCHAG_STAGE_BWD_SOFTMAX, st);
    const long T_total = (long)B * Cin * N;
    k_dalpha<T><<<dim3((unsigned)((T_total + 3) / 4)), 256, 0, st>>>(T_total, Cin, N, D, heads, g, G, zin, w, dalpha);
    if ((rc = launch_status())) return rc;
    const long total = (long)B * G * N * heads;
    k_softmax_group_backward<<<dim3((unsigned)((total + 255) / 256)), 256, 0, st>>>(Cin, N, heads, g, G, total, alpha,
                                                                                   dalpha);
    if ((rc = launch_status())) return rc;
  }
  {
    StageTimer tm(DCHAG_STAGE_BWD_TOKENS, st);
    k_dz_attention<T><<<dim3(Cin, N, B), 256, 0, st>>>(Cin, N, D, heads, g, G, alpha, dalpha, w, Mf, dz);
    if ((rc = launch_status())) return rc;
  }
  StageTimer tm(DCHAG_STAGE_BWD_KEY_QUERY, st);
  if (gr->dbk) {
    const long n = (long)G * D;
    k_fill_zero<T><<<dim3((unsigned)((n + 255) / 256)), 256, 0, st>>>(n, static_cast<T*>(gr->dbk));
    if ((rc = launch_status())) return rc;
  }
  if (!gr->dWk && !gr->dWq && !gr->dbq && !gr->dquery) return DCHAG_OK;
  {
    GemmDesc d{};                                               // r[k][a][j] = sum over the group's tokens of ds[., a] z[., j]
    d.M = heads; d.N = D; d.K = g * N; d.nb = B; d.nk = G; d.na = 1; d.reduce_b = 1;
    d.ragged = 2; d.ragged_total = Cin * N; d.ragged_nominal = g * N;
    d.A = {(long)Cin * N * heads, (long)g * N * heads, 0, 1, (long)heads};
    d.Bm = {(long)Cin * N * D, (long)g * N * D, 0, (long)D, 1};
    d.C = {0, (long)heads * D, 0, (long)D, 1};
    d.scale = 1.f;
    if ((rc = launch_gemm<float, T, float>(d, dalpha, zin, nullptr, r, st))) return rc;
  }
  if (gr->dWk) {
    k_outer_rows<float, T><<<dim3((D + 255) / 256, D, G), 256, 0, st>>>(D, dh, 1.f / sqrtf((float)dh), Qp, r,
                                                                        static_cast<T*>(gr->dWk));
    if ((rc = launch_status())) return rc;
  }
  if (!gr->dWq && !gr->dbq && !gr->dquery) return DCHAG_OK;
  k_query_grad<T><<<dim3((D + 3) / 4, G), 256, 0, st>>>(D, heads, static_cast<const T*>(lv->Wk), r, dQ,
                                                        static_cast<T*>(gr->dbq));
  if ((rc = launch_status())) return rc;
  if (gr->dWq) {
    k_outer_rows<T, T><<<dim3((D + 255) / 256, D, G), 256, 0, st>>>(D, D, 1.f, dQ, static_cast<const T*>(lv->query),
                                                                    static_cast<T*>(gr->dWq));
    if ((rc = launch_status())) return rc;
  }
  if (gr->dquery) {
    k_query_input_grad<T><<<dim3((D + 255) / 256, G), 256, 0, st>>>(D, static_cast<const T*>(lv->Wq), dQ,
                                                                   static_cast<T*>(gr->dquery));
    if ((rc = launch_status())) return rc;
  }
  return DCHAG_OK;
}

template <typename T>
int linear_level_backward(int B, int Cin, int N, int D, const dchag_level* lv, const dchag_level_grads* gr,
                          const T* zin, const T* dy, T* dz, hipStream_t st) {
  const int g = lv->group_size, G = groups_of(Cin, g);
  int rc;
  StageTimer tm(DCHAG_STAGE_BWD_CHANNEL_MIX, st);
  const long total = (long)B * Cin * N * D;
  k_channel_mix_dz<T><<<dim3((unsigned)((total + 255) / 256)), 256, 0, st>>>(total, Cin, N, D, g, G,
                                                                            static_cast<const T*>(lv->Wv), dy, dz);
  if ((rc = launch_status())) return rc;
  if (gr->dWv) {
    k_channel_mix_dw<T><<<dim3((D + 63) / 64, G * g), 256, 0, st>>>(B, Cin, N, D, g, G, zin, dy,
                                                                    static_cast<T*>(gr->dWv));
    if ((rc = launch_status())) return rc;
  }
  if (gr->dbv) return colsum<T>(B, D, RowBlocks{G, G * N, N}, dy, static_cast<T*>(gr->dbv), st);
  return DCHAG_OK;
}

template <typename T>
int tokenizer_backward(int B, int C, int H, int W, int p, int D, const T* x, const T* We, const T* dt_, T* dx,
                       T* dWe, T* dtok_bias, T* patches, hipStream_t st) {
  const int N = (H / p) * (W / p), pp = p * p;
  int rc;
  StageTimer tm(DCHAG_STAGE_BWD_TOKENIZE, st);
  if (dtok_bias && (rc = colsum<T>(B, D, RowBlocks{C, C * N, N}, dt_, dtok_bias, st))) return rc;
  const long pixels = (long)B * C * H * W;
  if (pixels > ((long)1 << 39)) return DCHAG_ERR_SHAPE;
  if (dWe) {
    k_patch_rows<T, false><<<dim3((unsigned)((pixels + 255) / 256)), 256, 0, st>>>(pixels, H, W, p, const_cast<T*>(x),
                                                                                  patches);
    if ((rc = launch_status())) return rc;
    GemmDesc d{};                                               // dWe[c][d][kk] = sum_{b,n} dt[b,c,n,d] patch[b,c,n,kk]
    d.M = D; d.N = pp; d.K = N; d.nb = B; d.nk = C; d.na = 1; d.reduce_b = 1;
    d.A = {(long)C * N * D, (long)N * D, 0, 1, (long)D};
    d.Bm = {(long)C * N * pp, (long)N * pp, 0, (long)pp, 1};
    d.C = {0, (long)D * pp, 0, (long)pp, 1};
    d.scale = 1.f;
    if ((rc = launch_gemm<T, T, T>(d, dt_, patches, nullptr, dWe, st))) return rc;
  }
  if (dx) {
    GemmDesc d{};                                               // dpatch[b,c,n,kk] = sum_d dt[b,c,n,d] We[c][d][kk]
    d.M = N; d.N = pp; d.K = D; d.nb = B; d.nk = C; d.na = 1;
    d.A = {(long)C * N * D, (long)N * D, 0, (long)D, 1};
    d.Bm = {0, (long)D * pp, 0, (long)pp, 1};
    d.C = {(long)C * N * pp, (long)N * pp, 0, (long)pp, 1};
    d.scale = 1.f;
    if ((rc = launch_gemm<T, T, T>(d, dt_, We, nullptr, patches, st))) return rc;
    k_patch_rows<T, true><<<dim3((unsigned)((pixels + 255) / 256)), 256, 0, st>>>(pixels, H, W, p, dx, patches);
    if ((rc = launch_status())) return rc;
  }
  return DCHAG_OK;
}

template <typename T>
int backward_impl(dchag_dtype dt, int B, int C, int H, int W, int p, int D, int heads, const void* x, const void* We,
                  const void* be, const void* ce, int n_levels, const dchag_level* levels, const int32_t* gs,
                  const void* dout, void* dx, void* dWe, void* dtok_bias, const dchag_level_grads* grads,
                  unsigned char* ws, const BackwardWs& w, hipStream_t st) {
  const int N = (H / p) * (W / p);
  // forward sweep, keeping alpha, u, o (and the inputs) of every level
  g_level = 0;
  int rc = dchag_tokenize(dt, B, C, H, W, p, D, x, We, be, ce, ws + w.tokens, st);
  if (rc) return rc;
  const T* zins[16];
  KeptLevel kl[16];
  int cins[17];
  cins[0] = C;
  zins[0] = reinterpret_cast<const T*>(ws + w.tokens);
  for (int l = 0; l < n_levels; ++l) {
    g_level = l + 1;
    const bool linear = levels[l].kind == DCHAG_LEVEL_LINEAR, last = l + 1 == n_levels;
    kl[l] = kept_level(dt, B, cins[l], N, D, heads, gs[l], linear, !last);
    unsigned char* lw = ws + w.kept[l];
    T* y = last ? nullptr : reinterpret_cast<T*>(lw + kl[l].y);
    if (linear)
      rc = run_level_linear<T>(B, cins[l], N, D, &levels[l], zins[l], y, st);
    else
      rc = folded_level_forward<T>(B, cins[l], N, D, heads, &levels[l], zins[l], y,
                                   reinterpret_cast<float*>(lw + kl[l].qp), reinterpret_cast<float*>(lw + kl[l].mf),
                                   reinterpret_cast<float*>(lw + kl[l].alpha), reinterpret_cast<T*>(lw + kl[l].u),
                                   reinterpret_cast<T*>(lw + kl[l].o), st);
    if (rc) return rc;
    cins[l + 1] = groups_of(cins[l], gs[l]);
    zins[l + 1] = y;
  }
  // reverse sweep
  const T* dy = static_cast<const T*>(dout);
  for (int l = n_levels - 1; l >= 0; --l) {
    g_level = l + 1;
    unsigned char* lw = ws + w.kept[l];
    T* dz = reinterpret_cast<T*>(ws + w.dz[l & 1]);
    if (levels[l].kind == DCHAG_LEVEL_LINEAR)
      rc = linear_level_backward<T>(B, cins[l], N, D, &levels[l], &grads[l], zins[l], dy, dz, st);
    else
      rc = attention_level_backward<T>(B, cins[l], N, D, heads, &levels[l], &grads[l], zins[l], dy, dz,
                                       reinterpret_cast<const float*>(lw + kl[l].qp),
                                       reinterpret_cast<const float*>(lw + kl[l].mf),
                                       reinterpret_cast<const float*>(lw + kl[l].alpha),
                                       reinterpret_cast<const T*>(lw + kl[l].u), reinterpret_cast<const T*>(lw + kl[l].o),
                                       reinterpret_cast<float*>(ws + w.dalpha), reinterpret_cast<T*>(ws + w.w),
                                       reinterpret_cast<T*>(ws + w.d_o), reinterpret_cast<float*>(ws + w.r),
                                       reinterpret_cast<float*>(ws + w.dq), st);
    if (rc) return rc;
    dy = dz;
  }
  g_level = 0;
  if (!dx && !dWe && !dtok_bias) return DCHAG_OK;
  return tokenizer_backward<T>(B, C, H, W, p, D, static_cast<const T*>(x), static_cast<const T*>(We), dy,
                               static_cast<T*>(dx), static_cast<T*>(dWe), static_cast<T*>(dtok_bias),
                               reinterpret_cast<T*>(ws + w.patches), st);
}
