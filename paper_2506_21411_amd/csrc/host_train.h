// Host side of dchag_forward_folded and dchag_backward: workspace layout, level scheduler, launches.
// Included by dchag_api.hip inside its anonymous namespace (it uses that file's helpers).
//
// Both calls evaluate an attention level with the value projection behind the weighted sum:
//   alpha = softmax over the group of (z . M),  u_a = sum_c alpha[c,a] z[c],  o_a = Wv_a u_a + bv_a,
//   y = Wo o + bo.
// The inference call takes its first level straight from the pixels where the shape allows (tokens are linear in
// the pixels, so Wv moves into the tokenizer weights: attend_pixels_forward).
// The backward call keeps alpha, u and o of every level in its workspace and then walks the levels
// in reverse (paper Section 3.3: the backward pass is local, the plain reverse of the forward).

// Per-level pieces that a forward sweep leaves behind for the reverse sweep.
struct KeptLevel {
  size_t qp, mf, mb, alpha_f, alpha, u, o, y, total;
};

// Shapes whose scores go through the score kernels of the bf16 forward path.
inline bool train_fast(dchag_dtype dt, int D, int heads) {
  return fast_level(dt, D, heads) && !dbg(SW_GENERIC_LEVEL);
}

inline KeptLevel kept_level(dchag_dtype dt, int B, int Cin, int N, int D, int heads, int g, bool linear,
                            bool keep_y) {
  const int G = groups_of(Cin, g);
  const size_t es = elem_size(dt);
  KeptLevel w{};
  size_t off = 0;
  if (!linear) {
    w.qp = off; off += align_up((size_t)G * D * 4);
    w.mf = off; off += align_up((size_t)G * heads * D * 4);
    w.mb = off; off += align_up((size_t)G * heads * D * 2);
    if (train_fast(dt, D, heads)) {
      w.alpha_f = off; off += align_up((size_t)B * G * round_up(g, 8) * heads * round_up(N, 32) * 4);
    }
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
  size_t tokens, ping, pong, level, ms, msb, cs, mft, prep[16], total;
};

// Scratch of the first level's pixel-score shortcut (composed score weights, fp32 and bf16; constants;
// transposed folded keys).
inline size_t pixel_scratch(size_t off, int C, int pp, int D, int heads, int G0, size_t* ms, size_t* msb, size_t* cs,
                            size_t* mft) {
  *ms = off; off += align_up((size_t)C * heads * pp * 4);
  *msb = off; off += align_up((size_t)C * heads * pp * 2);
  *cs = off; off += align_up((size_t)C * heads * 4);
  *mft = off; off += align_up((size_t)G0 * D * heads * 4);
  return off;
}

// Tokenizer weights with the first level's value projection folded in, Wf [C,D,pp], and the folded token bias [C,D].
inline size_t value_fold_bytes(int C, int D, int pp) {
  return align_up((size_t)C * D * pp * 2) + align_up((size_t)C * D * 2);
}

inline FoldedWs folded_ws(dchag_dtype dt, int B, int C, int N, int pp, int D, int heads, int n_levels,
                          const int32_t* group_sizes) {
  FoldedWs w{};
  const size_t es = elem_size(dt);
  size_t off = 0;
  // the tokens, or (bf16, 16 or 64 pixels per patch) what replaces them when the first level's values come from the pixels
  w.tokens = off; off += std::max(align_up((size_t)B * C * N * D * es), dt == DCHAG_BF16 && (pp == 16 || pp == 64) ? value_fold_bytes(C, D, pp) : 0);
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
  off = pixel_scratch(off, C, pp, D, heads, groups_of(C, group_sizes[0]), &w.ms, &w.msb, &w.cs, &w.mft);
  c_in = C;
  for (int l = 0; l < n_levels; ++l) {                   // every level's projected query and folded keys (one launch)
    const int G = groups_of(c_in, group_sizes[l]);
    w.prep[l] = off; off += prep_bytes(G, D, heads);
    c_in = G;
  }
  w.total = off;
  return w;
}

// Patches per block of the token-gradient kernels: 16 (the softmax weights and ds of a tile must fit 64 KiB of
// LDS), fewer while that leaves compute units without a block.
inline int dz_patches(int B, int G, int N, int D, int g) {
  int pt = 16;
  if (const char* e = dbg(SW_DZ_PT)) pt = atoi(e) > 0 ? atoi(e) : pt;
  while (pt > 1 && (size_t)2 * pt * g * 16 * 4 > 64 * 1024) pt >>= 1;
  while (pt > 1 && (long)B * G * ((N + pt - 1) / pt) * ((D + 1023) / 1024) < 2L * compute_units()) pt >>= 1;
  return pt;
}

struct BackwardWs {
  size_t tokens, patches, kept[16], dz[2], dalpha, w, d_o, r, dq, rpart, ms, msb, cs, mft, total;
};

inline BackwardWs backward_ws(dchag_dtype dt, int B, int C, int N, int pp, int D, int heads, int n_levels,
                              const int32_t* group_sizes, const int32_t* kinds) {
  BackwardWs w{};
  const size_t es = elem_size(dt);
  size_t off = 0;
  w.tokens = off; off += align_up((size_t)B * C * N * D * es);
  w.patches = off; off += align_up((size_t)B * C * N * pp * es);
  int c_in = C;
  size_t dal = 0, wv = 0, dov = 0, rv = 0, dqv = 0, dz0 = 0, dz1 = 0, rp = 0;
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
      const int pt = dz_patches(B, G, N, D, g);
      rp = std::max(rp, align_up((size_t)B * G * ((N + pt - 1) / pt) * heads * D * 4));
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
  w.rpart = off; off += rp;
  off = pixel_scratch(off, C, pp, D, heads, groups_of(C, group_sizes[0]), &w.ms, &w.msb, &w.cs, &w.mft);
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

// bf16 products go to the MFMA kernel when it tiles them: K a multiple of 64 and not ragged, each operand with
// one unit stride, every other stride and offset a multiple of 8 elements (16-byte rows).
inline bool mult8(long v) { return (v & 7) == 0; }
inline bool gemm_mfma_ok(const GemmDesc& d) {
  if (d.K % 64 || d.ragged == 2 || dbg(SW_GEMM_GENERIC)) return false;
  const bool at = d.A.s1 != 1, bt = d.Bm.s0 != 1;
  if (at && (d.A.s0 != 1 || d.M % 8 || d.M < 8 || d.ragged)) return false;
  if (bt && (d.Bm.s1 != 1 || d.N % 8 || d.N < 8)) return false;
  return mult8(d.A.sb) && mult8(d.A.sk) && mult8(d.A.sa) && mult8(at ? d.A.s1 : d.A.s0) && mult8(d.Bm.sb) &&
         mult8(d.Bm.sk) && mult8(d.Bm.sa) && mult8(bt ? d.Bm.s0 : d.Bm.s1);
}

template <int BM, int BN, int WM, int WN, typename TC>
int launch_gemm_mfma_tile(const GemmDesc& d, const bf16* A, const bf16* Bm, const bf16* bias, TC* C, TC* rowsum,
                          hipStream_t st) {
  const long batch = (long)(d.reduce_b ? 1 : d.nb) * d.nk * d.na;
  const long mt = (d.M + BM - 1) / BM;
  if (batch > 65535 || mt > 65535 || d.M < 1 || d.N < 1) return DCHAG_ERR_SHAPE;
  const bool at = d.A.s1 != 1, bt = d.Bm.s0 != 1;
  auto kern = at ? (bt ? k_gemm_mfma<BM, BN, WM, WN, true, true, TC> : k_gemm_mfma<BM, BN, WM, WN, true, false, TC>)
                 : (bt ? k_gemm_mfma<BM, BN, WM, WN, false, true, TC> : k_gemm_mfma<BM, BN, WM, WN, false, false, TC>);
  constexpr int lds = 2 * (BM + BN) * 128;
  if (ensure_dynamic_lds(reinterpret_cast<const void*>(kern), lds)) return DCHAG_ERR_LAUNCH;
  kern<<<dim3((d.N + BN - 1) / BN, (unsigned)mt, (unsigned)batch), 256, lds, st>>>(d, A, Bm, bias, C, rowsum);
  return launch_status();
}

// Tile shape by the extent of the output: a narrow N (one head, one patch of pixels) or a short M (the rows
// of one head) takes the 64-wide tile on that side.
// rowsum (optional, only with a transposed A on the MFMA kernel: see gemm_rowsum_ok): sums of A's rows.
template <typename TC>
int launch_gemm_bf16(const GemmDesc& d0, const bf16* A, const bf16* Bm, const bf16* bias, TC* C, hipStream_t st,
                     TC* rowsum = nullptr) {
  if (!gemm_mfma_ok(d0)) return launch_gemm<bf16, bf16, TC>(d0, A, Bm, bias, C, st);
  GemmDesc d = d0;
  d.c_vec = sizeof(TC) == 2 && d.C.s1 == 1 && d.N % 8 == 0 && mult8(d.C.sb) && mult8(d.C.sk) && mult8(d.C.sa) &&
            mult8(d.C.s0) && !(reinterpret_cast<uintptr_t>(C) & 15) && !dbg(SW_GEMM_SCALAR_STORES);
  if (d.N <= 64) return launch_gemm_mfma_tile<128, 64, 4, 1, TC>(d, A, Bm, bias, C, rowsum, st);
  if (d.M <= 64) return launch_gemm_mfma_tile<64, 128, 1, 4, TC>(d, A, Bm, bias, C, rowsum, st);
  // a product of few 128 x 128 tiles (the one-group top level) takes 64 x 64 tiles: four times the blocks
  const long batch = (long)(d.reduce_b ? 1 : d.nb) * d.nk * d.na;
  if ((long)((d.N + 127) / 128) * ((d.M + 127) / 128) * batch * 2 < compute_units())
    return launch_gemm_mfma_tile<64, 64, 2, 2, TC>(d, A, Bm, bias, C, rowsum, st);
  return launch_gemm_mfma_tile<128, 128, 2, 2, TC>(d, A, Bm, bias, C, rowsum, st);
}
// True when launch_gemm_bf16 will deliver the row sums of A along with the product.
inline bool gemm_rowsum_ok(const GemmDesc& d) { return gemm_mfma_ok(d) && d.A.s1 != 1 && !dbg(SW_COLSUM); }

// Same-type products of the level kernels: MFMA for bf16 where it tiles, the fp32-FMA kernel otherwise.
inline int gemm_tt(const GemmDesc& d, const float* A, const float* Bm, const float* bias, float* C, hipStream_t st) {
  return launch_gemm<float, float, float>(d, A, Bm, bias, C, st);
}
inline int gemm_tt(const GemmDesc& d, const bf16* A, const bf16* Bm, const bf16* bias, bf16* C, hipStream_t st) {
  return launch_gemm_bf16<bf16>(d, A, Bm, bias, C, st);
}

// A weight gradient  dW = sum over rows of X^T Y  together with the bias gradient  db = sum over rows of X
// (the row sums of the product's transposed A operand).  rb describes the rows for the separate column-sum
// kernel, which runs when the product kernel cannot deliver the sums.
inline int gemm_with_bias_grad(GemmDesc d, int B, int D, RowBlocks rb, const float* X, const float* Y, float* dW,
                               float* db, hipStream_t st) {
  int rc = DCHAG_OK;
  if (db) {
    k_colsum<float, float><<<dim3((D + 63) / 64, rb.G), 1024, 0, st>>>(B, D, rb, X, db);
    if ((rc = launch_status())) return rc;
  }
  return dW ? launch_gemm<float, float, float>(d, X, Y, nullptr, dW, st) : DCHAG_OK;
}
inline int gemm_with_bias_grad(GemmDesc d, int B, int D, RowBlocks rb, const bf16* X, const bf16* Y, bf16* dW, bf16* db,
                               hipStream_t st) {
  if (dW && db && gemm_rowsum_ok(d)) return launch_gemm_bf16<bf16>(d, X, Y, nullptr, dW, st, db);
  int rc = DCHAG_OK;
  if (db) {
    k_colsum<bf16, bf16><<<dim3((D + 63) / 64, rb.G), 1024, 0, st>>>(B, D, rb, X, db);
    if ((rc = launch_status())) return rc;
  }
  return dW ? launch_gemm_bf16<bf16>(d, X, Y, nullptr, dW, st) : DCHAG_OK;
}

// Buffers of one attention level (see KeptLevel); alpha_f and Mb are used by the bf16 kernels only.
template <typename T>
struct LevelBufs {
  float *Qp, *Mf;
  bf16* Mb;
  float *alpha_f, *alpha;
  T *u, *o;
};

template <typename T>
LevelBufs<T> level_bufs(unsigned char* lw, const KeptLevel& kl) {
  return LevelBufs<T>{reinterpret_cast<float*>(lw + kl.qp),      reinterpret_cast<float*>(lw + kl.mf),
                      reinterpret_cast<bf16*>(lw + kl.mb),       reinterpret_cast<float*>(lw + kl.alpha_f),
                      reinterpret_cast<float*>(lw + kl.alpha),   reinterpret_cast<T*>(lw + kl.u),
                      reinterpret_cast<T*>(lw + kl.o)};
}

// alpha of one level, token-major [B,Cin,N,heads], on the shape-generic kernels.
template <typename T>
int generic_alpha(int B, int Cin, int N, int D, int heads, const dchag_level* lv, const T* zin, const LevelBufs<T>& lb,
                  hipStream_t st) {
  const int g = lv->group_size, G = groups_of(Cin, g);
  int rc;
  {
    StageTimer tm(DCHAG_STAGE_QUERY, st);
    k_project_query<T><<<dim3((D + 3) / 4, G), 256, 0, st>>>(D, static_cast<const T*>(lv->query),
                                                             static_cast<const T*>(lv->Wq),
                                                             static_cast<const T*>(lv->bq), lb.Qp);
    if ((rc = launch_status())) return rc;
  }
  {
    StageTimer tm(DCHAG_STAGE_FOLD, st);
    k_fold_query_into_key<T><<<dim3((D + 63) / 64, heads, G), 256, 0, st>>>(D, heads, static_cast<const T*>(lv->Wk),
                                                                            lb.Qp, lb.Mf, lb.Mb, nullptr);
    if ((rc = launch_status())) return rc;
  }
  StageTimer tm(DCHAG_STAGE_SCORES, st);
  const long T_total = (long)B * Cin * N;
  k_scores_generic<T, 8><<<dim3((unsigned)((T_total + 3) / 4)), 256, 0, st>>>(T_total, Cin, N, D, heads, g, zin, lb.Mf,
                                                                             lb.alpha);
  if ((rc = launch_status())) return rc;
  const long total = (long)B * G * N * heads;
  k_softmax_group<<<dim3((unsigned)((total + 255) / 256)), 256, 0, st>>>(Cin, N, heads, g, G, total, lb.alpha);
  return launch_status();
}

// alpha of one level through the score kernels of the bf16 forward path, then re-laid token-major.
inline int fast_alpha(int B, int Cin, int N, int D, int heads, const dchag_level* lv, const bf16* zin,
                      const LevelBufs<bf16>& lb, hipStream_t st, const PixelScores* px, int phase = 0) {
  const int g = lv->group_size, G = groups_of(Cin, g);
  bool tm_done = false;
  int rc = fast_scores(B, Cin, N, D, heads, lv, zin, lb.Qp, lb.Mf, lb.Mb, lb.alpha_f, st, px, lb.alpha, &tm_done, phase);
  if (rc || tm_done) return rc;
  StageTimer tm(DCHAG_STAGE_SCORES, st);
  const long total = (long)B * Cin * N * heads;
  k_alpha_token_major<<<dim3((unsigned)((total + 255) / 256)), 256, 0, st>>>(total, Cin, N, heads, g, round_up(g, 8), G,
                                                                            round_up(N, 32), lb.alpha_f, lb.alpha);
  return launch_status();
}

inline int head_sums(int B, int Cin, int N, int D, int heads, int g, const float* alpha, const float* z, float* u,
                     hipStream_t st) {
  k_head_sums<float, 16><<<dim3(N, groups_of(Cin, g), B), 256, 0, st>>>(Cin, N, D, heads, g, alpha, z, u);
  return launch_status();
}
inline int head_sums(int B, int Cin, int N, int D, int heads, int g, const float* alpha, const bf16* z, bf16* u,
                     hipStream_t st) {
  const size_t lds = (size_t)std::min(g, Cin) * 16 * 4;
  if (D % 4 == 0 && lds <= 160 * 1024 - 4096 && !dbg(SW_GENERIC_LEVEL)) {
    if (ensure_dynamic_lds(reinterpret_cast<const void*>(k_head_sums_bf16), (int)lds)) return DCHAG_ERR_LAUNCH;
    k_head_sums_bf16<<<dim3(N, groups_of(Cin, g), B), 256, lds, st>>>(Cin, N, D, heads, g, alpha, z, u);
  } else {
    k_head_sums<bf16, 16><<<dim3(N, groups_of(Cin, g), B), 256, 0, st>>>(Cin, N, D, heads, g, alpha, z, u);
  }
  return launch_status();
}

inline int oproj(int B, int D, RowBlocks rb, const float* o, const float* Wo, const float* bo, float* y, hipStream_t st) {
  return launch_linear<float>(B, D, rb, o, Wo, bo, y, st);
}
inline int oproj(int B, int D, RowBlocks rb, const bf16* o, const bf16* Wo, const bf16* bo, bf16* y, hipStream_t st) {
  if (D % 256 == 0 && !force_generic()) return launch_linear_dl(B, D, rb, o, Wo, bo, y, st);
  return launch_linear<bf16>(B, D, rb, o, Wo, bo, y, st);
}

// One attention level evaluated as  alpha -> u -> o -> y  (y skipped when zout is NULL).  px: the first
// level of the bf16 path may take its scores from the pixels.  phase = 2: the level's weight-only prep (projected
// query, folded keys) is already in lb (bf16 score-kernel path only).
template <typename T>
int folded_level_forward(dchag_dtype dt, int B, int Cin, int N, int D, int heads, const dchag_level* lv, const T* zin,
                         T* zout, const LevelBufs<T>& lb, hipStream_t st, const PixelScores* px, int phase = 0) {
  const int g = lv->group_size, G = groups_of(Cin, g), dh = D / heads;
  const T* Wv = static_cast<const T*>(lv->Wv);
  int rc;
  if constexpr (std::is_same<T, bf16>::value) {
    if (train_fast(dt, D, heads)) rc = fast_alpha(B, Cin, N, D, heads, lv, zin, lb, st, px, phase);
    else rc = generic_alpha<T>(B, Cin, N, D, heads, lv, zin, lb, st);
  } else {
    rc = generic_alpha<T>(B, Cin, N, D, heads, lv, zin, lb, st);
  }
  if (rc) return rc;
  {
    StageTimer tm(DCHAG_STAGE_HEAD_SUMS, st);
    if ((rc = head_sums(B, Cin, N, D, heads, g, lb.alpha, zin, lb.u, st))) return rc;
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
    if ((rc = gemm_tt(d, lb.u, Wv, static_cast<const T*>(lv->bv), lb.o, st))) return rc;
  }
  if (!zout) return DCHAG_OK;
  StageTimer tm(DCHAG_STAGE_OPROJ, st);
  return oproj(B, D, RowBlocks{G, G * N, N}, lb.o, static_cast<const T*>(lv->Wo), static_cast<const T*>(lv->bo), zout,
               st);
}

template <typename T>
PixelScores pixel_scores_of(const void* x, const void* We, const void* be, const void* ce, int H, int W, int p,
                            unsigned char* ws, size_t ms, size_t msb, size_t cs, size_t mft) {
  return PixelScores{static_cast<const bf16*>(x), static_cast<const bf16*>(We), static_cast<const bf16*>(be),
                     static_cast<const bf16*>(ce), H, W, p, reinterpret_cast<float*>(ws + ms),
                     reinterpret_cast<float*>(ws + cs), reinterpret_cast<float*>(ws + mft),
                     reinterpret_cast<bf16*>(ws + msb)};
}

template <typename TC>
int gemm_per_channel(GemmDesc d, int C, int g, long a_grp, long b_ch, long c_ch, const bf16* A, const bf16* Bm, TC* Cm,
                     hipStream_t st);

// First attention level of the inference path with the value projection folded into the tokenizer (bf16, 4 x 4 or
// 8 x 8 patches): Wf[c] = Wv[k(c)] We[c] and the folded biases Wv be, Wv ce are weight-only products, then one kernel
// goes from pixels and softmax weights to the pre-projection output o [B,G,N,D]; neither tokens nor per-head token
// averages exist.  fold: scratch of fold_bytes >= value_fold_bytes(C, D, p*p); what is left behind the folded weights
// takes partial sums.  attend_ring_ok: the shape takes the ring kernel; attend_wide_ok: the kernel that passes the
// operands through registers.
inline bool attend_wide_ok(int p, int D, int heads, const dchag_level* lv) {
  const int pp = p * p, dh = D / heads;
  return lv->kind != DCHAG_LEVEL_LINEAR && (pp == 16 || pp == 64) && D % 256 == 0 && D % heads == 0 && dh % 32 == 0 &&
         (256 % dh == 0 || dh % 256 == 0) && !dbg(SW_VALUE_UNFOLDED);
}
inline bool attend_ring_ok(int p, int W, int D, int heads, const void* x, const dchag_level* lv) {
  return attend_wide_ok(p, D, heads, lv) && reduce_ring_ok(p, W, D, x, nullptr, nullptr, nullptr, nullptr) &&
         (D / heads) % 64 == 0;
}
// Shapes whose first level dchag_forward_folded takes from the pixels (scores through composed score weights, values
// through folded tokenizer weights).
inline bool values_from_pixels(dchag_dtype dt, int p, int D, int heads, const dchag_level* lv) {
  return dt == DCHAG_BF16 && train_fast(dt, D, heads) && pixel_scores_ok(p, heads) && attend_wide_ok(p, D, heads, lv);
}

// The weight-only part: fold (value_fold_bytes(C, D, p*p) bytes) receives Wf [C,D,p*p] and Wv (be + ce) [C,D].
inline int fold_value_weights(int C, int p, int D, const dchag_level* lv, const bf16* We, const bf16* be, const bf16* ce,
                              unsigned char* fold, hipStream_t st) {
  const int g = lv->group_size, G = groups_of(C, g), pp = p * p;
  const bf16* Wv = static_cast<const bf16*>(lv->Wv);
  const size_t wf_bytes = align_up((size_t)C * D * pp * 2);
  bf16* Wf = reinterpret_cast<bf16*>(fold);
  bf16* fb = reinterpret_cast<bf16*>(fold + wf_bytes);   // Wv (be + ce), [C,D]
  int rc;
  StageTimer tm(DCHAG_STAGE_FOLD_VALUE, st);
  // Wf[c](o, kk) = sum_d Wv[k](o, d) We[c](d, kk).  64 pixels per patch: four channels per work item share a 256-row
  // tile of Wv (DCHAG_FOLD_VALUE_GEMM, a debugging aid, takes the general product kernel, one channel per workgroup)
  if (pp == 64 && aligned16(Wv) && aligned16(We) && !dbg(SW_FOLD_VALUE_GEMM)) {
    TileWork tw{};
    tw.n_tiles = (std::min(g, C) + 3) / 4;
    tw.m_tiles = D / kGemmBM;
    tw.nb = 1;
    const long total = (long)G * tw.m_tiles * tw.n_tiles;
    if (total > (1L << 30)) return DCHAG_ERR_SHAPE;
    tw.total = (int)total;
    const int per = (tw.total + kXcds - 1) / kXcds;
    if (ensure_dynamic_lds(reinterpret_cast<const void*>(k_fold_value_dl), kGemmRingBytes)) return DCHAG_ERR_LAUNCH;
    k_fold_value_dl<<<dim3((unsigned)(per * kXcds)), 512, kGemmRingBytes, st>>>(C, D, g, tw, Wv, We, Wf);
    if ((rc = launch_status())) return rc;
  } else {
    GemmDesc d{};
    d.M = D; d.N = pp; d.K = D; d.nb = 1;
    d.A = {0, 0, 0, (long)D, 1};
    d.Bm = {0, 0, 0, (long)pp, 1};
    d.C = {0, 0, 0, (long)pp, 1};
    d.scale = 1.f;
    if ((rc = gemm_per_channel<bf16>(d, C, g, (long)D * D, (long)D * pp, (long)D * pp, Wv, We, Wf, st))) return rc;
  }
  if ((be || ce) && aligned16(Wv) && aligned16(be) && aligned16(ce) && G <= 65535 && !dbg(SW_FOLD_VALUE_GEMM)) {
    k_fold_token_bias<<<dim3(D / 32, G), 256, 0, st>>>(C, D, g, Wv, be, ce, fb);
    if ((rc = launch_status())) return rc;
  } else if (be || ce) {
    // (Wv (be + ce))[c](o) = sum over the vectors v present, sum_d v[c](d) Wv[k](o, d): one product whose batch
    // index walks from be to ce (their distance in elements, taken on the integer addresses: the two are separate
    // allocations in one flat device address space) and is summed over
    const bf16* first = be ? be : ce;
    const long be_to_ce = be && ce ? (long)((reinterpret_cast<intptr_t>(ce) - reinterpret_cast<intptr_t>(be)) /
                                            (intptr_t)sizeof(bf16))
                                   : 0;
    GemmDesc e{};
    e.M = g; e.N = D; e.K = D; e.nk = G; e.na = 1;
    e.nb = be && ce ? 2 : 1;
    e.reduce_b = 1;
    e.ragged = 1; e.ragged_total = C; e.ragged_nominal = g;
    e.A = {be_to_ce, (long)g * D, 0, (long)D, 1};
    e.Bm = {0, (long)D * D, 0, 1, (long)D};
    e.C = {0, (long)g * D, 0, (long)D, 1};
    e.scale = 1.f;
    if ((rc = launch_gemm_bf16<bf16>(e, first, Wv, nullptr, fb, st))) return rc;
  }
  return DCHAG_OK;
}

// From pixels, softmax weights and the folded weights (fold, as fold_value_weights leaves it) to the pre-projection
// output o [B,G,N,D].  part / part_bytes: scratch for partial sums (few groups: members dealt to several workgroups).
inline int attend_pixels_forward(int B, int C, int H, int W, int p, int D, int heads, const dchag_level* lv,
                                 const bf16* x, bool token_bias, const float* alpha, const unsigned char* fold,
                                 unsigned char* part, size_t part_bytes, bf16* o, hipStream_t st) {
  const int g = lv->group_size, G = groups_of(C, g), pp = p * p, N = (H / p) * (W / p);
  const bf16* Wf = reinterpret_cast<const bf16*>(fold);
  const bf16* fb = reinterpret_cast<const bf16*>(fold + align_up((size_t)C * D * pp * 2));
  StageTimer tm(DCHAG_STAGE_TOKENIZE_ATTEND, st);
  const bf16* v1 = token_bias ? fb : nullptr;
  const bf16* v2 = nullptr;
  const bf16* bv = static_cast<const bf16*>(lv->bv);
  if (attend_ring_ok(p, W, D, heads, x, lv))
    return launch_reduce_ring<true>(B, C, H, W, D, g, heads, x, Wf, nullptr, v1, v2, alpha, bv, o, st,
                                    reinterpret_cast<float*>(part), part_bytes);
  if (B > 65535 || G > 65535) return DCHAG_ERR_SHAPE;
  const int dh = D / heads, nhs = dh >= 256 ? 1 : 256 / dh;
  const size_t lds = (size_t)2 * 128 * (pp * 2 + 16) + (size_t)2 * nhs * 512;
  auto kern = pp == 16 ? k_tokenize_attend_wide<1> : k_tokenize_attend_wide<4>;
  if (ensure_dynamic_lds(reinterpret_cast<const void*>(kern), (int)lds)) return DCHAG_ERR_LAUNCH;
  kern<<<dim3((unsigned)(((N + 127) / 128) * (D / 256)), G, B), 512, lds, st>>>(
      C, H, W, p, D, g, heads, round_up(g, 8), round_up(N, 32), x, Wf, v1, v2, alpha, bv, o);
  return launch_status();
}

// What dchag_fold_value leaves in the caller's buffer: the folded tokenizer weights and token bias of the first level,
// then every attention level's weight-only prep (projected query, folded keys fp32 + bf16) and the first level's composed
// score weights.
struct PreparedLayout {
  size_t fold, qp[16], mf[16], mb[16], ms, msb, cs, mft, total;
};
inline PreparedLayout prepared_layout(int C, int pp, int D, int heads, int n_levels, const dchag_level* levels) {
  PreparedLayout L{};
  size_t off = 0;
  L.fold = off; off += value_fold_bytes(C, D, pp);
  int c_in = C;
  for (int l = 0; l < n_levels; ++l) {
    const int G = groups_of(c_in, levels[l].group_size);
    if (levels[l].kind != DCHAG_LEVEL_LINEAR) {
      L.qp[l] = off; off += align_up((size_t)G * D * 4);
      L.mf[l] = off; off += align_up((size_t)G * heads * D * 4);
      L.mb[l] = off; off += align_up((size_t)G * heads * D * 2);
    }
    c_in = G;
  }
  off = pixel_scratch(off, C, pp, D, heads, groups_of(C, levels[0].group_size), &L.ms, &L.msb, &L.cs, &L.mft);
  L.total = off;
  return L;
}
// The pieces of level l inside a prepared buffer, in the form the level code takes them.
inline void use_prepared(const unsigned char* pf, const PreparedLayout& L, int l, LevelBufs<bf16>& lb) {
  unsigned char* q = const_cast<unsigned char*>(pf);     // read only from here on (phase 2 of the score code)
  lb.Qp = reinterpret_cast<float*>(q + L.qp[l]);
  lb.Mf = reinterpret_cast<float*>(q + L.mf[l]);
  lb.Mb = reinterpret_cast<bf16*>(q + L.mb[l]);
}
inline int prepare_folded(int C, int H, int W, int p, int D, int heads, const void* We, const void* be, const void* ce,
                          int n_levels, const dchag_level* levels, unsigned char* pf, hipStream_t st) {
  const PreparedLayout L = prepared_layout(C, p * p, D, heads, n_levels, levels);
  int rc;
  set_level(1);
  if ((rc = fold_value_weights(C, p, D, &levels[0], static_cast<const bf16*>(We), static_cast<const bf16*>(be),
                               static_cast<const bf16*>(ce), pf + L.fold, st)))
    return rc;
  const PixelScores px = pixel_scores_of<bf16>(nullptr, We, be, ce, H, W, p, pf, L.ms, L.msb, L.cs, L.mft);
  int c_in = C;
  for (int l = 0; l < n_levels; ++l) {
    set_level(l + 1);
    if (levels[l].kind != DCHAG_LEVEL_LINEAR) {
      LevelBufs<bf16> lb{};
      use_prepared(pf, L, l, lb);
      if ((rc = fast_scores(1, c_in, 1, D, heads, &levels[l], nullptr, lb.Qp, lb.Mf, lb.Mb, nullptr, st,
                            l == 0 ? &px : nullptr, nullptr, nullptr, 1)))
        return rc;
    }
    c_in = groups_of(c_in, levels[l].group_size);
  }
  return DCHAG_OK;
}

template <typename T>
int forward_folded_impl(dchag_dtype dt, int B, int C, int H, int W, int p, int D, int heads, const void* x,
                        const void* We, const void* be, const void* ce, int n_levels, const dchag_level* levels,
                        const int32_t* gs, void* out, unsigned char* ws, const FoldedWs& w, hipStream_t st,
                        const unsigned char* prefolded = nullptr) {
  const int N = (H / p) * (W / p);
  set_level(0);
  int rc;
  const T* zin = reinterpret_cast<const T*>(ws + w.tokens);
  int c_in = C, first = 0;
  if constexpr (std::is_same<T, bf16>::value) {
    if (n_levels > 1 && tokenize_mix_ok(dt, levels, p * p, D)) {      // tokenizer and linear first level in one kernel
      set_level(1);
      bf16* y = reinterpret_cast<bf16*>(ws + w.ping);
      if ((rc = tokenize_mix_forward(B, C, H, W, p, D, x, We, be, ce, &levels[0], y, st))) return rc;
      zin = y;
      c_in = groups_of(C, gs[0]);
      first = 1;
    }
  }
  const PixelScores px = pixel_scores_of<T>(x, We, be, ce, H, W, p, ws, w.ms, w.msb, w.cs, w.mft);
  const bool use_px = dt == DCHAG_BF16 && train_fast(dt, D, heads) && pixel_scores_ok(p, heads);
  PreparedLayout PL{};
  if (prefolded) PL = prepared_layout(C, p * p, D, heads, n_levels, levels);
  // every attention level's weight-only prep (projected query, query folded into the key weights) in ONE launch
  PrepBufs ready[16];
  bool hoisted = false;
  if constexpr (std::is_same<T, bf16>::value) {
    if (!prefolded && train_fast(dt, D, heads)) {
      KeyPrepJob jobs[16];
      int nj = 0, cl = c_in;
      for (int l = first; l < n_levels; ++l) {
        const int G = groups_of(cl, gs[l]);
        if (levels[l].kind != DCHAG_LEVEL_LINEAR) {
          ready[l] = prep_bufs(ws + w.prep[l], G, D, heads);
          jobs[nj++] = KeyPrepJob{&levels[l], G, ready[l], l == 0 ? px.MfT : nullptr};
        }
        cl = G;
      }
      set_level(0);
      if (nj && (rc = launch_query_keys(D, heads, jobs, nj, st))) return rc;
      hoisted = nj > 0;
    }
  }
  if constexpr (std::is_same<T, bf16>::value) {
    // an attention first level straight from the pixels: scores through the composed score weights, values through
    // the folded tokenizer weights (which sit where the tokens would have been)
    if (!first && values_from_pixels(dt, p, D, heads, &levels[0])) {
      set_level(1);
      const KeptLevel kl = kept_level(dt, B, C, N, D, heads, gs[0], false, false);
      LevelBufs<bf16> lb = level_bufs<bf16>(ws + w.level, kl);
      PixelScores px0 = px;
      if (prefolded) {                                   // the level's weight-only prep comes with the folded weights
        use_prepared(prefolded, PL, 0, lb);
        px0 = pixel_scores_of<bf16>(x, We, be, ce, H, W, p, const_cast<unsigned char*>(prefolded), PL.ms, PL.msb, PL.cs,
                                    PL.mft);
      } else if (hoisted) {
        lb.Qp = ready[0].Qp;
        lb.Mf = ready[0].Mf;
        lb.Mb = ready[0].Mb;
      }
      if ((rc = fast_scores(B, C, N, D, heads, &levels[0], nullptr, lb.Qp, lb.Mf, lb.Mb, lb.alpha_f, st, &px0, nullptr,
                            nullptr, prefolded ? 2 : (hoisted ? 3 : 0))))
        return rc;
      // the folded weights: the caller's (prepared once for fixed weights), else formed here, where the tokens would
      // have been; what is left of that region takes partial sums
      unsigned char* region = ws + w.tokens;
      size_t used = 0;
      const unsigned char* fold = prefolded ? prefolded + PL.fold : nullptr;
      if (!fold) {
        if ((rc = fold_value_weights(C, p, D, &levels[0], static_cast<const bf16*>(We), static_cast<const bf16*>(be),
                                     static_cast<const bf16*>(ce), region, st)))
          return rc;
        fold = region;
        used = value_fold_bytes(C, D, p * p);
      }
      if ((rc = attend_pixels_forward(B, C, H, W, p, D, heads, &levels[0], static_cast<const bf16*>(x), be || ce,
                                      lb.alpha_f, fold, region + used, (w.ping - w.tokens) - used, lb.o, st)))
        return rc;
      bf16* zout = n_levels == 1 ? static_cast<bf16*>(out) : reinterpret_cast<bf16*>(ws + w.ping);
      {
        StageTimer tm(DCHAG_STAGE_OPROJ, st);
        const int G0 = groups_of(C, gs[0]);
        if ((rc = oproj(B, D, RowBlocks{G0, G0 * N, N}, lb.o, static_cast<const bf16*>(levels[0].Wo),
                        static_cast<const bf16*>(levels[0].bo), zout, st)))
          return rc;
      }
      zin = zout;
      c_in = groups_of(C, gs[0]);
      first = 1;
    }
  }
  if (!first && (rc = dchag_tokenize(dt, B, C, H, W, p, D, x, We, be, ce, ws + w.tokens, st))) return rc;
  for (int l = first; l < n_levels; ++l) {
    set_level(l + 1);
    T* zout = (l + 1 == n_levels) ? static_cast<T*>(out) : reinterpret_cast<T*>(ws + ((l & 1) ? w.pong : w.ping));
    if (levels[l].kind == DCHAG_LEVEL_LINEAR)
      rc = run_level_linear<T>(B, c_in, N, D, &levels[l], zin, zout, st);
    else {
      const KeptLevel kl = kept_level(dt, B, c_in, N, D, heads, gs[l], false, false);
      LevelBufs<T> lb = level_bufs<T>(ws + w.level, kl);
      int phase = 0;
      if constexpr (std::is_same<T, bf16>::value) {
        if (prefolded && l > 0 && train_fast(dt, D, heads)) {
          use_prepared(prefolded, PL, l, lb);
          phase = 2;
        } else if (hoisted) {
          lb.Qp = ready[l].Qp;
          lb.Mf = ready[l].Mf;
          lb.Mb = ready[l].Mb;
          phase = 3;
        }
      }
      rc = folded_level_forward<T>(dt, B, c_in, N, D, heads, &levels[l], zin, zout, lb, st,
                                   (l == 0 && use_px) ? &px : nullptr, phase);
    }
    if (rc) return rc;
    zin = zout;
    c_in = groups_of(c_in, gs[l]);
  }
  return DCHAG_OK;
}

template <typename T>
int colsum(int B, int D, RowBlocks rb, const T* X, T* out, hipStream_t st) {
  k_colsum<T, T><<<dim3((D + 63) / 64, rb.G), 1024, 0, st>>>(B, D, rb, X, out);
  return launch_status();
}

// d alpha -> ds (softmax Jacobian), token-major.
inline int softmax_backward(int B, int Cin, int N, int D, int heads, int g, const float* z, const float* w,
                            const float* alpha, float* ds, hipStream_t st) {
  const int G = groups_of(Cin, g);
  const long T_total = (long)B * Cin * N;
  k_dalpha<float><<<dim3((unsigned)((T_total + 3) / 4)), 256, 0, st>>>(T_total, Cin, N, D, heads, g, G, z, w, ds);
  int rc = launch_status();
  if (rc) return rc;
  const long total = (long)B * G * N * heads;
  k_softmax_group_backward<<<dim3((unsigned)((total + 255) / 256)), 256, 0, st>>>(Cin, N, heads, g, G, total, alpha, ds);
  return launch_status();
}
inline int softmax_backward(int B, int Cin, int N, int D, int heads, int g, const bf16* z, const bf16* w,
                            const float* alpha, float* ds, hipStream_t st) {
  const int G = groups_of(Cin, g);
  const int mt = (std::min(g, Cin) + 15) / 16;
  if (D % 32 == 0 && mt <= 4 && !dbg(SW_GENERIC_LEVEL)) {
    const long items = (long)B * G * N;
    const dim3 grid((unsigned)((items + 3) / 4));
    if (mt == 1) k_dalpha_softmax_mfma<1><<<grid, 256, 0, st>>>(items, Cin, N, D, heads, g, G, z, w, alpha, ds);
    else if (mt == 2) k_dalpha_softmax_mfma<2><<<grid, 256, 0, st>>>(items, Cin, N, D, heads, g, G, z, w, alpha, ds);
    else k_dalpha_softmax_mfma<4><<<grid, 256, 0, st>>>(items, Cin, N, D, heads, g, G, z, w, alpha, ds);
    return launch_status();
  }
  const size_t big_lds = ((size_t)16 * ((std::min(g, Cin) + 15) / 16) + 17) * 16 * 4;
  const long items = (long)B * G * N;
  if (D % 32 == 0 && big_lds <= 128 * 1024 && items <= 0x7fffffffL && !dbg(SW_GENERIC_LEVEL)) {
    if (ensure_dynamic_lds(reinterpret_cast<const void*>(k_dalpha_softmax_group), (int)big_lds)) return DCHAG_ERR_LAUNCH;
    k_dalpha_softmax_group<<<dim3((unsigned)items), 256, big_lds, st>>>(Cin, N, D, heads, g, G, z, w, alpha, ds);
    return launch_status();
  }
  const long T_total = (long)B * Cin * N;
  k_dalpha<bf16><<<dim3((unsigned)((T_total + 3) / 4)), 256, 0, st>>>(T_total, Cin, N, D, heads, g, G, z, w, ds);
  int rc = launch_status();
  if (rc) return rc;
  const long total = (long)B * G * N * heads;
  k_softmax_group_backward<<<dim3((unsigned)((total + 255) / 256)), 256, 0, st>>>(Cin, N, heads, g, G, total, alpha, ds);
  return launch_status();
}

// True when one kernel (k_tokens_backward_fused) takes the whole reverse step at the tokens of a level -- ds, the token
// gradients and the key-path partial sums: the shapes of the MFMA token-gradient path with at most 16 heads,
// D <= 2048 and groups of at most 32 channels.  DCHAG_TOKENS_UNFUSED (debugging aid) keeps the three kernels apart.
inline bool tokens_fused(int B, int Cin, int N, int D, int heads, int g) {
  const int G = groups_of(Cin, g);
  const size_t lds = (size_t)2 * dz_patches(B, G, N, D, g) * g * 16 * 4;
  return D % 256 == 0 && D <= 2048 && heads <= 16 && std::min(g, Cin) <= 32 && lds <= 128 * 1024 &&
         !dbg(SW_DZ_VALU) && !dbg(SW_GENERIC_LEVEL) && !dbg(SW_TOKENS_UNFUSED) &&
         !dbg(SW_RPART_VALU);
}
inline int sum_key_path_partials(int B, int G, int n_tiles, int heads, int D, const float* rpart, float* r,
                                 hipStream_t st) {
  const long per = (long)heads * D;
  k_sum_partials<<<dim3((unsigned)((per + 63) / 64), G), 1024, 0, st>>>(B, G, n_tiles, per, rpart, r);
  return launch_status();
}
inline int tokens_backward_fused(int B, int Cin, int N, int D, int heads, int g, const bf16* z, const bf16* w,
                                 const float* alpha, const bf16* Mb, bf16* dz, float* r, float* rpart, hipStream_t st) {
  const int G = groups_of(Cin, g);
  const int pt = dz_patches(B, G, N, D, g);
  const int n_tiles = (N + pt - 1) / pt;
  int rc;
  {
    StageTimer tm(DCHAG_STAGE_BWD_TOKENS, st);
    const dim3 grid((unsigned)n_tiles, G, B);
    const bool small = std::min(g, Cin) <= 16;
    if (D <= 1024) {
      if (small) k_tokens_backward_fused<1, 1><<<grid, 512, 0, st>>>(Cin, N, D, heads, g, pt, z, w, alpha, Mb, dz, rpart);
      else k_tokens_backward_fused<2, 1><<<grid, 512, 0, st>>>(Cin, N, D, heads, g, pt, z, w, alpha, Mb, dz, rpart);
    } else {
      if (small) k_tokens_backward_fused<1, 2><<<grid, 512, 0, st>>>(Cin, N, D, heads, g, pt, z, w, alpha, Mb, dz, rpart);
      else k_tokens_backward_fused<2, 2><<<grid, 512, 0, st>>>(Cin, N, D, heads, g, pt, z, w, alpha, Mb, dz, rpart);
    }
    if ((rc = launch_status())) return rc;
  }
  StageTimer tm(DCHAG_STAGE_BWD_KEY_QUERY, st);
  return sum_key_path_partials(B, G, n_tiles, heads, D, rpart, r, st);
}

// dz (value and key path) and r[k][a][:] = sum over the group's tokens of ds[., a] z[., :].
template <typename T>
int tokens_backward_generic(int B, int Cin, int N, int D, int heads, int g, const T* zin, const T* w, const float* alpha,
                            const float* ds, const float* Mf, T* dz, float* r, bool want_r, hipStream_t st) {
  const int G = groups_of(Cin, g);
  int rc;
  {
    StageTimer tm(DCHAG_STAGE_BWD_TOKENS, st);
    k_dz_attention<T><<<dim3(Cin, N, B), 256, 0, st>>>(Cin, N, D, heads, g, G, alpha, ds, w, Mf, dz);
    if ((rc = launch_status())) return rc;
  }
  if (!want_r) return DCHAG_OK;
  StageTimer tm(DCHAG_STAGE_BWD_KEY_QUERY, st);
  GemmDesc d{};
  d.M = heads; d.N = D; d.K = g * N; d.nb = B; d.nk = G; d.na = 1; d.reduce_b = 1;
  d.ragged = 2; d.ragged_total = Cin * N; d.ragged_nominal = g * N;
  d.A = {(long)Cin * N * heads, (long)g * N * heads, 0, 1, (long)heads};
  d.Bm = {(long)Cin * N * D, (long)g * N * D, 0, (long)D, 1};
  d.C = {0, (long)heads * D, 0, (long)D, 1};
  d.scale = 1.f;
  return launch_gemm<float, T, float>(d, ds, zin, nullptr, r, st);
}

inline int tokens_backward(int B, int Cin, int N, int D, int heads, int g, const float* zin, const float* w,
                           const float* alpha, const float* ds, const float* Mf, const bf16*, float* dz, float* r,
                           float*, bool want_r, hipStream_t st) {
  return tokens_backward_generic<float>(B, Cin, N, D, heads, g, zin, w, alpha, ds, Mf, dz, r, want_r, st);
}
inline int tokens_backward(int B, int Cin, int N, int D, int heads, int g, const bf16* zin, const bf16* w,
                           const float* alpha, const float* ds, const float* Mf, const bf16* Mb, bf16* dz, float* r,
                           float* rpart, bool want_r, hipStream_t st) {
  const int G = groups_of(Cin, g);
  const int pt = dz_patches(B, G, N, D, g);
  const size_t lds = (size_t)2 * pt * g * 16 * 4;
  const bool mfma = D % 256 == 0 && heads <= 32 && !dbg(SW_DZ_VALU);
  if ((!mfma && heads > 16) || D % 4 || lds > 128 * 1024 || dbg(SW_GENERIC_LEVEL))
    return tokens_backward_generic<bf16>(B, Cin, N, D, heads, g, zin, w, alpha, ds, Mf, dz, r, want_r, st);
  const int n_tiles = (N + pt - 1) / pt;
  int rc;
  {
    StageTimer tm(DCHAG_STAGE_BWD_TOKENS, st);
    const dim3 grid((unsigned)(n_tiles * ((D + 1023) / 1024)), G, B);
    if (mfma) {
      if (heads <= 16) k_dz_mfma<1><<<grid, 256, 0, st>>>(Cin, N, D, heads, g, n_tiles, pt, alpha, ds, w, Mb, dz);
      else k_dz_mfma<2><<<grid, 256, 0, st>>>(Cin, N, D, heads, g, n_tiles, pt, alpha, ds, w, Mb, dz);
      if ((rc = launch_status())) return rc;
      if (want_r) {                                               // DCHAG_RPART_VALU (debugging aid): vector-ALU sums
        const bool valu = dbg(SW_RPART_VALU) != nullptr;
        const size_t rl = (size_t)pt * g * (heads <= 16 ? 16 : 32) * 4;
        auto rk = valu ? (heads <= 16 ? k_rpart_bf16<1> : k_rpart_bf16<2>)
                       : (heads <= 16 ? k_rpart_mfma<1> : k_rpart_mfma<2>);
        const size_t rlds = valu ? lds / 2 : rl;
        if (ensure_dynamic_lds(reinterpret_cast<const void*>(rk), (int)rlds)) return DCHAG_ERR_LAUNCH;
        rk<<<grid, 256, rlds, st>>>(Cin, N, D, heads, g, n_tiles, pt, ds, zin, rpart);
        if ((rc = launch_status())) return rc;
      }
    } else {
      if (ensure_dynamic_lds(reinterpret_cast<const void*>(k_dz_rpart_bf16), (int)lds)) return DCHAG_ERR_LAUNCH;
      k_dz_rpart_bf16<<<grid, 256, lds, st>>>(Cin, N, D, heads, g, n_tiles, pt, alpha, ds, zin, w, Mb, dz, rpart);
      if ((rc = launch_status())) return rc;
    }
  }
  if (!want_r) return DCHAG_OK;
  StageTimer tm(DCHAG_STAGE_BWD_KEY_QUERY, st);
  return sum_key_path_partials(B, G, n_tiles, heads, D, rpart, r, st);
}

// Rank-one weight gradient out[k][i][:] = scale * rowv[k][i] * colv[k][i / rows_per_vec][:]: 16 bytes per thread where
// the rows allow it.
template <typename TV, typename T>
int outer_rows(int D, int G, int rows_per_vec, float scale, const float* rowv, const TV* colv, T* out, hipStream_t st) {
  const bool vec = D % 8 == 0 && !((reinterpret_cast<uintptr_t>(colv) | reinterpret_cast<uintptr_t>(out)) & 15) &&
                   !dbg(SW_GEMM_SCALAR_STORES);
  if (vec) {
    const long chunks = (long)D * (D / 8);
    k_outer_rows_vec<TV, T><<<dim3((unsigned)((chunks + 2047) / 2048), G), 256, 0, st>>>(D, rows_per_vec, scale, rowv,
                                                                                       colv, out);
  } else {
    k_outer_rows<TV, T><<<dim3((D + 255) / 256, D, G), 256, 0, st>>>(D, rows_per_vec, scale, rowv, colv, out);
  }
  return launch_status();
}

// Reverse of one attention level.  dy is the gradient at the level's output [B,G,N,D]; dz receives the
// gradient at its input [B,Cin,N,D].
template <typename T>
int attention_level_backward(int B, int Cin, int N, int D, int heads, const dchag_level* lv,
                             const dchag_level_grads* gr, const T* zin, const T* dy, T* dz, const LevelBufs<T>& lb,
                             float* dalpha, T* w, T* d_o, float* r, float* dQ, float* rpart, hipStream_t st) {
  const int g = lv->group_size, G = groups_of(Cin, g), dh = D / heads;
  const T* Wv = static_cast<const T*>(lv->Wv);
  const T* Wo = static_cast<const T*>(lv->Wo);
  const RowBlocks rbo{G, G * N, N};
  const long sBG = (long)G * N * D, sG = (long)N * D;          // strides of a [B,G,N,D] tensor
  const long uB = (long)G * N * heads * D, uG = (long)N * heads * D;
  int rc;
  {
    StageTimer tm(DCHAG_STAGE_BWD_OPROJ, st);
    {                                                           // dWo[k][i][j] = sum_{b,n} dy[..,i] o[..,j];  dbo = sum dy
      GemmDesc d{};
      d.M = D; d.N = D; d.K = N; d.nb = B; d.nk = G; d.na = 1; d.reduce_b = 1;
      d.A = {sBG, sG, 0, 1, (long)D};
      d.Bm = {sBG, sG, 0, (long)D, 1};
      d.C = {0, (long)D * D, 0, (long)D, 1};
      d.scale = 1.f;
      d.rs_sk = D;
      if ((rc = gemm_with_bias_grad(d, B, D, rbo, dy, lb.o, static_cast<T*>(gr->dWo), static_cast<T*>(gr->dbo), st)))
        return rc;
    }
    GemmDesc d{};                                               // d_o[.., j] = sum_i dy[.., i] Wo[k][i][j]
    d.M = N; d.N = D; d.K = D; d.nb = B; d.nk = G; d.na = 1;
    d.A = {sBG, sG, 0, (long)D, 1};
    d.Bm = {0, (long)D * D, 0, (long)D, 1};
    d.C = {sBG, sG, 0, (long)D, 1};
    d.scale = 1.f;
    if ((rc = gemm_tt(d, dy, Wo, nullptr, d_o, st))) return rc;
  }
  {
    StageTimer tm(DCHAG_STAGE_BWD_VALUE, st);
    {                                                           // dWv[k][a*dh+i][j] = sum_{b,n} d_o[.., a*dh+i] u[.., a, j]
      GemmDesc d{};                                             // dbv = sum d_o
      d.M = dh; d.N = D; d.K = N; d.nb = B; d.nk = G; d.na = heads; d.reduce_b = 1;
      d.A = {sBG, sG, (long)dh, 1, (long)D};
      d.Bm = {uB, uG, (long)D, (long)heads * D, 1};
      d.C = {0, (long)D * D, (long)dh * D, (long)D, 1};
      d.scale = 1.f;
      d.rs_sk = D; d.rs_sa = dh;
      if ((rc = gemm_with_bias_grad(d, B, D, rbo, d_o, lb.u, static_cast<T*>(gr->dWv), static_cast<T*>(gr->dbv), st)))
        return rc;
    }
    GemmDesc d{};                                               // w[.., a, j] = sum_i d_o[.., a*dh+i] Wv[k][a*dh+i][j]
    d.M = N; d.N = D; d.K = dh; d.nb = B; d.nk = G; d.na = heads;
    d.A = {sBG, sG, (long)dh, (long)D, 1};
    d.Bm = {0, (long)D * D, (long)dh * D, (long)D, 1};
    d.C = {uB, uG, (long)D, (long)heads * D, 1};
    d.scale = 1.f;
    if ((rc = gemm_tt(d, d_o, Wv, nullptr, w, st))) return rc;
  }
  const bool want_q = gr->dWq || gr->dbq || gr->dquery;
  const bool want_r = gr->dWk || want_q;
  bool fused = false;
  if constexpr (std::is_same<T, bf16>::value) {
    if (want_r && tokens_fused(B, Cin, N, D, heads, g)) {
      if ((rc = tokens_backward_fused(B, Cin, N, D, heads, g, zin, w, lb.alpha, lb.Mb, dz, r, rpart, st))) return rc;
      fused = true;
    }
  }
  if (!fused) {
    {
      StageTimer tm(DCHAG_STAGE_BWD_SOFTMAX, st);
      if ((rc = softmax_backward(B, Cin, N, D, heads, g, zin, w, lb.alpha, dalpha, st))) return rc;
    }
    if ((rc = tokens_backward(B, Cin, N, D, heads, g, zin, w, lb.alpha, dalpha, lb.Mf, lb.Mb, dz, r, rpart, want_r, st)))
      return rc;
  }
  StageTimer tm(DCHAG_STAGE_BWD_KEY_QUERY, st);
  if (gr->dbk) {
    const long n = (long)G * D;
    k_fill_zero<T><<<dim3((unsigned)((n + 255) / 256)), 256, 0, st>>>(n, static_cast<T*>(gr->dbk));
    if ((rc = launch_status())) return rc;
  }
  if (gr->dWk && (rc = outer_rows<float, T>(D, G, dh, 1.f / sqrtf((float)dh), lb.Qp, r, static_cast<T*>(gr->dWk), st)))
    return rc;
  if (!want_q) return DCHAG_OK;
  k_query_grad<T><<<dim3((D + 3) / 4, G), 256, 0, st>>>(D, heads, static_cast<const T*>(lv->Wk), r, dQ,
                                                        static_cast<T*>(gr->dbq));
  if ((rc = launch_status())) return rc;
  if (gr->dWq && (rc = outer_rows<T, T>(D, G, D, 1.f, dQ, static_cast<const T*>(lv->query), static_cast<T*>(gr->dWq), st)))
    return rc;
  if (gr->dquery) {
    k_query_input_grad<T><<<dim3((D + 63) / 64, G), 1024, 0, st>>>(D, static_cast<const T*>(lv->Wq), dQ,
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
  const bool vec = D % 8 == 0 && Cin <= 65535 && B <= 65535 && !dbg(SW_GEMM_SCALAR_STORES) &&
                   !((reinterpret_cast<uintptr_t>(lv->Wv) | reinterpret_cast<uintptr_t>(dy) |
                      reinterpret_cast<uintptr_t>(dz) | reinterpret_cast<uintptr_t>(zin) |
                      reinterpret_cast<uintptr_t>(gr->dWv)) & 15);
  if (vec)
    k_channel_mix_dz_vec<T><<<dim3((N + 15) / 16, Cin, B), 256, 0, st>>>(Cin, N, D, g, G, static_cast<const T*>(lv->Wv),
                                                                        dy, dz);
  else
    k_channel_mix_dz<T><<<dim3((unsigned)((total + 255) / 256)), 256, 0, st>>>(total, Cin, N, D, g, G,
                                                                              static_cast<const T*>(lv->Wv), dy, dz);
  if ((rc = launch_status())) return rc;
  if (gr->dWv) {
    if (vec)
      k_channel_mix_dw_vec<T><<<dim3((D + 1023) / 1024, G * g), 256, 0, st>>>(B, Cin, N, D, g, G, zin, dy,
                                                                             static_cast<T*>(gr->dWv));
    else
      k_channel_mix_dw<T><<<dim3((D + 63) / 64, G * g), 256, 0, st>>>(B, Cin, N, D, g, G, zin, dy,
                                                                      static_cast<T*>(gr->dWv));
    if ((rc = launch_status())) return rc;
  }
  if (gr->dbv) return colsum<T>(B, D, RowBlocks{G, G * N, N}, dy, static_cast<T*>(gr->dbv), st);
  return DCHAG_OK;
}

// Copy between the image layout and patch rows, in runs of 8, 4, 2 or 1 pixels (the widest that divides p).
template <typename T, bool TO_IMAGE>
int patch_rows(long pixels, int H, int W, int p, T* img, T* patches, hipStream_t st) {
  const int V = (p % 8 == 0 && sizeof(T) == 2) ? 8 : (p % 4 == 0 ? 4 : (p % 2 == 0 ? 2 : 1));
  const long runs = pixels / V;
  const dim3 grid((unsigned)((runs + 255) / 256));
  if (V == 8) k_patch_rows<T, 8, TO_IMAGE><<<grid, 256, 0, st>>>(runs, H, W, p, img, patches);
  else if (V == 4) k_patch_rows<T, 4, TO_IMAGE><<<grid, 256, 0, st>>>(runs, H, W, p, img, patches);
  else if (V == 2) k_patch_rows<T, 2, TO_IMAGE><<<grid, 256, 0, st>>>(runs, H, W, p, img, patches);
  else k_patch_rows<T, 1, TO_IMAGE><<<grid, 256, 0, st>>>(runs, H, W, p, img, patches);
  return launch_status();
}

template <typename T>
int tokenizer_backward(int B, int C, int H, int W, int p, int D, const T* x, const T* We, const T* dt_, T* dx,
                       T* dWe, T* dtok_bias, T* patches, hipStream_t st) {
  const int N = (H / p) * (W / p), pp = p * p;
  int rc;
  StageTimer tm(DCHAG_STAGE_BWD_TOKENIZE, st);
  const long pixels = (long)B * C * H * W;
  if (pixels > ((long)1 << 39)) return DCHAG_ERR_SHAPE;
  if (dWe && (rc = patch_rows<T, false>(pixels, H, W, p, const_cast<T*>(x), patches, st))) return rc;
  {
    GemmDesc d{};                                               // dWe[c][d][kk] = sum_{b,n} dt[b,c,n,d] patch[b,c,n,kk]
    d.M = D; d.N = pp; d.K = N; d.nb = B; d.nk = C; d.na = 1; d.reduce_b = 1;   // dtok_bias[c][d] = sum_{b,n} dt
    d.A = {(long)C * N * D, (long)N * D, 0, 1, (long)D};
    d.Bm = {(long)C * N * pp, (long)N * pp, 0, (long)pp, 1};
    d.C = {0, (long)D * pp, 0, (long)pp, 1};
    d.scale = 1.f;
    d.rs_sk = D;
    if ((rc = gemm_with_bias_grad(d, B, D, RowBlocks{C, C * N, N}, dt_, patches, dWe, dtok_bias, st))) return rc;
  }
  if (dx) {
    GemmDesc d{};                                               // dpatch[b,c,n,kk] = sum_d dt[b,c,n,d] We[c][d][kk]
    d.M = N; d.N = pp; d.K = D; d.nb = B; d.nk = C; d.na = 1;
    d.A = {(long)C * N * D, (long)N * D, 0, (long)D, 1};
    d.Bm = {0, (long)D * pp, 0, (long)pp, 1};
    d.C = {(long)C * N * pp, (long)N * pp, 0, (long)pp, 1};
    d.scale = 1.f;
    if ((rc = gemm_tt(d, dt_, We, nullptr, patches, st))) return rc;
    if ((rc = patch_rows<T, true>(pixels, H, W, p, dx, patches, st))) return rc;
  }
  return DCHAG_OK;
}

// A linear first level needs neither its input tokens nor their gradients in HBM (see k_linear_first_grads): true
// when the reverse sweep takes that route.  The products' intermediates (P fp32, the scaled weights, S) go where the
// tokens would have been.  DCHAG_LINEAR_TOKENS (debugging aid) keeps the route through the tokens.
inline bool linear_first_without_tokens(dchag_dtype dt, int B, int C, int N, int pp, int D, int n_levels,
                                        const dchag_level* levels) {
  if (dt != DCHAG_BF16 || n_levels < 2 || levels[0].kind != DCHAG_LEVEL_LINEAR || dbg(SW_LINEAR_TOKENS))
    return false;
  const int cpr = pp / 8;
  if (pp % 8 || (cpr & (cpr - 1)) || cpr > 64 || D % 8) return false;
  const size_t G = groups_of(C, levels[0].group_size);
  const size_t need = align_up((size_t)C * D * pp * 4) + align_up((size_t)C * D * pp * 2) + align_up(G * D * 4);
  return need <= align_up((size_t)B * C * N * D * 2);
}

// One product per channel with the group's operand shared by its members: full groups in one launch, a short last
// group in a second one.  dA / dB / dC: element offsets per channel of the three operands (0 for the shared one).
template <typename TC>
int gemm_per_channel(GemmDesc d, int C, int g, long a_grp, long b_ch, long c_ch, const bf16* A, const bf16* Bm, TC* Cm,
                     hipStream_t st) {
  const int full = C / g, tail = C % g;
  int rc = DCHAG_OK;
  d.A.sk = a_grp; d.A.sa = 0;
  d.Bm.sk = b_ch * g; d.Bm.sa = b_ch;
  d.C.sk = c_ch * g; d.C.sa = c_ch;
  if (full) {
    d.nk = full; d.na = g;
    if ((rc = launch_gemm_bf16<TC>(d, A, Bm, nullptr, Cm, st))) return rc;
  }
  if (tail) {
    d.nk = 1; d.na = tail;
    rc = launch_gemm_bf16<TC>(d, A + a_grp * full, Bm + b_ch * g * full, nullptr, Cm + c_ch * g * full, st);
  }
  return rc;
}

// Reverse of (tokenizer, linear first level) given dy [B,G,N,D]: dmix / dbias of the level, dWe, dtok_bias, dx.
inline int linear_first_backward(int B, int C, int H, int W, int p, int D, const dchag_level* lv,
                                 const dchag_level_grads* gr, const bf16* x, const bf16* We, const bf16* be,
                                 const bf16* ce, const bf16* dy, bf16* dx, bf16* dWe, bf16* dtok_bias, bf16* patches,
                                 unsigned char* scratch, hipStream_t st) {
  const int N = (H / p) * (W / p), pp = p * p, g = lv->group_size, G = groups_of(C, g);
  float* P = reinterpret_cast<float*>(scratch);
  bf16* Ws = reinterpret_cast<bf16*>(scratch + align_up((size_t)C * D * pp * 4));
  float* S = reinterpret_cast<float*>(scratch + align_up((size_t)C * D * pp * 4) + align_up((size_t)C * D * pp * 2));
  const long pixels = (long)B * C * H * W;
  if (pixels > ((long)1 << 39)) return DCHAG_ERR_SHAPE;
  int rc;
  bf16* dmix = static_cast<bf16*>(gr->dWv);
  const bool want_p = dWe || dmix;
  {
    StageTimer tm(DCHAG_STAGE_BWD_CHANNEL_MIX, st);
    k_colsum<bf16, float><<<dim3((D + 63) / 64, G), 1024, 0, st>>>(B, D, RowBlocks{G, G * N, N}, dy, S);
    if ((rc = launch_status())) return rc;
    if (gr->dbv && (rc = colsum<bf16>(B, D, RowBlocks{G, G * N, N}, dy, static_cast<bf16*>(gr->dbv), st))) return rc;
    if (dmix && G * g > C) {                                      // members a short last group lacks: zero
      const long n = (long)(G * g - C) * D;
      k_fill_zero<bf16><<<dim3((unsigned)((n + 255) / 256)), 256, 0, st>>>(n, dmix + (size_t)C * D);
      if ((rc = launch_status())) return rc;
    }
  }
  StageTimer tm(DCHAG_STAGE_BWD_TOKENIZE, st);
  if (want_p) {
    if ((rc = patch_rows<bf16, false>(pixels, H, W, p, const_cast<bf16*>(x), patches, st))) return rc;
    GemmDesc d{};                                                 // P[c][d][kk] = sum_{b,n} dy[b,k,n,d] patch[b,c,n,kk]
    d.M = D; d.N = pp; d.K = N; d.nb = B; d.reduce_b = 1;
    d.A = {(long)G * N * D, 0, 0, 1, (long)D};
    d.Bm = {(long)C * N * pp, 0, 0, (long)pp, 1};
    d.C = {0, 0, 0, (long)pp, 1};
    d.scale = 1.f;
    if ((rc = gemm_per_channel<float>(d, C, g, (long)N * D, (long)N * pp, (long)D * pp, dy, patches, P, st))) return rc;
  }
  {
    const long chunks = (long)C * D * (pp / 8);
    k_linear_first_grads<<<dim3((unsigned)((chunks + 255) / 256)), 256, 0, st>>>(
        chunks, C, D, pp, g, want_p ? P : nullptr, S, We, be, ce, static_cast<const bf16*>(lv->Wv), dWe, dtok_bias, dmix,
        dx ? Ws : nullptr);
    if ((rc = launch_status())) return rc;
  }
  if (dx) {
    GemmDesc d{};                                                 // dpatch[b,c,n,kk] = sum_d dy[b,k,n,d] Ws[c][d][kk]
    d.M = N; d.N = pp; d.K = D; d.nb = B;
    d.A = {(long)G * N * D, 0, 0, (long)D, 1};
    d.Bm = {0, 0, 0, (long)pp, 1};
    d.C = {(long)C * N * pp, 0, 0, (long)pp, 1};
    d.scale = 1.f;
    if ((rc = gemm_per_channel<bf16>(d, C, g, (long)N * D, (long)D * pp, (long)N * pp, dy, Ws, patches, st))) return rc;
    if ((rc = patch_rows<bf16, true>(pixels, H, W, p, dx, patches, st))) return rc;
  }
  return DCHAG_OK;
}

// The two halves of a training step.  keep_forward fills the workspace with what the reverse sweep reads
// (tokens, and per level: inputs, folded keys, softmax weights, per-head token averages, pre-projection outputs)
// and, if asked, writes the path's output; reverse_sweep walks the levels backwards over that workspace.
template <typename T>
int keep_forward(dchag_dtype dt, int B, int C, int H, int W, int p, int D, int heads, const void* x, const void* We,
                 const void* be, const void* ce, int n_levels, const dchag_level* levels, const int32_t* gs, void* out,
                 unsigned char* ws, const BackwardWs& w, hipStream_t st) {
  const int N = (H / p) * (W / p);
  set_level(0);
  int rc;
  const T* zin = reinterpret_cast<const T*>(ws + w.tokens);
  int c_in = C, first = 0;
  if constexpr (std::is_same<T, bf16>::value) {
    // a linear first level whose reverse needs no tokens: tokenizer and level in one kernel, nothing else kept
    if (linear_first_without_tokens(dt, B, C, N, p * p, D, n_levels, levels) && tokenize_mix_ok(dt, levels, p * p, D)) {
      set_level(1);
      const KeptLevel kl = kept_level(dt, B, C, N, D, heads, gs[0], true, true);
      bf16* y = reinterpret_cast<bf16*>(ws + w.kept[0] + kl.y);
      if ((rc = tokenize_mix_forward(B, C, H, W, p, D, x, We, be, ce, &levels[0], y, st))) return rc;
      zin = y;
      c_in = groups_of(C, gs[0]);
      first = 1;
    }
  }
  if (!first && (rc = dchag_tokenize(dt, B, C, H, W, p, D, x, We, be, ce, ws + w.tokens, st))) return rc;
  const PixelScores px = pixel_scores_of<T>(x, We, be, ce, H, W, p, ws, w.ms, w.msb, w.cs, w.mft);
  const bool use_px = dt == DCHAG_BF16 && train_fast(dt, D, heads) && pixel_scores_ok(p, heads);
  // every attention level's weight-only prep in ONE launch, straight into the level's kept buffers
  int phase = 0;
  if constexpr (std::is_same<T, bf16>::value) {
    if (train_fast(dt, D, heads)) {
      KeyPrepJob jobs[16];
      int nj = 0, cl = c_in;
      for (int l = first; l < n_levels; ++l) {
        const bool linear = levels[l].kind == DCHAG_LEVEL_LINEAR;
        const int G = groups_of(cl, gs[l]);
        if (!linear) {
          const LevelBufs<bf16> lb = level_bufs<bf16>(ws + w.kept[l], kept_level(dt, B, cl, N, D, heads, gs[l], false,
                                                                                 l + 1 < n_levels));
          jobs[nj++] = KeyPrepJob{&levels[l], G, PrepBufs{lb.Qp, lb.Mf, lb.Mb}, (l == 0 && use_px) ? px.MfT : nullptr};
        }
        cl = G;
      }
      set_level(0);
      if (nj && (rc = launch_query_keys(D, heads, jobs, nj, st))) return rc;
      if (nj) phase = 3;
    }
  }
  for (int l = first; l < n_levels; ++l) {
    set_level(l + 1);
    const bool linear = levels[l].kind == DCHAG_LEVEL_LINEAR, last = l + 1 == n_levels;
    const KeptLevel kl = kept_level(dt, B, c_in, N, D, heads, gs[l], linear, !last);
    unsigned char* lw = ws + w.kept[l];
    T* y = last ? static_cast<T*>(out) : reinterpret_cast<T*>(lw + kl.y);     // out may be NULL: the reverse sweep
    if (linear)                                                               // does not read the last output
      rc = run_level_linear<T>(B, c_in, N, D, &levels[l], zin, y, st);
    else
      rc = folded_level_forward<T>(dt, B, c_in, N, D, heads, &levels[l], zin, y, level_bufs<T>(lw, kl), st,
                                   (l == 0 && use_px) ? &px : nullptr, phase);
    if (rc) return rc;
    c_in = groups_of(c_in, gs[l]);
    zin = y;
  }
  return DCHAG_OK;
}

template <typename T>
int reverse_sweep(dchag_dtype dt, int B, int C, int H, int W, int p, int D, int heads, const void* x, const void* We,
                  const void* be, const void* ce, int n_levels, const dchag_level* levels, const int32_t* gs,
                  const void* dout, void* dx, void* dWe,
                  void* dtok_bias, const dchag_level_grads* grads, unsigned char* ws, const BackwardWs& w,
                  hipStream_t st) {
  const int N = (H / p) * (W / p);
  const T* zins[16];
  KeptLevel kl[16];
  int cins[17];
  cins[0] = C;
  zins[0] = reinterpret_cast<const T*>(ws + w.tokens);
  for (int l = 0; l < n_levels; ++l) {
    const bool linear = levels[l].kind == DCHAG_LEVEL_LINEAR, last = l + 1 == n_levels;
    kl[l] = kept_level(dt, B, cins[l], N, D, heads, gs[l], linear, !last);
    cins[l + 1] = groups_of(cins[l], gs[l]);
    zins[l + 1] = last ? nullptr : reinterpret_cast<const T*>(ws + w.kept[l] + kl[l].y);
  }
  int rc;
  const T* dy = static_cast<const T*>(dout);
  bool no_tokens = false;
  if constexpr (std::is_same<T, bf16>::value) no_tokens = linear_first_without_tokens(dt, B, C, N, p * p, D, n_levels, levels);
  for (int l = n_levels - 1; l >= 0; --l) {
    set_level(l + 1);
    unsigned char* lw = ws + w.kept[l];
    T* dz = reinterpret_cast<T*>(ws + w.dz[l & 1]);
    if constexpr (std::is_same<T, bf16>::value) {
      if (l == 0 && no_tokens) {
        rc = linear_first_backward(B, C, H, W, p, D, &levels[0], &grads[0], static_cast<const bf16*>(x),
                                   static_cast<const bf16*>(We), static_cast<const bf16*>(be),
                                   static_cast<const bf16*>(ce), dy, static_cast<bf16*>(dx), static_cast<bf16*>(dWe),
                                   static_cast<bf16*>(dtok_bias), reinterpret_cast<bf16*>(ws + w.patches),
                                   ws + w.tokens, st);
        set_level(0);
        return rc;
      }
    }
    if (levels[l].kind == DCHAG_LEVEL_LINEAR)
      rc = linear_level_backward<T>(B, cins[l], N, D, &levels[l], &grads[l], zins[l], dy, dz, st);
    else
      rc = attention_level_backward<T>(B, cins[l], N, D, heads, &levels[l], &grads[l], zins[l], dy, dz,
                                       level_bufs<T>(lw, kl[l]), reinterpret_cast<float*>(ws + w.dalpha),
                                       reinterpret_cast<T*>(ws + w.w), reinterpret_cast<T*>(ws + w.d_o),
                                       reinterpret_cast<float*>(ws + w.r), reinterpret_cast<float*>(ws + w.dq),
                                       reinterpret_cast<float*>(ws + w.rpart), st);
    if (rc) return rc;
    dy = dz;
  }
  set_level(0);
  if (!dx && !dWe && !dtok_bias) return DCHAG_OK;
  return tokenizer_backward<T>(B, C, H, W, p, D, static_cast<const T*>(x), static_cast<const T*>(We), dy,
                               static_cast<T*>(dx), static_cast<T*>(dWe), static_cast<T*>(dtok_bias),
                               reinterpret_cast<T*>(ws + w.patches), st);
}
