/*
 * D-CHAG forward oracle: plain fp64 CPU definition.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the yardstick the GPU library is checked against.  It shares no
 * code with that library and must never be linked into, called from, or used as
 * a fallback by the product path.  It is slow on purpose: every quantity is
 * computed exactly as the definition states it, one patch at a time, with no
 * blocking, fusion, folding of weights or reordering.
 *
 * What it computes (paper Section 2.1, "The Channel Aggregation Module";
 * Section 3.2, "Hierarchical Cross-Channel Aggregation"; Section 3.3, D-CHAG):
 *
 *   - tokenization: every p x p patch of every channel is embedded on its own by
 *     that channel's own linear map (a 2-D convolution whose kernel and stride
 *     are the patch size), plus that channel's ID embedding (Section 2.1);
 *   - channel aggregation: a cross-attention layer reduces the tokens of a set
 *     of channels at one spatial patch to one token (Section 2.1).  The paper
 *     gives no formula; the reading taken is standard multi-head scaled
 *     dot-product attention with one learned query per layer, projections
 *     W_q, W_k, W_v, W_o with optional biases, scale 1/sqrt(D/heads), no norm,
 *     no residual;
 *   - hierarchy: the channels are split in contiguous groups of at most g
 *     ("up to" g, Section 3.2), each group has its own layer, the outputs of a
 *     level are the inputs of the next, and the last level is one
 *     cross-attention layer over everything that is left (Section 3.3);
 *   - D-CHAG-L (Sections 3.2, 3.3): a partial-aggregation level may be a
 *     "lightweight linear layer" instead of cross-attention, the last level
 *     stays cross-attention.  The paper does not define that layer beyond
 *     saying that it has fewer parameters than a cross-attention layer; the
 *     reading taken is a learned mixing along the channel axis with one weight
 *     per member and feature:  y = sum_c w[c] * z[c] + b  (elementwise in the
 *     feature), g*D + D parameters per group.
 *
 * Inputs are float (exactly representable bf16 or fp32 values); all arithmetic
 * and all outputs are double.  Rows are summed left to right.
 *
 * The second half of the file is the backward pass of the same path (the paper
 * is a training method; Section 3.3): the chain rule through the steps above in
 * reverse, one patch and one group at a time.
 *
 * Pins: the tests under tests/ (not marked gpu) check this file against a
 * library grouped conv2d, a library multi-head attention with a length-1
 * query, a pure-Python brute force in another loop order, and the invariants
 * the definition fixes; the backward against central finite differences of
 * the (pinned) forward, against a library autograd through the library
 * conv2d / multi-head-attention composition, and against the identities the
 * derivative fixes.  The paper prints no worked numerical example, so there
 * is no pin to values of the paper itself.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
  int32_t group_size;                  /* nominal g; the last group may be shorter            */
  int32_t kind;                        /* 0: cross-attention; 1: linear mixing (Wv = [G,g,D] weights, bv = bias) */
  const float *query;                  /* [G, D]                                               */
  const float *Wq, *Wk, *Wv, *Wo;      /* [G, D, D], row-major (out, in): y = W x              */
  const float *bq, *bk, *bv, *bo;      /* [G, D] or NULL (= 0)                                 */
} oracle_level;

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

void oracle_set_threads(int n) {
#ifdef _OPENMP
  if (n > 0) omp_set_num_threads(n);
#else
  (void)n;
#endif
}

static int groups_of(int c_in, int g) { return (c_in + g - 1) / g; }

/* y = W x + b   with W [rows, cols] float row-major, x double, b float or NULL */
static void affine(const float *W, const float *b, const double *x, int rows, int cols, double *y) {
  for (int i = 0; i < rows; ++i) {
    double acc = 0.0;
    const float *w = W + (size_t)i * cols;
    for (int j = 0; j < cols; ++j) acc += (double)w[j] * x[j];
    y[i] = acc + (b ? (double)b[i] : 0.0);
  }
}

/*
 * Tokens of one patch (Section 2.1): for channel c,
 *   t[c] = W_e[c] . vec(patch) + b_e[c] + e[c],
 * vec() taking the p x p pixels row by row; patch n = (i, j) counts row by row
 * over the (H/p) x (W/p) grid.  W_e[c] is [D, p*p] (a conv2d weight [D,1,p,p]).
 */
static void tokens_of_patch(int C, int H, int W, int p, int D, const float *x_b /* [C,H,W] */,
                            const float *We, const float *be, const float *ce, int n,
                            double *t /* [C, D] */) {
  const int pw = W / p;
  const int pi = n / pw, pj = n % pw;
  const int pp = p * p;
  double *u = (double *)malloc(sizeof(double) * (size_t)pp);
  for (int c = 0; c < C; ++c) {
    const float *img = x_b + (size_t)c * H * W;
    for (int r = 0; r < p; ++r)
      for (int s = 0; s < p; ++s) u[r * p + s] = (double)img[(size_t)(pi * p + r) * W + (pj * p + s)];
    double *tc = t + (size_t)c * D;
    affine(We + (size_t)c * D * pp, be ? be + (size_t)c * D : NULL, u, D, pp, tc);
    if (ce)
      for (int d = 0; d < D; ++d) tc[d] += (double)ce[(size_t)c * D + d];
  }
  free(u);
}

/*
 * One linear partial-aggregation level at one patch (D-CHAG-L, Sections 3.2, 3.3, in the
 * reading stated at the top): group k holds inputs k*g .. min((k+1)*g, c_in)-1 and
 *   y[k][d] = sum over members c of w[k][c - k*g][d] * z[c][d] + b[k][d],
 * with w = lv->Wv laid out [G, g, D] and b = lv->bv [G, D] (or NULL).
 */
static void linear_level_of_patch(int c_in, int D, const oracle_level *lv, const double *z, double *y) {
  const int g = lv->group_size;
  const int G = groups_of(c_in, g);
  for (int k = 0; k < G; ++k) {
    const int c0 = k * g;
    const int c1 = (c0 + g < c_in) ? c0 + g : c_in;
    for (int d = 0; d < D; ++d) {
      double acc = 0.0;
      for (int c = c0; c < c1; ++c)
        acc += (double)lv->Wv[((size_t)k * g + (c - c0)) * D + d] * z[(size_t)c * D + d];
      y[(size_t)k * D + d] = acc + (lv->bv ? (double)lv->bv[(size_t)k * D + d] : 0.0);
    }
  }
}

/*
 * One aggregation level at one patch (Sections 2.1, 3.2): group k holds the
 * inputs k*g .. min((k+1)*g, c_in)-1.  Per group: project the learned query,
 * project every member to a key and a value, per head take the scaled dot
 * products, a softmax over the members, the weighted sum of the values, then
 * the output projection of the concatenated heads.
 * alpha (optional) receives the softmax weights [c_in, heads]; pre (optional)
 * the concatenated heads before W_o, [G, D].
 */
static void level_of_patch(int c_in, int D, int heads, const oracle_level *lv, const double *z /* [c_in, D] */,
                           double *y /* [G, D] */, double *alpha, double *pre) {
  if (lv->kind == 1) {
    linear_level_of_patch(c_in, D, lv, z, y);
    return;
  }
  const int g = lv->group_size;
  const int G = groups_of(c_in, g);
  const int dh = D / heads;
  const double scale = 1.0 / sqrt((double)dh);
  double *Q = (double *)malloc(sizeof(double) * (size_t)D);
  double *K = (double *)malloc(sizeof(double) * (size_t)g * D);
  double *V = (double *)malloc(sizeof(double) * (size_t)g * D);
  double *s = (double *)malloc(sizeof(double) * (size_t)g);
  double *o = (double *)malloc(sizeof(double) * (size_t)D);
  double *qv = (double *)malloc(sizeof(double) * (size_t)D);
  for (int k = 0; k < G; ++k) {
    const int c0 = k * g;
    const int c1 = (c0 + g < c_in) ? c0 + g : c_in;
    const int m = c1 - c0;
    const size_t wo = (size_t)k * D * D, bo = (size_t)k * D;
    for (int d = 0; d < D; ++d) qv[d] = (double)lv->query[bo + d];
    affine(lv->Wq + wo, lv->bq ? lv->bq + bo : NULL, qv, D, D, Q);
    for (int c = 0; c < m; ++c) {
      affine(lv->Wk + wo, lv->bk ? lv->bk + bo : NULL, z + (size_t)(c0 + c) * D, D, D, K + (size_t)c * D);
      affine(lv->Wv + wo, lv->bv ? lv->bv + bo : NULL, z + (size_t)(c0 + c) * D, D, D, V + (size_t)c * D);
    }
    for (int a = 0; a < heads; ++a) {
      const int r0 = a * dh;
      double smax = -INFINITY;
      for (int c = 0; c < m; ++c) {
        double acc = 0.0;
        for (int i = 0; i < dh; ++i) acc += Q[r0 + i] * K[(size_t)c * D + r0 + i];
        s[c] = acc * scale;
        if (s[c] > smax) smax = s[c];
      }
      double den = 0.0;
      for (int c = 0; c < m; ++c) {
        s[c] = exp(s[c] - smax);
        den += s[c];
      }
      for (int c = 0; c < m; ++c) {
        s[c] /= den;
        if (alpha) alpha[(size_t)(c0 + c) * heads + a] = s[c];
      }
      for (int i = 0; i < dh; ++i) {
        double acc = 0.0;
        for (int c = 0; c < m; ++c) acc += s[c] * V[(size_t)c * D + r0 + i];
        o[r0 + i] = acc;
      }
    }
    if (pre) memcpy(pre + (size_t)k * D, o, sizeof(double) * (size_t)D);
    affine(lv->Wo + wo, lv->bo ? lv->bo + bo : NULL, o, D, D, y + (size_t)k * D);
  }
  free(Q); free(K); free(V); free(s); free(o); free(qv);
}

/*
 * Tokens of S sampled patches (sample_b[i], sample_n[i]); tokens is [S, C, D].
 */
int oracle_tokenize(int B, int C, int H, int W, int p, int D, const float *x, const float *We,
                    const float *be, const float *ce, int S, const int32_t *sample_b,
                    const int32_t *sample_n, double *tokens) {
  if (p <= 0 || H % p || W % p) return -2;
  const int N = (H / p) * (W / p);
  for (int i = 0; i < S; ++i)
    if (sample_b[i] < 0 || sample_b[i] >= B || sample_n[i] < 0 || sample_n[i] >= N) return -2;
#pragma omp parallel for schedule(dynamic, 1)
  for (int i = 0; i < S; ++i)
    tokens_of_patch(C, H, W, p, D, x + (size_t)sample_b[i] * C * H * W, We, be, ce, sample_n[i],
                    tokens + (size_t)i * C * D);
  return 0;
}

/*
 * One level on S independent patches: z is [S, c_in, D], y is [S, G, D];
 * alpha [S, c_in, heads] and pre [S, G, D] are optional (NULL to skip).
 */
int oracle_aggregate_level(int S, int c_in, int D, int heads, const oracle_level *lv, const double *z,
                           double *y, double *alpha, double *pre) {
  if (heads <= 0 || D % heads || lv->group_size < 1 || c_in < 1) return -2;
  if (lv->kind != 0 && lv->kind != 1) return -2;
  if (lv->kind == 1 && (alpha || pre)) return -2;      /* a linear level has no softmax weights */
  const int G = groups_of(c_in, lv->group_size);
#pragma omp parallel for schedule(dynamic, 1)
  for (int i = 0; i < S; ++i)
    level_of_patch(c_in, D, heads, lv, z + (size_t)i * c_in * D, y + (size_t)i * G * D,
                   alpha ? alpha + (size_t)i * c_in * heads : NULL, pre ? pre + (size_t)i * G * D : NULL);
  return 0;
}

/*
 * The whole path on S sampled patches: tokenize, then every level in turn; the
 * last level must leave one token.  out is [S, D].
 */
int oracle_forward(int B, int C, int H, int W, int p, int D, int heads, const float *x, const float *We,
                   const float *be, const float *ce, int n_levels, const oracle_level *levels, int S,
                   const int32_t *sample_b, const int32_t *sample_n, double *out) {
  if (p <= 0 || H % p || W % p || heads <= 0 || D % heads || n_levels < 1) return -2;
  const int N = (H / p) * (W / p);
  int c_in = C, c_max = C;
  for (int l = 0; l < n_levels; ++l) {
    if (levels[l].group_size < 1) return -2;
    if (levels[l].kind != 0 && levels[l].kind != 1) return -2;
    c_in = groups_of(c_in, levels[l].group_size);
    if (c_in > c_max) c_max = c_in;
  }
  if (c_in != 1) return -2;
  if (levels[n_levels - 1].kind != 0) return -2;        /* the final layer is always cross-attention (Section 3.3) */
  for (int i = 0; i < S; ++i)
    if (sample_b[i] < 0 || sample_b[i] >= B || sample_n[i] < 0 || sample_n[i] >= N) return -2;
#pragma omp parallel for schedule(dynamic, 1)
  for (int i = 0; i < S; ++i) {
    double *za = (double *)malloc(sizeof(double) * (size_t)c_max * D);
    double *zb = (double *)malloc(sizeof(double) * (size_t)c_max * D);
    tokens_of_patch(C, H, W, p, D, x + (size_t)sample_b[i] * C * H * W, We, be, ce, sample_n[i], za);
    int c = C;
    for (int l = 0; l < n_levels; ++l) {
      level_of_patch(c, D, heads, &levels[l], za, zb, NULL, NULL);
      c = groups_of(c, levels[l].group_size);
      double *t = za; za = zb; zb = t;
    }
    memcpy(out + (size_t)i * D, za, sizeof(double) * (size_t)D);
    free(za); free(zb);
  }
  return 0;
}

/*
 * Positional embedding (Section 2.1: before the aggregated tokens enter the ViT they receive a positional
 * embedding): one learned vector per patch, shared by all batch items, added to the path's output.
 *   out[i][:] += pos[sample_n[i]][:]          pos is [N, D]
 */
int oracle_add_positional(int N, int D, int S, const int32_t *sample_n, const float *pos, double *out) {
  for (int i = 0; i < S; ++i) {
    if (sample_n[i] < 0 || sample_n[i] >= N) return -2;
    for (int d = 0; d < D; ++d) out[(size_t)i * D + d] += (double)pos[(size_t)sample_n[i] * D + d];
  }
  return 0;
}

/* ==========================================================================================
 * Backward pass (the paper trains through this module: Section 3.3 notes that the backward
 * of the partial-channel aggregation needs no communication, i.e. it is the plain reverse of
 * the forward above).  For a scalar loss L with dL/d(out) = dout given on S sampled patches
 * (every other patch has dout = 0 and, the path being independent per patch, contributes
 * nothing), this computes dL/d(every weight) summed over the sampled patches and
 * dL/d(pixels of the sampled patches), by the chain rule through the same steps in reverse.
 * ========================================================================================== */

typedef struct {
  double *dquery;                      /* [G, D]                                               */
  double *dWq, *dWk, *dWv, *dWo;       /* [G, D, D]  (linear level: dWv is [G, g, D])          */
  double *dbq, *dbk, *dbv, *dbo;       /* [G, D]     (linear level: only dbv)                  */
} oracle_level_grad;

/* x += W^T y   with W [rows, cols] float row-major */
static void affine_transposed_add(const float *W, const double *y, int rows, int cols, double *x) {
  for (int i = 0; i < rows; ++i) {
    const float *w = W + (size_t)i * cols;
    const double yi = y[i];
    for (int j = 0; j < cols; ++j) x[j] += (double)w[j] * yi;
  }
}

/* G += y (outer) x   with G [rows, cols] double */
static void outer_add(double *G, const double *y, const double *x, int rows, int cols) {
  for (int i = 0; i < rows; ++i) {
    double *gr = G + (size_t)i * cols;
    const double yi = y[i];
    for (int j = 0; j < cols; ++j) gr[j] += yi * x[j];
  }
}

/*
 * Reverse of one cross-attention layer (group k of a level) at one patch.  z holds the m member
 * tokens [m, D], dy the gradient at the layer's output [D]; dz [m, D] receives the gradient at
 * the members; the weight gradients of group k are accumulated into gr.
 * Forward recap: Q = Wq q + bq; K[c] = Wk z[c] + bk; V[c] = Wv z[c] + bv;
 *   s[c,a] = <Q_a, K_a[c]> / sqrt(dh); alpha = softmax_c s; o_a = sum_c alpha[c,a] V_a[c]; y = Wo o + bo.
 */
static void attention_group_backward(int D, int heads, const oracle_level *lv, int k, int m, const double *z,
                                     const double *dy, double *dz, const oracle_level_grad *gr) {
  const int dh = D / heads;
  const double scale = 1.0 / sqrt((double)dh);
  const size_t wo = (size_t)k * D * D, bo = (size_t)k * D;
  double *qv = (double *)malloc(sizeof(double) * (size_t)D);
  double *Q = (double *)malloc(sizeof(double) * (size_t)D);
  double *K = (double *)malloc(sizeof(double) * (size_t)m * D);
  double *V = (double *)malloc(sizeof(double) * (size_t)m * D);
  double *al = (double *)malloc(sizeof(double) * (size_t)m * heads);    /* alpha[c][a] */
  double *o = (double *)calloc((size_t)D, sizeof(double));
  double *d_o = (double *)calloc((size_t)D, sizeof(double));
  double *dQ = (double *)calloc((size_t)D, sizeof(double));
  double *dK = (double *)malloc(sizeof(double) * (size_t)m * D);
  double *dV = (double *)malloc(sizeof(double) * (size_t)m * D);
  double *dal = (double *)malloc(sizeof(double) * (size_t)m);
  /* forward, kept */
  for (int d = 0; d < D; ++d) qv[d] = (double)lv->query[bo + d];
  affine(lv->Wq + wo, lv->bq ? lv->bq + bo : NULL, qv, D, D, Q);
  for (int c = 0; c < m; ++c) {
    affine(lv->Wk + wo, lv->bk ? lv->bk + bo : NULL, z + (size_t)c * D, D, D, K + (size_t)c * D);
    affine(lv->Wv + wo, lv->bv ? lv->bv + bo : NULL, z + (size_t)c * D, D, D, V + (size_t)c * D);
  }
  for (int a = 0; a < heads; ++a) {
    const int r0 = a * dh;
    double smax = -INFINITY, den = 0.0;
    for (int c = 0; c < m; ++c) {
      double acc = 0.0;
      for (int i = 0; i < dh; ++i) acc += Q[r0 + i] * K[(size_t)c * D + r0 + i];
      al[(size_t)c * heads + a] = acc * scale;
      if (acc * scale > smax) smax = acc * scale;
    }
    for (int c = 0; c < m; ++c) {
      al[(size_t)c * heads + a] = exp(al[(size_t)c * heads + a] - smax);
      den += al[(size_t)c * heads + a];
    }
    for (int c = 0; c < m; ++c) al[(size_t)c * heads + a] /= den;
    for (int i = 0; i < dh; ++i)
      for (int c = 0; c < m; ++c) o[r0 + i] += al[(size_t)c * heads + a] * V[(size_t)c * D + r0 + i];
  }
  /* y = Wo o + bo */
  if (gr->dbo) for (int i = 0; i < D; ++i) gr->dbo[bo + i] += dy[i];
  outer_add(gr->dWo + wo, dy, o, D, D);
  affine_transposed_add(lv->Wo + wo, dy, D, D, d_o);
  /* heads: weighted sum, softmax, scaled dot product */
  for (int a = 0; a < heads; ++a) {
    const int r0 = a * dh;
    double dot = 0.0;
    for (int c = 0; c < m; ++c) {
      double acc = 0.0;
      for (int i = 0; i < dh; ++i) {
        acc += d_o[r0 + i] * V[(size_t)c * D + r0 + i];
        dV[(size_t)c * D + r0 + i] = al[(size_t)c * heads + a] * d_o[r0 + i];
      }
      dal[c] = acc;
      dot += al[(size_t)c * heads + a] * acc;
    }
    for (int c = 0; c < m; ++c) {
      const double ds = al[(size_t)c * heads + a] * (dal[c] - dot);      /* softmax Jacobian */
      for (int i = 0; i < dh; ++i) {
        dQ[r0 + i] += scale * ds * K[(size_t)c * D + r0 + i];
        dK[(size_t)c * D + r0 + i] = scale * ds * Q[r0 + i];
      }
    }
  }
  /* K[c] = Wk z[c] + bk,  V[c] = Wv z[c] + bv */
  for (int c = 0; c < m; ++c) {
    double *dzc = dz + (size_t)c * D;
    for (int j = 0; j < D; ++j) dzc[j] = 0.0;
    affine_transposed_add(lv->Wk + wo, dK + (size_t)c * D, D, D, dzc);
    affine_transposed_add(lv->Wv + wo, dV + (size_t)c * D, D, D, dzc);
    outer_add(gr->dWk + wo, dK + (size_t)c * D, z + (size_t)c * D, D, D);
    outer_add(gr->dWv + wo, dV + (size_t)c * D, z + (size_t)c * D, D, D);
    for (int i = 0; i < D; ++i) {
      if (gr->dbk) gr->dbk[bo + i] += dK[(size_t)c * D + i];
      if (gr->dbv) gr->dbv[bo + i] += dV[(size_t)c * D + i];
    }
  }
  /* Q = Wq q + bq */
  if (gr->dbq) for (int i = 0; i < D; ++i) gr->dbq[bo + i] += dQ[i];
  outer_add(gr->dWq + wo, dQ, qv, D, D);
  affine_transposed_add(lv->Wq + wo, dQ, D, D, gr->dquery + bo);
  free(qv); free(Q); free(K); free(V); free(al); free(o); free(d_o); free(dQ); free(dK); free(dV); free(dal);
}

/* Reverse of one linear mixing layer (group k) at one patch: y[d] = sum_c w[c][d] z[c][d] + b[d]. */
static void linear_group_backward(int D, const oracle_level *lv, int k, int m, const double *z, const double *dy,
                                  double *dz, const oracle_level_grad *gr) {
  const int g = lv->group_size;
  for (int c = 0; c < m; ++c)
    for (int d = 0; d < D; ++d) {
      const size_t wi = ((size_t)k * g + c) * D + d;
      gr->dWv[wi] += dy[d] * z[(size_t)c * D + d];
      dz[(size_t)c * D + d] = (double)lv->Wv[wi] * dy[d];
    }
  if (gr->dbv) for (int d = 0; d < D; ++d) gr->dbv[(size_t)k * D + d] += dy[d];
}

/*
 * Gradients of L = sum over the S sampled patches of <dout[i], out[i]>.
 *   dout [S, D];  dx [S, C, p*p] (pixels of each sampled patch, row by row; NULL to skip);
 *   dWe [C, D, p*p];  dtok_bias [C, D] = dL/d be = dL/d ce (the two enter the token as a sum);
 *   grads[l]: arrays of level l, zero-filled by the caller and accumulated into; bias-gradient
 *   pointers may be NULL.  A patch listed twice counts twice.
 */
int oracle_backward(int B, int C, int H, int W, int p, int D, int heads, const float *x, const float *We,
                    const float *be, const float *ce, int n_levels, const oracle_level *levels, int S,
                    const int32_t *sample_b, const int32_t *sample_n, const double *dout, double *dx,
                    double *dWe, double *dtok_bias, const oracle_level_grad *grads) {
  if (p <= 0 || H % p || W % p || heads <= 0 || D % heads || n_levels < 1 || n_levels > 16) return -2;
  const int N = (H / p) * (W / p), pp = p * p, pw = W / p;
  int cin[17];
  cin[0] = C;
  for (int l = 0; l < n_levels; ++l) {
    if (levels[l].group_size < 1 || (levels[l].kind != 0 && levels[l].kind != 1)) return -2;
    cin[l + 1] = groups_of(cin[l], levels[l].group_size);
  }
  if (cin[n_levels] != 1 || levels[n_levels - 1].kind != 0) return -2;
  for (int i = 0; i < S; ++i)
    if (sample_b[i] < 0 || sample_b[i] >= B || sample_n[i] < 0 || sample_n[i] >= N) return -2;
  /* forward: inputs of every level for every sampled patch, zs[l] is [S, cin[l], D] */
  double *zs[17], *dzs[17];
  for (int l = 0; l <= n_levels; ++l) {
    zs[l] = (double *)malloc(sizeof(double) * (size_t)S * cin[l] * D);
    dzs[l] = (double *)malloc(sizeof(double) * (size_t)S * cin[l] * D);
  }
#pragma omp parallel for schedule(dynamic, 1)
  for (int i = 0; i < S; ++i) {
    tokens_of_patch(C, H, W, p, D, x + (size_t)sample_b[i] * C * H * W, We, be, ce, sample_n[i],
                    zs[0] + (size_t)i * C * D);
    for (int l = 0; l < n_levels; ++l)
      level_of_patch(cin[l], D, heads, &levels[l], zs[l] + (size_t)i * cin[l] * D,
                     zs[l + 1] + (size_t)i * cin[l + 1] * D, NULL, NULL);
  }
  memcpy(dzs[n_levels], dout, sizeof(double) * (size_t)S * D);
  /* levels in reverse; a group's weight gradients are touched by one thread only */
  for (int l = n_levels - 1; l >= 0; --l) {
    const oracle_level *lv = &levels[l];
    const int g = lv->group_size, G = cin[l + 1];
#pragma omp parallel for schedule(dynamic, 1)
    for (int k = 0; k < G; ++k) {
      const int c0 = k * g;
      const int m = (c0 + g < cin[l]) ? g : cin[l] - c0;
      for (int i = 0; i < S; ++i) {
        const double *z = zs[l] + ((size_t)i * cin[l] + c0) * D;
        const double *dy = dzs[l + 1] + ((size_t)i * G + k) * D;
        double *dz = dzs[l] + ((size_t)i * cin[l] + c0) * D;
        if (lv->kind == 1) linear_group_backward(D, lv, k, m, z, dy, dz, &grads[l]);
        else attention_group_backward(D, heads, lv, k, m, z, dy, dz, &grads[l]);
      }
    }
  }
  /* tokenizer: t[c] = We[c] u + be[c] + ce[c] */
#pragma omp parallel for schedule(dynamic, 1)
  for (int c = 0; c < C; ++c) {
    double *u = (double *)malloc(sizeof(double) * (size_t)pp);
    double *du = (double *)malloc(sizeof(double) * (size_t)pp);
    for (int i = 0; i < S; ++i) {
      const float *img = x + ((size_t)sample_b[i] * C + c) * H * W;
      const int pi = sample_n[i] / pw, pj = sample_n[i] % pw;
      for (int r = 0; r < p; ++r)
        for (int s = 0; s < p; ++s) u[r * p + s] = (double)img[(size_t)(pi * p + r) * W + (pj * p + s)];
      const double *dt = dzs[0] + ((size_t)i * C + c) * D;
      outer_add(dWe + (size_t)c * D * pp, dt, u, D, pp);
      for (int d = 0; d < D; ++d) dtok_bias[(size_t)c * D + d] += dt[d];
      if (dx) {
        for (int kk = 0; kk < pp; ++kk) du[kk] = 0.0;
        affine_transposed_add(We + (size_t)c * D * pp, dt, D, pp, du);
        memcpy(dx + ((size_t)i * C + c) * pp, du, sizeof(double) * (size_t)pp);
      }
    }
    free(u); free(du);
  }
  for (int l = 0; l <= n_levels; ++l) { free(zs[l]); free(dzs[l]); }
  return 0;
}
