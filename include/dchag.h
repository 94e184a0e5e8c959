/*
 * dchag.h -- C ABI of the MI355X (gfx950) D-CHAG library (forward and backward).
 *
 * D-CHAG = Distributed Cross-Channel Hierarchical Aggregation.  The library
 * computes the forward pass of per-channel patch tokenization followed by
 * hierarchical learned-query cross-channel cross-attention, on ONE GPU:
 *
 *   x[B,C,H,W] --tokenize--> t[B,C,N,D] --level 1--> [B,G1,N,D] --...--> out[B,N,D]
 *
 * with N = (H/p)*(W/p) patches per image, numbered row by row over the patch
 * grid; the pixels of a patch are flattened row by row.
 *
 * Conventions for every entry point
 *   - All tensor arguments are DEVICE pointers on the current HIP device, dense,
 *     row-major, last index fastest, 16-byte aligned.  Element type of every
 *     tensor is given by `dt` (DCHAG_F32: float, DCHAG_BF16: bfloat16);
 *     accumulation is always fp32.  The `dchag_level` structs themselves live
 *     in HOST memory and hold device pointers.
 *   - The caller owns every buffer (inputs, weights, outputs, workspace).  The
 *     library allocates no device memory and keeps no state between calls that
 *     changes a result.  Process-wide state, all of it listed here: the table of
 *     debugging switches read from the environment at load time (dchag_debug_reload),
 *     per-device caches of the compute-unit count and of the dynamic-LDS limits
 *     already raised (both mutex- or atomic-guarded), the stage-timing records of
 *     dchag_profile_begin/end, and the fixed scratch array of
 *     dchag_aggregate_level_static.  Calls on different host threads are safe as
 *     long as they do not share a workspace and no profile is being taken.
 *     Inputs and weights are only read; outputs are fully overwritten; the
 *     workspace contents are undefined afterwards.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls are asynchronous on that stream: no device synchronisation happens
 *     inside.  Calls that share a workspace must be ordered by the caller.
 *   - Return value: DCHAG_OK (0) or a negative dchag_status.  Arguments are
 *     validated on the host BEFORE anything is launched; on a validation error
 *     nothing has been launched and no output has been touched.
 */
#ifndef DCHAG_H_
#define DCHAG_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { DCHAG_F32 = 0, DCHAG_BF16 = 1 } dchag_dtype;

typedef enum {
  DCHAG_OK = 0,
  DCHAG_ERR_NULL = -1,      /* a required pointer is NULL                                   */
  DCHAG_ERR_SHAPE = -2,     /* sizes that do not fit together (see each call)               */
  DCHAG_ERR_DTYPE = -3,     /* unknown dtype                                                */
  DCHAG_ERR_WORKSPACE = -4, /* workspace NULL, misaligned or smaller than required          */
  DCHAG_ERR_LAUNCH = -5,    /* the HIP runtime refused a launch                             */
  DCHAG_ERR_ALIGN = -6      /* a tensor pointer is not 16-byte aligned                      */
} dchag_status;

typedef enum {
  DCHAG_LEVEL_ATTENTION = 0,        /* learned-query multi-head cross-attention (D-CHAG-C)        */
  DCHAG_LEVEL_LINEAR = 1            /* linear mixing along the channel axis (D-CHAG-L)            */
} dchag_level_kind;

/*
 * One aggregation level (paper Section 3.2: "multiple cross-attention layers",
 * each handling "up to" g channels; Section 3.3: partial-channel aggregation
 * modules followed by a final cross-attention layer).  A level with Cin inputs
 * per patch has G = ceil(Cin / group_size) groups; group k holds inputs
 * k*g .. min((k+1)*g, Cin)-1 and owns slice k of every array below.
 */
typedef struct {
  int32_t group_size;               /* nominal g >= 1; the last group may be shorter              */
  int32_t kind;                     /* dchag_level_kind                                           */
  const void *query;                /* [G, D]    learned query of each group                      */
  const void *Wq, *Wk, *Wv, *Wo;    /* [G, D, D] row-major (out, in): y = W x                     */
  const void *bq, *bk, *bv, *bo;    /* [G, D]    each may be NULL (= 0)                           */
} dchag_level;
/*
 * DCHAG_LEVEL_LINEAR (paper Section 3.2: intermediate cross-attention layers may be replaced by
 * lightweight linear layers; Section 3.3: the D-CHAG-L variant, whose final layer stays
 * cross-attention).  The paper does not define the layer; the reading built here mixes the members
 * of a group along the channel axis with one learned weight per member and feature:
 *
 *   tokens_out[b,k,n,d] = sum over members c of group k of  w[k][c - k*g][d] * z[b,c,n,d]  +  bias[k][d]
 *
 * For such a level `Wv` holds w as [G, g, D] and `bv` the bias [G, D] (or NULL); every other
 * pointer of the struct is ignored and may be NULL.  The last level of dchag_forward must be
 * DCHAG_LEVEL_ATTENTION.
 */

/*
 * Per-channel patch tokenization (paper Section 2.1: every 2-D patch of every
 * channel is tokenized independently by a convolution with kernel = stride =
 * patch size; each channel is assigned an ID embedding):
 *
 *   tokens[b,c,n,:] = We[c] . vec(patch n of x[b,c]) + be[c] + ce[c]
 *
 *   x      [B,C,H,W]   in     We  [C,D,p*p]  in  (the conv weight [D,1,p,p] of channel c)
 *   be     [C,D] or NULL      ce  [C,D] or NULL  (channel-ID embedding, added)
 *   tokens [B,C,N,D]   out
 * Errors: NULL x/We/tokens; B,C,D,p < 1; H % p or W % p != 0; D % 8 != 0.
 */
int dchag_tokenize(dchag_dtype dt, int B, int C, int H, int W, int p, int D,
                   const void *x, const void *We, const void *be, const void *ce,
                   void *tokens, void *stream);

/*
 * One level of cross-channel aggregation (paper Section 2.1: a cross-attention
 * layer reduces the channels to one representation; Section 3.2: one such layer
 * per group of at most g channels).  For every batch item b, patch n and
 * group k, with S_k the members of the group, Q = Wq[k] query[k] + bq[k],
 * d_h = D / heads and per head a (rows a*d_h .. (a+1)*d_h-1):
 *
 *   s[c]   = < Q_a , (Wk[k] z[b,c,n] + bk[k])_a > / sqrt(d_h)      c in S_k
 *   alpha  = softmax over c in S_k of s
 *   o_a    = sum over c in S_k of alpha[c] (Wv[k] z[b,c,n] + bv[k])_a
 *   tokens_out[b,k,n,:] = Wo[k] concat_a(o_a) + bo[k]
 *
 *   tokens_in  [B,Cin,N,D] in      tokens_out [B,G,N,D] out
 *   workspace: at least dchag_workspace_bytes(..., which = 0) bytes, 256-byte aligned.
 * A DCHAG_LEVEL_LINEAR level computes the weighted sum given with dchag_level instead; it uses no
 * workspace (NULL is accepted) and `heads` only has to pass the shape check (1 will do).
 * Errors: NULL tokens/lvl/required weight; Cin,N,D,heads < 1; D % heads != 0;
 * D % 8 != 0; group_size < 1; unknown kind; workspace too small.
 */
int dchag_aggregate_level(dchag_dtype dt, int B, int Cin, int N, int D, int heads,
                          const dchag_level *lvl, const void *tokens_in, void *tokens_out,
                          void *workspace, size_t workspace_bytes, void *stream);

/*
 * dchag_aggregate_level for callers that cannot allocate device memory (code under HIP graph capture, serving loops,
 * harnesses that forbid hipMalloc): same arguments without the workspace, same result bit for bit.  The workspace is
 * a fixed array of DCHAG_STATIC_SCRATCH_BYTES bytes inside the library's code object (every GPU the library runs on
 * holds its own copy until the process ends); the call allocates nothing and frees nothing.  Its address is looked up
 * on the first call on a device, so make that first call outside any stream capture.
 *   - A level that needs more than DCHAG_STATIC_SCRATCH_BYTES (dchag_workspace_bytes(..., which = 0)) is rejected
 *     with DCHAG_ERR_WORKSPACE before anything is launched.
 *   - Every call on one GPU uses the same array: calls that overlap on one GPU (two streams, two threads) race and
 *     must be ordered by the caller.  Nothing in the array has to start at zero; the kernels write all they read.
 * Errors otherwise as dchag_aggregate_level.
 */
#define DCHAG_STATIC_SCRATCH_BYTES (32u << 20)
int dchag_aggregate_level_static(dchag_dtype dt, int B, int Cin, int N, int D, int heads,
                                 const dchag_level *lvl, const void *tokens_in, void *tokens_out,
                                 void *stream);

/*
 * The whole path (paper Section 3.3, run on one GPU: tokenize every channel,
 * aggregate groups level by level, finish with one cross-attention layer over
 * what is left):  out[b,n,:] = level_L( ... level_1( tokenize(x) ) ... ).
 * levels[l] takes the G_{l-1} outputs of the level before it as its inputs
 * (C for the first); the last level must have exactly one group.
 *
 *   out [B,N,D]; workspace: at least dchag_workspace_bytes(..., which = 1) bytes.
 * Errors: as the two calls above; n_levels < 1; last level leaves more than one group or is not
 * DCHAG_LEVEL_ATTENTION.
 */
int dchag_forward(dchag_dtype dt, int B, int C, int H, int W, int p, int D, int heads,
                  const void *x, const void *We, const void *be, const void *ce,
                  int n_levels, const dchag_level *levels, void *out,
                  void *workspace, size_t workspace_bytes, void *stream);

/*
 * dchag_forward with the positional embedding added in the epilogue of the last output projection
 * (paper Section 2.1: the aggregated token of every patch receives positional and metadata tokens before it
 * enters the ViT; the learned positional embedding is one vector per patch, shared by the batch):
 *
 *   out[b,n,:] = dchag_forward(...)[b,n,:] + pos[n,:]          pos [N,D] in, required
 *
 * The sum is taken in fp32 before the one rounding of the output; no extra pass over `out` is made.
 * Everything else as dchag_forward (same workspace, which = 1).
 */
int dchag_forward_pos(dchag_dtype dt, int B, int C, int H, int W, int p, int D, int heads,
                      const void *x, const void *We, const void *be, const void *ce,
                      int n_levels, const dchag_level *levels, const void *pos, void *out,
                      void *workspace, size_t workspace_bytes, void *stream);

/*
 * The whole path with the value projection moved behind the softmax-weighted sum (an inference
 * variant; same arguments, same result up to rounding as dchag_forward).  The weights of a softmax
 * sum to one, so for every head a
 *
 *   o_a = sum_c alpha[c,a] (Wv z[c] + bv)_a = Wv_a ( sum_c alpha[c,a] z[c] ) + bv_a :
 *
 * the group's tokens are averaged per head first (u_a, one D-vector per head) and Wv is applied once
 * per (group, patch, head) instead of once per member -- g*D*D multiply-adds per group and patch
 * become D*D + g*heads*D.  The paper states the layer as plain cross-attention (Section 2.1); this
 * is the same function evaluated in another order, kept as a call of its own so that the as-defined
 * path stays measurable.
 * At the first level the tokens are themselves linear in the pixels (Section 2.1: z[c] = We[c] u[c] + be[c] +
 * ce[c] for the patch u[c]), so there the projection moves one step further, into the tokenizer:
 *
 *   o_a = sum_c alpha[c,a] ( (Wv We[c]) u[c] + Wv (be[c] + ce[c]) )_a + bv_a .
 *
 * For bf16 inputs with 4 x 4 or 8 x 8 patches, D a multiple of 256 and heads of 32, 64, 128, ... columns (32 times a
 * power of two; and the shapes whose scores come from the pixels: a multiple of 4 heads, at most 32) the call forms the weight-only
 * products Wv We[c], Wv be, Wv ce first and then goes from pixels and softmax weights to o in one kernel; the
 * per-channel tokens and the per-head averages u_a of that level never exist.  Other shapes, fp32 and the upper
 * levels take the u_a route.  workspace: dchag_workspace_bytes(..., which = 2).
 */
int dchag_forward_folded(dchag_dtype dt, int B, int C, int H, int W, int p, int D, int heads,
                         const void *x, const void *We, const void *be, const void *ce,
                         int n_levels, const dchag_level *levels, void *out,
                         void *workspace, size_t workspace_bytes, void *stream);

/*
 * dchag_forward_folded for callers whose weights stay fixed between calls (inference).  Everything in that call
 * that depends on the weights alone is formed once by dchag_fold_value into a caller-owned device buffer `folded`:
 * the first level's folded tokenizer weights and token bias (paper Section 2.1's tokenizer and first cross-attention
 * layer composed, see above),
 *
 *   Wf[c] = Wv[k(c)] We[c]   [C, D, p*p]      and      Wv[k(c)] (be[c] + ce[c])   [C, D],
 *
 * and, for every attention level, the projected query Q = Wq q + bq, the query folded into the key weights, and (first
 * level) their composition with the tokenizer weights that scores the pixels directly.  dchag_forward_prefolded is
 * dchag_forward_folded without that work (same arguments otherwise, same result bit for bit; workspace which = 2).
 *   dchag_value_fold_bytes: size of `folded` for a shape, 0 if dchag_forward_folded does not take that shape's first
 *     level from the pixels (then there is nothing to prepare: use dchag_forward_folded).  levels: host array as in
 *     dchag_forward (only kinds and group sizes are read).
 *   dchag_fold_value: We, be, ce as in dchag_tokenize (be, ce may be NULL), levels as in dchag_forward; folded
 *     256-byte aligned, folded_bytes at least dchag_value_fold_bytes(...).  Asynchronous on `stream`.
 *   The caller redoes dchag_fold_value whenever a weight changes; the library cannot check that.
 * Errors: as dchag_forward; DCHAG_ERR_SHAPE for a shape with dchag_value_fold_bytes(...) == 0; DCHAG_ERR_WORKSPACE for
 * a NULL, misaligned or short `folded`.
 */
size_t dchag_value_fold_bytes(dchag_dtype dt, int C, int p, int D, int heads,
                              int n_levels, const dchag_level *levels);
int dchag_fold_value(dchag_dtype dt, int C, int p, int D, int heads,
                     const void *We, const void *be, const void *ce,
                     int n_levels, const dchag_level *levels,
                     void *folded, size_t folded_bytes, void *stream);
int dchag_forward_prefolded(dchag_dtype dt, int B, int C, int H, int W, int p, int D, int heads,
                            const void *x, const void *We, const void *be, const void *ce,
                            int n_levels, const dchag_level *levels, const void *folded, void *out,
                            void *workspace, size_t workspace_bytes, void *stream);

/*
 * Gradients of one level, shaped like the weights of dchag_level (host struct, device pointers).
 * Any pointer may be NULL: that gradient is not written.  A DCHAG_LEVEL_LINEAR level uses dWv
 * ([G, g, D]) and dbv only.
 */
typedef struct {
  void *dquery;                     /* [G, D]                                                     */
  void *dWq, *dWk, *dWv, *dWo;      /* [G, D, D]                                                  */
  void *dbq, *dbk, *dbv, *dbo;      /* [G, D]                                                     */
} dchag_level_grads;

/*
 * Backward pass of dchag_forward (the paper's module is trained through; Section 3.3 notes that the
 * backward of the partial aggregation needs no communication, it is the plain reverse of the forward).
 * Given dout = dL/d(out) for a scalar loss L, writes dL/d(every weight) and, if asked, dL/dx:
 *
 *   dout      [B,N,D]    in
 *   dx        [B,C,H,W]  out, or NULL
 *   dWe       [C,D,p*p]  out, or NULL
 *   dtok_bias [C,D]      out, or NULL: dL/d(be) = dL/d(ce) (the two enter a token as a sum)
 *   grads     n_levels entries (host), grads[l] for levels[l]
 *
 * Every gradient tensor has element type `dt` and is overwritten (not accumulated into); sums over
 * patches and members are fp32 in a fixed order (results are reproducible run to run).  The key bias
 * shifts all scores of a softmax equally, so dbk is written as zeros.  Nothing is kept from a forward
 * call: the activations the reverse sweep needs (tokens, softmax weights, per-head token averages,
 * pre-projection outputs) are recomputed into the workspace first, with the value projection applied
 * after the weighted sum (see dchag_forward_folded), so a training step is dchag_forward (or nothing,
 * if `out` is not needed) followed by this call.
 * workspace: dchag_workspace_bytes(..., which = 3).
 * Errors: as dchag_forward; NULL dout or grads.
 */
int dchag_backward(dchag_dtype dt, int B, int C, int H, int W, int p, int D, int heads,
                   const void *x, const void *We, const void *be, const void *ce,
                   int n_levels, const dchag_level *levels, const void *dout,
                   void *dx, void *dWe, void *dtok_bias, const dchag_level_grads *grads,
                   void *workspace, size_t workspace_bytes, void *stream);

/*
 * A training step without the recomputation: dchag_forward_keep is dchag_forward_folded that leaves, in a
 * workspace of dchag_backward's size and layout (which = 3), everything the reverse sweep reads (tokens; per
 * level its inputs, folded keys, softmax weights, per-head token averages, pre-projection outputs), and
 * dchag_backward_kept is the reverse sweep alone.  dchag_backward_kept must be given the same arguments and the
 * workspace of the dchag_forward_keep call, untouched in between (the library cannot check that); any number of
 * dchag_backward_kept calls (different dout) may follow one dchag_forward_keep.  The gradients equal those of
 * dchag_backward bit for bit; the output equals dchag_forward_folded's bit for bit wherever that call takes the
 * u_a route at the first level, and up to rounding where it folds the projection into the tokenizer (the kept
 * forward always forms tokens and u_a: the reverse sweep reads them).  For callers that keep activations between the two passes,
 * as training loops do; the paper describes the two passes of its module (Section 3.3), not how they share state.
 */
int dchag_forward_keep(dchag_dtype dt, int B, int C, int H, int W, int p, int D, int heads,
                       const void *x, const void *We, const void *be, const void *ce,
                       int n_levels, const dchag_level *levels, void *out,
                       void *workspace, size_t workspace_bytes, void *stream);
int dchag_backward_kept(dchag_dtype dt, int B, int C, int H, int W, int p, int D, int heads,
                        const void *x, const void *We, const void *be, const void *ce,
                        int n_levels, const dchag_level *levels, const void *dout,
                        void *dx, void *dWe, void *dtok_bias, const dchag_level_grads *grads,
                        void *workspace, size_t workspace_bytes, void *stream);

/*
 * Workspace size in bytes (0 on invalid arguments).
 *   which = 0: one dchag_aggregate_level call with Cin = C inputs, N = (H/p)*(W/p)
 *              (pass H = N, W = 1, p = 1 when only N is known), group size group_sizes[0];
 *   which = 1: one dchag_forward call with the n_levels nominal group sizes;
 *   which = 2: one dchag_forward_folded call;   which = 3: one dchag_backward call, or a
 *              dchag_forward_keep / dchag_backward_kept pair.
 * The size also depends on the current device (how a level's work is split follows its number of compute units;
 * without a device 256 are assumed): ask on the device and in the process that makes the call.
 */
size_t dchag_workspace_bytes(dchag_dtype dt, int B, int C, int H, int W, int p, int D, int heads,
                             int n_levels, const int32_t *group_sizes, int which);

/*
 * Stage timing, a diagnostic for benchmarks (not part of the paper's method).  Between
 * dchag_profile_begin and dchag_profile_end every kernel the library launches is bracketed
 * by a pair of HIP events recorded on the call's own stream; dchag_profile_end waits for the
 * recorded events, writes up to `cap` records in launch order and returns how many there
 * were in total (or a negative status).  It is not thread-safe and it creates HIP events,
 * so it must not be used under stream capture.  `records` is HOST memory.
 */
typedef enum {
  DCHAG_STAGE_TOKENIZE = 0,        /* per-channel patch embedding                              */
  DCHAG_STAGE_QUERY = 1,           /* Q = Wq q + bq (weight-only)                              */
  DCHAG_STAGE_FOLD = 2,            /* query folded into the key weights (weight-only)          */
  DCHAG_STAGE_SCORES = 3,          /* scores of every token against the folded keys            */
  DCHAG_STAGE_VPROJ = 4,           /* value projection                                         */
  DCHAG_STAGE_SOFTMAX_AGG = 5,     /* softmax over the group and weighted sum of the values    */
  DCHAG_STAGE_OPROJ = 6,           /* output projection                                        */
  DCHAG_STAGE_FUSED_VAGG = 7,      /* value projection with the softmax-weighted sum over the
                                      group in its epilogue (weights computed beforehand)      */
  DCHAG_STAGE_CHANNEL_MIX = 8,     /* linear (D-CHAG-L) level: weighted sum over the group      */
  DCHAG_STAGE_TOKENIZE_MIX = 9,    /* tokenizer fused with a linear first level                 */
  DCHAG_STAGE_HEAD_SUMS = 10,      /* per-head softmax-weighted token averages u_a              */
  DCHAG_STAGE_HEAD_VPROJ = 11,     /* value projection applied to u_a, one head at a time       */
  DCHAG_STAGE_BWD_OPROJ = 12,      /* backward of the output projection (dWo, dbo, d o)         */
  DCHAG_STAGE_BWD_VALUE = 13,      /* backward of the value path (dWv, dbv, w = Wv_a^T d o_a)   */
  DCHAG_STAGE_BWD_SOFTMAX = 14,    /* d alpha, softmax Jacobian                                 */
  DCHAG_STAGE_BWD_TOKENS = 15,     /* gradient at the level's input tokens                      */
  DCHAG_STAGE_BWD_KEY_QUERY = 16,  /* key / query weight gradients (rank-one per head)          */
  DCHAG_STAGE_BWD_TOKENIZE = 17,   /* tokenizer backward (dWe, token bias, dx)                  */
  DCHAG_STAGE_BWD_CHANNEL_MIX = 18,/* backward of a linear level                                */
  DCHAG_STAGE_FOLD_VALUE = 19,     /* value projection folded into the tokenizer (weight-only)  */
  DCHAG_STAGE_TOKENIZE_ATTEND = 20,/* tokenizer fused with an attention first level             */
  DCHAG_STAGE_KEY_PREP = 21        /* projected queries and query-folded keys of one level (level
                                      >= 1) or of all levels of the call at once (level 0); the
                                      bf16 path's form of stages 1 and 2 (weight-only)            */
} dchag_stage;

typedef struct {
  int32_t stage;                   /* dchag_stage                                              */
  int32_t level;                   /* 0 for the tokenizer, 1.. for the aggregation levels      */
  float ms;                        /* elapsed time between the two events                      */
} dchag_stage_time;

int dchag_profile_begin(void);
int dchag_profile_end(dchag_stage_time *records, int cap);

/*
 * Yardsticks for benchmarks (not part of the paper's method): what this GPU reaches on a loop of nothing but bf16
 * MFMAs and on a plain stream copy, so that a kernel's rate can be quoted against the achievable rate as well as
 * against the nominal peak.  Both are asynchronous on `stream`; the caller times them (HIP events).
 *   dchag_yardstick_mfma: every wavefront of 4 x (compute units) workgroups of 256 threads runs `iters` rounds of
 *     eight independent 32x32x16 bf16 MFMAs on registers; *flops (HOST) receives the number of flops launched.
 *     sink: device scratch of sink_floats >= 1024 x (compute units) floats (one value per thread is written).
 *   dchag_yardstick_copy: dst[0 .. bytes) = src[0 .. bytes) in 16-byte pieces (bytes % 16 == 0): reads `bytes`,
 *     writes `bytes`.
 *   dchag_yardstick_read: reads src[0 .. bytes) in 16-byte pieces and stores nothing (sink: device scratch of at
 *     least 256 floats, never written in practice): the streaming-read rate.
 */
int dchag_yardstick_mfma(int iters, float *sink, size_t sink_floats, double *flops, void *stream);
int dchag_yardstick_copy(void *dst, const void *src, size_t bytes, void *stream);
int dchag_yardstick_read(const void *src, size_t bytes, float *sink, void *stream);

/*
 * Debugging switches.  The library reads a set of DCHAG_* environment variables (kernel-route overrides used by its
 * tests) ONCE, when it is loaded; calls never read the environment.  dchag_debug_reload reads them again.  It is a
 * test aid, not thread-safe, and must not run while another thread is inside a call; change a switch that alters how
 * work is split (and with it workspace sizes) only between a dchag_workspace_bytes / call pair, never inside one.
 */
void dchag_debug_reload(void);

/* Static, never-NULL description of a status code. */
const char *dchag_strerror(int status);

/* Library version, "major.minor". */
const char *dchag_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DCHAG_H_ */
