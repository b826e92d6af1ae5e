/*
 * ficoco.h -- C ABI of the MI355X (gfx950) FiCoCo token-reduction library.
 *
 * One call of a *_step function runs one per-layer "filter, correlate, compress" step of
 * the paper "Filter, Correlate, Compress" (arxiv 2411.17686): Algorithm 1 (FiCoCo-V, vision
 * encoder) or Algorithm 2 (FiCoCo-L, LLM decoder, text guided).  The stage functions expose
 * the same path in four pieces: score -> filter -> correlate -> compress.
 *
 * Conventions that hold for every entry point
 *   - Plain C: no C++ types, no exceptions cross this boundary.
 *   - Every data pointer is a DEVICE pointer owned by the caller (tokens, maps, outputs and
 *     the workspace), on the device the ctx was created for, which must be the calling
 *     thread's current device (checked: FICOCO_EINVAL otherwise).  The library allocates no
 *     device memory and frees nothing of the caller's.  Outputs must not alias inputs
 *     (X_out overlapping X or the workspace is rejected with FICOCO_EINVAL; the small index
 *     and edge outputs are not checked).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All work is
 *     enqueued on it asynchronously; no call synchronises the device or copies to the host.
 *   - Return value: a ficoco_status.  Argument errors are found on the host before anything
 *     is launched (FICOCO_EINVAL), a workspace that is too small gives FICOCO_ENOMEM, a
 *     failed launch FICOCO_EHIP, a legal but unimplemented combination
 *     FICOCO_EUNSUPPORTED.  ficoco_last_error(ctx) describes the last failure on that ctx.
 *   - Inputs are assumed finite (no NaN / Inf); behaviour is undefined otherwise.
 *   - Attention maps P[b][h][q][k] are row-stochastic over k (query q attends key k), the
 *     key axis contiguous.  The paper describes its first score term as the attention a
 *     token receives, so the paper's A_{i,j} for a visual token i is P[j][i].
 *   - Scores, thresholds and merge weights are computed and compared in double precision;
 *     tokens are read and written in `dtype`.  Ties in the top-K filter go to the lower
 *     token index.
 */
#ifndef FICOCO_H
#define FICOCO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ficoco_ctx ficoco_ctx; /* opaque: device id + last error text */

typedef enum {
  FICOCO_OK = 0,
  FICOCO_EINVAL = 1,
  FICOCO_ENOMEM = 2,
  FICOCO_EHIP = 3,
  FICOCO_EUNSUPPORTED = 4
} ficoco_status;
/* There is no status for "a discarded token had more than k_max targets": whether that
 * happened is known only once the kernels have run, and no call waits for them.  It is
 * reported per image through the `overflow` array on the device instead, which the caller
 * reads whenever it next synchronises. */

typedef enum { FICOCO_F32 = 0, FICOCO_BF16 = 1 } ficoco_dtype;

/* Which algorithm of the paper the problem describes. */
typedef enum { FICOCO_VARIANT_V = 0, FICOCO_VARIANT_L = 1 } ficoco_variant;

/* First score term R_i of Eq. 1 / Eq. 3 (the token's received attention). */
typedef enum {
  FICOCO_R_ATTN_RECV = 0, /* (1/N) sum over visual queries q of headmean P[q][i]              */
  FICOCO_R_VECTOR = 1,    /* headmean of the caller's pre-reduced recv_vec[b][h][i]          */
  FICOCO_R_SIM_MEAN = 2   /* extension: (1/N) sum_j cos(F_i, F_j), when no map is available  */
} ficoco_red_src;

/* Second score term G_i (entered with a minus sign). */
typedef enum {
  FICOCO_G_CLS_ATTN = 0,  /* Eq. 1: headmean P[CLS][i]                                        */
  FICOCO_G_TEXT_ATTN = 1, /* Eq. 3: (1/M) sum over text queries k of headmean P[k][i]         */
  FICOCO_G_VECTOR = 2,    /* headmean of sem_vec[b][h][i]                                     */
  FICOCO_G_EQ_TOKEN = 3   /* appendix "Implementation of the Equivalent Token": -cos(mu,F_i) */
} ficoco_sem_src;

/* Direct correlation C_ij between discarded i and preserved j. */
typedef enum {
  FICOCO_C_ATTN = 0,  /* Algorithm 1 stage 2: headmean P[j][i], held in single precision      */
  FICOCO_C_COSINE = 1 /* extension: max(0, xh_i . xh_j), xh = bfloat16(F / |F|)                */
} ficoco_corr_src;

/* How the targets of a discarded token are chosen (Sec. "Correlation-based Information
 * Recycling" and the "Correlate" rows of the two ablation tables). */
typedef enum {
  FICOCO_K_ADAPTIVE = 0,  /* the method: token-wise eps-quantile threshold                       */
  FICOCO_K_FIXED = 1,     /* ablation "fixed K": the fixed_k largest C_ij of the row, ties to the
                             lower position; fixed_k = 0 is pruning                              */
  FICOCO_K_CONVERGENT = 2 /* ablation "convergent correlation": the preserved tokens stay as they
                             are; ONE extra token, the plain mean of the discarded tokens, is
                             written directly behind the last preserved visual token           */
} ficoco_k_mode;

/* How a preserved token takes up its sources (Sec. "Compress", Eq. 2, and the "Compress" row
 * of the ablation tables). */
typedef enum {
  FICOCO_COMPRESS_SELF = 0,   /* Eq. 2, self-preserving compression                            */
  FICOCO_COMPRESS_AVERAGE = 1 /* ablation "average compression": every weight is one           */
} ficoco_compress_mode;

/*
 * Problem description (host struct, passed by pointer, read during the call only).
 * Token indices are positions in the sequence of n_tot tokens; the reducible visual tokens
 * are the span [vis_begin, vis_begin + N).  "Visual token i" below means sequence position
 * vis_begin + i.  Strides are in ELEMENTS of `dtype`.
 */
typedef struct {
  int32_t variant; /* ficoco_variant */
  int32_t dtype;   /* ficoco_dtype of X, A, A_text, recv_vec, sem_vec, F and X_out */
  int32_t B, H, D;
  int32_t n_tot;     /* tokens per sequence in X (V: [CLS]+N or N;  L: system+N+text)  */
  int32_t vis_begin; /* first reducible visual token                                     */
  int32_t N;         /* number of reducible visual tokens                                */
  int32_t n_keep;    /* N^T = tokens preserved;  N^S = N - n_keep are discarded          */
  int32_t cls_index; /* sequence position of [CLS] (FICOCO_G_CLS_ATTN), else -1         */

  const void *X; /* [B][n_tot][D], D contiguous */
  int64_t x_stride_b, x_stride_n;

  /* Attention block that holds the visual queries x visual keys (and the [CLS] query row
   * when used): row r is the query at sequence position a_q_begin + r, column c the key at
   * a_k_begin + c.  NULL when neither FICOCO_R_ATTN_RECV, FICOCO_G_CLS_ATTN nor
   * FICOCO_C_ATTN is selected. */
  const void *A; /* [B][H][a_nq][a_nk], a_nk contiguous */
  int64_t a_stride_b, a_stride_h, a_stride_q;
  int32_t a_q_begin, a_nq, a_k_begin, a_nk;

  /* FiCoCo-L: attention of the M text queries, columns covering the visual keys: column c
   * is the key at sequence position at_k_begin + c.  May point into the same map as A. */
  const void *A_text; /* [B][H][M][at_nk] */
  int64_t at_stride_b, at_stride_h, at_stride_q;
  int32_t M, at_k_begin, at_nk;

  const void *recv_vec; /* [B][H][N] contiguous, FICOCO_R_VECTOR */
  const void *sem_vec;  /* [B][H][N] contiguous, FICOCO_G_VECTOR */

  /* Features of the visual tokens for the cosine-based terms (EQ_TOKEN: head-mean keys).
   * NULL = use the visual rows of X (then Df is ignored and D is used). */
  const void *F; /* [B][N][Df] */
  int64_t f_stride_b, f_stride_n;
  int32_t Df;

  /* Local penalty (FiCoCo-V): pos[b][i] = grid cell of visual token i in grid_g stacked
   * grid_h x grid_w grids, row-major; NULL = cell i.  window = 0 switches it off. */
  const int32_t *pos;
  int32_t grid_g, grid_h, grid_w, window;
  float penalty_coef;

  float w_score; /* lambda (Eq. 1) or beta (Eq. 3) */
  float gamma;   /* Eq. 4; ignored by FiCoCo-V      */
  float eps;     /* quantile of the token-wise threshold, in [0, 1] */

  int32_t red_src, sem_src, corr_src;
  int32_t k_max; /* capacity of targets per discarded token in the edge lists (>= 1) */

  /* Ablation variants; all zero = the method as published.  With FICOCO_K_CONVERGENT and at
   * least one discarded token X_out has one row more: n_tot - N^S + 1 (see ficoco_out_rows). */
  int32_t k_mode;        /* ficoco_k_mode                                                  */
  int32_t fixed_k;       /* FICOCO_K_FIXED: targets per discarded token, 0 <= fixed_k <= k_max */
  int32_t compress_mode; /* ficoco_compress_mode                                           */

  /* Queries and keys instead of the map (Sec. "Self-Attention": A = Softmax(Q K^T / sqrt(D))).
   * FiCoCo-V: used when A is NULL and an attention-derived term is selected: the step then
   * forms softmax(qk_scale * Q_h K_h^T) of every head itself, row by row over all qk_n keys,
   * unmasked, and reduces it on the fly -- the [B][H][n][n] maps are never stored.  Row r of Q
   * and of K is the token at sequence position qk_begin + r; the block must cover the visual
   * span and, for FICOCO_G_CLS_ATTN, cls_index.
   * FiCoCo-L: used when both A and A_text are NULL (M must be set): the maps are the decoder's,
   * causal (row r attends rows 0 .. r of the block); the M text tokens are the positions
   * vis_begin + N .. vis_begin + N + M - 1 and must lie inside the block; their rows give the
   * text profiles of Eq. 3 / Eq. 4, the visual rows the visual-to-visual terms where selected.  bfloat16 only (qk_dtype = FICOCO_BF16, whatever
   * `dtype` the tokens have), d_head in {32, 64, 128}; with qk_n > 640 (the keys are then taken in blocks of 640, in two
   * sweeps) and for FiCoCo-L at most 64 heads: FICOCO_EUNSUPPORTED otherwise.  Logits, exponentials and row sums are single precision (bf16 products are exact
   * in it), so scores and map entries agree with a double-precision evaluation to about 1e-6
   * relative, not to the last bit: a top-K or threshold decision whose margin is below that may
   * differ from one taken on double-precision values. */
  const void *Q; /* [B][H][qk_n][d_head], d_head contiguous */
  const void *K; /* same shape and strides */
  int64_t qk_stride_b, qk_stride_h, qk_stride_n;
  int32_t qk_begin, qk_n, d_head, qk_dtype;
  float qk_scale; /* the 1/sqrt(D) of the equation */
} ficoco_problem;

/* ctx: create once per device (and calling thread); not thread safe.  ficoco_create also
 * looks up, for that device, the address of the static scratch of ficoco_v_step_static. */
int ficoco_create(ficoco_ctx **out, int device);
int ficoco_destroy(ficoco_ctx *ctx);
const char *ficoco_last_error(const ficoco_ctx *ctx);
const char *ficoco_version(void);

/*
 * Measurement hook (not part of the paper's method).  With two non-NULL hipEvent_t handles
 * (created by the caller with timing enabled, passed as void*), every following call on this
 * ctx that launches the chosen kernel records `start` immediately before and `stop`
 * immediately after that launch, on the call's stream, so the dominant kernel can be timed
 * inside a running pipeline.  NULL, NULL switches it off.
 *   kernel = FICOCO_PROBE_REDUCE : the attention-reduction kernel (bandwidth bound)
 *   kernel = FICOCO_PROBE_GRAM   : the bf16 matrix-core tile kernel of the cosine correlation
 *   kernel = FICOCO_PROBE_GRAM_X16 : the same kernel launched FICOCO_PROBE_REPEAT times in a row
 *            between the two events (every launch writes the same block, so results do not
 *            change): elapsed / FICOCO_PROBE_REPEAT is the launch duration without the cost of
 *            recording an event around a single short launch.  For ficoco_correlate loops only.
 */
typedef enum { FICOCO_PROBE_REDUCE = 0, FICOCO_PROBE_GRAM = 1, FICOCO_PROBE_GRAM_X16 = 2 } ficoco_probe_kernel;
#define FICOCO_PROBE_REPEAT 16
int ficoco_set_probe(ficoco_ctx *ctx, int kernel, void *start_event, void *stop_event);

/* Bytes of device workspace the calls below need for this problem (256-byte aligned
 * pointer expected).  The workspace carries state from one stage to the next: the stage
 * functions must be called in order, on one stream, with the same problem and workspace. */
int ficoco_workspace_bytes(const ficoco_problem *p, size_t *out_bytes);

/*
 * Reduction schedule from the appendix "Theoretical FLOPs Calculation" (host arithmetic only,
 * no GPU): how many visual tokens to discard in every layer so that the model's transformer
 * layers stay within a FLOPs budget.
 *
 * Cost model of one layer over n visual tokens (hidden size D, feed-forward size F):
 *   FiCoCo-V: 4 n D^2 + 2 n^2 D + 2 n D F              (the vision encoder sees the visual tokens)
 *   FiCoCo-L: the same with p = n + M in place of n     (the decoder also sees M text tokens)
 * plus, in a layer that reduces from n to n' = n - s tokens, the method's own work
 *   V:  n^2 + 2n + s (n' + 2D + 1) + D        L:  2 (n^2 + 2n) + s (n' + 2D + 1) + D.
 * A reducing layer is charged with n' tokens (the appendix's "after" expression).  Layers
 * before start_layer keep all N tokens; from start_layer on every layer discards the same
 * count s (Sec. "Implementation Details": reduction starts at the 12th encoder / 4th decoder
 * layer, a fixed number of tokens per layer) but never goes below min_keep tokens.  The result
 * is the smallest s whose total cost is within the budget.
 *   n_discard [layers] int32, out: tokens discarded in each layer (host memory).
 *   total_flops          out: cost of the returned schedule (may be NULL).
 * Returns FICOCO_OK, FICOCO_EINVAL for bad arguments, FICOCO_EUNSUPPORTED when even the
 * strongest schedule (every layer from start_layer on drops to min_keep) exceeds the budget;
 * that schedule is then the one returned.
 */
typedef struct {
  int32_t variant;     /* ficoco_variant                                            */
  int32_t layers;      /* transformer layers of the model part that is scheduled    */
  int32_t start_layer; /* first layer that reduces, 0-based (the paper: 11 for V, 3 for L) */
  int32_t N;           /* visual tokens entering the first layer                     */
  int32_t M;           /* text tokens (FiCoCo-L), else 0                            */
  int32_t D;           /* hidden size                                               */
  int32_t F;           /* feed-forward size (the appendix calls it H)               */
  int32_t min_keep;    /* lower bound of visual tokens after any layer (>= 1)        */
  double budget_flops; /* budget for the sum over the layers                         */
} ficoco_schedule_problem;
int ficoco_schedule(const ficoco_schedule_problem *p, int32_t *n_discard, double *total_flops);

/* Rows per sequence of X_out for this problem: n_tot - N^S, plus one for the additional
 * token of FICOCO_K_CONVERGENT when N^S > 0.  Host arithmetic only. */
int ficoco_out_rows(const ficoco_problem *p, int32_t *out_rows);

/*
 * Attention reduction alone (the first term of Eq. 1 / Eq. 3, the [CLS] / text terms and
 * the head-mean maps of Algorithm 1/2 stage 2): the one pass over the [B][H][q][k] maps,
 * leaving per-column partial sums and the head-mean maps in the workspace.  ficoco_score
 * runs this itself; the separate entry point exists so the dominant, bandwidth-bound pass
 * can be timed and profiled on its own.
 */
int ficoco_reduce(ficoco_ctx *ctx, const ficoco_problem *p, void *ws, size_t ws_bytes, void *stream);

/*
 * Filter, part 1 (Eq. 1 / Eq. 3 and the local penalty, Sec. "Redundancy-based Token
 * Discard"; Sec. "Task-Aware Improvements for FiCoCo-L"): reduces the attention maps /
 * features once and writes the redundancy score of every visual token.  Also leaves the
 * head-mean maps needed by ficoco_correlate in the workspace.
 *   scores  [B][N] double, out: penalised scores (what the filter ranks).
 */
int ficoco_score(ficoco_ctx *ctx, const ficoco_problem *p, void *ws, size_t ws_bytes,
                 double *scores, void *stream);

/*
 * Filter, part 2 (Algorithm 1/2, stage 1): the N^S visual tokens with the highest score
 * (ties: lower index first) are discarded.
 *   scores       [B][N] double, in.
 *   discard_idx  [B][N^S] int32, out: visual token indices of the source set, ascending.
 *   keep_idx     [B][N^T] int32, out: visual token indices of the target set, ascending.
 */
int ficoco_filter(ficoco_ctx *ctx, const ficoco_problem *p, void *ws, size_t ws_bytes,
                  const double *scores, int32_t *discard_idx, int32_t *keep_idx, void *stream);

/*
 * Correlate (Sec. "Correlation-based Information Recycling", Eq. 4, and the threshold /
 * weight lines of Algorithm 1/2 stage 3): for every discarded token the correlation row
 * over the preserved tokens, its eps-quantile tau_i (linear interpolation between order
 * statistics), the targets J_i = { j : C_ij >= tau_i } and the weights
 * alpha_ij = C_ij / sum_{J_i} C_ij.  Needs the workspace left by ficoco_score.
 *   edge_cnt   [B][N^S] int32, out: |J_i| stored for discarded row i (0 = pruned).
 *   edge_tgt   [B][N^S][k_max] int32, out: slots into keep_idx, ascending.
 *   edge_alpha [B][N^S][k_max] double, out.
 *   overflow   [B] int32, out: set to 1 when some row had more than k_max targets (that
 *              image's result is then incomplete: rerun with a larger k_max), else 0.
 */
int ficoco_correlate(ficoco_ctx *ctx, const ficoco_problem *p, void *ws, size_t ws_bytes,
                     const int32_t *discard_idx, const int32_t *keep_idx, int32_t *edge_cnt,
                     int32_t *edge_tgt, double *edge_alpha, int32_t *overflow, void *stream);

/*
 * Pairwise token correlation gap (Sec. "Correlation-based Information Recycling": the
 * difference between the top-1 and the top-2 correlation of every discarded token, the
 * diagnostic behind the token-adaptive K), evaluated in double precision on the exact
 * correlation values.  Needs the workspace state ficoco_correlate needs.
 *   gap [B][N^S] double, out: 0 where fewer than two tokens are preserved.
 */
int ficoco_correlation_gap(ficoco_ctx *ctx, const ficoco_problem *p, void *ws, size_t ws_bytes,
                           const int32_t *discard_idx, const int32_t *keep_idx, double *gap,
                           void *stream);

/*
 * Compress (Eq. 2, self-preserving compression; last lines of Algorithm 1/2): every
 * preserved visual token becomes (X_j + sum_i alpha_ij X_i) / (1 + sum_i alpha_ij), sources
 * added in ascending order; discarded tokens are dropped and every other token of the
 * sequence is copied unchanged, order preserved.
 *   X_out   [B][ficoco_out_rows][D] dtype, out (dense); compress_mode / k_mode select the
 *           ablation variants (average weights; the additional token of the convergent form).
 *   pos_out [B][N^T] int32, out: grid cells of the preserved tokens (may be NULL).
 */
int ficoco_compress(ficoco_ctx *ctx, const ficoco_problem *p, void *ws, size_t ws_bytes,
                    const int32_t *discard_idx, const int32_t *keep_idx, const int32_t *edge_cnt,
                    const int32_t *edge_tgt, const double *edge_alpha, void *X_out,
                    int32_t *pos_out, void *stream);

/*
 * Apply a step's selection to another per-token tensor of the same sequences -- in a decoder
 * the key / value cache of the layers already computed and the position ids have to lose the
 * rows of the discarded visual tokens too (Algorithm 2 removes them from the sequence the
 * following layers see).  out[b][r] = in[b][src(r)] byte for byte, where src(r) walks the
 * sequence in order and skips the discarded tokens: r below vis_begin, then
 * vis_begin + keep_idx[b][r - vis_begin], then r + N^S behind the visual span.
 *   in   [B][n_tot][row_bytes] device, strides in BYTES (row contiguous); row_bytes % 4 == 0.
 *   out  [B][n_tot - N^S][row_bytes] device, dense.
 * Not defined for FICOCO_K_CONVERGENT (its additional token has no row in such tensors):
 * FICOCO_EUNSUPPORTED.  Needs no workspace.
 */
int ficoco_gather_tokens(ficoco_ctx *ctx, const ficoco_problem *p, const int32_t *keep_idx, const void *in,
                         int64_t in_stride_b, int64_t in_stride_n, int32_t row_bytes, void *out,
                         void *stream);

/*
 * Algorithm 1 (FiCoCo-V) / Algorithm 2 (FiCoCo-L) as one call: the four stages above on
 * one stream and one workspace without host synchronisation.  Every output of the stage
 * functions is produced (scores, index sets, edge lists, overflow flags, X_out, pos_out);
 * pos_out may be NULL.  n_keep == N is legal: X_out is then a bit-exact copy of X.
 */
int ficoco_v_step(ficoco_ctx *ctx, const ficoco_problem *p, void *ws, size_t ws_bytes,
                  void *X_out, int32_t *pos_out, int32_t *keep_idx, int32_t *discard_idx,
                  int32_t *edge_cnt, int32_t *edge_tgt, double *edge_alpha, double *scores,
                  int32_t *overflow, void *stream);
int ficoco_l_step(ficoco_ctx *ctx, const ficoco_problem *p, void *ws, size_t ws_bytes,
                  void *X_out, int32_t *pos_out, int32_t *keep_idx, int32_t *discard_idx,
                  int32_t *edge_cnt, int32_t *edge_tgt, double *edge_alpha, double *scores,
                  int32_t *overflow, void *stream);

/*
 * ficoco_v_step for callers that cannot allocate or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and results as
 * ficoco_v_step without `ws` / `ws_bytes`: the step's workspace is a static device array of
 * FICOCO_STATIC_SCRATCH_BYTES inside the library (one copy per GPU, held until the process
 * ends).  The call allocates and frees nothing and launches the same kernels.
 *   - A problem whose ficoco_workspace_bytes exceeds FICOCO_STATIC_SCRATCH_BYTES is rejected
 *     with FICOCO_ENOMEM before anything is launched (the batched 576-token ViT shape,
 *     B = 16, needs about 25 MB and fits).
 *   - All calls on one GPU share that GPU's array: calls that overlap in time on one GPU
 *     (two streams, two threads) race and give undefined results; calls on one stream are
 *     ordered and safe.  The array keeps the previous call's contents; every kernel writes
 *     what it later reads, so nothing has to be cleared between calls.
 */
#define FICOCO_STATIC_SCRATCH_BYTES ((size_t)32 << 20)
int ficoco_v_step_static(ficoco_ctx *ctx, const ficoco_problem *p, void *X_out, int32_t *pos_out,
                         int32_t *keep_idx, int32_t *discard_idx, int32_t *edge_cnt,
                         int32_t *edge_tgt, double *edge_alpha, double *scores, int32_t *overflow,
                         void *stream);

#ifdef __cplusplus
}
#endif
#endif /* FICOCO_H */
