/*
 * stageverify.h -- C ABI of the MI355X (gfx950) stage verifier.
 *
 * A verifier node sits between two pipeline stages and checks what a stage worker
 * submits: activations h^(s) = f_s(h^(s-1); theta^(s)) on the forward pass and
 * activation gradients g^(s) = dL/dh^(s-1) on the backward pass (paper, Problem
 * Statement, "Threat Model" paragraph and Def. threat_model).  This library is the
 * data-parallel part of that node:
 *
 *   sv_verify_forward   recompute f_s on the worker's own micro-batch (duplicate-work
 *                       verification, "Proposed Method" paragraph / FAQ Q9) and score the
 *                       claimed h^(s) against it;
 *   sv_verify_backward  recompute the forward, then the input-gradient backward from the
 *                       downstream gradient, and score the claimed g^(s) (a backward request
 *                       carries the stage input again: SWARM appendix, trainer description);
 *   sv_score_and_flag   the test statistic Gamma = Omega(signal, reference) and the flag rule
 *                       Gamma > tau (Eq. test_statistic) for the distance family of the
 *                       paragraph "Choice of Distance Measure" (mean absolute difference,
 *                       normalised Euclidean, sign flip ratio) plus a per-token relative L2;
 *                       the reference is any tensor: a recomputation or the EMA m_{t-1};
 *   sv_ema_update       Eq. momentum_def over the un-flagged submissions (R_clean of
 *                       Alg. momentum_verification);
 *   sv_score_and_sum, sv_ema_from_sum, sv_sw_against_projection, sv_sw_projection_ema
 *                       the same statistics and update arranged so that a verifier that keeps the
 *                       EMA reads every submission twice instead of three times and never projects
 *                       the EMA (the sum over the clean set from the score pass; the EMA's
 *                       projections carried along by linearity);
 *   sv_sliced_wasserstein, sv_adaptive_iqr / sv_policy_*, sv_replace_with_ema, sv_sentinel_*
 *                       the remaining statistic of that paragraph, the adaptive thresholds and
 *                       counters, gradient replacement, and the whole verifier loop of
 *                       Alg. momentum_verification (declared further down).
 * The stage may carry a dense MLP or a routed mixture of experts (sv_stage_desc); a check only
 * enqueues kernels, so a caller may capture it into a HIP graph after one eager call.
 *
 * Conventions
 *   - Every tensor pointer is a DEVICE pointer owned by the caller; row-major, the feature
 *     dimension innermost.  Activations are [B, S, D] (T = B*S tokens), weights [out, in].
 *     The library never frees or keeps a caller pointer after the stream work it enqueued.
 *   - Every call is asynchronous on `stream` (a hipStream_t passed as void*; NULL = the null
 *     stream) and returns after enqueueing.  Results are written to device memory.
 *   - Errors are returned as sv_status; sv_last_error(ctx) gives a text.  Shapes a kernel
 *     does not support are rejected with SV_EUNSUPPORTED, never mis-computed.
 *   - A context is bound to the device current at sv_create, owns only its workspace, and
 *     is not thread-safe: use one context per stream.
 */
#ifndef STAGEVERIFY_H
#define STAGEVERIFY_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct sv_ctx sv_ctx;

typedef enum { SV_OK = 0, SV_EINVAL = 1, SV_EUNSUPPORTED = 2, SV_ENOMEM = 3, SV_EHIP = 4 } sv_status;
typedef enum { SV_F32 = 0, SV_BF16 = 1 } sv_dtype;
typedef enum { SV_MLP_GELU = 0, SV_MLP_SWIGLU = 1 } sv_mlp;
typedef enum { SV_NORM_LN = 0, SV_NORM_RMS = 1 } sv_norm;
typedef enum { SV_REDUCE_GLOBAL = 0, SV_REDUCE_MAX_TOKEN = 1 } sv_reduce;
typedef enum { SV_ROUTER_SIGMOID = 0, SV_ROUTER_SOFTMAX = 1 } sv_router;

/* metric indices into score[] / tau[] and their mask bits (1 << index) */
enum { SV_IDX_RELL2 = 0, SV_IDX_L1 = 1, SV_IDX_ZL2 = 2, SV_IDX_SFR = 3 };
enum { SV_M_RELL2 = 1, SV_M_L1 = 2, SV_M_ZL2 = 4, SV_M_SFR = 8 };
/* mask bit of the sliced Wasserstein statistic (computed by sv_sliced_wasserstein, no score[] slot) */
enum { SV_M_SW = 16 };

/* sv_create flags */
enum {
  SV_FLAG_BACKWARD = 1,       /* also allocate what sv_verify_backward needs                       */
  SV_FLAG_PLAIN_KERNELS = 2,  /* run the plain fp32-math kernels for every dtype (validation aid)  */
  SV_FLAG_SLICED_W = 4,       /* also allocate the projection scratch of sv_sliced_wasserstein       */
  SV_FLAG_FUSE_NORM = 8       /* bf16 stages with RMSNorm: the two norms of a block run inside the products
                                 around them (the product before leaves each row's sum of squares, the product
                                 after reads the residual stream itself against a copy of its weights with the
                                 norm's gain folded in and scales its rows by 1 / rms); the context then holds
                                 that copy of wq, wk, wv and of the dense MLP's first weights (a mixture of
                                 experts keeps its second norm as a pass of its own).  sv_prepare_weights makes
                                 the copies once; without it every call makes them.  Ignored for fp32 stages,
                                 LayerNorm and SV_FLAG_PLAIN_KERNELS.                                  */
};

/* One pipeline stage = n_blocks identical pre-norm decoder blocks
 *   x1 = x + Attn(Norm1(x)) Wo^T,  y = x1 + MLP(Norm2(x1)).
 * Attention: n_heads query heads of width d_model/n_heads, n_kv_heads key/value heads
 * (query head h reads kv head h / (n_heads/n_kv_heads)), softmax scale 1/sqrt(head_dim),
 * optional causal mask, optional RoPE on interleaved pairs (2i, 2i+1) with angle
 * p * rope_theta^(-2i/head_dim) at in-sequence position p.  No linear biases.            */
typedef struct {
  int32_t n_blocks, d_model, n_heads, n_kv_heads, ffn_hidden;
  int32_t mlp;        /* sv_mlp  */
  int32_t norm;       /* sv_norm */
  int32_t rope;       /* 0 | 1   */
  int32_t causal;     /* 0 | 1   */
  float   norm_eps;
  float   rope_theta;
  int32_t dtype;      /* sv_dtype: storage type of activations, weights, claims */
  /* Mixture-of-experts MLP (the second model family of the paragraph "Alternative Architectures"; expert,
   * shared-expert and top-k counts as in Table model_config).  n_experts = 0: the dense MLP above.  Otherwise
   *   l = n Wr^T,  s = sigmoid(l) or softmax(l) over the experts,  S_t = the top_k experts of token t by s
   *   (decided on l, which orders the experts as s does; ties to the lower index),  g = s on S_t, divided by its sum over S_t if router_norm,
   *   MLP(n) = sum_{e in S_t} g_e SwiGLU_e(n) + SwiGLU_shared(n),
   * every routed expert a SwiGLU MLP of width ffn_hidden, the shared experts side by side as one SwiGLU MLP of
   * width ffn_shared.  No capacity limit: no token is dropped.  Needs mlp = SV_MLP_SWIGLU.                  */
  int32_t n_experts;    /* 0 | 1..16 */
  int32_t top_k;        /* 1..min(8, n_experts) */
  int32_t ffn_shared;   /* 0 = no shared expert */
  int32_t router_score; /* sv_router */
  int32_t router_norm;  /* 0 | 1 */
} sv_stage_desc;

/* Weights of one block, device pointers in the stage dtype, matrices [out, in] row-major. */
typedef struct {
  const void *wq;      /* [n_heads*hd,    d_model] */
  const void *wk;      /* [n_kv_heads*hd, d_model] */
  const void *wv;      /* [n_kv_heads*hd, d_model] */
  const void *wo;      /* [d_model, n_heads*hd]    */
  const void *w_gate;  /* [ffn, d_model]  SwiGLU only; NULL for the GELU MLP      */
  const void *w_up;    /* [ffn, d_model]  (fc1 of the GELU MLP)                   */
  const void *w_down;  /* [d_model, ffn]  (fc2 of the GELU MLP)                   */
  const void *norm1_g; /* [d_model] */
  const void *norm1_b; /* [d_model] LayerNorm only; NULL for RMSNorm              */
  const void *norm2_g;
  const void *norm2_b;
  /* mixture-of-experts blocks only (else NULL): then w_gate / w_up are [n_experts, ffn, d_model] and w_down is
   * [n_experts, d_model, ffn], expert after expert                                                        */
  const void *w_router; /* [n_experts, d_model]  */
  const void *ws_gate;  /* [ffn_shared, d_model] shared experts; NULL when ffn_shared = 0 */
  const void *ws_up;    /* [ffn_shared, d_model] */
  const void *ws_down;  /* [d_model, ffn_shared] */
} sv_block_weights;

/* Verdict for one submission (device memory, 32 bytes). */
typedef struct {
  float    score[4];        /* by SV_IDX_*; the relative L2 always, the others only if in the mask (else 0) */
  uint32_t flag;            /* 1 iff score[i] > tau[i] for some enabled metric i (strict '>')   */
  uint32_t metric_mask;     /* echo of the request                                               */
  float    max_token_rell2; /* max over tokens of ||c_t - r_t|| / max(||r_t||, 1e-30)            */
  int32_t  argmax_token;    /* lowest token index attaining it                                   */
} sv_result;

/* Host-only check of a descriptor against what the kernels support.  No GPU needed.
 * Returns SV_OK, SV_EINVAL (malformed) or SV_EUNSUPPORTED; `msg` (may be NULL) receives a
 * NUL-terminated explanation of at most msg_len bytes.                                     */
sv_status sv_check_desc(const sv_stage_desc *desc, uint32_t flags, char *msg, int32_t msg_len);

/* Workspace bytes sv_create would allocate on the device (host-only arithmetic).            */
int64_t sv_workspace_bytes(const sv_stage_desc *desc, int64_t max_tokens, int32_t max_seq, uint32_t flags);

/* Create a context on the current device for micro-batches of at most max_tokens = B*S
 * tokens and sequences of at most max_seq tokens.  Allocates the workspace (hipMalloc): the
 * intermediates of one block (and, in backward mode, what every block stashes and the
 * transposed weights), the score pass's partial records, and for bf16 stages two fp32 scratch
 * areas that products with few output tiles use (small micro-batches) -- partial products split along k (at most
 * 84 MB) and, in backward mode with grouped-query attention, per-query-head dk | dv
 * contributions (n_heads / n_kv_heads x min(max_tokens, 131072 / n_kv_heads) x 2 x kv width
 * floats).  sv_workspace_bytes gives the total.                                              */
sv_status sv_create(const sv_stage_desc *desc, int64_t max_tokens, int32_t max_seq, uint32_t flags,
                    sv_ctx **out);
void sv_destroy(sv_ctx *ctx);
const char *sv_last_error(const sv_ctx *ctx);  /* ctx may be NULL: last error, on this thread, of a call that takes no context */

/* Forward check.  w: host array of n_blocks sv_block_weights (device pointers inside).
 * h_in [B,S,D] stage input.  claimed_h (nullable) [B,S,D]: scored against the recomputation
 * with metric_mask / tau[4] / reduce; then result_dev (device, 1 element) must be non-NULL.
 * h_hat_out (nullable) receives the recomputed stage output [B,S,D] in the stage dtype.
 * token_scores_out (nullable) receives the per-token relative L2, [B*S] float.              */
sv_status sv_verify_forward(sv_ctx *ctx, const sv_block_weights *w, const void *h_in, int32_t B, int32_t S,
                            const void *claimed_h, uint32_t metric_mask, const float *tau, int32_t reduce,
                            void *h_hat_out, float *token_scores_out, sv_result *result_dev, void *stream);

/* Backward check.  Recomputes the forward from h_in keeping what backward needs, then the
 * gradient with respect to h_in from g_out = dL/d(stage output) [B,S,D]; no weight gradients.
 * claimed_g (nullable) is scored against it.  g_hat_out / h_hat_out (nullable) receive the
 * recomputed input gradient / stage output.  Needs SV_FLAG_BACKWARD at sv_create.           */
sv_status sv_verify_backward(sv_ctx *ctx, const sv_block_weights *w, const void *h_in, const void *g_out,
                             int32_t B, int32_t S, const void *claimed_g, uint32_t metric_mask,
                             const float *tau, int32_t reduce, void *g_hat_out, void *h_hat_out,
                             float *token_scores_out, sv_result *result_dev, void *stream);

/* Mixture-of-experts stages: copy out the routing that the most recent sv_verify_forward / sv_verify_backward call
 * on this context used in block `block`: experts_out [B*S, top_k] int32 in decreasing score order, gates_out
 * [B*S, top_k] float (device pointers, either may be NULL), enqueued on `stream`.  A forward-only context keeps the
 * routing of its last block only (SV_EINVAL for others); a backward context keeps every block's.  A recomputation
 * in another precision may choose differently for a token whose k-th and (k+1)-th scores nearly tie; this call
 * lets a caller tell such tokens from a deviation.                                                         */
sv_status sv_last_routing(sv_ctx *ctx, int32_t block, int32_t *experts_out, float *gates_out, void *stream);

/* Optional, the bf16 matrix-core path: make the context's copies of the stage's weight matrices once (on `stream`)
 * -- for a backward context the matrices transposed to [in, out], with SV_FLAG_FUSE_NORM the gain-folded ones -- so that
 * later sv_verify_forward / sv_verify_backward calls with the SAME sv_block_weights (same pointers) skip making them
 * per call.  The stage parameters are fixed for a whole training iteration while many micro-batches are checked
 * against them.  The caller promises that the weight contents do not change until the next sv_prepare_weights
 * call; w = NULL forgets the copies.  A call with other pointers than the prepared ones makes its copies per call
 * as before.  No-op for contexts that keep no copies.                                                */
sv_status sv_prepare_weights(sv_ctx *ctx, const sv_block_weights *w, void *stream);

/* Stand-alone statistic for n_claims submissions [T, D] (claim i at claims + i*claim_stride
 * elements) against references (ref + i*ref_stride elements; ref_stride 0 = one shared
 * reference, e.g. the EMA).  results_dev: n_claims sv_result.  token_scores_out (nullable):
 * [n_claims, T] float.  ctx is required (it owns the partial-sum scratch); its stage
 * descriptor is not consulted, so any context of the device serves.  D must be a multiple
 * of 8; T * D of one claim must fit int64 and T <= 2^31-1.                                  */
sv_status sv_score_and_flag(sv_ctx *ctx, const void *claims, int64_t claim_stride, int32_t n_claims,
                            const void *ref, int64_t ref_stride, int32_t claim_dtype, int32_t ref_dtype,
                            int64_t T, int32_t D, uint32_t metric_mask, const float *tau, int32_t reduce,
                            float *token_scores_out, sv_result *results_dev, void *stream);

/* sv_score_and_flag for callers that cannot allocate device memory and so cannot call sv_create: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments without the context, same kernels, same
 * results; the partial records (one per submission and 16 tokens) live in a device array that is part of the library's
 * code object: 65536 records = 5 MiB per GPU the library runs on, held until the process ends.  Calls no hipMalloc,
 * hipFree or allocating library routine.  Limit: n_claims * ceil(T / 16) <= 65536 (e.g. 128 submissions of 8192
 * tokens), SV_EUNSUPPORTED beyond it with nothing enqueued; the other limits are sv_score_and_flag's.  The first call
 * on a device looks the array's address up (hipGetSymbolAddress): make it outside a stream capture.  All calls on one
 * GPU share the one array: calls that overlap in time on the same GPU (two streams, two threads) race -- serialise
 * them on one stream.  Nothing has to be cleared between calls: a call writes every record it later reads.
 * Error text: sv_last_error(NULL) on the calling thread.                                                          */
sv_status sv_score_and_flag_noalloc(const void *claims, int64_t claim_stride, int32_t n_claims, const void *ref,
                                    int64_t ref_stride, int32_t claim_dtype, int32_t ref_dtype, int64_t T, int32_t D,
                                    uint32_t metric_mask, const float *tau, int32_t reduce, float *token_scores_out,
                                    sv_result *results_dev, void *stream);

/* m [T, D] float, in place:  m <- beta m + (1-beta) mean_{i: flags[i]==0} claim_i ; unchanged
 * when every claim is flagged.  flags_dev: n_claims bytes on the device (e.g. copied from
 * sv_result.flag), NULL = all clean.  n_claims <= 1024.                                      */
sv_status sv_ema_update(sv_ctx *ctx, float *m, const void *claims, int64_t claim_stride, int32_t n_claims,
                        int32_t claim_dtype, const uint8_t *flags_dev, int64_t T, int32_t D, float beta,
                        void *stream);

/* sv_score_and_flag against ONE shared reference (the momentum of Eq. momentum_def) that also writes what the
 * EMA update over these submissions needs, so that the update does not have to read them again:
 *   sum_out [T, D] float (device) <- sum over the submissions i with skip_host[i] == 0, added in index order.
 * skip_host: n_claims bytes in HOST memory (read during the call), NULL = none skipped: the submissions known to be
 * excluded before they are scored (banned or tainted workers, Alg. momentum_verification).  If the verdicts then
 * exclude nobody else, sv_ema_from_sum finishes the update; otherwise call sv_ema_update with the final flags.
 * Restrictions beyond sv_score_and_flag's: n_claims <= 32 and a row (D elements of the submissions' dtype) must
 * be a multiple of 2 KB -- SV_EUNSUPPORTED otherwise, nothing enqueued (use the two separate calls).           */
sv_status sv_score_and_sum(sv_ctx *ctx, const void *claims, int64_t claim_stride, int32_t n_claims,
                           const void *ref, int32_t claim_dtype, int32_t ref_dtype, int64_t T, int32_t D,
                           uint32_t metric_mask, const float *tau, int32_t reduce, float *token_scores_out,
                           sv_result *results_dev, const uint8_t *skip_host, float *sum_out, void *stream);

/* m [T, D] float, in place:  m <- beta m + (1-beta) / n_summed * sum  (Eq. momentum_def with the mean taken from
 * sv_score_and_sum's sum_out over its n_summed un-skipped submissions); n_summed = 0 leaves m unchanged.
 * D must be a multiple of 8.                                                                               */
sv_status sv_ema_from_sum(sv_ctx *ctx, float *m, const float *sum, int32_t n_summed, int64_t T, int32_t D,
                          float beta, void *stream);

/* Sliced Wasserstein statistic (paragraph "Choice of Distance Measure", Omega_SW): the mean over
 * n_dirs directions u of the 1-Wasserstein distance between the two signals projected on u.  The
 * samples of a signal are its T token vectors in R^D; both sides have T samples, so W1 on the line
 * is the mean absolute difference of the sorted projections.
 *   claims / ref / strides / dtypes : as in sv_score_and_flag (ref_stride 0 = one shared reference,
 *                  projected and sorted once).
 *   directions   : device, bf16 [n_dirs, D] row-major, drawn and normalised by the caller (the
 *                  paper draws them from the unit sphere; they are used as given).
 *   n_dirs       : a multiple of 32, at most 128.   D: a multiple of 64.   n_claims <= 4096.
 *   tau          : threshold; a submission is flagged iff not (Omega_SW <= tau).
 *   sw_out       : device, nullable, [n_claims] float: Omega_SW per submission.
 *   results_dev  : device, nullable, [n_claims] sv_result that an earlier sv_score_and_flag /
 *                  sv_verify_* call on the same stream filled: metric_mask gets SV_M_SW and flag is
 *                  set (never cleared), which keeps the any-metric rule.
 * Needs a context created with SV_FLAG_SLICED_W and T <= its max_tokens; submissions are processed
 * in groups that fit the context's projection scratch.  bf16 signals are projected exactly
 * (bf16 x bf16 products, fp32 accumulation); fp32 signals are split into three bf16 terms first.
 * Errors: SV_EINVAL (null pointers, negative sizes, context without the flag), SV_EUNSUPPORTED
 * (n_dirs, D, n_claims or T outside the limits above), SV_EHIP.                                  */
sv_status sv_sliced_wasserstein(sv_ctx *ctx, const void *claims, int64_t claim_stride, int32_t n_claims,
                                const void *ref, int64_t ref_stride, int32_t claim_dtype, int32_t ref_dtype,
                                int64_t T, int32_t D, const void *directions, int32_t n_dirs, float tau,
                                float *sw_out, sv_result *results_dev, void *stream);

/* The sliced Wasserstein statistic against a reference that is known only through its projections, for a caller
 * that keeps the EMA of Eq. momentum_def: the projection is linear, so the projections of the EMA follow from those
 * of the submissions and the reference itself never has to be projected.
 *   sv_sw_row_len(T)            row length Tpad >= T of the projection arrays below (a power of two)
 *   sv_sw_against_projection    ref_proj [n_dirs, Tpad] float (device, unsorted <u_l, ref_t>; entries t >= T are
 *                               ignored) stands for the reference; claim_proj_out [n_claims, n_dirs, Tpad] float
 *                               (device) receives the submissions' unsorted projections; otherwise as
 *                               sv_sliced_wasserstein.  Needs Tpad <= 16384 and n_claims <= 256 (SV_EUNSUPPORTED beyond).
 *   sv_sw_projection_ema        ref_proj <- beta ref_proj + (1-beta) mean_{i: skip_host[i]==0} claim_proj_i over the
 *                               T samples (skip_host: n_claims bytes in HOST memory, NULL = none; nobody left:
 *                               unchanged); n_claims <= 32.                                                  */
int64_t sv_sw_row_len(int64_t T);
sv_status sv_sw_against_projection(sv_ctx *ctx, const void *claims, int64_t claim_stride, int32_t n_claims,
                                   int32_t claim_dtype, int64_t T, int32_t D, const void *directions, int32_t n_dirs,
                                   const float *ref_proj, float *claim_proj_out, float tau, float *sw_out,
                                   sv_result *results_dev, void *stream);
sv_status sv_sw_projection_ema(sv_ctx *ctx, float *ref_proj, const float *claim_proj, int32_t n_claims,
                               const uint8_t *skip_host, int64_t T, int32_t n_dirs, float beta, void *stream);

/* ---- decision policy (host side: plain double arithmetic on the scalar statistics the kernels emit;
 *      every pointer below is a HOST pointer and no call touches the GPU) -------------------------
 * Tukey fences around the median of a history window (Eq. tukey_fences) with the multiplier k
 * adapted to a target false-positive rate (Alg. adaptive_iqr), and the per-stage bookkeeping of
 * Alg. activation_verification / Alg. gradient_verification.  Readings: percentiles interpolate
 * linearly between order statistics; "outside" the fences is strict; the narrowing loop runs while
 * the outside fraction is below alpha / 10; the history is cut to its last `window` VALUES at the start of a
 * verified step (so the fences adapted at its end see up to window + n_workers values) and at the end of a warm-up
 * step; a deviation
 * of `severe` (paper: 100) times k * IQR from the median bans at once; after t_forgive consecutive
 * clean steps a worker's counter drops by one and the streak restarts.                          */
typedef struct {
  int32_t c;              /* violations that ban a worker (paper: 5)                               */
  int32_t t_forgive;      /* consecutive clean steps that take one violation back (paper: 100)      */
  int32_t window;         /* history length l, in values                                            */
  int32_t n_max;          /* iteration cap of the widening and of the narrowing loop                */
  double  k0;             /* initial multiplier                                                     */
  double  alpha;          /* target false-positive rate                                             */
  double  grow, shrink;   /* gamma_g >= 1, gamma_s in (0, 1]                                        */
  double  min_dist_mult;  /* Lambda: the fences keep at least |median| * Lambda from the median     */
  double  eps;            /* floor of the inter-quartile range                                      */
  double  severe;         /* immediate-ban factor                                                   */
} sv_policy_cfg;
typedef struct sv_policy sv_policy;

/* One run of Alg. adaptive_iqr on history[0..n): returns the fences and the adapted multiplier.    */
sv_status sv_adaptive_iqr(const double *history, int32_t n, double k_prev, const sv_policy_cfg *cfg,
                          double *lower, double *upper, double *k_out);
/* State of one verifier for one stage and one signal kind: n_workers counters, n_metrics histories. */
sv_status sv_policy_create(int32_t n_workers, int32_t n_metrics, const sv_policy_cfg *cfg, sv_policy **out);
void      sv_policy_destroy(sv_policy *p);
/* Warm-up iteration: gamma [n_workers, n_metrics] enters the histories, nothing is flagged.         */
sv_status sv_policy_warmup(sv_policy *p, const double *gamma);
/* One verified iteration.  skip (nullable) [n_workers]: workers not examined (tainted by an earlier
 * stage in this iteration, or absent).  pre_tainted (nullable) [n_workers]: workers that enter this
 * stage's tainted set without being examined (tainted downstream, backward pass).  tainted_out
 * [n_workers]: 1 for workers tainted here (all 0 when more than half of the active workers are in the
 * set).  A worker is flagged iff for some metric not (lower < gamma < upper); before any history
 * exists the fences are infinite.  Banned workers are ignored whatever the masks say.               */
sv_status sv_policy_step(sv_policy *p, const double *gamma, const uint8_t *skip, const uint8_t *pre_tainted,
                         uint8_t *tainted_out);
/* Any output may be NULL: violations/banned [n_workers]; lower/upper/k/history_len [n_metrics].     */
sv_status sv_policy_state(const sv_policy *p, int32_t *violations, uint8_t *banned, double *lower,
                          double *upper, double *k, int32_t *history_len);

/* Alg. gradient_replacement: every signal i in [0, n) with mask_dev[i] != 0 is overwritten with the
 * reference point m [T, D] float (rounded to the signal's dtype); the others are left alone.
 * signals: device, n tensors [T, D] at signals + i*stride elements; mask_dev: device, n bytes.
 * D must be a multiple of 8; n <= 65535.                                                          */
sv_status sv_replace_with_ema(sv_ctx *ctx, void *signals, int64_t stride, int32_t n, int32_t dtype,
                              const uint8_t *mask_dev, const float *m, int64_t T, int32_t D, void *stream);

/* ---- the whole verifier loop (Alg. momentum_verification with Alg. activation_verification,
 *      Alg. gradient_verification and Alg. gradient_replacement) for n_stages pipeline stages with
 *      n_workers workers each; worker r of every stage belongs to data-parallel pipe r.
 * Per stage and signal kind the object owns an EMA m [T, D] float on the device (m_0 = 0) and a
 * decision policy on the host.  One iteration is: sv_sentinel_begin_iteration, sv_sentinel_forward for
 * stage 0 .. n_stages-1, sv_sentinel_backward for stage n_stages-1 .. 0.  A forward / backward call
 *   1. computes Gamma [n_workers, n_metrics] of the workers' signals against the EMA (whole-signal
 *      form of every enabled statistic, columns in the order rel-L2, L1, z-scored L2, sign flips, SW),
 *   2. waits for the stream and runs the policy (warm-up: every value enters the history; else: workers
 *      of a pipe tainted at an earlier stage of this iteration are not examined (forward), workers of a
 *      pipe tainted at a later stage are tainted without examination (backward)),
 *   3. backward only: overwrites the gradient of every worker tainted at this stage in this iteration
 *      (forward or backward) with the gradient EMA of before this call,
 *   4. updates the EMA over the clean set: forward -- not banned, pipe not tainted so far in this
 *      iteration; backward -- not banned, not tainted at this stage.
 * signals: device, [n_workers, T, D] contiguous; tainted_out: HOST, n_workers bytes; gamma_out: HOST,
 * nullable, [n_workers, n_metrics] doubles.  `directions` (device, bf16 [n_dirs, D]) must stay valid
 * while the object lives; SV_M_SW needs a context created with SV_FLAG_SLICED_W and max_tokens >= T.
 * The context must outlive the object; calls on one object must not overlap.
 * Device memory the object holds: two EMAs [T, D] float per stage, and -- with at most 32 workers -- one more
 * [T, D] float (the score pass leaves the sum over the signals there: sv_score_and_sum) and, with SV_M_SW and
 * sv_sw_row_len(T) <= 16384, the projections of the EMAs and of the current signals
 * ((2 n_stages + n_workers) [n_dirs, sv_sw_row_len(T)] floats: sv_sw_against_projection).             */
typedef struct {
  int32_t n_stages, n_workers;
  int64_t T;
  int32_t D;
  uint32_t metric_mask;            /* SV_M_RELL2 | SV_M_L1 | SV_M_ZL2 | SV_M_SFR | SV_M_SW, at least one */
  int32_t n_dirs;
  const void *directions;
  float beta_h, beta_g;            /* EMA coefficients of activations / gradients                      */
  sv_policy_cfg policy_h, policy_g;
} sv_sentinel_cfg;
typedef struct sv_sentinel sv_sentinel;
sv_status sv_sentinel_create(sv_ctx *ctx, const sv_sentinel_cfg *cfg, sv_sentinel **out);
void      sv_sentinel_destroy(sv_sentinel *s);
const char *sv_sentinel_last_error(const sv_sentinel *s);
sv_status sv_sentinel_begin_iteration(sv_sentinel *s, int32_t warmup);
sv_status sv_sentinel_forward(sv_sentinel *s, int32_t stage, const void *h, int32_t dtype, uint8_t *tainted_out,
                              double *gamma_out, void *stream);
sv_status sv_sentinel_backward(sv_sentinel *s, int32_t stage, void *g, int32_t dtype, uint8_t *tainted_out,
                               double *gamma_out, void *stream);
/* kind 0 = activations, 1 = gradients.  Any output may be NULL: *ema_dev = the device EMA (owned by the
 * object); violations/banned [n_workers]; lower/upper/k [n_metrics] (HOST).                          */
sv_status sv_sentinel_state(const sv_sentinel *s, int32_t stage, int32_t kind, const float **ema_dev,
                            int32_t *violations, uint8_t *banned, double *lower, double *upper, double *k);

/* Copies the EMA of (stage, kind) to out_host (HOST, T*D floats) after the work queued on `stream`.   */
sv_status sv_sentinel_read_ema(sv_sentinel *s, int32_t stage, int32_t kind, float *out_host, void *stream);
/* How the stage calls so far were served: counts[0] stage calls, counts[1] EMA updates finished from the score pass's
 * sum, counts[2] EMA updates that read the signals themselves (shape not taken by the summing pass, no buffer, or a
 * verdict that excluded somebody beyond the workers known beforehand), counts[3] sliced Wasserstein checks against
 * carried projections of the EMA.  counts: HOST, 4 entries.                                                */
sv_status sv_sentinel_counters(const sv_sentinel *s, int64_t *counts);

/* Per-operation timing with HIP events recorded on the caller's stream around each launch.
 * sv_profile_enable(ctx, 1) clears the accumulators and starts recording; (ctx, 0) stops.
 * sv_profile_read waits for the recorded events and returns, per operation class, the summed
 * kernel time in ms, the algorithmic FLOP (2 M N K per product, causal attention at half the
 * dense count) and the number of launches.  Recording adds two event records per launch.    */
enum {
  SV_OP_NORM = 0, SV_OP_GEMM_QKV, SV_OP_ROPE, SV_OP_ATTN, SV_OP_GEMM_O, SV_OP_GEMM_GATEUP, SV_OP_GEMM_DOWN,
  SV_OP_SCORE, SV_OP_BWD_GEMM_DA, SV_OP_BWD_GEMM_DN2, SV_OP_BWD_NORM, SV_OP_BWD_GEMM_DO, SV_OP_BWD_ATTN,
  SV_OP_BWD_ROPE, SV_OP_BWD_GEMM_DN1, SV_OP_BWD_WTRANSPOSE, SV_OP_SW_PROJECT, SV_OP_SW_SORT, SV_OP_MOE_ROUTE,
  SV_OP_MOE_PERMUTE, SV_OP_BWD_MOE,
  SV_OP_NORM_PIECES,   /* SV_FLAG_FUSE_NORM: the rows' 1 / rms (from the stream or from the partial sums) and gain folding */
  SV_OP_COUNT
};
typedef struct {
  double  ms[SV_OP_COUNT];
  double  flop[SV_OP_COUNT];
  int64_t launches[SV_OP_COUNT];
} sv_profile;
sv_status sv_profile_enable(sv_ctx *ctx, int32_t on);
sv_status sv_profile_read(sv_ctx *ctx, sv_profile *out);
/* Bracket only the operation classes whose bit (1 << SV_OP_*) is set in op_mask; 0 = all of them again (the
 * default).  Events around every launch cost a check of many short launches a few per cent; a caller that times
 * whole checks and wants one kernel's duration from the same run selects that class alone.              */
sv_status sv_profile_select(sv_ctx *ctx, uint64_t op_mask);

/* Tuning and test aid: one bf16 product C[M,N] = A[M,K] * op(B) on the MFMA GEMM kernels that
 * the block recompute uses (fp32 accumulation, bf16 result).  b_is_kn = 0: B stored [N,K]
 * (C = A B^T); 1: B stored [K,N] (C = A B).  tile: 0 = automatic, 1 = 256x256 (direct-to-LDS
 * loads when B is [N,K]), 2 = 128x128, 3 = 256x256 with register-staged loads, 4 = 128 rows x 64
 * columns (B stored [N,K] only; what the automatic choice takes when 128x128 tiles would leave CUs idle).
 * Returns SV_EUNSUPPORTED for shapes outside the kernels' limits (N % 128, K % 64, 16-byte
 * aligned rows).  No context is needed.                                                      */
sv_status sv_gemm_bf16(const void *A, int64_t lda, const void *B, int64_t ldb, int32_t b_is_kn, void *C, int64_t ldc,
                       int32_t M, int32_t N, int32_t K, int32_t tile, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* STAGEVERIFY_H */
