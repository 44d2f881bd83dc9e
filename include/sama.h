/*
 * sama.h -- C ABI of the MI355X (gfx950) implementation of SAMA's per-iteration meta-gradient step
 * ("Making Scalable Meta Learning Practical", Sec. 2-3) on the data-reweighting bilevel problem of Sec. 4.1:
 *
 *     base:  theta*(lambda) = argmin_theta (1/B_eff) sum_i mask_i w(l_i; lambda) l_i(theta)      (noisy batch)
 *     meta:  lambda*        = argmin_lambda mean_j l_j(theta*(lambda))                           (clean batch)
 *
 * l_i is the per-sample cross-entropy of the base learner f(x_i; theta); w(.; lambda) is a 1 -> H -> 1
 * weighting net (ReLU hidden layer, sigmoid output) applied to l_i.
 *
 * Conventions
 *  - Every pointer marked DEVICE is memory of the GPU that was current at sama_init; HOST is ordinary memory.
 *  - The library allocates no device memory: the caller hands sama_init one workspace of
 *    sama_workspace_bytes() bytes (256-byte aligned) and keeps it alive until sama_destroy.
 *  - All work is enqueued on the hipStream_t given to sama_init and returns without waiting for it, except
 *    where a function says it synchronises.  Batches and outputs must stay valid until the stream has passed
 *    the call.  Calls on one context must not overlap from several threads.  The encoder's backward passes also use
 *    a second stream of the library's own (default priority, created at the first such pass, destroyed by
 *    sama_destroy); it forks from and joins the given stream by events inside each call, so the ordering a caller
 *    sees is that of the given stream alone.
 *  - sama_base_step / sama_meta_grad / sama_meta_step (and their sama_aux_* forms) may be captured into a HIP graph on
 *    the context's stream once each of them has run eagerly (the first calls create the second stream and set
 *    kernel attributes): step counts and the optimizer's step-dependent scalars live on the device, so a replay
 *    continues where the last execution stopped.  Batch and output pointers are baked into the capture.  The
 *    host-side check that a meta gradient follows a base step looks at eager calls only.  sama_set_state(COUNTERS)
 *    and the profile functions synchronise or record timing events and do not belong into a capture.
 *  - Return value: SAMA_OK or an error detected on the host (nothing is enqueued after an error).  Conditions
 *    only the device can see (a zero or non-finite ||v||) set a status word readable through
 *    sama_get_state(SAMA_STATE_COUNTERS) and turn that meta step into a no-op with a zero hypergradient.
 *
 * Parameter layout (theta, and every theta-sized state vector), flat fp32, n = sama_param_count():
 *    all GEMM weight matrices, each [out x in] row-major, in layer order; then every other tensor in layer order.
 *    MLP  dims = {d0, d1, ..., dL}:    W_0[d1 x d0] ... W_{L-1}[dL x d_{L-1}],  b_0[d1] ... b_{L-1}[dL]
 *         (two dims = multinomial logistic regression; hidden layers use ReLU)
 *    ENCODER dims = {L, d, heads, ffn, S, V, C}  (post-LN, learned positions, erf-GELU, LN eps 1e-5,
 *         softmax(q k^T / sqrt(d/heads)) over the real tokens of a sequence (sama_batch.seq_len), classifier on the
 *         position-0 hidden state; supported shapes: S = 64, 128 or 256, d / heads = 64, d <= 2048, ffn % 64 = 0,
 *         at most 8192 token rows per batch):
 *         per layer l: Wqkv[3d x d] (rows 0..d-1 = Q, d..2d-1 = K, 2d..3d-1 = V; head h owns rows h*d/heads..),
 *                      Wo[d x d], W1[ffn x d], W2[d x ffn];
 *         then per layer l: bqkv[3d], bo[d], ln1_g[d], ln1_b[d], b1[ffn], b2[d], ln2_g[d], ln2_b[d];
 *         then tok_emb[V x d], pos_emb[S x d], emb_ln_g[d], emb_ln_b[d], Wc[C x d], bc[C].
 *         With aux_mlm = 1 (masked-token head, token logits = x_L[row] Wmlm^T + bmlm): Wmlm[V x d] follows the last
 *         layer's W2 among the matrices and bmlm[V] sits between emb_ln_b and Wc.
 *    sama_param_tensor() enumerates the same table.
 * lambda layout, flat fp32, n_lambda = sama_lambda_count():  the weighting net W1[H], b1[H], W2[H], b2[1]; then, when
 *    label correction is on (corr_hidden = Hc > 0), the corrector  W1c[Hc x 2C], b1c[Hc], W2c[C x Hc], b2c[C].
 *
 * Label correction (the second meta learner of Sec. 4.1): the base loss of a noisy sample becomes the cross-entropy
 * against a corrected soft label, l_i = -sum_k c_ik log softmax(z_i)_k.  The paper names the corrector only as a
 * 2-layer MLP; here c_i = softmax(kappa onehot(y_i) + W2c relu(W1c [onehot(y_i), softmax(z_i)] + b1c) + b2c), with
 * softmax(z_i) entering as a constant.  The meta batch keeps its hard labels.
 */
#ifndef SAMA_H
#define SAMA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct sama_ctx sama_ctx; /* opaque; owned by the library, freed by sama_destroy */

typedef enum {
  SAMA_OK = 0,
  SAMA_EINVAL = 1,     /* bad argument or unsupported shape */
  SAMA_ESTATE = 2,     /* call order: sama_meta_grad / sama_meta_step before any sama_base_step */
  SAMA_EWORKSPACE = 3, /* workspace missing, misaligned or too small */
  SAMA_EHIP = 4,       /* a HIP runtime call failed; see sama_last_error */
  SAMA_ENONFINITE = 5  /* never returned by the library (non-finite values are only visible on the device): the code a
                          caller may use to report a raised status word */
} sama_status;

enum { SAMA_MODEL_MLP = 0, SAMA_MODEL_ENCODER = 1 };
enum { SAMA_DTYPE_FP32 = 0, SAMA_DTYPE_BF16 = 1 }; /* BF16: bf16 GEMM operands, fp32 master weights / moments / gradients */
enum { SAMA_OPT_SGD = 0, SAMA_OPT_ADAM = 1 };
enum { SAMA_ADAPT_OPTIMIZER = 0, SAMA_ADAPT_NONE = 1 };

/* Plain data, copied by sama_init. */
typedef struct {
  int32_t model_kind;  /* SAMA_MODEL_* */
  int32_t n_dims;      /* number of entries used in dims */
  int32_t dims[8];     /* see "Parameter layout" */
  int32_t param_dtype; /* SAMA_DTYPE_*; the encoder requires BF16, the MLP requires FP32 */
  int32_t wnet_hidden; /* H, 1..256 */
  int32_t base_opt;    /* SAMA_OPT_*: the base-level solver u of Sec. 2 */
  float base_lr, beta1, beta2, adam_eps; /* gamma, beta_1, beta_2, epsilon of App. C */
  float weight_decay;  /* L2 coefficient (the wdecay column of App. B): weight_decay * theta is added to the base gradient
                        * before the solver; the G state and the adaptation of Eq. 4 use that sum */
  float momentum;      /* SGD only: heavy-ball momentum mu in [0, 1), b <- mu b + g, theta <- theta - base_lr b (the velocity b
                        * is the M state).  du/dg stays base_lr, so the adaptation of Eq. 4 is unchanged.  Must be 0 for Adam */
  float meta_lr, meta_beta1, meta_beta2, meta_eps; /* Adam on lambda (Table 4) */
  float alpha;         /* eps = alpha / ||v||_2, Sec. 3.2 below Eq. 5 */
  int32_t adapt_mode;  /* SAMA_ADAPT_OPTIMIZER: du/dg of base_opt (App. C for Adam, gamma for SGD);
                          SAMA_ADAPT_NONE: identity, the SAMA-NA ablation of Sec. 4.1 */
  int32_t max_batch;      /* largest train batch that will be passed, 1..2048 */
  int32_t max_meta_batch; /* largest meta batch, 1..2048 */
  int32_t fast_meta_pass; /* BF16 models only.  0 (default): the direct-gradient pass of Eq. 1 contracts with the
                             two-term split hi + lo of the fp32 master weights, so dL_meta/dtheta is taken at theta
                             and not at bf16(theta) (costs two extra forward-equivalents of GEMM work per meta
                             step).  1: that pass uses the bf16 working copy like a base step. */
  int32_t fast_base_pass; /* BF16 models only.  0 (default): the base step's forward and input-gradient GEMMs contract with the
                             same two-term split hi + lo, so the base gradient g (and with it the adaptation of Eq. 4) is
                             taken at the fp32 master theta; this is what matches the float64 reference from any state (costs
                             two extra forward-equivalents of GEMM work per base step).  1: ordinary mixed precision -- the
                             base step sees only the bf16 working copy, whose rounding hides updates smaller than half a
                             bf16 ulp of a weight (every update at learning rates around 1e-5). */
  int32_t corr_hidden;    /* Hc: hidden width of the label corrector, 0 = no label correction, at most 128; needs C <= 16 */
  float corr_kappa;       /* kappa >= 0: fixed prior on the given label inside the corrector */
  int32_t aux_mlm;        /* 1: auxiliary-task reweighting (Sec. 4.3).  ENCODER only; theta gains a masked-token head
                             (Wmlm [V x d] after the layers' matrices, bmlm [V] before Wc); V must be a multiple of 64;
                             cannot be combined with corr_hidden > 0.  The sama_aux_* entry points need it. */
  int32_t max_aux_batch;  /* aux_mlm: largest number of auxiliary sequences per batch; (max_batch + max_aux_batch) * S
                             and max_meta_batch * S must stay within the encoder's 8192-token limit */
  int32_t max_aux_masked; /* aux_mlm: largest number of masked positions per auxiliary batch, 1..max_aux_batch * S */
} sama_config;

/* One batch.  x: DEVICE, fp32 [n x d0] row-major (MLP) or int32 token ids [n x S] (ENCODER), ids in [0, V).
 * y: DEVICE int32 [n], labels in [0, C).  Token ids and labels outside their range are clamped into it on the device,
 * not reported (the same rule as for the rows and targets of sama_aux_batch).  sample_mask: DEVICE uint8 [n], 1 = use, 0 = ignore, or NULL = use all.
 * seq_len (ENCODER; ignored by the MLP): DEVICE int32 [n], the number of real tokens of each padded sequence, or NULL =
 * every sequence fills all S positions.  Keys at positions >= seq_len get no attention weight (key-padding mask);
 * values are clamped into [1, S]; what sits in the padded positions of x then has no influence on any result.
 * Read-only; owned by the caller. */
typedef struct {
  const void* x;
  const int32_t* y;
  const uint8_t* sample_mask;
  int32_t n;
  const int32_t* seq_len;
} sama_batch;

/* One batch of the auxiliary (masked-token) task.  ids: DEVICE int32 [n_seq x S], the input tokens with the masked
 * positions already replaced by the caller.  mask_row: DEVICE int32 [n_mask], token row sequence * S + position of
 * each masked position, all distinct, every sequence owning at least one; mask_tgt: DEVICE int32 [n_mask], the token
 * to predict there.  Out-of-range rows / targets are clamped into range, not reported.  seq_len: as in sama_batch
 * ([n_seq] or NULL); masked positions should be real tokens.  Read-only; caller-owned. */
typedef struct {
  const int32_t* ids;
  const int32_t* mask_row;
  const int32_t* mask_tgt;
  int32_t n_seq, n_mask;
  const int32_t* seq_len;
} sama_aux_batch;

/* Selectors of sama_get_state / sama_set_state.  Sizes in elements:
 * THETA, M, V, G, GMETA, VDIR: n fp32 (M, V = Adam moments m, v of App. C; G = g_base of the last base step,
 * Eq. 4; GMETA = dL_meta/dtheta, Eq. 1; VDIR = the perturbation vector v of Eq. 5);
 * LAMBDA, META_M, META_V, HYPERGRAD, GLAM_PLUS, GLAM_MINUS: n_lambda fp32;
 * COUNTERS: 4 int64 = {base step count t, meta step count, status word (0 ok, 1 = last meta step skipped: ||v|| was zero or
 * not finite, or the hypergradient was not finite; lambda, theta and the meta moments are then left as they were, up to
 * one fp32 rounding of theta's GEMM block, which is nudged early and nudged back), 0};
 * SCALARS: 4 fp32 = {eps of the last meta gradient, ||v||_2, L_base of the last base step, L_meta of the last meta pass};
 * LOSSES: max(max_batch (+ max_aux_batch with aux_mlm), max_meta_batch) fp32, per-sample losses of the most recent
 * forward pass. */
enum {
  SAMA_STATE_THETA = 0, SAMA_STATE_LAMBDA = 1, SAMA_STATE_M = 2, SAMA_STATE_V = 3, SAMA_STATE_G = 4,
  SAMA_STATE_GMETA = 5, SAMA_STATE_VDIR = 6, SAMA_STATE_META_M = 7, SAMA_STATE_META_V = 8,
  SAMA_STATE_COUNTERS = 9, SAMA_STATE_HYPERGRAD = 10, SAMA_STATE_GLAM_PLUS = 11, SAMA_STATE_GLAM_MINUS = 12,
  SAMA_STATE_SCALARS = 13, SAMA_STATE_LOSSES = 14
};

/* Shape queries (host only, no GPU needed).  Return -1 / 0 on an invalid config. */
int64_t sama_param_count(const sama_config* cfg);      /* n = dim theta */
int64_t sama_gemm_param_count(const sama_config* cfg); /* leading part of theta held by GEMM weight matrices */
int32_t sama_lambda_count(const sama_config* cfg);     /* 3H + 1 */
int32_t sama_param_tensor_count(const sama_config* cfg);
/* idx-th tensor of the layout table: name (<= 31 chars + NUL) copied to name_out[32], flat offset, rows, cols
 * (cols = 1 for vectors).  SAMA_EINVAL when idx is out of range. */
sama_status sama_param_tensor(const sama_config* cfg, int32_t idx, char* name_out, int64_t* offset,
                              int64_t* rows, int64_t* cols);
size_t sama_workspace_bytes(const sama_config* cfg);

/* Create a context (the bilevel problem statement of Sec. 2 with the solver of Eq. 2): copies theta0 (DEVICE
 * fp32 [n]) and lambda0 (DEVICE fp32 [n_lambda]) into the workspace, zeroes moments and counters.
 * hip_stream: a hipStream_t (NULL = the default stream).  *out is set only on SAMA_OK. */
sama_status sama_init(const sama_config* cfg, void* workspace /*DEVICE*/, size_t workspace_bytes,
                      const float* theta0 /*DEVICE*/, const float* lambda0 /*DEVICE*/, void* hip_stream,
                      sama_ctx** out);

/* One step of the base solver u on L_base (Sec. 2; Sec. 4.1 objective): forward, w_i = w(l_i; lambda) held
 * constant in the backward pass, g = dL_base/dtheta, Adam (bias-corrected) or SGD update; keeps g and the
 * post-update moments for the adaptation of Eq. 4.  loss_out: DEVICE fp32 scalar receiving L_base, or NULL. */
sama_status sama_base_step(sama_ctx* ctx, const sama_batch* train, float* loss_out /*DEVICE*/);

/* The meta gradient of Eq. 5 at the current state:
 *   g_meta = dL_meta/dtheta on `meta` (Eq. 1);  v = (du/dg_base) . g_meta (Eq. 4, App. C);  eps = alpha/||v||_2;
 *   h = -(dL_base(theta + eps v, lambda)/dlambda - dL_base(theta - eps v, lambda)/dlambda) / (2 eps)
 * with both lambda-gradients taken on `train` (the batch of the last base step).  Leaves theta, lambda and all
 * moments unchanged.  hypergrad_out: DEVICE fp32 [n_lambda] or NULL; eps_out: DEVICE fp32 scalar or NULL.
 * SAMA_ESTATE before the first sama_base_step. */
sama_status sama_meta_grad(sama_ctx* ctx, const sama_batch* train, const sama_batch* meta,
                           float* hypergrad_out /*DEVICE*/, float* eps_out /*DEVICE*/);

/* sama_meta_grad, then one Adam step on lambda with h (Table 4), then theta <- theta - eps v (end of
 * Sec. 3.2).  The base moments and step count are not touched.
 * Note for Adam base solvers: after the very first base step from zero moments the update is lr * sign(g), so the
 * adaptation of Eq. 4 vanishes analytically and v holds nothing but rounding noise, which eps = alpha / ||v|| scales to
 * a step of norm alpha.  Only an exactly zero ||v|| is skipped; run at least two base steps before the first meta step. */
sama_status sama_meta_step(sama_ctx* ctx, const sama_batch* train, const sama_batch* meta);

/* Auxiliary-task reweighting (Sec. 4.3): L_base = L_ft(ft) + (1/n_seq) sum_x w(L_pt(x); lambda) L_pt(x) over the
 * auxiliary sequences x, L_ft the mean classifier cross-entropy on `ft` (its sample_mask honoured), L_pt(x) the mean
 * masked-token cross-entropy over x's masked positions, w the weight net on that loss (a constant of the backward
 * pass).  One forward / backward over the concatenated batch, then the base solver's update as in sama_base_step.
 * ft->n <= max_batch, pt->n_seq <= max_aux_batch, pt->n_mask <= max_aux_masked.  Afterwards LOSSES holds
 * [classifier losses of ft | L_pt of the auxiliary sequences].  loss_out as in sama_base_step. */
sama_status sama_aux_base_step(sama_ctx* ctx, const sama_batch* ft, const sama_aux_batch* pt, float* loss_out /*DEVICE*/);

/* Eq. 5 for that problem: g_meta = dL_ft/dtheta on `meta`; v, eps as in sama_meta_grad; the two lambda-gradients are
 * taken on `pt` alone (the finetuning term of L_base does not depend on lambda).  `pt` is the auxiliary batch of the
 * last sama_aux_base_step.  sama_aux_meta_step then updates lambda and nudges theta like sama_meta_step. */
sama_status sama_aux_meta_grad(sama_ctx* ctx, const sama_aux_batch* pt, const sama_batch* meta,
                               float* hypergrad_out /*DEVICE*/, float* eps_out /*DEVICE*/);
sama_status sama_aux_meta_step(sama_ctx* ctx, const sama_aux_batch* pt, const sama_batch* meta);

/* A forward-only look at a batch through the current theta and lambda, as the base step of Sec. 4.1 sees it:
 * logits_out [n x C] (row-major), losses_out [n] = l_i (against the corrected soft label when label correction is on),
 * weights_out [n] = w(l_i; lambda) -- the per-sample importance the meta learner has learned (what the reweighting and
 * pruning applications of Sec. 4 read off it).  DEVICE pointers, each may be NULL.  n up to max(max_batch,
 * max_meta_batch); sample_mask is ignored, seq_len honoured.  bf16 models evaluate with the weights the base
 * step's forward uses (fast_base_pass).  Changes no state (LOSSES and SCALARS keep what the last step left). */
sama_status sama_eval(sama_ctx* ctx, const sama_batch* batch, float* logits_out /*DEVICE*/, float* losses_out /*DEVICE*/,
                      float* weights_out /*DEVICE*/);

/* The same look at an auxiliary batch (Sec. 4.3): losses_out [n_seq] = L_pt(x), the mean masked-token loss of each
 * sequence, and weights_out [n_seq] = w(L_pt(x); lambda), how much the meta learner lets each auxiliary sequence count.
 * DEVICE pointers, each may be NULL; changes no state. */
sama_status sama_aux_eval(sama_ctx* ctx, const sama_aux_batch* pt, float* losses_out /*DEVICE*/, float* weights_out /*DEVICE*/);

/* Learning-rate schedule hook (the lr_scheduler column of the App. B tables: cosine, linear decay with warm-up, ...;
 * the schedule itself is the caller's).  base_lr applies from the next base step, meta_lr from the next meta update;
 * the adaptation of Eq. 4 keeps using the rate of the base step it differentiates, whenever this is called.  Host
 * side only, nothing is enqueued; both must be finite and > 0.  Rates are kernel arguments: a captured graph replays
 * with the rates in force at capture. */
sama_status sama_set_lr(sama_ctx* ctx, float base_lr, float meta_lr);

/* Copy a state vector out of / into the context (DEVICE pointers; sizes above).  Enqueued on the context's
 * stream.  sama_set_state(COUNTERS) synchronises the stream (the base step count lives on the host);
 * setting THETA also refreshes the bf16 working copy.  SCALARS, LOSSES, HYPERGRAD, GLAM_* are read-only.
 * The settable selectors (THETA, M, V, G, LAMBDA, META_M, META_V, COUNTERS) are a complete checkpoint: a fresh context
 * of the same configuration that is handed them continues a run with the same bits (set the learning rates in force
 * with sama_set_lr before COUNTERS). */
sama_status sama_get_state(sama_ctx* ctx, int32_t which, void* dst /*DEVICE*/);
sama_status sama_set_state(sama_ctx* ctx, int32_t which, const void* src /*DEVICE*/);

/* Text of the last error on this context (HOST string owned by the context; "" if none).  ctx may be NULL,
 * which returns the text of the last failed sama_init on this thread. */
const char* sama_last_error(const sama_ctx* ctx);

/* Optional per-kernel timing, for roofline reports (not part of the method).  While enabled, every kernel launch
 * of this library in the process is bracketed by two HIP events on its stream, which costs a few microseconds
 * per launch: keep it off in throughput runs.  sama_profile_enable(ctx, 1) clears earlier records.
 * sama_profile_read synchronises with the recorded events and returns, for kernel family `family`
 * (0 .. sama_profile_family_count()-1): its name (HOST string owned by the library), the number of launches, their
 * summed duration in milliseconds and their summed algorithmic work: flops for the GEMM and attention families,
 * bytes for the others (Adam 28 B per parameter + 4 B per GEMM weight -- the bf16 working copy and its residual half;
 * adaptation 20 B; +-eps halves 12 B per GEMM weight, or 18 B when sama_meta_step nudges the GEMM block in the same
 * pass; residual half alone 6 B; nudge 12 B + 2 B per bf16 array it refreshes over the elements it covers).  Two-term (hi + lo) GEMM launches are families of their own
 * ("..._hilo") and count 2 M N (2K): they contract over the concatenated operand. */
int32_t sama_profile_family_count(void);
sama_status sama_profile_enable(sama_ctx* ctx, int32_t on);
sama_status sama_profile_read(sama_ctx* ctx, int32_t family, const char** name, int64_t* launches, double* total_ms,
                              double* units);

/* Free the host-side context.  The workspace stays with the caller.  Does not synchronise. */
void sama_destroy(sama_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* SAMA_H */
