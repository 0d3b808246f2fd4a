/*
 * spo.h - C ABI of the MI355X (gfx950) hot path of Single-stream Policy
 * Optimization (SPO, arXiv 2509.13232).
 *
 * Conventions for every entry point
 *   - All array arguments are DEVICE pointers owned by the caller; the library
 *     never allocates or frees memory.  Scratch comes from a caller-provided
 *     workspace whose size the matching *_workspace_bytes() query returns.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*; NULL is the
 *     default stream) and the call returns without waiting for it.
 *   - Scalars are host values.  Argument errors are detected on the host
 *     before anything is launched: the call returns a negative status and
 *     leaves all outputs untouched.  0 is success.
 *   - No global state (the optional kernel timing at the end of this file
 *     aside).  Calls that share output or workspace memory must be ordered by
 *     the caller (same stream or events).
 *
 * One training iteration calls, in this order (training-loop algorithm of the
 * paper): spo_sample_prompts -> [rollout, outside this library] ->
 * spo_advantages -> spo_tracker_update -> per mini-batch spo_pg_loss_fwd /
 * spo_pg_loss_bwd, or spo_pg_loss_fwd_bwd when the weight of the loss in the
 * total is known beforehand.  spo_advantages must see the tracker BEFORE
 * spo_tracker_update: the baseline of an advantage is the pre-update estimate.
 */
#ifndef SPO_H_
#define SPO_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SPO_OK 0
#define SPO_EINVAL (-1)       /* a size, flag or scalar is out of its domain   */
#define SPO_ENULL (-2)        /* a required pointer is NULL                    */
#define SPO_ERANGE (-3)       /* a size exceeds what the kernels support       */
#define SPO_EWORKSPACE (-4)   /* workspace missing or smaller than required    */
#define SPO_EUNSUPPORTED (-5) /* valid request that this build does not cover  */
#define SPO_EHIP (-6)         /* the HIP runtime reported an error at launch   */

#define SPO_FP32 0
#define SPO_BF16 1

/* Memory order of the LM-head matrix W (logical shape H x V). */
#define SPO_W_VH 0 /* W[v*H + h]: one contiguous row of H values per vocabulary entry */
#define SPO_W_HV 1 /* W[h*V + v]: one contiguous row of V values per hidden unit      */

typedef void *spo_stream_t;

const char *spo_status_string(int status);

/* ---------------------------------------------------------------------------
 * Prioritized prompt sampling (Method, "Prioritized Prompt Sampling": the
 * sampling-weight equation w(x) ~ sqrt(v(1-v)) + eps with v = alpha/(alpha+beta)
 * the tracker mean, and the step of the training loop that draws a batch of B
 * prompts according to these weights).
 *
 * The draw is defined so that it has exactly one answer on any machine:
 *   weight    w_i  = sqrt(v_i (1 - v_i)) + eps_explore, evaluated in IEEE fp64
 *                    from the fp32 tracker (an entry with alpha+beta <= 0 gets
 *                    eps_explore alone);
 *   code      c_i  = floor(w_i * 2^32) as a 64-bit integer;
 *   CDF       C_i  = c_0 + ... + c_i (exact integers);
 *   slot k, attempt a: 64 random bits r = lo | hi<<32 of the first two words of
 *                    Philox4x32-10 with key (seed lo, seed hi) and counter
 *                    (k, a, iteration lo, iteration hi);
 *                    t = floor(r * C_{N-1} / 2^64); index = first i with C_i > t;
 *   replace = 1:     slot k takes attempt 0 (independent weighted draws);
 *   replace = 0:     slot k takes its first attempt whose index is not held by
 *                    a lower slot (successive weighted sampling without
 *                    replacement); needs B <= N.
 *
 * alpha, beta   [N] fp32, read only.
 * idx_out       [B] int32.
 * info          optional int32[2]: info[0] = 0, or 1 if some slot ran out of
 *               attempts (its idx_out entries are then -1); info[1] = largest
 *               attempt number used.  If every weight is zero (eps_explore = 0
 *               and every v_i is 0 or 1) nothing can be drawn: all entries are
 *               -1 and info[0] = 1.
 * max_attempts  bound on attempts per slot (0 selects 65536).  Without replacement the
 *               draw runs in one workgroup, one sweep over the B slots per attempt
 *               level (about 2 us each): a batch that takes most of the prompts
 *               with non-zero weight needs many levels for its last slots (about
 *               N ln N draws to collect the last of N equal weights), so such a
 *               call can take max_attempts sweeps before it gives up; info[0] and
 *               info[1] tell.
 * ws            spo_sample_prompts_workspace_bytes(N, B) bytes, 256-byte aligned.
 * Limits: 1 <= N < 2^31, 1 <= B <= 16384 (replace = 0) or B < 2^31 (replace = 1).
 * ------------------------------------------------------------------------- */
size_t spo_sample_prompts_workspace_bytes(int64_t N, int32_t B);
int spo_sample_prompts(const float *alpha, const float *beta, int64_t N, int32_t B,
                       double eps_explore, uint64_t seed, uint64_t iteration, int replace,
                       uint32_t max_attempts, int32_t *idx_out, int32_t *info, void *ws,
                       size_t ws_bytes, spo_stream_t stream);

/* The same draw for callers that cannot allocate device memory or carry a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Arguments, result and errors are those of spo_sample_prompts
 * without ws / ws_bytes; the CDF, the block sums and the owner table live in a
 * fixed array of about 12.6 MB in device memory that belongs to the library (one
 * copy per GPU, held until the process ends).  The call allocates nothing; its
 * first call on a device looks the array's address up once.
 * Limit: N <= SPO_SAMPLE_STATIC_MAX_N, otherwise SPO_ERANGE.
 * Every call on a GPU uses that GPU's one array: calls that overlap in time on
 * one GPU (different streams, different threads) race; order them.  Nothing has
 * to be cleared between calls: each call rewrites what it reads. */
#define SPO_SAMPLE_STATIC_MAX_N (1 << 20)
int spo_sample_prompts_static(const float *alpha, const float *beta, int64_t N, int32_t B,
                              double eps_explore, uint64_t seed, uint64_t iteration, int replace,
                              uint32_t max_attempts, int32_t *idx_out, int32_t *info,
                              spo_stream_t stream);

/* ---------------------------------------------------------------------------
 * Advantages (Method, "Advantage Estimation and Policy Optimization": the raw
 * advantage A = r - v_{-1} with the PRE-update tracker mean as baseline, and the
 * global normalisation (A - mu_B) / sigma_B over the whole batch).  One value per
 * response; the loss applies it to every token of that response.
 *
 * alpha, beta  [N] fp32 tracker state before this iteration's update.  beta may
 *              be NULL: alpha then holds the estimate v_hat itself (the state of
 *              spo_tracker_update_ema).
 * idx, reward  [B]: prompt id and reward of each response.
 * ddof         0 = population standard deviation (the default reading), 1 = sample.
 * eps_norm     added to sigma in the denominator (0 for the paper's form).
 *              sigma + eps_norm == 0 gives adv_norm = 0, not NaN.
 * use_baseline 0 selects the paper's "no baseline" variant (v = 0).
 * adv_raw      optional [B]; adv_norm [B]; stats optional [2] = (mu, sigma).
 * info         optional int32[1]: 0, or 1 if some idx[k] lies outside [0, N).  Such an
 *              id is never used as an index: its advantage is NaN, and so are the
 *              batch statistics and every normalised value.
 * ws           optional, spo_advantages_workspace_bytes(B) bytes, 256-byte aligned.
 *              Without it one workgroup does all the work (three passes over the
 *              batch: right for the batches of the paper, slow beyond ~10^5
 *              responses); with it, batches of 16384 responses or more are spread
 *              over the chip (partial sums of 4096 responses each, added in a fixed
 *              order).  Both forms are bitwise reproducible; between them the
 *              statistics agree to fp64 rounding.
 * Statistics are accumulated in fp64 in a fixed order.
 * Limits: 1 <= B < 2^31.  Errors: ws too small -> SPO_EWORKSPACE.
 * ------------------------------------------------------------------------- */
size_t spo_advantages_workspace_bytes(int32_t B);
int spo_advantages(const float *alpha, const float *beta, int64_t N, const int32_t *idx,
                   const float *reward, int32_t B, int ddof, float eps_norm, int use_baseline,
                   float *adv_raw, float *adv_norm, float *stats, int32_t *info, void *ws,
                   size_t ws_bytes, spo_stream_t stream);

/* Diagnostics of the unnormalised advantages that the paper's analysis tracks
 * (Experiments, "Signal Efficiency and Information Loss" and "Signal Stability and
 * Advantage Variance"): diag[0], diag[1] = share of responses with |A| <= tau_tight
 * and |A| <= tau_loose (the paper uses 1e-4 and 0.02), diag[2] = population
 * variance of A, diag[3] = population variance of the rewards (the "no baseline"
 * reference).  adv_raw, reward [B] fp32; diag fp32[4]; tau_tight <= tau_loose. */
int spo_advantage_diagnostics(const float *adv_raw, const float *reward, int32_t B, float tau_tight,
                              float tau_loose, float *diag, spo_stream_t stream);

/* ---------------------------------------------------------------------------
 * Tracker update (Method, "A KL-Adaptive Value Tracker"): for every observed
 * response, rho = 2^(-D/D_half) kept inside [rho_min, rho_max],
 * alpha <- rho*alpha + r, beta <- rho*beta + (1 - r), in place.
 *
 * alpha, beta  [N] fp32, updated in place at the B listed entries.
 * idx, reward, kl [B]; kl is D(x) >= 0, the divergence between the current
 *              policy and the one that last acted on the prompt (negative
 *              values are read as 0).
 * ids_unique   1: the caller guarantees that idx holds no repeated id (one
 *              response per prompt).  0: repeated ids are applied one after the
 *              other in batch order, as if the responses arrived in sequence
 *              (needs ws); the cost is one pass over the batch per repeat of the
 *              most repeated id, in a single workgroup.
 * n_obs        optional uint32[N] visit counters, incremented per observation.
 * v_prev_out   optional [B]: tracker mean right before observation k.
 * info         optional int32[1], bits: 1 = some idx[k] lies outside [0, N) (that
 *              observation is skipped, nothing is written for it, its v_prev_out is
 *              NaN); 2 = ids_unique = 1 but an id repeats (only looked for when ws is
 *              given; the entry of such an id then holds one of its updates).
 * ws           spo_tracker_update_workspace_bytes(N) bytes, 256-byte aligned: a table
 *              of one int32 per prompt.  Required for ids_unique = 0; with
 *              ids_unique = 1 it is optional and only serves the repeat check.
 * Arithmetic: rho and the products are formed in fp64 and rounded once to fp32,
 * so rho_min = rho_max = 1 reproduces Beta posterior counts exactly.
 * Limits: 1 <= B < 2^31.
 * Errors: d_half <= 0, rho_min > rho_max, rho outside [0, 1] -> SPO_EINVAL;
 * ids_unique = 0 without ws, or ws too small -> SPO_EWORKSPACE.
 * ------------------------------------------------------------------------- */
size_t spo_tracker_update_workspace_bytes(int64_t N);
int spo_tracker_update(float *alpha, float *beta, int64_t N, const int32_t *idx,
                       const float *reward, const float *kl, int32_t B, float d_half,
                       float rho_min, float rho_max, int ids_unique, uint32_t *n_obs,
                       float *v_prev_out, int32_t *info, void *ws, size_t ws_bytes,
                       spo_stream_t stream);

/* ---------------------------------------------------------------------------
 * The tracker in its moving-average form, for rewards that are not binary
 * (Method, "A KL-Adaptive Value Tracker": the EMA form of the update and the
 * remark on general rewards).  State per prompt: the estimate v_hat and the
 * effective sample size n_eff (alpha + beta of the Beta form):
 *     eta = 1 / (rho * n_eff + 1),  v_hat <- v_hat + eta * (r - v_hat),
 *     n_eff <- rho * n_eff + 1,
 * with rho as in spo_tracker_update.  With v_hat = alpha / (alpha + beta) and
 * n_eff = alpha + beta the two forms describe the same estimate; this one puts
 * no bound on r.  All other arguments, the fp64-then-one-rounding arithmetic,
 * limits and errors are those of spo_tracker_update.  spo_advantages accepts the
 * state of this form as alpha = v_hat, beta = NULL.
 * ------------------------------------------------------------------------- */
int spo_tracker_update_ema(float *v_hat, float *n_eff, int64_t N, const int32_t *idx,
                           const float *reward, const float *kl, int32_t B, float d_half,
                           float rho_min, float rho_max, int ids_unique, uint32_t *n_obs,
                           float *v_prev_out, int32_t *info, void *ws, size_t ws_bytes,
                           spo_stream_t stream);

/* Tracker initialisation (Method, "Initialization"; Appendix "SPO
 * Initialization"): N0 = 1/(1 - rho_min), alpha0 = N0*v0, beta0 = N0*(1 - v0),
 * with v0 [N] the mean of the offline outcomes of each prompt.  rho_min < 1. */
int spo_tracker_init(const float *v0, int64_t N, float rho_min, float *alpha, float *beta,
                     spo_stream_t stream);

/* ---------------------------------------------------------------------------
 * Token-level clipped policy-gradient loss over the full vocabulary (Method, the
 * PPO-Clip objective; clip bounds eps_low / eps_high as in Appendix "Training and
 * Evaluation Details").
 *
 * For token t of response b (cu_seqlens[b]-cu_seqlens[0] <= t <
 * cu_seqlens[b+1]-cu_seqlens[0]):
 *   z_t     = W^T h_t                         (V logits; or row t of `logits`)
 *   lse_t   = log sum_v exp z_t[v];  logp_t = z_t[target_t] - lse_t
 *   ratio_t = exp(logp_t - old_logp_t)
 *   obj_t   = min(ratio_t * A_b, clip(ratio_t, 1-eps_low, 1+eps_high) * A_b)
 *   loss    = - sum_t mask_t obj_t / M,  M = sum_t mask_t   (0 if M = 0)
 * The exported loss is MINUS the objective the paper maximises.  Its gradient
 * w.r.t. the logits is g_t * (onehot(target_t) - softmax(z_t)) with
 * g_t = -(mask_t/M) * A_b * ratio_t * [unclipped branch is the minimum] * grad_loss
 * (ties count as unclipped); old_logp carries no gradient.
 *
 * Fused form (logits == NULL): the [T x V] logits are never written to memory.
 * Logits-in form (logits != NULL; hidden and W ignored): streams existing logits.
 * ------------------------------------------------------------------------- */
typedef struct {
    size_t struct_size;      /* sizeof(spo_pg_desc), checked                         */
    int dtype;               /* SPO_BF16 or SPO_FP32: element type of hidden, W, logits */
    int w_layout;            /* SPO_W_VH or SPO_W_HV                                  */
    int64_t T, H, V;         /* tokens (packed), hidden size, vocabulary size        */
    int32_t B;               /* responses                                            */
    const void *hidden;      /* [T, H] row-major                                     */
    const void *W;           /* H*V elements in w_layout                             */
    const void *logits;      /* [T, V] row-major, or NULL                            */
    const int32_t *target;   /* [T] sampled token ids in [0, V); an id outside that
                                range is not an error code: the token's logp is NaN
                                (and with it the loss, if the token is unmasked) and
                                its gradient row carries no one-hot term              */
    const float *old_logp;   /* [T] log-probs under the behaviour policy             */
    const uint8_t *mask;     /* [T] 0/1 loss mask, or NULL for all ones              */
    const float *adv_norm;   /* [B] normalised advantage per response                */
    const int32_t *cu_seqlens; /* [B+1] non-decreasing token offsets; only differences
                                  to cu_seqlens[0] are used; last - first = T        */
    float eps_low, eps_high; /* clip range [1-eps_low, 1+eps_high]                   */
} spo_pg_desc;

/* Forward.
 * loss  [1] fp32.   logp, lse [T] fp32 (inputs of the backward).
 * stats optional fp32[4]: M, share of unmasked tokens whose clipped branch is the
 *       minimum, mean ratio over unmasked tokens, sum_t mask_t*obj_t.
 * Reductions run in a fixed order: results are bitwise reproducible.
 * Requirements (fused form): H a multiple of 64, H <= 65536, pointers 16-byte
 * aligned.  T = 0 is allowed (loss = 0, the per-token
 * pointers may then be NULL). */
size_t spo_pg_loss_fwd_workspace_bytes(const spo_pg_desc *d);
int spo_pg_loss_fwd(const spo_pg_desc *d, float *loss, float *logp, float *lse, float *stats,
                    void *ws, size_t ws_bytes, spo_stream_t stream);

/* Backward.
 * logp, lse     [T] from the forward of the same desc.
 * grad_loss     d(total)/d(loss), a host scalar.
 * d_hidden      [T, H] in d_hidden_dtype (fused form; may be NULL to skip).
 * d_W           H*V elements in W's layout, in d_W_dtype (fused form; may be NULL).
 * accumulate_dW 1: add to the existing contents of d_W (mini-batch accumulation;
 *               needs d_W_dtype = SPO_FP32); 0: overwrite.
 * d_logits      [T, V] in desc dtype (logits-in form only).
 * chunk_tokens  tokens whose logit gradients are held in the workspace at once,
 *               rounded up to a multiple of 256.  The backward recomputes the logits
 *               tile by tile; a chunk's bf16 logit gradients (2 * V bytes per token,
 *               V rounded up to 256) live in the workspace between the three
 *               contractions: at most chunk_tokens x V of them at a time, which is the
 *               whole [T x V] array whenever T <= chunk_tokens.  0 lets the library
 *               choose: as many tokens as keep that buffer within 8 GiB (24576 at
 *               V = 151936, H = 4096).  Fewer, larger chunks cost workspace and save
 *               passes over d_W, which is read and rewritten once per chunk.
 * Tokens whose gradient factor is zero (masked, on the clipped branch, or in a
 * response with zero advantage) are left out of the recompute and of both
 * contractions: the cost of the backward follows the number of remaining tokens,
 * and their rows of d_hidden are exact zeros. */
size_t spo_pg_loss_bwd_workspace_bytes(const spo_pg_desc *d, int64_t chunk_tokens);
int spo_pg_loss_bwd(const spo_pg_desc *d, const float *logp, const float *lse, float grad_loss,
                    void *d_hidden, int d_hidden_dtype, void *d_W, int d_W_dtype,
                    int accumulate_dW, void *d_logits, int64_t chunk_tokens, void *ws,
                    size_t ws_bytes, spo_stream_t stream);

/* Forward and backward in one call (fused form only), for callers that know
 * grad_loss = d(total)/d(loss) before the forward: a loss that enters the total with
 * a fixed weight, which is how the policy-gradient objective is used (Method, the
 * PPO-Clip objective is the whole training loss).  Same results as spo_pg_loss_fwd
 * followed by spo_pg_loss_bwd, up to the rounding of what is stored (below), at
 * three contractions of size T x V x H instead of four: the logits are not formed
 * a second time.
 * The batch is walked in pieces of chunk_tokens tokens (rounded up to a multiple of
 * 256).  The forward sweep of a piece also stores, at 2 * V bytes per token in the
 * workspace, what the backward needs of its logits; the piece's log-probs then give
 * the gradient factors and the two contractions follow.  What is stored depends on
 * the desc:
 *  - mask == NULL: bf16 of q[t][v] = exp(z[t][v] - r_t) with r_t = z[t][target_t] -
 *    old_logp_t, known before the sweep; q = softmax / ratio_t lies near the
 *    probabilities, and the logit gradient is c_t * (q - onehot / ratio_t) with
 *    c_t = -g_t * ratio_t.  After the sweep one entry per token is rewritten and the
 *    contractions read q as it is: d_hidden_t = c_t * (q_t W), d_W = q^T (c X).
 *    Every token of the piece is multiplied, also those whose factor is zero (the
 *    clipped ones); exponents are capped so that nothing stored is infinite.  c_t
 *    grows with the square of the ratio: an unclipped token whose ratio exceeds
 *    about e^40 overflows it (spo_pg_loss_bwd, whose factor is linear in the ratio,
 *    reaches e^80).
 *  - mask != NULL: fp16 of the logit minus an offset per (token, 128 vocabulary
 *    entries), the largest logit the sweep has met for that token up to there.  An
 *    entry within d of its row's largest logit is stored within d of zero, where
 *    fp16 resolves d * 2^-11: the error this adds to a probability p is at most
 *    p * ln(1/p) * 2^-11.  One pass then turns the stored logits of the tokens with a
 *    non-zero factor into bf16 logit gradients (as much workspace again), and the
 *    contractions run over those tokens only, as in spo_pg_loss_bwd.
 * chunk_tokens = 0 lets the library choose: the most tokens, in multiples of 4096,
 * whose stored values stay within 8 GiB (24576 at V = 151936).  Shorter pieces cost
 * more passes over d_W.
 * Arguments as in spo_pg_loss_fwd and spo_pg_loss_bwd; d_hidden and d_W may each be
 * NULL.  The workspace size depends on whether the desc has a mask.  Errors as
 * there; a desc with logits != NULL -> SPO_EUNSUPPORTED. */
size_t spo_pg_loss_fwd_bwd_workspace_bytes(const spo_pg_desc *d, int64_t chunk_tokens);
int spo_pg_loss_fwd_bwd(const spo_pg_desc *d, float grad_loss, float *loss, float *logp,
                        float *lse, float *stats, void *d_hidden, int d_hidden_dtype,
                        void *d_W, int d_W_dtype, int accumulate_dW, int64_t chunk_tokens,
                        void *ws, size_t ws_bytes, spo_stream_t stream);

/* ---------------------------------------------------------------------------
 * Per-kernel timing (measurement aid, not part of the method; with the static
 * buffer of spo_sample_prompts_static the only state the library keeps).  While enabled, the loss entry points bracket each launch
 * of their heavy kernels with a pair of HIP events on the launch stream.
 * spo_kernel_timing_read waits for the recorded events, writes the summed
 * milliseconds and the number of launches per kernel class, and forgets them.
 * Classes: 0 fused forward vocabulary sweep, 1 backward logits recompute,
 * 2 backward dHidden contraction, 3 backward dW contraction, 4 logits-in forward
 * pass, 5 logits-in backward pass, 6 stored logits -> logit gradients (one-call
 * forward + backward).  ms and launches are HOST arrays of 7.
 * ------------------------------------------------------------------------- */
#define SPO_TIMING_CLASSES 7
int spo_kernel_timing_enable(int enable);
int spo_kernel_timing_read(float *ms, int32_t *launches);

#ifdef __cplusplus
}
#endif
#endif /* SPO_H_ */
