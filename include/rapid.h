/*
 * rapid.h -- C ABI of the MI355X (gfx950) library for the hot path of RAPID's off-policy update
 * step (arXiv 2510.03515): the fused importance-weighted group-advantage policy-gradient loss.
 *
 * Conventions shared by every call
 * --------------------------------
 *  - Every data pointer is a DEVICE pointer owned by the caller.  The library never allocates,
 *    frees or keeps device memory: scratch comes from the caller's `workspace`, whose size is
 *    given by rapid_workspace_bytes().  `opts` of rapid_iw_pg_loss_fwd_bwd is a HOST pointer.
 *  - All work is enqueued on the caller's HIP stream (`stream` is a hipStream_t passed as
 *    void*; NULL = the default stream).  Calls are asynchronous and never synchronise the
 *    device; outputs are valid once the stream has reached the end of the call's work.
 *  - Return value: RAPID_OK or a negative RAPID_ERR_*.  Every code except RAPID_ERR_HIP is found on
 *    the host before any launch (nothing has been enqueued then).  RAPID_ERR_HIP after the
 *    validation means that the HIP runtime reported an error while or after the call's kernels were
 *    enqueued (hipGetLastError at the end of the call, which also returns an error another library
 *    left behind on this thread): part of the work may be on the stream and the outputs are not
 *    usable.  rapid_last_error() gives a thread-local message.
 *  - Errors only the device can see (token id outside [0,V) at an unmasked position, group id
 *    outside [0,K), non-finite reward or behaviour log-prob; with opts->logits_cache also the two
 *    conditions documented at RAPID_STATUS_LOGIT_RANGE and RAPID_STATUS_TOKEN_BOUND) OR a bit into
 *    the caller's `dev_status` word (may be NULL); the offending element is treated as token 0 /
 *    skipped / 0 and nothing faults.  The library only ORs bits in: the caller clears the word.
 *  - Layouts: hidden [N,T,d] row-major (padded), dtype bf16 or fp32; hidden row (n,t) is the
 *    state that predicts tokens[n,t].  W is logically [d,V]; w_layout says how it is stored:
 *    RAPID_W_DV = [d,V] row-major, RAPID_W_VD = [V,d] row-major.  tokens [N,T] int32;
 *    mask [N,T] uint8 (any 0/1 pattern); per-token outputs [N,T] fp32 (0 at masked positions);
 *    rewards [N] fp32; group_ids [N] int32 in [0,K), groups need not be contiguous or equal.
 *  - Only gfx950 devices are accepted (RAPID_ERR_ARCH otherwise).
 */
#ifndef RAPID_H
#define RAPID_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* host-side error codes */
#define RAPID_OK 0
#define RAPID_ERR_NULL (-1)      /* a required pointer is NULL */
#define RAPID_ERR_SHAPE (-2)     /* a size is <= 0, too large (limits: N * T <= 2e9 positions, d <= 65536,
                                    V <= 4e6), or unsupported (bf16 needs d % 8 == 0) */
#define RAPID_ERR_DTYPE (-3)     /* unknown dtype / layout / mode enum */
#define RAPID_ERR_WORKSPACE (-4) /* workspace NULL, misaligned (256 B) or below the minimum */
#define RAPID_ERR_ARCH (-5)      /* current device is not gfx950 */
#define RAPID_ERR_HIP (-6)       /* a HIP runtime call failed */

/* bits OR-ed into *dev_status by kernels */
#define RAPID_STATUS_BAD_TOKEN 1
#define RAPID_STATUS_BAD_GROUP 2
#define RAPID_STATUS_NONFINITE_REWARD 4
#define RAPID_STATUS_NONFINITE_LOGP 8
#define RAPID_STATUS_LOGIT_RANGE 16 /* logits_cache = 1 only: in some row a logit, or the log-sum-exp, is more than 79
                                       away from the reference the cached values are relative to (the sampled
                                       token's logit minus its behaviour log-prob; the sampled token's logit alone
                                       without logp_behav).  Loss and log-probs are exact, that row's share of
                                       dhidden and dW is truncated */
#define RAPID_STATUS_TOKEN_BOUND 32 /* more valid tokens than opts->max_tokens promised (logits_cache = 1): the tokens
                                      past the bound were left out; the call's outputs are not usable */
#define RAPID_STATUS_GROUP_LAYOUT 64 /* logits_cache = 1 with a workspace that cannot cache the whole batch: the batch is
                                      then worked through in chunks of whole groups, which needs the members of every
                                      group next to each other in the batch and every group's tokens to fit into the
                                      cache rows the workspace affords.  Set when one of the two does not hold; the
                                      call's outputs are not usable.  Repeat the call with logits_cache = 0, or with
                                      the workspace of rapid_workspace_bytes_max_tokens (one chunk, any layout) */

/* enums */
#define RAPID_DTYPE_F32 0
#define RAPID_DTYPE_BF16 1
#define RAPID_W_DV 0
#define RAPID_W_VD 1
#define RAPID_OP_LOGPROB_FWD 0
#define RAPID_OP_GROUP_ADVANTAGE 1
#define RAPID_OP_IW_PG_FWD_BWD 2
#define RAPID_OP_IW_PG_FWD_BWD_CACHED 3 /* workspace query only: rapid_iw_pg_loss_fwd_bwd with logits_cache = 1 */

/* Options of rapid_iw_pg_loss_fwd_bwd (host struct).  rapid_iw_pg_default_opts() fills the
 * paper's defaults: eta = 2.0 (Appendix A, RL hyper-parameter table), everything else as
 * Sec. 3.4 states the estimator. */
typedef struct rapid_iw_pg_opts {
    float eta;             /* clip of the generation-level ratio in the baseline, Eq. (5); +inf => Eq. (4) */
    int coef_mode;         /* 0: outer weight is the unclipped ratio (Eq. (3) as printed);
                              1: outer weight is the clipped weight, held constant */
    int baseline_mode;     /* 0: Eq. (5), sum over the whole group; 1: leave-one-out sum of Sec. 3.4
                              divided by N_k as printed; 2: leave-one-out divided by N_k - 1 */
    float loss_scale;      /* multiplies loss and gradients (fold in N/N_global, accumulation steps) */
    float temperature;     /* logits are divided by it; 1.0 */
    int w_layout;          /* RAPID_W_DV | RAPID_W_VD, for W and for dW_out */
    int dw_dtype;          /* RAPID_DTYPE_F32 (default) | RAPID_DTYPE_BF16 */
    int accumulate_dw;     /* 0: dW_out is overwritten; 1: dW_out += gradient (fp32 dW only) */
    int normalized_grads;  /* 1: loss, dhidden and dW are returned multiplied by exp(-lambda), with
                              lambda = log max_n |g_n| reported in diag->grad_log_scale, so that
                              ratios that underflow fp32 still give usable gradients */
    int logits_cache;      /* 0 (default): the backward regenerates the logits tile by tile from hidden and W;
                              nothing of size rows x V outlives a row chunk.  1 (bf16 inputs only): the
                              forward also stores, in the workspace, exp(z_v - r) (bf16) for every vocabulary
                              entry, r = the sampled token's logit minus its behaviour log-prob (an estimate
                              of the row's log-sum-exp that is known before the sweep, so the stored value
                              is close to the probability p_v), and the backward contracts those directly
                              (dz = -g exp(r - lse) (stored - onehot exp(lse - r))): one contraction fewer
                              and no pass over rows x V in between.  The cache holds as many token rows as
                              the workspace affords (2 bytes x V per row).  If that is every token of the batch
                              (rapid_workspace_bytes_max_tokens), the call is one sweep.  If not
                              (rapid_workspace_bytes(RAPID_OP_IW_PG_FWD_BWD_CACHED, ...): 90112 rows), the batch is
                              worked through in chunks of whole groups, in order, each chunk as many groups as the
                              cache holds: forward with store, the chunk's ratios, advantages (Eq. (5) needs only
                              the group) and coefficients (Eq. (3)'s 1/N is known beforehand), dHidden and dW of
                              the chunk, then the next; with normalized_grads the sums are rescaled on the way
                              whenever a chunk raises the maximum.  This needs every group's members adjacent in
                              the batch (see RAPID_STATUS_GROUP_LAYOUT).  Same single bf16 rounding per element
                              of the rows x V intermediate as mode 0; see RAPID_STATUS_LOGIT_RANGE for its one
                              limit */
    int ratio_level;       /* 0 (default): the outer weight of Eq. (3) is the generation-level ratio rho_n, as
                              the paper defines it.  1: a variant the paper does not define (its token-level
                              ratios are a diagnostic, Sec. 4.3): every token carries its own ratio,
                              loss = -(loss_scale/N) sum_n A_n sum_t c_{n,t}, c_{n,t} = rho_{n,t} (coef_mode 0)
                              or min(rho_{n,t}, eta) held constant (coef_mode 1); the advantages stay those of
                              Eq. (5) with generation-level clipped weights.  grad_log_scale is then
                              log max |dLoss/dlogp_{n,t}| over tokens.  Ignored with coef_override */
    int64_t max_tokens;    /* 0, or the caller's upper bound on the number of valid tokens (sum of mask), which it
                              knows from its sampler: with logits_cache = 1 the cache holds the whole batch
                              once it has that many rows instead of N*T (rapid_workspace_bytes_max_tokens), and
                              a chunked call is laid out for that many tokens.  Checked on the device:
                              RAPID_STATUS_TOKEN_BOUND */
    const float* coef_override; /* DEVICE [N] or NULL: use these per-generation coefficients g_n
                              = dLoss/dlogp_{n,t} instead of the estimator's (loss = sum g_n) */
    const void* rms_weight; /* NULL, or DEVICE [d] (bf16; bf16 inputs only): `hidden` is then the input x of the
                              model's final RMSNorm and the path runs on h = x * rms_weight / sqrt(mean(x^2) +
                              rms_eps), formed (and rounded to bf16) while the rows are packed; dhidden_out
                              is dLoss/dx.  Not part of the paper's method, whose path starts at h */
    float* drms_weight_out; /* NULL, or DEVICE [d] fp32: dLoss/d rms_weight (only read with rms_weight) */
    float rms_eps;          /* >= 0; 1e-6 */
} rapid_iw_pg_opts;

/* Diagnostics written by rapid_iw_pg_loss_fwd_bwd (device struct).
 * mean_log_w / mean_abs_log_w: mean over generations of log(clipped weight) and of its absolute
 * value (staleness of Sec. 4.3); n_clipped: generations with ratio > eta (clip proportion,
 * Sec. 4.3 "Importance-weight clipping"). */
typedef struct rapid_iw_pg_diag {
    int64_t n_tokens;
    int32_t n_clipped;
    int32_t n_sequences;
    float mean_log_w;
    float mean_abs_log_w;
    float max_abs_s;
    float grad_log_scale;
} rapid_iw_pg_diag;

/* Library/ABI version (monotone integer) and the last error text of the calling thread. */
int rapid_version(void);
const char* rapid_last_error(void);

/* Fills *opts with the defaults described above.  Host pointer. */
void rapid_iw_pg_default_opts(rapid_iw_pg_opts* opts);

/* Workspace sizes in bytes for `op` at the given problem size.  rapid_workspace_bytes is the
 * recommended size (backward row-chunks large enough to fill the chip); rapid_workspace_min_bytes
 * the smallest the call accepts (smaller chunks, same results).  RAPID_OP_GROUP_ADVANTAGE needs
 * none (returns 0).  RAPID_OP_IW_PG_FWD_BWD_CACHED are the sizes for rapid_iw_pg_loss_fwd_bwd with
 * opts->logits_cache = 1 (bf16 only): recommended = a cache of 90112 token rows (or of all N * T positions
 * if those are fewer), minimum = a cache of 256 rows; the call uses as many cache rows as the workspace
 * it is given affords.  rapid_workspace_bytes_max_tokens (cached op only; the others ignore the bound) is
 * the size with which the cache holds every token of a batch of at most max_tokens valid tokens (0 = N * T)
 * at once: the largest useful size, and the one that puts no condition on where the members of a group
 * lie in the batch.  Returns 0 for invalid arguments. */
size_t rapid_workspace_bytes(int op, int64_t N, int64_t T, int64_t d, int64_t V, int64_t K, int dtype);
size_t rapid_workspace_min_bytes(int op, int64_t N, int64_t T, int64_t d, int64_t V, int64_t K, int dtype);
size_t rapid_workspace_bytes_max_tokens(int op, int64_t N, int64_t T, int64_t d, int64_t V, int64_t K, int dtype,
                                        int64_t max_tokens);

/* Host arithmetic only: the number of token rows the cache of a logits_cache = 1 call would hold if it were given
 * `workspace_bytes` of workspace and opts->max_tokens = max_tokens (0 = N * T).  Every token of the batch (one chunk) if
 * that fits, otherwise the largest window that does; a window's chunks are whole groups in batch order, each as many
 * groups as fit.  0 if the workspace is below the minimum or an argument is invalid. */
int64_t rapid_logits_cache_rows(int64_t N, int64_t T, int64_t d, int64_t V, int64_t K, int64_t max_tokens,
                                size_t workspace_bytes);

/*
 * Behaviour / current-policy log-probabilities of the sampled tokens (Sec. 3.1: pi(y_t | .) is
 * the softmax of the LM head; Alg. 1, the step that snapshots the current policy as the behaviour
 * policy mu: these are the log mu(y_t) the ratio of Eq. (3) divides by).
 *   logp_out[n,t] = z[y] - logsumexp(z),  z = hidden[n,t,:] . W / temperature   (0 where mask = 0)
 *   lse_out[n,t]  = logsumexp(z) (optional, may be NULL)
 * The [N*T, V] logits are never written to memory.
 */
int rapid_logprob_fwd(const void* hidden, const void* W, const int32_t* tokens, const uint8_t* mask,
                      int64_t N, int64_t T, int64_t d, int64_t V, int dtype, int w_layout,
                      float temperature, float* logp_out, float* lse_out, int32_t* dev_status,
                      void* workspace, size_t workspace_bytes, void* stream);

/*
 * rapid_logprob_fwd for callers that cannot allocate device memory or pass a workspace: code under
 * HIP graph capture, tight serving loops that score behaviour log-probs between decoding steps,
 * harnesses that forbid hipMalloc.  Same arguments without `workspace`, same results, bit for bit:
 * the scratch is a static device array inside the library (768 MiB, RAPID_STATIC_SCRATCH_BYTES in the
 * source; each GPU the entry point is used on holds its own copy from first use until the process
 * ends).  The call allocates and frees nothing, on the device or through any allocating library.
 *  - Shapes whose scratch (rapid_workspace_min_bytes(RAPID_OP_LOGPROB_FWD, ...)) exceeds the array
 *    are refused with RAPID_ERR_WORKSPACE before any launch; the message names both sizes.  The
 *    Qwen2.5-3B-shaped head (d = 2048, V = 151936, bf16) fits with up to 4096 positions per call.
 *  - The first call on a device looks the array's address up (hipGetSymbolAddress, once per device,
 *    kept): make that first call outside stream capture.
 *  - All calls on one GPU share that GPU's array, which keeps the previous call's contents (every
 *    word a call reads it has written itself first): calls that overlap in time on one GPU, on
 *    whatever streams, race.  Serialise them.
 */
int rapid_logprob_fwd_static(const void* hidden, const void* W, const int32_t* tokens, const uint8_t* mask,
                             int64_t N, int64_t T, int64_t d, int64_t V, int dtype, int w_layout,
                             float temperature, float* logp_out, float* lse_out, int32_t* dev_status,
                             void* stream);

/* rapid_logprob_fwd on h = hidden * rms_weight / sqrt(mean(hidden^2) + rms_eps) (see
 * rapid_iw_pg_opts.rms_weight; rms_weight: DEVICE [d] bf16, dtype must be RAPID_DTYPE_BF16): the
 * log-probs a behaviour policy with that final norm assigns.  Same workspace size, same errors,
 * plus RAPID_ERR_NULL / RAPID_ERR_DTYPE / RAPID_ERR_SHAPE for rms_weight, dtype and rms_eps. */
int rapid_logprob_fwd_rmsnorm(const void* hidden, const void* W, const int32_t* tokens, const uint8_t* mask,
                              int64_t N, int64_t T, int64_t d, int64_t V, int dtype, int w_layout,
                              float temperature, const void* rms_weight, float rms_eps, float* logp_out,
                              float* lse_out, int32_t* dev_status, void* workspace, size_t workspace_bytes,
                              void* stream);

/*
 * Group advantage (Sec. 3.3 Eq. (2); Sec. 3.4 Eq. (4), (5)).
 *   w_n = 1 if seq_logratio == NULL (on-policy, Eq. (2)), else min(exp(seq_logratio[n]), eta)
 *   baseline_mode 0:  adv[n] = R_n - (1/N_k) sum_{n' in group(n)} w_n' R_n'
 *   baseline_mode 1/2: the sum leaves n out; divided by N_k (as printed) / by N_k - 1
 * group_mean_out / group_std_out [K]: plain mean and population std of R per group (diagnostic;
 * the paper never divides by the std); group_size_out [K] int32.  Optional outputs may be NULL.
 * A group with no member gets size 0, mean 0, std 0.
 */
int rapid_group_advantage(const float* rewards, const int32_t* group_ids, const float* seq_logratio,
                          int64_t N, int64_t K, float eta, int baseline_mode, float* adv_out,
                          float* weight_out, float* group_mean_out, float* group_std_out,
                          int32_t* group_size_out, int32_t* dev_status, void* stream);

/*
 * Token- and generation-level log ratios (Sec. 3.4, the ratio of Eq. (3); Sec. 4.3: token ratios are accumulated
 * over the generation, the clip acts on the result), the reduction step of the fused call as a call of its own:
 *   tok_logratio_out[n,t] = mask (logp_cur - logp_behav)   ([N,T] fp32, may be NULL)
 *   seq_logratio_out[n]   = sum_t tok_logratio[n,t]        ([N] fp32, fp64 accumulation in a fixed order)
 * A non-finite behaviour log-prob at a valid position counts as a log ratio of 0 and sets
 * RAPID_STATUS_NONFINITE_LOGP.  No workspace.
 */
int rapid_seq_logratio(const float* logp_cur, const float* logp_behav, const uint8_t* mask, int64_t N, int64_t T,
                       float* tok_logratio_out, float* seq_logratio_out, int32_t* dev_status, void* stream);

/*
 * One mini-batch of Alg. 1's IW-GRPG: advantages by Eq. (5), loss and gradients by Eq. (3).
 *   logp      = as rapid_logprob_fwd on the current W
 *   s_n       = sum_t mask (logp - logp_behav)            (generation-level log ratio, Sec. 4.3)
 *   A_n       = rapid_group_advantage(rewards, group_ids, s, eta, baseline_mode)
 *   loss      = -(loss_scale/N) sum_n c_n A_n,  c_n = exp(s_n)  (coef_mode 0)
 *   g_n       = -(loss_scale/N) c_n A_n  = d loss / d logp[n,t] for every valid t
 *   dhidden[n,t,:] = g_n (W[:,y] - W p) / temperature  (0 where mask = 0), dtype of hidden
 *   dW        = sum_{valid n,t} outer(hidden[n,t,:], g_n (e_y - p)) / temperature, layout w_layout
 * logp_behav == NULL means on-policy: every ratio is exactly 1 and the call is the group relative
 * policy gradient of Sec. 3.3 (Eq. (1) with the advantages of Eq. (2)).
 * Optional outputs (NULL to skip): logp_cur_out, tok_logratio_out [N,T]; seq_logratio_out,
 * adv_out [N]; diag_out.  loss_out [1], dhidden_out [N,T,d] and dW_out are required.
 * Generations without gradient (bf16 inputs): if every reward of a group is exactly 0, Eq. (5) gives its members
 * A_n = 0 whatever their ratios are (the weighted baseline of zeros is 0; likewise both leave-one-out forms), so their
 * rows of dhidden are zero and they add nothing to dW.  The call decides this from the rewards (or from zeros in
 * coef_override) before the forward, orders such generations behind the others and ends the backward's contractions
 * in front of them; their log-probs, ratios and diagnostics are computed as for any other generation.
 */
int rapid_iw_pg_loss_fwd_bwd(const void* hidden, const void* W, const int32_t* tokens,
                             const uint8_t* mask, const float* logp_behav, const float* rewards,
                             const int32_t* group_ids, int64_t N, int64_t T, int64_t d, int64_t V,
                             int64_t K, int dtype, const rapid_iw_pg_opts* opts, float* loss_out,
                             void* dhidden_out, void* dW_out, float* logp_cur_out,
                             float* tok_logratio_out, float* seq_logratio_out, float* adv_out,
                             rapid_iw_pg_diag* diag_out, int32_t* dev_status, void* workspace,
                             size_t workspace_bytes, void* stream);

/*
 * Loss steps of the paper's RL baselines on the same kernels (Sec. 4.1, "Baselines": GRPO and DAPO; Appendix A:
 * KL coefficient 0.04 for GRPO only), for a like-for-like comparison of one update step.  The paper does not
 * print their objectives; they follow the papers it cites for them:
 *   A_n     = (R_n - mean_k) / (std_k + adv_eps)   over the group k of n (std with divisor N_k - std_ddof; a group
 *             of equal rewards has A = 0)
 *   r_{n,t} = exp(logp_cur - logp_old)             token-level ratio (logp_old == NULL: all ratios 1)
 *   surr    = min(r A_n, clip(r, 1 - eps_low, 1 + eps_high) A_n)
 *   kl      = exp(logp_ref - logp_cur) - (logp_ref - logp_cur) - 1     (only if kl_beta != 0; logp_ref required then)
 *   loss    = - loss_scale sum_{valid n,t} omega_{n,t} (surr - kl_beta kl)
 *   omega   = 1 / (N L_n)  (norm_mode 0: mean over a generation's tokens, then over the N generations: GRPO)
 *           = 1 / M        (norm_mode 1: mean over the M valid tokens of the call: DAPO)
 * and its gradients dhidden and dW through the LM head, as in rapid_iw_pg_loss_fwd_bwd (same layouts, same
 * workspace sizes: RAPID_OP_IW_PG_FWD_BWD, or RAPID_OP_IW_PG_FWD_BWD_CACHED with logits_cache = 1, same
 * conditions).  A token whose ratio has left the clip range in the direction its advantage pushes gets no
 * gradient from the surrogate.  rapid_clip_pg_default_opts: variant 0 = GRPO (eps 0.2 / 0.2, kl_beta 0.04, norm_mode 0),
 * 1 = DAPO (eps 0.2 / 0.28, kl_beta 0, norm_mode 1; its sample filtering and reward shaping are the caller's).
 * Optional outputs (NULL to skip): logp_cur_out [N,T], adv_out [N], diag_out (device).
 */
typedef struct rapid_clip_pg_opts {
    float eps_low, eps_high;
    float kl_beta;
    int norm_mode;
    float adv_eps;         /* 1e-4 */
    int std_ddof;          /* 0 (default): population std; 1: sample std (0 for a group of one) */
    float loss_scale;
    float temperature;
    int w_layout, dw_dtype, accumulate_dw, logits_cache;   /* as in rapid_iw_pg_opts */
    int64_t max_tokens;    /* as in rapid_iw_pg_opts */
} rapid_clip_pg_opts;

typedef struct rapid_clip_pg_diag {
    int64_t n_tokens;
    int64_t n_clipped;     /* tokens whose surrogate took the clipped branch */
    int32_t n_sequences;
    float mean_kl;         /* mean over valid tokens of the KL estimate (0 without the term) */
} rapid_clip_pg_diag;

void rapid_clip_pg_default_opts(rapid_clip_pg_opts* opts, int variant);

int rapid_clip_pg_loss_fwd_bwd(const void* hidden, const void* W, const int32_t* tokens, const uint8_t* mask,
                               const float* logp_old, const float* logp_ref, const float* rewards,
                               const int32_t* group_ids, int64_t N, int64_t T, int64_t d, int64_t V, int64_t K,
                               int dtype, const rapid_clip_pg_opts* opts, float* loss_out, void* dhidden_out,
                               void* dW_out, float* logp_cur_out, float* adv_out, rapid_clip_pg_diag* diag_out,
                               int32_t* dev_status, void* workspace, size_t workspace_bytes, void* stream);

/*
 * The parameter update of Alg. 1's inner loop (the step after the gradient of Eq. (3)), for
 * the LM head alone and as plain gradient descent on the returned loss:
 *   master[i] -= lr * grad[i]   (fp32, n elements, same layout as dW_out)
 * and, if w_out != NULL, w_out[i] = the updated weight in `dtype` (the W of the next call).
 */
int rapid_sgd_step(float* master, const float* grad, int64_t n, float lr, void* w_out, int dtype, void* stream);

/*
 * The same update with AdamW (decoupled weight decay), the optimiser family of the paper's training runs
 * (Appendix A gives the learning rate, 1e-6; the remaining constants are the caller's).  Step number `step` >= 1:
 *   m = beta1 m + (1 - beta1) g;  v = beta2 v + (1 - beta2) g^2
 *   master -= lr * ( (m / (1 - beta1^step)) / (sqrt(v / (1 - beta2^step)) + eps) + weight_decay * master )
 * master, exp_avg (m) and exp_avg_sq (v) are fp32 device arrays of n elements that the caller keeps between
 * steps (m and v start at zero); w_out as in rapid_sgd_step.
 */
int rapid_adamw_step(float* master, const float* grad, float* exp_avg, float* exp_avg_sq, int64_t n, float lr,
                     float beta1, float beta2, float eps, float weight_decay, int64_t step, void* w_out, int dtype,
                     void* stream);

/*
 * Integer bookkeeping of the padding mask (device outputs; seq_len_out and cu_seqlen_out are
 * required, RAPID_ERR_NULL otherwise; row_index_out may be NULL):
 *   seq_len_out [N] int32, cu_seqlen_out [N+1] int32 (exclusive prefix sum, last = M),
 *   row_index_out [N*T] int32: the first M entries are the flat positions n*T+t of the valid
 *   tokens in row-major order.  This is the first step of both calls above, exported so that it
 *   can be checked bit for bit.
 */
int rapid_compaction(const uint8_t* mask, int64_t N, int64_t T, int32_t* seq_len_out,
                     int32_t* cu_seqlen_out, int32_t* row_index_out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* RAPID_H */
