/*
 * pg_head.h -- C ABI of the MI355X policy-gradient head.
 *
 * The library computes, for one packed microbatch of a multi-turn RL step, the
 * per-token policy-gradient quantities over the vocabulary without ever writing
 * the [tokens x vocab] logits to device memory:
 *
 *   trloo_advantage   turn returns and leave-one-out advantages   (Sec. 4.2, Eq. 2 and 5)
 *   pg_logprob_fwd    LM-head log-prob / entropy / logsumexp of the sampled tokens
 *                     (pi_train(a_t|s_t) of Sec. 5.1; entropy is the monitor of Sec. 5.1)
 *   pg_loss_fwd_bwd   mismatch correction (Sec. 5.1), clipped surrogate whose gradient is
 *                     grad log pi * A (App. A), backward to dH and dW
 *
 * and the small stages around that path:
 *
 *   pg_sft_fwd_bwd    token-mean cross-entropy of the same head, forward and backward
 *                     (the cold-start SFT stage of Sec. 3.3)
 *   grpo_advantage    turn returns and group-mean advantages          (Sec. 4.2, Eq. 2 and 3)
 *   turn_reward       per-turn reward with speedup cap and profiling ratio (Eq. 1, Eq. 6-7)
 *   prs_retain        profiling-based rejection sampling               (Sec. 5.2, Eq. 8)
 *   pg_monitors       entropy, perplexities and gradient norms         (Sec. 5.1)
 *   pg_rmsnorm_fwd/bwd  the RMS normalisation in front of the head in the Qwen3 policies of Sec. 6.1
 *   pg_head_shard_fwd, pg_head_partials_merge, pg_head_partials_finish, pg_loss_shard_bwd
 *                     pg_logprob_fwd / pg_loss_fwd_bwd with the head's vocabulary rows split over
 *                     devices: one device's share of the work and the reduction operator of the exchange
 *
 * Conventions
 *   - Every pointer is a DEVICE pointer unless its name starts with h_ (pg_params is
 *     passed by host pointer).  The caller owns all buffers; the library allocates
 *     and frees nothing and keeps no state between calls except lazily initialised
 *     kernel attributes.
 *   - All work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the
 *     default stream).  No call synchronises with the host; scalar results are
 *     written to device memory.
 *   - Arguments are validated on the host before anything is enqueued: for PG_ERR_INVALID_ARG,
 *     PG_ERR_UNSUPPORTED_SHAPE and PG_ERR_WORKSPACE_TOO_SMALL nothing has been enqueued and
 *     nothing is written.  PG_ERR_HIP reports a launch that the runtime refused; the kernels
 *     enqueued before it still run and the outputs are then undefined.  Only an error that
 *     arises during the call is reported: an error state that an earlier HIP call of the caller
 *     left behind is neither returned nor cleared.  pg_last_error() gives a thread-local message.
 *   - The first call on a device sets kernel attributes and must not happen inside a stream
 *     capture: run one call eagerly, or pg_init(), before capturing.
 *   - A workspace belongs to one call at a time: it holds the call's intermediate results and the
 *     tile counters of its kernels.  Calls that may overlap (different streams or threads) need
 *     workspaces of their own; calls ordered on one stream may share one.
 *   - H is [T,d] row-major, W is [V,d] row-major (LM-head weight, no bias), y[t] is
 *     the token whose log-prob row t predicts (the caller has already shifted).
 *     dtype 0: H, W, dH are bf16 (fp32 accumulation; the logit gradient dS is rounded to bf16 before
 *     the two backward contractions).  dtype 1: H, W, dH are fp32; every contraction then runs on
 *     operands split into a bf16 value plus a bf16 remainder (H, W and dS alike), the product of two
 *     remainders dropped: about 16 mantissa bits per product, at three times the matrix work.
 *   - Shapes: d must be a multiple of 64, 1 <= d, 1 <= V <= 2^30, 0 <= T < 2^23, and 256 rows of
 *     any operand (256 x d, x 3 for fp32 inputs) must stay below 4 GiB, and ceil(T/256) x ceil(V/256),
 *     the number of 256 x 256 logits tiles, below 2^28; otherwise
 *     PG_ERR_UNSUPPORTED_SHAPE.  Operands as a whole may be of any size.
 *     H, W, dH, dW and workspace must be 16-byte aligned.
 *   - y[t] outside [0,V) on an active row is not detected: that row's log-prob is
 *     then -logsumexp and its gradient has no one-hot term.  No memory is addressed
 *     through y.
 */
#ifndef PG_HEAD_H
#define PG_HEAD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PG_OK 0
#define PG_ERR_INVALID_ARG (-1)
#define PG_ERR_UNSUPPORTED_SHAPE (-2)
#define PG_ERR_WORKSPACE_TOO_SMALL (-3)
#define PG_ERR_HIP (-4)

#define PG_DTYPE_BF16 0
#define PG_DTYPE_F32 1

#define PG_MISMATCH_NONE 0      /* c_t = 1 */
#define PG_MISMATCH_GEOMETRIC 1 /* Sec. 5.1: keep a sample iff exp(mean log-ratio) in [geo_lo, geo_hi] */
#define PG_MISMATCH_TRUNCATE 2  /* c_t = min(pi_train/pi_rollout, trunc_c) per token */

#define PG_CALL_LOGPROB_FWD 0
#define PG_CALL_LOSS_FWD_BWD 1
#define PG_CALL_LOSS_FWD_BWD_NORMED 2

/* indices into counters_out[8] */
#define PG_CNT_ACTIVE 0      /* loss tokens of kept samples */
#define PG_CNT_CLIP_HI 1     /* A >= 0 and ratio > 1 + eps_hi (no gradient) */
#define PG_CNT_CLIP_LO 2     /* A <  0 and ratio < 1 - eps_lo (no gradient) */
#define PG_CNT_SEG_GEO 3     /* samples outside the geometric window (mode 1) */
#define PG_CNT_SEG_VETO 4    /* samples with a token ratio below veto_ratio */
#define PG_CNT_TRUNCATED 5   /* tokens whose weight was capped (mode 2) */
#define PG_CNT_LOSS_TOKENS 6 /* rows with loss_mask = 1 in samples that were not dropped */
#define PG_CNT_SEG_DROPPED 7 /* samples with loss rows whose sample_keep flag is 0 (or whose table index is out of range) */

typedef struct pg_params {
  int32_t dtype;         /* PG_DTYPE_* of H, W and dH */
  float temperature;     /* tau > 0: logits are divided by tau before the softmax */
  float clip_eps_lo;     /* clip range of pi_theta/pi_old is [1-eps_lo, 1+eps_hi] */
  float clip_eps_hi;
  int32_t mismatch_mode; /* PG_MISMATCH_* */
  float geo_lo;          /* 0.999 in Sec. 5.1 */
  float geo_hi;          /* 1.001 in Sec. 5.1 */
  float veto_ratio;      /* 1e-4 in Sec. 5.1; 0 disables the token veto */
  float trunc_c;         /* cap of mode 2 */
  float norm_override;   /* <= 0: normalise by the number of active tokens (at least 1);
                            > 0: divide by this value (e.g. a global token count) */
  int32_t accumulate_dW; /* 0: dW is overwritten; 1: dW += */
  int32_t dW_dtype;      /* 0: fp32, 1: bf16 */
  int32_t n_samples;     /* entries in the adv and sample_keep tables of the loss calls; a segment whose
                            table index (seg_sample[s], or s) lies outside [0, n_samples) is treated as a
                            dropped sample and counted in PG_CNT_SEG_DROPPED.  0: the length is not given
                            and the indices are used as they are (an index outside the tables then reads
                            memory that is not the caller's: undefined) */
  void* w_transposed;    /* optional, loss calls only: DEVICE buffer of pg_w_transposed_bytes(d, V) bytes that
                            caches the transposed head weight the dH contraction reads (for fp32 heads its bf16
                            values; their remainders are rebuilt in the workspace on every call).  NULL: the
                            transpose is rebuilt in the workspace on every call */
  int32_t w_transposed_valid; /* 0: this call fills w_transposed from W; 1: it already holds the transpose of
                            this very W (filled by an earlier call, W unchanged since: e.g. the further
                            microbatches of one optimizer step) and the call skips the transposition */
} pg_params;

/* Message for the last error returned on this thread ("" if none). */
const char* pg_last_error(void);

/*
 * One-time set-up for the CURRENT device: raises the MFMA kernels' dynamic shared-memory limit and
 * resolves the device address of the library's static scratch array.  Every entry point does this
 * by itself on its first call on a device; call pg_init() beforehand (once per device, outside any
 * stream capture) if the first real call is to be recorded into a HIP graph.  Allocates nothing.
 */
int32_t pg_init(void);

/*
 * Bytes of device workspace the given call needs for these sizes (S is ignored for
 * PG_CALL_LOGPROB_FWD).  Returns 0 if the arguments are invalid or unsupported.
 * The workspace need not be initialised and holds nothing the caller may rely on.
 */
size_t pg_workspace_bytes(int64_t T, int64_t d, int64_t V, int32_t S, const pg_params* h_params,
                          int32_t which_call);

/* Bytes of the optional W^T cache (pg_params.w_transposed) for a [V, d] head; 0 if unsupported. */
size_t pg_w_transposed_bytes(int64_t d, int64_t V);

/*
 * Inspection hook (tests, tuning): the number of vocabulary rows per chunk of the backward pass of
 * pg_loss_fwd_bwd / pg_sft_fwd_bwd for these sizes (chunk c covers rows [c n, (c+1) n) of W and dW;
 * it follows from the scratch budget, PG_HEAD_DS_BUDGET_BYTES).  0 if the arguments are invalid.
 */
int64_t pg_backward_chunk_rows(int64_t T, int64_t d, int64_t V, int32_t S, const pg_params* h_params);

/*
 * Sec. 4.2, Eq. (2) and Eq. (5).
 *   rewards[(p*K+k)*Tmax+t]  per-turn reward R of rollout k of prompt p at turn t (0 where the
 *                            turn was never generated)
 *   valid  (same indexing)   1 iff the rollout belongs to the turn group G_t of its prompt
 *   returns_out (nullable)   G = sum_{t'>=t} gamma^(t'-t) R, for every entry
 *   adv_out                  A = G - mean of the other valid rollouts' G of the same prompt
 *                            and turn; 0 for invalid entries and for groups with N_t < 2
 *   group_n_out (nullable)   [P*Tmax] N_t
 * Accumulation and outputs are fp64.  P, K, Tmax >= 1.
 */
int32_t trloo_advantage(const float* rewards, const uint8_t* valid, int32_t P, int32_t K, int32_t Tmax,
                        float gamma, double* returns_out, double* adv_out, int32_t* group_n_out,
                        void* stream);

/*
 * Log-prob of y[t], entropy and logsumexp of softmax(H W^T / tau) for the rows with
 * row_mask[t] != 0 (row_mask NULL = all rows).  Outputs are float32 [T]; rows that are
 * masked out are written as 0.  entropy_out and lse_out may be NULL.
 */
int32_t pg_logprob_fwd(const void* H, const void* W, const int32_t* y, const uint8_t* row_mask, int64_t T,
                       int64_t d, int64_t V, const pg_params* h_params, float* logp_out,
                       float* entropy_out, float* lse_out, void* workspace, size_t workspace_bytes,
                       void* stream);

/*
 * Loss forward and backward for one packed microbatch of S segments; segment s covers
 * rows cu_seqlens[s] .. cu_seqlens[s+1]-1 (cu_seqlens[0] = 0, cu_seqlens[S] = T) and is one
 * training sample, i.e. one (prompt, rollout, turn).
 *
 *   loss_mask[t]      1 on response tokens (context / feedback rows are 0)
 *   adv               fp64 table of advantages (e.g. adv_out of trloo_advantage), h_params->n_samples
 *                     entries
 *   seg_sample        [S] index into adv of each segment; NULL = segment s uses adv[s]
 *   sample_keep       uint8 table indexed like adv (e.g. keep_out of prs_retain), nullable: a
 *                     segment whose flag is 0 was filtered out before training (Sec. 5.2) and is
 *                     treated exactly as if its loss_mask rows were 0 -- no loss, no gradient, not
 *                     in the normaliser, not examined by the mismatch correction
 *   old_logp          [T] log-prob under the policy that the update starts from; NULL =
 *                     on-policy (ratio 1, gradient of log-prob times advantage)
 *   rollout_logp      [T] log-prob reported by the rollout engine; required unless
 *                     mismatch_mode is PG_MISMATCH_NONE (old_logp is then required too)
 *
 * With delta_t = old_logp - rollout_logp on loss tokens, a sample is rejected if
 * exp(min delta) < veto_ratio, and in mode 1 also unless geo_lo <= exp(mean delta) <= geo_hi;
 * c_t is 1 (modes 0, 1) or min(exp(delta_t), trunc_c) (mode 2).  Active rows are the loss
 * tokens of samples that were not rejected.  For active rows, with r = exp(logp - old_logp)
 * and A the segment's advantage,
 *   l_t   = -min(r A, clip(r, 1-eps_lo, 1+eps_hi) A)
 *   loss  = (1/norm) sum_t c_t l_t
 *   dS    = (c_t (dl_t/dlogp_t) / (norm tau)) (onehot(y_t) - softmax_t)
 *   dH    = dS W   (rows that are not active are written as 0)
 *   dW    = dS^T H (added to dW if accumulate_dW)
 *
 * Outputs: loss_out (one float), dH [T,d] in the dtype of H, dW [V,d] in dW_dtype,
 * logp_out [T] and entropy_out [T] (nullable; 0 on rows that are not active),
 * counters_out [8] int64 (nullable; see PG_CNT_*).
 */
int32_t pg_loss_fwd_bwd(const void* H, const void* W, const int32_t* y, const uint8_t* loss_mask,
                        const int32_t* cu_seqlens, int32_t S, const double* adv,
                        const int32_t* seg_sample, const uint8_t* sample_keep, const float* old_logp,
                        const float* rollout_logp, int64_t T, int64_t d, int64_t V, const pg_params* h_params,
                        float* loss_out, void* dH, void* dW, float* logp_out, float* entropy_out,
                        int64_t* counters_out, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Cold-start SFT (Sec. 3.3): token-mean cross-entropy of the head over the rows with
 * loss_mask[t] != 0,
 *   loss = -(1/norm) sum_t log softmax(H_t W^T / tau)[y_t],   dS = (softmax_t - onehot(y_t)) / (norm tau),
 *   dH = dS W (0 on masked rows), dW = dS^T H (added to dW if accumulate_dW).
 * Of pg_params only dtype, temperature, norm_override, accumulate_dW and dW_dtype are used.
 * Outputs, workspace (pg_workspace_bytes with PG_CALL_LOSS_FWD_BWD, any S) and error behaviour
 * as for pg_loss_fwd_bwd; counters_out[PG_CNT_ACTIVE] = counters_out[PG_CNT_LOSS_TOKENS] = the
 * number of loss rows, the other counters are 0.
 */
int32_t pg_sft_fwd_bwd(const void* H, const void* W, const int32_t* y, const uint8_t* loss_mask, int64_t T,
                       int64_t d, int64_t V, const pg_params* h_params, float* loss_out, void* dH, void* dW,
                       float* logp_out, float* entropy_out, int64_t* counters_out, void* workspace,
                       size_t workspace_bytes, void* stream);

/*
 * Sec. 4.2, Eq. (2) and Eq. (3): as trloo_advantage, but with the group-mean baseline the paper
 * compares against, A = G - mean of the valid rollouts' G of the same prompt and turn (own
 * return included); 0 for invalid entries.
 */
int32_t grpo_advantage(const float* rewards, const uint8_t* valid, int32_t P, int32_t K, int32_t Tmax,
                       float gamma, double* returns_out, double* adv_out, int32_t* group_n_out,
                       void* stream);

/*
 * Sec. 4.2, Eq. (1) and Sec. 5.2, Eq. (6)-(7), for n samples (one sample = one turn of one rollout):
 *   speedup = min(t_reference / t_kernel, speedup_cap)        (the paper's cap is 3)
 *   PR      = t_generated / t_total                            (only if both are given)
 *   reward  = C + C speedup + C PR,   C = (correct != 0)
 * correct [n] uint8, times [n] float32 (> 0 where correct; ignored where not), t_generated and
 * t_total both NULL = Eq. (1) without the PR term.  rewards_out [n] float32; pr_out [n] float32
 * (nullable) receives C * PR.  Arithmetic is fp64, results are rounded to float32.
 */
int32_t turn_reward(const uint8_t* correct, const float* t_reference, const float* t_kernel,
                    const float* t_generated, const float* t_total, int64_t n, float speedup_cap,
                    float* rewards_out, float* pr_out, void* stream);

/*
 * Sec. 5.2, Eq. (8): sample i is retained with probability p_i = clip((pr_i - tau) / s, 0, 1)
 * (the paper's tau = 0.3, s = 0.1), or, with hard != 0, iff pr_i >= tau (the ablation without
 * softness).  The draw is reproducible: u_i = (x + 0.5) / 2^32 with x the first output word of
 * Philox-4x32-10 at counter (i mod 2^32, i div 2^32, 0, 0) and key (seed mod 2^32, seed div 2^32);
 * keep_i = u_i < p_i, decided in fp64.  valid (nullable) = 0 marks samples that were never
 * generated: they are not kept.  keep_out [n] uint8, p_out [n] float32 (nullable).  s > 0.
 */
int32_t prs_retain(const float* pr, const uint8_t* valid, int64_t n, float tau, float s, int32_t hard,
                   uint64_t seed, uint8_t* keep_out, float* p_out, void* stream);

/*
 * Sec. 5.1 monitors over the rows with loss_mask[t] != 0 (n of them):
 *   out[PG_MON_ENTROPY]      (1/n) sum entropy[t]                 (0 if entropy is NULL)
 *   out[PG_MON_PPL_TRAIN]    exp(-(1/n) sum logp_train[t])
 *   out[PG_MON_PPL_ROLLOUT]  exp(-(1/n) sum logp_rollout[t])       (0 if logp_rollout is NULL)
 *   out[PG_MON_DH_NORM]      Euclidean norm of dH [dH_elems]       (0 if dH is NULL)
 *   out[PG_MON_DW_NORM]      Euclidean norm of dW [dW_elems]       (0 if dW is NULL)
 *   out[PG_MON_TOKENS]       n
 * (n = 0 divides by 1.)  out is fp64 [8] in device memory.  dH_dtype / dW_dtype: 0 bf16, 1 fp32.
 * Sums are fp64 in a fixed order (bitwise repeatable).  workspace: pg_monitors_workspace_bytes().
 */
#define PG_MON_ENTROPY 0
#define PG_MON_PPL_TRAIN 1
#define PG_MON_PPL_ROLLOUT 2
#define PG_MON_DH_NORM 3
#define PG_MON_DW_NORM 4
#define PG_MON_TOKENS 5
size_t pg_monitors_workspace_bytes(void);
int32_t pg_monitors(const float* logp_train, const float* logp_rollout, const float* entropy,
                    const uint8_t* loss_mask, int64_t T, const void* dH, int32_t dH_dtype, int64_t dH_elems,
                    const void* dW, int32_t dW_dtype, int64_t dW_elems, double* out, void* workspace,
                    size_t workspace_bytes, void* stream);

/*
 * pg_monitors for callers that cannot allocate device memory (code under HIP graph capture, tight
 * loops, harnesses that forbid hipMalloc): same arguments, results and error behaviour, without the
 * workspace.  The partial sums (6 x 1024 fp64 = 49 152 bytes, for any input size) live in a static
 * device array inside the library; each GPU the library runs on holds one copy until the process
 * ends.  The call allocates and frees nothing.  Limits: T <= PG_MONITORS_STATIC_MAX_ROWS and
 * dH_elems, dW_elems <= PG_MONITORS_STATIC_MAX_ELEMS, else PG_ERR_UNSUPPORTED_SHAPE (use pg_monitors
 * with a workspace of the caller's).  All calls on one GPU share that GPU's array: calls that
 * overlap on one GPU (two streams, two threads) race and give undefined monitors; calls that
 * follow each other on a stream, or are otherwise ordered, are fine - every call rewrites all
 * partial sums before it reads them, so nothing is carried from one call to the next.  The array's
 * address is resolved on the first call on a device (or by pg_init()), which must not happen
 * inside a stream capture.
 */
#define PG_MONITORS_STATIC_MAX_ROWS 2147483648LL      /* 2^31 */
#define PG_MONITORS_STATIC_MAX_ELEMS 1099511627776LL  /* 2^40 */
int32_t pg_monitors_static(const float* logp_train, const float* logp_rollout, const float* entropy,
                           const uint8_t* loss_mask, int64_t T, const void* dH, int32_t dH_dtype, int64_t dH_elems,
                           const void* dW, int32_t dW_dtype, int64_t dW_elems, double* out, void* stream);

/*
 * The step in front of the head in the policies the paper trains (Qwen3, Sec. 6.1): per row,
 *   h = x * rstd * gamma,   rstd = 1 / sqrt(mean_j x_j^2 + eps),
 * and its backward for g = dL/dh (e.g. dH of pg_loss_fwd_bwd):
 *   xhat = x rstd,   dx = rstd (gamma g - xhat mean_j(gamma_j g_j xhat_j)),   dgamma = sum_rows g xhat.
 * X, H_out, dH, dX_out are [T,d], gamma is [d], all in `dtype` (PG_DTYPE_*); arithmetic is fp32;
 * rstd_out [T] float32 (nullable); dgamma_out [d] float32 (overwritten).  d must be a multiple of 8
 * and at most 8192 (PG_ERR_UNSUPPORTED_SHAPE otherwise); X, gamma, H_out, dH, dX_out must be 16-byte aligned.  The backward
 * needs pg_rmsnorm_bwd_workspace_bytes(d) bytes of workspace; its sums have a fixed order (bitwise
 * repeatable).  dX_out may alias dH.
 */
int32_t pg_rmsnorm_fwd(const void* X, const void* gamma, int64_t T, int64_t d, float eps, int32_t dtype,
                       void* H_out, float* rstd_out, void* stream);
size_t pg_rmsnorm_bwd_workspace_bytes(int64_t d);
int32_t pg_rmsnorm_bwd(const void* X, const void* gamma, const void* dH, int64_t T, int64_t d, float eps,
                       int32_t dtype, void* dX_out, float* dgamma_out, void* workspace, size_t workspace_bytes,
                       void* stream);

/*
 * pg_loss_fwd_bwd with that normalisation fused around the head: the hidden states that enter the head
 * are h_t = x_t rstd_t gamma (computed in fp32, rounded once to the storage dtype, exactly what
 * pg_rmsnorm_fwd writes) and the call returns dX and dgamma instead of dH, i.e. what pg_rmsnorm_bwd
 * gives for dH of pg_loss_fwd_bwd - except that dH reaches the normalisation's backward in fp32, not
 * rounded to the storage dtype in between.  The forward is applied while the active rows are
 * compacted (rows that are not active are never read) and the backward while the gradient rows are
 * scattered, so the two extra passes over [T, d] of the separate calls disappear.
 *   X [T,d], gamma [d]   in the dtype of h_params->dtype;  norm_eps >= 0
 *   dX [T,d]             same dtype; rows that are not active are written as 0
 *   dgamma_out [d]       float32, overwritten: sum over the active rows of dH_t xhat_t
 * All other arguments, outputs and errors as pg_loss_fwd_bwd.  d must not exceed 8192.
 * Workspace: pg_workspace_bytes(..., PG_CALL_LOSS_FWD_BWD_NORMED).
 */
int32_t pg_loss_fwd_bwd_normed(const void* X, const void* gamma, float norm_eps, const void* W, const int32_t* y,
                               const uint8_t* loss_mask, const int32_t* cu_seqlens, int32_t S, const double* adv,
                               const int32_t* seg_sample, const uint8_t* sample_keep, const float* old_logp,
                               const float* rollout_logp, int64_t T, int64_t d, int64_t V, const pg_params* h_params,
                               float* loss_out, void* dX, float* dgamma_out, void* dW, float* logp_out,
                               float* entropy_out, int64_t* counters_out, void* workspace, size_t workspace_bytes,
                               void* stream);

/*
 * Vocab-sharded head: the quantities of pg_logprob_fwd and pg_loss_fwd_bwd (pi_train of Sec. 5.1,
 * the estimator of App. A) when W is split by vocabulary rows and each device holds
 * W_shard = W[v_offset : v_offset + V_shard, :].  y holds token ids of the WHOLE vocabulary.
 * One device's share is two calls with one exchange between them:
 *
 * pg_head_shard_fwd: for the rows with row_mask[t] != 0 (NULL = all rows) writes the row's softmax
 * state over this shard's logits z = H_t W_shard^T / tau,
 *   partials_out[t] = (m, s, u, z_y) = (max_v z_v, sum_v e^(z_v - m), sum_v e^(z_v - m)(z_v - m),
 *                                      z at y[t] if v_offset <= y[t] < v_offset + V_shard else 0),
 * [T][4] fp32, natural-log units; rows that are masked out are written as (0, 0, 0, 0), the empty
 * state.  Workspace: pg_workspace_bytes(T, d, V_shard, 0, params, PG_CALL_LOGPROB_FWD).
 *
 * pg_head_partials_merge: out[t] = a[t] (+) b[t], the state of the union of two disjoint vocab
 * ranges: m = max(m_a, m_b), s = e^(m_a - m) s_a + e^(m_b - m) s_b,
 * u = e^(m_a - m)(u_a + (m_a - m) s_a) + e^(m_b - m)(u_b + (m_b - m) s_b), z_y = z_y,a + z_y,b;
 * an empty state (s = 0) is the neutral element.  This is the operator an all-reduce over the
 * shards applies (16 bytes per token); on one device it merges states computed one after the
 * other.  out may alias a or b.  From the merged state: logsumexp = m + ln s,
 * log-prob = z_y - logsumexp, entropy = ln s - u / s.
 *
 * pg_head_partials_finish: those three per row from a merged state, logp_out [T] (required),
 * entropy_out and lse_out [T] (nullable); rows with the empty state give 0.  With it the
 * forward-only recompute of pg_logprob_fwd runs on a sharded head: shard_fwd, exchange, finish.
 *
 * pg_loss_shard_bwd: arguments, loss, counters, logp_out and entropy_out as pg_loss_fwd_bwd, except
 * that the forward contraction is not run: the rows' log-prob, entropy and logsumexp are taken
 * from `partials` ([T][4], the state merged over ALL shards; read on active rows only).  Writes
 *   dW_shard   = dS[:, shard]^T H            [V_shard, d], complete (added to if accumulate_dW),
 *   dH_partial = dS[:, shard] W_shard        [T, d], this shard's term of the sum over shards that
 *                gives dH; fp32 if dH_f32 != 0 (what a sum all-reduce wants), else the dtype of H.
 * loss_out, logp_out, entropy_out and the counters are the same on every shard.
 * With the whole head as the one shard (v_offset = 0, V_shard = V) this is pg_loss_fwd_bwd without its
 * forward contraction: a caller whose old-policy recompute (pg_head_shard_fwd + pg_head_partials_finish)
 * ran on the same H and W can hand its states over and save a quarter of the step's flops.
 * Workspace: pg_workspace_bytes(T, d, V_shard, S, params, PG_CALL_LOSS_FWD_BWD).
 * Errors as for pg_loss_fwd_bwd; partials and partials_out must be 16-byte aligned.
 */
int32_t pg_head_shard_fwd(const void* H, const void* W_shard, const int32_t* y, const uint8_t* row_mask, int64_t T,
                          int64_t d, int64_t V_shard, int64_t v_offset, const pg_params* h_params, float* partials_out,
                          void* workspace, size_t workspace_bytes, void* stream);
int32_t pg_head_partials_merge(const float* a, const float* b, float* out, int64_t T, void* stream);
int32_t pg_head_partials_finish(const float* partials, int64_t T, float* logp_out, float* entropy_out, float* lse_out,
                                void* stream);
int32_t pg_loss_shard_bwd(const void* H, const void* W_shard, const int32_t* y, const uint8_t* loss_mask,
                          const int32_t* cu_seqlens, int32_t S, const double* adv, const int32_t* seg_sample,
                          const uint8_t* sample_keep, const float* old_logp, const float* rollout_logp,
                          const float* partials, int64_t T, int64_t d, int64_t V_shard, int64_t v_offset, const pg_params* h_params, float* loss_out, void* dH_partial,
                          int32_t dH_f32, void* dW_shard, float* logp_out, float* entropy_out, int64_t* counters_out,
                          void* workspace, size_t workspace_bytes, void* stream);

/*
 * Measurement hooks (host-side state, not thread-safe; the only calls that create HIP events
 * or wait on the device).  pg_profile_enable(1, n) creates a pool for n kernel launches; from
 * then on each launch of the MFMA kernels is bracketed by two events on the caller's stream.
 * pg_profile_read waits for the recorded events, returns the summed durations in milliseconds
 * and the launch counts per kernel class (host arrays of PG_KERNEL_CLASSES entries), and
 * empties the pool.  pg_profile_enable(0, 0) releases the events.
 */
#define PG_KERNEL_FWD 0      /* logits + online softmax statistics               */
#define PG_KERNEL_DLOGITS 1  /* logits recompute + dS in both orientations       */
#define PG_KERNEL_DW 2       /* dW = dS^T H   (gemm_store_kernel)                */
#define PG_KERNEL_DH 3       /* dH = dS W     (gemm_store_kernel)                */
#define PG_KERNEL_CLASSES 4
int32_t pg_profile_enable(int32_t on, int32_t max_launches);
int32_t pg_profile_read(double* h_ms, int64_t* h_launches);

#ifdef __cplusplus
}
#endif
#endif /* PG_HEAD_H */
