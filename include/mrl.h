/*
 * mrl.h - C ABI of the MI355X (gfx950) GRPO scoring library.
 *
 * The library computes the data-parallel hot path of a GRPO-based training
 * step as used by the Mutual RL paper: per-token log-probabilities of the
 * sampled tokens under the learner (LM-head projection, log-softmax over the
 * full vocabulary, gather at the target id), group-relative advantages, the
 * clipped importance-ratio surrogate with a KL term to a reference policy,
 * and the backward pass to the hidden states and the LM-head weight.
 *
 * Conventions for every entry point
 *   - Returns an mrl_status (0 = MRL_OK, negative = error).  Never throws,
 *     never aborts.  Arguments are validated on the host before any device
 *     work is enqueued; on error nothing has been launched (the two data-dependent
 *     codes of the debug_sync mode of call (3) are the exception, see there).
 *   - Every tensor pointer is a DEVICE pointer owned by the caller.  The
 *     library allocates no device memory: scratch space comes from the
 *     caller's workspace, whose size is obtained from the matching
 *     *_workspace() query (256-byte aligned base required).
 *   - Work is enqueued on the caller's stream (a hipStream_t passed as
 *     void*, NULL = the default stream) and is asynchronous: outputs are
 *     valid once the caller has synchronised that stream.  No host
 *     synchronisation happens inside a call (debug_sync of call (3) excepted).
 *   - Inputs are never modified.  Outputs are fully overwritten, except
 *     out_dW when accumulate_dw = 1.
 *   - All tensors are dense and row-major.  lm_head_w is [V, d], one row per
 *     vocabulary id (the layout of a linear layer's weight).  Row n of hidden
 *     is the final hidden state that PREDICTS target_ids[n]; the shift
 *     between inputs and labels is the caller's business.  No bias, sampling
 *     temperature 1.
 *   - dtype MRL_BF16: hidden / lm_head_w are bfloat16, matrix products run on
 *     the bf16 MFMA units with fp32 accumulation; d must be a multiple of 8 (rows of 16-byte
 *     vectors).  Widths that are not a multiple of 128 run on zero-padded copies of the operands
 *     (a little extra workspace and time); multiples of 256 use the matrix cores best.
 *     dtype MRL_F32: hidden / lm_head_w are float, plain fp32 arithmetic (a
 *     small-shape sanity path, not tuned); any d >= 1.
 *   - Only gfx950 devices are supported; there is no fallback path.
 */
#ifndef MRL_H
#define MRL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  MRL_OK = 0,
  MRL_ERR_NULL = -1,             /* a required pointer is NULL                          */
  MRL_ERR_SHAPE = -2,            /* a size is <= 0, too large, or violates a divisibility rule */
  MRL_ERR_DTYPE = -3,            /* unknown mrl_dtype                                   */
  MRL_ERR_TARGET_RANGE = -4,     /* debug_sync only: a scored slot has a target id outside [0, V) */
  MRL_ERR_GROUP_RANGE = -5,      /* debug_sync only: a sequence has a group id outside [0, G)     */
  MRL_ERR_WORKSPACE = -6,        /* workspace NULL, misaligned or too small             */
  MRL_ERR_CONFIG = -7,           /* a configuration value is out of its domain          */
  MRL_ERR_DEVICE = -8,           /* no usable device / a HIP call failed                */
  MRL_ERR_UNSUPPORTED_ARCH = -9, /* the current device is not gfx950                    */
  MRL_ERR_SCRATCH_LIMIT = -10    /* mrl_token_logprobs_static: the input needs more scratch memory
                                    than the library's built-in buffer holds                      */
} mrl_status;

typedef enum { MRL_F32 = 0, MRL_BF16 = 1 } mrl_dtype;

typedef enum {
  MRL_ADV_CENTER = 0,   /* A = r - mean(group)                     (Sec. 3, A-tilde)            */
  MRL_ADV_GROUP_ZN = 1, /* A = (r - mean) / (std(group) + eps)     (Sec. 3, A-tilde-zn)         */
  MRL_ADV_BATCH_ZN = 2  /* centre per group, divide by the std over all scored entries (App. A) */
} mrl_adv_mode;

/* bits of out_flags[g] of mrl_group_advantages (SGT gate, Sec. 5.3 / App. B) */
#define MRL_FLAG_ALL_FAIL 1u     /* every own rollout of the group has reward < neg_thresh */
#define MRL_FLAG_PEER_SUCCESS 2u /* some non-own entry has reward > pos_thresh             */
#define MRL_FLAG_RESCUE 4u       /* both: the gate fires for this prompt                   */

const char* mrl_status_string(int status);
int mrl_version(void);

/* ------------------------------------------------------------------------
 * (1) Token log-probabilities  l_theta[n] = log pi_theta(y_n | context)
 *     (Sec. 3, GRPO paragraph: the entries of the trace l_theta(x, y)).
 *
 *   z[n, v] = sum_k hidden[n, k] * lm_head_w[v, k]
 *   lse[n]  = log sum_v exp z[n, v]
 *   out_logp[n] = z[n, target_ids[n]] - lse[n]
 *
 * The N x V logits are never written to memory.  token_mask (uint8, 0/1) may
 * be NULL (= every row is scored); rows with mask 0 or with a target id
 * outside [0, V) are skipped and report out_logp = out_lse = 0.  out_lse may
 * be NULL.  N >= 0 (N = 0 is a no-op).
 * ---------------------------------------------------------------------- */
size_t mrl_token_logprobs_workspace(int64_t N, int32_t d, int32_t V, int32_t dtype);
int mrl_token_logprobs(const void* hidden /*[N,d] dev*/, const void* lm_head_w /*[V,d] dev*/,
                       const int32_t* target_ids /*[N] dev*/,
                       const uint8_t* token_mask /*[N] dev | NULL*/,
                       int64_t N, int32_t d, int32_t V, int32_t dtype,
                       float* out_logp /*[N] dev*/, float* out_lse /*[N] dev | NULL*/,
                       void* workspace /*dev*/, size_t workspace_bytes, void* stream);

/* (1c) mrl_token_logprobs for callers that cannot allocate device memory or hand over a
 *      workspace: code under HIP graph capture, tight serving loops, harnesses that forbid
 *      allocation.  Same arguments minus the workspace, same kernels, same results (bit for bit).
 *      The scratch space is a buffer of MRL_STATIC_SCRATCH_BYTES built into the library's device
 *      image: every GPU the library runs on holds one copy from the first call until the process
 *      ends.  The call allocates and frees nothing, on the host side of HIP or the device.
 *      Limits: the buffer must hold about 8 bytes per row of N plus, for the smallest pass of
 *      256 rows, 8 bytes per vocabulary id (partial sums) and 512 bytes per hidden column (the
 *      pass's gathered rows); at V = 151936, d = 4096 that allows N up to about 3.7 million rows.
 *      Widths that are not a multiple of 128 also need a padded copy of lm_head_w in the buffer.
 *      An input beyond the limit returns MRL_ERR_SCRATCH_LIMIT and launches nothing.
 *      All calls on one GPU share that GPU's buffer: two calls whose work overlaps in time on the
 *      same GPU (different streams, or different host threads) race on it and give undefined
 *      results; calls on one stream, or otherwise ordered, are fine.  Nothing in the buffer needs
 *      to survive between calls and nothing needs clearing: every call writes what it reads. */
#define MRL_STATIC_SCRATCH_BYTES (32u << 20)
int mrl_token_logprobs_static(const void* hidden /*[N,d] dev*/, const void* lm_head_w /*[V,d] dev*/,
                              const int32_t* target_ids /*[N] dev*/,
                              const uint8_t* token_mask /*[N] dev | NULL*/,
                              int64_t N, int32_t d, int32_t V, int32_t dtype,
                              float* out_logp /*[N] dev*/, float* out_lse /*[N] dev | NULL*/,
                              void* stream);

/* (1b) Scoring pass with diagnostics: the same log-probs plus, when out_entropy is not
 *      NULL, the entropy of the next-token distribution of every scored row,
 *        out_entropy[n] = - sum_v p[n, v] log p[n, v] = lse[n] - sum_v p[n, v] z[n, v],
 *      the per-token quantity behind the entropy traces of Sec. 5 ("Optimization
 *      Diagnostics").  This is the forward-only pass that produces the behaviour and
 *      reference traces and re-scores pooled peer rollouts before the loss call.
 *      Unscored rows report 0.  out_lse and out_entropy may be NULL; with out_entropy
 *      NULL the call is mrl_token_logprobs.  The workspace query is its own because the
 *      entropy needs a third partial per row and vocabulary tile. */
size_t mrl_token_scores_workspace(int64_t N, int32_t d, int32_t V, int32_t dtype);
int mrl_token_scores(const void* hidden /*[N,d] dev*/, const void* lm_head_w /*[V,d] dev*/,
                     const int32_t* target_ids /*[N] dev*/,
                     const uint8_t* token_mask /*[N] dev | NULL*/,
                     int64_t N, int32_t d, int32_t V, int32_t dtype,
                     float* out_logp /*[N] dev*/, float* out_lse /*[N] dev | NULL*/,
                     float* out_entropy /*[N] dev | NULL*/,
                     void* workspace /*dev*/, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------
 * (2) Group-relative advantages and the SGT gate.
 *     Sec. 3: rbar = mean of the group's rewards, A~ = r - rbar,
 *     A~zn = A~ / (std + eps).  Sec. 5.1 (PRP): own and peer rollouts of a
 *     prompt form one group and are normalised together.  App. I.1 (XGRPO):
 *     the baseline mean / std pool the rewards of every policy while only
 *     own rollouts are scored.  Sec. 5.3 / App. B (SGT): the gate fires for a
 *     prompt when every own rollout failed and some peer succeeded.
 *
 * Entries b = 0..B-1 are rollouts (or bare peer rewards); group_id[b] in
 * [0, G) names the prompt; entries of a group need not be contiguous.
 *   in_stats[b] = 1 : the reward enters the group's mean / std   (NULL = all 1)
 *   scored[b]   = 1 : an advantage is emitted, else out_adv[b] = 0 (NULL = all 1)
 *   is_own[b]   = 1 : the rollout is the learner's own             (NULL = all 1)
 * std uses divisor (count - ddof), ddof in {0, 1}; std = 0 if count <= ddof.
 * mix_alpha in [0, 1]: A = (1 - alpha) * A_own + alpha * A_pool, where A_own
 * uses statistics over (in_stats & is_own) entries only; 1 = pooled rule.
 * baseline_shift (NULL = none): baseline_shift[g] is added to the per-prompt baseline
 * of group g, its pooled and its own-only mean alike, before the rewards are centred;
 * the std stays that of the unshifted rewards and out_group_mean reports the unshifted
 * pooled mean.  It is the perturbed-baseline control of App. C.4 (shared-normalisation
 * ablation); the caller draws the perturbations.
 * An entry whose group id is outside [0, G) gets advantage 0 and enters no
 * statistic.  Sums are accumulated in fp64 in a fixed order (bit-reproducible).
 * Optional outputs (NULL to skip): out_group_mean / out_group_std (pooled
 * statistics), out_flags (MRL_FLAG_* bits).
 * ---------------------------------------------------------------------- */
int mrl_group_advantages(const float* rewards /*[B] dev*/, const int32_t* group_id /*[B] dev*/,
                         const uint8_t* in_stats /*[B] dev | NULL*/,
                         const uint8_t* scored /*[B] dev | NULL*/,
                         const uint8_t* is_own /*[B] dev | NULL*/,
                         const float* baseline_shift /*[G] dev | NULL*/,
                         int64_t B, int32_t G, int32_t adv_mode, float eps_norm, int32_t ddof,
                         float mix_alpha, float neg_thresh, float pos_thresh,
                         float* out_adv /*[B] dev*/, float* out_group_mean /*[G] dev | NULL*/,
                         float* out_group_std /*[G] dev | NULL*/, uint8_t* out_flags /*[G] dev | NULL*/,
                         void* stream);

/* ------------------------------------------------------------------------
 * (3) Fused scoring + GRPO loss, forward and backward.
 *     Eq. (1): L_GRPO = - E_x (1/K) sum_i E_tok[ min(w A, clip(w, 1-eps, 1+eps) A) ]
 *              + beta * R(theta),  w = exp(l_theta - l_behaviour);
 *     R(theta) is the k3 estimator exp(rho) - rho - 1, rho = l_ref - l_theta,
 *     averaged with the same weights.  Eq. (2): auxiliary SGT rows add
 *     lambda * (- token-mean l_theta), averaged over the auxiliary rows.
 *     behav_logp carries l_old for own rollouts and the aligned peer trace
 *     for pooled peer rollouts (Sec. 5.1, the two denominators); advantages,
 *     behaviour and reference traces are constants of the differentiation.
 *
 * Tokens are [B, T] right- or arbitrarily padded, token_mask marks scored
 * slots.  seq_kind[b]: 0 = GRPO row, 1 = SGT auxiliary row (NULL = all 0).
 * Weights (loss_agg = 0): c = mask / (P * K_g * L_b) for GRPO rows, with L_b
 * the row's scored tokens, K_g the GRPO rows of its group, P the groups with
 * a GRPO row; c_sgt = mask / (S_aux * L_b), S_aux = auxiliary rows with
 * L_b > 0.  loss_agg = 1: c = mask / (all scored GRPO tokens).
 * Backward: g = dL/dl; dz[n, v] = g[n] (1[v = y_n] - softmax[n, v]);
 * out_dH = dz W (rows of unscored slots are zero), out_dW (+)= dz^T H in fp32.
 * Every reduction runs in a fixed order (no floating-point atomics): results are
 * bit-reproducible from run to run, so there is no separate deterministic mode.
 * out_dH and/or out_dW may be NULL to skip that gradient.
 * Numerical range (bf16 path): logits of any offset and scale are handled (exponentials
 * are taken relative to the row's target logit, in fp32, straight from the accumulators);
 * the backward operands are exact to bf16 rounding as long as the target's log-prob is
 * above about -97.  A row below that (a token the learner deems impossible, p < 1e-42)
 * reports a finite, saturated log-prob <= -97, contributes nothing to the loss and the
 * gradients (it still counts in its sequence's length), and is counted in
 * n_saturated_rows.
 * ref_logp may be NULL when kl_beta = 0.  group_id[b] must lie in [0, G); a
 * row with an id outside gets weight 0.
 * ---------------------------------------------------------------------- */
typedef struct {
  float clip_eps_low;    /* lower clip: ratios below 1 - clip_eps_low are clipped; paper: 0.2 */
  float clip_eps_high;   /* upper clip: 1 + clip_eps_high; paper: 0.2                         */
  float kl_beta;         /* coefficient of the KL term (paper's runs: 1e-3)                   */
  float sgt_lambda;      /* weight of the SGT auxiliary loss (paper: 0.1)                     */
  int32_t loss_agg;      /* 0 = Eq. (1) literal (seq-mean of token-means), 1 = global token mean */
  int32_t accumulate_dw; /* 0 = overwrite out_dW, 1 = add into it                             */
  int32_t dh_dtype;      /* mrl_dtype of out_dH                                               */
  int32_t chunk_rows;    /* 0 = automatic; else scored rows per pass (multiple of 256)        */
  int64_t scored_rows_hint; /* 0 = unknown.  Else an upper bound on the number of scored slots the
                               caller vouches for (it usually knows the sequence lengths): only
                               ceil(hint / chunk_rows) passes are enqueued instead of the worst case
                               ceil(B*T / chunk_rows).  If the mask holds more scored slots than the
                               hint, the excess rows are NOT processed: their out_logp is NaN and
                               n_unprocessed_rows reports how many.                              */
  int32_t ratio_level;   /* which importance ratio enters Eq. (1):
                            0 = per token, w_t = exp(l_t - l_beh,t)                (Sec. 3)
                            1 = per response, exp{L_theta - L_behavior}, L = sums over the
                                response's scored tokens                           (App. I.1)
                            2 = per response, exp of the per-token mean of the same sum (the
                                magnitudes of App. E.3's sequence-ratio table are those of a mean)
                            Levels 1 and 2 need loss_agg = 0; the KL term stays per token; the
                            ratio statistics then count each token with its response's ratio.
                            They run the forward contraction twice (the response sums must be
                            complete before any token's gradient weight is known).           */
  int32_t debug_sync;    /* 0 = fully asynchronous (default): target and group ids are range-checked on
                            the device only, offenders are skipped and counted (n_bad_targets; a bad
                            group id gives its row weight 0).
                            1 = debugging aid: after the preparation kernels the call waits for the
                            stream, reads the two counters back and returns MRL_ERR_TARGET_RANGE or
                            MRL_ERR_GROUP_RANGE if either is non-zero; no GEMM has been enqueued then
                            and the outputs hold nothing defined.  Not for timed or captured code.  */
} mrl_loss_config;

typedef struct {
  double loss_total, loss_pg, loss_kl, loss_sgt; /* L = pg + beta*kl + lambda*sgt */
  double mean_ratio, max_ratio, mean_k3;         /* over scored GRPO tokens       */
  int64_t n_scored_tokens;                       /* scored slots with a valid target */
  int64_t n_clipped_tokens;                      /* ratio outside [1-eps_low, 1+eps_high] */
  int64_t n_zero_grad_tokens;                    /* clipped branch active (no surrogate gradient) */
  int64_t n_bad_targets;                         /* masked-in slots whose target id is outside [0,V) */
  int64_t n_unprocessed_rows;                    /* scored slots beyond scored_rows_hint (0 unless the hint was wrong) */
  int64_t n_saturated_rows;                      /* bf16 path: scored rows whose target log-prob is below about -97,
                                                    outside the range the backward operands represent (see
                                                    "Numerical range" above): dropped from the loss and the gradients */
} mrl_loss_stats;

size_t mrl_grpo_loss_workspace(int64_t B, int32_t T, int32_t d, int32_t V, int32_t dtype,
                               const mrl_loss_config* cfg);
int mrl_grpo_loss_fwd_bwd(const void* hidden /*[B*T,d] dev*/, const void* lm_head_w /*[V,d] dev*/,
                          const int32_t* target_ids /*[B*T] dev*/,
                          const uint8_t* token_mask /*[B*T] dev*/,
                          const float* behav_logp /*[B*T] dev*/,
                          const float* ref_logp /*[B*T] dev | NULL*/,
                          const float* seq_adv /*[B] dev*/, const int32_t* group_id /*[B] dev*/,
                          const uint8_t* seq_kind /*[B] dev | NULL*/,
                          int64_t B, int32_t T, int32_t G, int32_t d, int32_t V, int32_t dtype,
                          const mrl_loss_config* cfg /*host*/,
                          float* out_logp /*[B*T] dev*/, void* out_dH /*[B*T,d] dev | NULL*/,
                          float* out_dW /*[V,d] dev | NULL*/, mrl_loss_stats* out_stats /*dev*/,
                          void* workspace /*dev*/, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------
 * (4) THL word-level trace alignment on integer word maps (Sec. 4.3; App. D,
 *     "THL WordAlignLogProbs", Alg. 2).  A peer's per-token log-probs on its own
 *     token grid (source) are carried over to the learner's grid (target): the
 *     source log-probs of the response tokens of a word are summed (Z_w) and every
 *     target response token of that word receives Z_w / C_w, C_w being the number
 *     of target tokens of the word.  The result is the behaviour trace of a pooled
 *     peer rollout (behav_logp of call (3)); positions left at ignore_value are
 *     the ones the caller clears in token_mask.
 *
 *   src_logp     [B, S_src] float, finite, |value| < 2^30.
 *   src_mask     [B, S_src] 1 = response token of the source grid.
 *   src_word_map [B, S_src] entry p of row i is the word index, in [0, max_words),
 *                of the p-th response token (the p-th set bit of src_mask row i), or
 *                -1 for a token that belongs to no word (leading delimiters); only
 *                the first src_map_len[i] entries are meaningful.
 *   src_map_len  [B] length of row i's map.  When it differs from the number of
 *                response tokens, the shorter of the two is used (Alg. 2).
 *   tgt_*        likewise on the target grid.
 *   out          [B, S_tgt] fully overwritten: ignore_value everywhere except at the
 *                target response tokens that carry a word.  A word without source
 *                tokens has Z_w = 0.  A sequence whose source side carries no word at
 *                all stays entirely at ignore_value.
 *   out_bad_words [1] | NULL: number of map entries outside [-1, max_words) among the
 *                entries in use; they are treated as -1.
 *   max_words <= 8192 (per-word sums and counts live in on-chip memory).
 *   Sums are accumulated exactly in 2^-32 fixed point: results do not depend on the
 *   order of evaluation and are bit-reproducible.  No workspace.  Asynchronous on
 *   `stream`.  All tensor pointers are device pointers owned by the caller.
 *   Errors: MRL_ERR_SHAPE (sizes, max_words), MRL_ERR_NULL.
 * ---------------------------------------------------------------------- */
int mrl_thl_word_align(const float* src_logp /*[B,S_src] dev*/, const uint8_t* src_mask /*[B,S_src] dev*/,
                       const int32_t* src_word_map /*[B,S_src] dev*/, const int32_t* src_map_len /*[B] dev*/,
                       const uint8_t* tgt_mask /*[B,S_tgt] dev*/, const int32_t* tgt_word_map /*[B,S_tgt] dev*/,
                       const int32_t* tgt_map_len /*[B] dev*/, int64_t B, int32_t S_src, int32_t S_tgt,
                       int32_t max_words, float ignore_value, float* out /*[B,S_tgt] dev*/,
                       int64_t* out_bad_words /*[1] dev | NULL*/, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MRL_H */
