/*
 * libgrpo - token-level GRPO policy objective with two-sided clipping,
 * forward and fused backward, for AMD MI355X (gfx950).
 *
 * The operation is the objective of section 3.4 of the INTELLECT-2 paper
 * (second displayed objective, the one that adds the bound delta):
 *
 *   J_t  = min( min(r_t, delta) A_t , clip(r_t, 1 - eps_low, 1 + eps_high) A_t )
 *   r_t  = pi_theta(y_t) / pi_theta_old(y_t) = exp(l_t - l_old_t)
 *   l_t  = log softmax(z_t / T)[y_t]
 *   loss = -(1/D) sum_t m_t J_t          (token-level mean, section 4.1)
 *
 * with z_t the row of policy logits of token t, y_t the sampled token, A_t the
 * group-relative advantage (section 3.4), m_t the response mask.  The paper uses
 * eps_low = eps_high = 0.2 and delta = 4 (section 4.1).
 *
 * Conventions shared by every entry point
 *  - All data pointers are DEVICE pointers owned by the caller.  The library
 *    allocates nothing, frees nothing and keeps no per-call state; scratch comes
 *    from the caller's workspace (one entry point, grpo_loss_fwd_bwd_noalloc, uses an
 *    array built into the library instead; see there).
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All
 *    work is enqueued on it; nothing synchronises with the host, so results are
 *    device-resident and valid once the stream has reached that point.
 *  - Arguments are validated on the host BEFORE any GPU call; a failed
 *    validation returns a code below and launches nothing.  Problems that only
 *    the data can reveal (a token id outside [0, vocab)) cannot be returned as a
 *    code; see each function.
 *  - NaN or Inf in the logits of an unmasked row propagate to that row's
 *    outputs and to the loss; they are never hidden.
 *  - Rows are independent; 64-bit indexing throughout (n_tokens * vocab may
 *    exceed 2^31).  vocab itself must lie in [1, 2^28].
 */
#ifndef GRPO_H
#define GRPO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    GRPO_OK = 0,
    GRPO_ERR_NULL = 1,      /* a required pointer is NULL                              */
    GRPO_ERR_SHAPE = 2,     /* a size is negative/zero where it may not be, stride < vocab */
    GRPO_ERR_DTYPE = 3,     /* dtype is not one of grpo_dtype                          */
    GRPO_ERR_ALIGN = 4,     /* logits/grad base or row pitch not 16-byte aligned       */
    GRPO_ERR_PARAM = 5,     /* temperature <= 0, eps out of range, delta <= 1+eps_high */
    GRPO_ERR_WORKSPACE = 6, /* workspace NULL, misaligned or too small                 */
    GRPO_ERR_HIP = 7,       /* the HIP runtime reported an error at launch             */
    GRPO_ERR_CAPACITY = 8   /* more rows than the library's built-in scratch array holds
                               (grpo_loss_fwd_bwd_noalloc only)                         */
} grpo_status;

typedef enum {
    GRPO_F32 = 0, /* IEEE binary32 logits and gradients            */
    GRPO_BF16 = 1 /* bfloat16 logits and gradients (RNE on store)  */
} grpo_dtype;

/* Index of each counter in counts_out of grpo_loss_fwd_bwd. */
enum {
    GRPO_COUNT_TOKENS = 0,     /* M = number of rows with mask 1                       */
    GRPO_COUNT_CLIP_HIGH = 1,  /* A > 0 and r > 1 + eps_high (gradient cut)            */
    GRPO_COUNT_CLIP_LOW = 2,   /* A < 0 and r < 1 - eps_low  (gradient cut)            */
    GRPO_COUNT_DELTA = 3,      /* A < 0 and r > delta        (gradient cut, sec. 3.4)  */
    GRPO_COUNT_OUT_OF_BAND = 4 /* r outside [1-eps_low, 1+eps_high], any A: the "token
                                  probability clip ratio" tracked in section 3.5       */
};

/* Static, human-readable text for a status code.  Never NULL. */
const char *grpo_status_string(grpo_status status);

/* Bytes of device workspace grpo_loss_fwd_bwd / grpo_loss_aux_fwd_bwd need for n_tokens rows (a pure host
 * function; returns 0 for n_tokens < 0).  The workspace must be 256-byte aligned. */
size_t grpo_workspace_bytes(int64_t n_tokens);

/*
 * Which row kernel serves logits rows of a given width (a pure host function, for
 * reading profiles and for sizing expectations; it launches nothing).  The path of
 * section 3.4 reads every logit at least once and writes every gradient once; how
 * often a row is read a second time depends on whether it stays on the chip between
 * the softmax statistics and the gradient:
 *   streaming = 0: one workgroup of `lanes` lanes holds `register_slots` 16-byte
 *     vectors per lane in registers and `lds_slots` more per lane in LDS
 *     (`resident_vectors` of the row's `vectors` in all); these are read once.
 *     With streamed_remainder = 1 the vectors beyond them are read twice.
 *     ragged_tail_slot = 1: the instantiation also serves a vocabulary that ends
 *     inside a 16-byte vector.  workgroups_per_cu of them share a compute unit.
 *   streaming = 1: the row is read twice (online maximum and sum, then the gradient).
 * Errors: GRPO_ERR_DTYPE, GRPO_ERR_SHAPE (vocab outside [1, 2^28]), GRPO_ERR_NULL.
 */
typedef struct grpo_row_plan {
    int64_t vectors;           /* ceil(vocab / 8) for bf16, ceil(vocab / 4) for f32 */
    int64_t resident_vectors;  /* of those, how many stay on the chip between the passes */
    int32_t streaming;
    int32_t lanes;
    int32_t register_slots;
    int32_t lds_slots;
    int32_t workgroups_per_cu;
    int32_t ragged_tail_slot;
    int32_t streamed_remainder;
    int32_t reserved;
} grpo_row_plan;
grpo_status grpo_row_kernel_plan(grpo_dtype dtype, int64_t vocab, grpo_row_plan *plan_out /* host */);

/*
 * Group-relative advantages (section 3.4: each prompt's G sampled outputs are
 * scored relative to one another; section 3.3: a group whose rewards are all
 * equal has zero advantages).  The paper gives no formula; this library uses
 *     A_i = (R_i - mean_g) / (std_g + eps_std),
 *     std_g = sqrt( sum_{i in g} (R_i - mean_g)^2 / (G - ddof) ),
 * and A_i = 0 when G - ddof <= 0 or std_g + eps_std == 0.
 *
 *  rewards          [n_rollouts] f32, device, read.
 *  group_offsets    [n_groups+1] i32, device, read, or NULL.  Group g owns rollouts
 *                   [group_offsets[g], group_offsets[g+1]).  Offsets outside
 *                   [0, n_rollouts] or decreasing are clamped on the device (no
 *                   out-of-bounds access; the affected advantages are unspecified).
 *  group_size       used when group_offsets is NULL: every group has group_size
 *                   rollouts and n_rollouts must equal n_groups * group_size.
 *  eps_std >= 0, ddof in {0, 1}.
 *  adv_out          [n_rollouts] f32, device, written (rollouts no group owns are
 *                   left untouched).
 *  rollout_of_token [n_tokens] i32, device, read, or NULL: rollout index of every
 *                   token row.  With it, adv_tok_out[t] = adv_out[rollout_of_token[t]]
 *                   (NaN if the index is outside [0, n_rollouts)).
 *  adv_tok_out      [n_tokens] f32, device, written; required iff rollout_of_token
 *                   is given.
 * Accumulation is in fp64, so results are independent of launch shape.
 * n_groups == 0 and n_tokens == 0 are legal and do nothing.
 */
grpo_status grpo_group_advantages(const float *rewards, int64_t n_rollouts,
                                  const int32_t *group_offsets, int64_t n_groups,
                                  int64_t group_size, float eps_std, int ddof,
                                  float *adv_out, const int32_t *rollout_of_token,
                                  int64_t n_tokens, float *adv_tok_out, void *stream);

/*
 * Total reward with the length penalty of section 3.1,
 *     rewards_out[i] = task_rewards[i] - alpha * | target_lengths[i] - lengths[i] |,
 * lengths in tokens (alpha = 3e-4 in section 4.1).  The result feeds
 * grpo_group_advantages.
 *  task_rewards [n_rollouts] f32, lengths and target_lengths [n_rollouts] i32, device, read;
 *  rewards_out [n_rollouts] f32, device, written (may be task_rewards itself).
 *  alpha finite.  n_rollouts == 0 does nothing.
 */
grpo_status grpo_total_rewards(const float *task_rewards, const int32_t *lengths,
                               const int32_t *target_lengths, int64_t n_rollouts, float alpha,
                               float *rewards_out, void *stream);

/*
 * Online data filtering of section 3.3: a group whose completions all received the same
 * reward has zero advantages and carries no training signal; the trainer keeps sampling
 * until it has a batch of groups that do.  This call finds them.
 *  rewards, n_rollouts, group_offsets | NULL, n_groups, group_size: as in
 *               grpo_group_advantages (invalid offsets are clamped on the device).
 *  keep_out        [n_groups] u8, device, written: 1 iff the rewards of the group are
 *                  not all equal (exact fp32 comparison); 0 for an empty group.
 *  kept_groups_out [n_groups] i32, device, written: indices of the kept groups in
 *                  increasing order, then -1.
 *  n_kept_out      [1] i32, device, written: how many groups are kept.
 *  rollout_keep_out[n_rollouts] u8, device, written, or NULL: the group's flag per rollout
 *                  (rollouts no group owns are left untouched).
 * n_groups == 0 writes n_kept_out = 0.
 */
grpo_status grpo_filter_groups(const float *rewards, int64_t n_rollouts, const int32_t *group_offsets,
                               int64_t n_groups, int64_t group_size, uint8_t *keep_out,
                               int32_t *kept_groups_out, int32_t *n_kept_out,
                               uint8_t *rollout_keep_out, void *stream);

/*
 * Packed (variable-length) batches (section 4.1, sequence packing: samples are collated
 * along the sequence dimension instead of being padded).  The response tokens of rollout
 * i are the rows [cu_seqlens[i], cu_seqlens[i+1]) of the batch.  Writes per row
 *   rollout_of_token_out[t] = i            (-1 for rows no rollout owns), as
 *                             grpo_group_advantages wants it, and
 *   weights_out[t] = 1 (sample_level = 0) or 1/|o_i| (sample_level != 0), the 1/|o_i| of
 *                    the objective as printed in section 3.4; 0 for rows no rollout owns,
 * ready to be passed as token_weights to grpo_loss_aux_fwd_bwd.
 *  cu_seqlens [n_rollouts+1] i64, device, read; expected non-decreasing within
 *             [0, n_tokens]; other values are clamped on the device (no out-of-bounds
 *             access, affected rows unspecified).
 *  weights_out [n_tokens] f32 and rollout_of_token_out [n_tokens] i32, device, written;
 *             either may be NULL, not both.
 */
grpo_status grpo_packed_layout(const int64_t *cu_seqlens, int64_t n_rollouts, int64_t n_tokens,
                               int sample_level, float *weights_out, int32_t *rollout_of_token_out,
                               void *stream);

/*
 * Per-token log-probabilities of the sampled tokens,
 *     logprobs_out[t] = log softmax(logits[t, :] / temperature)[tokens[t]],
 * i.e. log pi_theta(o_{i,t} | q, o_{i,<t}) of section 3.4.  This is how the trainer
 * obtains the old-policy log-probs at the start of an optimisation step
 * (section 4.1: recomputed with the policy weights rather than taken from the
 * inference workers).  One streaming read of the logits.
 *
 *  logits      [n_tokens, vocab] row-major, device, read; row t starts
 *              row_stride ELEMENTS after row t-1 (row_stride >= vocab).  The base
 *              pointer and the row pitch in bytes must be multiples of 16.
 *  tokens      [n_tokens] i64, device, read.
 *  mask        [n_tokens] u8 (0 or non-zero), device, read, or NULL = all ones.
 *              Rows with mask 0 give logprobs_out = 0 and none of their inputs
 *              (logits, token) is read.
 *  logprobs_out[n_tokens] f32, device, written.
 *  workspace   device, optional (NULL allowed): at least grpo_workspace_bytes(0) bytes,
 *              256-byte aligned,
 *              contents ignored on entry.  With it rows are handed to workgroups
 *              through a queue, which keeps the GPU evenly loaded when many rows are
 *              masked; without it rows are assigned in a fixed strided pattern.  The
 *              results are identical either way.
 * A token id outside [0, vocab) at an unmasked row gives logprobs_out = NaN there.
 * n_tokens == 0 is legal and does nothing.
 */
grpo_status grpo_logprobs_fwd(const void *logits, grpo_dtype dtype, int64_t n_tokens,
                              int64_t vocab, int64_t row_stride, const int64_t *tokens,
                              const uint8_t *mask, float temperature, float *logprobs_out,
                              void *workspace, size_t workspace_bytes, void *stream);

/*
 * Objective forward and fused backward (section 3.4 objective with delta,
 * token-level normalisation of section 4.1; see the top of this file).
 *
 *  logits, dtype, n_tokens, vocab, row_stride, tokens, mask: as above.
 *  old_logprobs [n_tokens] f32, device, read: l_old_t.
 *  advantages   [n_tokens] f32, device, read: A_t per token.
 *  eps_low in [0, 1], eps_high >= 0, delta > 1 + eps_high (section 3.4 asks for
 *               delta above 1 + eps), temperature > 0.
 *  denom        D.  denom > 0: used as given (a caller that splits a batch over
 *               micro-batches or GPUs passes the global token count).  denom <= 0:
 *               D = M = number of rows with mask 1 in this call; if that is 0 the
 *               loss and all gradients are 0.
 *  grad_scale   upstream gradient dL/dloss; multiplies grad_logits only.
 *  loss_out     [1] f32, device, written: -(1/D) sum_t m_t J_t.
 *  logprobs_out [n_tokens] f32, device, written, or NULL: l_t (0 at masked rows).
 *  counts_out   [5] i64, device, written, or NULL: see GRPO_COUNT_*; counted over
 *               rows with mask 1.  Clip fractions are counts / M.
 *  grad_logits  [n_tokens, vocab] same dtype and row_stride as logits, device,
 *               written:  grad_scale * dloss/dlogits
 *                 = c_t / T * (1[j = y_t] - softmax(z_t / T)_j),
 *               c_t = -grad_scale * m_t * (dJ_t/dl_t) / D,
 *               dJ_t/dl_t = r_t A_t where the objective is not clipped, else 0
 *               (a ratio exactly on a boundary counts as not clipped).
 *               Rows with c_t = 0 (masked, clipped, delta-capped, A_t = 0) are
 *               zero-filled.  bf16 gradients are rounded to nearest even.  May be
 *               the same buffer as logits (in-place); no other aliasing is allowed.
 *               Padding elements [vocab, row_stride) are never read or written.
 *  workspace    device, >= grpo_workspace_bytes(n_tokens) bytes, 256-byte aligned;
 *               contents on entry are ignored; on return it holds a sticky error
 *               word readable with grpo_workspace_error.
 * A token id outside [0, vocab) at an unmasked row makes that row behave as a
 * masked row (it still counts towards M) and sets the error word.
 * The loss is reduced in fp64 in a fixed order: results are bitwise reproducible.
 * n_tokens == 0 is legal: loss 0, counts 0.
 */
grpo_status grpo_loss_fwd_bwd(const void *logits, grpo_dtype dtype, int64_t n_tokens,
                              int64_t vocab, int64_t row_stride, const int64_t *tokens,
                              const float *old_logprobs, const float *advantages,
                              const uint8_t *mask, float eps_low, float eps_high,
                              float delta, float temperature, double denom,
                              float grad_scale, float *loss_out, float *logprobs_out,
                              int64_t *counts_out, void *grad_logits, void *workspace,
                              size_t workspace_bytes, void *stream);

/*
 * grpo_loss_fwd_bwd for callers that cannot allocate device memory or size a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same computation, same kernels and bit-identical outputs, but the per-row scratch
 * (objective terms, indicator bits, row queue, denominator) lives in an array built into
 * the library's device image instead of a caller-supplied workspace, so the call takes
 * no workspace and neither it nor anything it calls allocates or frees memory.
 *
 *  All arguments as in grpo_loss_fwd_bwd, without workspace / workspace_bytes, plus
 *  error_out    [1] i32, device, written, or NULL: the sticky data-error word that
 *               grpo_workspace_error reads for the workspace variant (0 = none, bit 0 =
 *               an unmasked row had a token id outside [0, vocab)).
 *  Limit:       n_tokens <= GRPO_NOALLOC_MAX_TOKENS, else GRPO_ERR_CAPACITY (nothing is
 *               launched).  The array takes about 8.5 MiB of every GPU the library is
 *               used on, for the life of the process.
 *  Concurrency: all calls on one GPU share that GPU's array (each GPU has its own).  A
 *               call clears what it needs at its start; two calls that overlap in time
 *               on the same GPU (different streams, or host threads) race and give
 *               undefined results.  Calls on one stream, or otherwise ordered, are fine.
 *  The address of the array is looked up once per device, on the first call made with
 *  that device current (hipGetSymbolAddress: a query, not an allocation); a failure of
 *  that lookup returns GRPO_ERR_HIP.  A caller that captures the call into a graph makes
 *  one call on that device before the capture begins, so that the lookup is not part of it.
 */
#define GRPO_NOALLOC_MAX_TOKENS 524288
grpo_status grpo_loss_fwd_bwd_noalloc(const void *logits, grpo_dtype dtype, int64_t n_tokens,
                                      int64_t vocab, int64_t row_stride, const int64_t *tokens,
                                      const float *old_logprobs, const float *advantages,
                                      const uint8_t *mask, float eps_low, float eps_high,
                                      float delta, float temperature, double denom,
                                      float grad_scale, float *loss_out, float *logprobs_out,
                                      int64_t *counts_out, void *grad_logits, int32_t *error_out,
                                      void *stream);

/*
 * The same objective with the trainer's two auxiliary terms fused into the same pass
 * over the logits (section 2.1.1: GRPO "along with auxiliary KL and entropy losses";
 * section 4.1: KL coefficient 0.001, entropy coefficient 1e-4).  The paper prints
 * neither estimator; this library uses
 *   kl_t = exp(d_t) - d_t - 1,  d_t = ref_logprobs[t] - l_t    (sampled-token estimator
 *          of KL(pi_theta || pi_ref), the one of the GRPO paper; >= 0),
 *   H_t  = - sum_j p_j log p_j,  p = softmax(z_t / T)           (entropy, in nats),
 *   total = -(1/D) sum m J  +  kl_coef (1/D) sum m kl  -  entropy_coef (1/D) sum m H
 * (the entropy enters as a bonus; pass a negative coefficient to penalise it).
 *
 * Arguments as grpo_loss_fwd_bwd, plus
 *  ref_logprobs [n_tokens] f32, device, read: log pi_ref(y_t); may be NULL iff
 *               kl_coef == 0.
 *  token_weights [n_tokens] f32, device, read, or NULL (= all ones): omega_t multiplies
 *               row t in all three sums, -(1/D) sum m omega J etc.  omega = 1 with
 *               D = M is the token-level loss of section 4.1; omega_t = 1/|o_i| with
 *               denom = number of rollouts is the sample-level normalisation the
 *               objective is printed with in section 3.4 (grpo_packed_layout writes
 *               those weights).  A row with omega_t = 0 is treated exactly like a
 *               masked row (never read, zero gradient, not counted in M).
 *  kl_coef, entropy_coef: finite.
 *  loss_out     [4] f32, device, written: total, policy part -(1/D) sum m omega J,
 *               (1/D) sum m omega kl, (1/D) sum m omega H.
 *  entropy_out  [n_tokens] f32, device, written, or NULL: H_t (0 at masked rows).
 *  grad_logits  grad_scale * dtotal/dlogits
 *                 = c_t/T (1[j = y_t] - p_j) + b_t/T p_j (log p_j + H_t),
 *               c_t = grad_scale m_t omega_t (-dJ_t/dl_t + kl_coef (1 - exp(d_t))) / D,
 *               b_t = grad_scale m_t omega_t entropy_coef / D.
 *               Rows with c_t = 0 and b_t = 0 are zero-filled.
 * With kl_coef = 0 and entropy_coef = 0 the loss and the gradient equal those of
 * grpo_loss_fwd_bwd.  Entropies below about 1e-7 nats are at the resolution of the
 * fp32 normaliser and are reported with that absolute accuracy.
 */
grpo_status grpo_loss_aux_fwd_bwd(const void *logits, grpo_dtype dtype, int64_t n_tokens,
                                  int64_t vocab, int64_t row_stride, const int64_t *tokens,
                                  const float *old_logprobs, const float *ref_logprobs,
                                  const float *advantages, const uint8_t *mask,
                                  const float *token_weights, float eps_low, float eps_high,
                                  float delta, float temperature, float kl_coef,
                                  float entropy_coef, double denom, float grad_scale,
                                  float *loss_out, float *logprobs_out, float *entropy_out,
                                  int64_t *counts_out, void *grad_logits, void *workspace,
                                  size_t workspace_bytes, void *stream);

/*
 * Reads the sticky error word the last grpo_loss_fwd_bwd left in `workspace`:
 * waits for `stream`, copies one int to *flag_out (HOST pointer).  0 = no data
 * error, bit 0 = some unmasked row had a token id outside [0, vocab).
 */
grpo_status grpo_workspace_error(const void *workspace, int32_t *flag_out, void *stream);

/* ------------------------------------------------------------------------- *
 * Language-model head fused with the objective.
 *
 * The policy pi_theta of section 3.4 is the softmax of the logits z_t = W h_t that
 * the model's last linear layer (no bias) computes from the final hidden state
 * h_t of each token position.  These two calls take h and W instead of z: the
 * logits are formed tile by tile on the matrix cores and reduced from the fp32
 * accumulators, so log pi(y) is not affected by a bf16 rounding of z.
 *
 *  hidden   [n_tokens, d_model] bf16, device, read; row pitch hidden_stride
 *           elements (>= d_model), base and pitch 16-byte aligned.
 *  weight   [vocab, d_model] bf16, device, read; row v holds the d_model weights of
 *           vocabulary entry v; row pitch weight_stride, aligned like hidden.
 *  d_model  a multiple of 64 (one step of the contraction), at most 2^20.  vocab in [1, 2^28].
 *  tokens, mask, temperature, old_logprobs, advantages, eps_low, eps_high, delta,
 *  denom, grad_scale, loss_out, logprobs_out, counts_out: as in
 *           grpo_logprobs_fwd / grpo_loss_fwd_bwd.
 *  workspace  device, 256-byte aligned.  Forward only: at least
 *           grpo_lmhead_workspace_bytes(n_tokens, vocab, d_model, 0) bytes; it holds a
 *           compacted copy of the hidden states of the rows that take part and 8 bytes
 *           per token and 256 vocabulary entries.  With the backward the rows that take
 *           part are worked through in chunks, and per chunk row the workspace also holds
 *           the logits in fp32 and their gradient in bf16, 6 bytes per chunk row and
 *           vocabulary entry, next to a transposed copy of the chunk's hidden states (W is
 *           never copied): its size follows the chunk, not
 *           the number of tokens.  grpo_lmhead_workspace_bytes(.., 1) is the size for
 *           the default chunk of 10240 rows (about 9.6 GB at vocab 152064, d_model 5120,
 *           for any n_tokens >= 10240); grpo_lmhead_workspace_bytes_for_chunk gives the
 *           size for another chunk.  The call uses the largest chunk (a multiple of 256
 *           rows, at most n_tokens rounded up to 256) that fits into workspace_bytes:
 *           a caller short of memory brings less, down to a chunk of 256 rows, a caller
 *           with memory to spare brings more and gets fewer, larger chunks.  Less than
 *           the 256-row size is GRPO_ERR_WORKSPACE.  Contents on entry are
 *           ignored; the error word is read with grpo_workspace_error.
 *  Results do not depend on the chunk except for dL/dW, whose sum over the rows is taken
 *  chunk by chunk in fp32 (the same as accumulating micro-batches).
 *  With the backward vocab may not exceed 8388544 (byte offsets inside an operand tile of
 *  the two gradient products are 32-bit): larger values are GRPO_ERR_SHAPE.
 * Rows with mask 0 cost no matrix work, and neither do, in the backward, rows whose
 * objective has no gradient (clipped, delta-capped, zero advantage): the rows that
 * take part are compacted on the device first.
 * Errors as for grpo_loss_fwd_bwd; additionally GRPO_ERR_SHAPE when d_model is not
 * a multiple of 64 or a pitch is smaller than d_model.  All work is enqueued on
 * `stream`; nothing is allocated.
 * ------------------------------------------------------------------------- */

/* Pure host functions; 0 for invalid sizes.  The second: the backward's workspace for chunks of
 * chunk_rows rows (rounded up to a multiple of 256, at most n_tokens rounded up likewise). */
size_t grpo_lmhead_workspace_bytes(int64_t n_tokens, int64_t vocab, int64_t d_model, int with_backward);
size_t grpo_lmhead_workspace_bytes_for_chunk(int64_t n_tokens, int64_t vocab, int64_t d_model,
                                             int64_t chunk_rows);

/*
 * logprobs_out[t] = log softmax(W h_t / T)[y_t] for rows with mask 1 (0 at masked
 * rows, NaN where the token id is outside [0, vocab)): what the trainer recomputes
 * as the old policy's log-probs before its optimiser steps (section 4.1).  The
 * logits never reach memory.
 */
grpo_status grpo_lmhead_logprobs_fwd(const void *hidden, int64_t hidden_stride, const void *weight,
                                     int64_t weight_stride, int64_t n_tokens, int64_t vocab,
                                     int64_t d_model, const int64_t *tokens, const uint8_t *mask,
                                     float temperature, float *logprobs_out, void *workspace,
                                     size_t workspace_bytes, void *stream);

/*
 * The objective of grpo_loss_fwd_bwd on z = h W^T and its gradient with respect to
 * h and W (chain rule through the head: dL/dh_t = sum_v G[t][v] W[v][:],
 * dL/dW[v][:] = sum_t G[t][v] h_t, with G = grad_scale * dloss/dz as defined for
 * grpo_loss_fwd_bwd).
 *  grad_hidden  [n_tokens, d_model] bf16, device, written (zero rows where the
 *               objective has no gradient); row pitch grad_hidden_stride elements.
 *  grad_weight  [vocab, d_model] f32, device; row pitch grad_weight_stride elements.
 *               accumulate_grad_weight == 0: overwritten; != 0: added to, which is
 *               how a trainer sums micro-batches (pass the global token count as
 *               denom in that case).
 * G is rounded to bf16 (8 significant bits: relative error at most 2^-8 per element)
 * before the two products, which accumulate in fp32.
 */
grpo_status grpo_lmhead_loss_fwd_bwd(const void *hidden, int64_t hidden_stride, const void *weight,
                                     int64_t weight_stride, int64_t n_tokens, int64_t vocab,
                                     int64_t d_model, const int64_t *tokens, const float *old_logprobs,
                                     const float *advantages, const uint8_t *mask, float eps_low,
                                     float eps_high, float delta, float temperature, double denom,
                                     float grad_scale, float *loss_out, float *logprobs_out,
                                     int64_t *counts_out, void *grad_hidden, int64_t grad_hidden_stride,
                                     float *grad_weight, int64_t grad_weight_stride,
                                     int accumulate_grad_weight, void *workspace, size_t workspace_bytes,
                                     void *stream);

/*
 * The total objective of grpo_loss_aux_fwd_bwd (policy term of section 3.4, sampled-token
 * KL against a reference policy and entropy bonus with the coefficients of section 4.1,
 * per-token weights for packed batches and the sample-level normalisation) on z = h W^T,
 * and its gradient with respect to h and W.  Arguments as grpo_lmhead_loss_fwd_bwd, plus
 * ref_logprobs, token_weights, kl_coef, entropy_coef, entropy_out and the four-entry
 * loss_out exactly as documented for grpo_loss_aux_fwd_bwd; G = grad_scale * dtotal/dz as
 * defined there, rounded to bf16 before the two products.  A row with weight 0 is treated
 * like a masked row and costs no matrix work.  With entropy_coef != 0 every row that takes
 * part has a gradient.  The same workspace rules as grpo_lmhead_loss_fwd_bwd.
 */
grpo_status grpo_lmhead_loss_aux_fwd_bwd(const void *hidden, int64_t hidden_stride, const void *weight,
                                         int64_t weight_stride, int64_t n_tokens, int64_t vocab,
                                         int64_t d_model, const int64_t *tokens, const float *old_logprobs,
                                         const float *ref_logprobs, const float *advantages,
                                         const uint8_t *mask, const float *token_weights, float eps_low,
                                         float eps_high, float delta, float temperature, float kl_coef,
                                         float entropy_coef, double denom, float grad_scale, float *loss_out,
                                         float *logprobs_out, float *entropy_out, int64_t *counts_out,
                                         void *grad_hidden, int64_t grad_hidden_stride, float *grad_weight,
                                         int64_t grad_weight_stride, int accumulate_grad_weight,
                                         void *workspace, size_t workspace_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* GRPO_H */
