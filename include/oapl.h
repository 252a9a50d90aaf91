/*
 * oapl.h - C ABI of the OAPL trainer-step loss head for AMD MI355X (gfx950).
 *
 * The library scores sampled rollouts under the current policy pi and
 * evaluates the OAPL objective on them ("LLMs Can Learn to Reason Via
 * Off-Policy RL", Sec. 3.1), with its backward pass to the final hidden states
 * and the LM-head weights.
 *
 * Notation (Sec. 3.1): x is a prompt, y_1..y_G the group of rollouts sampled
 * for it from the lagged inference policy pi_vllm, r(x, y) the reward, beta
 * the regularisation constant.
 *
 *   T         packed number of scored tokens over all rollouts
 *   d, V      hidden size and vocabulary size
 *   H [T, d]  final hidden states, row-major; row t predicts token y_t (the
 *             caller has applied the next-token shift and dropped prompt and
 *             padding positions)
 *   W [V, d]  LM-head weights, row-major, no bias; logits z_t = W h_t
 *
 * General rules for every entry point
 *   - Every pointer is DEVICE memory on the current HIP device unless the
 *     comment says "host".  The caller owns all buffers; the library never
 *     allocates, frees or keeps a pointer after the call returns.
 *   - All work is enqueued on `stream` (a hipStream_t passed as void*, NULL =
 *     the default stream).  No entry point synchronises with the host except
 *     oapl_read_device_status.
 *   - Inputs are never modified; outputs are fully overwritten.
 *   - `workspace` must hold at least oapl_workspace_bytes(...) bytes for the
 *     same sizes, aligned to 256 bytes (the loss calls also accept less or more,
 *     see oapl_workspace_bytes_for).  Its contents are scratch.  Two calls
 *     may run concurrently only with distinct workspaces.  The library keeps
 *     no state between calls: there are no process-wide switches.
 *   - The return value is an oapl_status.  Errors the host can see (null
 *     pointers, bad sizes, bad beta, short workspace) return before anything
 *     is launched.  Errors in device data (token id outside [0, V), group id
 *     outside [0, n_groups), empty group, offsets not starting at 0 / not
 *     ending at T / decreasing) cannot be seen without a sync: the kernels
 *     record the first such status in the workspace, never read or write out
 *     of bounds because of it, and write NaN to the affected outputs (the
 *     log-prob of a bad token; the loss for bad offsets or groups).
 *     oapl_read_device_status fetches the record.
 */
#ifndef OAPL_H
#define OAPL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  OAPL_OK = 0,
  OAPL_ERR_NULL = 1,        /* a required pointer is NULL */
  OAPL_ERR_SHAPE = 2,       /* a size is non-positive or unsupported */
  OAPL_ERR_DTYPE = 3,       /* dtype is not an oapl_dtype */
  OAPL_ERR_OFFSETS = 4,     /* device: seq_offsets malformed */
  OAPL_ERR_GROUP = 5,       /* device: group id out of range or empty group */
  OAPL_ERR_BETA = 6,        /* beta (or loss_scale) not finite or beta <= 0 */
  OAPL_ERR_WORKSPACE = 7,   /* workspace NULL, misaligned or too small */
  OAPL_ERR_HIP = 8,         /* a HIP launch or runtime call failed */
  OAPL_ERR_TOKEN_RANGE = 9, /* device: sampled token outside [0, V) */
  OAPL_ERR_SCRATCH_LIMIT = 10 /* oapl_loss_fwd_bwd_noalloc: the sizes need more than the static scratch */
} oapl_status;

typedef enum {
  OAPL_F32 = 0,  /* H, W, dH are float; plain fp32 FMA arithmetic */
  OAPL_BF16 = 1  /* H, W, dH are bfloat16 (raw uint16 bit patterns); MFMA with fp32 accumulation */
} oapl_dtype;

/* Human-readable name of a status (host pointer to a static string). */
const char* oapl_status_string(int32_t status);

/*
 * Shape limits: T >= 0 (T == 0 is legal and yields loss = sum of squared
 * advantages), 1 <= d <= 2^21, 1 <= V <= 2^21, 0 <= n_seq, 1 <= n_groups,
 * n_seq * n_groups <= 2^32 (each prompt's wavefront walks all rollouts to find
 * its own).  OAPL_BF16 additionally needs d to be a multiple of 8 (16-byte
 * rows) and T <= 65535 * 256; OAPL_F32 needs T <= 65535 * 64.  Anything else
 * is OAPL_ERR_SHAPE.
 */

/* Options of the loss entry points that take a `flags` argument (bit set). */
typedef enum {
  OAPL_FLAG_TWO_PASS = 1  /* never try the single sweep: log-sum-exp pass first, then soft-max recompute per panel */
} oapl_flags;

/* Bytes of workspace the two calls below need for these sizes (host call, no
 * GPU work).  with_backward = 0 sizes it for oapl_logprob_fwd and for
 * oapl_loss_fwd_bwd with dH = dW = NULL.  Returns 0 for invalid sizes. */
size_t oapl_workspace_bytes(int64_t T, int32_t d, int32_t V, int32_t n_seq,
                            int32_t n_groups, int32_t dtype, int32_t with_backward);

/*
 * The workspace is the memory budget of a loss call.  The gradients are
 * produced panel by panel (a panel = a range of token rows whose soft-max
 * values are held, bf16, until the dH and dW contractions have consumed them),
 * and nearly all of the workspace is panel storage: panel rows x V x 4 bytes
 * per panel buffer.  Two things can be chosen:
 *   - the panel size.  oapl_workspace_bytes uses the library's own (at most
 *     12288 rows for OAPL_BF16 -- the fastest measured -- and 4096 for
 *     OAPL_F32); max_panel_rows caps it lower (rounded down to whole 384-row
 *     tiles for OAPL_BF16, at least one tile; <= 0 or larger = the library's);
 *   - the number of panel buffers (OAPL_BF16).  The single sweep finishes a
 *     panel's gradients only when every rollout touching it is scored, so it
 *     keeps a ring of panels: 1 + ceil(longest rollout / panel rows) buffers
 *     serve rollouts of that length.  oapl_workspace_bytes sizes two buffers
 *     (rollouts up to one panel); pass max_rollout_len to size more (<= 0 =
 *     two).  More than two buffers exist only at the library's own panel size
 *     (a plan with smaller panels always has two: the loss call sees only a
 *     byte count, and prefers larger panels to more buffers).  Longer rollouts
 *     than the buffers serve are not an error: the call then takes the
 *     two-pass schedule (decided on the device).
 * Returns the bytes needed, and the panel rows / buffers of that plan through
 * the host pointers (each may be NULL).  Returns 0 for invalid sizes.
 *
 * A loss call derives its plan from workspace_bytes alone: the library's panel
 * size if two buffers of it fit, else the largest panel that does
 * (OAPL_ERR_WORKSPACE if not even a one-tile panel fits); then as many buffers
 * as fit.  Results do not depend on the plan beyond rounding (summation order
 * of dW over panels).
 */
size_t oapl_workspace_bytes_for(int64_t T, int32_t d, int32_t V, int32_t n_seq,
                                int32_t n_groups, int32_t dtype, int32_t with_backward,
                                int64_t max_panel_rows, int64_t max_rollout_len,
                                int64_t* panel_rows_out, int32_t* panel_buffers_out);

/*
 * Per-token log-probability of the sampled token under pi (the ln pi(y_t | x,
 * y_<t) whose sum over a rollout is the ln pi(y_i | x) of Eq. 3; soft-max over
 * the full vocabulary at temperature 1, as the appendix's generation settings
 * imply):
 *
 *     lse_t      = ln sum_v exp(z_{t,v}),   z_{t,v} = sum_k H[t,k] W[v,k]
 *     logprob[t] = z_{t, tokens[t]} - lse_t          (<= 0)
 *
 * The T x V logits are produced tile by tile and reduced on the fly; they are
 * never stored.
 *
 * Optionally also the entropy of pi(. | x, y_<t), the quantity whose collapse
 * or stability the paper's training-dynamics discussion follows (Sec. 6.1):
 *
 *     entropy[t] = - sum_v p_{t,v} ln p_{t,v} = lse_t - sum_v p_{t,v} z_{t,v}
 *
 * accumulated in the same streaming pass (one more running sum per token).
 *
 *   tokens      [T] int32, each in [0, V)
 *   logprob_out [T] float
 *   lse_out     [T] float, or NULL if not wanted
 *   entropy_out [T] float, or NULL if not wanted (in [0, ln V])
 */
int32_t oapl_logprob_fwd(const void* H, const void* W, const int32_t* tokens,
                         int64_t T, int32_t d, int32_t V, int32_t dtype,
                         float* logprob_out, float* lse_out, float* entropy_out,
                         void* workspace, size_t workspace_bytes, void* stream);

/*
 * Sampling step of Alg. 1 ("sample a batch from pi_vllm") on the same fused
 * LM head, for harnesses that need rollouts' tokens without an inference
 * engine: one draw per row from softmax(z_t / temperature) (the appendix's
 * generation settings are temperature 1, top-p 1) by the Gumbel-max
 * construction,
 *
 *     tokens_out[t] = argmax_v ( z_{t,v} / temperature + g_{t,v} ),   ties to the smaller v,
 *     g_{t,v} = -ln(-ln u_{t,v}),  u = ((x >> 9) + 1/2) 2^-23,
 *     x = word (v mod 4) of Philox-4x32-10( counter = (v / 4, t mod 2^32, t / 2^32, 0),
 *                                           key = (seed mod 2^32, seed / 2^32) ),
 *
 * so a draw depends only on (seed, t, v) and can be reproduced anywhere.  The
 * logits are never stored.
 *   temperature > 0 and finite (else OAPL_ERR_BETA)
 *   tokens_out [T] int32
 *   score_out  [T] float or NULL: the winning perturbed logit
 * Workspace: oapl_workspace_bytes(T, d, V, 0, 1, dtype, 0).
 */
int32_t oapl_sample_tokens(const void* H, const void* W, int64_t T, int32_t d, int32_t V,
                           int32_t dtype, float temperature, uint64_t seed,
                           int32_t* tokens_out, float* score_out,
                           void* workspace, size_t workspace_bytes, void* stream);

/*
 * OAPL objective and gradients on one packed batch (Sec. 3.1).
 *
 *   Delta_s = sum_{t in rollout s} (logprob[t] - logq[t])     ln pi(y|x)/pi_vllm(y|x), no length normalisation
 *   V*_g    = beta ln( (1/G_g) sum_{s in group g} exp(r_s / beta) )                    Eq. 2
 *   delta_s = beta Delta_s - (r_s - V*_{g(s)})
 *   loss    = loss_scale * sum_s delta_s^2                                             Eq. 3
 *   dH, dW  = d loss / d H, d loss / d W; V* and logq are constants (V* depends
 *             on rewards only), so with c_t = loss_scale * 2 beta delta_{s(t)}
 *             and p_t = softmax(z_t):
 *               dH[t,:] = c_t (W[y_t,:] - sum_v p_{t,v} W[v,:])
 *               dW[v,:] = sum_t c_t (1[v = y_t] - p_{t,v}) H[t,:]
 *
 * How the gradients are scheduled (bf16): the logits are visited ONCE.  Panels of
 * token rows (12288 by default, see oapl_workspace_bytes_for) are swept with the
 * soft-max written unnormalised (bf16, against a per-row reference exponent
 * fixed before the sweep), their row sums give lse and the log-probs, and the
 * dH / dW contractions consume a panel as soon as every rollout touching it is
 * scored.  That needs (a) no rollout longer than the panel buffers serve (one
 * panel with the default workspace) and (b) every row's largest logit within
 * about 97 nats of the largest among its first 256 vocabulary entries and the
 * sampled token.  Both are checked on the device; if either fails, the same
 * call recomputes everything in two passes (log-sum-exp first, then soft-max
 * recompute per panel), in stream order, with no host involvement.  The
 * results of the two schedules agree to rounding.  fp32 and batches of fewer
 * than 64 tokens always run two passes (nothing is gained by a sweep there).
 *
 * The same beta is used in Eq. 2 and Eq. 3, as the method section writes
 * them.  loss_scale = 1 gives the paper's plain sum; it exists so a caller can
 * average over a batch.
 *
 *   logq         [T] float, inference-policy log-probs of the same tokens
 *   seq_offsets  [n_seq + 1] int64; rollout s owns tokens [off[s], off[s+1]);
 *                off[0] = 0, off[n_seq] = T, non-decreasing (empty rollouts legal)
 *   rewards      [n_seq] float (the paper's are binary; any finite value works)
 *   group_ids    [n_seq] int32 in [0, n_groups), any order; G_g is the number
 *                of rollouts carrying id g and must be >= 1 for every g
 *   loss_out         [1] float
 *   logprob_out      [T] float or NULL
 *   seq_logratio_out [n_seq] float or NULL   (Delta_s)
 *   vstar_out        [n_groups] float or NULL
 *   dH  [T, d] in `dtype`, dW [V, d] float (overwritten, not accumulated);
 *       pass both NULL to get the loss only.
 */
int32_t oapl_loss_fwd_bwd(const void* H, const void* W, const int32_t* tokens,
                          const float* logq, const int64_t* seq_offsets,
                          const float* rewards, const int32_t* group_ids,
                          int64_t T, int32_t d, int32_t V, int32_t n_seq, int32_t n_groups,
                          int32_t dtype, float beta, float loss_scale,
                          float* loss_out, float* logprob_out, float* seq_logratio_out,
                          float* vstar_out, void* dH, float* dW,
                          void* workspace, size_t workspace_bytes, void* stream);

/*
 * Same as oapl_loss_fwd_bwd with separate constants, as the experimental
 * section (Sec. 5) uses: beta_value in Eq. 2 and beta_loss in Eq. 3, and with
 * per-call options: flags is 0 or a set of oapl_flags (unknown bits are
 * OAPL_ERR_SHAPE).
 */
int32_t oapl_loss_fwd_bwd_two_beta(const void* H, const void* W, const int32_t* tokens,
                                   const float* logq, const int64_t* seq_offsets,
                                   const float* rewards, const int32_t* group_ids,
                                   int64_t T, int32_t d, int32_t V, int32_t n_seq, int32_t n_groups,
                                   int32_t dtype, float beta_value, float beta_loss, float loss_scale,
                                   uint32_t flags, float* loss_out, float* logprob_out, float* seq_logratio_out,
                                   float* vstar_out, void* dH, float* dW,
                                   void* workspace, size_t workspace_bytes, void* stream);

/*
 * oapl_loss_fwd_bwd for callers that cannot allocate device memory at all (code
 * under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc) and so cannot bring a workspace either: the same computation with
 * the same kernels, its scratch taken from an array the library itself holds in
 * device memory (64 MiB on every GPU the library runs on, from the first call
 * on that GPU until the process ends).  The call allocates and frees nothing.
 *   - Sizes whose plan (with the largest backward panel that fits) needs more
 *     than 64 MiB return OAPL_ERR_SCRATCH_LIMIT before anything is launched;
 *     small heads and batches fit (d = 256, V = 1544, T = 1000 needs about 12 MiB).
 *   - All calls on one GPU share that GPU's array, which keeps the last call's
 *     contents; the call clears what it needs cleared.  Calls that overlap on
 *     one GPU (different streams or host threads) race: serialise them.
 *   - The first call on a GPU resolves the array's device address (a HIP
 *     runtime call that may load the code object): make that call outside any
 *     graph capture.
 *   - The device-side status record lives in the library's scratch and cannot
 *     be read back; errors in device data show as NaN in the affected outputs.
 * Arguments as for oapl_loss_fwd_bwd, without workspace and workspace_bytes.
 */
int32_t oapl_loss_fwd_bwd_noalloc(const void* H, const void* W, const int32_t* tokens,
                                  const float* logq, const int64_t* seq_offsets,
                                  const float* rewards, const int32_t* group_ids,
                                  int64_t T, int32_t d, int32_t V, int32_t n_seq, int32_t n_groups,
                                  int32_t dtype, float beta, float loss_scale,
                                  float* loss_out, float* logprob_out, float* seq_logratio_out,
                                  float* vstar_out, void* dH, float* dW, void* stream);

/*
 * The paper's baseline on the same fused head: GRPO with token-level importance
 * sampling (Sec. 2, the displayed GRPO objective; appendix: clip ratio 0.2,
 * length normalisation on).  With A_s the group-normalised advantage of rollout s,
 *
 *   A_s     = (r_s - mean_g r) / (std_g r + adv_eps)          population std over the prompt's group
 *   r_t     = pi(y_t) / pi_old(y_t) = exp(logprob[t] - logp_old[t])
 *   IS_t    = pi_old(y_t) / pi_vllm(y_t) = exp(logp_old[t] - logq[t])
 *   loss    = - loss_scale * sum_g (1/G_g) sum_{s in g} (1/|y_s|) sum_{t in s}
 *                 IS_t min( r_t A_s, clip(r_t, 1 - clip_eps, 1 + clip_eps) A_s )
 *
 * (the objective is maximised in the paper; the loss is its negative; empty
 * rollouts contribute 0), and dH, dW = d loss / dH, d loss / dW with pi_old,
 * pi_vllm and A constants: tokens on a clipped branch get zero gradient.  The
 * paper does not spell out the normalisation of A: population standard
 * deviation plus adv_eps is this library's reading.
 *   logp_old [T] float: log-probs of the tokens under the previous trainer policy
 *   0 <= clip_eps < 1, adv_eps >= 0, all finite (else OAPL_ERR_BETA)
 *   adv_out [n_seq] float or NULL; flags as for oapl_loss_fwd_bwd_two_beta; other
 *   arguments as for oapl_loss_fwd_bwd.
 */
int32_t oapl_grpo_loss_fwd_bwd(const void* H, const void* W, const int32_t* tokens,
                               const float* logq, const float* logp_old, const int64_t* seq_offsets,
                               const float* rewards, const int32_t* group_ids,
                               int64_t T, int32_t d, int32_t V, int32_t n_seq, int32_t n_groups,
                               int32_t dtype, float clip_eps, float adv_eps, float loss_scale,
                               uint32_t flags, float* loss_out, float* logprob_out, float* adv_out,
                               void* dH, float* dW,
                               void* workspace, size_t workspace_bytes, void* stream);

/*
 * Per-rollout sums over a packed stream (the reduction behind Delta_s in
 * Eq. 3), exposed on its own: out[s] = sum_{t in [off[s], off[s+1])} x[t],
 * accumulated in double in a fixed order (bit-reproducible).
 *   x [off[n_seq]] float, seq_offsets [n_seq + 1] int64 (must be non-decreasing),
 *   out [n_seq] double.  Needs no workspace.
 */
int32_t oapl_segmented_sum_f32(const float* x, const int64_t* seq_offsets, int32_t n_seq,
                               double* out, void* stream);

/*
 * Waits for `stream`, then copies the device-side status recorded in
 * `workspace` by the last call that used it into *status_out (host pointer).
 */
int32_t oapl_read_device_status(const void* workspace, void* stream, int32_t* status_out);

/*
 * Which schedule the last loss call on `workspace` ended up using: waits for
 * `stream`, then *two_pass_out (host pointer) = 1 if the device sent the call
 * down the two-pass path, 0 if the single sweep was valid (also 0 for calls
 * that never try the sweep: fp32, forward-only, empty, OAPL_FLAG_TWO_PASS).
 */
int32_t oapl_read_path_taken(const void* workspace, void* stream, int32_t* two_pass_out);

/*
 * Measurement aid, not part of the method.  The path's time is spent in the
 * dense bf16 kernels: 0 = LM-head contraction fused with the streaming
 * log-sum-exp (forward-only scoring, and pass one of the two-pass loss),
 * 1 = soft-max recompute producing the logit gradient (pass two of the two-pass loss),
 * 2 = the dH contraction, 3 = the dW contraction, 4 = the sampling kernel,
 * 5 = the single sweep (contraction + unnormalised soft-max panel + row sums).  After
 * oapl_timing_enable(1), every launch of these kernels is bracketed by a pair
 * of HIP events recorded on the launch stream; oapl_timing_read waits for the
 * recorded events of one kernel and returns the summed duration (milliseconds)
 * and the number of launches since the last enable call (host pointers).
 * oapl_timing_enable(0) switches recording off and drops the records.  Calls
 * made while recording must not overlap on different host threads' streams if
 * per-kernel attribution matters; the events themselves are stream-ordered.
 */
int32_t oapl_timing_enable(int32_t enable);
int32_t oapl_timing_read(int32_t kernel, double* total_ms, int64_t* launches);

#ifdef __cplusplus
}
#endif
#endif /* OAPL_H */
