/*
 * tppo.h -- C ABI of the MI355X (gfx950) per-token core of Truncated PPO.
 *
 * Four operations of one T-PPO training step (Algorithm 1, lines 6, 8, 9):
 *   tppo_select          token filter of Sec. 3.2 -> compact gather indices
 *   tppo_token_logprobs  log pi_theta(a_t|s_t) of the kept tokens (the quantity
 *                        in the ratio of Eq. (ppoloss)), LM head fused with
 *                        log-softmax and target gather; logits are never stored
 *   tppo_egae            Extended GAE advantages (Eq. (egae), Sec. 3.1) and
 *                        Monte-Carlo returns R_t (Sec. 2.4)
 *   tppo_ppo_losses      clipped surrogate (Eq. (ppoloss)) and clipped value
 *                        loss (Eqs. (valueclip), (valueloss)) over the policy /
 *                        value token sets of Sec. 3.2
 *
 * Conventions common to every entry point
 *   - Every array pointer is DEVICE memory owned by the caller, valid until the
 *     work enqueued by the call has finished.  The library allocates nothing and
 *     frees nothing.  The state it keeps: a process-wide call counter (each
 *     launch that lets workgroups exchange partial results tags them with its
 *     call number, which is why scratch memory needs no clearing between
 *     calls), and what it learns or sets once per device on first use -- the
 *     number of compute units, the large-LDS attribute of the
 *     tppo_token_logprobs* kernels, the address of tppo_egae_static's array.
 *     All of it is kept in atomics; calls from several threads are safe.  No
 *     environment variable is read.
 *   - The matrix-core kernels of tppo_token_logprobs* are scheduled for the
 *     whole MI355X (256 compute units in 8 XCDs).  On a device that reports
 *     another number of compute units (a partition of the chip) the bf16 path
 *     returns TPPO_ERR_LAUNCH instead of running with its workgroups taking
 *     turns.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     All work is enqueued asynchronously on it; no call synchronises with the
 *     host, which is why scalar results are written to device memory.
 *   - Scratch memory comes from the caller: `*_workspace_bytes` gives the size
 *     for the same size arguments; the workspace needs no initialisation and
 *     must be 256-byte aligned.  One workspace must not be shared by calls
 *     that may overlap in time.
 *   - Return value: 0 on success, a negative tppo_error otherwise.  On error
 *     nothing has been enqueued.  Errors the host cannot see (bad indices in
 *     device arrays) set bits of the optional device word `status` (may be
 *     NULL; the caller zeroes it) and the offending element is skipped.
 *   - Indices and offsets are int32, sizes int64; address arithmetic in the
 *     kernels is 64-bit.
 *
 * Batch layout (Sec. 2.1, Sec. 3.2).  B sequences packed back to back.
 * Sequence i owns packed positions cu_seqlens[i] .. cu_seqlens[i+1]-1: first
 * ctx_len[i] >= 1 context tokens (prompt and tokens generated in earlier
 * steps), then win_len[i] tokens generated in the current step.  done[i] = 1 if
 * it emitted end-of-sequence inside the window, 0 if it was cut at the window
 * length.  The "response-packed" domain numbers only window tokens: element
 * resp_off[i]+t is window token t of sequence i, n_resp = resp_off[B].
 */
#ifndef TPPO_H
#define TPPO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    TPPO_OK = 0,
    TPPO_ERR_NULL = -1,      /* a required pointer is NULL */
    TPPO_ERR_SIZE = -2,      /* negative, inconsistent or unsupported size */
    TPPO_ERR_PARAM = -3,     /* scalar out of range (gamma, lambda outside [0,1]; negative eps, xi, tail_drop) */
    TPPO_ERR_DTYPE = -4,     /* unknown tppo_dtype */
    TPPO_ERR_WORKSPACE = -5, /* workspace NULL, misaligned or too small */
    TPPO_ERR_LAUNCH = -6     /* the HIP runtime refused a launch, or the device is not one the kernel is scheduled for */
} tppo_error;

/* bits of the device status word */
enum {
    TPPO_STATUS_BAD_TARGET = 1,   /* a target id outside [0, V): its logp is NaN */
    TPPO_STATUS_BAD_LAYOUT = 2,   /* ctx_len < 1, negative window length, non-monotone offsets, or a plan that
                                     was built for another batch (nothing is computed then) */
    TPPO_STATUS_CAPACITY = 4,     /* more kept tokens than `capacity`: excess not written */
    TPPO_STATUS_BAD_ROW = 8,      /* a row index outside [0, n_rows): its logp is NaN */
    TPPO_STATUS_TIMEOUT = 16      /* an inter-workgroup wait gave up (results invalid) */
};

typedef enum { TPPO_F32 = 0, TPPO_BF16 = 1 } tppo_dtype;

/* Library version, for the binding's sanity check. */
int tppo_version(void);

/* ---------------------------------------------------------------------------
 * tppo_select -- token filter (Sec. 3.2; abstract: prompt and truncated tokens
 * are filtered out of the policy update).
 *
 * Policy tokens: every window token of every sequence, finished or not, except
 * the `tail_drop` latest tokens of an unfinished sequence:
 *   keep_len[i] = done[i] ? win_len[i] : max(win_len[i] - tail_drop, 0).
 * Value tokens: all window tokens of finished sequences.  Context tokens are in
 * neither set.  For kept token t of sequence i, in order of (i, t), at compact
 * index m = sel_off[i] + t:
 *   sel_rows[m]     = cu_seqlens[i] + ctx_len[i] + t - 1   (the state s_t that
 *                     predicts it: Sec. 2.1, s_t holds the tokens before t)
 *   sel_targets[m]  = input_ids[cu_seqlens[i] + ctx_len[i] + t]
 *   sel_resp_idx[m] = resp_off[i] + t
 *
 * in : cu_seqlens[B+1], ctx_len[B], done[B] int32; input_ids[n_tok] int32
 *      (may be NULL together with sel_targets).
 * out: resp_off[B+1], sel_off[B+1], keep_len[B] int32; sel_rows, sel_targets,
 *      sel_resp_idx: `capacity` int32 each (each may be NULL = not wanted;
 *      n_tok is always a sufficient capacity); counts[3] int64 =
 *      { M = sel_off[B], n_resp = resp_off[B], N_val = number of value tokens }.
 *      workspace: tppo_select_workspace_bytes(B, max(capacity, n_tok)) bytes; only
 *      needed (may be NULL otherwise) when one of the three index arrays is wanted.
 *      plan (optional, may be NULL): receives the work plan of this batch's
 *      response-packed domain (see tppo_plan_build), ready for tppo_egae* and
 *      the loss entry points; plan_bytes >= tppo_plan_bytes(n_tok, B), since the
 *      number of window tokens is not known to the host before the call.
 * Errors: NULL required pointer, B < 0, n_tok < 0, capacity < 0 ->
 *      TPPO_ERR_NULL / TPPO_ERR_SIZE; tail_drop < 0 -> TPPO_ERR_PARAM.
 *      B = 0 is valid (counts = 0).  Sequences with a bad layout set
 *      TPPO_STATUS_BAD_LAYOUT and are treated as having an empty window.
 */
size_t tppo_select_workspace_bytes(int64_t B, int64_t capacity);
int tppo_select(const int32_t* cu_seqlens, const int32_t* ctx_len, const int32_t* done,
                const int32_t* input_ids, int64_t B, int64_t n_tok, int32_t tail_drop,
                int32_t* resp_off, int32_t* sel_off, int32_t* keep_len,
                int32_t* sel_rows, int32_t* sel_targets, int32_t* sel_resp_idx,
                int64_t capacity, int64_t* counts, void* workspace, size_t workspace_bytes,
                void* plan, size_t plan_bytes, int32_t* status, void* stream);

/* ---------------------------------------------------------------------------
 * tppo_plan_build -- the work plan of a batch layout: the response-packed
 * domain cut into tiles of <= 1024 tokens of one sequence (what the scan
 * walks), one descriptor per aligned block of 1024 tokens naming the sequences
 * that meet there (what the loss passes walk), the sizes of the policy /
 * value token sets of Sec. 3.2, and zeroed words through which the
 * workgroups of a later launch hand partial results to each other.  Every
 * entry point below that takes `plan` builds the same thing in its workspace
 * when plan is NULL; building it once per batch (here, or as a by-product of
 * tppo_select) saves each of them that launch.
 *
 * in : resp_off[B+1], done[B] int32; keep_len[B] int32 or NULL (a plan built
 *      without keep_len serves tppo_egae* only).
 * out: plan, tppo_plan_bytes(n_resp, B) bytes, 256-byte aligned.  It stays
 *      valid for any number of calls with the same resp_off / keep_len / done;
 *      calls that use one plan must not overlap in time.  Under HIP graph
 *      capture, capture the call that builds a plan together with the calls
 *      that use it (a replayed launch repeats its call number).
 * A consumer given a plan that was built for other sizes sets
 * TPPO_STATUS_BAD_LAYOUT and computes nothing.
 */
size_t tppo_plan_bytes(int64_t n_resp, int64_t B);
int tppo_plan_build(const int32_t* resp_off, const int32_t* keep_len, const int32_t* done,
                    int64_t B, int64_t n_resp, void* plan, size_t plan_bytes,
                    int32_t* status, void* stream);

/* ---------------------------------------------------------------------------
 * tppo_token_logprobs -- log-probability of each kept token under the current
 * policy, log pi_theta(a_t|s_t), the numerator of the ratio in Eq. (ppoloss):
 *   z = W_head h_{sel_rows[m]}           (V logits, never written to memory)
 *   lse[m]  = log sum_v exp z[v]
 *   logp[m] = z[sel_targets[m]] - lse[m]
 * Only the M kept rows are projected; prompt rows and dropped tails cost
 * nothing (the filtered policy update of Sec. 3.2).  No bias, temperature 1.
 *
 * in : hidden  [n_rows, H] row-major with leading dimension ld_hidden (elements);
 *      w_head  [V, H] row-major (torch Linear.weight layout), leading dim ld_w;
 *      both of type `dt` (TPPO_BF16: bf16 inputs, fp32 accumulation on the
 *      matrix cores when H % 64 == 0 and both leading dimensions are multiples
 *      of 8 and the base pointers 16-byte aligned, otherwise a slower generic
 *      kernel; TPPO_F32: fp32 FMA kernel; the generic and the fp32 kernel keep
 *      one hidden row in LDS and take H <= 16320, beyond that TPPO_ERR_SIZE);
 *      sel_rows[M], sel_targets[M] int32;
 *      m_actual: optional device int64 (e.g. counts+0 of tppo_select): only the
 *      first min(M, *m_actual) tokens are computed, so M can be a host-side
 *      upper bound and no read-back is needed.  NULL = M.
 *      out_index: optional int32[M]; result m is written to logp[out_index[m]]
 *      (e.g. sel_resp_idx, to scatter into the response-packed domain).
 * out: logp fp32, lse fp32 (NULL = not wanted), indexed by m or out_index[m].
 * Errors: M, H, V, n_rows < 0, H = 0 or V = 0 with M > 0, ld < H ->
 *      TPPO_ERR_SIZE; M = 0 is valid and does nothing.  Bad row / target ids set
 *      status bits and yield NaN for that token.
 */
size_t tppo_token_logprobs_workspace_bytes(int64_t M, int64_t H, int64_t V, tppo_dtype dt);
int tppo_token_logprobs(const void* hidden, int64_t n_rows, int64_t H, int64_t ld_hidden,
                        const void* w_head, int64_t V, int64_t ld_w, tppo_dtype dt,
                        const int32_t* sel_rows, const int32_t* sel_targets, int64_t M,
                        const int64_t* m_actual, const int32_t* out_index,
                        float* logp, float* lse,
                        void* workspace, size_t workspace_bytes,
                        int32_t* status, void* stream);

/* ---------------------------------------------------------------------------
 * tppo_egae -- Extended GAE (Sec. 3.1, Eq. (egae)) and returns (Sec. 2.4), for
 * every window token of every sequence (the filter applies to the losses, not
 * to the recurrence).  With l = win_len[i], per sequence:
 *   delta_t = r_t + gamma V(s_{t+1}) - V(s_t)                       (Eq. (TD))
 *   V(s_l)  = 0                 if done[i]   (terminal state)
 *           = bootstrap[i]      if bootstrap != NULL
 *           = V(s_{l-1})        otherwise    (the assumption of Sec. 3.1)
 *   A_t = sum_{k=t}^{l-1} (gamma lambda)^{k-t} delta_k            (Eq. (egae))
 *   R_t = sum_{k=t}^{l-1} gamma^{k-t} r_k     (observed rewards only)
 * Finished sequences therefore get standard GAE (Eq. (gae)).
 *
 * in : rewards[n_resp], values[n_resp] fp32, response-packed, values[j] = V(s_t)
 *      of the rollout-time critic; resp_off[B+1], done[B] int32;
 *      bootstrap[B] fp32 or NULL.
 * out: adv[n_resp], ret[n_resp] fp32.  May not alias the inputs.
 * workspace / plan: with plan = NULL the call builds its own plan in workspace
 *      (tppo_egae_workspace_bytes); with a plan of this layout (tppo_select,
 *      tppo_plan_build) the workspace is not used and may be NULL.
 * Errors: gamma or lambda outside [0,1] -> TPPO_ERR_PARAM; negative sizes ->
 *      TPPO_ERR_SIZE.  n_resp = 0 is valid.  resp_off must be non-decreasing
 *      with resp_off[0] = 0 and resp_off[B] = n_resp (empty sequences allowed).
 */
size_t tppo_egae_workspace_bytes(int64_t n_resp, int64_t B);
int tppo_egae(const float* rewards, const float* values, const int32_t* resp_off,
              const int32_t* done, const float* bootstrap,
              int64_t B, int64_t n_resp, float gamma, float lambda,
              float* adv, float* ret, void* workspace, size_t workspace_bytes,
              void* plan, int32_t* status, void* stream);

/* tppo_egae_static -- tppo_egae for callers that cannot allocate device memory
 * or may not call anything that does: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same inputs, outputs,
 * results and errors as tppo_egae with plan = NULL, but there is no workspace
 * argument: the call builds its plan in a fixed array of 5.3 MiB that
 * is part of the library's image on every GPU the library runs on (it stays
 * there until the process ends).  It calls no hipMalloc / hipFree and no
 * library routine that allocates; the first call on a device asks the runtime
 * for the array's address there and keeps it.
 * Limit: n_resp / 1024 + B + 1 <= tppo_egae_static_max_tiles() (47872: e.g.
 * 40 M tokens in 8704 sequences); larger batches -> TPPO_ERR_SIZE, nothing is
 * launched.
 * All calls on one GPU share the array: two calls may not overlap in time on
 * the same GPU (calls on one stream never do; calls on different streams, or
 * from different threads on different streams, race).  Nothing has to be
 * cleared between calls: each call rebuilds the list and zeroes the words it
 * is going to use.
 */
int64_t tppo_egae_static_max_tiles(void);
int tppo_egae_static(const float* rewards, const float* values, const int32_t* resp_off,
                     const int32_t* done, const float* bootstrap,
                     int64_t B, int64_t n_resp, float gamma, float lambda,
                     float* adv, float* ret, int32_t* status, void* stream);

/* tppo_egae_terminal -- the same with the sparse reward of Sec. 2.1 (one
 * rule-based reward at the end of a finished response, nothing else): instead
 * of a dense array, terminal_reward[B] gives r of the last window token of
 * sequence i; it is read only where done[i] != 0, every other reward is 0.
 * Identical results to tppo_egae on the dense array so built; 12 instead of
 * 16 bytes of traffic per token.  Same workspace, arguments and errors.
 */
int tppo_egae_terminal(const float* terminal_reward, const float* values, const int32_t* resp_off,
                       const int32_t* done, const float* bootstrap,
                       int64_t B, int64_t n_resp, float gamma, float lambda,
                       float* adv, float* ret, void* workspace, size_t workspace_bytes,
                       void* plan, int32_t* status, void* stream);

/* ---------------------------------------------------------------------------
 * tppo_ppo_losses -- token-level losses (Sec. 4.1.1) of one update:
 *   rho_t = exp(logp_new - logp_old)
 *   policy_sum = - sum_{policy tokens} min(rho_t A_t, clip(rho_t, 1-eps_low, 1+eps_high) A_t)
 *   policy_loss = policy_sum / n_policy            (= -J_PPO, Eq. (ppoloss))
 *   V_clip = clip(v_new, v_old - xi_low, v_old + xi_high)        (Eq. (valueclip))
 *   value_sum = 1/2 sum_{value tokens} max((v_new - R)^2, (V_clip - R)^2)
 *   value_loss = value_sum / n_value               (= J_value, Eq. (valueloss))
 * Policy tokens of sequence i: window tokens t < keep_len[i]; value tokens: all
 * window tokens of sequences with done[i] != 0 (Sec. 3.2).  Entries outside a
 * set are not read, so whatever they hold cannot influence the result.  An
 * entry INSIDE a set that is not a number is not clipped away: that loss is
 * NaN.  Empty sets give a loss of 0.  The un-normalised sums and counts let the caller
 * combine minibatches.  Reductions are deterministic (no float atomics).
 *
 * in : six fp32 arrays [n_resp], response-packed; the three policy arrays
 *      (logp_new, logp_old, adv) may all be NULL to skip the policy half,
 *      likewise (v_new, v_old, ret); resp_off[B+1], keep_len[B], done[B] int32.
 * out: one tppo_loss_out in device memory.
 * workspace / plan: as for tppo_egae (the plan must have been built with keep_len).
 * Errors: eps or xi negative -> TPPO_ERR_PARAM; a half with only some of its
 *      arrays NULL -> TPPO_ERR_NULL.
 */
typedef struct {
    float policy_loss, value_loss, policy_sum, value_sum;
    int64_t n_policy, n_value;
} tppo_loss_out;

size_t tppo_ppo_losses_workspace_bytes(int64_t n_resp, int64_t B);
int tppo_ppo_losses(const float* logp_new, const float* logp_old, const float* adv,
                    const float* v_new, const float* v_old, const float* ret,
                    const int32_t* resp_off, const int32_t* keep_len, const int32_t* done,
                    int64_t B, int64_t n_resp,
                    float eps_low, float eps_high, float xi_low, float xi_high,
                    tppo_loss_out* out, void* workspace, size_t workspace_bytes,
                    void* plan, int32_t* status, void* stream);

/* ---------------------------------------------------------------------------
 * tppo_ppo_losses_backward -- the step after the losses in Alg. 1 (policy and
 * value updates): derivatives of Eq. (ppoloss) and Eqs. (valueclip),
 * (valueloss) with respect to the new policy's log-probs and the new values,
 * in one streaming pass that also yields the losses themselves and the
 * fraction of tokens whose clip is active.
 *
 *   grad_logp[j] = policy_scale * d policy_loss / d logp_new[j]
 *                = -policy_scale * rho_j A_j / N_policy  where rho A <= clip(rho) A
 *                  (the unclipped surrogate is the minimum), 0 where the clip is
 *                  saturated ("clipped" token) and 0 outside the policy set;
 *   grad_v[j]    = value_scale * d value_loss / d v_new[j]
 *                = value_scale * (V_j - R_j) / N_value  where (V-R)^2 >= (V_clip-R)^2,
 *                  0 where the clipped square is larger ("clipped") and 0 outside
 *                  the value set.
 * N_policy / N_value are this call's token counts (token-level mean, Sec.
 * 4.1.1) unless policy_denominator / value_denominator > 0 replace them (a
 * batch spread over several calls or devices).  Sets, masking by selection and
 * determinism as in tppo_ppo_losses.  Decisions are taken in fp32.  A token of
 * a set with a NaN among its inputs gets the derivative NaN and counts neither
 * as clipped nor as unclipped.
 *
 * in : as tppo_ppo_losses, plus the two scales (finite) and denominators.
 * out: grad_logp[n_resp], grad_v[n_resp] device fp32, every element written
 *      (NULL exactly when the corresponding input half is NULL); out and stats
 *      device, each may be NULL.
 * Errors: as tppo_ppo_losses; a gradient pointer that does not match its half
 *      -> TPPO_ERR_NULL; NaN scale -> TPPO_ERR_PARAM.
 */
typedef struct {
    float ratio_mean;          /* mean of rho over the policy set */
    float policy_clip_frac;    /* n_policy_clipped / n_policy */
    float value_clip_frac;     /* n_value_clipped / n_value */
    float reserved;
    int64_t n_policy_clipped, n_value_clipped;
} tppo_loss_stats;

size_t tppo_ppo_losses_backward_workspace_bytes(int64_t n_resp, int64_t B);
int tppo_ppo_losses_backward(const float* logp_new, const float* logp_old, const float* adv,
                             const float* v_new, const float* v_old, const float* ret,
                             const int32_t* resp_off, const int32_t* keep_len, const int32_t* done,
                             int64_t B, int64_t n_resp,
                             float eps_low, float eps_high, float xi_low, float xi_high,
                             float policy_scale, float value_scale,
                             int64_t policy_denominator, int64_t value_denominator,
                             float* grad_logp, float* grad_v,
                             tppo_loss_out* out, tppo_loss_stats* stats,
                             void* workspace, size_t workspace_bytes,
                             void* plan, int32_t* status, void* stream);

/* ---------------------------------------------------------------------------
 * tppo_token_logprobs_backward -- derivatives of the kept tokens' log-probs
 * (the quantity inside the ratio of Eq. (ppoloss)) with respect to the hidden
 * rows and the head matrix: the policy update of Alg. 1 carried one layer down.
 * With z = W h and logp_t = z_t[target_t] - lse_t,
 *     dz[t, v]          = g_t * ([v == target_t] - exp(z[t, v] - lse_t)),
 *     grad_hidden[t, :] = sum_v dz[t, v] * W[v, :],
 *     grad_w[v, :]     (+)= sum_t dz[t, v] * hidden[sel_rows[t], :],
 * where g_t is the upstream derivative d L / d logp_t (for instance grad_logp
 * of tppo_ppo_losses_backward) and lse_t the forward pass's log-sum-exp.  No
 * logits are kept from the forward pass: they are recomputed tile by tile.
 * dz is rounded to bf16 (round to nearest even) before the two products, which
 * accumulate in fp32.
 *
 * in : hidden, w_head, sel_rows, sel_targets, M as in tppo_token_logprobs
 *      (bf16 only; H % 64 == 0, leading dimensions % 8 == 0, 16-byte aligned
 *      bases, else TPPO_ERR_PARAM; fp32 -> TPPO_ERR_DTYPE);
 *      lse, grad_logp  device fp32; token t's entries are element in_index[t]
 *                      (in_index NULL: element t).
 * out: grad_hidden[M, H]  device fp32, row t belongs to hidden row sel_rows[t];
 *      grad_w[V, H]       device fp32, overwritten, or added to when
 *                         accumulate_w != 0.  Either may be NULL to skip it.
 * status is not written by this call (bad rows and targets were reported by
 * the forward pass; rows are clamped, a bad target matches no column).
 * workspace: tppo_token_logprobs_backward_workspace_bytes(M, ...) holds dZ in
 *      both layouts for min(M, 98304) tokens at once (about 4 V bytes per
 *      token plus W^T: 46 GB for the 77 000 kept tokens of the 32B-shaped
 *      head) and is the fastest.  The call works with any workspace that
 *      holds 256 tokens (the size the same function returns for M = 256): it
 *      then goes through chunks of as many tokens, a multiple of 256, as the
 *      workspace holds, more slowly (fewer tiles per sweep, grad_w re-read and
 *      re-written per chunk); smaller than that -> TPPO_ERR_WORKSPACE.
 */
size_t tppo_token_logprobs_backward_workspace_bytes(int64_t M, int64_t H, int64_t V, tppo_dtype dt);
int tppo_token_logprobs_backward(const void* hidden, int64_t n_rows, int64_t H, int64_t ld_hidden,
                                 const void* w_head, int64_t V, int64_t ld_w, tppo_dtype dt,
                                 const int32_t* sel_rows, const int32_t* sel_targets, int64_t M,
                                 const float* lse, const float* grad_logp, const int32_t* in_index,
                                 float* grad_hidden, float* grad_w, int32_t accumulate_w,
                                 void* workspace, size_t workspace_bytes,
                                 int32_t* status, void* stream);

/* ---------------------------------------------------------------------------
 * tppo_batcher_* -- slot bookkeeping of successive batching (Sec. 3.2 first
 * paragraph, Alg. 1 line 2).  HOST code and HOST pointers only, integers only.
 * A constant number of slots; a sequence ends when it emits the
 * end-of-sequence token or when its response reaches max_response tokens (the
 * actual maximum length L); one step adds at most `window` (l) tokens.  Ended
 * sequences are replaced by new prompts at the next refill, the others stay and
 * their previous window becomes context.
 *
 *   create(slots, window, max_response)   NULL on bad sizes or no memory; the
 *                                         caller owns the object until destroy.
 *   refill(b, prompt_len, n_available, n_taken)
 *        new prompts (>= 1 token each) go into empty or finished slots in slot
 *        order, ids count up from 0; *n_taken (may be NULL) says how many.
 *        An empty prompt among those that would be taken -> TPPO_ERR_PARAM,
 *        nothing changed.
 *   advance(b, gen_len[slots], eos[slots])
 *        one rollout window.  Every slot must hold an unfinished sequence
 *        (else TPPO_ERR_PARAM); 0 <= gen_len <= window and the response may not
 *        pass max_response (TPPO_ERR_SIZE); a sequence that stops short of both
 *        limits must have eos set (TPPO_ERR_PARAM).  A rejected call changes nothing.
 *   layout(b, cu_seqlens[slots+1], ctx_len, prompt_len, done, seq_id)
 *        the packed layout of the current training batch (seq_id may be NULL).
 *        For the policy tokens call tppo_select with ctx_len; for the value
 *        tokens (every response token of finished sequences, whichever window
 *        produced it) call it with prompt_len in place of ctx_len and
 *        tail_drop = INT32_MAX.
 */
typedef struct tppo_batcher tppo_batcher;
tppo_batcher* tppo_batcher_create(int64_t slots, int32_t window, int32_t max_response);
void tppo_batcher_destroy(tppo_batcher* b);
int tppo_batcher_refill(tppo_batcher* b, const int32_t* prompt_len, int64_t n_available, int64_t* n_taken);
int tppo_batcher_advance(tppo_batcher* b, const int32_t* gen_len, const int32_t* eos);
int tppo_batcher_layout(const tppo_batcher* b, int32_t* cu_seqlens, int32_t* ctx_len, int32_t* prompt_len,
                        int32_t* done, int64_t* seq_id);

/* ---------------------------------------------------------------------------
 * tppo_value_head -- V(s_t) = w_value . h_t + bias for a list of hidden rows of
 * the value model (Sec. 2.2): the projection that yields the v_new consumed by
 * Eq. (valueloss).  bf16 rows and weights, fp32 accumulation and output.
 *
 * in : hidden [n_rows, H] device bf16, row stride ld_hidden (H % 8 == 0,
 *      ld_hidden % 8 == 0, 16-byte aligned base, else TPPO_ERR_PARAM;
 *      H <= 16384); w_value [H] device bf16; bias host scalar;
 *      rows[M] device int32 (NULL: rows 0 .. M-1); m_actual as in
 *      tppo_token_logprobs.
 * out: v_out[out_index[t]] (out_index NULL: v_out[t]) device fp32.
 * A row index outside [0, n_rows) gives NaN and sets TPPO_STATUS_BAD_ROW.
 */
int tppo_value_head(const void* hidden, int64_t n_rows, int64_t H, int64_t ld_hidden,
                    const void* w_value, float bias, tppo_dtype dt,
                    const int32_t* rows, const int32_t* out_index, int64_t M, const int64_t* m_actual,
                    float* v_out, int32_t* status, void* stream);

/* ---------------------------------------------------------------------------
 * tppo_diag_mfma_rate -- a measuring stick, not a step of the method: runs the
 * inner loop of the LM-head kernel (v_mfma_f32_16x16x32_bf16, 8 wavefronts per
 * workgroup, one workgroup per CU, 32 MFMAs per wavefront and iteration) on
 * operands held in registers, with no memory traffic.  Timing it gives the
 * matrix-core rate this chip sustains under its power limit, the practical
 * ceiling beside the datasheet peak in the benchmark's roofline entry.
 *
 * in : operands  device, 6144 bf16 values (16-byte aligned); finite values of
 *                the magnitude of real inputs make the power draw realistic.
 *      iters     loop count (0 .. 2^24).
 * out: out       device, 131072 floats (one checksum per thread; contents are
 *                not specified).  *flop (host, may be NULL): floating-point
 *                operations the launch performs.
 */
int tppo_diag_mfma_rate(const void* operands, float* out, int64_t iters, double* flop, void* stream);

/* tppo_diag_streams -- the streaming counterpart: one elementwise pass over
 * n_read input streams (src + k * stride_bytes) and n_write output streams
 * (dst + k * stride_bytes), each bytes_per_stream long; every output is the
 * sum of the inputs.  Lanes on consecutive 16 bytes, one element per thread
 * and stream, non-temporal accesses, small workgroups: the shape measured
 * fastest on this chip.  Timing it gives the rate the memory system sustains for as many
 * concurrent streams as one of this library's kernels has: (n_read, n_write) =
 * (2,2) EGAE, (1,2) EGAE from terminal rewards, (6,0) losses, (6,2) loss
 * derivatives, (1,1) plain copy, (1,0) plain read; other shapes ->
 * TPPO_ERR_PARAM.  Sizes positive multiples of 16, pointers 16-byte aligned.
 * (With n_write = 0 nothing is written, unless the sum of everything read is
 * exactly 1.2345e-30, in which case src[0] receives it.)
 */
int tppo_diag_streams(const void* src, void* dst, int64_t bytes_per_stream, int64_t stride_bytes,
                      int32_t n_read, int32_t n_write, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* TPPO_H */
