"""Fast oracle: numpy fp64.  This is what the HIP results are compared with.

Test infrastructure only: the product path never imports this module.

Same definitions as ``oracle.definitional`` (which pins it on tiny inputs),
evaluated in O(T): the sums of Eq. (gae)/(egae) and of the return R_t are
computed by the backward recurrences they telescope into, and the LM head is
one BLAS matrix product followed by the textbook log-softmax.  All arithmetic
is fp64 on the exact fp32 / bf16 values of the inputs.
"""
import numpy as np


def decode(x):
    """Input array -> fp64.  ``uint16`` arrays hold bfloat16 bit patterns
    (the upper half of an IEEE binary32); everything else is a plain cast."""
    x = np.asarray(x)
    if x.dtype == np.uint16:
        return (x.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return x.astype(np.float64)


# --------------------------------------------------------------------------
# Token filter (Sec. 3.2)
# --------------------------------------------------------------------------
def select(cu_seqlens, ctx_len, done, input_ids, tail_drop):
    """Policy tokens = window tokens of every sequence minus the ``tail_drop``
    latest of unfinished ones; value tokens = window tokens of finished
    sequences (Sec. 3.2).  The row that predicts a token is the packed position
    before it (Sec. 2.1)."""
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    ctx = np.asarray(ctx_len, dtype=np.int64)
    dn = np.asarray(done, dtype=np.int64) != 0
    ids = np.asarray(input_ids)
    B = ctx.shape[0]
    win_len = cu[1:] - cu[:-1] - ctx
    keep_len = np.where(dn, win_len, np.maximum(win_len - int(tail_drop), 0))
    resp_off = np.concatenate([[0], np.cumsum(win_len)])
    sel_off = np.concatenate([[0], np.cumsum(keep_len)])
    rows, tgts, ridx = [], [], []
    for i in range(B):
        t = np.arange(keep_len[i], dtype=np.int64)
        pos = cu[i] + ctx[i] + t
        rows.append(pos - 1)
        tgts.append(ids[pos].astype(np.int64))
        ridx.append(resp_off[i] + t)
    cat = (lambda xs: np.concatenate(xs) if xs else np.zeros(0, np.int64))
    return dict(resp_off=resp_off.astype(np.int32), sel_off=sel_off.astype(np.int32),
                keep_len=keep_len.astype(np.int32),
                sel_rows=cat(rows).astype(np.int32),
                sel_targets=cat(tgts).astype(np.int32),
                sel_resp_idx=cat(ridx).astype(np.int32),
                M=int(sel_off[B]), N_resp=int(resp_off[B]),
                N_val=int(win_len[dn].sum()))


# --------------------------------------------------------------------------
# log pi_theta(a_t | s_t)  (inside the ratio of Eq. (ppoloss))
# --------------------------------------------------------------------------
def token_logprobs(hidden, w_head, sel_rows, sel_targets, row_block=256,
                   vocab_block=8192):
    """``log softmax(W h_row)[target]`` for each kept token.

    The logits of a block of rows are formed in full (the matrix product is
    evaluated a block of vocabulary columns at a time only so that the fp64
    copy of ``w_head`` never has to exist whole; each logit is still one dot
    product), then reduced with the plain definition
    ``lse = max + log(sum(exp(z - max)))``.  Returns ``(logp, lse)`` in fp64.
    """
    sel_rows = np.asarray(sel_rows, dtype=np.int64)
    sel_targets = np.asarray(sel_targets, dtype=np.int64)
    M = sel_rows.shape[0]
    V = w_head.shape[0]
    logp = np.empty(M, np.float64)
    lse = np.empty(M, np.float64)
    if M == 0:
        return logp, lse
    for r0 in range(0, M, row_block):
        r1 = min(r0 + row_block, M)
        h = decode(hidden[sel_rows[r0:r1]])
        z = np.empty((r1 - r0, V), np.float64)
        for v0 in range(0, V, vocab_block):
            v1 = min(v0 + vocab_block, V)
            z[:, v0:v1] = h @ decode(w_head[v0:v1]).T
        zmax = z.max(axis=1)
        block_lse = zmax + np.log(np.exp(z - zmax[:, None]).sum(axis=1))
        lse[r0:r1] = block_lse
        logp[r0:r1] = z[np.arange(r1 - r0), sel_targets[r0:r1]] - block_lse
    return logp, lse


# --------------------------------------------------------------------------
# Extended GAE (Sec. 3.1) and Monte-Carlo return (Sec. 2.4)
# --------------------------------------------------------------------------
def egae(rewards, values, resp_off, done, gamma, lam, bootstrap=None):
    """Backward form of Eq. (egae): with delta_t from Eq. (TD),
    ``A_t = delta_t + gamma*lam*A_{t+1}`` and ``R_t = r_t + gamma*R_{t+1}``,
    both zero past the last window token.  The value of the state after the
    last token is 0 for a finished sequence and, for a truncated one, the
    value of the last state (Sec. 3.1) unless ``bootstrap[i]`` overrides it.
    Returns ``(adv, ret)`` in fp64, response-packed.
    """
    r = decode(rewards)
    v = decode(values)
    n = r.shape[0]
    adv = np.zeros(n, np.float64)
    ret = np.zeros(n, np.float64)
    c = float(gamma) * float(lam)
    g = float(gamma)
    for i in range(len(done)):
        lo, hi = int(resp_off[i]), int(resp_off[i + 1])
        if hi <= lo:
            continue
        rs = r[lo:hi].tolist()
        vs = v[lo:hi].tolist()
        if int(done[i]) != 0:
            v_next = 0.0
        elif bootstrap is not None:
            v_next = float(bootstrap[i])
        else:
            v_next = vs[-1]
        a_next = 0.0
        r_next = 0.0
        a_out = [0.0] * (hi - lo)
        r_out = [0.0] * (hi - lo)
        for t in range(hi - lo - 1, -1, -1):
            delta = rs[t] + g * v_next - vs[t]
            a_next = delta + c * a_next
            r_next = rs[t] + g * r_next
            a_out[t] = a_next
            r_out[t] = r_next
            v_next = vs[t]
        adv[lo:hi] = a_out
        ret[lo:hi] = r_out
    return adv, ret


# --------------------------------------------------------------------------
# Losses: Eq. (ppoloss), Eq. (valueclip), Eq. (valueloss)
# --------------------------------------------------------------------------
def loss_masks(resp_off, keep_len, done):
    """Boolean masks over the response-packed domain: policy set and value set
    of Sec. 3.2."""
    resp_off = np.asarray(resp_off, dtype=np.int64)
    n = int(resp_off[-1])
    pol = np.zeros(n, bool)
    val = np.zeros(n, bool)
    for i in range(len(done)):
        lo, hi = int(resp_off[i]), int(resp_off[i + 1])
        pol[lo:lo + int(keep_len[i])] = True
        if int(done[i]) != 0:
            val[lo:hi] = True
    return pol, val


def ppo_losses(logp_new, logp_old, adv, v_new, v_old, ret,
               resp_off, keep_len, done,
               eps_low, eps_high, xi_low, xi_high):
    """policy_loss = -mean_policy min(rho A, clip(rho, 1-eps_low, 1+eps_high) A)
    with rho = exp(logp_new - logp_old)  (Eq. (ppoloss));
    value_loss = 1/2 mean_value max((V-R)^2, (V_clip-R)^2) with V_clip from
    Eq. (valueclip)  (Eq. (valueloss)).  Token-level means (Sec. 4.1.1).
    Masked-out entries are selected away before any arithmetic, so whatever
    they hold (NaN, Inf) cannot reach the result.  An entry INSIDE a set that
    is not a number makes its term, and hence that loss, not a number (the
    paper is silent; min, max and clip here all propagate NaN).
    """
    pol, val = loss_masks(resp_off, keep_len, done)
    n_pol, n_val = int(pol.sum()), int(val.sum())
    policy_sum = 0.0
    value_sum = 0.0
    if n_pol:
        ln, lo_, a = (decode(x)[pol] for x in (logp_new, logp_old, adv))
        rho = np.exp(ln - lo_)
        surr = np.minimum(rho * a, np.clip(rho, 1.0 - eps_low, 1.0 + eps_high) * a)
        policy_sum = -float(np.sum(surr))
    if n_val:
        v, vo, r = (decode(x)[val] for x in (v_new, v_old, ret))
        v_clip = np.clip(v, vo - xi_low, vo + xi_high)
        value_sum = 0.5 * float(np.sum(np.maximum((v - r) ** 2, (v_clip - r) ** 2)))
    return dict(policy_loss=policy_sum / n_pol if n_pol else 0.0,
                value_loss=value_sum / n_val if n_val else 0.0,
                policy_sum=policy_sum, value_sum=value_sum,
                n_policy=n_pol, n_value=n_val)


def ppo_loss_grads(logp_new, logp_old, adv, v_new, v_old, ret,
                   resp_off, keep_len, done,
                   eps_low, eps_high, xi_low, xi_high,
                   policy_scale=1.0, value_scale=1.0,
                   policy_denominator=None, value_denominator=None):
    """Derivatives of policy_scale * policy_loss with respect to logp_new and of
    value_scale * value_loss with respect to v_new (Eq. (ppoloss);
    Eqs. (valueclip), (valueloss); token-level means), zero outside the sets:
    -rho A / N where the unclipped surrogate is the minimum, 0 where the clip is
    saturated; (V - R) / N where the unclipped square is the maximum, 0 where
    the clipped one is.  Plus clipped-token counts and the mean ratio.
    A token of a set with a NaN among its inputs has an undefined term: its
    derivative is NaN and it is counted neither as clipped nor as unclipped."""
    pol, val = loss_masks(resp_off, keep_len, done)
    n = pol.shape[0]
    n_pol, n_val = int(pol.sum()), int(val.sum())
    den_p = float(policy_denominator) if policy_denominator else float(n_pol)
    den_v = float(value_denominator) if value_denominator else float(n_val)
    g_lp, g_v = np.zeros(n), np.zeros(n)
    pol_clipped = val_clipped = 0
    ratio_mean = 0.0
    if n_pol:
        ln, lo_, a = (decode(x)[pol] for x in (logp_new, logp_old, adv))
        rho = np.exp(ln - lo_)
        undefined = np.isnan(rho * a)
        unclipped = rho * a <= np.clip(rho, 1.0 - eps_low, 1.0 + eps_high) * a
        g_lp[pol] = np.where(undefined, np.nan, np.where(unclipped, -policy_scale * rho * a / den_p, 0.0))
        pol_clipped = int((~unclipped & ~undefined).sum())
        ratio_mean = float(rho.mean())
    if n_val:
        v, vo, r = (decode(x)[val] for x in (v_new, v_old, ret))
        d0 = v - r
        d1 = np.clip(v, vo - xi_low, vo + xi_high) - r
        undefined = np.isnan(d0) | np.isnan(d1)
        unclipped = d0 * d0 >= d1 * d1
        g_v[val] = np.where(undefined, np.nan, np.where(unclipped, value_scale * d0 / den_v, 0.0))
        val_clipped = int((~unclipped & ~undefined).sum())
    return dict(grad_logp=g_lp, grad_v=g_v, n_policy=n_pol, n_value=n_val,
                n_policy_clipped=pol_clipped, n_value_clipped=val_clipped, ratio_mean=ratio_mean)


def token_logprob_grads(hidden, w_head, sel_rows, sel_targets, grad_logp, row_block=256, want_w=True,
                        return_abs_bounds=False):
    """Derivatives of L = sum_t g_t logp_t with respect to the kept hidden rows
    and the head matrix: with z = W h, p = softmax(z),
        dz[t, v] = g_t ([v = target_t] - p[t, v]),
        grad_hidden[t] = dz[t] W,    grad_w = dz^T Hid.
    All logits of a block of rows are formed in full, fp64 throughout.  With
    ``return_abs_bounds`` also returns |dz| |W| and |dz|^T |Hid| (the sums of
    the magnitudes of the terms of each output element), which tests use to
    bound the effect of rounding dz."""
    sel_rows = np.asarray(sel_rows, dtype=np.int64)
    sel_targets = np.asarray(sel_targets, dtype=np.int64)
    g = decode(grad_logp)
    M = sel_rows.shape[0]
    V, H = w_head.shape
    w = decode(w_head)
    grad_hidden = np.zeros((M, H))
    grad_w = np.zeros((V, H)) if want_w else None
    abs_h = np.zeros((M, H)) if return_abs_bounds else None
    abs_w = np.zeros((V, H)) if (return_abs_bounds and want_w) else None
    for r0 in range(0, M, row_block):
        r1 = min(r0 + row_block, M)
        h = decode(hidden[sel_rows[r0:r1]])
        z = h @ w.T
        z -= z.max(axis=1, keepdims=True)
        p = np.exp(z)
        p /= p.sum(axis=1, keepdims=True)
        dz = -p
        dz[np.arange(r1 - r0), sel_targets[r0:r1]] += 1.0
        dz *= g[r0:r1, None]
        grad_hidden[r0:r1] = dz @ w
        if want_w:
            grad_w += dz.T @ h
        if return_abs_bounds:
            abs_h[r0:r1] = np.abs(dz) @ np.abs(w)
            if want_w:
                abs_w += np.abs(dz).T @ np.abs(h)
    if return_abs_bounds:
        return grad_hidden, grad_w, abs_h, abs_w
    return grad_hidden, grad_w


def value_head(hidden, w_value, bias, rows, return_abs_bound=False):
    """V(s_t) = w_value . hidden[rows[t]] + bias in fp64 on the exact bf16 / fp32
    inputs (Sec. 2.2).  ``return_abs_bound`` adds sum_k |w_k h_k| per row."""
    rows = np.asarray(rows, dtype=np.int64)
    w = decode(w_value)
    v = np.empty(rows.shape[0])
    bound = np.empty(rows.shape[0])
    for r0 in range(0, rows.shape[0], 4096):
        h = decode(hidden[rows[r0:r0 + 4096]])
        v[r0:r0 + 4096] = h @ w + bias
        if return_abs_bound:
            bound[r0:r0 + 4096] = np.abs(h) @ np.abs(w)
    return (v, bound) if return_abs_bound else v
