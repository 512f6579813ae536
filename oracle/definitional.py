"""Definitional oracle: every quantity evaluated exactly as the paper prints it.

Pure Python, fp64 (``float``), explicit loops and ``math.fsum``.  Slow on
purpose; meant for inputs of a few hundred tokens.  Test infrastructure only.

Indexing (Sec. 2.1): the state ``s_t`` holds the prompt and the response tokens
before position ``t``; the action ``a_t`` is response token ``t``.  So the
hidden state that predicts window token ``t`` of a sequence is the one at the
packed position just before that token, and ``values[t]`` is ``V(s_t)``.

Batch layout: ``B`` sequences packed back to back.  Sequence ``i`` occupies
packed positions ``cu_seqlens[i] .. cu_seqlens[i+1]-1``: first ``ctx_len[i]``
context tokens (prompt plus tokens generated in earlier steps), then
``win_len[i]`` tokens generated in the current step.  ``done[i]`` is 1 when the
sequence emitted its end-of-sequence token inside the window and 0 when it was
cut at the window length (Sec. 3.2).
"""
import math


# --------------------------------------------------------------------------
# Token filter (Sec. 3.2; abstract: prompt and truncated tokens are filtered)
# --------------------------------------------------------------------------
def select(cu_seqlens, ctx_len, done, input_ids, tail_drop):
    """Token filter of Sec. 3.2.

    Policy tokens: every token generated in the current step, finished or not,
    except the ``tail_drop`` latest tokens of an unfinished sequence.  Value
    tokens: all window tokens of finished sequences.  Prompt/context tokens
    belong to neither set.
    """
    B = len(ctx_len)
    resp_off = [0]
    sel_off = [0]
    keep_len = []
    sel_rows, sel_targets, sel_resp_idx = [], [], []
    n_val = 0
    for i in range(B):
        seq_start = int(cu_seqlens[i])
        win_len = int(cu_seqlens[i + 1]) - seq_start - int(ctx_len[i])
        first_window_pos = seq_start + int(ctx_len[i])
        if int(done[i]) != 0:
            keep = win_len
            n_val += win_len
        else:
            keep = max(win_len - int(tail_drop), 0)
        for t in range(win_len):
            if t < keep:
                pos = first_window_pos + t          # packed position of a_t
                sel_rows.append(pos - 1)            # hidden state of s_t
                sel_targets.append(int(input_ids[pos]))
                sel_resp_idx.append(resp_off[i] + t)
        keep_len.append(keep)
        resp_off.append(resp_off[i] + win_len)
        sel_off.append(sel_off[i] + keep)
    return dict(resp_off=resp_off, sel_off=sel_off, keep_len=keep_len,
                sel_rows=sel_rows, sel_targets=sel_targets,
                sel_resp_idx=sel_resp_idx,
                M=sel_off[B], N_resp=resp_off[B], N_val=n_val)


# --------------------------------------------------------------------------
# log pi_theta(a_t | s_t): the quantity inside the ratio of Eq. (ppoloss)
# --------------------------------------------------------------------------
def token_logprobs(hidden, w_head, sel_rows, sel_targets):
    """``log softmax(W h)[target]`` for each kept token, by brute force.

    ``hidden`` is a list of rows (lists of floats), ``w_head`` a list of V rows
    of H floats (``Linear.weight`` layout, no bias, temperature 1).
    Returns ``(logp, lse)``.
    """
    logp, lse = [], []
    for row, tgt in zip(sel_rows, sel_targets):
        h = hidden[row]
        z = [math.fsum(hk * wk for hk, wk in zip(h, w_v)) for w_v in w_head]
        zmax = max(z)
        log_sum = zmax + math.log(math.fsum(math.exp(zv - zmax) for zv in z))
        lse.append(log_sum)
        logp.append(z[tgt] - log_sum)
    return logp, lse


# --------------------------------------------------------------------------
# Extended GAE, Eq. (egae) with Eq. (TD), and the return R_t of Sec. 2.4
# --------------------------------------------------------------------------
def td_residuals(rewards, values, done, gamma, bootstrap=None):
    """delta_t = r_t + gamma V(s_{t+1}) - V(s_t), Eq. (TD), for one sequence.

    The state after the last window token has no value estimate.  For a
    finished response it is terminal, V = 0.  For a truncated one Sec. 3.1
    assumes V(s_l) = V(s_{l-1}); a caller-supplied ``bootstrap`` replaces that
    assumption.
    """
    l = len(rewards)
    delta = []
    for t in range(l):
        if t + 1 < l:
            v_next = values[t + 1]
        elif done:
            v_next = 0.0
        elif bootstrap is not None:
            v_next = bootstrap
        else:
            v_next = values[l - 1]
        delta.append(rewards[t] + gamma * v_next - values[t])
    return delta


def egae_sequence(rewards, values, done, gamma, lam, bootstrap=None):
    """A_t = sum_{k=t}^{l-1} (gamma lam)^{k-t} delta_k  (Eq. (egae)), and
    R_t = sum_i gamma^i r_{t+i} (Sec. 2.4), for one sequence, as double sums."""
    l = len(rewards)
    delta = td_residuals(rewards, values, done, gamma, bootstrap)
    c = gamma * lam
    adv = [math.fsum((c ** (k - t)) * delta[k] for k in range(t, l))
           for t in range(l)]
    ret = [math.fsum((gamma ** i) * rewards[t + i] for i in range(l - t))
           for t in range(l)]
    return adv, ret


def egae(rewards, values, resp_off, done, gamma, lam, bootstrap=None):
    """Eq. (egae) over a response-packed batch: element ``resp_off[i]+t`` of
    each array is window token ``t`` of sequence ``i``."""
    adv, ret = [], []
    for i in range(len(done)):
        lo, hi = int(resp_off[i]), int(resp_off[i + 1])
        b = None if bootstrap is None else float(bootstrap[i])
        a, r = egae_sequence([float(x) for x in rewards[lo:hi]],
                             [float(x) for x in values[lo:hi]],
                             int(done[i]) != 0, gamma, lam, b)
        adv += a
        ret += r
    return adv, ret


# --------------------------------------------------------------------------
# Clipped surrogate, Eq. (ppoloss); clipped value loss, Eqs. (valueclip/loss)
# --------------------------------------------------------------------------
def _clip(x, lo, hi):
    return min(max(x, lo), hi)


def ppo_losses(logp_new, logp_old, adv, v_new, v_old, ret,
               resp_off, keep_len, done,
               eps_low, eps_high, xi_low, xi_high):
    """Token-level means (Sec. 4.1.1) over the policy set and the value set.

    policy_loss = -J_PPO (the paper maximises J_PPO), value_loss = +J_value.
    Empty sets give 0.  Tokens outside a set are never touched.  A token of a
    set with a NaN among its three inputs has the term NaN (Python's min / max
    would return either operand depending on the order, so the rule is spelled out).
    """
    pol_terms, val_terms = [], []
    for i in range(len(done)):
        lo, hi = int(resp_off[i]), int(resp_off[i + 1])
        for t in range(hi - lo):
            j = lo + t
            if t < int(keep_len[i]):
                ratio = math.exp(float(logp_new[j]) - float(logp_old[j]))
                a = float(adv[j])
                if math.isnan(ratio) or math.isnan(a):        # not a number in, not a number out
                    pol_terms.append(math.nan)
                else:
                    pol_terms.append(min(ratio * a,
                                         _clip(ratio, 1.0 - eps_low, 1.0 + eps_high) * a))
            if int(done[i]) != 0:
                v, vo, r = float(v_new[j]), float(v_old[j]), float(ret[j])
                if math.isnan(v) or math.isnan(vo) or math.isnan(r):
                    val_terms.append(math.nan)
                else:
                    v_clip = _clip(v, vo - xi_low, vo + xi_high)
                    val_terms.append(max((v - r) ** 2, (v_clip - r) ** 2))
    policy_sum = -math.fsum(pol_terms)
    value_sum = 0.5 * math.fsum(val_terms)
    n_pol, n_val = len(pol_terms), len(val_terms)
    return dict(policy_loss=policy_sum / n_pol if n_pol else 0.0,
                value_loss=value_sum / n_val if n_val else 0.0,
                policy_sum=policy_sum, value_sum=value_sum,
                n_policy=n_pol, n_value=n_val)


# --------------------------------------------------------------------------
# Derivatives of the two losses with respect to the new policy's log-probs and
# the new values (the step after the losses in Alg. 1: the policy and value
# updates).  Written out branch by branch from Eq. (ppoloss) and
# Eqs. (valueclip), (valueloss).
# --------------------------------------------------------------------------
def ppo_loss_grads(logp_new, logp_old, adv, v_new, v_old, ret,
                   resp_off, keep_len, done,
                   eps_low, eps_high, xi_low, xi_high,
                   policy_scale=1.0, value_scale=1.0,
                   policy_denominator=None, value_denominator=None):
    """d(policy_scale * policy_loss)/d logp_new and d(value_scale * value_loss)/d v_new.

    Policy token: the surrogate is min(u, c) with u = rho A, c = clip(rho) A,
    rho = exp(logp_new - logp_old), so d rho / d logp_new = rho.  Where u <= c
    the unclipped branch is the minimum (inside the clip range the two are the
    same function) and the derivative of the term is rho A; where c < u the
    clip is saturated, c is constant and the derivative is 0 ("clipped").
    Value token: the term is 1/2 max(d0^2, d1^2), d0 = V - R, d1 = V_clip - R.
    Where d0^2 >= d1^2 the derivative is d0; where d1^2 > d0^2 V lies outside
    the clip range (inside it V_clip = V and the squares are equal), V_clip is
    constant and the derivative is 0 ("clipped").
    Token-level means: each derivative is divided by the number of tokens of
    its set (or by the given denominator, for a batch spread over several
    calls).  policy_loss = -J_PPO, hence the minus sign.  Entries outside a set
    get 0.  Also returns the clipped-token counts and the mean ratio.  A token
    of a set with a NaN among its inputs gets the derivative NaN and is counted
    neither as clipped nor as unclipped.
    """
    n = int(resp_off[len(done)])
    g_lp, g_v = [0.0] * n, [0.0] * n
    n_pol = sum(min(int(keep_len[i]), int(resp_off[i + 1]) - int(resp_off[i])) for i in range(len(done)))
    n_val = sum(int(resp_off[i + 1]) - int(resp_off[i]) for i in range(len(done)) if int(done[i]) != 0)
    den_p = float(policy_denominator) if policy_denominator else float(n_pol)
    den_v = float(value_denominator) if value_denominator else float(n_val)
    pol_clipped = val_clipped = 0
    ratios = []
    for i in range(len(done)):
        lo, hi = int(resp_off[i]), int(resp_off[i + 1])
        for t in range(hi - lo):
            j = lo + t
            if t < int(keep_len[i]):
                ratio = math.exp(float(logp_new[j]) - float(logp_old[j]))
                a = float(adv[j])
                u = ratio * a
                c = _clip(ratio, 1.0 - eps_low, 1.0 + eps_high) * a
                ratios.append(ratio)
                if math.isnan(u):                             # undefined term: neither branch
                    g_lp[j] = math.nan
                elif u <= c:
                    g_lp[j] = -policy_scale * ratio * a / den_p
                else:
                    pol_clipped += 1
            if int(done[i]) != 0:
                v, vo, r = float(v_new[j]), float(v_old[j]), float(ret[j])
                d0 = v - r
                d1 = _clip(v, vo - xi_low, vo + xi_high) - r
                if math.isnan(d0) or math.isnan(vo):
                    g_v[j] = math.nan
                elif d0 * d0 >= d1 * d1:
                    g_v[j] = value_scale * d0 / den_v
                else:
                    val_clipped += 1
    return dict(grad_logp=g_lp, grad_v=g_v, n_policy=n_pol, n_value=n_val,
                n_policy_clipped=pol_clipped, n_value_clipped=val_clipped,
                ratio_mean=math.fsum(ratios) / len(ratios) if ratios else 0.0)


# --------------------------------------------------------------------------
# Derivatives of the kept tokens' log-probs (the policy update of Alg. 1 one
# layer down): d/dh and d/dW of  L = sum_t g_t logp_t,  logp_t = z_t[a_t] - lse_t,
# z_t = W h_t.  Since d lse / d z_v = softmax(z)_v, d logp_t / d z_v = [v = a_t] - p_v.
# --------------------------------------------------------------------------
def token_logprob_grads(hidden, w_head, sel_rows, sel_targets, grad_logp):
    """Returns (grad_hidden, grad_w): grad_hidden[t] = sum_v dz[t][v] W[v],
    grad_w[v] = sum_t dz[t][v] h_t with dz[t][v] = g_t ([v = a_t] - p_t[v]).
    Brute force; lists of lists in, lists of lists out."""
    V, H = len(w_head), len(w_head[0])
    grad_w = [[0.0] * H for _ in range(V)]
    grad_hidden = []
    for row, tgt, g in zip(sel_rows, sel_targets, grad_logp):
        h = hidden[row]
        z = [math.fsum(hk * wk for hk, wk in zip(h, w_v)) for w_v in w_head]
        zmax = max(z)
        total = math.fsum(math.exp(zv - zmax) for zv in z)
        dz = [g * ((1.0 if v == tgt else 0.0) - math.exp(z[v] - zmax) / total) for v in range(V)]
        grad_hidden.append([math.fsum(dz[v] * w_head[v][k] for v in range(V)) for k in range(H)])
        for v in range(V):
            for k in range(H):
                grad_w[v][k] += dz[v] * h[k]
    return grad_hidden, grad_w


# --------------------------------------------------------------------------
# Value head (Sec. 2.2: the value model maps a state to one scalar)
# --------------------------------------------------------------------------
def value_head(hidden, w_value, bias, rows):
    """V(s_t) = w_value . hidden[rows[t]] + bias, one dot product per row."""
    return [math.fsum(hk * wk for hk, wk in zip(hidden[r], w_value)) + bias for r in rows]


# --------------------------------------------------------------------------
# Successive batching (Sec. 3.2 first paragraph, Alg. 1 line 2): a constant
# number K of slots; a sequence that reached an ending condition is removed
# before the next step and a new prompt takes its place, unfinished ones stay.
# --------------------------------------------------------------------------
class SuccessiveBatch:
    """Book-keeping of the slots across steps.  A sequence ends when it emits
    the end-of-sequence token or when its response reaches ``max_response``
    tokens (the actual maximum response length L; the window length l bounds
    what one step may add)."""

    def __init__(self, slots, window, max_response):
        self.window, self.max_response = window, max_response
        self.seq = [None] * slots          # per slot: dict(id, prompt, ctx, win, done) or None
        self.next_id = 0

    def refill(self, prompt_lens):
        """Put new prompts into empty slots (and slots whose sequence is finished),
        in slot order; returns how many prompts were taken."""
        taken = 0
        for k in range(len(self.seq)):
            s = self.seq[k]
            if (s is None or s["done"]) and taken < len(prompt_lens):
                self.seq[k] = dict(id=self.next_id, prompt=int(prompt_lens[taken]), ctx=int(prompt_lens[taken]),
                                   win=0, done=False)
                self.next_id += 1
                taken += 1
        return taken

    def advance(self, gen_len, eos):
        """One rollout window: slot k generated gen_len[k] tokens and (eos[k]) ended
        with the end-of-sequence token.  Tokens of the previous window become context."""
        for k, s in enumerate(self.seq):
            if s is None or s["done"]:
                raise ValueError("advance() on an empty or finished slot: refill first")
            g = int(gen_len[k])
            so_far = s["ctx"] + s["win"] - s["prompt"]
            if g < 0 or g > self.window or so_far + g > self.max_response:
                raise ValueError("window or maximum response length exceeded")
            if not eos[k] and g < self.window and so_far + g < self.max_response:
                raise ValueError("a sequence stops short of the window only by ending")
            s["ctx"] += s["win"]
            s["win"] = g
            s["done"] = bool(eos[k]) or so_far + g == self.max_response

    def layout(self):
        """(cu_seqlens, ctx_len, prompt_len, done, seq_id) of the current training batch."""
        cu, ctx, prompt, done, ids = [0], [], [], [], []
        for s in self.seq:
            cu.append(cu[-1] + s["ctx"] + s["win"])
            ctx.append(s["ctx"])
            prompt.append(s["prompt"])
            done.append(1 if s["done"] else 0)
            ids.append(s["id"])
        return cu, ctx, prompt, done, ids
