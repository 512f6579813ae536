"""CPU pins for the oracle: closed forms, special cases, hand-worked examples,
library routines and brute force.  None of these touches the GPU path."""
import math
import os

import numpy as np
import pytest
import scipy.signal
import scipy.special

from oracle import definitional as odef
from oracle import fast as ofast

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------ helpers
def _random_batch(rng, B, max_ctx=5, max_win=12, vocab=50):
    ctx = rng.integers(1, max_ctx + 1, size=B)
    win = rng.integers(1, max_win + 1, size=B)
    done = rng.integers(0, 2, size=B)
    cu = np.concatenate([[0], np.cumsum(ctx + win)])
    ids = rng.integers(0, vocab, size=cu[-1])
    return cu, ctx, win, done, ids


def _parse_cases(path):
    cases, cur = [], None
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, val = line.split(":", 1)
        if key == "case":
            cur = dict(name=val.strip())
            cases.append(cur)
        else:
            cur[key] = [float(x) for x in val.split()]
    return cases


# ------------------------------------------------------------------ select
@pytest.mark.parametrize("seed", range(5))
@pytest.mark.parametrize("tail_drop", [0, 1, 3, 100])
def test_select_fast_equals_definitional_and_invariants(seed, tail_drop):
    rng = np.random.default_rng(seed)
    cu, ctx, win, done, ids = _random_batch(rng, B=7)
    d = odef.select(cu, ctx, done, ids, tail_drop)
    f = ofast.select(cu, ctx, done, ids, tail_drop)
    for k in ("resp_off", "sel_off", "keep_len", "sel_rows", "sel_targets", "sel_resp_idx"):
        assert list(d[k]) == list(f[k]), k
    for k in ("M", "N_resp", "N_val"):
        assert d[k] == f[k]
    rows = np.asarray(f["sel_rows"], np.int64)
    tg = np.asarray(f["sel_targets"])
    # invariants fixed by Sec. 2.1 / Sec. 3.2
    assert f["M"] == int(np.sum(f["keep_len"])) == rows.shape[0]
    assert np.all(np.diff(rows) > 0)
    assert np.array_equal(tg, ids[rows + 1])
    last_rows = cu[1:] - 1
    assert not np.isin(rows, last_rows).any()        # nothing is predicted from the last token
    prompt_rows = np.concatenate([np.arange(cu[i], cu[i] + ctx[i] - 1) for i in range(7)])
    assert not np.isin(rows, prompt_rows).any()      # prompt tokens are never targets
    for i in range(7):
        if f["keep_len"][i] > 0:
            assert rows[f["sel_off"][i]] == cu[i] + ctx[i] - 1   # first kept row = last context position
        expect = win[i] if done[i] else max(win[i] - tail_drop, 0)
        assert f["keep_len"][i] == expect
    assert f["N_val"] == int(win[done != 0].sum())
    assert f["N_resp"] == int(win.sum())


def test_select_extremes():
    rng = np.random.default_rng(11)
    cu, ctx, win, done, ids = _random_batch(rng, B=6)
    all_done = np.ones(6, int)
    assert ofast.select(cu, ctx, all_done, ids, 5)["M"] == int(win.sum())
    none_done = np.zeros(6, int)
    assert ofast.select(cu, ctx, none_done, ids, int(win.max()))["M"] == 0
    assert ofast.select(cu, ctx, none_done, ids, 0)["M"] == int(win.sum())


# ------------------------------------------------------------------ log-probs
def test_bf16_decode_known_patterns():
    bits = np.array([0x3F80, 0xC000, 0x3DCC, 0x0000, 0xBF00], np.uint16)
    assert ofast.decode(bits).tolist() == [1.0, -2.0, 0.099609375, 0.0, -0.5]


def test_logprob_fast_equals_definitional_tiny():
    rng = np.random.default_rng(0)
    H, V, N = 5, 11, 9
    hidden = rng.normal(size=(N, H))
    w = rng.normal(size=(V, H))
    rows = [0, 3, 3, 8, 5]
    tg = [10, 0, 7, 4, 4]
    dl, dlse = odef.token_logprobs(hidden.tolist(), w.tolist(), rows, tg)
    fl, flse = ofast.token_logprobs(hidden, w, rows, tg, row_block=2, vocab_block=4)
    assert np.allclose(dl, fl, rtol=0, atol=1e-12)
    assert np.allclose(dlse, flse, rtol=0, atol=1e-12)


def test_logprob_matches_library_log_softmax():
    rng = np.random.default_rng(1)
    H, V, N = 16, 37, 20              # H != V and nothing symmetric: catches a transposed operand
    hidden = rng.normal(size=(N, H)).astype(np.float32)
    w = (0.5 * rng.normal(size=(V, H))).astype(np.float32)
    rows = rng.integers(0, N, size=50)
    tg = rng.integers(0, V, size=50)
    z = np.einsum("nh,vh->nv", hidden.astype(np.float64), w.astype(np.float64))
    ref = scipy.special.log_softmax(z, axis=1)[rows, tg]
    got, lse = ofast.token_logprobs(hidden, w, rows, tg, row_block=7, vocab_block=10)
    assert np.allclose(got, ref, rtol=0, atol=1e-12)
    assert np.allclose(lse, scipy.special.logsumexp(z, axis=1)[rows], rtol=0, atol=1e-12)


def test_logprob_closed_forms():
    rng = np.random.default_rng(2)
    H, V = 8, 13
    hidden = rng.normal(size=(4, H))
    # zero head: uniform distribution
    lp, lse = ofast.token_logprobs(hidden, np.zeros((V, H)), [0, 1, 2], [0, 5, 12])
    assert np.allclose(lp, -math.log(V), atol=1e-15)
    assert np.allclose(lse, math.log(V), atol=1e-15)
    # probabilities of one row over every target sum to one
    w = rng.normal(size=(V, H))
    lp, _ = ofast.token_logprobs(hidden, w, [2] * V, list(range(V)))
    assert abs(np.exp(lp).sum() - 1.0) < 1e-12
    lpd, _ = odef.token_logprobs(hidden.tolist(), w.tolist(), [2] * V, list(range(V)))
    assert abs(sum(math.exp(x) for x in lpd) - 1.0) < 1e-12
    # one dominant logit: log-prob tends to 0 for it, to -(gap) for the others
    w2 = np.zeros((V, H))
    w2[3] = 50.0 * hidden[1] / np.dot(hidden[1], hidden[1])     # logit 50 at v=3, 0 elsewhere
    lp, _ = ofast.token_logprobs(hidden, w2, [1, 1], [3, 4])
    assert abs(lp[0]) < 1e-15 * 1e6
    assert abs(lp[1] + 50.0) < 1e-9
    # large logits do not overflow (max is subtracted)
    lp, _ = ofast.token_logprobs(hidden, 1e3 * w, [0], [1])
    assert np.isfinite(lp).all()


def test_logprob_bf16_inputs_are_used_exactly():
    # bf16 bit patterns must decode to the same values as their fp32 images
    from paper_2506_15050_amd import synth
    rng = np.random.default_rng(3)
    h32 = rng.normal(size=(6, 8)).astype(np.float32)
    w32 = rng.normal(size=(9, 8)).astype(np.float32)
    hb, wb = synth.f32_to_bf16_bits(h32), synth.f32_to_bf16_bits(w32)
    a, _ = ofast.token_logprobs(hb, wb, [0, 5], [1, 8])
    b, _ = ofast.token_logprobs(synth.bf16_bits_to_f32(hb), synth.bf16_bits_to_f32(wb), [0, 5], [1, 8])
    assert np.array_equal(a, b)


# ------------------------------------------------------------------ EGAE
@pytest.mark.parametrize("case", _parse_cases(os.path.join(GOLDEN, "egae_worked_examples.txt")),
                         ids=lambda c: c["name"])
def test_egae_worked_examples(case):
    g, lam, done = case["gamma"][0], case["lam"][0], int(case["done"][0])
    boot = case.get("bootstrap", [None])[0]
    v, r = case["values"], case["rewards"]
    assert np.allclose(odef.td_residuals(r, v, bool(done), g, boot), case["delta"], atol=1e-12)
    a, ret = odef.egae_sequence(r, v, bool(done), g, lam, boot)
    assert np.allclose(a, case["adv"], atol=1e-12) and np.allclose(ret, case["ret"], atol=1e-12)
    off = [0, len(v)]
    fa, fr = ofast.egae(np.array(r), np.array(v), off, [done], g, lam,
                        None if boot is None else [boot])
    assert np.allclose(fa, case["adv"], atol=1e-12) and np.allclose(fr, case["ret"], atol=1e-12)


def _random_resp(rng, B, max_len=40):
    lens = rng.integers(1, max_len + 1, size=B)
    off = np.concatenate([[0], np.cumsum(lens)])
    n = int(off[-1])
    return off, rng.normal(size=n), rng.uniform(-1, 1, size=n), rng.integers(0, 2, size=B)


@pytest.mark.parametrize("gamma,lam", [(1.0, 0.95), (0.99, 0.9), (1.0, 1.0), (1.0, 0.0), (0.5, 0.5)])
def test_egae_fast_equals_double_sum(gamma, lam):
    rng = np.random.default_rng(4)
    off, r, v, done = _random_resp(rng, 9)
    boot = rng.uniform(-1, 1, size=9)
    for b in (None, boot):
        da, dr = odef.egae(r, v, off, done, gamma, lam, b)
        fa, fr = ofast.egae(r, v, off, done, gamma, lam, b)
        assert np.allclose(da, fa, rtol=0, atol=1e-12)
        assert np.allclose(dr, fr, rtol=0, atol=1e-12)


def _textbook_gae_lfilter(r, v, gamma, lam):
    """GAE of a finished episode through a library IIR filter: reversed in
    time, A[n] = delta[n] + c*A[n-1] is ``lfilter([1], [1, -c])``."""
    v_next = np.append(v[1:], 0.0)
    delta = r + gamma * v_next - v
    adv = scipy.signal.lfilter([1.0], [1.0, -gamma * lam], delta[::-1])[::-1]
    ret = scipy.signal.lfilter([1.0], [1.0, -gamma], r[::-1])[::-1]
    return adv, ret


@pytest.mark.parametrize("gamma,lam", [(1.0, 0.95), (0.97, 0.8)])
def test_complete_responses_reduce_to_standard_gae(gamma, lam):
    rng = np.random.default_rng(5)
    off, r, v, _ = _random_resp(rng, 6, max_len=200)
    done = np.ones(6, int)
    fa, fr = ofast.egae(r, v, off, done, gamma, lam)
    for i in range(6):
        a, ret = _textbook_gae_lfilter(r[off[i]:off[i + 1]], v[off[i]:off[i + 1]], gamma, lam)
        assert np.allclose(fa[off[i]:off[i + 1]], a, rtol=0, atol=1e-11)
        assert np.allclose(fr[off[i]:off[i + 1]], ret, rtol=0, atol=1e-11)


def test_egae_special_cases():
    rng = np.random.default_rng(6)
    off, r, v, done = _random_resp(rng, 8, max_len=60)
    n = int(off[-1])
    last = off[1:] - 1
    # lambda = 0: one-step TD residual
    a, _ = ofast.egae(r, v, off, done, 0.9, 0.0)
    v_next = np.append(v[1:], 0.0)
    v_next[last] = np.where(done != 0, 0.0, v[last])
    assert np.allclose(a, r + 0.9 * v_next - v, atol=1e-13)
    # gamma = lambda = 1: finished -> return minus value; truncated -> observed
    # rewards plus the bootstrap (= last value) minus value
    a, ret = ofast.egae(r, v, off, done, 1.0, 1.0)
    for i in range(8):
        s = slice(off[i], off[i + 1])
        tail_sum = np.cumsum(r[s][::-1])[::-1]
        assert np.allclose(ret[s], tail_sum, atol=1e-12)
        if done[i]:
            assert np.allclose(a[s], ret[s] - v[s], atol=1e-12)
        else:
            assert np.allclose(a[s], tail_sum + v[last[i]] - v[s], atol=1e-12)
    # constant value, no reward, truncated, gamma = 1: every residual vanishes
    a, ret = ofast.egae(np.zeros(n), np.full(n, 0.37), off, np.zeros(8, int), 1.0, 0.95)
    assert np.all(a == 0.0) and np.all(ret == 0.0)
    # zero intermediate reward, gamma = 1: last token of a truncated sequence has advantage 0
    a, _ = ofast.egae(np.zeros(n), v, off, np.zeros(8, int), 1.0, 0.95)
    assert np.all(a[last] == 0.0)


def test_egae_bootstrap_equivalence_and_sensitivity():
    rng = np.random.default_rng(7)
    off, r, v, _ = _random_resp(rng, 5, max_len=50)
    gamma, lam = 0.98, 0.9
    trunc = np.zeros(5, int)
    boot = rng.uniform(-1, 1, size=5)
    last = off[1:] - 1
    a_b, ret_b = ofast.egae(r, v, off, trunc, gamma, lam, boot)
    # EGAE with bootstrap b == finished-episode GAE with gamma*b added to the last reward
    r2 = r.copy()
    r2[last] += gamma * boot
    a_g, _ = ofast.egae(r2, v, off, np.ones(5, int), gamma, lam)
    assert np.allclose(a_b, a_g, atol=1e-12)
    # default bootstrap is the last value (Sec. 3.1)
    a_default, _ = ofast.egae(r, v, off, trunc, gamma, lam)
    a_explicit, _ = ofast.egae(r, v, off, trunc, gamma, lam, v[last])
    assert np.array_equal(a_default, a_explicit)
    # bootstrap is ignored for finished sequences, and never enters the return
    a_done, ret_done = ofast.egae(r, v, off, np.ones(5, int), gamma, lam, boot)
    a_done0, ret_done0 = ofast.egae(r, v, off, np.ones(5, int), gamma, lam)
    assert np.array_equal(a_done, a_done0) and np.array_equal(ret_b, ret_done0)
    # the cut is forgotten geometrically: d A_t / d b = gamma (gamma lam)^(l-1-t)
    a_b2, _ = ofast.egae(r, v, off, trunc, gamma, lam, boot + 0.25)
    for i in range(5):
        l = off[i + 1] - off[i]
        t = np.arange(l)
        expect = gamma * (gamma * lam) ** (l - 1 - t) * 0.25
        assert np.allclose((a_b2 - a_b)[off[i]:off[i + 1]], expect, atol=1e-12)


def test_egae_segment_independence():
    rng = np.random.default_rng(8)
    off, r, v, done = _random_resp(rng, 6)
    a, ret = ofast.egae(r, v, off, done, 1.0, 0.95)
    for i in range(6):
        s = slice(off[i], off[i + 1])
        ai, ri = ofast.egae(r[s], v[s], [0, off[i + 1] - off[i]], [done[i]], 1.0, 0.95)
        assert np.array_equal(a[s], ai) and np.array_equal(ret[s], ri)


# ------------------------------------------------------------------ losses
def _loss_golden():
    pol, val, exp = [], [], {}
    for line in open(os.path.join(GOLDEN, "loss_worked_examples.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, v = line.split(":")
        nums = [float(x) for x in v.split()]
        if key == "policy":
            pol.append(nums)
        elif key == "value":
            val.append(nums)
        else:
            exp[key] = nums[0]
    return np.array(pol), np.array(val), exp


@pytest.mark.parametrize("impl", [odef, ofast], ids=["definitional", "fast"])
def test_loss_worked_examples(impl):
    pol, val, exp = _loss_golden()
    n = len(pol)
    assert len(val) == n
    zeros = np.zeros(n)
    # per-token terms, one token at a time
    for k in range(n):
        out = impl.ppo_losses([math.log(pol[k, 1])], [0.0], [pol[k, 0]],
                              [val[k, 0]], [val[k, 1]], [val[k, 2]],
                              [0, 1], [1], [1], 0.2, 0.28, 0.5, 0.6)
        assert abs(out["policy_loss"] + pol[k, 2]) < 1e-12
        assert abs(out["value_loss"] - 0.5 * val[k, 3]) < 1e-12
    out = impl.ppo_losses(np.log(pol[:, 1]), zeros, pol[:, 0], val[:, 0], val[:, 1], val[:, 2],
                          [0, n], [n], [1], 0.2, 0.28, 0.5, 0.6)
    assert abs(out["policy_loss"] - exp["policy_loss"]) < 1e-12
    assert abs(out["value_loss"] - exp["value_loss"]) < 1e-12
    assert out["n_policy"] == n and out["n_value"] == n


def _random_loss_inputs(rng, B=7, max_len=30):
    lens = rng.integers(1, max_len + 1, size=B)
    off = np.concatenate([[0], np.cumsum(lens)])
    n = int(off[-1])
    done = rng.integers(0, 2, size=B)
    keep = np.where(done != 0, lens, np.maximum(lens - 5, 0))
    arrs = dict(logp_new=-np.abs(rng.normal(size=n)), adv=rng.normal(size=n),
                v_new=rng.normal(size=n), ret=rng.normal(size=n))
    arrs["logp_old"] = arrs["logp_new"] + rng.normal(0, 0.3, size=n)
    arrs["v_old"] = arrs["v_new"] + rng.normal(0, 0.6, size=n)
    return off, keep, done, arrs


def _call(impl, a, off, keep, done, eps=(0.2, 0.28), xi=(0.5, 0.6)):
    return impl.ppo_losses(a["logp_new"], a["logp_old"], a["adv"], a["v_new"], a["v_old"],
                           a["ret"], off, keep, done, eps[0], eps[1], xi[0], xi[1])


def test_losses_fast_equals_definitional():
    rng = np.random.default_rng(9)
    off, keep, done, a = _random_loss_inputs(rng)
    d, f = _call(odef, a, off, keep, done), _call(ofast, a, off, keep, done)
    for k in d:
        assert abs(d[k] - f[k]) <= 1e-12 * max(1.0, abs(d[k])), k


def test_losses_closed_forms_masks_and_additivity():
    rng = np.random.default_rng(10)
    off, keep, done, a = _random_loss_inputs(rng, B=9)
    pol, val = ofast.loss_masks(off, keep, done)
    assert pol.sum() == keep.sum() and val.sum() == (off[1:] - off[:-1])[done != 0].sum()
    # same policy: ratio 1, loss is minus the mean advantage over the policy set
    b = dict(a, logp_old=a["logp_new"].copy(), v_old=a["v_new"].copy())
    out = _call(ofast, b, off, keep, done)
    assert abs(out["policy_loss"] + a["adv"][pol].mean()) < 1e-12
    # same value function: clip is a no-op, plain half mean squared error
    assert abs(out["value_loss"] - 0.5 * ((a["v_new"] - a["ret"])[val] ** 2).mean()) < 1e-12
    # masked-out entries contribute exactly zero, whatever they hold
    ref = _call(ofast, a, off, keep, done)
    c = {k: v.copy() for k, v in a.items()}
    for k in ("logp_new", "logp_old", "adv"):
        c[k][~pol] = np.nan
    for k in ("v_new", "v_old", "ret"):
        c[k][~val] = np.inf
    poisoned = _call(ofast, c, off, keep, done)
    assert poisoned == ref
    assert _call(odef, c, off, keep, done)["policy_loss"] == pytest.approx(ref["policy_loss"], abs=1e-12)
    # additivity of the un-normalised sums over a split batch
    k = 4
    cut = off[k]
    first = {n_: v[:cut] for n_, v in a.items()}
    second = {n_: v[cut:] for n_, v in a.items()}
    o1 = _call(ofast, first, off[:k + 1], keep[:k], done[:k])
    o2 = _call(ofast, second, off[k:] - cut, keep[k:], done[k:])
    assert abs(o1["policy_sum"] + o2["policy_sum"] - ref["policy_sum"]) < 1e-11
    assert abs(o1["value_sum"] + o2["value_sum"] - ref["value_sum"]) < 1e-11
    assert o1["n_policy"] + o2["n_policy"] == ref["n_policy"]
    assert o1["n_value"] + o2["n_value"] == ref["n_value"]


def test_losses_empty_sets():
    out = ofast.ppo_losses(np.zeros(3), np.zeros(3), np.ones(3), np.zeros(3), np.zeros(3),
                           np.ones(3), [0, 3], [0], [0], 0.2, 0.28, 0.5, 0.6)
    assert out["policy_loss"] == 0.0 and out["value_loss"] == 0.0
    assert out["n_policy"] == 0 and out["n_value"] == 0
    out = odef.ppo_losses([], [], [], [], [], [], [0], [], [], 0.2, 0.28, 0.5, 0.6)
    assert out["policy_loss"] == 0.0 and out["value_loss"] == 0.0


def test_clip_is_asymmetric():
    # ratio 1.25 is inside [0.8, 1.28] but outside [0.8, 1.2]
    args = ([math.log(1.25)], [0.0], [1.0], [0.0], [0.0], [0.0], [0, 1], [1], [1])
    assert ofast.ppo_losses(*args, 0.2, 0.28, 0.5, 0.6)["policy_loss"] == pytest.approx(-1.25)
    assert ofast.ppo_losses(*args, 0.2, 0.2, 0.5, 0.6)["policy_loss"] == pytest.approx(-1.2)
    # value 0.55 above v_old is inside +0.6 but would be outside +0.5
    vargs = ([0.0], [0.0], [0.0], [0.55], [0.0], [2.0], [0, 1], [1], [1])
    assert ofast.ppo_losses(*vargs, 0.2, 0.28, 0.5, 0.6)["value_loss"] == pytest.approx(0.5 * 1.45 ** 2)
    assert ofast.ppo_losses(*vargs, 0.2, 0.28, 0.6, 0.5)["value_loss"] == pytest.approx(0.5 * 1.5 ** 2)


# ------------------------------------------------------------------ loss derivatives
def _grad_call(impl, a, off, keep, done, eps=(0.2, 0.28), xi=(0.5, 0.6), **kw):
    return impl.ppo_loss_grads(a["logp_new"], a["logp_old"], a["adv"], a["v_new"], a["v_old"],
                               a["ret"], off, keep, done, eps[0], eps[1], xi[0], xi[1], **kw)


def _loss_grad_golden():
    pol, val, exp = [], [], {}
    for line in open(os.path.join(GOLDEN, "loss_grad_worked_examples.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, v = line.split(":")
        nums = [float(x) for x in v.split()]
        if key == "policy":
            pol.append(nums)
        elif key == "value":
            val.append(nums)
        else:
            exp[key] = nums[0]
    return np.array(pol), np.array(val), exp


@pytest.mark.parametrize("impl", [odef, ofast], ids=["definitional", "fast"])
def test_loss_grad_worked_examples(impl):
    pol, val, exp = _loss_grad_golden()
    n = len(pol)
    out = impl.ppo_loss_grads(np.log(pol[:, 1]), np.zeros(n), pol[:, 0], val[:, 0], val[:, 1], val[:, 2],
                              [0, n], [n], [1], 0.2, 0.28, 0.5, 0.6)
    assert np.allclose(np.asarray(out["grad_logp"]) * n, pol[:, 2], rtol=0, atol=1e-12)
    assert np.allclose(np.asarray(out["grad_v"]) * n, val[:, 3], rtol=0, atol=1e-12)
    assert out["n_policy_clipped"] == int(pol[:, 3].sum()) and out["n_value_clipped"] == int(val[:, 4].sum())
    assert abs(out["ratio_mean"] - exp["ratio_mean"]) < 1e-12
    # scales multiply, denominators replace the token counts
    out2 = impl.ppo_loss_grads(np.log(pol[:, 1]), np.zeros(n), pol[:, 0], val[:, 0], val[:, 1], val[:, 2],
                               [0, n], [n], [1], 0.2, 0.28, 0.5, 0.6, policy_scale=2.0, value_scale=-3.0,
                               policy_denominator=10, value_denominator=20)
    assert np.allclose(np.asarray(out2["grad_logp"]) * 10 / 2.0, pol[:, 2], rtol=0, atol=1e-12)
    assert np.allclose(np.asarray(out2["grad_v"]) * 20 / -3.0, val[:, 3], rtol=0, atol=1e-12)


def test_loss_grads_fast_equals_definitional():
    rng = np.random.default_rng(21)
    off, keep, done, a = _random_loss_inputs(rng)
    d, f = _grad_call(odef, a, off, keep, done), _grad_call(ofast, a, off, keep, done)
    for k in ("grad_logp", "grad_v"):
        assert np.allclose(np.asarray(d[k]), f[k], rtol=1e-13, atol=1e-15), k
    for k in ("n_policy", "n_value", "n_policy_clipped", "n_value_clipped"):
        assert d[k] == f[k], k
    assert abs(d["ratio_mean"] - f["ratio_mean"]) < 1e-13


def test_loss_grads_match_autograd():
    """The derivative formulas against reverse-mode differentiation of the loss
    written with library tensor ops (an independent mechanism: nothing of the
    branch analysis is shared)."""
    import torch
    rng = np.random.default_rng(22)
    off, keep, done, a = _random_loss_inputs(rng, B=11, max_len=40)
    pol, val = ofast.loss_masks(off, keep, done)
    ln = torch.tensor(a["logp_new"], dtype=torch.float64, requires_grad=True)
    v = torch.tensor(a["v_new"], dtype=torch.float64, requires_grad=True)
    lo_, adv, vo, r = (torch.tensor(a[k], dtype=torch.float64) for k in ("logp_old", "adv", "v_old", "ret"))
    pm, vm = torch.tensor(pol), torch.tensor(val)
    rho = torch.exp(ln - lo_)
    surr = torch.minimum(rho * adv, torch.clamp(rho, 0.8, 1.28) * adv)
    policy_loss = -(surr[pm]).sum() / int(pol.sum())
    v_clip = torch.maximum(torch.minimum(v, vo + 0.6), vo - 0.5)
    value_loss = 0.5 * torch.maximum((v - r) ** 2, (v_clip - r) ** 2)[vm].sum() / int(val.sum())
    (1.7 * policy_loss - 0.4 * value_loss).backward()
    out = _grad_call(ofast, a, off, keep, done, policy_scale=1.7, value_scale=-0.4)
    assert np.allclose(out["grad_logp"], ln.grad.numpy(), rtol=1e-12, atol=1e-15)
    assert np.allclose(out["grad_v"], v.grad.numpy(), rtol=1e-12, atol=1e-15)
    assert np.all(out["grad_logp"][~pol] == 0.0) and np.all(out["grad_v"][~val] == 0.0)
    assert out["n_policy_clipped"] > 0 and out["n_value_clipped"] > 0       # both branches exercised
    assert out["n_policy_clipped"] < pol.sum() and out["n_value_clipped"] < val.sum()


def test_loss_grads_match_finite_differences_of_the_pinned_loss():
    rng = np.random.default_rng(23)
    off, keep, done, a = _random_loss_inputs(rng, B=4, max_len=8)
    g = _grad_call(odef, a, off, keep, done)
    h = 1e-6
    for name, key, loss in (("logp_new", "grad_logp", "policy_loss"), ("v_new", "grad_v", "value_loss")):
        for j in range(len(a[name])):
            up, dn = {k: x.copy() for k, x in a.items()}, {k: x.copy() for k, x in a.items()}
            up[name][j] += h
            dn[name][j] -= h
            fd = (_call(odef, up, off, keep, done)[loss] - _call(odef, dn, off, keep, done)[loss]) / (2 * h)
            assert abs(fd - g[key][j]) < 1e-7, (name, j)     # kinks have measure zero for these draws


def test_loss_grads_masks_poison_and_counts():
    rng = np.random.default_rng(24)
    off, keep, done, a = _random_loss_inputs(rng, B=9)
    pol, val = ofast.loss_masks(off, keep, done)
    ref = _grad_call(ofast, a, off, keep, done)
    c = {k: v.copy() for k, v in a.items()}
    for k in ("logp_new", "logp_old", "adv"):
        c[k][~pol] = np.nan
    for k in ("v_new", "v_old", "ret"):
        c[k][~val] = np.inf
    out = _grad_call(ofast, c, off, keep, done)
    assert np.array_equal(out["grad_logp"], ref["grad_logp"]) and np.array_equal(out["grad_v"], ref["grad_v"])
    # same policy and same value function: nothing is clipped, ratio 1
    b = dict(a, logp_old=a["logp_new"].copy(), v_old=a["v_new"].copy())
    same = _grad_call(ofast, b, off, keep, done)
    assert same["n_policy_clipped"] == 0 and same["n_value_clipped"] == 0 and same["ratio_mean"] == 1.0
    assert np.allclose(same["grad_logp"][pol], -a["adv"][pol] / pol.sum(), rtol=1e-13)
    assert np.allclose(same["grad_v"][val], (a["v_new"] - a["ret"])[val] / val.sum(), rtol=1e-13)
    # empty sets
    e = ofast.ppo_loss_grads(np.zeros(3), np.zeros(3), np.ones(3), np.zeros(3), np.zeros(3), np.ones(3),
                             [0, 3], [0], [0], 0.2, 0.28, 0.5, 0.6)
    assert not e["grad_logp"].any() and not e["grad_v"].any() and e["ratio_mean"] == 0.0


# ------------------------------------------------------------------ log-prob derivatives
def _head_case(rng, M=7, n_rows=9, V=11, H=5):
    hidden = rng.normal(size=(n_rows, H))
    w = rng.normal(0, 0.5, size=(V, H))
    rows = rng.integers(0, n_rows, size=M)
    tg = rng.integers(0, V, size=M)
    g = rng.normal(size=M)
    return hidden, w, rows, tg, g


def test_logprob_grads_fast_equals_definitional():
    hidden, w, rows, tg, g = _head_case(np.random.default_rng(31))
    dh_d, dw_d = odef.token_logprob_grads(hidden.tolist(), w.tolist(), rows.tolist(), tg.tolist(), g.tolist())
    dh_f, dw_f = ofast.token_logprob_grads(hidden, w, rows, tg, g)
    assert np.allclose(dh_f, np.array(dh_d), rtol=1e-12, atol=1e-14)
    assert np.allclose(dw_f, np.array(dw_d), rtol=1e-12, atol=1e-14)


def test_logprob_grads_match_autograd():
    import torch
    hidden, w, rows, tg, g = _head_case(np.random.default_rng(32), M=13, n_rows=13, V=17, H=6)
    rows = np.arange(13)                                   # distinct rows: row derivative = hidden derivative
    ht = torch.tensor(hidden, dtype=torch.float64, requires_grad=True)
    wt = torch.tensor(w, dtype=torch.float64, requires_grad=True)
    logp = torch.log_softmax(ht[torch.tensor(rows)] @ wt.T, dim=1)[torch.arange(13), torch.tensor(tg)]
    (logp * torch.tensor(g)).sum().backward()
    dh, dw = ofast.token_logprob_grads(hidden, w, rows, tg, g)
    assert np.allclose(dh, ht.grad.numpy(), rtol=1e-12, atol=1e-14)
    assert np.allclose(dw, wt.grad.numpy(), rtol=1e-12, atol=1e-14)


def test_logprob_grads_match_finite_differences_of_the_pinned_forward():
    hidden, w, rows, tg, g = _head_case(np.random.default_rng(33), M=4, n_rows=4, V=6, H=3)
    rows = np.arange(4)
    dh, dw = ofast.token_logprob_grads(hidden, w, rows, tg, g)
    eps = 1e-6

    def loss(hid, wm):
        lp, _ = ofast.token_logprobs(hid, wm, rows, tg)
        return float((lp * g).sum())
    for t in range(4):
        for k in range(3):
            up, dn = hidden.copy(), hidden.copy()
            up[t, k] += eps
            dn[t, k] -= eps
            assert abs((loss(up, w) - loss(dn, w)) / (2 * eps) - dh[t, k]) < 1e-8
    for v in range(6):
        for k in range(3):
            up, dn = w.copy(), w.copy()
            up[v, k] += eps
            dn[v, k] -= eps
            assert abs((loss(hidden, up) - loss(hidden, dn)) / (2 * eps) - dw[v, k]) < 1e-8


def test_logprob_grads_closed_forms_and_invariants():
    rng = np.random.default_rng(34)
    hidden, w, rows, tg, g = _head_case(rng, M=9, n_rows=5, V=8, H=4)       # rows repeat
    dh, dw, abs_h, abs_w = ofast.token_logprob_grads(hidden, w, rows, tg, g, return_abs_bounds=True)
    # softmax derivative sums to zero over the vocabulary: so do the columns of grad_w
    assert np.allclose(dw.sum(axis=0), 0.0, atol=1e-13)
    assert np.all(np.abs(dh) <= abs_h + 1e-15) and np.all(np.abs(dw) <= abs_w + 1e-15)
    # zero head matrix: uniform softmax, grad_hidden = 0, grad_w[v] = sum_t g_t ([v = a_t] - 1/V) h_t
    dh0, dw0 = ofast.token_logprob_grads(hidden, np.zeros_like(w), rows, tg, g)
    assert not dh0.any()
    expect = np.zeros_like(w)
    for t in range(9):
        for v in range(8):
            expect[v] += g[t] * ((1.0 if v == tg[t] else 0.0) - 1.0 / 8) * hidden[rows[t]]
    assert np.allclose(dw0, expect, rtol=1e-13, atol=1e-15)
    # a vocabulary of one entry: log-prob is identically 0, every derivative vanishes
    dh1, dw1 = ofast.token_logprob_grads(hidden, w[:1], rows, np.zeros(9, int), g)
    assert np.allclose(dh1, 0.0, atol=1e-15) and np.allclose(dw1, 0.0, atol=1e-15)
    # linear in g; tokens with g = 0 contribute nothing
    dh2, dw2 = ofast.token_logprob_grads(hidden, w, rows, tg, 2.0 * g)
    assert np.allclose(dh2, 2 * dh) and np.allclose(dw2, 2 * dw)
    gz = g.copy()
    gz[3:] = 0.0
    dh3, dw3 = ofast.token_logprob_grads(hidden, w, rows, tg, gz)
    dh4, dw4 = ofast.token_logprob_grads(hidden, w, rows[:3], tg[:3], g[:3])
    assert np.allclose(dh3[:3], dh4) and not dh3[3:].any() and np.allclose(dw3, dw4)
    # bf16 inputs are decoded, not cast
    from paper_2506_15050_amd.synth import f32_to_bf16_bits
    hb, wb = f32_to_bf16_bits(hidden.astype(np.float32)), f32_to_bf16_bits(w.astype(np.float32))
    dh5, dw5 = ofast.token_logprob_grads(hb, wb, rows, tg, g)
    dh6, dw6 = ofast.token_logprob_grads(ofast.decode(hb), ofast.decode(wb), rows, tg, g)
    assert np.array_equal(dh5, dh6) and np.array_equal(dw5, dw6)


# ------------------------------------------------------------------ value head
def test_value_head_definition_and_closed_forms():
    rng = np.random.default_rng(41)
    hidden = rng.normal(size=(9, 16))
    w = rng.normal(size=16)
    rows = rng.integers(0, 9, size=13)
    d = odef.value_head(hidden.tolist(), w.tolist(), 0.25, rows.tolist())
    f, bound = ofast.value_head(hidden, w, 0.25, rows, return_abs_bound=True)
    assert np.allclose(f, d, rtol=1e-14, atol=1e-15)
    assert np.all(np.abs(f - 0.25) <= bound + 1e-15)
    # a unit weight vector picks one column; all-ones sums the row; the bias is added once
    e3 = np.zeros(16)
    e3[3] = 1.0
    assert np.array_equal(ofast.value_head(hidden, e3, 0.0, rows), hidden[rows, 3])
    ones = ofast.value_head(hidden, np.ones(16), 1.5, rows)
    assert np.allclose(ones, [math.fsum(hidden[r]) + 1.5 for r in rows], rtol=1e-14)
    # linear in the weights
    w2 = rng.normal(size=16)
    assert np.allclose(ofast.value_head(hidden, w + 2 * w2, 0.0, rows),
                       ofast.value_head(hidden, w, 0.0, rows) + 2 * ofast.value_head(hidden, w2, 0.0, rows))
    # bf16 bit patterns are decoded
    from paper_2506_15050_amd.synth import f32_to_bf16_bits
    hb, wb = f32_to_bf16_bits(hidden.astype(np.float32)), f32_to_bf16_bits(w.astype(np.float32))
    assert np.array_equal(ofast.value_head(hb, wb, 0.0, rows),
                          ofast.value_head(ofast.decode(hb), ofast.decode(wb), 0.0, rows))


# ------------------------------------------------------------------ successive batching
def test_successive_batching_paper_example():
    rows = {}
    for line in open(os.path.join(GOLDEN, "successive_batching_example.txt")):
        line = line.strip()
        if line and not line.startswith("#"):
            k, v = line.split(":")
            rows[k] = [int(x) for x in v.split()]
    sb = odef.SuccessiveBatch(slots=5, window=8, max_response=24)
    assert sb.refill([3, 4, 5, 6, 7, 8, 9]) == 5                      # only five slots: two prompts wait
    assert sb.layout()[4] == rows["step0"]
    eos = [1 if k in rows["finished0"] else 0 for k in range(5)]
    sb.advance([8, 8, 5, 2, 8], eos)
    assert [k for k, d in enumerate(sb.layout()[3]) if d] == rows["finished0"]
    assert sb.refill([8, 9]) == 2
    assert sb.layout()[4] == rows["step1"]


def test_successive_batching_worked_example():
    """Three steps worked by hand (lengths included): context accumulation, both ending rules,
    refill order and id numbering, and the calls the rules forbid."""
    g = {}
    for line in open(os.path.join(GOLDEN, "successive_batching_worked.txt")):
        line = line.strip()
        if line and not line.startswith("#"):
            k, v = line.split(":")
            g[k] = [int(x) for x in v.split()]
    sb = odef.SuccessiveBatch(g["slots"][0], g["window"][0], g["max_response"][0])
    for step in (1, 2, 3):
        assert sb.refill(g[f"refill{step - 1}"]) == g[f"taken{step - 1}"][0]
        if step == 1:
            with pytest.raises(ValueError):
                sb.advance([5, 4, 4], [0, 0, 0])                    # one step adds at most `window` tokens
        sb.advance(g[f"gen{step}"], g[f"eos{step}"])
        cu, ctx, prompt, done, ids = sb.layout()
        assert [list(map(int, x)) for x in (cu, ctx, prompt, done, ids)] == \
               [g[f"cu{step}"], g[f"ctx{step}"], g[f"prompt{step}"], g[f"done{step}"], g[f"ids{step}"]], step
    # value tokens of the sequence that ended at the maximum length: its whole response, 10 tokens over 3 windows
    assert cu[1] - cu[0] - prompt[0] == 10 and done[0] == 1 and g["eos3"][0] == 0
    with pytest.raises(ValueError):
        sb.advance([1, 1, 1], [0, 0, 0])                            # slots 0 and 2 hold ended sequences
    sb.refill([4, 4])
    with pytest.raises(ValueError):
        sb.advance([4, 3, 4], [0, 0, 0])                            # slot 1 would pass max_response (8 + 3)
    with pytest.raises(ValueError):
        sb.advance([3, 2, 4], [0, 1, 0])                            # slot 0 stops short of the window without ending
    sb.advance([4, 2, 4], [0, 0, 0])                                # slot 1 reaches max_response exactly
    assert list(sb.layout()[3]) == [0, 1, 0]


def test_nan_inside_a_set_makes_the_loss_and_its_derivative_nan():
    """The paper is silent on inputs that are not numbers.  Reading: inside a token set a NaN is never
    clipped away -- the term and its derivative are NaN, the token counts towards N but is neither
    clipped nor unclipped; outside the sets it still cannot reach anything."""
    rng = np.random.default_rng(61)
    off, keep, done, a = _random_loss_inputs(rng, B=9)
    pol, val = ofast.loss_masks(off, keep, done)
    for impl in (odef, ofast):
        clean, gclean = _call(impl, a, off, keep, done), _grad_call(impl, a, off, keep, done)
        for key, mask, bad, good, gkey, gother in (
                ("logp_new", pol, "policy_loss", "value_loss", "grad_logp", "grad_v"),
                ("logp_old", pol, "policy_loss", "value_loss", "grad_logp", "grad_v"),
                ("adv", pol, "policy_loss", "value_loss", "grad_logp", "grad_v"),
                ("v_new", val, "value_loss", "policy_loss", "grad_v", "grad_logp"),
                ("v_old", val, "value_loss", "policy_loss", "grad_v", "grad_logp"),
                ("ret", val, "value_loss", "policy_loss", "grad_v", "grad_logp")):
            j = int(np.flatnonzero(mask)[3])
            c = {k: np.array(v, dtype=np.float64) for k, v in a.items()}
            c[key][j] = np.nan
            out, g = _call(impl, c, off, keep, done), _grad_call(impl, c, off, keep, done)
            assert math.isnan(out[bad]) and out[good] == clean[good], (key, out)
            assert out["n_policy"] == clean["n_policy"] and out["n_value"] == clean["n_value"]
            gv, gc = np.asarray(g[gkey], dtype=np.float64), np.asarray(gclean[gkey], dtype=np.float64)
            assert math.isnan(gv[j]), key
            others = np.arange(gv.size) != j
            assert np.array_equal(gv[others], gc[others])
            assert np.array_equal(np.asarray(g[gother]), np.asarray(gclean[gother]))
            # the undefined token leaves the clipped counts of everybody else alone
            was_clipped = gc[j] == 0.0
            n_key = "n_policy_clipped" if gkey == "grad_logp" else "n_value_clipped"
            assert g[n_key] == gclean[n_key] - (1 if was_clipped else 0)


def test_successive_batching_invariants():
    rng = np.random.default_rng(51)
    K, l, L = 6, 8, 24
    sb = odef.SuccessiveBatch(K, l, L)
    sb.refill(rng.integers(1, 9, size=K))
    trained_policy = {}                                              # seq id -> response tokens seen by the policy
    finished = {}
    for step in range(12):
        cu, ctx, prompt, done, ids = sb.layout()
        gen, eos = [], []
        for k in range(K):
            so_far = ctx[k] - prompt[k] + (cu[k + 1] - cu[k] - ctx[k])
            room = min(l, L - so_far)
            stop = rng.random() < 0.3
            g = int(rng.integers(1, room + 1)) if stop else room
            gen.append(g)
            eos.append(1 if stop else 0)
        sb.advance(gen, eos)
        cu, ctx, prompt, done, ids = sb.layout()
        assert len(ids) == K and len(set(ids)) == K                 # constant batch, no duplicates
        for k in range(K):
            win = cu[k + 1] - cu[k] - ctx[k]
            assert win == gen[k] and 0 < win <= l
            trained_policy[ids[k]] = trained_policy.get(ids[k], 0) + win
            resp = ctx[k] + win - prompt[k]
            assert resp <= L and trained_policy[ids[k]] == resp      # every response token is in exactly one window
            if done[k]:
                assert eos[k] or resp == L
                finished[ids[k]] = resp                              # value tokens: the whole response
            else:
                assert win == l                                      # unfinished sequences fill the window
        sb.refill(rng.integers(1, 9, size=sum(done)))
    assert len(finished) > K                                         # slots were reused
    with pytest.raises(ValueError):
        sb.advance([l + 1] * K, [0] * K)


def test_value_set_is_the_whole_window_whatever_keep_len():
    """Sec. 3.2: value tokens are all window tokens of finished sequences; the policy
    set's keep_len has no say in it (a caller may drop policy tokens of a finished sequence)."""
    pol, val = ofast.loss_masks([0, 5, 9], [2, 1], [1, 0])
    assert pol.tolist() == [True, True, False, False, False, True, False, False, False]
    assert val.tolist() == [True] * 5 + [False] * 4
    z = np.zeros(9)
    for impl in (odef, ofast):
        out = impl.ppo_losses(z, z, z + 1, z + 1, z, z, [0, 5, 9], [2, 1], [1, 0], 0.2, 0.28, 0.5, 0.6)
        assert out["n_policy"] == 3 and out["n_value"] == 5
        assert out["value_loss"] == pytest.approx(0.5)             # v = 1, R = 0, clipped 0.6: max(1, 0.36) / 2
