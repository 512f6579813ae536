"""The pins must bite: each plausible mistake below is planted in a COPY of the
fast oracle's source (on the CPU, never in the GPU path), and at least one pin of
tests/test_oracle_pins.py must fail against the mutated copy.  A mutation that
survives means a pin is missing."""
import importlib
import os
import sys
import types

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
FAST_SRC = open(os.path.join(os.path.dirname(HERE), "oracle", "fast.py")).read()
DEF_SRC = open(os.path.join(os.path.dirname(HERE), "oracle", "definitional.py")).read()

# (what is broken, text to find, replacement)
MUTATIONS = [
    ("filter: predicting row is the token's own position", "rows.append(pos - 1)", "rows.append(pos)"),
    ("filter: tail dropped from finished sequences too",
     "keep_len = np.where(dn, win_len, np.maximum(win_len - int(tail_drop), 0))",
     "keep_len = np.maximum(win_len - int(tail_drop), 0)"),
    ("filter: value tokens counted over unfinished sequences", "N_val=int(win_len[dn].sum())", "N_val=int(win_len.sum())"),
    ("log-prob: sum without the max shift's compensation",
     "block_lse = zmax + np.log(np.exp(z - zmax[:, None]).sum(axis=1))",
     "block_lse = np.log(np.exp(z - zmax[:, None]).sum(axis=1))"),
    ("log-prob: transposed target gather", "logp[r0:r1] = z[np.arange(r1 - r0), sel_targets[r0:r1]] - block_lse",
     "logp[r0:r1] = z[np.arange(r1 - r0), sel_targets[r0:r1][::-1]] - block_lse"),
    ("EGAE: residual with the wrong sign of V(s_t)", "delta = rs[t] + g * v_next - vs[t]", "delta = rs[t] + g * v_next + vs[t]"),
    ("EGAE: residual without gamma", "delta = rs[t] + g * v_next - vs[t]", "delta = rs[t] + v_next - vs[t]"),
    ("EGAE: lambda dropped from the recursion", "a_next = delta + c * a_next", "a_next = delta + g * a_next"),
    ("EGAE: truncated sequence bootstraps with 0", "            v_next = vs[-1]", "            v_next = 0.0"),
    ("EGAE: finished sequence bootstraps with its last value", "        if int(done[i]) != 0:\n            v_next = 0.0",
     "        if int(done[i]) != 0:\n            v_next = vs[-1]"),
    ("return: discounted with gamma*lambda", "r_next = rs[t] + g * r_next", "r_next = rs[t] + c * r_next"),
    ("loss: symmetric clip", "np.clip(rho, 1.0 - eps_low, 1.0 + eps_high) * a)\n        policy_sum",
     "np.clip(rho, 1.0 - eps_low, 1.0 + eps_low) * a)\n        policy_sum"),
    ("loss: max instead of min in the surrogate", "surr = np.minimum(rho * a,", "surr = np.maximum(rho * a,"),
    ("loss: policy loss with the sign of J_PPO", "policy_sum = -float(np.sum(surr))", "policy_sum = float(np.sum(surr))"),
    ("loss: value loss without the 1/2", "value_sum = 0.5 * float(", "value_sum = float("),
    ("loss: value clip around the return", "v_clip = np.clip(v, vo - xi_low, vo + xi_high)", "v_clip = np.clip(v, r - xi_low, r + xi_high)"),
    ("loss: min instead of max of the two squares", "np.sum(np.maximum((v - r) ** 2, (v_clip - r) ** 2))",
     "np.sum(np.minimum((v - r) ** 2, (v_clip - r) ** 2))"),
    ("masks: value set ends at keep_len", "            val[lo:hi] = True", "            val[lo:lo + int(keep_len[i])] = True"),
    ("loss derivative: ratio factor forgotten", "-policy_scale * rho * a / den_p", "-policy_scale * a / den_p"),
    ("loss derivative: clipped branch passes the derivative", "np.where(unclipped, -policy_scale * rho * a / den_p, 0.0))",
     "-policy_scale * rho * a / den_p)"),
    ("loss derivative: strict comparison inside the clip range", "unclipped = rho * a <= np.clip(", "unclipped = rho * a < np.clip("),
    ("loss derivative: value derivative of the clipped branch", "np.where(unclipped, value_scale * d0 / den_v, 0.0))",
     "np.where(unclipped, value_scale * d0 / den_v, value_scale * d1 / den_v))"),
    ("log-prob derivative: one-hot with the wrong sign", "dz[np.arange(r1 - r0), sel_targets[r0:r1]] += 1.0",
     "dz[np.arange(r1 - r0), sel_targets[r0:r1]] -= 1.0"),
    ("log-prob derivative: head derivative not transposed over tokens", "grad_w += dz.T @ h", "grad_w += (dz.T @ h)[::-1]"),
    ("log-prob derivative: upstream derivative not applied", "        dz *= g[r0:r1, None]\n", ""),
    ("value head: bias forgotten", "v[r0:r0 + 4096] = h @ w + bias", "v[r0:r0 + 4096] = h @ w"),
    ("loss: a NaN inside the policy set is clipped away (min / max that return the other operand)",
     "surr = np.minimum(rho * a, np.clip(rho, 1.0 - eps_low, 1.0 + eps_high) * a)",
     "surr = np.fmin(rho * a, np.fmin(np.fmax(rho, 1.0 - eps_low), 1.0 + eps_high) * a)"),
    ("loss: a NaN inside the value set is dropped by the max", "np.sum(np.maximum((v - r) ** 2, (v_clip - r) ** 2))",
     "np.sum(np.fmax((v - r) ** 2, np.nan_to_num((v_clip - r) ** 2)))"),
    ("loss derivative: a NaN token counted as clipped with derivative 0",
     "g_lp[pol] = np.where(undefined, np.nan, np.where(unclipped, -policy_scale * rho * a / den_p, 0.0))",
     "g_lp[pol] = np.where(unclipped, -policy_scale * rho * a / den_p, 0.0)"),
    ("loss derivative: a NaN value token gets derivative 0",
     "g_v[val] = np.where(undefined, np.nan, np.where(unclipped, value_scale * d0 / den_v, 0.0))",
     "g_v[val] = np.where(unclipped, value_scale * d0 / den_v, 0.0)"),
]

# the same for the slot bookkeeping of successive batching, which lives in the definitional oracle
DEF_MUTATIONS = [
    ("batching: reaching the maximum response length does not end a sequence",
     's["done"] = bool(eos[k]) or so_far + g == self.max_response', 's["done"] = bool(eos[k])'),
    ("batching: the previous window does not become context", 's["ctx"] += s["win"]', 's["ctx"] = s["prompt"]'),
    ("batching: response length counted over the current window only",
     'so_far = s["ctx"] + s["win"] - s["prompt"]', 'so_far = s["win"]'),
    ("batching: refill walks the slots backwards", "for k in range(len(self.seq)):\n            s = self.seq[k]",
     "for k in reversed(range(len(self.seq))):\n            s = self.seq[k]"),
    ("batching: refill also replaces unfinished sequences", '(s is None or s["done"]) and taken', "True and taken"),
    ("batching: every new sequence gets the same id", "                self.next_id += 1\n", ""),
    ("batching: a sequence may stop short of the window without ending",
     'if not eos[k] and g < self.window and so_far + g < self.max_response:', "if False:"),
    ("batching: the window bound is not enforced", "if g < 0 or g > self.window or so_far + g > self.max_response:",
     "if g < 0 or so_far + g > self.max_response:"),
]


def _pin_functions(mod):
    return [getattr(mod, n) for n in dir(mod) if n.startswith("test_") and callable(getattr(mod, n))]


def _cases(fn, real_fast, mutated):
    """The keyword-argument sets pytest would call `fn` with (its parametrize marks
    expanded), with the real oracle module replaced by the mutated copy."""
    sets = [{}]
    for m in getattr(fn, "pytestmark", []):
        if m.name != "parametrize":
            continue
        names = [n.strip() for n in m.args[0].split(",")]
        expanded = []
        for values in m.args[1]:
            values = values if len(names) > 1 else (values,)
            kw = {n: (mutated if v is real_fast else v) for n, v in zip(names, values)}
            expanded += [dict(base, **kw) for base in sets]
        sets = expanded
    return sets


def _run_pins(pins, real_fast, mutated):
    failed = []
    for fn in _pin_functions(pins):
        for kw in _cases(fn, real_fast, mutated):
            try:
                fn(**kw)
            except (AssertionError, pytest.fail.Exception):              # pytest.raises reports through the latter
                failed.append(fn.__name__)
            except (ArithmeticError, ValueError, IndexError, KeyError) as e:     # a mutation may also crash a pin
                failed.append(f"{fn.__name__}: {type(e).__name__}")
    return failed


def _load(src):
    mod = types.ModuleType("oracle_fast_copy")
    mod.__file__ = "oracle/fast.py (copy)"
    exec(compile(src, mod.__file__, "exec"), mod.__dict__)
    return mod


def test_an_unmutated_copy_passes_every_pin(monkeypatch):
    """The harness itself: a verbatim copy must fail nothing (and TypeErrors from a
    wrong call signature are not swallowed, they propagate)."""
    pins = importlib.import_module("test_oracle_pins")
    real = pins.ofast
    copy = _load(FAST_SRC)
    monkeypatch.setattr(pins, "ofast", copy)
    assert _run_pins(pins, real, copy) == []


@pytest.mark.parametrize("what,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_a_pin_catches(what, old, new, monkeypatch):
    assert FAST_SRC.count(old) >= 1, f"mutation target not found: {old!r}"
    pins = importlib.import_module("test_oracle_pins")
    real = pins.ofast
    mutated = _load(FAST_SRC.replace(old, new, 1))
    monkeypatch.setattr(pins, "ofast", mutated)
    assert _run_pins(pins, real, mutated), f"no pin noticed: {what}"


@pytest.mark.parametrize("what,old,new", DEF_MUTATIONS, ids=[m[0] for m in DEF_MUTATIONS])
def test_a_pin_catches_batching_mistakes(what, old, new, monkeypatch):
    assert DEF_SRC.count(old) >= 1, f"mutation target not found: {old!r}"
    pins = importlib.import_module("test_oracle_pins")
    real = pins.odef
    mutated = _load(DEF_SRC.replace(old, new, 1))
    monkeypatch.setattr(pins, "odef", mutated)
    only = types.SimpleNamespace(**{n: getattr(pins, n) for n in dir(pins) if n.startswith("test_successive_batching")})
    assert _run_pins(only, real, mutated), f"no pin noticed: {what}"
