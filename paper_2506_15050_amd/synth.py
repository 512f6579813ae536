"""Seeded synthetic inputs shaped like the T-PPO training workloads.

This module only draws random inputs (lengths, flags, token ids, hidden
states, head weights, values, rewards, noise).  It contains none of the
method's arithmetic and imports neither the HIP binding nor the CPU oracle, so
both can be fed from it.  The inputs stand in for the paper's Qwen2.5-32B /
DAPO-Math-17K runs (Sec. 4.1): only shapes, length mixes and hyper-parameters
are taken from there (window 8k, lambda 0.95, gamma 1, eps 0.2/0.28,
xi 0.5/0.6, sparse terminal reward).

bfloat16 tensors are returned as ``uint16`` bit patterns.
"""
from concurrent.futures import ThreadPoolExecutor
import math
import os

import numpy as np

# Named workloads.  ``len_dist``: ("fixed_trunc", lo, hi) = window length for
# truncated sequences, uniform lo..hi for finished ones; ("uniform", lo, hi);
# ("loguniform", lo, hi).  ``p_done`` = probability that a sequence finished
# inside the window (``done_pattern`` fixes the flags instead).
CONFIGS = {
    "tiny": dict(B=4, ctx=16, window=64, len_dist=("fixed_trunc", 8, 64),
                 done_pattern=(1, 0, 1, 0), H=64, V=1000, dtype="f32",
                 tail_drop=8, eps=(0.2, 0.2), seed=0),
    "small": dict(B=32, ctx=256, window=1024, len_dist=("uniform", 64, 1024),
                  p_done=0.5, H=1024, V=32000, dtype="bf16",
                  tail_drop=128, eps=(0.2, 0.28), seed=1002),
    "head7b": dict(B=64, ctx=512, window=2048, len_dist=("uniform", 256, 2048),
                   p_done=0.6, H=3584, V=152064, dtype="bf16",
                   drop_fraction=0.25, eps=(0.2, 0.28), seed=1003),
    "head32b": dict(B=32, ctx=1024, window=8192, len_dist=("loguniform", 512, 8192),
                    p_done=0.4, H=5120, V=152064, dtype="bf16",
                    tail_drop=1024, eps=(0.2, 0.28), seed=1004,
                    ids_from_policy=True),
    "longcot": dict(B=512, ctx=1, window=20480, len_dist=("loguniform", 256, 20480),
                    p_done=0.3, H=0, V=0, dtype="f32",
                    tail_drop=1024, eps=(0.2, 0.28), seed=1005),
    "longcot5x": dict(B=2176, ctx=1, window=20480, len_dist=("loguniform", 256, 20480),
                      p_done=0.3, H=0, V=0, dtype="f32",
                      tail_drop=1024, eps=(0.2, 0.28), seed=1006),
    # same distribution, 42 M tokens: shows the streaming kernels' rate once launch ramp and drain are small
    "longcot20x": dict(B=8704, ctx=1, window=20480, len_dist=("loguniform", 256, 20480),
                       p_done=0.3, H=0, V=0, dtype="f32",
                       tail_drop=1024, eps=(0.2, 0.28), seed=1007),
}
GAMMA = 1.0
LAMBDA = 0.95
XI = (0.5, 0.6)

_STREAM = dict(meta=0, ids=1, hidden=2, w=3, values=4, rewards=5, logp=6,
               vgap=7, uniforms=8, bootstrap=9)


def _rng(seed, stream, block=0):
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence(
        [int(seed), _STREAM[stream], int(block)])))


def f32_to_bf16_bits(x):
    """Round fp32 to bfloat16 (nearest, ties to even); returns uint16 bits."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    return ((u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
            >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b):
    return (np.asarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _normal_matrix(seed, stream, rows, cols, std, dtype, block_rows=4096):
    """rows x cols N(0, std) matrix, one child seed per row block so the result
    does not depend on the number of worker threads."""
    out = np.empty((rows, cols), np.uint16 if dtype == "bf16" else np.float32)

    def fill(b):
        r0 = b * block_rows
        r1 = min(r0 + block_rows, rows)
        x = _rng(seed, stream, b).standard_normal((r1 - r0, cols), dtype=np.float32)
        if std != 1.0:
            x *= np.float32(std)
        out[r0:r1] = f32_to_bf16_bits(x) if dtype == "bf16" else x

    nblocks = (rows + block_rows - 1) // block_rows
    workers = max(1, min(8, len(os.sched_getaffinity(0)), nblocks))
    with ThreadPoolExecutor(workers) as ex:
        list(ex.map(fill, range(nblocks)))
    return out


def _draw_lengths(rng, cfg, done):
    kind, lo, hi = cfg["len_dist"]
    B = cfg["B"]
    if kind == "fixed_trunc":
        finished = rng.integers(lo, hi + 1, size=B)
        return np.where(done != 0, finished, cfg["window"]).astype(np.int64)
    if kind == "uniform":
        return rng.integers(lo, hi + 1, size=B).astype(np.int64)
    if kind == "loguniform":
        x = np.exp(rng.uniform(math.log(lo), math.log(hi), size=B))
        return np.clip(np.rint(x), lo, hi).astype(np.int64)
    raise ValueError(kind)


def make_batch(name, with_head=True, **overrides):
    """Draw one batch of the named workload.  ``overrides`` replace entries of
    the config (e.g. ``B=``, ``H=``, ``V=``, ``seed=``) for reduced-size runs.

    Draw order: flags, lengths, token ids, hidden, head weights, values,
    rewards, log-prob noise, value noise (each from its own seeded stream).
    """
    cfg = dict(CONFIGS[name])
    cfg.update(overrides)
    seed, B = cfg["seed"], cfg["B"]
    meta = _rng(seed, "meta")
    if "done_pattern" in cfg and len(cfg["done_pattern"]) == B:
        done = np.asarray(cfg["done_pattern"], np.int32)
    else:
        done = (meta.random(B) < cfg["p_done"]).astype(np.int32)
    win_len = _draw_lengths(meta, cfg, done)
    ctx_len = np.full(B, cfg["ctx"], np.int64)
    seq_len = ctx_len + win_len
    cu_seqlens = np.concatenate([[0], np.cumsum(seq_len)])
    resp_off = np.concatenate([[0], np.cumsum(win_len)])
    n_tok, n_resp = int(cu_seqlens[-1]), int(resp_off[-1])

    if "drop_fraction" in cfg:
        # smallest tail_drop whose dropped share of window tokens reaches the
        # requested fraction
        trunc = win_len[done == 0]
        lo_d, hi_d = 0, int(cfg["window"])
        while lo_d < hi_d:
            mid = (lo_d + hi_d) // 2
            if np.minimum(trunc, mid).sum() >= cfg["drop_fraction"] * n_resp:
                hi_d = mid
            else:
                lo_d = mid + 1
        tail_drop = lo_d
    else:
        tail_drop = int(cfg["tail_drop"])

    out = dict(name=name, cfg=cfg, B=B, n_tok=n_tok, n_resp=n_resp,
               cu_seqlens=cu_seqlens.astype(np.int32), ctx_len=ctx_len.astype(np.int32),
               done=done, win_len=win_len.astype(np.int32),
               resp_off=resp_off.astype(np.int32), tail_drop=tail_drop,
               gamma=GAMMA, lam=LAMBDA, eps_low=cfg["eps"][0], eps_high=cfg["eps"][1],
               xi_low=XI[0], xi_high=XI[1], H=cfg["H"], V=cfg["V"], dtype=cfg["dtype"])

    if cfg["V"] > 0:
        out["input_ids"] = _rng(seed, "ids").integers(0, cfg["V"], size=n_tok).astype(np.int32)
        # one uniform per packed position, used when ids are re-drawn from the
        # policy's own distribution (inverse-CDF sampling)
        out["id_uniforms"] = _rng(seed, "uniforms").random(n_tok)
    if cfg["V"] > 0 and with_head:
        out["hidden"] = _normal_matrix(seed, "hidden", n_tok, cfg["H"], 1.0, cfg["dtype"])
        out["w_head"] = _normal_matrix(seed, "w", cfg["V"], cfg["H"], 0.02, cfg["dtype"])

    out["values"] = _rng(seed, "values").uniform(-1.0, 1.0, size=n_resp).astype(np.float32)
    rewards = np.zeros(n_resp, np.float32)
    signs = _rng(seed, "rewards").integers(0, 2, size=B) * 2 - 1
    fin = np.nonzero((done != 0) & (win_len > 0))[0]
    rewards[resp_off[fin + 1] - 1] = signs[fin].astype(np.float32)
    out["rewards"] = rewards
    out["bootstrap"] = _rng(seed, "bootstrap").uniform(-1.0, 1.0, size=B).astype(np.float32)
    lg = _rng(seed, "logp")
    # stand-in new log-probs for stages run without the head, and the gap to
    # the old policy's log-probs
    out["logp_new_synth"] = (-np.abs(lg.normal(0.0, 3.0, size=n_resp)) - 0.01).astype(np.float32)
    out["logp_gap"] = lg.normal(0.0, 0.1, size=n_resp).astype(np.float32)
    out["v_gap"] = _rng(seed, "vgap").normal(0.0, 0.3, size=n_resp).astype(np.float32)
    out["v_new"] = (out["values"] + out["v_gap"]).astype(np.float32)
    return out


def sample_ids_from_policy(batch, device="cpu", row_block=2048):
    """Re-draw every window token from softmax(W h) at temperature 1, where h is
    the hidden state of the position before it (inverse-CDF sampling with the
    batch's per-position uniforms).  This emulates the rollout stage, which is
    outside the library; it runs in plain torch ops on ``device`` and its result
    is a frozen input for both the oracle and the HIP path.  Hidden states are
    not changed (they are synthetic and independent of the ids)."""
    import torch
    dt = torch.bfloat16 if batch["dtype"] == "bf16" else torch.float32

    def as_t(a):
        t = torch.from_numpy(a)
        if a.dtype == np.uint16:
            t = t.view(torch.int16).view(torch.bfloat16)
        return t.to(device)

    hidden, w = as_t(batch["hidden"]), as_t(batch["w_head"])
    V = w.shape[0]
    cu, ctx = batch["cu_seqlens"].astype(np.int64), batch["ctx_len"].astype(np.int64)
    pos = np.concatenate([np.arange(cu[i] + ctx[i], cu[i + 1]) for i in range(batch["B"])])
    ids = batch["input_ids"].copy()
    u_all = batch["id_uniforms"]
    for p0 in range(0, pos.shape[0], row_block):
        p = pos[p0:p0 + row_block]
        rows = torch.from_numpy(p - 1).to(device)
        logits = (hidden[rows].to(dt) @ w.t()).float()
        cdf = torch.cumsum(torch.softmax(logits, dim=1).double(), dim=1)
        u = torch.from_numpy(u_all[p]).to(device).unsqueeze(1) * cdf[:, -1:]
        tok = torch.searchsorted(cdf, u).clamp_(max=V - 1).squeeze(1)
        ids[p] = tok.cpu().numpy().astype(np.int32)
    batch["input_ids"] = ids
    return batch
