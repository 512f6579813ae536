"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by
element on the same seeded inputs.  Tolerances: indices bit-exact; log-probs
abs 2e-3; EGAE |x-y| <= 1e-5*max(|y|,1); losses rel 1e-3."""
import numpy as np
import pytest

from oracle import fast as ofast
from paper_2506_15050_amd import synth

pytestmark = pytest.mark.gpu

LOGP_ATOL = 2e-3
EGAE_RTOL = 1e-5
LOSS_RTOL = 1e-3


@pytest.fixture(scope="module")
def tp():
    import torch
    from paper_2506_15050_amd import binding
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    binding.load()
    return binding


def dev(a):
    import torch
    if a is None:
        return None
    t = torch.from_numpy(np.ascontiguousarray(a))
    if a.dtype == np.uint16:
        t = t.view(torch.int16).view(torch.bfloat16)
    return t.cuda()


def host(t):
    return t.detach().cpu().numpy()


def assert_egae_close(got, ref, what):
    ref = np.asarray(ref, np.float64)
    err = np.abs(got.astype(np.float64) - ref)
    tol = EGAE_RTOL * np.maximum(np.abs(ref), 1.0)
    bad = np.nonzero(err > tol)[0]
    assert bad.size == 0, f"{what}: {bad.size} mismatches, first at {bad[:5]}, err {err[bad[:5]]}"


def run_select(tp, b, tail_drop=None, capacity=None, with_ids=True):
    st = tp.new_status("cuda")
    out = tp.tppo_select(dev(b["cu_seqlens"]), dev(b["ctx_len"]), dev(b["done"]),
                         dev(b["input_ids"]) if with_ids else None,
                         b["tail_drop"] if tail_drop is None else tail_drop,
                         capacity=capacity, status=st, n_tok=b["n_tok"])
    return out, int(host(st)[0])


def check_select(tp, b, tail_drop=None):
    td = b["tail_drop"] if tail_drop is None else tail_drop
    out, status = run_select(tp, b, td)
    ref = ofast.select(b["cu_seqlens"], b["ctx_len"], b["done"], b["input_ids"], td)
    assert status == 0
    counts = host(out["counts"])
    assert counts.tolist() == [ref["M"], ref["N_resp"], ref["N_val"]]
    M = ref["M"]
    for k in ("resp_off", "sel_off", "keep_len"):
        assert np.array_equal(host(out[k]), ref[k]), k
    for k in ("sel_rows", "sel_targets", "sel_resp_idx"):
        assert np.array_equal(host(out[k])[:M], ref[k]), k
    return out, ref


# ------------------------------------------------------------------ select
@pytest.mark.parametrize("name", ["tiny", "small"])
def test_select_configs(tp, name):
    b = synth.make_batch(name, with_head=False)
    check_select(tp, b)
    check_select(tp, b, tail_drop=0)
    check_select(tp, b, tail_drop=10 ** 6)


def test_select_large_configs(tp):
    for name in ("head7b", "head32b"):
        check_select(tp, synth.make_batch(name, with_head=False))


def test_select_many_sequences_offsets_only(tp):
    b = synth.make_batch("longcot5x")                     # B = 2176 > one scan chunk
    out, status = run_select(tp, b, with_ids=False)
    ids = np.zeros(b["n_tok"], np.int32)
    ref = ofast.select(b["cu_seqlens"], b["ctx_len"], b["done"], ids, b["tail_drop"])
    assert status == 0
    for k in ("resp_off", "sel_off", "keep_len"):
        assert np.array_equal(host(out[k]), ref[k]), k
    assert host(out["counts"]).tolist() == [ref["M"], ref["N_resp"], ref["N_val"]]
    assert np.array_equal(host(out["sel_rows"])[:ref["M"]], ref["sel_rows"])
    assert np.array_equal(host(out["sel_resp_idx"])[:ref["M"]], ref["sel_resp_idx"])


def test_select_edge_cases(tp):
    import torch
    # empty batch
    z = torch.zeros(1, dtype=torch.int32, device="cuda")
    e = torch.zeros(0, dtype=torch.int32, device="cuda")
    out = tp.tppo_select(z, e, e, e, 0)
    assert host(out["counts"]).tolist() == [0, 0, 0] and host(out["resp_off"]).tolist() == [0]
    # windows of length 1 and sequences whose whole window is dropped
    b = synth.make_batch("tiny", with_head=False, len_dist=("fixed_trunc", 1, 1), window=1)
    check_select(tp, b, tail_drop=0)
    check_select(tp, b, tail_drop=1)
    # capacity smaller than M: excess not written, status says so
    b = synth.make_batch("tiny", with_head=False)
    ref = ofast.select(b["cu_seqlens"], b["ctx_len"], b["done"], b["input_ids"], b["tail_drop"])
    out, status = run_select(tp, b, capacity=10)
    assert status == tp.STATUS_CAPACITY
    assert np.array_equal(host(out["sel_rows"]), ref["sel_rows"][:10])
    # bad layout (ctx_len = 0) is flagged and that sequence contributes nothing
    b2 = synth.make_batch("tiny", with_head=False)
    b2["ctx_len"] = b2["ctx_len"].copy()
    b2["ctx_len"][1] = 0
    out, status = run_select(tp, b2)
    assert status & tp.STATUS_BAD_LAYOUT
    assert host(out["keep_len"])[1] == 0


@pytest.mark.parametrize("K,l,L", [(12, 512, 1536), (8, 8192, 24576)])
def test_select_across_successive_batching_steps(tp, K, l, L):
    """Several training steps of successive batching (window l of a maximum L, as in
    the paper's 8k of 24k): the policy tokens are the current window, the value
    tokens every response token of the finished sequences, whichever step made them."""
    rng = np.random.default_rng(K + l)
    bt = tp.Batcher(K, l, L)
    bt.refill(rng.integers(16, 200, size=K))
    tail = l // 8
    seen_value = {}
    for step in range(5):
        cu, ctx, prompt, done, ids = bt.layout()
        gen, eos = [], []
        for k in range(K):
            room = min(l, L - (cu[k + 1] - cu[k] - prompt[k]))
            stop = rng.random() < 0.4
            gen.append(int(rng.integers(1, room + 1)) if stop else room)
            eos.append(1 if stop else 0)
        bt.advance(gen, eos)
        cu, ctx, prompt, done, ids = bt.layout()
        b = dict(cu_seqlens=cu, ctx_len=ctx, done=done, n_tok=int(cu[-1]),
                 input_ids=rng.integers(0, 50000, size=int(cu[-1])).astype(np.int32), tail_drop=tail)
        _, pol = check_select(tp, b)                                       # policy tokens: the current window
        assert pol["N_resp"] == sum(gen)
        _, val = check_select(tp, dict(b, ctx_len=prompt), tail_drop=2**31 - 1)   # value tokens
        lens = (cu[1:] - cu[:-1] - prompt)[done != 0]
        assert val["M"] == int(lens.sum())
        for k in np.flatnonzero(done):                                     # the whole response, in order
            lo, hi = val["sel_off"][k], val["sel_off"][k + 1]
            assert np.array_equal(val["sel_rows"][lo:hi], np.arange(cu[k] + prompt[k] - 1, cu[k + 1] - 1))
            assert ids[k] not in seen_value
            seen_value[ids[k]] = hi - lo
        bt.refill(rng.integers(16, 200, size=int(done.sum())))
    assert len(seen_value) >= 3
    bt.close()


# ------------------------------------------------------------------ log-probs
def check_logprobs(tp, hidden, w, rows, targets, **kw):
    st = tp.new_status("cuda")
    logp, lse = tp.tppo_token_logprobs(dev(hidden), dev(w), dev(rows.astype(np.int32)),
                                       dev(targets.astype(np.int32)), status=st, **kw)
    ref_lp, ref_lse = ofast.token_logprobs(hidden, w, rows, targets)
    assert int(host(st)[0]) == 0
    got_lp, got_lse = host(logp), host(lse)
    assert np.abs(got_lp - ref_lp).max() <= LOGP_ATOL, np.abs(got_lp - ref_lp).max()
    assert np.abs(got_lse - ref_lse).max() <= LOGP_ATOL, np.abs(got_lse - ref_lse).max()
    return np.abs(got_lp - ref_lp).max()


def test_logprobs_tiny_fp32(tp):
    b = synth.make_batch("tiny")
    sel = ofast.select(b["cu_seqlens"], b["ctx_len"], b["done"], b["input_ids"], b["tail_drop"])
    err = check_logprobs(tp, b["hidden"], b["w_head"], sel["sel_rows"], sel["sel_targets"])
    assert err < 1e-4          # fp32 inputs: far inside the bf16 tolerance


def test_logprobs_generic_bf16_odd_shapes(tp):
    rng = np.random.default_rng(0)
    H, V, N = 72, 333, 40                                 # H not a multiple of 64 -> generic kernel
    hidden = synth.f32_to_bf16_bits(rng.normal(size=(N, H)).astype(np.float32))
    w = synth.f32_to_bf16_bits((0.1 * rng.normal(size=(V, H))).astype(np.float32))
    rows = rng.integers(0, N, size=57)
    check_logprobs(tp, hidden, w, rows, rng.integers(0, V, size=57))


@pytest.mark.parametrize("M,V,H", [(1, 256, 64), (37, 1000, 128), (300, 1000, 256), (513, 2049, 192),
                                   (256, 512, 64), (700, 5000, 1024)])
def test_logprobs_mfma_ragged_shapes(tp, M, V, H):
    rng = np.random.default_rng(M + V)
    N = M + 5
    hidden = synth.f32_to_bf16_bits(rng.normal(size=(N, H)).astype(np.float32))
    w = synth.f32_to_bf16_bits((rng.normal(size=(V, H)) / np.sqrt(H)).astype(np.float32))
    rows = rng.integers(0, N, size=M)
    # targets sweep every residue of the accumulator layout, plus both ends
    targets = (np.arange(M) * 7 + 3) % V
    targets[0], targets[-1] = 0, V - 1
    check_logprobs(tp, hidden, w, rows, targets)


def test_logprobs_every_target_of_one_row_sums_to_one(tp):
    rng = np.random.default_rng(5)
    H, V = 128, 777
    hidden = synth.f32_to_bf16_bits(rng.normal(size=(3, H)).astype(np.float32))
    w = synth.f32_to_bf16_bits((rng.normal(size=(V, H)) / np.sqrt(H)).astype(np.float32))
    rows = np.full(V, 1)
    logp, lse = tp.tppo_token_logprobs(dev(hidden), dev(w), dev(rows.astype(np.int32)),
                                       dev(np.arange(V, dtype=np.int32)))
    lp = host(logp).astype(np.float64)
    assert abs(np.exp(lp).sum() - 1.0) < 1e-4
    ref, _ = ofast.token_logprobs(hidden, w, rows, np.arange(V))
    assert np.abs(lp - ref).max() <= LOGP_ATOL


_SMALL_FULL = {}


def small_full_oracle():
    """Config 2 at its own size (32 sequences, H = 1024, V = 32000): batch, oracle selection and oracle
    log-probs of every kept token, computed once per test session."""
    if not _SMALL_FULL:
        b = synth.make_batch("small")
        sel = ofast.select(b["cu_seqlens"], b["ctx_len"], b["done"], b["input_ids"], b["tail_drop"])
        lp, lse = ofast.token_logprobs(b["hidden"], b["w_head"], sel["sel_rows"], sel["sel_targets"])
        _SMALL_FULL.update(b=b, sel=sel, logp=lp, lse=lse)
    return _SMALL_FULL["b"], _SMALL_FULL["sel"], _SMALL_FULL["logp"], _SMALL_FULL["lse"]


@pytest.mark.timeout(600)
def test_logprobs_small_config_full(tp):
    """Config 2 with all 32 sequences: every kept token against the oracle."""
    b, sel, ref_lp, ref_lse = small_full_oracle()
    assert sel["M"] > 12000
    st = tp.new_status("cuda")
    logp, lse = tp.tppo_token_logprobs(dev(b["hidden"]), dev(b["w_head"]), dev(sel["sel_rows"]),
                                       dev(sel["sel_targets"]), status=st)
    assert int(host(st)[0]) == 0
    assert np.abs(host(logp) - ref_lp).max() <= LOGP_ATOL
    assert np.abs(host(lse) - ref_lse).max() <= LOGP_ATOL


@pytest.mark.parametrize("M,V,H", [(18600, 2048, 64), (21000, 1100, 128), (4200, 9000, 64)])
def test_logprobs_many_token_tiles_every_output(tp, M, V, H):
    """Many 256-token tiles against a small vocabulary and hidden size, so the oracle can afford
    every output: the persistent schedule then has several rounds of units per XCD, more than one
    unit column, a ragged last group of unit rows and a ragged last token tile."""
    rng = np.random.default_rng(M)
    N = M // 3 + 11                                       # rows are revisited, in no order
    hidden = synth.f32_to_bf16_bits(rng.normal(size=(N, H)).astype(np.float32))
    w = synth.f32_to_bf16_bits((rng.normal(size=(V, H)) / np.sqrt(H)).astype(np.float32))
    rows = rng.integers(0, N, size=M)
    targets = rng.integers(0, V, size=M)
    targets[:V] = np.arange(V)[:M]                        # every vocabulary id is some token's target
    check_logprobs(tp, hidden, w, rows, targets)


def test_logprobs_scatter_count_and_status(tp):
    import torch
    b = synth.make_batch("small", B=3, V=1500, H=128)
    sel = ofast.select(b["cu_seqlens"], b["ctx_len"], b["done"], b["input_ids"], b["tail_drop"])
    M, n_resp = sel["M"], sel["N_resp"]
    ref, _ = ofast.token_logprobs(b["hidden"], b["w_head"], sel["sel_rows"], sel["sel_targets"])
    # scatter into the response-packed domain, with M given as an upper bound
    # and the true count read from device memory
    cap = b["n_tok"]
    rows = np.zeros(cap, np.int32); rows[:M] = sel["sel_rows"]
    tg = np.zeros(cap, np.int32); tg[:M] = sel["sel_targets"]
    oi = np.zeros(cap, np.int32); oi[:M] = sel["sel_resp_idx"]
    m_dev = torch.tensor([M], dtype=torch.int64, device="cuda")
    logp, _ = tp.tppo_token_logprobs(dev(b["hidden"]), dev(b["w_head"]), dev(rows), dev(tg), M=cap,
                                     m_actual=m_dev, out_index=dev(oi), out_size=n_resp)
    got = host(logp)[sel["sel_resp_idx"]]
    assert np.abs(got - ref).max() <= LOGP_ATOL
    # a bad target id yields NaN for that token only and sets the status bit
    tg_bad = sel["sel_targets"].copy()
    tg_bad[5] = 1500
    st = tp.new_status("cuda")
    logp, _ = tp.tppo_token_logprobs(dev(b["hidden"]), dev(b["w_head"]), dev(sel["sel_rows"]),
                                     dev(tg_bad), status=st)
    got = host(logp)
    assert np.isnan(got[5]) and int(host(st)[0]) == tp.STATUS_BAD_TARGET
    keep = np.arange(M) != 5
    assert np.abs(got[keep] - ref[keep]).max() <= LOGP_ATOL


def _sampled_rows(sel, n, seed):
    rng = np.random.default_rng(seed)
    M = sel["M"]
    pick = set(rng.choice(M, size=min(n, M), replace=False).tolist())
    so = sel["sel_off"]
    for i in range(len(so) - 1):                          # first and last kept token of every sequence
        if so[i + 1] > so[i]:
            pick.add(int(so[i])); pick.add(int(so[i + 1] - 1))
    return np.array(sorted(pick))


def _stratified_rows(sel, seed):
    """One kept token out of every run of 16 consecutive compact indices (so every 256-token tile of the
    MFMA sweep contributes 16 outputs, one per 16-column accumulator block, at positions that rotate through
    all 16 columns), plus the first and last kept token of every sequence and of the batch."""
    rng = np.random.default_rng(seed)
    M = sel["M"]
    starts = np.arange(0, M, 16)
    pick = set(np.minimum(starts + (starts // 16 + rng.integers(0, 16)) % 16, M - 1).tolist())
    so = sel["sel_off"]
    for i in range(len(so) - 1):
        if so[i + 1] > so[i]:
            pick.add(int(so[i])); pick.add(int(so[i + 1] - 1))
    pick.update((0, M - 1))
    return np.array(sorted(pick))


def _split_edge_targets(V, tile=256):
    """Vocabulary ids on both sides of every boundary between vocabulary splits, for every split count
    the kernel may choose (a split owns tiles [tiles*s/S, tiles*(s+1)/S) of `tile` ids), and both ends."""
    tiles = (V + tile - 1) // tile
    edges = set()
    for S in (1, 2, 3) + tuple(range(4, 65, 4)):
        for s in range(1, S):
            edges.add((tiles * s // S) * tile)
    ids = {0, V - 1}
    for e in edges:
        if 0 < e < V:
            ids.update((e - 1, e))
    return np.array(sorted(ids))


@pytest.mark.timeout(1200)
@pytest.mark.parametrize("name", ["head7b", "head32b"])
def test_logprobs_full_size_stratified(tp, name):
    """Full-size shapes in the launch configuration the benchmark times.  The oracle checks, one by
    one, a stratified sample of the outputs: 16 per 256-token tile (one per accumulator block), each
    sequence's first and last kept token; a few hundred of the sampled tokens get their target moved
    onto the edges of the vocabulary splits."""
    import torch
    b = synth.make_batch(name)
    if b["cfg"].get("ids_from_policy"):
        synth.sample_ids_from_policy(b, device="cuda")
    sel = ofast.select(b["cu_seqlens"], b["ctx_len"], b["done"], b["input_ids"], b["tail_drop"])
    pick = _stratified_rows(sel, seed=1)
    assert pick.size >= 2048 and pick.size >= sel["M"] // 16
    targets = sel["sel_targets"].copy()
    edge_ids = _split_edge_targets(b["V"])
    moved = pick[np.linspace(0, pick.size - 1, edge_ids.size).astype(np.int64)]
    targets[moved] = edge_ids
    hidden, w = dev(b["hidden"]), dev(b["w_head"])
    rows, tg = dev(sel["sel_rows"]), dev(targets)
    st = tp.new_status("cuda")
    logp, lse = tp.tppo_token_logprobs(hidden, w, rows, tg, status=st)
    logp2, _ = tp.tppo_token_logprobs(hidden, w, rows, tg)
    torch.cuda.synchronize()
    assert int(host(st)[0]) == 0
    got, got_lse = host(logp), host(lse)
    assert np.array_equal(got, host(logp2))               # deterministic
    assert np.isfinite(got).all() and (got <= 0).all()
    ref, ref_lse = ofast.token_logprobs(b["hidden"], b["w_head"], sel["sel_rows"][pick], targets[pick])
    assert np.abs(got[pick] - ref).max() <= LOGP_ATOL, np.abs(got[pick] - ref).max()
    assert np.abs(got_lse[pick] - ref_lse).max() <= LOGP_ATOL


# ------------------------------------------------------------------ log-prob derivatives
# dz is rounded to bf16 (relative error <= 2^-9 per element) before the two
# products; an output element is a sum of terms dz * w (or dz * h), so its error
# is at most 2^-9 times the sum of the terms' magnitudes.  The tests allow twice
# that, plus 1e-6 of the largest such sum for the fp32 arithmetic in front.
DZ_RTOL = 2.0 ** -8


def assert_within_term_bound(got, ref, abs_bound, what):
    tol = DZ_RTOL * abs_bound + 1e-6 * abs_bound.max() + 1e-30
    err = np.abs(got.astype(np.float64) - ref)
    bad = err > tol
    assert not bad.any(), (what, int(bad.sum()), float((err / tol).max()))


def check_logprob_grads(tp, hidden, w, rows, targets, g, workspace=None, via_index=False):
    import torch
    _, lse = ofast.token_logprobs(hidden, w, rows, targets)
    M = len(rows)
    lse32, g32 = lse.astype(np.float32), g.astype(np.float32)
    kw = {}
    if via_index:                                           # scalars stored in a permuted, larger array
        perm = np.random.default_rng(1).permutation(M + 9)[:M].astype(np.int32)
        big_l, big_g = np.full(M + 9, np.nan, np.float32), np.full(M + 9, np.nan, np.float32)
        big_l[perm], big_g[perm] = lse32, g32
        lse_d, g_d, kw["in_index"] = dev(big_l), dev(big_g), dev(perm)
    else:
        lse_d, g_d = dev(lse32), dev(g32)
    dh, dw = tp.tppo_token_logprobs_backward(dev(hidden), dev(w), dev(np.asarray(rows, np.int32)),
                                             dev(np.asarray(targets, np.int32)), lse_d, g_d,
                                             workspace=workspace, **kw)
    torch.cuda.synchronize()
    ref_h, ref_w, abs_h, abs_w = ofast.token_logprob_grads(hidden, w, rows, targets, g32, return_abs_bounds=True)
    assert_within_term_bound(host(dh), ref_h, abs_h, "grad_hidden")
    assert_within_term_bound(host(dw), ref_w, abs_w, "grad_w")
    return host(dh), host(dw)


def _bf16_case(M, V, H, seed):
    rng = np.random.default_rng(seed)
    N = M + 5
    hidden = synth.f32_to_bf16_bits(rng.normal(size=(N, H)).astype(np.float32))
    w = synth.f32_to_bf16_bits((rng.normal(size=(V, H)) / np.sqrt(H)).astype(np.float32))
    rows = rng.permutation(N)[:M]
    targets = (np.arange(M) * 7 + 3) % V
    targets[0], targets[-1] = 0, V - 1
    return hidden, w, rows, targets, rng.normal(size=M)


@pytest.mark.parametrize("M,V,H", [(1, 256, 64), (37, 1000, 128), (300, 1000, 256), (513, 2049, 192),
                                   (700, 5000, 1024)])
def test_logprob_grads_ragged_shapes(tp, M, V, H):
    check_logprob_grads(tp, *_bf16_case(M, V, H, seed=M + V))


def test_logprob_grads_index_chunks_halves_accumulate(tp):
    import torch
    hidden, w, rows, targets, g = _bf16_case(700, 1000, 128, seed=77)
    dh, dw = check_logprob_grads(tp, hidden, w, rows, targets, g, via_index=True)
    # a workspace that only holds 256 tokens at a time: three chunks, same result up to fp32 summation order
    lib = tp.load()
    small_ws = tp._workspace(lib.tppo_token_logprobs_backward_workspace_bytes(256, 128, 1000, tp.TPPO_BF16), "cuda")
    dh_c, dw_c = check_logprob_grads(tp, hidden, w, rows, targets, g, workspace=small_ws)
    assert np.array_equal(dh_c, dh)                         # rows do not interact
    assert np.allclose(dw_c, dw, rtol=0, atol=1e-5 * np.abs(dw).max())
    # one output at a time, and accumulation into grad_w
    _, lse = ofast.token_logprobs(hidden, w, rows, targets)
    args = (dev(hidden), dev(w), dev(rows.astype(np.int32)), dev(targets.astype(np.int32)),
            dev(lse.astype(np.float32)), dev(g.astype(np.float32)))
    only_h, none_w = tp.tppo_token_logprobs_backward(*args, want_w=False)
    none_h, only_w = tp.tppo_token_logprobs_backward(*args, want_hidden=False)
    assert none_w is None and none_h is None
    assert np.array_equal(host(only_h), dh) and np.array_equal(host(only_w), dw)
    acc = only_w.clone()
    tp.tppo_token_logprobs_backward(*args, want_hidden=False, grad_w=acc, accumulate_w=True)
    torch.cuda.synchronize()
    assert np.allclose(host(acc), 2 * dw, rtol=1e-6, atol=0)
    # tokens with a zero upstream derivative contribute exactly nothing
    g0 = g.copy()
    g0[100:] = 0.0
    dh0, _ = check_logprob_grads(tp, hidden, w, rows, targets, g0)
    assert not dh0[100:].any()


def test_logprob_grads_small_config_slice(tp):
    b = synth.make_batch("small", B=4)
    sel = ofast.select(b["cu_seqlens"], b["ctx_len"], b["done"], b["input_ids"], b["tail_drop"])
    g = np.random.default_rng(3).normal(size=sel["M"]) / sel["M"]
    check_logprob_grads(tp, b["hidden"], b["w_head"], sel["sel_rows"], sel["sel_targets"], g)


@pytest.mark.timeout(900)
def test_logprob_grads_full_vocabulary_few_tokens(tp):
    """Vocabulary and hidden size of the 32B-shaped workload, 192 kept tokens:
    every element of both outputs against the oracle."""
    b = synth.make_batch("head32b")
    sel = ofast.select(b["cu_seqlens"], b["ctx_len"], b["done"], b["input_ids"], b["tail_drop"])
    pick = _sampled_rows(sel, 160, seed=4)[:192]
    g = np.random.default_rng(5).normal(size=len(pick))
    check_logprob_grads(tp, b["hidden"], b["w_head"], sel["sel_rows"][pick], sel["sel_targets"][pick], g)


@pytest.mark.timeout(900)
def test_logprob_grads_full_size_sampled(tp):
    """The 32B-shaped workload at full size: grad_hidden on a seeded sample of
    tokens one by one; for grad_w, which needs every token, the properties that
    hold at any size (its columns sum to zero; bit-identical reruns)."""
    import torch
    b = synth.make_batch("head32b")
    synth.sample_ids_from_policy(b, device="cuda")
    sel = ofast.select(b["cu_seqlens"], b["ctx_len"], b["done"], b["input_ids"], b["tail_drop"])
    M = sel["M"]
    hidden, w = dev(b["hidden"]), dev(b["w_head"])
    rows, tg = dev(sel["sel_rows"]), dev(sel["sel_targets"])
    _, lse = tp.tppo_token_logprobs(hidden, w, rows, tg)      # the backward entry point's own input
    g = (np.random.default_rng(6).normal(size=M) / M).astype(np.float32)
    ws = tp._workspace(tp.load().tppo_token_logprobs_backward_workspace_bytes(M, b["H"], b["V"], tp.TPPO_BF16), "cuda")
    dh, dw = tp.tppo_token_logprobs_backward(hidden, w, rows, tg, lse, dev(g), workspace=ws)
    dh2, dw2 = tp.tppo_token_logprobs_backward(hidden, w, rows, tg, lse, dev(g), workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(dh, dh2) and torch.equal(dw, dw2)
    assert bool(torch.isfinite(dh).all()) and bool(torch.isfinite(dw).all())
    col = dw.double().sum(dim=0).abs().cpu().numpy()
    mass = dw.double().abs().sum(dim=0).cpu().numpy()
    assert (col <= 1e-2 * mass).all(), float((col / mass).max())
    pick = _sampled_rows(sel, 40, seed=7)[:64]
    ref_h, _, abs_h, _ = ofast.token_logprob_grads(b["hidden"], b["w_head"], sel["sel_rows"][pick],
                                                   sel["sel_targets"][pick], g[pick], want_w=False,
                                                   return_abs_bounds=True)
    assert_within_term_bound(dh[torch.from_numpy(pick).cuda()].cpu().numpy(), ref_h, abs_h, "grad_hidden")


# ------------------------------------------------------------------ value head
def check_value_head(tp, hidden, w, bias, rows, **kw):
    got = host(tp.tppo_value_head(dev(hidden), dev(w), bias, None if rows is None else dev(np.asarray(rows, np.int32)), **kw))
    idx = np.arange(hidden.shape[0]) if rows is None else rows
    ref, bound = ofast.value_head(hidden, w, float(np.float32(bias)), idx, return_abs_bound=True)
    # fp32 accumulation of H products: error <= a few sqrt(H) 2^-24 of the sum of the terms' magnitudes
    tol = 1e-5 * (bound + abs(bias)) + 1e-30
    assert np.all(np.abs(got - ref) <= tol), float((np.abs(got - ref) / tol).max())
    return got


@pytest.mark.parametrize("M,N,H", [(1, 3, 8), (57, 60, 64), (300, 305, 200), (1000, 1500, 1024), (777, 800, 5120)])
def test_value_head_shapes(tp, M, N, H):
    rng = np.random.default_rng(M + H)
    hidden = synth.f32_to_bf16_bits(rng.normal(size=(N, H)).astype(np.float32))
    w = synth.f32_to_bf16_bits((rng.normal(size=H) / np.sqrt(H)).astype(np.float32))
    check_value_head(tp, hidden, w, 0.125, rng.integers(0, N, size=M))
    check_value_head(tp, hidden, w, -2.0, None)             # no list: every row in order


def test_value_head_scatter_count_status(tp):
    import torch
    rng = np.random.default_rng(9)
    N, H, M = 400, 256, 333
    hidden = synth.f32_to_bf16_bits(rng.normal(size=(N, H)).astype(np.float32))
    w = synth.f32_to_bf16_bits((rng.normal(size=H) / 16).astype(np.float32))
    rows = rng.integers(0, N, size=M)
    ref = ofast.value_head(hidden, w, 0.0, rows)
    # scatter through an index, count read from device memory, capacity larger than the count
    cap = 500
    rows_c = np.zeros(cap, np.int32); rows_c[:M] = rows
    oi = np.zeros(cap, np.int32); oi[:M] = rng.permutation(600)[:M]
    out = torch.full((600,), 7.0, device="cuda")
    tp.tppo_value_head(dev(hidden), dev(w), 0.0, dev(rows_c), M=cap,
                       m_actual=torch.tensor([M], dtype=torch.int64, device="cuda"), out_index=dev(oi), out=out)
    got = host(out)
    assert np.abs(got[oi[:M]] - ref).max() < 1e-4
    untouched = np.ones(600, bool); untouched[oi[:M]] = False
    assert (got[untouched] == 7.0).all()
    # a bad row index: NaN for that token only, status bit set
    bad = rows.copy(); bad[10] = N
    st = tp.new_status("cuda")
    got = host(tp.tppo_value_head(dev(hidden), dev(w), 0.0, dev(bad.astype(np.int32)), status=st))
    assert np.isnan(got[10]) and int(host(st)[0]) == tp.STATUS_BAD_ROW
    keep = np.arange(M) != 10
    assert np.abs(got[keep] - ref[keep]).max() < 1e-4


def test_value_head_32b_shape_value_tokens(tp):
    """Hidden size and value-token rows of the 32B-shaped workload (window tokens of finished sequences)."""
    b = synth.make_batch("head32b")
    sel = ofast.select(b["cu_seqlens"], b["ctx_len"], b["done"], b["input_ids"], b["tail_drop"])
    fin = np.repeat(b["done"] != 0, np.diff(sel["sel_off"]))
    rows = sel["sel_rows"][fin]
    assert len(rows) == sel["N_val"]
    w = synth.f32_to_bf16_bits((np.random.default_rng(2).normal(size=b["H"]) / np.sqrt(b["H"])).astype(np.float32))
    check_value_head(tp, b["hidden"], w, 0.0, rows)


@pytest.mark.timeout(600)
def test_hidden_matrix_beyond_4_GiB(tp):
    """Rows of a 9.2 GB hidden matrix (byte offsets past 2^32 and 2^33): log-probs, their derivatives
    and the value head gather rows through 64-bit arithmetic.  The matrix is drawn on the device; the
    picked rows travel to the host for the oracle."""
    import torch
    N, H, V, M = 900_001, 5120, 32000, 320
    rng = np.random.default_rng(31)
    gen = torch.Generator(device="cuda").manual_seed(31)
    hidden = torch.empty(N, H, dtype=torch.bfloat16, device="cuda")
    for r0 in range(0, N, 100_000):
        hidden[r0:r0 + 100_000].normal_(generator=gen)
    edge = [0, 1, N - 2, N - 1] + [2**32 // (2 * H) + d for d in (-1, 0, 1)] + [2**33 // (2 * H) + d for d in (-1, 0, 1)]
    rows = np.unique(np.concatenate([edge, rng.integers(0, N, size=M - len(edge))])).astype(np.int32)
    rng.shuffle(rows)
    M = rows.size
    picked = host(hidden[torch.from_numpy(rows.astype(np.int64)).cuda()].view(torch.int16)).view(np.uint16)
    w = synth.f32_to_bf16_bits((rng.normal(size=(V, H)) * 0.02).astype(np.float32))
    targets = rng.integers(0, V, size=M).astype(np.int32)
    ident = np.arange(M)
    st = tp.new_status("cuda")
    logp, lse = tp.tppo_token_logprobs(hidden, dev(w), dev(rows), dev(targets), status=st)
    ref, ref_lse = ofast.token_logprobs(picked, w, ident, targets)
    assert int(host(st)[0]) == 0
    assert np.abs(host(logp) - ref).max() <= LOGP_ATOL and np.abs(host(lse) - ref_lse).max() <= LOGP_ATOL
    g = rng.normal(size=M).astype(np.float32)
    dh, dw = tp.tppo_token_logprobs_backward(hidden, dev(w), dev(rows), dev(targets), dev(ref_lse.astype(np.float32)), dev(g))
    ref_h, ref_w, abs_h, abs_w = ofast.token_logprob_grads(picked, w, ident, targets, g, return_abs_bounds=True)
    assert_within_term_bound(host(dh), ref_h, abs_h, "grad_hidden")
    assert_within_term_bound(host(dw), ref_w, abs_w, "grad_w")
    wv = synth.f32_to_bf16_bits((rng.normal(size=H) / np.sqrt(H)).astype(np.float32))
    got_v = host(tp.tppo_value_head(hidden, dev(wv), 0.25, dev(rows)))
    ref_v, bound = ofast.value_head(picked, wv, 0.25, ident, return_abs_bound=True)
    assert np.all(np.abs(got_v - ref_v) <= 1e-5 * (bound + 0.25))
    del hidden
    torch.cuda.empty_cache()


# ------------------------------------------------------------------ EGAE
def check_egae(tp, rewards, values, resp_off, done, gamma, lam, bootstrap=None):
    st = tp.new_status("cuda")
    adv, ret = tp.tppo_egae(dev(rewards), dev(values), dev(resp_off.astype(np.int32)),
                            dev(done.astype(np.int32)), gamma, lam,
                            bootstrap=dev(bootstrap), status=st)
    # the ABI takes gamma and lambda as fp32: the oracle gets the same rounded values
    ref_a, ref_r = ofast.egae(rewards, values, resp_off, done, float(np.float32(gamma)),
                              float(np.float32(lam)), bootstrap)
    assert int(host(st)[0]) == 0
    assert_egae_close(host(adv), ref_a, "adv")
    assert_egae_close(host(ret), ref_r, "ret")
    return host(adv), host(ret)


@pytest.mark.timeout(300)
@pytest.mark.parametrize("name", ["tiny", "small", "head7b", "head32b", "longcot"])
@pytest.mark.parametrize("lam", [0.0, 0.95, 1.0])
def test_egae_configs(tp, name, lam):
    b = synth.make_batch(name, with_head=False)
    check_egae(tp, b["rewards"], b["values"], b["resp_off"], b["done"], b["gamma"], lam)


@pytest.mark.timeout(600)
def test_egae_longcot5x(tp):
    """The 10.5 M-token reading of the long-CoT workload (2176 sequences), paper rule and bootstrap array."""
    b = synth.make_batch("longcot5x", with_head=False)
    check_egae(tp, b["rewards"], b["values"], b["resp_off"], b["done"], b["gamma"], b["lam"])
    check_egae(tp, b["rewards"], b["values"], b["resp_off"], b["done"], b["gamma"], 1.0, b["bootstrap"])


def test_egae_one_very_long_sequence(tp):
    """Sequences of 140 k - 300 k tokens between short ones: the carry of such a sequence is
    collected from well over a hundred work units to its right."""
    rng = np.random.default_rng(21)
    lens = np.array([5, 140001, 1, 2048, 300017, 1024, 3, 163840])
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    n = int(off[-1])
    done = np.array([1, 0, 1, 0, 1, 1, 0, 0], np.int32)
    r = np.where(rng.random(n) < 0.01, rng.normal(size=n), 0.0).astype(np.float32)
    v = rng.uniform(-1, 1, size=n).astype(np.float32)
    boot = rng.uniform(-1, 1, size=lens.size).astype(np.float32)
    for g, l in ((1.0, 1.0), (1.0, 0.95), (0.9999, 1.0)):
        check_egae(tp, r, v, off, done, g, l)
        check_egae(tp, r, v, off, done, g, l, boot)


def test_egae_bootstrap_and_discount(tp):
    b = synth.make_batch("longcot", with_head=False, B=64)
    check_egae(tp, b["rewards"], b["values"], b["resp_off"], b["done"], 1.0, 0.95, b["bootstrap"])
    check_egae(tp, b["rewards"], b["values"], b["resp_off"], b["done"], 0.999, 0.9, b["bootstrap"])
    dense = np.random.default_rng(3).normal(size=b["n_resp"]).astype(np.float32) * 0.01
    check_egae(tp, dense, b["values"], b["resp_off"], b["done"], 0.9995, 1.0)


def test_egae_exact_zero_cases(tp):
    b = synth.make_batch("small", with_head=False)
    n = b["n_resp"]
    trunc = np.zeros_like(b["done"])
    adv, ret = check_egae(tp, np.zeros(n, np.float32), np.full(n, 0.37, np.float32), b["resp_off"],
                          trunc, 1.0, 0.95)
    assert np.all(adv == 0.0) and np.all(ret == 0.0)
    adv, _ = check_egae(tp, np.zeros(n, np.float32), b["values"], b["resp_off"], trunc, 1.0, 0.95)
    assert np.all(adv[b["resp_off"][1:] - 1] == 0.0)     # last token of a truncated sequence


def test_egae_ragged_segment_shapes(tp):
    rng = np.random.default_rng(12)
    # length-1 sequences, empty sequences, many short ones inside one tile, one
    # sequence spanning many tiles, a total that is not a multiple of the vector width
    lens = np.concatenate([[1, 1, 0, 3, 0, 0, 2], rng.integers(1, 9, size=700), [30011], [1],
                           rng.integers(1, 5000, size=9), [0, 7]])
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    n = int(off[-1])
    done = rng.integers(0, 2, size=lens.size).astype(np.int32)
    r = rng.normal(size=n).astype(np.float32)
    v = rng.uniform(-1, 1, size=n).astype(np.float32)
    boot = rng.uniform(-1, 1, size=lens.size).astype(np.float32)
    for g, l in ((1.0, 0.95), (1.0, 1.0), (0.99, 0.5), (0.0, 0.7), (1.0, 0.0)):
        check_egae(tp, r, v, off, done, g, l)
        check_egae(tp, r, v, off, done, g, l, boot)


def test_egae_unaligned_pointers(tp):
    import torch
    b = synth.make_batch("small", with_head=False)
    n = b["n_resp"]
    pad = lambda a: torch.cat([torch.zeros(1, device="cuda"), dev(a)])[1:]    # 4-byte aligned only
    r, v = pad(b["rewards"]), pad(b["values"])
    assert r.data_ptr() % 16 != 0
    adv, ret = tp.tppo_egae(r, v, dev(b["resp_off"]), dev(b["done"]), 1.0, 0.95)
    ref_a, ref_r = ofast.egae(b["rewards"], b["values"], b["resp_off"], b["done"], 1.0,
                              float(np.float32(0.95)))
    assert_egae_close(host(adv), ref_a, "adv")
    assert_egae_close(host(ret), ref_r, "ret")
    assert n == adv.numel()


def test_egae_empty(tp):
    import torch
    e = torch.zeros(0, device="cuda")
    z = torch.zeros(1, dtype=torch.int32, device="cuda")
    adv, ret = tp.tppo_egae(e, e, z, torch.zeros(0, dtype=torch.int32, device="cuda"), 1.0, 0.95)
    assert adv.numel() == 0 and ret.numel() == 0


@pytest.mark.parametrize("name,lam,gamma", [("tiny", 0.95, 1.0), ("small", 1.0, 1.0), ("longcot", 0.95, 0.999)])
def test_egae_terminal_reward_equals_dense(tp, name, lam, gamma):
    """One reward per finished sequence (Sec. 2.1) instead of a dense array: the
    oracle evaluates the dense array built from it; the two entry points agree bit for bit."""
    b = synth.make_batch(name, with_head=False)
    off, done = b["resp_off"], b["done"]
    rng = np.random.default_rng(11)
    terminal = rng.choice([-1.0, 1.0], size=len(done)).astype(np.float32)   # also set for unfinished ones: ignored
    dense = np.zeros(b["n_resp"], np.float32)
    for i in range(len(done)):
        if done[i] != 0 and off[i + 1] > off[i]:
            dense[off[i + 1] - 1] = terminal[i]
    st = tp.new_status("cuda")
    adv, ret = tp.tppo_egae_terminal(dev(terminal), dev(b["values"]), dev(off.astype(np.int32)),
                                     dev(done.astype(np.int32)), gamma, lam, status=st)
    ref_a, ref_r = ofast.egae(dense, b["values"], off, done, float(np.float32(gamma)), float(np.float32(lam)))
    assert int(host(st)[0]) == 0
    assert_egae_close(host(adv), ref_a, "adv")
    assert_egae_close(host(ret), ref_r, "ret")
    adv2, ret2 = tp.tppo_egae(dev(dense), dev(b["values"]), dev(off.astype(np.int32)),
                              dev(done.astype(np.int32)), gamma, lam)
    assert np.array_equal(host(adv), host(adv2)) and np.array_equal(host(ret), host(ret2))


# ------------------------------------------------------------------ losses
def loss_inputs(b, rng=None):
    adv, ret = ofast.egae(b["rewards"], b["values"], b["resp_off"], b["done"], b["gamma"], b["lam"])
    keep = np.where(b["done"] != 0, b["win_len"], np.maximum(b["win_len"] - b["tail_drop"], 0)).astype(np.int32)
    arrs = dict(logp_new=b["logp_new_synth"], logp_old=(b["logp_new_synth"] + b["logp_gap"]).astype(np.float32),
                adv=adv.astype(np.float32), v_new=b["v_new"], v_old=b["values"], ret=ret.astype(np.float32))
    return arrs, keep


def run_losses(tp, a, b, keep, eps=None, skip=None):
    eps = eps or (b["eps_low"], b["eps_high"])
    d = {k: dev(v) for k, v in a.items()}
    if skip == "policy":
        d["logp_new"] = d["logp_old"] = d["adv"] = None
    if skip == "value":
        d["v_new"] = d["v_old"] = d["ret"] = None
    res = tp.tppo_ppo_losses(d["logp_new"], d["logp_old"], d["adv"], d["v_new"], d["v_old"], d["ret"],
                             dev(b["resp_off"]), dev(keep), dev(b["done"]), eps[0], eps[1],
                             b["xi_low"], b["xi_high"])
    return tp.read_loss_out(res)


def assert_loss_close(got, ref):
    for k in ("policy_loss", "value_loss", "policy_sum", "value_sum"):
        assert abs(got[k] - ref[k]) <= LOSS_RTOL * abs(ref[k]) + 1e-12, (k, got[k], ref[k])
    assert got["n_policy"] == ref["n_policy"] and got["n_value"] == ref["n_value"]


@pytest.mark.timeout(600)
@pytest.mark.parametrize("name", ["tiny", "small", "head7b", "head32b", "longcot", "longcot5x"])
def test_losses_configs(tp, name):
    b = synth.make_batch(name, with_head=False)
    a, keep = loss_inputs(b)
    ref = ofast.ppo_losses(a["logp_new"], a["logp_old"], a["adv"], a["v_new"], a["v_old"], a["ret"],
                           b["resp_off"], keep, b["done"], b["eps_low"], b["eps_high"], b["xi_low"], b["xi_high"])
    got = run_losses(tp, a, b, keep)
    assert_loss_close(got, ref)
    assert got == run_losses(tp, a, b, keep)              # deterministic reduction
    if name == "tiny":                                    # the literal "clip 0.2" and the paper's 0.2/0.28
        ref2 = ofast.ppo_losses(a["logp_new"], a["logp_old"], a["adv"], a["v_new"], a["v_old"], a["ret"],
                                b["resp_off"], keep, b["done"], 0.2, 0.28, b["xi_low"], b["xi_high"])
        assert_loss_close(run_losses(tp, a, b, keep, eps=(0.2, 0.28)), ref2)


def test_losses_keep_len_outside_the_window(tp):
    """keep_len beyond the window means every window token, a negative one none (the policy set is the window
    tokens t < keep_len[i]): losses and derivatives as with the clamped values."""
    b = synth.make_batch("small", with_head=False)
    a, keep = loss_inputs(b)
    win = np.diff(b["resp_off"])
    wild = keep.copy()
    wild[::3] = win[::3] + 7
    wild[1::3] = -5
    clamped = np.clip(wild, 0, win).astype(np.int32)
    ref = ofast.ppo_losses(a["logp_new"], a["logp_old"], a["adv"], a["v_new"], a["v_old"], a["ret"],
                           b["resp_off"], clamped, b["done"], b["eps_low"], b["eps_high"], b["xi_low"], b["xi_high"])
    got = run_losses(tp, a, b, wild)
    assert_loss_close(got, ref)
    assert got == run_losses(tp, a, b, clamped)
    g_wild, g_clamped = run_loss_grads(tp, a, b, wild), run_loss_grads(tp, a, b, clamped)
    assert np.array_equal(g_wild[0], g_clamped[0]) and np.array_equal(g_wild[1], g_clamped[1])


def test_losses_masked_entries_contribute_exactly_zero(tp):
    b = synth.make_batch("small", with_head=False)
    a, keep = loss_inputs(b)
    clean = run_losses(tp, a, b, keep)
    pol, val = ofast.loss_masks(b["resp_off"], keep, b["done"])
    p = {k: v.copy() for k, v in a.items()}
    for k in ("logp_new", "logp_old", "adv"):
        p[k][~pol] = np.nan
    for k in ("v_new", "v_old", "ret"):
        p[k][~val] = np.inf
    assert run_losses(tp, p, b, keep) == clean            # bit-identical


def test_nan_inside_a_set_reaches_the_loss_and_its_derivative(tp):
    """A NaN in an entry that IS in a token set (a diverged model, a bad log-prob) must not be clipped
    away: the loss of that half is NaN, the derivative at that token is NaN, every other derivative and
    the other half are untouched.  Entries outside the sets still cannot reach anything."""
    b = synth.make_batch("small", with_head=False)
    a, keep = loss_inputs(b)
    pol, val = ofast.loss_masks(b["resp_off"], keep, b["done"])
    clean = run_losses(tp, a, b, keep)
    g_lp, g_v, _, _ = run_loss_grads(tp, a, b, keep)
    ip, iv = int(np.flatnonzero(pol)[777]), int(np.flatnonzero(val)[555])
    for key, idx, half in (("logp_new", ip, "policy"), ("logp_old", ip, "policy"), ("adv", ip, "policy"),
                           ("v_new", iv, "value"), ("v_old", iv, "value"), ("ret", iv, "value")):
        p = {k: v.copy() for k, v in a.items()}
        p[key][idx] = np.nan
        ref = ofast.ppo_losses(p["logp_new"], p["logp_old"], p["adv"], p["v_new"], p["v_old"], p["ret"],
                               b["resp_off"], keep, b["done"], b["eps_low"], b["eps_high"], b["xi_low"], b["xi_high"])
        og = ofast.ppo_loss_grads(p["logp_new"], p["logp_old"], p["adv"], p["v_new"], p["v_old"], p["ret"],
                                  b["resp_off"], keep, b["done"], b["eps_low"], b["eps_high"], b["xi_low"], b["xi_high"])
        got = run_losses(tp, p, b, keep)
        q_lp, q_v, q_loss, q_stats = run_loss_grads(tp, p, b, keep)
        bad, good = (("policy_loss", "value_loss") if half == "policy" else ("value_loss", "policy_loss"))
        assert np.isnan(ref[bad]) and np.isnan(got[bad]) and np.isnan(q_loss[bad]), (key, got)
        assert got[good] == clean[good] and not np.isnan(ref[good])
        assert got["n_policy"] == clean["n_policy"] and got["n_value"] == clean["n_value"]
        g_bad, g_ref, g_clean = (q_lp, og["grad_logp"], g_lp) if half == "policy" else (q_v, og["grad_v"], g_v)
        assert np.isnan(g_ref[idx]) and np.isnan(g_bad[idx]), key
        others = np.arange(g_bad.size) != idx
        assert np.array_equal(g_bad[others], g_clean[others])
        assert np.array_equal(q_v if half == "policy" else q_lp, g_v if half == "policy" else g_lp)
        # a token whose inputs are NaN is neither "clipped" nor "unclipped"
        assert q_stats["n_policy_clipped"] == og["n_policy_clipped"] and q_stats["n_value_clipped"] == og["n_value_clipped"]


def test_losses_halves_and_empty_sets(tp):
    b = synth.make_batch("small", with_head=False)
    a, keep = loss_inputs(b)
    full = run_losses(tp, a, b, keep)
    only_v = run_losses(tp, a, b, keep, skip="policy")
    only_p = run_losses(tp, a, b, keep, skip="value")
    assert only_v["value_loss"] == full["value_loss"] and only_v["policy_loss"] == 0.0 and only_v["n_policy"] == 0
    assert only_p["policy_loss"] == full["policy_loss"] and only_p["value_loss"] == 0.0 and only_p["n_value"] == 0
    # policy tokens dropped from finished sequences too: the value set is still their whole window
    half = (keep // 2).astype(np.int32)
    ref = ofast.ppo_losses(a["logp_new"], a["logp_old"], a["adv"], a["v_new"], a["v_old"], a["ret"],
                           b["resp_off"], half, b["done"], b["eps_low"], b["eps_high"], b["xi_low"], b["xi_high"])
    got = run_losses(tp, a, b, half)
    assert_loss_close(got, ref)
    assert got["n_value"] == full["n_value"] and got["n_policy"] < full["n_policy"]
    # nothing kept and nothing finished
    none_done = dict(b, done=np.zeros_like(b["done"]))
    got = run_losses(tp, a, none_done, np.zeros_like(keep))
    assert got["policy_loss"] == 0.0 and got["value_loss"] == 0.0 and got["n_policy"] == 0 and got["n_value"] == 0


def test_losses_split_batch_additivity(tp):
    b = synth.make_batch("small", with_head=False)
    a, keep = loss_inputs(b)
    full = run_losses(tp, a, b, keep)
    k = 13
    cut = int(b["resp_off"][k])
    first = dict(b, resp_off=b["resp_off"][:k + 1], done=b["done"][:k])
    second = dict(b, resp_off=(b["resp_off"][k:] - cut).astype(np.int32), done=b["done"][k:])
    g1 = run_losses(tp, {n: v[:cut] for n, v in a.items()}, first, keep[:k])
    g2 = run_losses(tp, {n: v[cut:] for n, v in a.items()}, second, keep[k:])
    assert abs(g1["policy_sum"] + g2["policy_sum"] - full["policy_sum"]) <= 1e-4 * abs(full["policy_sum"])
    assert abs(g1["value_sum"] + g2["value_sum"] - full["value_sum"]) <= 1e-4 * abs(full["value_sum"])
    assert g1["n_policy"] + g2["n_policy"] == full["n_policy"]
    assert g1["n_value"] + g2["n_value"] == full["n_value"]


# ------------------------------------------------------------------ loss derivatives
GRAD_RTOL = 1e-5      # fp32 exp, two products and one scale: a few 1e-7 relative; 1e-5 leaves a decade


def run_loss_grads(tp, a, b, keep, skip=None, **kw):
    d = {k: dev(v) for k, v in a.items()}
    if skip == "policy":
        d["logp_new"] = d["logp_old"] = d["adv"] = None
    if skip == "value":
        d["v_new"] = d["v_old"] = d["ret"] = None
    g_lp, g_v, res, st = tp.tppo_ppo_losses_backward(
        d["logp_new"], d["logp_old"], d["adv"], d["v_new"], d["v_old"], d["ret"], dev(b["resp_off"]),
        dev(keep), dev(b["done"]), b["eps_low"], b["eps_high"], b["xi_low"], b["xi_high"], **kw)
    return (None if g_lp is None else g_lp.cpu().numpy(), None if g_v is None else g_v.cpu().numpy(),
            tp.read_loss_out(res), tp.read_loss_stats(st))


def near_kinks(a, b, keep):
    """Tokens whose branch (clipped or not) is decided by less than 1e-5: there the
    fp32 decision of the kernel may legitimately differ from the fp64 one."""
    pol, val = ofast.loss_masks(b["resp_off"], keep, b["done"])
    f = {k: v.astype(np.float64) for k, v in a.items()}
    with np.errstate(all="ignore"):
        rho = np.exp(f["logp_new"] - f["logp_old"])
        kp = pol & ((np.abs(rho - (1 - np.float32(b["eps_low"]))) < 1e-5) | (np.abs(rho - (1 + np.float32(b["eps_high"]))) < 1e-5))
        lo, hi = f["v_old"] - b["xi_low"], f["v_old"] + b["xi_high"]
        d0 = f["v_new"] - f["ret"]
        d1 = np.clip(f["v_new"], lo, hi) - f["ret"]
        scale = np.maximum(1.0, np.abs(f["v_new"]))
        kv = val & ((np.abs(f["v_new"] - lo) < 1e-5 * scale) | (np.abs(f["v_new"] - hi) < 1e-5 * scale) |
                    ((d0 != d1) & (np.abs(d0 * d0 - d1 * d1) < 1e-5 * np.maximum(d0 * d0, 1e-12))))
    return kp, kv


def assert_grads_close(got, ref, kink, unclipped_value):
    """Element by element; at a near-kink token either branch's value is accepted."""
    tol = GRAD_RTOL * np.abs(ref) + 1e-30
    ok = np.abs(got - ref) <= tol
    alt = kink & ((got == 0.0) | (np.abs(got - unclipped_value) <= GRAD_RTOL * np.abs(unclipped_value) + 1e-30))
    bad = ~(ok | alt)
    assert not bad.any(), (int(bad.sum()), np.flatnonzero(bad)[:5], got[bad][:5], ref[bad][:5])


@pytest.mark.timeout(600)
@pytest.mark.parametrize("name", ["tiny", "small", "head7b", "head32b", "longcot", "longcot5x"])
def test_loss_grads_configs(tp, name):
    b = synth.make_batch(name, with_head=False)
    a, keep = loss_inputs(b)
    kw = dict(policy_scale=1.0, value_scale=0.5)
    ref = ofast.ppo_loss_grads(a["logp_new"], a["logp_old"], a["adv"], a["v_new"], a["v_old"], a["ret"],
                               b["resp_off"], keep, b["done"], float(np.float32(b["eps_low"])),
                               float(np.float32(b["eps_high"])), float(np.float32(b["xi_low"])),
                               float(np.float32(b["xi_high"])), **kw)
    g_lp, g_v, losses, stats = run_loss_grads(tp, a, b, keep, **kw)
    kp, kv = near_kinks(a, b, keep)
    f = {k: v.astype(np.float64) for k, v in a.items()}
    with np.errstate(all="ignore"):
        free_p = -np.exp(f["logp_new"] - f["logp_old"]) * f["adv"] / max(ref["n_policy"], 1)
        free_v = 0.5 * (f["v_new"] - f["ret"]) / max(ref["n_value"], 1)
    assert_grads_close(g_lp, ref["grad_logp"], kp, free_p)
    assert_grads_close(g_v, ref["grad_v"], kv, free_v)
    pol, val = ofast.loss_masks(b["resp_off"], keep, b["done"])
    assert not g_lp[~pol].any() and not g_v[~val].any()            # exact zeros outside the sets
    assert abs(stats["n_policy_clipped"] - ref["n_policy_clipped"]) <= int(kp.sum())
    assert abs(stats["n_value_clipped"] - ref["n_value_clipped"]) <= int(kv.sum())
    assert abs(stats["ratio_mean"] - ref["ratio_mean"]) <= 1e-5 * ref["ratio_mean"]
    assert ref["n_policy_clipped"] > 0 and ref["n_value_clipped"] > 0  # both branches are exercised
    # the losses of the same pass agree with the forward entry point
    fwd = run_losses(tp, a, b, keep)
    for k in ("policy_loss", "value_loss"):
        assert abs(losses[k] - fwd[k]) <= 1e-6 * abs(fwd[k]) + 1e-12
    assert losses["n_policy"] == fwd["n_policy"] and losses["n_value"] == fwd["n_value"]
    # deterministic
    g2 = run_loss_grads(tp, a, b, keep, **kw)
    assert np.array_equal(g2[0], g_lp) and np.array_equal(g2[1], g_v) and g2[3] == stats


def test_loss_grads_poison_halves_denominators(tp):
    b = synth.make_batch("small", with_head=False)
    a, keep = loss_inputs(b)
    g_lp, g_v, _, stats = run_loss_grads(tp, a, b, keep)
    pol, val = ofast.loss_masks(b["resp_off"], keep, b["done"])
    p = {k: v.copy() for k, v in a.items()}
    for k in ("logp_new", "logp_old", "adv"):
        p[k][~pol] = np.nan
    for k in ("v_new", "v_old", "ret"):
        p[k][~val] = np.inf
    q_lp, q_v, _, qstats = run_loss_grads(tp, p, b, keep)
    assert np.array_equal(q_lp, g_lp) and np.array_equal(q_v, g_v) and qstats == stats   # bit-identical
    # one half only
    only_p = run_loss_grads(tp, a, b, keep, skip="value")
    only_v = run_loss_grads(tp, a, b, keep, skip="policy")
    assert only_p[1] is None and np.array_equal(only_p[0], g_lp)
    assert only_v[0] is None and np.array_equal(only_v[1], g_v)
    # explicit denominators and scales: a plain rescaling of the same derivatives
    n_pol, n_val = int(pol.sum()), int(val.sum())
    s_lp, s_v, _, _ = run_loss_grads(tp, a, b, keep, policy_scale=2.0, value_scale=-1.0,
                                     policy_denominator=4 * n_pol, value_denominator=2 * n_val)
    assert np.allclose(s_lp, 0.5 * g_lp, rtol=1e-6, atol=0) and np.allclose(s_v, -0.5 * g_v, rtol=1e-6, atol=0)
    # nothing kept, nothing finished: all zeros
    none_done = dict(b, done=np.zeros_like(b["done"]))
    z_lp, z_v, zl, zs = run_loss_grads(tp, a, none_done, np.zeros_like(keep))
    assert not z_lp.any() and not z_v.any() and zl["n_policy"] == 0 and zs["n_policy_clipped"] == 0


# ------------------------------------------------------------------ whole path
def test_whole_path_tiny(tp):
    """select -> log-probs -> EGAE -> losses chained on device buffers, against
    the same chain in the oracle (config 1, both clip settings)."""
    import torch
    b = synth.make_batch("tiny")
    sel = tp.tppo_select(dev(b["cu_seqlens"]), dev(b["ctx_len"]), dev(b["done"]), dev(b["input_ids"]),
                         b["tail_drop"])
    n_resp = b["n_resp"]
    logp, _ = tp.tppo_token_logprobs(dev(b["hidden"]), dev(b["w_head"]), sel["sel_rows"],
                                     sel["sel_targets"], M=b["n_tok"], m_actual=sel["counts"],
                                     out_index=sel["sel_resp_idx"], out_size=n_resp)
    adv, ret = tp.tppo_egae(dev(b["rewards"]), dev(b["values"]), sel["resp_off"], dev(b["done"]),
                            b["gamma"], b["lam"])
    # oracle chain
    osel = ofast.select(b["cu_seqlens"], b["ctx_len"], b["done"], b["input_ids"], b["tail_drop"])
    olp, _ = ofast.token_logprobs(b["hidden"], b["w_head"], osel["sel_rows"], osel["sel_targets"])
    o_new = np.zeros(n_resp); o_new[osel["sel_resp_idx"]] = olp
    o_old = o_new + b["logp_gap"]
    oadv, oret = ofast.egae(b["rewards"], b["values"], osel["resp_off"], b["done"], b["gamma"], b["lam"])
    logp_old = dev(o_old.astype(np.float32))
    for eps in ((0.2, 0.2), (0.2, 0.28)):
        res = tp.tppo_ppo_losses(logp, logp_old, adv, dev(b["v_new"]), dev(b["values"]), ret,
                                 sel["resp_off"], sel["keep_len"], dev(b["done"]), eps[0], eps[1],
                                 b["xi_low"], b["xi_high"])
        got = tp.read_loss_out(res)
        ref = ofast.ppo_losses(o_new, o_old.astype(np.float32), oadv, b["v_new"], b["values"], oret,
                               osel["resp_off"], osel["keep_len"], b["done"], eps[0], eps[1],
                               b["xi_low"], b["xi_high"])
        assert_loss_close(got, ref)
    torch.cuda.synchronize()


@pytest.mark.timeout(600)
def test_whole_path_small_config_full(tp):
    """Config 2 at its own size (bf16, H = 1024, V = 32000, 32 sequences), every stage fed by the stage
    before it on device buffers, lambda in {0, 0.95, 1}; against the same chain in the oracle."""
    b, osel, olp, _ = small_full_oracle()
    n_resp = b["n_resp"]
    st = tp.new_status("cuda")
    sel = tp.tppo_select(dev(b["cu_seqlens"]), dev(b["ctx_len"]), dev(b["done"]), dev(b["input_ids"]),
                         b["tail_drop"], status=st)
    logp, _ = tp.tppo_token_logprobs(dev(b["hidden"]), dev(b["w_head"]), sel["sel_rows"], sel["sel_targets"],
                                     M=b["n_tok"], m_actual=sel["counts"], out_index=sel["sel_resp_idx"],
                                     out_size=n_resp, status=st)
    o_new = np.zeros(n_resp); o_new[osel["sel_resp_idx"]] = olp
    o_old = (o_new + b["logp_gap"]).astype(np.float32)
    logp_old = dev(o_old)
    for lam in (0.0, 0.95, 1.0):
        adv, ret = tp.tppo_egae(dev(b["rewards"]), dev(b["values"]), sel["resp_off"], dev(b["done"]),
                                b["gamma"], lam, status=st)
        res = tp.tppo_ppo_losses(logp, logp_old, adv, dev(b["v_new"]), dev(b["values"]), ret, sel["resp_off"],
                                 sel["keep_len"], dev(b["done"]), b["eps_low"], b["eps_high"], b["xi_low"],
                                 b["xi_high"], status=st)
        oadv, oret = ofast.egae(b["rewards"], b["values"], osel["resp_off"], b["done"], b["gamma"],
                                float(np.float32(lam)))
        ref = ofast.ppo_losses(o_new, o_old, oadv, b["v_new"], b["values"], oret, osel["resp_off"],
                               osel["keep_len"], b["done"], b["eps_low"], b["eps_high"], b["xi_low"], b["xi_high"])
        assert_egae_close(host(adv), oadv, "adv")
        assert_loss_close(tp.read_loss_out(res), ref)
    assert int(host(st)[0]) == 0


def test_whole_update_step_small(tp):
    """Forward and backward chained on device buffers (a slice of config 2):
    select -> log-probs -> EGAE -> loss derivatives -> log-prob derivatives, i.e.
    d policy_loss / d hidden rows and / d W, against the same chain in the oracle."""
    import torch
    b = synth.make_batch("small", B=4, V=2000, H=256)
    sel = tp.tppo_select(dev(b["cu_seqlens"]), dev(b["ctx_len"]), dev(b["done"]), dev(b["input_ids"]),
                         b["tail_drop"])
    n_resp = b["n_resp"]
    M = int(host(sel["counts"])[0])
    hidden, w = dev(b["hidden"]), dev(b["w_head"])
    logp, lse = tp.tppo_token_logprobs(hidden, w, sel["sel_rows"], sel["sel_targets"], M=M,
                                       out_index=sel["sel_resp_idx"], out_size=n_resp)
    adv, ret = tp.tppo_egae(dev(b["rewards"]), dev(b["values"]), sel["resp_off"], dev(b["done"]),
                            b["gamma"], b["lam"])
    # oracle chain up to the old policy's log-probs (an input of the update)
    osel = ofast.select(b["cu_seqlens"], b["ctx_len"], b["done"], b["input_ids"], b["tail_drop"])
    olp, olse = ofast.token_logprobs(b["hidden"], b["w_head"], osel["sel_rows"], osel["sel_targets"])
    o_new = np.zeros(n_resp); o_new[osel["sel_resp_idx"]] = olp
    o_old = (o_new + b["logp_gap"]).astype(np.float32)
    oadv, oret = ofast.egae(b["rewards"], b["values"], osel["resp_off"], b["done"], b["gamma"], b["lam"])
    g_lp, g_v, res, st = tp.tppo_ppo_losses_backward(logp, dev(o_old), adv, dev(b["v_new"]), dev(b["values"]),
                                                     ret, sel["resp_off"], sel["keep_len"], dev(b["done"]),
                                                     b["eps_low"], b["eps_high"], b["xi_low"], b["xi_high"])
    dh, dw = tp.tppo_token_logprobs_backward(hidden, w, sel["sel_rows"], sel["sel_targets"], lse, g_lp, M=M,
                                             in_index=sel["sel_resp_idx"])
    torch.cuda.synchronize()
    og = ofast.ppo_loss_grads(o_new, o_old, oadv, b["v_new"], b["values"], oret, osel["resp_off"],
                              osel["keep_len"], b["done"], float(np.float32(b["eps_low"])),
                              float(np.float32(b["eps_high"])), float(np.float32(b["xi_low"])),
                              float(np.float32(b["xi_high"])))
    a = dict(logp_new=o_new.astype(np.float32), logp_old=o_old, adv=oadv.astype(np.float32), v_new=b["v_new"],
             v_old=b["values"], ret=oret.astype(np.float32))
    kp, kv = near_kinks(a, b, osel["keep_len"])
    assert not kp.any() and not kv.any()                     # this seed has no token within 1e-5 of a clip bound
    g_tok = og["grad_logp"][osel["sel_resp_idx"]]
    assert np.allclose(host(g_lp)[osel["sel_resp_idx"]], g_tok, rtol=1e-4, atol=1e-9)
    ref_h, ref_w, abs_h, abs_w = ofast.token_logprob_grads(b["hidden"], b["w_head"], osel["sel_rows"],
                                                           osel["sel_targets"], g_tok, return_abs_bounds=True)
    # on top of the bf16 term bound: the upstream derivative itself carries the log-probs' error (2e-3 absolute
    # on logp moves rho, hence g, by up to 2e-3 relative)
    tol_h = (DZ_RTOL + 4e-3) * abs_h + 1e-6 * abs_h.max()
    tol_w = (DZ_RTOL + 4e-3) * abs_w + 1e-6 * abs_w.max()
    assert np.all(np.abs(host(dh) - ref_h) <= tol_h) and np.all(np.abs(host(dw) - ref_w) <= tol_w)


def test_whole_step_captured_in_a_graph_replays_like_eager(tp):
    """The library neither allocates nor synchronises nor clears memory with memset nodes, so a whole
    step (select -> log-probs -> EGAE -> losses) can be captured in a HIP graph.  Every replay, with the
    inputs changed in place and eager work in between, must reproduce the eager step bit for bit."""
    import torch
    b = synth.make_batch("small", B=4, V=2000, H=256)
    n_resp, n_tok = b["n_resp"], b["n_tok"]
    rng = np.random.default_rng(77)
    cu, ctx, done, ids = dev(b["cu_seqlens"]), dev(b["ctx_len"]), dev(b["done"]), dev(b["input_ids"])
    hidden, w = dev(b["hidden"]), dev(b["w_head"])
    rewards, values, v_new = dev(b["rewards"]), dev(b["values"]), dev(b["v_new"])
    logp_old = dev((-np.abs(rng.normal(size=n_resp)) - 6.0).astype(np.float32))

    def step():
        sel = tp.tppo_select(cu, ctx, done, ids, b["tail_drop"], want_plan=True)
        logp, _ = tp.tppo_token_logprobs(hidden, w, sel["sel_rows"], sel["sel_targets"], M=n_tok,
                                         m_actual=sel["counts"], out_index=sel["sel_resp_idx"], out_size=n_resp)
        adv, ret = tp.tppo_egae(rewards, values, sel["resp_off"], done, b["gamma"], b["lam"], plan=sel["plan"])
        res = tp.tppo_ppo_losses(logp, logp_old, adv, v_new, values, ret, sel["resp_off"], sel["keep_len"], done,
                                 b["eps_low"], b["eps_high"], b["xi_low"], b["xi_high"], plan=sel["plan"])
        return sel, logp, adv, ret, res

    step()                                                    # first calls (occupancy queries, attributes) outside
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            g_sel, g_logp, g_adv, g_ret, g_res = step()
    torch.cuda.current_stream().wait_stream(side)
    for trial in range(4):
        if trial:                                             # new inputs, same buffers
            hidden.copy_(dev(synth.f32_to_bf16_bits(rng.normal(size=b["hidden"].shape).astype(np.float32))))
            values.copy_(dev(rng.uniform(-1, 1, size=n_resp).astype(np.float32)))
            rewards.copy_(dev(np.where(rng.random(n_resp) < 0.01, 1.0, 0.0).astype(np.float32)))
            ids.copy_(dev(rng.integers(0, 2000, size=n_tok).astype(np.int32)))
        graph.replay()
        torch.cuda.synchronize()
        got = [host(t).copy() for t in (g_sel["sel_resp_idx"], g_sel["counts"], g_logp, g_adv, g_ret, g_res)]
        e_sel, e_logp, e_adv, e_ret, e_res = step()           # eager work between the replays
        torch.cuda.synchronize()
        M = int(got[1][0])
        assert M > 0 and np.array_equal(got[1], host(e_sel["counts"]))
        kept = got[0][:M]
        assert np.array_equal(kept, host(e_sel["sel_resp_idx"])[:M])
        assert np.array_equal(got[2][kept], host(e_logp)[kept]), trial
        assert np.array_equal(got[3], host(e_adv)) and np.array_equal(got[4], host(e_ret)), trial
        assert np.array_equal(got[5], host(e_res)), trial
    # and the last replay against the oracle
    osel = ofast.select(b["cu_seqlens"], b["ctx_len"], b["done"], host(ids), b["tail_drop"])
    olp, _ = ofast.token_logprobs(host(hidden.view(torch.int16)).view(np.uint16), b["w_head"], osel["sel_rows"],
                                  osel["sel_targets"])
    assert np.max(np.abs(got[2][osel["sel_resp_idx"]] - olp)) <= LOGP_ATOL


# ------------------------------------------------------------------ one plan per batch
@pytest.mark.parametrize("name", ["small", "longcot"])
def test_plan_from_select_feeds_every_consumer(tp, name):
    """tppo_select hands out the work plan of the batch; EGAE (dense and terminal rewards), the losses and
    their derivatives take it instead of building their own, any number of times, with results bit-identical
    to the calls that build their own -- and correct against the oracle."""
    import torch
    b = synth.make_batch(name, with_head=False)
    st = tp.new_status("cuda")
    ids = dev(b["input_ids"]) if "input_ids" in b else None
    sel = tp.tppo_select(dev(b["cu_seqlens"]), dev(b["ctx_len"]), dev(b["done"]), ids, b["tail_drop"],
                         n_tok=b["n_tok"], status=st, want_plan=True)
    plan, off, keep, done = sel["plan"], sel["resp_off"], sel["keep_len"], dev(b["done"])
    a, keep_ref = loss_inputs(b)
    assert np.array_equal(host(keep), keep_ref)
    d = {k: dev(v) for k, v in a.items()}
    rewards, values = dev(b["rewards"]), dev(b["values"])
    eps = (b["eps_low"], b["eps_high"], b["xi_low"], b["xi_high"])
    order = ("logp_new", "logp_old", "adv", "v_new", "v_old", "ret")
    for trial, (gamma, lam) in enumerate(((1.0, 0.95), (0.999, 1.0), (1.0, 0.95))):      # the same plan again and again
        adv_p, ret_p = tp.tppo_egae(rewards, values, off, done, gamma, lam, status=st, plan=plan)
        adv_s, ret_s = tp.tppo_egae(rewards, values, off, done, gamma, lam, status=st)
        assert torch.equal(adv_p, adv_s) and torch.equal(ret_p, ret_s), trial
        ref_a, ref_r = ofast.egae(b["rewards"], b["values"], b["resp_off"], b["done"], float(np.float32(gamma)),
                                  float(np.float32(lam)))
        assert_egae_close(host(adv_p), ref_a, "adv")
        assert_egae_close(host(ret_p), ref_r, "ret")
        res_p = tp.read_loss_out(tp.tppo_ppo_losses(*(d[k] for k in order), off, keep, done, *eps, status=st, plan=plan))
        res_s = tp.read_loss_out(tp.tppo_ppo_losses(*(d[k] for k in order), off, keep, done, *eps, status=st))
        assert res_p == res_s
        g_p = tp.tppo_ppo_losses_backward(*(d[k] for k in order), off, keep, done, *eps, status=st, plan=plan)
        g_s = tp.tppo_ppo_losses_backward(*(d[k] for k in order), off, keep, done, *eps, status=st)
        assert torch.equal(g_p[0], g_s[0]) and torch.equal(g_p[1], g_s[1])
        assert tp.read_loss_out(g_p[2]) == res_p and tp.read_loss_stats(g_p[3]) == tp.read_loss_stats(g_s[3])
    ref = ofast.ppo_losses(*(a[k] for k in order), b["resp_off"], keep_ref, b["done"], *eps)
    assert_loss_close(res_p, ref)
    term = dev(np.ones(b["B"], np.float32))
    t_p = tp.tppo_egae_terminal(term, values, off, done, 1.0, 0.95, status=st, plan=plan)
    t_s = tp.tppo_egae_terminal(term, values, off, done, 1.0, 0.95, status=st)
    assert torch.equal(t_p[0], t_s[0]) and torch.equal(t_p[1], t_s[1])
    assert int(host(st)[0]) == 0


def test_plan_build_and_a_plan_of_another_batch(tp):
    import torch
    b = synth.make_batch("small", with_head=False)
    a, keep = loss_inputs(b)
    off, done, keepd = dev(b["resp_off"]), dev(b["done"]), dev(keep)
    rewards, values = dev(b["rewards"]), dev(b["values"])
    plan = tp.tppo_plan_build(off, keepd, done, b["n_resp"])
    adv, ret = tp.tppo_egae(rewards, values, off, done, 1.0, 0.95, plan=plan)
    adv_s, ret_s = tp.tppo_egae(rewards, values, off, done, 1.0, 0.95)
    assert torch.equal(adv, adv_s) and torch.equal(ret, ret_s)
    # a plan without keep_len serves the scan, not the losses
    scan_only = tp.tppo_plan_build(off, None, done, b["n_resp"])
    adv2, _ = tp.tppo_egae(rewards, values, off, done, 1.0, 0.95, plan=scan_only)
    assert torch.equal(adv2, adv)
    d = {k: dev(v) for k, v in a.items()}
    order = ("logp_new", "logp_old", "adv", "v_new", "v_old", "ret")
    st = tp.new_status("cuda")
    res = tp.read_loss_out(tp.tppo_ppo_losses(*(d[k] for k in order), off, keepd, done, 0.2, 0.28, 0.5, 0.6,
                                              status=st, plan=scan_only))
    assert int(host(st)[0]) == tp.STATUS_BAD_LAYOUT and np.isnan(res["policy_loss"])
    # a plan built for other sizes is refused: status bit, outputs untouched
    b2 = synth.make_batch("small", with_head=False, B=5)
    st = tp.new_status("cuda")
    out = (torch.full((b2["n_resp"],), 7.0, device="cuda"), torch.full((b2["n_resp"],), 7.0, device="cuda"))
    tp.tppo_egae(dev(b2["rewards"]), dev(b2["values"]), dev(b2["resp_off"]), dev(b2["done"]), 1.0, 0.95,
                 status=st, plan=plan, out=out)
    assert int(host(st)[0]) == tp.STATUS_BAD_LAYOUT and bool((out[0] == 7.0).all())
    # a frame descriptor that names no sequence: the loss kernels say so and leave its tokens out; one whose
    # other fields are nonsense only changes which tokens count (no access depends on them)
    cap = int(plan[32:36].view(torch.int32)[0])
    at = 256 + (16 * cap + 255) // 256 * 256
    frames = plan[at:at + 32 * cap].view(torch.int32).view(cap, 8)
    good = tp.read_loss_out(tp.tppo_ppo_losses(*(d[k] for k in order), off, keepd, done, 0.2, 0.28, 0.5, 0.6, plan=plan))
    saved = frames[:3].clone()
    frames[0, 0] = len(b["done"]) + 5                                # first sequence out of range
    frames[1, 4] = -1                                          # second sequence out of range
    frames[2, 1:4] = torch.tensor([2 ** 30, -5, 1], dtype=torch.int32, device="cuda")
    st = tp.new_status("cuda")
    res = tp.read_loss_out(tp.tppo_ppo_losses(*(d[k] for k in order), off, keepd, done, 0.2, 0.28, 0.5, 0.6,
                                              status=st, plan=plan))
    assert int(host(st)[0]) == tp.STATUS_BAD_LAYOUT and np.isfinite(res["policy_loss"])
    frames[:3] = saved
    st = tp.new_status("cuda")
    again = tp.read_loss_out(tp.tppo_ppo_losses(*(d[k] for k in order), off, keepd, done, 0.2, 0.28, 0.5, 0.6,
                                                status=st, plan=plan))
    assert int(host(st)[0]) == 0 and again == good


def expected_tiles(off, keep, done):
    """The plan's tiles as the header documents them, worked out on the host: a sequence is cut at multiples of
    1024 of the response-packed index; per tile (first token, tokens, tiles after it), keyed by (sequence, tile
    number in the sequence)."""
    out = {}
    for i in range(len(done)):
        lo, hi = int(off[i]), int(off[i + 1])
        if hi == lo:
            continue
        cuts = [lo] + list(range((lo // 1024 + 1) * 1024, hi, 1024)) + [hi]
        for c in range(len(cuts) - 1):
            first, n = cuts[c], cuts[c + 1] - cuts[c]
            out[(i, c)] = (first, n, len(cuts) - 2 - c)
    return out


def expected_frames(off, keep, done):
    """Per aligned block of 1024 tokens: (sequence of its first token, where that sequence ends, where its
    policy tokens end, finished) and the same for the sequence that follows it inside the block, if one does
    (else the first sequence again, as an empty range)."""
    n, B = int(off[-1]), len(done)
    rows = []
    for start in range(0, n, 1024):
        seg = int(np.searchsorted(off, start, side="right")) - 1  # the last sequence that begins at or before
        lo, hi = int(off[seg]), int(off[seg + 1])
        row = [seg, hi, lo + min(max(int(keep[seg]), 0), hi - lo), int(done[seg] != 0), seg, hi, hi, 0]
        if hi < start + 1024 and hi < n:
            j = seg + 1
            while off[j + 1] <= hi:                               # (the builder gives up after 64 empty sequences)
                j += 1
            assert j - seg <= 64
            hi2 = int(off[j + 1])
            row[4:] = [j, hi2, hi + min(max(int(keep[j]), 0), hi2 - hi), int(done[j] != 0)]
        rows.append(row)
    return np.array(rows, dtype=np.int32).reshape(-1, 8)


@pytest.mark.parametrize("case", ["small", "longcot", "many", "deep", "select"])
def test_plan_lists_every_tile_once_in_level_order(tp, case):
    """The work plan read back from the device: every tile of every sequence exactly once, with the fields the
    consumers rely on, sorted by the number of tiles after it in its sequence (beyond 32, sequence by sequence);
    every frame's descriptor; all tagged words zero after the build."""
    import torch
    rng = np.random.default_rng(77)
    if case in ("small", "longcot", "select"):
        b = synth.make_batch("longcot" if case == "longcot" else "small", with_head=False)
        win, done = np.diff(b["resp_off"]), b["done"]
    elif case == "many":                                     # several builder workgroups, several sequences per thread
        win = rng.integers(0, 3000, size=20011)
        win[rng.random(win.size) < 0.1] = 0
        done = (rng.random(win.size) < 0.5).astype(np.int32)
    else:                                                    # sequences beyond the 32 sorted levels, one of them very long
        win = np.concatenate([[70001, 5, 0, 40000], rng.integers(1, 9000, size=70), [33 * 1024 + 1]])
        done = (rng.random(win.size) < 0.5).astype(np.int32)
    off = np.concatenate([[0], np.cumsum(win)]).astype(np.int32)
    keep = np.where(done != 0, win, np.maximum(win - 128, 0)).astype(np.int32)
    n, B = int(off[-1]), len(done)
    if case == "select":                                     # the plan tppo_select writes: capacity sized for n_tok
        sel, st = run_select(tp, b)
        sel = tp.tppo_select(dev(b["cu_seqlens"]), dev(b["ctx_len"]), dev(b["done"]), None, b["tail_drop"],
                             n_tok=b["n_tok"], want_plan=True)
        plan, keep = sel["plan"], host(sel["keep_len"])
    else:
        plan = tp.tppo_plan_build(dev(off), dev(keep), dev(done.astype(np.int32)), n)
    torch.cuda.synchronize()
    raw = plan.cpu().numpy()
    hdr = raw[:256].view(np.int32)
    n_tiles, cap = int(hdr[0]), int(hdr[8])
    assert (int(hdr[1]), int(hdr[2])) == (B, n) and cap >= n // 1024 + B + 1
    want = expected_tiles(off, keep, done)
    assert n_tiles == len(want)
    tiles = raw[256:256 + 16 * cap].view(np.int32).reshape(cap, 4)[:n_tiles]
    at = 256 + (16 * cap + 255) // 256 * 256
    want_frames = expected_frames(off, keep, done)
    frames = raw[at:at + 32 * cap].view(np.int32).reshape(cap, 8)[:len(want_frames)]
    assert np.array_equal(frames, want_frames)
    at += (32 * cap + 255) // 256 * 256
    assert not raw[at:].any(), "tagged words must be zero after the build"
    seen = set()
    afters = []
    for start, pos_len, seg, after in tiles.tolist():
        key = (seg, pos_len >> 11)
        assert key in want and key not in seen, key
        seen.add(key)
        assert (start, (pos_len & 2047) + 1, after) == want[key], key
        afters.append(after)
    afters = np.array(afters)
    sorted_part = afters[afters < 32]
    assert np.all(np.diff(sorted_part) >= 0) and np.all(afters[:sorted_part.size] < 32)
    deep_seg, deep_after = tiles[sorted_part.size:, 2], afters[sorted_part.size:]
    for s_ in np.unique(deep_seg):                           # a sequence's deeper tiles: together, innermost first
        idx = np.nonzero(deep_seg == s_)[0]
        assert np.array_equal(idx, np.arange(idx[0], idx[0] + idx.size))
        assert np.array_equal(deep_after[idx], np.arange(32, 32 + idx.size))


# ------------------------------------------------------------------ randomised batches
SPECIAL_WINDOWS = np.array([0, 1, 2, 2047, 2048, 2049, 4096, 4097])


@pytest.mark.parametrize("seed", range(12))
def test_random_batches_all_stages(tp, seed):
    """Random layouts (1..40 sequences, windows of 0..5000 tokens, contexts of 1..50, any
    mix of finished / truncated, any tail_drop, chunk boundaries hit on purpose): select,
    EGAE (dense and terminal rewards), losses and their derivatives against the oracle."""
    rng = np.random.default_rng(1000 + seed)
    B = int(rng.integers(1, 41))
    win = np.where(rng.random(B) < 0.3, rng.choice(SPECIAL_WINDOWS, size=B), rng.integers(0, 5001, size=B))
    all_stages_against_oracle(tp, rng, win, seed)


@pytest.mark.parametrize("B", [2048, 2049, 5000, 17001])
def test_many_sequences_all_stages(tp, B):
    """Thousands of short sequences (empty ones and a few longer than a chunk among them):
    the work lists are then built by several workgroups, each for its own range of sequences."""
    rng = np.random.default_rng(2000 + B)
    win = np.where(rng.random(B) < 0.01, rng.choice(SPECIAL_WINDOWS, size=B), rng.integers(0, 200, size=B))
    all_stages_against_oracle(tp, rng, win, B)


@pytest.mark.parametrize("seed", range(3))
def test_long_runs_of_empty_sequences_all_stages(tp, seed):
    """Sequences that end in mid-frame and are followed by runs of up to 300 empty sequences (more than the plan
    builder skips when it describes a frame, so the loss kernels find the next sequence by themselves), by
    sequences of 1-3 tokens (several boundaries inside one frame) and by the end of the batch."""
    rng = np.random.default_rng(3000 + seed)
    parts = []
    for _ in range(12):
        parts += [rng.integers(1, 3000, size=1), np.zeros(int(rng.choice([1, 63, 64, 65, 100, 300])), np.int64),
                  rng.integers(1, 4, size=int(rng.integers(0, 5)))]
    if seed == 1:
        parts.append(np.zeros(200, np.int64))                # the batch ends with empty sequences
    all_stages_against_oracle(tp, rng, np.concatenate(parts), seed)


@pytest.mark.parametrize("win", [[1024], [1025], [1023, 1], [1, 1023], [4], [5], [3, 1], [2, 1], [2048], [1, 1023, 1024, 1],
                                 [1020, 3, 2, 1, 1022], [0, 1024, 0], [4096, 4], [1, 1, 1, 1, 1, 1, 1, 1, 1017, 3000]])
def test_frame_edges_all_stages(tp, win):
    """Layouts whose sequence ends fall on, just before and just after the ends of the aligned 1024-token frames,
    whose last frame is full, nearly empty or the only one, and batches of 3 and 4 tokens."""
    rng = np.random.default_rng(4000 + sum(win) + len(win))
    all_stages_against_oracle(tp, rng, np.asarray(win, dtype=np.int64), len(win))


def all_stages_against_oracle(tp, rng, win, seed):
    B = win.size
    ctx = rng.integers(1, 51, size=B)
    done = (rng.random(B) < rng.random()).astype(np.int32)
    cu = np.concatenate([[0], np.cumsum(ctx + win)]).astype(np.int32)
    n_tok = int(cu[-1])
    b = dict(cu_seqlens=cu, ctx_len=ctx.astype(np.int32), done=done, n_tok=n_tok,
             input_ids=rng.integers(0, 1000, size=n_tok).astype(np.int32),
             tail_drop=int(rng.choice([0, 1, 7, 1024, 6000])))
    _, sel = check_select(tp, b)
    off, keep, n = sel["resp_off"], sel["keep_len"], sel["N_resp"]
    if n == 0:
        return
    gamma, lam = float(rng.choice([1.0, 0.99])), float(rng.choice([0.0, 0.95, 1.0]))
    rewards = np.where(rng.random(n) < 0.05, rng.normal(size=n), 0.0).astype(np.float32)
    values = rng.uniform(-1, 1, size=n).astype(np.float32)
    boot = rng.uniform(-1, 1, size=B).astype(np.float32) if seed % 2 else None
    adv, ret = check_egae(tp, rewards, values, off, done, gamma, lam, bootstrap=boot)
    terminal = rng.choice([-1.0, 1.0], size=B).astype(np.float32)
    dense = np.zeros(n, np.float32)
    for i in range(B):
        if done[i] and off[i + 1] > off[i]:
            dense[off[i + 1] - 1] = terminal[i]
    ta, tr = tp.tppo_egae_terminal(dev(terminal), dev(values), dev(off), dev(done), gamma, lam)
    ref_a, ref_r = ofast.egae(dense, values, off, done, float(np.float32(gamma)), float(np.float32(lam)))
    assert_egae_close(host(ta), ref_a, "adv")
    assert_egae_close(host(tr), ref_r, "ret")
    a = dict(logp_new=(-np.abs(rng.normal(size=n)) - 0.01).astype(np.float32), adv=adv, ret=ret,
             v_new=(values + rng.normal(0, 0.3, size=n)).astype(np.float32), v_old=values)
    a["logp_old"] = (a["logp_new"] + rng.normal(0, 0.1, size=n)).astype(np.float32)
    bb = dict(resp_off=off, done=done, eps_low=0.2, eps_high=0.28, xi_low=0.5, xi_high=0.6)
    ref = ofast.ppo_losses(a["logp_new"], a["logp_old"], a["adv"], a["v_new"], a["v_old"], a["ret"], off, keep, done,
                           float(np.float32(0.2)), float(np.float32(0.28)), 0.5, float(np.float32(0.6)))
    assert_loss_close(run_losses(tp, a, bb, keep), ref)
    g_lp, g_v, losses, stats = run_loss_grads(tp, a, bb, keep)
    og = ofast.ppo_loss_grads(a["logp_new"], a["logp_old"], a["adv"], a["v_new"], a["v_old"], a["ret"], off, keep, done,
                              float(np.float32(0.2)), float(np.float32(0.28)), 0.5, float(np.float32(0.6)))
    kp, kv = near_kinks(a, bb, keep)
    f = {k: v.astype(np.float64) for k, v in a.items()}
    assert_grads_close(g_lp, og["grad_logp"], kp, -np.exp(f["logp_new"] - f["logp_old"]) * f["adv"] / max(og["n_policy"], 1))
    assert_grads_close(g_v, og["grad_v"], kv, (f["v_new"] - f["ret"]) / max(og["n_value"], 1))
    assert_loss_close(losses, ref)


# ------------------------------------------------------------------ maximum sizes
@pytest.mark.timeout(600)
def test_all_stages_at_the_largest_batch_the_abi_takes(tp):
    """~2^31 window tokens (the ABI's 32-bit token indices end there): a sub-batch of 40 sequences -- two
    of them hundreds of tiles long -- repeated 1800-odd times.  Every copy must reproduce the first one:
    bit for bit where the result is elementwise or an index (shifted by the copy's offset); to the EGAE
    tolerance for advantages and returns, whose tiles are cut at multiples of 1024 of the packed index,
    i.e. at different places in different copies.  The first and last copy are compared with the oracle
    element by element, and the loss sums with the oracle's sums for the sub-batch times the copies."""
    import torch
    rng = np.random.default_rng(4242)
    win = np.concatenate([[700001, 0, 300007], np.exp(rng.uniform(np.log(256), np.log(20480), size=37)).astype(np.int64)])
    Bs = win.size
    done_s = (rng.random(Bs) < 0.4).astype(np.int32)
    done_s[0], done_s[2] = 1, 0                               # one long finished, one long truncated sequence
    ctx_s = rng.integers(1, 4, size=Bs)
    n_sub, n_tok_sub = int(win.sum()), int((win + ctx_s).sum())
    copies = (2**31 - 4096 - 2048) // n_tok_sub
    B, n, n_tok = Bs * copies, n_sub * copies, n_tok_sub * copies
    assert n_tok < 2**31 - 2048 and n > 2**31 - 3 * n_tok_sub
    tail_drop = 1024
    off_s = np.concatenate([[0], np.cumsum(win)]).astype(np.int64)
    cu_s = np.concatenate([[0], np.cumsum(win + ctx_s)]).astype(np.int64)
    keep_s = np.where(done_s != 0, win, np.maximum(win - tail_drop, 0)).astype(np.int32)
    tile_off = lambda o, step: torch.from_numpy(np.concatenate(
        [(o[:-1][None, :] + step * np.arange(copies)[:, None]).ravel(), [step * copies]]).astype(np.int32)).cuda()
    rep = lambda a: dev(a).repeat(copies)
    done, keep = rep(done_s), rep(keep_s)
    resp_off = tile_off(off_s, n_sub)

    def same_in_every_copy(t, width, shift=0):
        """t[c*width + k] == t[k] + c*shift for every copy c, checked on the device in slices"""
        first = t[:width]
        for c0 in range(0, copies, 64):
            c1 = min(c0 + 64, copies)
            block = t[c0 * width:c1 * width].view(c1 - c0, width)
            if shift:
                block = block - (torch.arange(c0, c1, device="cuda", dtype=t.dtype) * shift)[:, None]
            if not torch.equal(block, first.expand(c1 - c0, width)):
                return False
        return True

    def close_in_every_copy(t, width, rtol):
        """|t[c*width + k] - t[k]| <= rtol * max(|t[k]|, 1) for every copy c, checked on the device in slices"""
        first = t[:width]
        tol = rtol * first.abs().clamp(min=1.0)
        for c0 in range(0, copies, 64):
            c1 = min(c0 + 64, copies)
            block = t[c0 * width:c1 * width].view(c1 - c0, width)
            if not bool(((block - first) .abs() <= tol).all()):
                return False
        return True

    # ---- select
    ids_s = rng.integers(0, 50000, size=n_tok_sub).astype(np.int32)
    st = tp.new_status("cuda")
    sel = tp.tppo_select(tile_off(cu_s, n_tok_sub), rep(ctx_s.astype(np.int32)), done, rep(ids_s), tail_drop, status=st)
    osel = ofast.select(cu_s.astype(np.int32), ctx_s.astype(np.int32), done_s, ids_s, tail_drop)
    M_s = osel["M"]
    assert int(host(st)[0]) == 0
    assert host(sel["counts"]).tolist() == [M_s * copies, n, osel["N_val"] * copies]
    assert torch.equal(sel["resp_off"], resp_off) and torch.equal(sel["keep_len"], keep)
    for k, shift in (("sel_rows", n_tok_sub), ("sel_targets", 0), ("sel_resp_idx", n_sub)):
        assert np.array_equal(host(sel[k][:M_s]), osel[k]), k
        assert same_in_every_copy(sel[k][:M_s * copies], M_s, shift), k
    del sel
    torch.cuda.empty_cache()

    # ---- EGAE
    r_s = np.where(rng.random(n_sub) < 0.01, rng.normal(size=n_sub), 0.0).astype(np.float32)
    v_s = rng.uniform(-1, 1, size=n_sub).astype(np.float32)
    gamma, lam = 1.0, 0.95
    values = rep(v_s)
    adv, ret = tp.tppo_egae(rep(r_s), values, resp_off, done, gamma, lam, status=st)
    ref_a, ref_r = ofast.egae(r_s, v_s, off_s.astype(np.int32), done_s, gamma, float(np.float32(lam)))
    assert int(host(st)[0]) == 0
    for c in (0, copies - 1):
        assert_egae_close(host(adv[c * n_sub:(c + 1) * n_sub]), ref_a, "adv")
        assert_egae_close(host(ret[c * n_sub:(c + 1) * n_sub]), ref_r, "ret")
    assert close_in_every_copy(adv, n_sub, 2 * EGAE_RTOL) and close_in_every_copy(ret, n_sub, 2 * EGAE_RTOL)
    del adv, ret
    torch.cuda.empty_cache()

    # ---- losses and their derivatives (advantages and returns: the oracle's, rounded to fp32)
    a_s = dict(logp_new=(-np.abs(rng.normal(size=n_sub)) - 0.01).astype(np.float32), adv=ref_a.astype(np.float32),
               ret=ref_r.astype(np.float32), v_new=(v_s + rng.normal(0, 0.3, size=n_sub)).astype(np.float32), v_old=v_s)
    a_s["logp_old"] = (a_s["logp_new"] + rng.normal(0, 0.1, size=n_sub)).astype(np.float32)
    eps = (float(np.float32(0.2)), float(np.float32(0.28)), 0.5, float(np.float32(0.6)))
    order = ("logp_new", "logp_old", "adv", "v_new", "v_old", "ret")
    ref = ofast.ppo_losses(*(a_s[k] for k in order), off_s.astype(np.int32), keep_s, done_s, *eps)
    og = ofast.ppo_loss_grads(*(a_s[k] for k in order), off_s.astype(np.int32), keep_s, done_s, *eps)
    d = dict(logp_new=rep(a_s["logp_new"]), logp_old=rep(a_s["logp_old"]), adv=rep(a_s["adv"]),
             v_new=rep(a_s["v_new"]), v_old=values, ret=rep(a_s["ret"]))
    got = tp.read_loss_out(tp.tppo_ppo_losses(*(d[k] for k in order), resp_off, keep, done, 0.2, 0.28, 0.5, 0.6, status=st))
    whole = dict(ref, policy_sum=ref["policy_sum"] * copies, value_sum=ref["value_sum"] * copies,
                 n_policy=ref["n_policy"] * copies, n_value=ref["n_value"] * copies)
    assert_loss_close(got, whole)
    g_lp, g_v, res, stats = tp.tppo_ppo_losses_backward(*(d[k] for k in order), resp_off, keep, done, 0.2, 0.28, 0.5, 0.6,
                                                        status=st)
    assert int(host(st)[0]) == 0
    assert_loss_close(tp.read_loss_out(res), whole)
    bb = dict(resp_off=off_s.astype(np.int32), done=done_s, eps_low=0.2, eps_high=0.28, xi_low=0.5, xi_high=0.6)
    kp, kv = near_kinks(a_s, bb, keep_s)
    f = {k: v.astype(np.float64) for k, v in a_s.items()}
    free_p = -np.exp(f["logp_new"] - f["logp_old"]) * f["adv"] / whole["n_policy"]
    free_v = (f["v_new"] - f["ret"]) / whole["n_value"]
    for c in (0, copies - 1):
        assert_grads_close(host(g_lp[c * n_sub:(c + 1) * n_sub]), og["grad_logp"] / copies, kp, free_p)
        assert_grads_close(host(g_v[c * n_sub:(c + 1) * n_sub]), og["grad_v"] / copies, kv, free_v)
    assert same_in_every_copy(g_lp, n_sub) and same_in_every_copy(g_v, n_sub)
    assert tp.read_loss_stats(stats)["n_policy_clipped"] % copies == 0
    del d, g_lp, g_v, values
    torch.cuda.empty_cache()
