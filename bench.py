#!/usr/bin/env python3
"""Benchmark of the T-PPO per-token core on one MI355X.

One "step" = one pass of the whole hot path over one synthetic batch resident
in HBM: tppo_select -> tppo_token_logprobs -> tppo_egae -> tppo_ppo_losses.
Metric: selected (kept) tokens per second.  Default workload: the 32B-shaped
head (32 sequences, prompt 1024 + window 8192, hidden 5120, vocabulary 152064,
bf16, token ids sampled from the policy).

Prints ONE JSON line with the whole-path throughput, the roofline position of
the dominant kernel (the fused LM-head MFMA kernel, timed with HIP events on
the launch stream inside the timed region), the roofline positions of the
HBM-bound kernels (EGAE scan, losses, loss derivatives) on long-CoT-sized
arrays that no cache holds, and the CPU oracle timed on a bounded sample of
the same batch on this machine's host cores.  The oracle's sample doubles as a
check: its log-probs are compared with those of the last timed step, and the
run fails if they differ by more than 2e-3.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0     # MI355X dense bf16 matrix peak
HBM_PEAK_GBS = 8000.0
PARITY_TOLERANCE = 2e-3            # |log-prob (timed run) - log-prob (oracle)| on the oracle's sample
STREAMING_WORKLOAD = "longcot20x"  # 40 M response tokens in 8704 sequences: 160 MB per array


def measured_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` on `workload`, from the committed
    rocprofv3 --pmc summary (FETCH_SIZE + WRITE_SIZE, calibrated on a copy
    kernel); None when no such summary exists."""
    path = os.path.join(ROOT, "profiles", f"{kernel}_{workload}_pmc.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="head32b",
                    choices=["small", "head7b", "head32b", "longcot", "longcot5x", "longcot20x"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-rows", type=int, default=4096)
    ap.add_argument("--metric-only", action="store_true",
                    help="skip everything outside the metric's four steps (measured ceilings, backward passes)")
    ap.add_argument("--no-streaming-rooflines", action="store_true",
                    help="skip the HBM-bound kernels' roofline entries on long-CoT-sized arrays")
    ap.add_argument("--no-reference-rates", action="store_true",
                    help="skip the two measuring sticks printed beside the datasheet peak")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MiB",
                    help="only run a plain device copy of this many MiB (reference for the "
                         "FETCH_SIZE / WRITE_SIZE counters) and exit")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2506_15050_amd import binding as tp, synth

    torch.cuda.set_device(0)
    if args.calibrate_copy:
        nbytes = args.calibrate_copy << 20
        src = torch.ones(nbytes // 4, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes_read": nbytes, "calibrate_copy_bytes_written": nbytes,
                          "launches": 5}))
        return
    tp.load()
    name = args.workload
    has_head = synth.CONFIGS[name]["V"] > 0
    t0 = time.time()
    b = synth.make_batch(name)

    def dev(a):
        t = torch.from_numpy(np.ascontiguousarray(a))
        if a.dtype == np.uint16:
            t = t.view(torch.int16).view(torch.bfloat16)
        return t.cuda()

    if has_head and b["cfg"].get("ids_from_policy"):
        synth.sample_ids_from_policy(b, device="cuda")
    d = {k: dev(b[k]) for k in ("cu_seqlens", "ctx_len", "done", "rewards", "values", "v_new")}
    ids = dev(b["input_ids"]) if has_head else None
    hidden = dev(b["hidden"]) if has_head else None
    w_head = dev(b["w_head"]) if has_head else None
    n_resp, n_tok = b["n_resp"], b["n_tok"]
    print(f"[bench] inputs for '{name}' ready in {time.time() - t0:.1f}s "
          f"(n_tok={n_tok}, n_resp={n_resp})", file=sys.stderr, flush=True)

    # --- set-up pass: the caller learns M once (it is fixed by the batch), and
    # the old policy's log-probs are the new ones plus the seeded gap
    sel = tp.tppo_select(d["cu_seqlens"], d["ctx_len"], d["done"], ids, b["tail_drop"], n_tok=n_tok)
    M = int(sel["counts"][0].item())
    if has_head:
        logp0, _ = tp.tppo_token_logprobs(hidden, w_head, sel["sel_rows"], sel["sel_targets"], M=M,
                                          out_index=sel["sel_resp_idx"], out_size=n_resp, want_lse=False)
        logp0 = torch.where(torch.isfinite(logp0), logp0, torch.zeros_like(logp0))
    else:
        logp0 = dev(b["logp_new_synth"])
    logp_old = logp0 + dev(b["logp_gap"])
    status = tp.new_status("cuda")
    lib = tp.load()
    H, V = b["H"], b["V"]
    ws_head = tp._workspace(lib.tppo_token_logprobs_workspace_bytes(M, H, V, tp.TPPO_BF16), "cuda") if has_head else None
    adv_ret = (torch.empty(n_resp, device="cuda"), torch.empty(n_resp, device="cuda"))
    loss_out = torch.empty(32, dtype=torch.uint8, device="cuda")

    ev = lambda: torch.cuda.Event(enable_timing=True)
    stage_names = ("select", "logprobs", "egae", "losses")
    marks = []
    last = {}

    def step(record):
        e = [ev() for _ in range(5)] if record else None
        if record:
            e[0].record()
        s = tp.tppo_select(d["cu_seqlens"], d["ctx_len"], d["done"], ids, b["tail_drop"], n_tok=n_tok,
                           status=status, want_plan=True)       # the work plan is built once, here
        if record:
            e[1].record()
        if has_head:
            logp, _ = tp.tppo_token_logprobs(hidden, w_head, s["sel_rows"], s["sel_targets"], M=M,
                                             out_index=s["sel_resp_idx"], out_size=n_resp,
                                             want_lse=False, status=status, workspace=ws_head)
        else:
            logp = logp0
        if record:
            e[2].record()
        adv, ret = tp.tppo_egae(d["rewards"], d["values"], s["resp_off"], d["done"], b["gamma"], b["lam"],
                                status=status, plan=s["plan"], out=adv_ret)
        if record:
            e[3].record()
        tp.tppo_ppo_losses(logp, logp_old, adv, d["v_new"], d["values"], ret, s["resp_off"],
                           s["keep_len"], d["done"], b["eps_low"], b["eps_high"], b["xi_low"],
                           b["xi_high"], status=status, plan=s["plan"], out=loss_out)
        if record:
            e[4].record()
            marks.append(e)
        last["logp"], last["sel"] = logp, s

    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for _ in range(args.steps):
        step(True)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    assert int(status.item()) == 0, f"device status {int(status.item())}"
    losses = tp.read_loss_out(loss_out)

    stage_ms = {n: float(np.mean([m[i].elapsed_time(m[i + 1]) for m in marks]))
                for i, n in enumerate(stage_names)}
    ms_per_step = elapsed / args.steps * 1e3
    value = M * args.steps / elapsed

    if has_head:
        flops = 2.0 * M * V * H
        achieved = flops / (stage_ms["logprobs"] * 1e-3) / 1e12
        roofline = dict(bound="mfma", kernel="head_mfma_kernel", achieved=achieved,
                        peak=MFMA_BF16_PEAK_TFLOPS, unit="TFLOP/s",
                        frac=achieved / MFMA_BF16_PEAK_TFLOPS,
                        traffic=measured_traffic(name, "head_mfma_kernel"),
                        flops_per_launch=flops, avg_ms=stage_ms["logprobs"])
    else:
        nbytes = 16.0 * n_resp
        achieved = nbytes / (stage_ms["egae"] * 1e-3) / 1e9
        roofline = dict(bound="hbm", kernel="egae_scan_kernel", achieved=achieved, peak=HBM_PEAK_GBS,
                        unit="GB/s", frac=achieved / HBM_PEAK_GBS,
                        traffic=measured_traffic(name, "egae_scan_kernel"),
                        bytes_per_launch=nbytes, avg_ms=stage_ms["egae"])

    if not has_head and not (args.no_reference_rates or args.metric_only):
        # what the memory system sustains for as many concurrent streams as each kernel has, on arrays of the
        # same length, cold (each launch walks its own part of a 2 GB pool: nothing comes from the 256 MB cache)
        per_stream = (4 * n_resp + 4095) // 4096 * 4096
        pool_r = torch.zeros(6 * 2 * per_stream // 4 + 1024, device="cuda")
        pool_w = torch.empty(2 * 2 * per_stream // 4 + 1024, device="cuda")
        skip_r, skip_w = (-pool_r.data_ptr()) % 4096 // 4, (-pool_w.data_ptr()) % 4096 // 4

        def rate(n_read, n_write):
            run = lambda half: tp.tppo_diag_streams(pool_r[skip_r + half * 6 * per_stream // 4:],
                                                    pool_w[skip_w + half * 2 * per_stream // 4:],
                                                    per_stream, per_stream, n_read, n_write)
            run(0); run(1)
            torch.cuda.synchronize()
            e0, e1 = ev(), ev()
            e0.record()
            total = sum(run(i & 1) for i in range(8))
            e1.record()
            torch.cuda.synchronize()
            return total / (e0.elapsed_time(e1) * 1e-3) / 1e9
        roofline["measured_ceilings"] = {
            "elementwise_2_read_2_write_streams_GBps (EGAE)": rate(2, 2),
            "elementwise_6_read_streams_GBps (losses)": rate(6, 0),
            "elementwise_6_read_2_write_streams_GBps (loss derivatives)": rate(6, 2)}
        del pool_r, pool_w
    if has_head and not (args.no_reference_rates or args.metric_only):
        roofline["measured_ceilings"] = reference_rates(tp, hidden, w_head, s_rows=sel["sel_rows"][:M])

    extra = None
    if not args.metric_only:
        # --- beyond the metric's four steps: the loss derivatives (one more streaming pass), timed on their own
        grads = (torch.empty(n_resp, device="cuda"), torch.empty(n_resp, device="cuda"))
        stats_out = torch.empty(32, dtype=torch.uint8, device="cuda")
        s_last = tp.tppo_select(d["cu_seqlens"], d["ctx_len"], d["done"], ids, b["tail_drop"], n_tok=n_tok,
                                want_plan=True)
        logp_last = logp0
        adv_last, ret_last = adv_ret

        def backward_pass():
            tp.tppo_ppo_losses_backward(logp_last, logp_old, adv_last, d["v_new"], d["values"], ret_last,
                                        s_last["resp_off"], s_last["keep_len"], d["done"], b["eps_low"],
                                        b["eps_high"], b["xi_low"], b["xi_high"], status=status,
                                        plan=s_last["plan"], out=loss_out, stats=stats_out, grads=grads)

        backward_pass()
        torch.cuda.synchronize()
        e0, e1 = ev(), ev()
        e0.record()
        for _ in range(args.steps):
            backward_pass()
        e1.record()
        torch.cuda.synchronize()
        bwd_ms = e0.elapsed_time(e1) / args.steps
        bwd_bytes = 16.0 * (losses["n_policy"] + losses["n_value"]) + 4.0 * (2 * n_resp - losses["n_policy"] - losses["n_value"])
        extra = {"ppo_losses_backward": {"ms": bwd_ms, "algorithmic_bytes": bwd_bytes,
                                         "GB/s": bwd_bytes / (bwd_ms * 1e-3) / 1e9,
                                         "clip_stats": tp.read_loss_stats(stats_out)}}

        # Extended GAE from one terminal reward per sequence (12 instead of 16 bytes per token)
        terminal = torch.ones(b["B"], dtype=torch.float32, device="cuda")
        run_t = lambda: tp.tppo_egae_terminal(terminal, d["values"], s_last["resp_off"], d["done"], b["gamma"],
                                              b["lam"], status=status, plan=s_last["plan"], out=adv_ret)
        run_t()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(args.steps):
            run_t()
        e1.record()
        torch.cuda.synchronize()
        t_ms = e0.elapsed_time(e1) / args.steps
        extra["egae_terminal"] = {"ms": t_ms, "algorithmic_bytes": 12.0 * n_resp,
                                  "GB/s": 12.0 * n_resp / (t_ms * 1e-3) / 1e9}
        if has_head:
            # value-head projection on the value tokens' rows (window tokens of finished sequences)
            fin = torch.repeat_interleave(d["done"] != 0, (sel["sel_off"][1:] - sel["sel_off"][:-1]).long())
            v_rows = sel["sel_rows"][:M][fin].contiguous()
            w_value = (torch.randn(H, device="cuda") / H ** 0.5).to(torch.bfloat16)
            v_out = torch.empty(v_rows.numel(), dtype=torch.float32, device="cuda")
            run_v = lambda: tp.tppo_value_head(hidden, w_value, 0.0, v_rows, out=v_out, status=status)
            run_v()
            torch.cuda.synchronize()
            e0.record()
            for _ in range(args.steps):
                run_v()
            e1.record()
            torch.cuda.synchronize()
            v_ms = e0.elapsed_time(e1) / args.steps
            v_bytes = 2.0 * H * v_rows.numel()
            extra["value_head"] = {"ms": v_ms, "rows": int(v_rows.numel()), "algorithmic_bytes": v_bytes,
                                   "GB/s": v_bytes / (v_ms * 1e-3) / 1e9}
            # derivatives of the log-probs with respect to hidden rows and head matrix (three sweeps of the same size)
            _, lse0 = tp.tppo_token_logprobs(hidden, w_head, sel["sel_rows"], sel["sel_targets"], M=M)
            g_tok = grads[0][sel["sel_resp_idx"][:M].long()].contiguous()
            ws_hb = tp._workspace(lib.tppo_token_logprobs_backward_workspace_bytes(M, H, V, tp.TPPO_BF16), "cuda")
            grad_w = torch.empty(V, H, dtype=torch.float32, device="cuda")
            run_hb = lambda: tp.tppo_token_logprobs_backward(hidden, w_head, sel["sel_rows"], sel["sel_targets"],
                                                             lse0, g_tok, M=M, grad_w=grad_w, workspace=ws_hb)
            run_hb()
            torch.cuda.synchronize()
            e0.record()
            for _ in range(2):
                run_hb()
            e1.record()
            torch.cuda.synchronize()
            hb_ms = e0.elapsed_time(e1) / 2
            extra["token_logprobs_backward"] = {"ms": hb_ms, "flop": 6.0 * M * V * H,
                                                "TFLOP/s": 6.0 * M * V * H / (hb_ms * 1e-3) / 1e12}
            del ws_hb, grad_w

    streaming = None
    if not (args.metric_only or args.no_streaming_rooflines):
        streaming = streaming_rooflines(tp, synth, args.steps)

    cpu, parity_ok = None, True
    if not args.no_cpu_baseline:
        gpu_logp = last["logp"].float().cpu().numpy() if has_head else None
        gpu_idx = last["sel"]["sel_resp_idx"][:M].cpu().numpy() if has_head else None
        cpu = cpu_baseline(b, M, args.cpu_sample_rows, has_head, gpu_logp, gpu_idx)
        parity_ok = cpu.get("parity_max_abs_err") is None or cpu["parity_max_abs_err"] <= PARITY_TOLERANCE

    out = {
        "metric": "selected tokens/sec (logprob+EGAE+loss) at 1 MI355X",
        "value": value, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if has_head else "f32", "data": "synthetic",
        "config": {"workload": name, "sequences": b["B"], "n_tok": n_tok, "n_resp": n_resp,
                   "kept_tokens_M": M, "hidden": H, "vocab": V, "tail_drop": b["tail_drop"],
                   "gamma": b["gamma"], "lambda": b["lam"]},
        "stages_ms": stage_ms,
        "losses": {k: losses[k] for k in ("policy_loss", "value_loss", "n_policy", "n_value")},
        "roofline": roofline, "roofline_streaming": streaming, "cpu_baseline": cpu,
        "beyond_the_metric": extra,
    }
    print(json.dumps(out))
    if not parity_ok:
        print(f"bench.py: the timed run's log-probs differ from the oracle's by {cpu['parity_max_abs_err']:.3g} "
              f"(> {PARITY_TOLERANCE}) on the oracle's sample", file=sys.stderr)
        sys.exit(1)


def reference_rates(tp, hidden, w_head, s_rows):
    """Two measured ceilings for the matrix-core roofline, taken after the timed
    region on the same GPU: the library's own MFMA loop on register-resident
    operands (what the chip sustains under its power limit), and the vendor
    GEMM (torch.matmul) on the same M x V x H problem, which writes the logits
    out and computes no softmax."""
    import torch
    ops = (torch.randn(6144, device="cuda") * 0.5).to(torch.bfloat16)
    out = torch.empty(131072, dtype=torch.float32, device="cuda")
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    tp.tppo_diag_mfma_rate(ops, out, 2000)
    torch.cuda.synchronize()
    e0.record()
    flop = tp.tppo_diag_mfma_rate(ops, out, 100000)
    e1.record()
    torch.cuda.synchronize()
    mfma_only = flop / (e0.elapsed_time(e1) * 1e-3) / 1e12
    rows = hidden[s_rows.long()]
    logits = torch.empty(rows.shape[0], w_head.shape[0], dtype=torch.bfloat16, device="cuda")
    torch.matmul(rows, w_head.t(), out=logits)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(2):
        torch.matmul(rows, w_head.t(), out=logits)
    e1.record()
    torch.cuda.synchronize()
    gemm = 2 * 2.0 * rows.shape[0] * w_head.shape[0] * w_head.shape[1] / (e0.elapsed_time(e1) * 1e-3) / 1e12
    return {"mfma_loop_in_registers_tflops": mfma_only, "library_gemm_logits_to_hbm_tflops": gemm}


def streaming_rooflines(tp, synth, steps):
    """Roofline entries of the HBM-bound kernels: tppo_egae, tppo_ppo_losses and
    tppo_ppo_losses_backward on arrays of the long-CoT batch (40 M response
    tokens, 160 MB per array), each launch on another of three array sets so that
    nothing is served from the 256 MB cache, with the plan built once (as in the
    whole path, where tppo_select builds it).  A kernel's launches are queued back
    to back between one pair of HIP events on the launch stream and the time is
    divided by their number -- the way the elementwise pass beside them is timed,
    and what the kernel trace's durations are compared with (an event pair around
    every single launch adds 3-5 us of command processing to each)."""
    import torch
    name = STREAMING_WORKLOAD
    cfg = dict(synth.CONFIGS[name])
    meta = synth._rng(cfg["seed"], "meta")
    done = (meta.random(cfg["B"]) < cfg["p_done"]).astype(np.int32)
    win = synth._draw_lengths(meta, cfg, done)
    off = np.concatenate([[0], np.cumsum(win)]).astype(np.int32)
    n, B = int(off[-1]), cfg["B"]
    keep = np.where(done != 0, win, np.maximum(win - cfg["tail_drop"], 0)).astype(np.int32)
    n_pol, n_val = int(np.minimum(keep, win).sum()), int(win[done != 0].sum())
    d_off, d_done, d_keep = (torch.from_numpy(x).cuda() for x in (off, done, keep))
    sets = []
    for k in range(3):
        g = torch.Generator(device="cuda").manual_seed(1000 + k)
        mk = lambda: torch.rand(n, device="cuda", generator=g) * 2 - 1
        a = dict(r=mk() * 0.1, v=mk(), adv=torch.empty(n, device="cuda"), ret=torch.empty(n, device="cuda"),
                 ln=-mk().abs() - 0.01, vn=mk(), glp=torch.empty(n, device="cuda"), gv=torch.empty(n, device="cuda"))
        a["lo"] = a["ln"] + 0.1 * mk()
        sets.append(a)
    plan = tp.tppo_plan_build(d_off, d_keep, d_done, n)
    st = tp.new_status("cuda")
    out = torch.empty(32, dtype=torch.uint8, device="cuda")
    stats = torch.empty(32, dtype=torch.uint8, device="cuda")
    eps = (cfg["eps"][0], cfg["eps"][1], synth.XI[0], synth.XI[1])

    def egae(a):
        tp.tppo_egae(a["r"], a["v"], d_off, d_done, synth.GAMMA, synth.LAMBDA, status=st, plan=plan,
                     out=(a["adv"], a["ret"]))

    def losses(a):
        tp.tppo_ppo_losses(a["ln"], a["lo"], a["adv"], a["vn"], a["v"], a["ret"], d_off, d_keep, d_done, *eps,
                           status=st, plan=plan, out=out)

    def grads(a):
        tp.tppo_ppo_losses_backward(a["ln"], a["lo"], a["adv"], a["vn"], a["v"], a["ret"], d_off, d_keep, d_done,
                                    *eps, status=st, plan=plan, out=out, stats=stats, grads=(a["glp"], a["gv"]))

    for a in sets:
        egae(a)
    torch.cuda.synchronize()
    # the elementwise pass beside each kernel: same number of streams, same bytes per stream, streams 4 KiB-aligned
    # (as the kernels' full tiles are; misaligned streams cost such a pass ~15 %)
    per_stream = (4 * n + 4095) // 4096 * 4096
    pool_r = torch.zeros(3 * 6 * per_stream // 4 + 1024, device="cuda")
    pool_w = torch.empty(3 * 2 * per_stream // 4 + 1024, device="cuda")
    skip_r, skip_w = (-pool_r.data_ptr()) % 4096 // 4, (-pool_w.data_ptr()) % 4096 // 4

    def timed(fn, reps):
        for a in sets:
            fn(a)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(reps):
            fn(sets[i % 3])
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / reps

    def ceiling(n_read, n_write):
        run = lambda k: tp.tppo_diag_streams(pool_r[skip_r + k * 6 * per_stream // 4:],
                                             pool_w[skip_w + k * 2 * per_stream // 4:],
                                             per_stream, per_stream, n_read, n_write)
        for k in range(3):
            run(k)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        total = sum(run(i % 3) for i in range(9))
        e1.record()
        torch.cuda.synchronize()
        return total / (e0.elapsed_time(e1) * 1e-3) / 1e9

    reps = max(6, 2 * steps)
    entries = []
    for kernel, fn, nbytes, mix in (
            ("egae_scan_kernel", egae, 16.0 * n, (2, 2)),
            ("loss_kernel", losses, 12.0 * (n_pol + n_val), (6, 0)),
            ("loss_grad_kernel", grads, 16.0 * (n_pol + n_val) + 4.0 * (2 * n - n_pol - n_val), (6, 2))):
        sec = timed(fn, reps)
        top = ceiling(*mix)
        achieved = nbytes / sec / 1e9
        entries.append(dict(bound="hbm", kernel=kernel, workload=name, achieved=achieved, peak=HBM_PEAK_GBS,
                            unit="GB/s", frac=achieved / HBM_PEAK_GBS, traffic=measured_traffic(name, kernel),
                            bytes_per_launch=nbytes, avg_us=sec * 1e6, launches=reps, cold=True,
                            elementwise_pass_same_streams_GBps=top, frac_of_elementwise_pass=achieved / top))
    assert int(st.item()) == 0, f"device status {int(st.item())} in the streaming kernels"
    return entries


def cpu_baseline(b, M, sample_rows, has_head, gpu_logp=None, gpu_resp_idx=None):
    """The CPU oracle, as it stands, on a bounded sample of the same batch:
    the LM head on `sample_rows` seeded kept rows, the other stages on the full
    batch; per-token costs are added.  With the timed run's log-probs
    (response-packed) and the kept tokens' response-packed indices, the sample
    is also a check: the largest difference is reported."""
    from oracle import fast as ofast
    t = time.perf_counter()
    ids = b["input_ids"] if has_head else np.zeros(b["n_tok"], np.int32)
    sel = ofast.select(b["cu_seqlens"], b["ctx_len"], b["done"], ids, b["tail_drop"])
    t_sel = time.perf_counter() - t
    t_head, n_head = 0.0, 0
    if has_head:
        pick = np.sort(np.random.default_rng(0).choice(M, size=min(sample_rows, M), replace=False))
        t = time.perf_counter()
        olp, _ = ofast.token_logprobs(b["hidden"], b["w_head"], sel["sel_rows"][pick], sel["sel_targets"][pick])
        t_head, n_head = time.perf_counter() - t, len(pick)
        logp_new = np.zeros(b["n_resp"], np.float32)
    else:
        logp_new = b["logp_new_synth"]
    t = time.perf_counter()
    adv, ret = ofast.egae(b["rewards"], b["values"], sel["resp_off"], b["done"], b["gamma"], b["lam"])
    t_egae = time.perf_counter() - t
    t = time.perf_counter()
    ofast.ppo_losses(logp_new, logp_new + b["logp_gap"], adv, b["v_new"], b["values"], ret,
                     sel["resp_off"], sel["keep_len"], b["done"], b["eps_low"], b["eps_high"],
                     b["xi_low"], b["xi_high"])
    t_loss = time.perf_counter() - t
    per_token = (t_sel + t_egae + t_loss) / max(M, 1) + (t_head / n_head if n_head else 0.0)
    err = None
    if has_head and gpu_logp is not None:
        assert np.array_equal(gpu_resp_idx[pick], sel["sel_resp_idx"][pick]), "kept-token indices differ from the oracle's"
        err = float(np.max(np.abs(gpu_logp[gpu_resp_idx[pick]].astype(np.float64) - olp.astype(np.float64))))
    return dict(value=1.0 / per_token, unit="tokens/s", cores=len(os.sched_getaffinity(0)),
                kind="oracle", parity_max_abs_err=err, parity_rows=n_head, parity_tolerance=PARITY_TOLERANCE,
                sample=(f"LM head on {n_head} seeded kept rows of {M} ({t_head:.1f}s); select, EGAE and "
                        f"losses on the full batch ({t_sel + t_egae + t_loss:.1f}s); per-token costs added"))


if __name__ == "__main__":
    main()
