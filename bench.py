#!/usr/bin/env python3
"""Benchmark of the T-PPO per-token core on one MI355X.

One "step" = one pass of the whole hot path over one synthetic batch resident
in HBM: tppo_select -> tppo_token_logprobs -> tppo_egae -> tppo_ppo_losses.
Metric: selected (kept) tokens per second.  Default workload: the 32B-shaped
head (32 sequences, prompt 1024 + window 8192, hidden 5120, vocabulary 152064,
bf16, token ids sampled from the policy).

Prints ONE JSON line with the whole-path throughput, the roofline position of
the dominant kernel (the fused LM-head MFMA kernel, timed with HIP events on
the launch stream inside the timed region) and the CPU oracle timed on a
bounded sample of the same batch on this machine's host cores.
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
    ws_egae = tp._workspace(lib.tppo_egae_workspace_bytes(n_resp, b["B"]), "cuda")
    ws_loss = tp._workspace(lib.tppo_ppo_losses_workspace_bytes(n_resp, b["B"]), "cuda")
    adv_ret = (torch.empty(n_resp, device="cuda"), torch.empty(n_resp, device="cuda"))
    loss_out = torch.empty(32, dtype=torch.uint8, device="cuda")

    ev = lambda: torch.cuda.Event(enable_timing=True)
    stage_names = ("select", "logprobs", "egae", "losses")
    marks = []

    def step(record):
        e = [ev() for _ in range(5)] if record else None
        if record:
            e[0].record()
        s = tp.tppo_select(d["cu_seqlens"], d["ctx_len"], d["done"], ids, b["tail_drop"], n_tok=n_tok,
                           status=status)
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
                                status=status, workspace=ws_egae, out=adv_ret)
        if record:
            e[3].record()
        tp.tppo_ppo_losses(logp, logp_old, adv, d["v_new"], d["values"], ret, s["resp_off"],
                           s["keep_len"], d["done"], b["eps_low"], b["eps_high"], b["xi_low"],
                           b["xi_high"], status=status, workspace=ws_loss, out=loss_out)
        if record:
            e[4].record()
            marks.append(e)

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
        per_stream = (4 * n_resp + 15) // 16 * 16
        pool_r = torch.zeros(6 * 2 * per_stream // 4 + 64, device="cuda")
        pool_w = torch.empty(2 * 2 * per_stream // 4 + 64, device="cuda")

        def rate(n_read, n_write):
            run = lambda half: tp.tppo_diag_streams(pool_r[half * 6 * per_stream // 4:], pool_w[half * 2 * per_stream // 4:],
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
        ws_bwd = tp._workspace(lib.tppo_ppo_losses_backward_workspace_bytes(n_resp, b["B"]), "cuda")
        grads = (torch.empty(n_resp, device="cuda"), torch.empty(n_resp, device="cuda"))
        stats_out = torch.empty(32, dtype=torch.uint8, device="cuda")
        s_last = tp.tppo_select(d["cu_seqlens"], d["ctx_len"], d["done"], ids, b["tail_drop"], n_tok=n_tok)
        logp_last = logp0
        adv_last, ret_last = adv_ret

        def backward_pass():
            tp.tppo_ppo_losses_backward(logp_last, logp_old, adv_last, d["v_new"], d["values"], ret_last,
                                        s_last["resp_off"], s_last["keep_len"], d["done"], b["eps_low"],
                                        b["eps_high"], b["xi_low"], b["xi_high"], status=status,
                                        workspace=ws_bwd, out=loss_out, stats=stats_out, grads=grads)

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
                                              b["lam"], status=status, workspace=ws_egae, out=adv_ret)
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

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(b, M, args.cpu_sample_rows, has_head)

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
        "roofline": roofline, "cpu_baseline": cpu, "beyond_the_metric": extra,
    }
    print(json.dumps(out))


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


def cpu_baseline(b, M, sample_rows, has_head):
    """The CPU oracle, as it stands, on a bounded sample of the same batch:
    the LM head on `sample_rows` seeded kept rows, the other stages on the full
    batch; per-token costs are added."""
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
    return dict(value=1.0 / per_token, unit="tokens/s", cores=len(os.sched_getaffinity(0)),
                kind="oracle",
                sample=(f"LM head on {n_head} seeded kept rows of {M} ({t_head:.1f}s); select, EGAE and "
                        f"losses on the full batch ({t_sel + t_egae + t_loss:.1f}s); per-token costs added"))


if __name__ == "__main__":
    main()
