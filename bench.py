#!/usr/bin/env python3
"""Benchmark of the SqueezeAttention hot path on one MI355X.

A "step" is one pass of the whole hot path over one synthetic batch that is
already resident in HBM: layer-importance probe -> budgets (host) -> prompt
compression of every layer -> S decode steps over all layers (append, evict,
attend, accumulate).  value = generated tokens per second = B*S*steps / time.

Prints ONE JSON line.  `roofline` is for the dominant kernel (the fused decode
step): algorithmic bytes per launch / mean launch duration, measured with HIP
events on the launch stream, against the 8 TB/s HBM peak.  `cpu_baseline` is
the fp64 numpy oracle timed on this machine's host cores on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0

# HBM bytes per decode launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by what the same
# counters read for a plain 1 GiB copy kernel (x2.0 / x1.0); see profiles/decode_importance_compress__<workload>.txt.
# Counters cannot be read from inside this process, so the figure is the one of the committed profile.
MEASURED_TRAFFIC_BYTES = {("llama2_7b", "squeeze", "h2o", "all_layers"): 820870.1 * 1024 * 2.0 + 19393.0 * 1024}


def cpu_baseline(sess, units_per_layer: int, steps: int):
    """Time the oracle's decode step (Algorithm 1 steps 14-21) on a sample:
    `units_per_layer` (sequence, KV head) units of every layer, `steps` steps."""
    import numpy as np
    import torch
    from oracle import sqa_oracle as O
    try:
        from threadpoolctl import threadpool_limits
    except Exception:  # pragma: no cover
        threadpool_limits = None
    wl = sess.wl
    g = wl.g
    f64 = lambda t: t.detach().cpu().to(torch.float64).numpy()
    units = [(i // wl.Hkv % wl.B, i % wl.Hkv) for i in range(units_per_layer)]
    ctx = threadpool_limits(limits=1) if threadpool_limits else None
    t_total = 0.0
    try:
        for l in range(wl.L):
            b_l = sess.budgets[l]
            for (b, h) in units:
                Kp, Vp = f64(sess.Kp[l][b, h]), f64(sess.Vp[l][b, h])
                # untimed set-up with a stand-in score vector: which prompt tokens
                # are kept does not change what a decode step costs
                s0 = np.linspace(0.0, 1.0, wl.P)
                c = O.prefill_compress(Kp, Vp, s0, b_l, wl.policy, wl.n_sink)
                q = f64(sess.q[:steps, l, b, h * g:(h + 1) * g])
                k = f64(sess.k_new[:steps, l, b, h]); v = f64(sess.v_new[:steps, l, b, h])
                t0 = time.perf_counter()
                for t in range(steps):
                    _, c = O.decode_step(c, q[t], k[t], v[t], wl.P + t, b_l, wl.policy, wl.n_sink)
                t_total += time.perf_counter() - t0
    finally:
        if ctx is not None:
            ctx.__exit__(None, None, None)
    frac = units_per_layer / float(wl.B * wl.Hkv)
    est_step_s = t_total / steps / frac                 # one decode step of the whole batch
    return {"value": wl.B / est_step_s, "unit": "tokens/s", "cores": 1, "kind": "oracle",
            "sample": "%d of %d units of each of %d layers, first %d decode steps, %.1f s of CPU"
                      % (units_per_layer, wl.B * wl.Hkv, wl.L, steps, t_total)}


def scores_only(args, wl):
    """The prompt-score producer alone: per layer one sqa_prefill_scores call (two kernels, row statistics then
    column sums) on generated prompt queries and keys; 2 passes x B*Hq*P(P+1)/2 logits x 2*D flops per layer."""
    import torch
    from paper_2404_04793_amd import binding as sqa
    from paper_2404_04793_amd import workloads as W
    dev = "cuda:0"
    n_gen = min(wl.L, 4)                                  # distinct layers' inputs, cycled
    u_dirs, mask = W.unit_dirs(wl), W.hh_mask(wl, dev)
    QK = [(W.prompt_q(wl, l, dev, u_dirs), W.prompt_kv(wl, l, dev, u_dirs, mask)[0]) for l in range(n_gen)]

    def one_pass():
        for l in range(wl.L):
            sqa.prefill_scores(QK[l % n_gen][0], QK[l % n_gen][1])

    for _ in range(args.warmup):
        one_pass()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(args.steps):
        one_pass()
    e1.record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    call_s = e0.elapsed_time(e1) * 1e-3 / (args.steps * wl.L)
    flops = 2 * wl.B * wl.Hq * (wl.P * (wl.P + 1) // 2) * 2 * wl.D
    peak = 2500.0 if (wl.dtype == "bf16" and wl.D == 128) else 157.3     # matrix cores (bf16, D = 128) or fp32 vector
    out = {
        "metric": "H2O prompt-score producer (causal softmax column sums), TFLOP/s", "value": flops / call_s / 1e12,
        "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": dt / args.steps * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": wl.name, "layers": wl.L, "q_heads": wl.Hq, "kv_heads": wl.Hkv, "head_dim": wl.D,
                   "batch": wl.B, "prompt": wl.P, "phases": "scores_only"},
        "roofline": {"bound": "mfma" if peak == 2500.0 else "alu",
                     "kernel": "score_rowstats + score_colsum (one call = both)", "achieved": flops / call_s / 1e12,
                     "peak": peak, "unit": "TFLOP/s", "frac": flops / call_s / 1e12 / peak, "traffic": None,
                     "flops_per_call": flops, "call_us": call_s * 1e6},
    }
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="llama2_7b")
    ap.add_argument("--per-layer", action="store_true", help="one decode launch per layer instead of one per step")
    ap.add_argument("--graph", action="store_true",
                    help="replay each decode step from a HIP graph recorded once (inputs copied into fixed buffers, "
                         "positions read from a device array); meant for --per-layer, where launches dominate")
    ap.add_argument("--ragged", action="store_true",
                    help="a ragged batch: prompt lengths from P down to about P/2, each sequence probed, budgeted and "
                         "positioned on its own (per-sequence budgets and positions from device arrays)")
    ap.add_argument("--uniform", action="store_true", help="sequence-only baseline: same budget in every layer")
    ap.add_argument("--full-cache", action="store_true", help="no compression (budget = P + S)")
    ap.add_argument("--policy", default=None, choices=["h2o", "streaming", "sliding"],
                    help="override the workload's sequence-wise policy")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timing leg")
    ap.add_argument("--decode-only", action="store_true",
                    help="time only the decode steps (probe, budgets and prompt compression run untimed before "
                         "each pass); for workloads whose whole pass does not fit one GPU's memory")
    ap.add_argument("--probe-tokens", type=int, default=None,
                    help="hidden-state rows per layer given to the probe (default: all B*P)")
    ap.add_argument("--fused-probe", action="store_true",
                    help="run the probe inside the residual add that writes h_out (reads 2, writes 1 tensor)")
    ap.add_argument("--order", default="evict_then_attend", choices=["evict_then_attend", "attend_then_evict"],
                    help="where the policy runs inside a decode step (default: Algorithm 1 as printed)")
    ap.add_argument("--decode-steps", type=int, default=None, help="decode steps per pass (default: the workload's)")
    ap.add_argument("--batch", type=int, default=None, help="override the workload's batch")
    ap.add_argument("--kv-heads", type=int, default=None,
                    help="override the workload's number of KV heads (grouped queries: q_heads / kv_heads per KV head)")
    ap.add_argument("--budget-pct", type=int, default=None, help="override b_init as a percentage of the prompt")
    ap.add_argument("--calib-copy", action="store_true",
                    help="after the timed region run one plain 1 GiB -> 1 GiB elementwise copy kernel "
                         "(reference point for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--scores-only", action="store_true",
                    help="time only the H2O prompt-score producer (sqa_prefill_scores; set-up work of the pass, "
                         "matrix-core bound): a step = the scores of all layers of one prompt batch")
    ap.add_argument("--progress", action="store_true", help="say on stderr when each phase of the run begins")
    ap.add_argument("--cpu-units", type=int, default=32)
    ap.add_argument("--cpu-steps", type=int, default=128)
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2404_04793_amd import workloads as W
    from paper_2404_04793_amd.session import Session

    wl = W.WORKLOADS[args.workload]
    if args.policy:
        wl = W.scaled(wl, policy=args.policy)
    if args.decode_steps:
        wl = W.scaled(wl, S=args.decode_steps)
    if args.batch:
        wl = W.scaled(wl, B=args.batch)
    if args.kv_heads:
        wl = W.scaled(wl, Hkv=args.kv_heads)
    if args.budget_pct:
        wl = W.scaled(wl, budget_pct=args.budget_pct)
    torch.cuda.set_device(0)
    if args.scores_only:
        return scores_only(args, wl)
    plen = [wl.P - (b * wl.P) // (2 * wl.B) for b in range(wl.B)] if args.ragged else None
    def say(what):
        if args.progress:
            print("bench.py: " + what, file=sys.stderr, flush=True)

    say("generating inputs for %s" % wl.name)
    sess = Session(wl, "cuda:0", uniform_budget=args.uniform, full_cache=args.full_cache,
                   probe_tokens=args.probe_tokens, fused_probe=args.fused_probe, order=args.order, prompt_len=plen)
    say("inputs ready")

    def do_decode():
        if args.graph:
            if getattr(sess, "graph", None) is None:
                sess.capture_step_graph(per_layer=args.per_layer)     # during the first (warm-up) pass
            sess.decode_graph()
        else:
            sess.decode(per_layer=args.per_layer)

    def one_pass(ev=None):
        if ev:
            ev[0].record()
        cos = sess.probe_and_allocate()
        if ev:
            ev[1].record()
        sess.compress_prompt()
        if ev:
            ev[2].record()
        do_decode()
        if ev:
            ev[3].record()
        return cos

    if args.decode_only:
        def one_pass(ev=None):                       # noqa: F811
            cos = sess.probe_and_allocate()
            sess.compress_prompt()
            torch.cuda.synchronize()
            t_a = time.perf_counter()
            if ev:
                ev[0].record(); ev[1].record(); ev[2].record()
            do_decode()
            if ev:
                ev[3].record()
            torch.cuda.synchronize()
            one_pass.timed += time.perf_counter() - t_a
            return cos
        one_pass.timed = 0.0

    for i in range(args.warmup):
        say("warm-up pass %d" % (i + 1))
        one_pass()
    torch.cuda.synchronize()
    say("timed passes")
    if args.decode_only:
        one_pass.timed = 0.0
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        cos = one_pass(evs[i])
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    if args.decode_only:
        dt = one_pass.timed

    if args.calib_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        torch.mul(src, 1.0, out=dst)          # reads 2^30 bytes, writes 2^30 bytes
        torch.cuda.synchronize()
        del src, dst

    from paper_2404_04793_amd import binding as sqa
    status = sqa.read_device_status(sess.dec_ws)
    probe_ms = sum(e[0].elapsed_time(e[1]) for e in evs) / args.steps
    comp_ms = sum(e[1].elapsed_time(e[2]) for e in evs) / args.steps
    dec_ms = sum(e[2].elapsed_time(e[3]) for e in evs) / args.steps
    launches = wl.S * (wl.L if args.per_layer else 1)
    bytes_steps = sess.decode_bytes_per_step()
    bytes_launch = sum(bytes_steps) / float(launches)
    launch_s = dec_ms * 1e-3 / launches
    achieved = bytes_launch / launch_s / 1e9
    tokens = wl.B * wl.S * args.steps
    mode = "full_cache" if args.full_cache else ("uniform" if args.uniform else "squeeze")
    launch = ("per_layer" if args.per_layer else "all_layers") + ("_graph" if args.graph else "")
    res = {
        "metric": "decode tokens/s + achieved HBM GB/s (attn+evict), 7B shape, 1 GPU",
        "value": tokens / dt, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": dt * 1e3 / args.steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": wl.name, "layers": wl.L, "q_heads": wl.Hq, "kv_heads": wl.Hkv, "head_dim": wl.D,
                   "batch": wl.B, "prompt": wl.P, "decode_steps": wl.S, "policy": wl.policy,
                   "budget_pct": wl.budget_pct, "p": wl.p,
                   "mode": mode, "launch": launch,
                   "phases": "decode_only" if args.decode_only else "whole_pass",
                   "probe_tokens": sess.probe_tokens, "fused_probe": args.fused_probe, "order": args.order,
                   "ragged_prompt_lengths": plen},
        "roofline": {"bound": "hbm", "kernel": "decode_unit_kernel", "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": MEASURED_TRAFFIC_BYTES.get((wl.name, mode, wl.policy, launch)),
                     "bytes_per_launch": bytes_launch, "launch_us": launch_s * 1e6},
        "phases_ms": {"probe_and_budgets": probe_ms, "prefill_compress": comp_ms, "decode": dec_ms},
        "decode_only_tokens_per_s": wl.B * wl.S / (dec_ms * 1e-3),
        "probe_GBps": None if args.decode_only else sess.probe_bytes() / (probe_ms * 1e-3) / 1e9,
        "compress_GBps": None if args.decode_only else sess.compress_bytes() / (comp_ms * 1e-3) / 1e9,
        "budgets": {"low": min(sess.budgets), "high": max(sess.budgets),
                    "n_G3": None if sess.groups is None else sum(1 for g in sess.groups if g == 2),
                    "sum": sum(sess.budgets)},
        "resident_kv_GB": sess.resident_kv_bytes() / 1e9,
        "device_status": status,
    }
    if not args.no_cpu:
        res["cpu_baseline"] = cpu_baseline(sess, args.cpu_units, min(args.cpu_steps, wl.S))
    print(json.dumps(res))


if __name__ == "__main__":
    main()
