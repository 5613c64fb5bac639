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

# HBM bytes per decode launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by what the same counters
# read for a plain 1 GiB copy kernel (x2.0 / x1.0).  Counters cannot be read from inside this process, so the
# figure is the one of the committed profile named beside it, and it is only reported while the decode
# kernel's source is byte for byte the one that profile was taken with (sha256 prefix below); otherwise
# `traffic` is null and `traffic_source` says that the profile is out of date.
MEASURED_TRAFFIC = {
    ("llama2_7b", "squeeze", "h2o", "all_layers", "dense"): {
        "bytes": 820874.5 * 1024 * 2.0 + 19390.9 * 1024,
        "source": "profiles/decode_importance_compress__llama2_7b.txt", "kernel_sha": "a6972dc5cfdd1b7e"},
    ("llama2_7b", "squeeze", "h2o", "all_layers", "blocked"): {
        "bytes": 821453.8 * 1024 * 2.0 + 19391.0 * 1024,
        "source": "profiles/decode_importance_compress__llama2_7b.txt", "kernel_sha": "a6972dc5cfdd1b7e"},
}


def decode_kernel_sha() -> str:
    import hashlib
    h = hashlib.sha256()
    for f in ("sqa_decode.hip", "sqa_common.h"):
        with open(os.path.join(ROOT, "paper_2404_04793_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def measured_traffic(key):
    m = MEASURED_TRAFFIC.get(key)
    if m is None:
        return None, None
    if m["kernel_sha"] != decode_kernel_sha():
        return None, m["source"] + " (taken with another version of the decode kernel: not reported)"
    return m["bytes"], m["source"]


# ---- the oracle on the host cores -------------------------------------------------------
def _oracle_worker_init():
    try:
        from threadpoolctl import threadpool_limits
        _oracle_worker_init.ctx = threadpool_limits(limits=1)      # one core per worker process
    except Exception:  # pragma: no cover
        pass


def _oracle_unit_task(task):
    """One (layer, sequence, KV head) unit: `steps` oracle decode steps from its compressed cache."""
    import numpy as np
    from oracle import sqa_oracle as O
    c, q, k, v, pos0, b_l, policy, n_sink = task
    c = {key: np.asarray(val, dtype=np.float64) if key != "pos" else val for key, val in c.items()}
    q, k, v = q.astype(np.float64), k.astype(np.float64), v.astype(np.float64)
    t0 = time.perf_counter()
    for t in range(q.shape[0]):
        _, c = O.decode_step(c, q[t], k[t], v[t], pos0 + t, b_l, policy, n_sink)
    return os.getpid(), time.perf_counter() - t0


def _oracle_worker_ready(_):
    _oracle_worker_init()
    time.sleep(0.3)
    return os.getpid()


def oracle_pool():
    """Worker processes for the oracle leg, one per host core of this box's share (at most 16).  Started
    before this process touches the GPU: a process that has initialised the GPU starts no new programs.
    (An executor, not multiprocessing.Pool: if a worker dies the leg fails instead of respawning for ever.)"""
    import multiprocessing as mp
    from concurrent.futures import ProcessPoolExecutor
    nproc = os.cpu_count() or 1
    cores = max(1, min(16, nproc))
    ex = ProcessPoolExecutor(cores, mp_context=mp.get_context("spawn"))
    pids = set(ex.map(_oracle_worker_ready, range(cores), timeout=120))      # every worker is up now
    return ex, len(pids), nproc


def cpu_baseline(sess, units_per_layer: int, steps: int, pool, cores: int, nproc: int):
    """Time the oracle's decode step (Algorithm 1 steps 14-21) on a bounded sample -- `units_per_layer`
    (sequence, KV head) units of every layer, `steps` steps -- spread over the worker processes of
    oracle_pool(), CPU only.  The rate is the sample's work over the busiest worker's time (set-up and
    moving the inputs to the workers are not timed)."""
    import numpy as np
    import torch
    from oracle import sqa_oracle as O
    wl = sess.wl
    g = wl.g
    f32 = lambda t: t.detach().cpu().to(torch.float32).numpy()      # (bf16 and fp32 values are exact in fp32)
    units = [(i // wl.Hkv % wl.B, i % wl.Hkv) for i in range(units_per_layer)]
    tasks = []
    for l in range(wl.L):
        b_l = sess.budgets[l]
        Kl, Vl = f32(sess.Kp[l]), f32(sess.Vp[l])
        ql, kl, vl = f32(sess.q[:steps, l]), f32(sess.k_new[:steps, l]), f32(sess.v_new[:steps, l])
        for (b, h) in units:
            # untimed set-up with a stand-in score vector: which prompt tokens are kept does not change
            # what a decode step costs
            c = O.prefill_compress(Kl[b, h], Vl[b, h], np.linspace(0.0, 1.0, wl.P), b_l, wl.policy, wl.n_sink)
            c = {"K": c["K"].astype(np.float32), "V": c["V"].astype(np.float32), "pos": c["pos"], "score": c["score"]}
            tasks.append((c, ql[:, b, h * g:(h + 1) * g], kl[:, b, h], vl[:, b, h], wl.P, b_l, wl.policy, wl.n_sink))
    busy = {}
    for pid, dt in pool.map(_oracle_unit_task, tasks, timeout=600, chunksize=max(1, len(tasks) // (cores * 8))):
        busy[pid] = busy.get(pid, 0.0) + dt
    pool.shutdown()
    cpu_s, wall_s = sum(busy.values()), max(busy.values())
    frac = units_per_layer / float(wl.B * wl.Hkv)
    est_step_s = wall_s / steps / frac                  # one decode step of the whole batch on these cores
    return {"value": wl.B / est_step_s, "unit": "tokens/s", "cores": len(busy), "nproc": nproc, "kind": "oracle",
            "sample": "%d of %d units of each of %d layers, first %d decode steps: %.1f s of CPU over %d worker "
                      "processes, busiest %.1f s" % (units_per_layer, wl.B * wl.Hkv, wl.L, steps, cpu_s, len(busy), wall_s),
            "single_core_value": wl.B / (cpu_s / steps / frac)}


# ---- short decode-only legs on the other workloads ------------------------------------------
def decode_leg(sess, label, per_layer=False, passes=2):
    """Decode steps only, over sess.wl.S steps: the prompt is (re)compressed untimed, one untimed pass warms
    up, the next `passes - 1` are timed with HIP events on the launch stream."""
    import torch
    wl = sess.wl
    ms = 0.0
    for i in range(passes):
        sess.probe_and_allocate()
        sess.compress_prompt()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        sess.decode(per_layer=per_layer)
        e1.record()
        torch.cuda.synchronize()
        if i > 0:
            ms += e0.elapsed_time(e1)
    ms /= (passes - 1)
    launches = wl.S * (wl.L if per_layer else 1)
    bytes_launch = sum(sess.decode_bytes_per_step()) / float(launches)
    launch_s = ms * 1e-3 / launches
    from paper_2404_04793_amd import binding as sqa
    return {"workload": label, "batch": wl.B, "policy": wl.policy, "launch": "per_layer" if per_layer else "all_layers",
            "decode_steps_timed": wl.S, "tokens_per_s": round(wl.B * wl.S / (ms * 1e-3), 1),
            "launch_us": round(launch_s * 1e6, 2), "bytes_per_launch": int(bytes_launch),
            "GBps": round(bytes_launch / launch_s / 1e9, 1), "frac": round(bytes_launch / launch_s / 1e9 / HBM_PEAK_GBS, 4),
            "resident_kv_GB": round(sess.resident_kv_bytes() / 1e9, 3),
            "device_status": sqa.read_device_status(sess.dec_ws)}


def other_workloads(main_sess, say):
    """The other BASELINE configurations at their real batch and layer count (decode only, a cut number of
    steps, the probe on 4096 token rows), one launch per layer at the headline shape, and the stress
    configuration's comparison with an uncompressed cache at equal batch and at equal memory."""
    import gc
    import torch
    from paper_2404_04793_amd import workloads as W
    from paper_2404_04793_amd.session import Session
    out = []
    say("llama2_7b, one launch per layer")
    out.append(decode_leg(main_sess, "llama2_7b", per_layer=True))
    if not main_sess.blocked and not main_sess.ragged:
        say("llama2_7b, K and V in 16-row blocks behind a shuffled block table")
        main_sess.blocked, main_sess.caches = True, None
        leg = decode_leg(main_sess, "llama2_7b blocked allocation")
        leg["kv_allocation"] = "blocked"
        out.append(leg)
        main_sess.blocked, main_sess.caches = False, None
    for name, steps in (("mistral_7b", 64), ("llama2_70b", 32), ("stress_7b", 128)):
        say("%s, %d decode steps" % (name, steps))
        wl = W.scaled(W.WORKLOADS[name], S=steps)
        sess = Session(wl, "cuda:0", probe_tokens=4096)
        leg = decode_leg(sess, name)
        out.append(leg)
        if name == "stress_7b":
            full = W.WORKLOADS[name]
            squeezed_bytes = sess.resident_kv_bytes()
            say("stress_7b, full cache at the same batch")
            sess.full_cache, sess.caches = True, None
            eq_batch = decode_leg(sess, "stress_7b full cache, same batch")
            del sess
            gc.collect(); torch.cuda.empty_cache()
            # the largest batch whose uncompressed cache, sized for the whole generation (P + S = 1536 tokens
            # per sequence, Sec. 2.1 size model), fits in the memory the squeezed run's caches occupy
            per_seq = W.full_cache_bytes_per_sequence(full)
            b_fit = max(1, W.equal_memory_batch(full, squeezed_bytes))
            say("stress_7b, full cache at batch %d (equal memory), all %d decode steps" % (b_fit, full.S))
            sess = Session(W.scaled(full, B=int(b_fit)), "cuda:0", full_cache=True, probe_tokens=4096)
            eq_mem = decode_leg(sess, "stress_7b full cache, equal memory")
            leg["vs_full_cache"] = {
                "same_batch": eq_batch, "equal_memory": eq_mem,
                "squeezed_kv_GB": round(squeezed_bytes / 1e9, 3), "full_cache_bytes_per_sequence": int(per_seq),
                "batch_gain": round(wl.B / float(b_fit), 2),
                "tokens_per_s_gain_same_batch": round(leg["tokens_per_s"] / eq_batch["tokens_per_s"], 2),
                "tokens_per_s_gain_equal_memory": round(leg["tokens_per_s"] / eq_mem["tokens_per_s"], 2)}
        del sess
        gc.collect(); torch.cuda.empty_cache()
    # H2O with grouped queries (the matrix-core variant that also accumulates scores): not a combination the
    # paper's throughput table uses, measured because the kernel supports it
    for name, steps in (("mistral_7b", 64), ("llama2_70b", 32)):
        say("%s under H2O, %d decode steps" % (name, steps))
        sess = Session(W.scaled(W.WORKLOADS[name], S=steps, policy="h2o"), "cuda:0", probe_tokens=4096)
        out.append(decode_leg(sess, name + " --policy h2o"))
        del sess
        gc.collect(); torch.cuda.empty_cache()
    return out


def launch_floor(args, wl):
    """What a single-layer decode call costs on the GPU whatever it streams: four groups of 100 launches over the
    units of ONE layer of the workload's shape (budget 143 tokens), each followed by a synchronisation so that a
    kernel trace (rocprofv3 --kernel-trace) shows them one by one, in this order: the H2O step; the same launch
    with every sequence sitting out (a workgroup returns after its first requests); the step with a sliding
    window; a sitting-out launch over 8-token units.  Prints its own HIP-event medians, which include the gap
    between two events (a few microseconds): the trace is the measurement."""
    import torch
    from paper_2404_04793_amd import binding as sqa
    dev, n = "cuda:0", 100
    B, H, D, P = wl.B, wl.Hkv, wl.D, wl.P
    res = []
    for label, budget, policy, sit in (("h2o_143", 143, "h2o", False), ("h2o_143_sitting_out", 143, "h2o", True),
                                       ("sliding_143", 143, "sliding", False), ("h2o_8_sitting_out", 8, "h2o", True)):
        caches = sqa.LayerCaches([budget], [min(budget, P + n + 40)], B, H, D, wl.torch_dtype, dev, True)
        K = torch.randn(B, H, P, D, device=dev).to(wl.torch_dtype)
        V = torch.randn(B, H, P, D, device=dev).to(wl.torch_dtype)
        sc = torch.rand(B, H, P, device=dev)
        sqa.prefill_compress(K, V, sc if policy == "h2o" else None, policy, wl.n_sink, caches, 0)
        ws = sqa.decode_workspace(caches, wl.Hq, policy)
        q = torch.randn(1, B, wl.Hq, D, device=dev).to(wl.torch_dtype)
        kv = torch.randn(1, B, H, D, device=dev).to(wl.torch_dtype)
        out = torch.empty_like(q)
        pos = torch.full((B,), -1 if sit else P, dtype=torch.int32, device=dev)
        opts = sqa.batch_opts(new_pos_seq=pos)
        times = []
        for i in range(n):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            sqa.decode_step(q, kv, kv, 0, policy, wl.n_sink, caches, out, ws, opts=opts)
            e1.record()
            torch.cuda.synchronize()
            times.append(e0.elapsed_time(e1) * 1e3)
            if not sit:
                pos += 1
        assert sqa.read_device_status(ws) == 0
        times = sorted(times[10:])
        res.append({"launches": label, "units": B * H, "median_us_between_events": round(times[len(times) // 2], 2)})
    print(json.dumps({"metric": "single-layer decode launch, microseconds (see the kernel trace)", "config": {"workload": wl.name},
                      "groups_in_launch_order": res}))
    return 0


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
    LSE = None
    if args.lse:
        # the ln-normalisers of the prompt's causal attention, as a fused attention kernel would hand them over
        # (input preparation with torch, untimed; one head at a time to keep the logit matrix small)
        LSE = []
        tri = torch.ones(wl.P, wl.P, dtype=torch.bool, device=dev).tril()
        for Q, K in QK:
            out = torch.empty(wl.B, wl.Hq, wl.P, dtype=torch.float32, device=dev)
            for b in range(wl.B):
                for h in range(wl.Hq):
                    s_ = (Q[b, h].float() @ K[b, h // wl.g].float().T) / (wl.D ** 0.5)
                    out[b, h] = torch.logsumexp(s_.masked_fill(~tri, float("-inf")), dim=-1)
            LSE.append(out)

    def one_pass():
        for l in range(wl.L):
            sqa.prefill_scores(QK[l % n_gen][0], QK[l % n_gen][1], row_lse=None if LSE is None else LSE[l % n_gen])

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
    flops = (1 if args.lse else 2) * wl.B * wl.Hq * (wl.P * (wl.P + 1) // 2) * 2 * wl.D
    peak = 2500.0 if (wl.dtype == "bf16" and wl.D == 128) else 157.3     # matrix cores (bf16, D = 128) or fp32 vector
    out = {
        "metric": "H2O prompt-score producer (causal softmax column sums), TFLOP/s", "value": flops / call_s / 1e12,
        "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": dt / args.steps * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": wl.name, "layers": wl.L, "q_heads": wl.Hq, "kv_heads": wl.Hkv, "head_dim": wl.D,
                   "batch": wl.B, "prompt": wl.P, "phases": "scores_only",
                   "passes": "column sums from given row normalisers" if args.lse else "row statistics + column sums"},
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
    ap.add_argument("--blocked", action="store_true",
                    help="K and V in pools of 16-row blocks scattered by a block table (sqa_layer_cache.block_table)")
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
    ap.add_argument("--launch-floor", action="store_true",
                    help="single-layer decode launches one by one, with and without work, for a kernel trace")
    ap.add_argument("--scores-only", action="store_true",
                    help="time only the H2O prompt-score producer (sqa_prefill_scores; set-up work of the pass, "
                         "matrix-core bound): a step = the scores of all layers of one prompt batch")
    ap.add_argument("--lse", action="store_true",
                    help="with --scores-only: the row normalisers are given (sqa_prefill_scores_lse), one pass instead of two")
    ap.add_argument("--progress", action="store_true", help="say on stderr when each phase of the run begins")
    ap.add_argument("--no-others", action="store_true",
                    help="skip the short decode-only legs on the other workloads (they run by default with the "
                         "headline workload and no other switch)")
    ap.add_argument("--cpu-units", type=int, default=32)
    ap.add_argument("--cpu-steps", type=int, default=128)
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    pool = None
    if not (args.no_cpu or args.scores_only):
        pool, cores, nproc = oracle_pool()          # (before the first GPU call)

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
    if args.launch_floor:
        return launch_floor(args, wl)
    plen = [wl.P - (b * wl.P) // (2 * wl.B) for b in range(wl.B)] if args.ragged else None
    def say(what):
        if args.progress:
            print("bench.py: " + what, file=sys.stderr, flush=True)

    say("generating inputs for %s" % wl.name)
    sess = Session(wl, "cuda:0", uniform_budget=args.uniform, full_cache=args.full_cache,
                   probe_tokens=args.probe_tokens, fused_probe=args.fused_probe, order=args.order, prompt_len=plen,
                   blocked=args.blocked)
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
    traffic, traffic_source = measured_traffic((wl.name, mode, wl.policy, launch, "blocked" if args.blocked else "dense"))
    launch_plan = None
    if not args.per_layer and plen is None:
        from paper_2404_04793_amd import binding as sqa_b
        lp = sqa_b.decode_plan(sess.budgets, sess.caches.capacities, wl.B, wl.Hq, wl.Hkv, wl.D, wl.dtype, wl.policy,
                               args.blocked)
        launch_plan = {"workgroups": lp["workgroups"], "lds_bytes_per_workgroup": lp["lds_bytes"],
                       "matrix_cores": bool(lp["matrix_cores"]),
                       "layers_one_wave_per_unit": sum(l["wave_per_unit"] for l in lp["layers"]),
                       "layers_whole_units": sum(l["workgroups_per_unit"] == 1 for l in lp["layers"]),
                       "layers_split_units": sum(l["workgroups_per_unit"] > 1 for l in lp["layers"])}
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
                   "ragged_prompt_lengths": plen, "kv_allocation": "blocked" if args.blocked else "dense"},
        "roofline": {"bound": "hbm", "kernel": "decode_unit_kernel", "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": traffic, "traffic_source": traffic_source,
                     "bytes_per_launch": bytes_launch, "launch_us": launch_s * 1e6, "launch_plan": launch_plan},
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
        say("oracle on the host cores")
        res["cpu_baseline"] = cpu_baseline(sess, args.cpu_units, min(args.cpu_steps, wl.S), pool, cores, nproc)
    headline = (args.workload == "llama2_7b" and not (args.per_layer or args.graph or args.ragged or args.uniform or
                                                      args.full_cache or args.policy or args.decode_only or args.batch or
                                                      args.kv_heads or args.budget_pct or args.decode_steps or
                                                      args.fused_probe or args.probe_tokens) and
                args.order == "evict_then_attend" and not args.blocked)
    if headline and not args.no_others:
        res["other_workloads"] = other_workloads(sess, say)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
