"""Attention-level analogue of the paper's throughput and memory comparisons
(Sec. 5.3 Fig. 4: KV memory per generated token; Sec. 5.4 Table 3: tokens/s
against batch size for the layer-wise budgets, the sequence-only baseline and
the full cache), on synthetic inputs of the paper's shapes.

    python -m paper_2404_04793_amd.report [--workload stress_7b] [--batches 1,32,64,128,224]
                                          [--decode-steps 64] [--equal-memory]

--equal-memory adds, per batch, the full-cache run at the largest batch whose
uncompressed cache -- sized for the workload's WHOLE generation, P + S tokens
per sequence, whatever --decode-steps cuts the timed run to -- fits in the bytes
the layer-wise run holds resident at that batch (the "same memory, larger
batch" reading of Table 3; workloads.equal_memory_batch, the rule bench.py uses).

Prints a markdown table.  Only the decode steps are timed (HIP events); every
number comes from the HIP library through the binding.
"""
from __future__ import annotations

import argparse
import sys

import torch

from . import workloads as W
from .session import Session


def run_mode(wl: W.Workload, mode: str, passes: int = 2):
    sess = Session(wl, "cuda:0", uniform_budget=(mode == "uniform"), full_cache=(mode == "full"),
                   probe_tokens=min(wl.B * wl.P, 4096))
    best = None
    for _ in range(passes):
        sess.probe_and_allocate()
        sess.compress_prompt()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        sess.decode()
        b.record()
        torch.cuda.synchronize()
        ms = a.elapsed_time(b)
        best = ms if best is None else min(best, ms)
    tok_s = wl.B * wl.S / (best * 1e-3)
    gbs = sum(sess.decode_bytes_per_step()) / (best * 1e-3) / 1e9
    kv_bytes = sess.resident_kv_bytes()
    del sess
    torch.cuda.empty_cache()
    return tok_s, gbs, kv_bytes / 1e9, kv_bytes / wl.B / 1e6, kv_bytes


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="stress_7b")
    ap.add_argument("--batches", default="1,32,64,128,224")
    ap.add_argument("--decode-steps", type=int, default=64)
    ap.add_argument("--budget-pct", type=int, default=None)
    ap.add_argument("--equal-memory", action="store_true")
    args = ap.parse_args(argv)
    whole = W.WORKLOADS[args.workload]
    if args.budget_pct:
        whole = W.scaled(whole, budget_pct=args.budget_pct)
    base = W.scaled(whole, S=args.decode_steps)
    print("| batch | mode | tokens/s | GB/s | resident KV (GB) | KV per sequence (MB) |")
    print("|---|---|---|---|---|---|")
    for bs in [int(x) for x in args.batches.split(",")]:
        wl = W.scaled(base, B=bs)
        held = {}
        for mode in ("squeeze", "uniform", "full"):
            try:
                tok_s, gbs, kv_gb, per_seq, kv_bytes = run_mode(wl, mode)
                held[mode] = (kv_gb, per_seq, kv_bytes)
                print("| %d | %s | %.0f | %.0f | %.2f | %.1f |" % (bs, mode, tok_s, gbs, kv_gb, per_seq))
            except torch.cuda.OutOfMemoryError:
                print("| %d | %s | OOM | | | |" % (bs, mode))
            sys.stdout.flush()
        if args.equal_memory and "squeeze" in held:
            fit = W.equal_memory_batch(whole, held["squeeze"][2])
            if fit >= 1:
                tok_s, gbs, kv_gb, per_seq, _ = run_mode(W.scaled(base, B=fit), "full")
                print("| %d | full, batch that fits in the squeezed run's %.2f GB | %.0f | %.0f | %.2f | %.1f |"
                      % (fit, held["squeeze"][0], tok_s, gbs, kv_gb, per_seq))
            else:
                print("| 0 | full: not even one sequence fits in %.2f GB | | | | |" % held["squeeze"][0])
            sys.stdout.flush()


if __name__ == "__main__":
    main()
