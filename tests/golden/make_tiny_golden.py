"""Writes tests/golden/tiny_end_to_end.json: configs[0] ("Tiny") run end to end
by the CPU oracle alone -- Algorithm 1 from the probe to the 16th decode step.
Calls only oracle/ and the seeded input generators.  Run from the repo root:
    python tests/golden/make_tiny_golden.py
"""
import json
import os
import sys

import numpy as np
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import pipeline as OP          # noqa: E402
from oracle import sqa_oracle as O         # noqa: E402
from paper_2404_04793_amd import workloads as W   # noqa: E402


def compute():
    wl = W.WORKLOADS["tiny"]
    f64 = lambda t: t.to(torch.float64).numpy()
    hs = [W.hidden_states(wl, l) for l in range(wl.L)]
    cos = O.layer_importance([f64(x[0]) for x in hs], [f64(x[1]) for x in hs])
    budgets, groups = O.allocate_budgets(cos.astype(np.float32), wl.total_budget, wl.p)
    u, mask = W.unit_dirs(wl), W.hh_mask(wl)
    units = {}
    for l in range(wl.L):
        K, V = W.prompt_kv(wl, l, "cpu", u, mask)
        Q = W.prompt_q(wl, l, "cpu", u)
        q, k, v = W.decode_qkv(wl, l, "cpu", u, mask)
        for h in range(wl.Hkv):
            s0 = O.prefill_scores(f64(Q)[0, h:h + 1], f64(K)[0, h])
            outs, c, states, first = OP.run_unit(f64(K)[0, h], f64(V)[0, h], s0, f64(q)[:, 0, h:h + 1], f64(k)[:, 0, h],
                                                 f64(v)[:, 0, h], budgets[l], wl.policy, wl.n_sink, keep_states=True)
            units["%d,%d" % (l, h)] = {
                "kept_after_prefill": first["pos"].tolist(),
                "kept_after_step": {str(t): states[t]["pos"].tolist() for t in (0, 7, 15)},
                "out_last_step_first4": [float("%.9e" % x) for x in outs[-1, 0, :4]],
                "score_sum_end": float("%.9e" % c["score"].sum()),
            }
    return {"workload": "tiny", "cos": [float("%.7f" % c) for c in cos], "budgets": budgets, "groups": groups,
            "units": units}


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_end_to_end.json")
    with open(path, "w") as f:
        json.dump(compute(), f, indent=0, separators=(",", ":"))
    print("wrote", path)
