"""Test infrastructure: drives the oracle over one (layer, sequence, KV head)
unit of a workload, step by step, in Algorithm 1's order.  Calls only
oracle.sqa_oracle; inputs are numpy arrays (already widened to fp64)."""
from __future__ import annotations

import numpy as np

from . import sqa_oracle as O


def run_unit(Kp, Vp, score0, q_steps, k_steps, v_steps, b, policy, n_sink=4, keep_states=False,
             order="evict_then_attend"):
    """Kp, Vp [P, D]; score0 [P] or None; q_steps [S, g, D]; k_steps, v_steps
    [S, D].  Compress the prompt to budget b, then S decode steps.
    Returns (outs [S, g, D], final cache, list of per-step caches or None)."""
    P = Kp.shape[0]
    c = O.prefill_compress(Kp, Vp, np.zeros(P) if score0 is None else score0, b, policy, n_sink)
    first = c
    S = q_steps.shape[0]
    outs = np.empty(q_steps.shape, dtype=np.float64)
    states = [] if keep_states else None
    for t in range(S):
        outs[t], c = O.decode_step(c, q_steps[t], k_steps[t], v_steps[t], P + t, b, policy, n_sink, order)
        if keep_states:
            states.append(c)
    return outs, c, states, first
