"""Helpers for the GPU parity tests: move one unit's cache state between the
oracle's representation and the library's device layout, and the tolerance
rule.  Test infrastructure only."""
from __future__ import annotations

import numpy as np
import torch

TOL = {"f32": 1e-5, "bf16": 2e-2}


def rel_err(x, ref) -> float:
    """max|x - ref| / max|ref| over one output vector (or a stack of them, row-wise worst)."""
    x = np.asarray(x, dtype=np.float64).reshape(-1, np.shape(ref)[-1])
    ref = np.asarray(ref, dtype=np.float64).reshape(x.shape)
    num = np.abs(x - ref).max(axis=1)
    den = np.maximum(np.abs(ref).max(axis=1), 1e-30)
    return float((num / den).max())


def np64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu").to(torch.float64).numpy()


def import_state(caches, layer: int, b: int, h: int, c: dict) -> None:
    """Write an oracle cache (ascending position) into unit (b, h) of a layer
    in the library's canonical layout: slot i = i-th smallest position, ring head 0."""
    n = len(c["pos"])
    dev = caches.K[layer].device
    dt = caches.dtype
    K, V, score, pos = caches.unit(layer, b, h)
    K[:n] = torch.from_numpy(c["K"]).to(dt).to(dev)
    V[:n] = torch.from_numpy(c["V"]).to(dt).to(dev)
    pos[:n] = torch.from_numpy(c["pos"].astype(np.int32)).to(dev)
    pos[n:] = -1
    if score is not None:
        score[:n] = torch.from_numpy(c["score"]).to(torch.float32).to(dev)
    caches.lens[layer][b, h] = n
    caches.head[layer][b, h] = 0
    caches.hint[layer][b, h] = -2          # scores were edited: no eviction decision carried over


def export_state(caches, layer: int, b: int, h: int) -> dict:
    """Unit (b, h) of a layer as an oracle-style cache sorted by position."""
    n = int(caches.lens[layer][b, h].item())
    K, V, score, pos_t = caches.unit(layer, b, h)
    pos = pos_t[:n].cpu().numpy().astype(np.int64)
    order = np.argsort(pos, kind="stable")
    out = {"pos": pos[order], "K": np64(K[:n])[order], "V": np64(V[:n])[order]}
    if score is not None:
        out["score"] = np64(score[:n])[order]
    else:
        out["score"] = np.zeros(n)
    return out


def round_scores_f32(c: dict) -> dict:
    d = dict(c)
    d["score"] = c["score"].astype(np.float32).astype(np.float64)
    return d


def near_tie_swap(got_pos, want_pos, c_before, c_after_full, rec, tol):
    """Attend-then-evict decides on scores updated in this very step, in fp32 on
    the GPU and fp64 in the oracle: when the two worst candidates are closer
    than the fp32 error either may go.  True if that is what happened."""
    a, b = set(got_pos) - set(want_pos), set(want_pos) - set(got_pos)
    if len(a) != 1 or len(b) != 1:
        return False
    cand = sorted(c_after_full)[: len(c_after_full) - rec]
    x, y = a.pop(), b.pop()
    if x not in cand or y not in cand:
        return False
    return abs(c_after_full[x] - c_after_full[y]) <= tol * max(abs(c_after_full[x]), abs(c_after_full[y]), 1e-30)
