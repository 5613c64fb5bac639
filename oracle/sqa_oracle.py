"""CPU oracle for the SqueezeAttention hot path -- TEST INFRASTRUCTURE ONLY.

Plain, slow, fp64 numpy (Python loops where order of evaluation matters),
written from the paper; it shares no code with the HIP library and is never
imported by the product path.  Only tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py may call it.

What each function follows:
  token_cosines / layer_importance   Sec. 3, the cosine-similarity equation;
                                     Algorithm 1 steps 1-4 (mean over prompt tokens)
  residual_hidden                    Sec. 3: the hidden state "after" the block is
                                     the block's input plus the attention output
  cluster_layers / allocate_budgets  Algorithm 1 steps 5-11; Sec. 4.2.2 (three
                                     groups, only G3 loses budget); Appendix A.2
                                     worked example (300 / 1544)
  prefill_scores                     Sec. 5.1 "Heavy-Hitter (H2O)": accumulated
                                     attention score of each token over the prompt
  prefill_row_lse /                  the same from given softmax normalisers (Sec. 2.1
  prefill_scores_from_lse            attention equation: the denominator of softmax)
  select_keep                        Sec. 2.2 / Sec. 5.1: sliding window, StreamingLLM
                                     (n sink tokens + recent), H2O (accumulated score)
  prefill_compress / decode_step     Algorithm 1 steps 12-21 with Eq. 2-3 (append)

Readings taken where the paper is silent:
  * one cosine per layer = mean over ALL tokens of the batch (b x p rows);
  * a zero-norm row contributes cosine 0 (each norm is clamped at 1e-8);
  * KMeans = the global optimum of 1-D 3-means on the sorted values (a
    contiguous split, cuts only between distinct values), ties -> smallest cut
    positions; fewer than 3 distinct values -> that many groups; 1 -> uniform;
    the sums are evaluated sequentially in sorted order in IEEE double so that
    an independent implementation of the same rule reproduces them bit for bit;
  * b_low = floor(total * p / L) (double), the rest is split evenly over the
    other layers, remainder +1 to the lowest layer indices: sum is exact;
  * decode order per layer: append -> evict if over budget -> attend -> accumulate
    (Algorithm 1 as printed); the other order, attend -> accumulate -> evict, is
    available as a variant;
  * H2O: per (layer, sequence, KV head); hh = floor(b/2) best by (score desc,
    position asc) among the non-recent tokens + the b-hh most recent; with
    grouped queries the probabilities of the g query heads are summed;
  * StreamingLLM sinks count against the budget.
Parity unpinned: which eviction order and which H2O accumulator scope the
authors' own code used (the paper does not say); everything else is pinned by
tests/test_oracle_*.py.
"""
from __future__ import annotations

import math
from typing import Dict, List, Sequence, Tuple

import numpy as np

EPS_NORM = 1e-8
POLICIES = ("sliding", "streaming", "h2o")


# --------------------------------------------------------------------------
# Sec. 3 cosine similarity, Algorithm 1 steps 1-4
# --------------------------------------------------------------------------

def token_cosines(A, B) -> np.ndarray:
    """A, B: [T, n] hidden rows before / after self-attention -> cos_j [T]."""
    A = np.asarray(A, dtype=np.float64)
    B = np.asarray(B, dtype=np.float64)
    ab = np.einsum("tn,tn->t", A, B)
    aa = np.einsum("tn,tn->t", A, A)
    bb = np.einsum("tn,tn->t", B, B)
    return ab / (np.maximum(np.sqrt(aa), EPS_NORM) * np.maximum(np.sqrt(bb), EPS_NORM))


def layer_importance(h_in, h_out) -> np.ndarray:
    """h_in, h_out: [L, T, n] -> cos_sim^(i) [L] = mean over the T tokens."""
    L = len(h_in)
    out = np.empty(L, dtype=np.float64)
    for i in range(L):
        c = token_cosines(h_in[i], h_out[i])
        out[i] = math.fsum(c.tolist()) / len(c)
    return out


def round_bf16(x32: np.ndarray) -> np.ndarray:
    """float32 array -> the nearest bfloat16 values (ties to even), returned as
    float32.  bfloat16 = the top 16 bits of the float32 pattern."""
    u = np.ascontiguousarray(x32, dtype=np.float32).view(np.uint32).astype(np.uint64)
    keep_odd = (u >> np.uint64(16)) & np.uint64(1)
    u = (u + np.uint64(0x7FFF) + keep_odd) & np.uint64(0xFFFF0000)
    return u.astype(np.uint32).view(np.float32).reshape(np.shape(x32))


def residual_hidden(h_in, attn_out, dtype: str) -> np.ndarray:
    """The hidden state after the self-attention block as the model stores it:
    h_in + attn_out (the residual connection), added in float32 and rounded to
    the storage type ("f32" or "bf16").  Sec. 3 takes the cosine between h_in
    and this tensor, so the stored (rounded) values are what the probe sees."""
    s = np.asarray(h_in, dtype=np.float32) + np.asarray(attn_out, dtype=np.float32)
    if dtype == "bf16":
        return round_bf16(s)
    if dtype == "f32":
        return s
    raise ValueError(dtype)


# --------------------------------------------------------------------------
# Algorithm 1 steps 5-11: groups and budgets
# --------------------------------------------------------------------------

def _sse(x: Sequence[float], lo: int, hi: int) -> float:
    """Sum of squared deviations of x[lo:hi] from its mean; sequential, double."""
    s = 0.0
    for t in range(lo, hi):
        s += x[t]
    mean = s / (hi - lo)
    e = 0.0
    for t in range(lo, hi):
        d = x[t] - mean
        e += d * d
    return e


def cluster_layers(cos) -> Tuple[List[int], int]:
    """cos [L] -> (group id per layer, k).  Group ids: 0 = G1 (lowest cos),
    1 = G2, 2 = G3 (largest cos).  With two groups the lower one is G2; with one
    group every layer is G2 (nothing to take budget from)."""
    L = len(cos)
    order = sorted(range(L), key=lambda i: (float(cos[i]), i))
    x = [float(cos[i]) for i in order]
    cut_ok = [False] + [x[c - 1] < x[c] for c in range(1, L)]   # cut before index c
    k = min(3, 1 + sum(cut_ok))
    group = [1] * L
    if k == 1:
        return group, 1
    if k == 2:
        best, best_c = None, None
        for c in range(1, L):
            if not cut_ok[c]:
                continue
            cost = _sse(x, 0, c) + _sse(x, c, L)
            if best is None or cost < best:
                best, best_c = cost, c
        for r in range(best_c, L):
            group[order[r]] = 2
        return group, 2
    best, best_c = None, None
    for c1 in range(1, L - 1):
        if not cut_ok[c1]:
            continue
        for c2 in range(c1 + 1, L):
            if not cut_ok[c2]:
                continue
            cost = _sse(x, 0, c1) + _sse(x, c1, c2) + _sse(x, c2, L)
            if best is None or cost < best:
                best, best_c = cost, (c1, c2)
    c1, c2 = best_c
    for r in range(L):
        group[order[r]] = 0 if r < c1 else (1 if r < c2 else 2)
    return group, 3


def allocate_budgets(cos, total_budget: int, p: float) -> Tuple[List[int], List[int]]:
    """cos [L], total token budget over all layers (= n_layer * b_init), p in
    (0,1] -> (budget per layer, group per layer).  Raises ValueError where the
    library reports SQA_ERR_BUDGET."""
    L = len(cos)
    if not (0.0 < p <= 1.0) or total_budget < L:
        raise ValueError("budget")
    group, k = cluster_layers(cos)
    if k == 1:
        base, r = divmod(total_budget, L)
        return [base + (1 if i < r else 0) for i in range(L)], group
    g3 = [i for i in range(L) if group[i] == 2]
    rest_layers = [i for i in range(L) if group[i] != 2]
    b_low = int(math.floor(float(total_budget) * p / float(L)))
    if b_low < 1:
        raise ValueError("budget")
    rest = total_budget - len(g3) * b_low
    b_high, r = divmod(rest, len(rest_layers))
    budget = [0] * L
    for i in g3:
        budget[i] = b_low
    for n, i in enumerate(rest_layers):          # ascending layer index
        budget[i] = b_high + (1 if n < r else 0)
    return budget, group


# --------------------------------------------------------------------------
# H2O accumulated attention over the prompt
# --------------------------------------------------------------------------

def prefill_scores(Q, K) -> np.ndarray:
    """Q [g, P, D] (the query heads sharing this KV head), K [P, D] ->
    score [P]: column sums of the causal softmax(Q K^T / sqrt(D)), added over
    the g heads."""
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    g, P, D = Q.shape
    score = np.zeros(P, dtype=np.float64)
    for h in range(g):
        S = (Q[h] @ K.T) / math.sqrt(D)
        for i in range(P):
            row = S[i, : i + 1]
            e = np.exp(row - row.max())
            score[: i + 1] += e / e.sum()
    return score


def prefill_row_lse(Q, K) -> np.ndarray:
    """Q [g, P, D], K [P, D] -> lse [g, P]: the natural logarithm of each prompt query's softmax normaliser,
    lse[h, i] = ln sum_{j<=i} exp(Q[h,i].K[j] / sqrt(D)) (what a fused attention kernel returns beside its
    output)."""
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    g, P, D = Q.shape
    out = np.empty((g, P), dtype=np.float64)
    for h in range(g):
        S = (Q[h] @ K.T) / math.sqrt(D)
        for i in range(P):
            row = S[i, : i + 1]
            m = row.max()
            out[h, i] = m + math.log(np.exp(row - m).sum())
    return out


def prefill_scores_from_lse(Q, K, lse) -> np.ndarray:
    """The same accumulated attention as prefill_scores, computed from given row normalisers:
    score[j] = sum over heads h and queries i >= j of exp(Q[h,i].K[j] / sqrt(D) - lse[h, i])."""
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    lse = np.asarray(lse, dtype=np.float64)
    g, P, D = Q.shape
    score = np.zeros(P, dtype=np.float64)
    for h in range(g):
        S = (Q[h] @ K.T) / math.sqrt(D)
        for i in range(P):
            score[: i + 1] += np.exp(S[i, : i + 1] - lse[h, i])
    return score


# --------------------------------------------------------------------------
# C_seq: which tokens a sequence-wise policy keeps
# --------------------------------------------------------------------------

def h2o_split(b: int) -> Tuple[int, int]:
    hh = b // 2
    return hh, b - hh


def select_keep(pos, score, b: int, policy: str, n_sink: int = 4) -> np.ndarray:
    """pos [n] distinct token positions, score [n] accumulated attention (used
    by h2o only) -> indices into pos (ascending by position) of the kept
    tokens; exactly min(n, b) of them."""
    pos = np.asarray(pos)
    n = len(pos)
    by_pos = sorted(range(n), key=lambda i: int(pos[i]))
    if n <= b:
        return np.array(by_pos, dtype=np.int64)
    if policy == "sliding":
        keep = by_pos[n - b:]
    elif policy == "streaming":
        sinks = [i for i in by_pos if pos[i] < n_sink][: min(n_sink, b)]
        n_recent = b - len(sinks)
        others = [i for i in by_pos if i not in set(sinks)]
        keep = sinks + (others[len(others) - n_recent:] if n_recent > 0 else [])
    elif policy == "h2o":
        hh, rec = h2o_split(b)
        recent = by_pos[n - rec:]
        older = by_pos[: n - rec]
        ranked = sorted(older, key=lambda i: (-float(score[i]), int(pos[i])))
        keep = ranked[:hh] + recent
    else:
        raise ValueError(policy)
    keep = sorted(keep, key=lambda i: int(pos[i]))
    return np.array(keep, dtype=np.int64)


# --------------------------------------------------------------------------
# one (layer, sequence, KV head) cache and Algorithm 1's decode loop body
# --------------------------------------------------------------------------

def new_cache(K, V, score=None, pos=None) -> Dict[str, np.ndarray]:
    K = np.array(K, dtype=np.float64)
    V = np.array(V, dtype=np.float64)
    n = K.shape[0]
    return {
        "K": K, "V": V,
        "pos": np.arange(n, dtype=np.int64) if pos is None else np.array(pos, dtype=np.int64),
        "score": np.zeros(n) if score is None else np.array(score, dtype=np.float64),
    }


def _take(c, idx):
    return {"K": c["K"][idx], "V": c["V"][idx], "pos": c["pos"][idx], "score": c["score"][idx]}


def prefill_compress(K, V, score, b: int, policy: str, n_sink: int = 4):
    """Prompt K, V [P, D] (+ H2O score [P]) -> cache compressed to min(P, b)
    tokens, in ascending position."""
    c = new_cache(K, V, score)
    return _take(c, select_keep(c["pos"], c["score"], b, policy, n_sink))


def attend(q, K, V) -> Tuple[np.ndarray, np.ndarray]:
    """q [g, D], K, V [n, D] -> out [g, D], probabilities [g, n]."""
    q = np.asarray(q, dtype=np.float64)
    D = q.shape[-1]
    s = (q @ K.T) / math.sqrt(D)
    s = s - s.max(axis=1, keepdims=True)
    e = np.exp(s)
    prob = e / e.sum(axis=1, keepdims=True)
    return prob @ V, prob


ORDERS = ("evict_then_attend", "attend_then_evict")


def decode_step(c, q, k_new, v_new, new_pos: int, b: int, policy: str, n_sink: int = 4,
                order: str = "evict_then_attend"):
    """One decode step of one (layer, sequence, KV head).
    order "evict_then_attend" (Algorithm 1 as printed): append (Eq. 2-3) ->
    compress if longer than b (steps 16-17) -> attention of the g query heads
    (step 19) -> H2O accumulation.
    order "attend_then_evict" (the other reading of Sec. 2.2, where the policy
    runs after the step's attention has been observed): append -> attention over
    all b+1 tokens -> H2O accumulation -> compress if longer than b.
    Returns (out [g, D], cache)."""
    if order not in ORDERS:
        raise ValueError(order)
    c = {
        "K": np.vstack([c["K"], np.asarray(k_new, dtype=np.float64)[None]]),
        "V": np.vstack([c["V"], np.asarray(v_new, dtype=np.float64)[None]]),
        "pos": np.append(c["pos"], np.int64(new_pos)),
        "score": np.append(c["score"], 0.0),
    }
    if order == "evict_then_attend" and len(c["pos"]) > b:
        c = _take(c, select_keep(c["pos"], c["score"], b, policy, n_sink))
    out, prob = attend(q, c["K"], c["V"])
    if policy == "h2o":
        c["score"] = c["score"] + prob.sum(axis=0)
    if order == "attend_then_evict" and len(c["pos"]) > b:
        c = _take(c, select_keep(c["pos"], c["score"], b, policy, n_sink))
    return out, c
