"""The comparison rules of the GPU parity tests, exercised on the CPU with planted mistakes: a rule that
would let a wrong victim, a wrong small score or a wrong carried decision through fails here."""
import numpy as np
import pytest

from oracle import sqa_oracle as O
from tests import harness as H


def _unit(n=12, D=8, seed=0):
    r = np.random.default_rng(seed)
    return O.new_cache(r.standard_normal((n, D)), r.standard_normal((n, D)), score=r.random(n) + 0.05)


def _step(c, budget, order="evict_then_attend", seed=1, g=2):
    r = np.random.default_rng(seed)
    D = c["K"].shape[1]
    return O.decode_step(c, r.standard_normal((g, D)), r.standard_normal(D), r.standard_normal(D),
                         int(c["pos"].max()) + 1, budget, "h2o", 4, order)


def test_score_rule_accepts_rounding_and_rejects_a_wrong_small_score():
    c = _unit()
    _, c2 = _step(c, 12)
    p = H.step_probabilities(c, c2)
    assert abs(p.sum() - 2.0) < 1e-12                       # two heads: the step's mass
    got = {"pos": c2["pos"], "score": c2["score"].astype(np.float32).astype(np.float64)}
    assert H.check_step_scores(got, c, c2, False) <= 1.0    # fp32 rounding of the exact result passes
    # a token whose increment is dropped: invisible to a max-norm over the vector, caught per element
    j = int(np.argmin(p))
    bad = dict(got); bad["score"] = got["score"].copy(); bad["score"][j] -= p[j]
    assert H.rel_err(bad["score"][None], c2["score"][None]) < 0.2
    with pytest.raises(AssertionError):
        H.check_step_scores(bad, c, c2, False)
    # a relative error of 1e-3 in the increment passes only under the matrix-core bound
    off = dict(got); off["score"] = c2["score"] + 1e-3 * p
    assert H.check_step_scores(off, c, c2, True) <= 1.0
    with pytest.raises(AssertionError):
        H.check_step_scores(off, c, c2, False)


def test_near_tie_rule():
    c = _unit()
    budget = 12
    _, want = _step(c, budget, "attend_then_evict")
    _, full = _step(c, 1 << 30, "attend_then_evict")
    rec = budget - budget // 2
    victim = (set(full["pos"].tolist()) - set(want["pos"].tolist())).pop()
    cand = sorted(full["pos"].tolist())[: len(full["pos"]) - rec]
    sc = dict(zip(full["pos"].tolist(), full["score"].tolist()))
    others = sorted((p for p in cand if p != victim), key=lambda p: sc[p])
    second = others[0]
    swapped = sorted((set(want["pos"].tolist()) - {second}) | {victim})
    # the runner-up is clearly better than the victim here: evicting it instead is a mistake
    assert sc[second] - sc[victim] > 1e-3
    assert not H.near_tie_swap(swapped, want["pos"].tolist(), c, full, rec, False)
    assert not H.near_tie_swap(swapped, want["pos"].tolist(), c, full, rec, True)
    # make the two indistinguishable in fp32: now either may go
    i, j = full["pos"].tolist().index(second), full["pos"].tolist().index(victim)
    tie = {k: v.copy() for k, v in full.items()}
    tie["score"][i] = tie["score"][j] * (1 + 1e-9)
    assert H.near_tie_swap(swapped, want["pos"].tolist(), c, tie, rec, False)
    # a token from the recent window is never a legitimate victim
    newest = int(full["pos"].max())
    wrong = sorted((set(want["pos"].tolist()) - {newest}) | {victim})
    assert not H.near_tie_swap(wrong, want["pos"].tolist(), c, tie, rec, False)
    # two tokens differing is never a tie
    wrong2 = sorted((set(want["pos"].tolist()) - {second, others[1]}) | {victim})
    assert not H.near_tie_swap(wrong2, want["pos"].tolist(), c, tie, rec, False)


def test_carried_decision_helpers():
    """oracle_next_victim_pos = what one more oracle step evicts; carried_victim_pos reads the slot layout
    (heavy region [0, hh), ring behind it, oldest ring token at hh + ring_head)."""
    c = _unit(n=10)
    budget = 10
    _, c2 = _step(c, budget)                       # full before and after: one token went
    expected = H.oracle_next_victim_pos(c2, budget)
    _, c3 = _step(c2, budget, seed=5)
    assert (set(c2["pos"].tolist()) | {int(c2["pos"].max()) + 1}) - set(c3["pos"].tolist()) == {expected}
    hh = budget // 2
    raw_pos = np.array([7, 3, 0, 5, 1, 12, 13, 9, 10, 11])      # heavy slots 0..4, ring 5..9 with its oldest at slot 7
    raw = {"raw_pos": raw_pos, "ring_head": 2, "hint": -1}
    assert H.carried_victim_pos(raw, budget) == 9
    assert H.carried_victim_pos(dict(raw, hint=3), budget) == 5
    assert H.carried_victim_pos(dict(raw, hint=-2), budget) is None
    assert H.carried_victim_pos(dict(raw, hint=hh), budget) is None


def test_clustering_margin():
    assert H.clustering_margin([0.1, 0.1, 0.5, 0.5, 0.9, 0.9]) > 0.5
    # two splits of equal cost: no margin
    assert H.clustering_margin([0.0, 1.0, 2.0, 3.0]) < 1e-12
    assert H.clustering_margin([0.3, 0.3, 0.7]) == float("inf")     # fewer than three distinct values
