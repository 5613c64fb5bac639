"""Pins for the oracle's sequence-wise policies and H2O prompt scores
(Sec. 2.2 and Sec. 5.1 policy descriptions; Algorithm 1 steps 16-17)."""
import math

import numpy as np
import pytest

from oracle import sqa_oracle as O


def _rng(s):
    return np.random.default_rng(s)


# ---------------- H2O prompt scores ----------------

def test_scores_mass_and_first_row():
    r = _rng(0)
    g, P, D = 3, 17, 8
    Q, K = r.standard_normal((g, P, D)), r.standard_normal((P, D))
    s = O.prefill_scores(Q, K)
    assert abs(s.sum() - g * P) < 1e-11            # every softmax row sums to 1
    assert s[0] >= g - 1e-12                       # first causal row is [1]
    assert np.all(s > 0)


def test_scores_p1_p2_by_hand():
    assert np.allclose(O.prefill_scores(np.ones((2, 1, 4)), np.ones((1, 4))), [2.0])
    q = np.array([[[1.0, 0.0], [2.0, 0.0]]]); k = np.array([[1.0, 0.0], [3.0, 0.0]])
    # row 0: [1]; row 1: logits (2, 6)/sqrt(2)
    a, b = 2 / math.sqrt(2), 6 / math.sqrt(2)
    p0 = math.exp(a) / (math.exp(a) + math.exp(b))
    assert np.allclose(O.prefill_scores(q, k), [1 + p0, 1 - p0], atol=1e-14)


def test_scores_equal_keys_harmonic():
    g, P, D = 2, 12, 4
    Q = _rng(1).standard_normal((g, P, D)); K = np.tile(_rng(2).standard_normal(D), (P, 1))
    want = [g * sum(1.0 / (i + 1) for i in range(j, P)) for j in range(P)]
    assert np.allclose(O.prefill_scores(Q, K), want, atol=1e-12)


def test_scores_bruteforce_loops():
    r = _rng(3)
    g, P, D = 2, 6, 3
    Q, K = r.standard_normal((g, P, D)), r.standard_normal((P, D))
    want = [0.0] * P
    for h in range(g):
        for i in range(P):
            logit = [sum(Q[h, i, d] * K[j, d] for d in range(D)) / math.sqrt(D) for j in range(i + 1)]
            z = sum(math.exp(x) for x in logit)
            for j in range(i + 1):
                want[j] += math.exp(logit[j]) / z
    assert np.allclose(O.prefill_scores(Q, K), want, atol=1e-13)


def test_row_lse_closed_forms_and_scores_from_it():
    """The softmax normalisers a fused attention kernel returns, and the column sums taken with them."""
    r = _rng(4)
    g, P, D = 2, 9, 4
    Q, K = r.standard_normal((g, P, D)), r.standard_normal((P, D))
    lse = O.prefill_row_lse(Q, K)
    # brute force: ln of the sum of exponentials, row by row, with plain loops
    for h in range(g):
        for i in range(P):
            logit = [sum(Q[h, i, d] * K[j, d] for d in range(D)) / math.sqrt(D) for j in range(i + 1)]
            assert abs(lse[h, i] - math.log(sum(math.exp(x) for x in logit))) < 1e-13
    # the first row attends to one key: its normaliser is that logit
    assert np.allclose(lse[:, 0], (Q[:, 0] * K[0]).sum(-1) / math.sqrt(D), atol=1e-14)
    # all keys equal: every logit of row i is the same s_i, so lse_i = s_i + ln(i + 1)
    Ke = np.tile(r.standard_normal(D), (P, 1))
    s_i = (Q @ Ke[0]) / math.sqrt(D)
    assert np.allclose(O.prefill_row_lse(Q, Ke), s_i + np.log(np.arange(1, P + 1)), atol=1e-13)
    # column sums taken with the true normalisers are the H2O prompt scores (pinned above on their own)
    assert np.allclose(O.prefill_scores_from_lse(Q, K, lse), O.prefill_scores(Q, K), atol=1e-12)
    # a normaliser that is too large by ln 2 halves every probability of that row: one row, by hand
    lse2 = lse.copy(); lse2[1, 5] += math.log(2.0)
    diff = O.prefill_scores(Q, K) - O.prefill_scores_from_lse(Q, K, lse2)
    row = np.exp((Q[1, 5] @ K[:6].T) / math.sqrt(D) - lse[1, 5])
    assert np.allclose(diff[:6], row / 2, atol=1e-13) and np.allclose(diff[6:], 0.0, atol=1e-15)


# ---------------- selection ----------------

@pytest.mark.parametrize("policy", O.POLICIES)
@pytest.mark.parametrize("seed", range(6))
def test_kept_sets_shape(policy, seed):
    r = _rng(10 + seed)
    n = int(r.integers(6, 80)); b = int(r.integers(5, 90))
    pos = np.sort(r.choice(500, size=n, replace=False)); pos[: min(4, n)] = np.arange(min(4, n))
    perm = r.permutation(n)
    score = r.random(n)
    keep = O.select_keep(pos[perm], score[perm], b, policy)
    kp = pos[perm][keep]
    assert len(keep) == min(n, b) and len(set(keep.tolist())) == len(keep)
    assert np.all(np.diff(kp) > 0)                              # ascending, unique
    if n <= b:
        assert sorted(kp.tolist()) == sorted(pos.tolist())
        return
    if policy == "sliding":
        assert kp.tolist() == pos[n - b:].tolist()
    if policy == "streaming":
        assert kp[:4].tolist() == [0, 1, 2, 3]                  # sinks never evicted
        assert kp[4:].tolist() == pos[n - (b - 4):].tolist()
    if policy == "h2o":
        hh, rec = b // 2, b - b // 2
        assert kp[-rec:].tolist() == pos[n - rec:].tolist()     # recent window kept
        older = [(float(-score[i]), int(pos[i])) for i in range(n - rec)]
        best = sorted(older)[:hh]
        assert sorted(kp[:hh].tolist()) == sorted(p for _, p in best)


def test_h2o_ties_keep_lowest_positions():
    pos = np.arange(20); score = np.full(20, 0.25)
    keep = O.select_keep(pos, score, 8, "h2o")
    assert pos[keep].tolist() == [0, 1, 2, 3, 16, 17, 18, 19]
    score[7] = 0.5
    assert pos[O.select_keep(pos, score, 8, "h2o")].tolist() == [0, 1, 2, 7, 16, 17, 18, 19]


def test_h2o_odd_budget_split():
    pos = np.arange(30); score = np.zeros(30); score[[2, 5, 9]] = [3, 2, 1]
    keep = O.select_keep(pos, score, 7, "h2o")                  # hh 3, recent 4
    assert pos[keep].tolist() == [2, 5, 9, 26, 27, 28, 29]


@pytest.mark.parametrize("policy", O.POLICIES)
def test_top_k_is_mergeable(policy):
    """Compressing the prompt at once, or token by token as it grows, ends in
    the same set (why compressing straight after prefill equals Algorithm 1's
    first compression inside the decode loop) -- scores held fixed."""
    r = _rng(42)
    n, b = 60, 13
    score = r.random(n)
    once = O.select_keep(np.arange(n), score, b, policy)
    cur = list(range(b))
    for t in range(b, n):
        cur = cur + [t]
        k = O.select_keep(np.array(cur), score[cur], b, policy)
        cur = [cur[i] for i in k]
    assert cur == once.tolist()


def test_streaming_sinks_are_positions_below_n_sink():
    """The sinks are the first n tokens of the sequence (Sec. 5.1), i.e. positions < n_sink -- not
    whatever happens to be oldest in the cache."""
    pos = np.array([0, 1, 4, 6, 7, 8, 9])
    assert pos[O.select_keep(pos, np.zeros(7), 5, "streaming")].tolist() == [0, 1, 7, 8, 9]
    assert pos[O.select_keep(pos, np.zeros(7), 5, "streaming", n_sink=1)].tolist() == [0, 6, 7, 8, 9]


def test_streaming_small_budget_and_short_prompt():
    assert O.select_keep(np.arange(10), np.zeros(10), 5, "streaming").tolist() == [0, 1, 2, 3, 9]
    assert O.select_keep(np.arange(3), np.zeros(3), 8, "streaming").tolist() == [0, 1, 2]
