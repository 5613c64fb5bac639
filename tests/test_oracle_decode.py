"""Pins for the oracle's decode step (Algorithm 1 steps 14-21, Eq. 2-3) and
prefill compression (step 12 + 16-17)."""
import math

import numpy as np
import pytest

from oracle import sqa_oracle as O


def _rng(s):
    return np.random.default_rng(s)


def _full_attention_loops(q, K, V):
    """Textbook softmax(q K^T / sqrt(D)) V, plain Python loops."""
    D = len(q)
    logit = [sum(q[d] * K[j][d] for d in range(D)) / math.sqrt(D) for j in range(len(K))]
    m = max(logit)
    w = [math.exp(x - m) for x in logit]
    z = sum(w)
    return [sum(w[j] * V[j][d] for j in range(len(K))) / z for d in range(D)], [x / z for x in w]


def _run(policy, b, P, S, g, D, seed, n_sink=4, score0=None):
    r = _rng(seed)
    K, V = r.standard_normal((P + S, D)), r.standard_normal((P + S, D))
    q = r.standard_normal((S, g, D))
    score = r.random(P) if score0 is None else score0
    c = O.prefill_compress(K[:P], V[:P], score, b, policy, n_sink)
    outs = []
    for t in range(S):
        out, c = O.decode_step(c, q[t], K[P + t], V[P + t], P + t, b, policy, n_sink)
        outs.append((out, c))
    return K, V, q, outs


@pytest.mark.parametrize("policy", O.POLICIES)
def test_budget_at_least_length_is_full_attention(policy):
    P, S, g, D = 9, 5, 2, 4
    K, V, q, outs = _run(policy, P + S, P, S, g, D, seed=1)
    for t, (out, c) in enumerate(outs):
        assert c["pos"].tolist() == list(range(P + t + 1))
        for h in range(g):
            want, _ = _full_attention_loops(q[t, h], K[: P + t + 1], V[: P + t + 1])
            assert np.allclose(out[h], want, atol=1e-13)


def test_sliding_equals_full_attention_over_last_b():
    P, S, g, D, b = 20, 8, 1, 4, 6
    K, V, q, outs = _run("sliding", b, P, S, g, D, seed=2)
    for t, (out, c) in enumerate(outs):
        n = P + t + 1
        assert c["pos"].tolist() == list(range(n - b, n))
        want, _ = _full_attention_loops(q[t, 0], K[n - b:n], V[n - b:n])
        assert np.allclose(out[0], want, atol=1e-13)


def test_streaming_keeps_sinks_and_window():
    P, S, g, D, b = 20, 8, 2, 4, 9
    K, V, q, outs = _run("streaming", b, P, S, g, D, seed=3)
    for t, (out, c) in enumerate(outs):
        n = P + t + 1
        idx = [0, 1, 2, 3] + list(range(n - 5, n))
        assert c["pos"].tolist() == idx
        for h in range(g):
            want, _ = _full_attention_loops(q[t, h], K[idx], V[idx])
            assert np.allclose(out[h], want, atol=1e-13)


@pytest.mark.parametrize("policy", O.POLICIES)
def test_equal_values_give_that_value(policy):
    r = _rng(4)
    P, S, D, b = 16, 6, 8, 7
    v0 = r.standard_normal(D)
    c = O.prefill_compress(r.standard_normal((P, D)), np.tile(v0, (P, 1)), r.random(P), b, policy)
    for t in range(S):
        out, c = O.decode_step(c, r.standard_normal((2, D)), r.standard_normal(D), v0, P + t, b, policy)
        assert np.allclose(out, v0, atol=1e-13)
        assert len(c["pos"]) == b


def test_zero_query_is_mean_and_scores_gain_g_over_n():
    r = _rng(5)
    P, D, b, g = 12, 4, 8, 3
    c = O.prefill_compress(r.standard_normal((P, D)), r.standard_normal((P, D)), r.random(P), b, "h2o")
    before = None
    out, c2 = O.decode_step(c, np.zeros((g, D)), r.standard_normal(D), r.standard_normal(D), P, b, "h2o")
    assert np.allclose(out, c2["V"].mean(axis=0), atol=1e-14)
    # every kept token gained exactly g / n
    old = dict(zip(c["pos"].tolist(), c["score"].tolist())); old[P] = 0.0
    for ps, sc in zip(c2["pos"].tolist(), c2["score"].tolist()):
        assert abs(sc - old[ps] - g / b) < 1e-14


def test_h2o_mass_conservation_and_eviction_rule():
    """Kept + evicted accumulated score = (prompt mass) + g per decode step;
    each eviction removes the worst non-recent token by (score, -position)."""
    r = _rng(6)
    P, S, D, b, g = 24, 10, 4, 9, 2
    K, V = r.standard_normal((P + S, D)), r.standard_normal((P + S, D))
    Qp = r.standard_normal((g, P, D))
    s0 = O.prefill_scores(Qp, K[:P])
    c = O.prefill_compress(K[:P], V[:P], s0, b, "h2o")
    evicted = s0.sum() - c["score"].sum()
    hh, rec = b // 2, b - b // 2
    for t in range(S):
        prev = dict(zip(c["pos"].tolist(), c["score"].tolist()))
        out, c = O.decode_step(c, r.standard_normal((g, D)), K[P + t], V[P + t], P + t, b, "h2o")
        gone = set(prev) - set(c["pos"].tolist())
        assert len(gone) == 1 and len(c["pos"]) == b
        victim = gone.pop()
        cand = sorted(prev)[: len(prev) + 1 - rec]          # non-recent after the append
        worst = min(cand, key=lambda ps: (prev[ps], -ps))
        assert victim == worst
        evicted += prev[victim]
        assert abs(c["score"].sum() + evicted - g * (P + t + 1)) < 1e-10
        assert c["pos"][-rec:].tolist() == list(range(P + t + 1 - rec, P + t + 1))


def test_prefill_compress_then_decode_equals_late_first_compression():
    """Algorithm 1 caches the whole prompt (step 12) and compresses inside the
    decode loop; compressing right after prefill gives the same first step."""
    r = _rng(7)
    P, D, b, g = 30, 4, 11, 2
    K, V = r.standard_normal((P + 1, D)), r.standard_normal((P + 1, D))
    q = r.standard_normal((g, D)); s0 = r.random(P)
    for policy in O.POLICIES:
        early = O.prefill_compress(K[:P], V[:P], s0, b, policy)
        o1, c1 = O.decode_step(early, q, K[P], V[P], P, b, policy)
        late = O.new_cache(K[:P], V[:P], s0)
        o2, c2 = O.decode_step(late, q, K[P], V[P], P, b, policy)
        assert c1["pos"].tolist() == c2["pos"].tolist()
        assert np.allclose(o1, o2, atol=1e-15) and np.allclose(c1["score"], c2["score"], atol=1e-15)


def test_probabilities_match_loop_softmax():
    r = _rng(8)
    K, V, q = r.standard_normal((7, 5)), r.standard_normal((7, 5)), r.standard_normal((1, 5))
    out, prob = O.attend(q, K, V)
    want_out, want_p = _full_attention_loops(q[0], K, V)
    assert np.allclose(out[0], want_out, atol=1e-14) and np.allclose(prob[0], want_p, atol=1e-15)


# -- the attend-then-evict variant ---------------------------------------------------

AE = "attend_then_evict"


@pytest.mark.parametrize("policy", O.POLICIES)
def test_orders_agree_while_nothing_is_evicted(policy):
    r = _rng(20)
    P, S, g, D = 7, 4, 2, 4
    K, V, q = r.standard_normal((P + S, D)), r.standard_normal((P + S, D)), r.standard_normal((S, g, D))
    a = O.prefill_compress(K[:P], V[:P], r.random(P), P + S, policy)
    b = {k: v.copy() for k, v in a.items()}
    for t in range(S):
        oa, a = O.decode_step(a, q[t], K[P + t], V[P + t], P + t, P + S, policy)
        ob, b = O.decode_step(b, q[t], K[P + t], V[P + t], P + t, P + S, policy, order=AE)
        assert np.array_equal(oa, ob) and np.array_equal(a["score"], b["score"]) and a["pos"].tolist() == b["pos"].tolist()


def test_attend_then_evict_sliding_sees_one_more_token():
    P, S, D, b = 15, 6, 4, 5
    r = _rng(21)
    K, V, q = r.standard_normal((P + S, D)), r.standard_normal((P + S, D)), r.standard_normal((S, 1, D))
    c = O.prefill_compress(K[:P], V[:P], np.zeros(P), b, "sliding")
    for t in range(S):
        n = P + t + 1
        out, c = O.decode_step(c, q[t], K[P + t], V[P + t], P + t, b, "sliding", order=AE)
        want, _ = _full_attention_loops(q[t, 0], K[n - b - 1:n], V[n - b - 1:n])     # b kept + the new one
        assert np.allclose(out[0], want, atol=1e-13)
        assert c["pos"].tolist() == list(range(n - b, n))


def test_attend_then_evict_streaming_kept_sets():
    P, S, D, b = 20, 5, 4, 9
    r = _rng(22)
    K, V, q = r.standard_normal((P + S, D)), r.standard_normal((P + S, D)), r.standard_normal((S, 2, D))
    c = O.prefill_compress(K[:P], V[:P], np.zeros(P), b, "streaming")
    for t in range(S):
        n = P + t + 1
        out, c = O.decode_step(c, q[t], K[P + t], V[P + t], P + t, b, "streaming", order=AE)
        seen = [0, 1, 2, 3] + list(range(n - 6, n))
        for h in range(2):
            want, _ = _full_attention_loops(q[t, h], K[seen], V[seen])
            assert np.allclose(out[h], want, atol=1e-13)
        assert c["pos"].tolist() == [0, 1, 2, 3] + list(range(n - 5, n))


def test_attend_then_evict_h2o_uses_the_updated_scores():
    """The victim is the worst non-recent token by the scores AFTER this step's
    probabilities (recomputed here with the loop softmax) were added; the mass
    kept + evicted grows by g per step."""
    r = _rng(23)
    P, S, D, b, g = 18, 9, 4, 8, 2
    K, V = r.standard_normal((P + S, D)), r.standard_normal((P + S, D))
    s0 = r.random(P)
    c = O.prefill_compress(K[:P], V[:P], s0, b, "h2o")
    hh, rec = b // 2, b - b // 2
    evicted = s0.sum() - c["score"].sum()
    for t in range(S):
        q = r.standard_normal((g, D))
        ps = c["pos"].tolist() + [P + t]
        upd = dict(zip(ps, c["score"].tolist() + [0.0]))
        for h in range(g):
            _, pr = _full_attention_loops(q[h], K[ps], V[ps])
            for x, w in zip(ps, pr):
                upd[x] += w
        out, c = O.decode_step(c, q, K[P + t], V[P + t], P + t, b, "h2o", order=AE)
        gone = set(ps) - set(c["pos"].tolist())
        assert len(gone) == 1
        victim = gone.pop()
        cand = sorted(ps)[: len(ps) - rec]
        assert victim == min(cand, key=lambda x: (upd[x], -x))
        evicted += upd[victim]
        assert abs(c["score"].sum() + evicted - (s0.sum() + g * (t + 1))) < 1e-10
        for x, sc in zip(c["pos"].tolist(), c["score"].tolist()):
            assert abs(sc - upd[x]) < 1e-13


def test_unknown_order_is_rejected():
    c = O.new_cache(np.zeros((2, 4)), np.zeros((2, 4)))
    with pytest.raises(ValueError):
        O.decode_step(c, np.zeros((1, 4)), np.zeros(4), np.zeros(4), 2, 4, "sliding", order="evict_first")
