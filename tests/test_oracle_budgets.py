"""Pins for the oracle's clustering and budget allocation (Algorithm 1 steps
5-11, Sec. 4.2.2, Appendix A.2 worked example)."""
import itertools
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import sqa_oracle as O

GOLD = os.path.join(os.path.dirname(__file__), "golden", "paper_budget_example.txt")


def _gold():
    d = {}
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        k, v = line.split()
        d[k] = float(v) if "." in v else int(v)
    return d


def _example_cos(n_imp, n_unimp, seed=0):
    r = np.random.default_rng(seed)
    n1 = 4
    cos = np.concatenate([0.40 + 0.05 * r.random(n1), 0.70 + 0.04 * r.random(n_imp - n1),
                          0.94 + 0.02 * r.random(n_unimp)]).astype(np.float32)
    perm = r.permutation(len(cos))
    return cos[perm]


def test_paper_worked_example():
    g = _gold()
    cos = _example_cos(g["n_important"], g["n_unimportant"])
    total = g["n_layer"] * g["b_init"]
    budget, group = O.allocate_budgets(cos, total, g["p"])
    unimp = [b for b, gr in zip(budget, group) if gr == 2]
    imp = [b for b, gr in zip(budget, group) if gr != 2]
    assert len(unimp) == g["n_unimportant"] and len(imp) == g["n_important"]
    assert set(unimp) == {g["b_unimportant"]}
    assert min(imp) == g["b_important"] and max(imp) - min(imp) <= 1
    assert sum(budget) == total                       # "the total budget remains unchanged"
    # the +1s go to the important layers with the lowest index
    imp_idx = [i for i, gr in enumerate(group) if gr != 2]
    r = total - g["n_unimportant"] * g["b_unimportant"] - g["n_important"] * g["b_important"]
    assert [budget[i] for i in imp_idx] == [g["b_important"] + 1] * r + [g["b_important"]] * (len(imp_idx) - r)


def test_g3_is_high_cosine_group_and_loses_budget():
    cos = _example_cos(18, 14, seed=3)
    budget, group = O.allocate_budgets(cos, 32 * 500, 0.4)
    hi = [c for c, gr in zip(cos, group) if gr == 2]
    lo = [c for c, gr in zip(cos, group) if gr != 2]
    assert min(hi) > max(lo)
    assert all(b == 200 for b, gr in zip(budget, group) if gr == 2)
    assert all(b > 500 for b, gr in zip(budget, group) if gr != 2)
    g1 = [c for c, gr in zip(cos, group) if gr == 0]
    g2 = [c for c, gr in zip(cos, group) if gr == 1]
    assert max(g1) < min(g2)


def test_p_equal_one_is_uniform():
    """Appendix A.2: p = 100 % leaves the cache structure unchanged."""
    cos = _example_cos(10, 6, seed=1)
    budget, _ = O.allocate_budgets(cos, 16 * 123, 1.0)
    assert budget == [123] * 16


@pytest.mark.parametrize("seed", range(20))
def test_sum_exact_and_shape_random(seed):
    r = np.random.default_rng(seed)
    L = int(r.integers(2, 60))
    cos = r.random(L).astype(np.float32)
    total = int(r.integers(L * 4, L * 5000))
    p = float(r.choice([0.1, 0.3, 0.35, 0.4, 0.7, 1.0]))
    budget, group = O.allocate_budgets(cos, total, p)
    assert sum(budget) == total
    low = {b for b, g in zip(budget, group) if g == 2}
    high = [b for b, g in zip(budget, group) if g != 2]
    assert len(low) <= 1 and max(high) - min(high) <= 1
    if low:
        assert low.pop() == int(np.floor(total * p / L))
        assert min(high) >= total // L


def _exact_sse(vals):
    n = len(vals)
    s = sum(vals)
    return sum((v - s / n) ** 2 for v in vals)


@pytest.mark.parametrize("seed", range(12))
def test_clustering_is_global_optimum_bruteforce(seed):
    """All 3^L assignments into 3 non-empty groups, exact rational SSE."""
    r = np.random.default_rng(100 + seed)
    L = int(r.integers(3, 9))
    cos = r.random(L).astype(np.float32)
    group, k = O.cluster_layers(cos)
    assert k == 3
    x = [Fraction(float(c)) for c in cos]
    best = None
    for assign in itertools.product(range(3), repeat=L):
        if len(set(assign)) < 3:
            continue
        cost = sum(_exact_sse([x[i] for i in range(L) if assign[i] == gid]) for gid in range(3))
        if best is None or cost < best[0]:
            best = (cost, assign)
    mine = sum(_exact_sse([x[i] for i in range(L) if group[i] == gid]) for gid in range(3))
    assert mine == best[0]
    # same partition (labels ordered by mean)
    parts = lambda a: sorted(tuple(i for i in range(L) if a[i] == gid) for gid in range(3))
    assert parts(group) == parts(best[1])
    means = [np.mean([cos[i] for i in range(L) if group[i] == gid]) for gid in range(3)]
    assert means[0] < means[1] < means[2]


def test_lloyd_fixed_point():
    cos = _example_cos(20, 12, seed=5)
    group, _ = O.cluster_layers(cos)
    cent = [np.mean([float(c) for c, g in zip(cos, group) if g == gid]) for gid in range(3)]
    again = [int(np.argmin([abs(float(c) - m) for m in cent])) for c in cos]
    assert again == group


def test_layer_permutation_permutes_groups():
    cos = _example_cos(12, 9, seed=6)
    group, _ = O.cluster_layers(cos)
    perm = np.random.default_rng(7).permutation(len(cos))
    group_p, _ = O.cluster_layers(cos[perm])
    assert group_p == [group[i] for i in perm]


def test_degenerate_distinct_value_counts():
    assert O.allocate_budgets(np.full(5, 0.9, np.float32), 103, 0.3)[0] == [21, 21, 21, 20, 20]
    budget, group = O.allocate_budgets(np.array([0.5, 0.9, 0.5, 0.9], np.float32), 400, 0.5)
    assert group == [1, 2, 1, 2] and budget == [150, 50, 150, 50]
    # ties in value never split: equal values share a group
    cos = np.array([0.2, 0.2, 0.5, 0.5, 0.9, 0.9, 0.9], np.float32)
    group, k = O.cluster_layers(cos)
    assert k == 3 and group == [0, 0, 1, 1, 2, 2, 2]


def test_tie_between_partitions_takes_smallest_cuts():
    # 0,1,2,3 evenly spaced: {0|1|2,3}, {0|1,2|3}, {0,1|2|3} all cost 0.5
    group, _ = O.cluster_layers(np.array([0.0, 1.0, 2.0, 3.0], np.float32))
    assert group == [0, 1, 2, 2]


def test_errors():
    cos = np.array([0.1, 0.5, 0.9], np.float32)
    for total, p in [(2, 0.3), (30, 0.0), (30, 1.5), (3, 0.3)]:
        with pytest.raises(ValueError):
            O.allocate_budgets(cos, total, p)
