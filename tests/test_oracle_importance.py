"""Pins for the oracle's layer-importance probe (Sec. 3 cosine equation;
Algorithm 1 steps 1-4).  None of these re-types the oracle's formula: they are
closed forms, invariances and an independently ordered exact summation."""
import math
from fractions import Fraction

import numpy as np
import pytest

from oracle import sqa_oracle as O


def _rng(seed):
    return np.random.default_rng(seed)


def test_identical_rows_give_one_and_negated_minus_one():
    A = _rng(0).standard_normal((7, 33))
    assert np.allclose(O.token_cosines(A, A), 1.0, rtol=0, atol=1e-15)
    assert np.allclose(O.token_cosines(A, -A), -1.0, rtol=0, atol=1e-15)


def test_orthogonal_rows_give_zero_and_axis_angles():
    A = np.array([[1.0, 0, 0], [2.0, 0, 0], [1.0, 1.0, 0]])
    B = np.array([[0, 5.0, 0], [2.0, 2.0, 0], [1.0, 0, 0]])
    c = O.token_cosines(A, B)
    assert c[0] == 0.0
    assert abs(c[1] - math.cos(math.pi / 4)) < 1e-15
    assert abs(c[2] - math.cos(math.pi / 4)) < 1e-15


def test_positive_scaling_invariance_and_sign():
    r = _rng(1)
    A, B = r.standard_normal((5, 64)), r.standard_normal((5, 64))
    c = O.token_cosines(A, B)
    assert np.allclose(O.token_cosines(3.5 * A, 0.01 * B), c, atol=1e-14)
    assert np.allclose(O.token_cosines(-A, B), -c, atol=1e-14)
    assert np.allclose(O.token_cosines(B, A), c, atol=1e-15)       # symmetric


def test_zero_row_contributes_zero():
    A = np.zeros((2, 8)); B = np.ones((2, 8)); A[1] = 1.0
    c = O.token_cosines(A, B)
    assert c[0] == 0.0 and abs(c[1] - 1.0) < 1e-15


def test_exact_rational_arithmetic_agrees():
    """Small-integer rows: the cosine squared is an exact rational."""
    r = _rng(2)
    A = r.integers(-9, 10, size=(6, 11)); B = r.integers(-9, 10, size=(6, 11))
    c = O.token_cosines(A, B)
    for j in range(6):
        ab = sum(Fraction(int(a)) * int(b) for a, b in zip(A[j], B[j]))
        aa = sum(Fraction(int(a)) ** 2 for a in A[j]); bb = sum(Fraction(int(b)) ** 2 for b in B[j])
        ref2 = ab * ab / (aa * bb)
        assert abs(c[j] * c[j] - float(ref2)) < 1e-14
        assert (c[j] >= 0) == (ab >= 0)


def test_layer_mean_is_mean_over_all_tokens():
    r = _rng(3)
    h_in = r.standard_normal((3, 10, 16)); h_out = r.standard_normal((3, 10, 16))
    cos = O.layer_importance(h_in, h_out)
    for l in range(3):
        tot = 0.0
        for j in range(10):                       # reversed order, plain loop
            tot += O.token_cosines(h_in[l, 9 - j:10 - j], h_out[l, 9 - j:10 - j])[0]
        assert abs(cos[l] - tot / 10) < 1e-14


@pytest.mark.parametrize("a", [2.0, 0.3, 1.5])
def test_additive_noise_closed_form(a):
    """B = A + a*N(0,I): E[cos] -> 1/sqrt(1+a^2) (configs[0] uses a = 2, .3, .3, 1.5)."""
    r = _rng(4)
    T, d = 512, 1024
    A = r.standard_normal((1, T, d)); B = A + a * r.standard_normal((1, T, d))
    cos = O.layer_importance(A, B)[0]
    assert abs(cos - 1.0 / math.sqrt(1 + a * a)) < 4.0 / math.sqrt(T * d) + 1.0 / d


def test_tiny_workload_pattern():
    from paper_2404_04793_amd import workloads as W
    wl = W.WORKLOADS["tiny"]
    h = [W.hidden_states(wl, l) for l in range(wl.L)]
    cos = O.layer_importance([x[0].double().numpy() for x in h], [x[1].double().numpy() for x in h])
    want = [0.4472, 0.9578, 0.9578, 0.5547]
    assert np.allclose(cos, want, atol=5e-3)
