"""Pins for the oracle's gate: projection, softmax, top-k, weights, capacity.

Each check is against something other than the oracle's own formula: a scipy
routine, a closed form, brute force with Python's sort, or an invariant.
"""
import math

import numpy as np
import pytest
from scipy.special import expit, softmax as scipy_softmax

from oracle import moe_oracle as O
from paper_2109_10465_amd import inputs as I


def rng(s):
    return np.random.default_rng(s)


def test_gate_logits_matches_python_loops():
    r = rng(1)
    x, Wg, b = r.standard_normal((5, 7)), r.standard_normal((7, 3)), r.standard_normal(3)
    got = O.gate_logits(x, Wg, b)
    for t in range(5):
        for e in range(3):
            want = math.fsum(x[t, i] * Wg[i, e] for i in range(7)) + b[e]
            assert got[t, e] == pytest.approx(want, rel=1e-13, abs=1e-13)
    assert np.array_equal(O.gate_logits(x, Wg), got - b[None, :]) or np.allclose(
        O.gate_logits(x, Wg), got - b[None, :], rtol=1e-13)


def test_softmax_rows_sum_to_one_and_match_scipy():
    l = rng(2).standard_normal((64, 17)) * 5
    p = O.softmax(l)
    assert np.all(np.abs(p.sum(axis=1) - 1.0) <= 1e-12)
    assert np.all(p > 0)
    np.testing.assert_allclose(p, scipy_softmax(l, axis=1), rtol=1e-12)


def test_softmax_shift_invariant_and_stable_for_huge_logits():
    l = rng(3).standard_normal((8, 5))
    np.testing.assert_allclose(O.softmax(l + 1000.0), O.softmax(l), rtol=1e-10)
    big = np.array([[1e4, 1e4 - 1.0, -1e4]])
    p = O.softmax(big)
    assert np.isfinite(p).all()
    assert p[0, 0] == pytest.approx(1 / (1 + math.exp(-1.0)), rel=1e-12)


def test_softmax_single_expert_and_two_expert_closed_form():
    assert np.array_equal(O.softmax(rng(4).standard_normal((9, 1))), np.ones((9, 1)))
    l = rng(5).standard_normal((32, 2))
    np.testing.assert_allclose(O.softmax(l)[:, 0], expit(l[:, 0] - l[:, 1]), rtol=1e-12)


@pytest.mark.parametrize("k", [1, 2])
def test_top_k_matches_full_sort(k):
    r = rng(6)
    # few distinct values -> plenty of ties
    l = r.integers(-2, 3, size=(200, 6)).astype(np.float32)
    got = O.top_k(l, k)
    for t in range(l.shape[0]):
        order = sorted(range(l.shape[1]), key=lambda e: (-float(l[t, e]), e))
        assert list(got[t]) == order[:k]


def test_top_k_order_and_distinct():
    l = rng(7).standard_normal((500, 9)).astype(np.float32)
    idx = O.top_k(l, 2)
    rows = np.arange(500)
    assert np.all(idx[:, 0] != idx[:, 1])
    l0, l1 = l[rows, idx[:, 0]], l[rows, idx[:, 1]]
    assert np.all(l0 >= l1)
    masked = l.copy()
    masked[rows, idx[:, 0]] = -np.inf
    masked[rows, idx[:, 1]] = -np.inf
    assert np.all(l1 >= masked.max(axis=1))


def test_top_k_signed_zero_is_a_tie():
    l = np.array([[-0.0, 0.0, -1.0], [0.0, -0.0, -1.0]], np.float32)
    assert O.top_k(l, 2).tolist() == [[0, 1], [0, 1]]


def test_gate_weights_invariants_and_closed_form():
    l = rng(8).standard_normal((300, 8)).astype(np.float32)
    p = O.softmax(l)
    i1 = O.top_k(l, 1)
    g1 = O.gate_weights(p, i1)
    assert g1.shape == (300, 1) and np.all(g1 >= 1.0 / 8)
    np.testing.assert_allclose(g1[:, 0], p.max(axis=1), rtol=0)
    i2 = O.top_k(l, 2)
    g2 = O.gate_weights(p, i2)
    np.testing.assert_allclose(g2.sum(axis=1), 1.0, rtol=1e-13)
    assert np.all(g2[:, 0] >= g2[:, 1])
    # two renormalised softmax probabilities = a sigmoid of the logit difference
    rows = np.arange(300)
    la, lb = l[rows, i2[:, 0]].astype(np.float64), l[rows, i2[:, 1]].astype(np.float64)
    np.testing.assert_allclose(g2[:, 0], expit(la - lb), rtol=1e-12)


def test_capacity_matches_the_workloads_stated_slots():
    # top-1, capacity factor 1.0: capacity = T / E (64 and 256 are stated)
    assert O.capacity(256, 4, 1, 1.0) == 64
    assert O.capacity(32768, 128, 1, 1.0) == 256
    for w in I.WORKLOADS.values():
        assert O.capacity(w.T, w.E, w.k, w.capacity_factor) == w.capacity
    assert O.capacity(10, 4, 1, 1.0) == 3          # ceil
    assert O.capacity(1, 64, 1, 1.0) == 1          # floor of one slot
    assert O.capacity(100, 8, 2, 2.0) == 50
