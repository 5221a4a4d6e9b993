"""Pins for the oracle's routing: brute force, closed forms, library routines,
exact-arithmetic inputs.  None of these re-types the oracle's own loops."""
import itertools
from fractions import Fraction

import numpy as np
import pytest
import scipy.special

import oracle


def _brute_topk(keys, k, eligible=None):
    """All C(E,k) subsets: max sum of keys, ties -> lexicographically smallest
    sorted id tuple; returned in (-key, id) order."""
    E = len(keys)
    cand = [e for e in range(E) if eligible is None or eligible[e]]
    best, best_sum = None, None
    for sub in itertools.combinations(cand, k):      # lexicographic order
        s = sum(Fraction(float(keys[e])) for e in sub)
        if best is None or s > best_sum:
            best, best_sum = sub, s
    return sorted(best, key=lambda e: (-keys[e], e))


def _brute_groups(keys, G, Kg, n_top):
    E = len(keys)
    gs = E // G
    gscore = []
    for g in range(G):
        srt = sorted((Fraction(float(v)) for v in keys[g * gs:(g + 1) * gs]), reverse=True)
        gscore.append(sum(srt[:n_top]))
    best, best_sum = None, None
    for sub in itertools.combinations(range(G), Kg):
        s = sum(gscore[g] for g in sub)
        if best is None or s > best_sum:
            best, best_sum = sub, s
    elig = np.zeros(E, bool)
    for g in best:
        elig[g * gs:(g + 1) * gs] = True
    return elig


@pytest.mark.parametrize("E,k", [(5, 1), (8, 2), (12, 4), (9, 9), (12, 6)])
def test_topk_brute_force_softmax(E, k):
    rng = np.random.default_rng(E * 100 + k)
    logits = rng.standard_normal((40, E)).astype(np.float32)
    gw = np.zeros((E, 4), np.float32)
    ids, w, margin = oracle.route(None, gw, k, "softmax", logits_in=logits)
    for t in range(logits.shape[0]):
        assert list(ids[t]) == _brute_topk(logits[t].astype(np.float64), k)
    assert np.all(margin > 0)


def test_topk_exact_ties_lowest_index():
    # keys drawn from 3 distinct values: many exact ties
    rng = np.random.default_rng(7)
    logits = rng.integers(0, 3, size=(60, 10)).astype(np.float32)
    gw = np.zeros((10, 4), np.float32)
    for k in (1, 3, 5):
        ids, w, margin = oracle.route(None, gw, k, "softmax", logits_in=logits)
        for t in range(60):
            assert list(ids[t]) == _brute_topk(logits[t].astype(np.float64), k)
    assert margin.min() == 0.0


def test_softmax_weights_closed_form():
    # renormalised top-k softmax weights == softmax over the selected logits
    rng = np.random.default_rng(3)
    logits = (3 * rng.standard_normal((50, 16))).astype(np.float32)
    gw = np.zeros((16, 4), np.float32)
    ids, w, _ = oracle.route(None, gw, 4, "softmax", logits_in=logits)
    sel = np.take_along_axis(logits.astype(np.float64), ids, axis=1)
    ref = scipy.special.softmax(sel, axis=1)
    np.testing.assert_allclose(w, ref, rtol=2e-7)
    np.testing.assert_allclose(w.sum(1), 1.0, atol=3e-7)
    # without renormalisation: the plain softmax probability, times the scale
    ids2, w2, _ = oracle.route(None, gw, 4, "softmax", renormalize=False, routed_scale=3.0,
                               logits_in=logits)
    assert np.array_equal(ids, ids2)
    full = scipy.special.softmax(logits.astype(np.float64), axis=1)
    np.testing.assert_allclose(w2, 3.0 * np.take_along_axis(full, ids, axis=1), rtol=2e-7)


def test_logit_bias_moves_selection_and_weights():
    logits = np.zeros((1, 6), np.float32)
    gw = np.zeros((6, 4), np.float32)
    lb = np.array([0, 0, 5, 0, 1, 0], np.float32)
    ids, w, _ = oracle.route(None, gw, 2, "softmax", logits_in=logits, logit_bias=lb)
    assert list(ids[0]) == [2, 4]
    ref = scipy.special.softmax(np.array([5.0, 1.0]))
    np.testing.assert_allclose(w[0], ref, rtol=2e-7)


def test_gate_dot_product_exact_integers():
    # small integers: the gate logits are exact integers in any order of summation
    rng = np.random.default_rng(11)
    x = rng.integers(-4, 5, size=(9, 32)).astype(np.float32)
    gw = rng.integers(-4, 5, size=(7, 32)).astype(np.float32)
    _, _, _, z = oracle.route(x, gw, 2, "softmax", return_logits=True)
    ref = np.array([[sum(int(a) * int(b) for a, b in zip(x[t], gw[e])) for e in range(7)]
                    for t in range(9)], dtype=np.float64)
    assert np.array_equal(z, ref)          # catches a transposed or mis-indexed operand
    # and the matmul special case on non-square float inputs
    xf = rng.standard_normal((5, 48)).astype(np.float32)
    gf = rng.standard_normal((11, 48)).astype(np.float32)
    _, _, _, z = oracle.route(xf, gf, 3, "softmax", return_logits=True)
    np.testing.assert_allclose(z, xf.astype(np.float64) @ gf.astype(np.float64).T, rtol=1e-12, atol=1e-13)


def test_sigmoid_plain_topk_and_weights():
    rng = np.random.default_rng(5)
    logits = rng.standard_normal((40, 12)).astype(np.float32)
    gw = np.zeros((12, 4), np.float32)
    sb = (0.3 * rng.standard_normal(12)).astype(np.float32)
    ids, w, _ = oracle.route(None, gw, 3, "sigmoid", routed_scale=2.5, logits_in=logits,
                             select_bias=sb)
    s = scipy.special.expit(logits.astype(np.float64))
    keys = s + sb.astype(np.float64)
    for t in range(40):
        assert list(ids[t]) == _brute_topk(keys[t], 3)
    sel = np.take_along_axis(s, ids, axis=1)          # weights use the un-biased score
    np.testing.assert_allclose(w, 2.5 * sel / sel.sum(1, keepdims=True), rtol=3e-7)
    np.testing.assert_allclose(w.sum(1), 2.5, rtol=3e-7)
    # no renormalisation: the raw score times the scale
    _, w2, _ = oracle.route(None, gw, 3, "sigmoid", renormalize=False, routed_scale=2.0,
                            logits_in=logits, select_bias=sb)
    np.testing.assert_allclose(w2, 2.0 * sel, rtol=3e-7)


def test_select_bias_changes_selection_not_weights():
    logits = np.array([[2.0, 1.0, 0.0, -1.0]], np.float32)
    gw = np.zeros((4, 4), np.float32)
    ids0, w0, _ = oracle.route(None, gw, 2, "sigmoid", logits_in=logits)
    assert list(ids0[0]) == [0, 1]
    sb = np.array([0, 0, 0, 5], np.float32)           # pushes expert 3 in, first
    ids1, w1, _ = oracle.route(None, gw, 2, "sigmoid", logits_in=logits, select_bias=sb)
    assert list(ids1[0]) == [3, 0]
    s = scipy.special.expit(np.array([-1.0, 2.0]))
    np.testing.assert_allclose(w1[0], s / s.sum(), rtol=3e-7)
    # a bias that leaves the set unchanged leaves the weights unchanged
    sb2 = np.array([0.01, 0.0, 0.0, 0.0], np.float32)
    ids2, w2, _ = oracle.route(None, gw, 2, "sigmoid", logits_in=logits, select_bias=sb2)
    assert np.array_equal(ids2, ids0) and np.array_equal(w2, w0)


@pytest.mark.parametrize("E,G,Kg,k,n_top", [(8, 4, 2, 2, 2), (12, 3, 2, 3, 2), (16, 4, 2, 4, 1),
                                             (16, 8, 4, 4, 2)])
def test_group_limited_brute_force(E, G, Kg, k, n_top):
    rng = np.random.default_rng(E + G + Kg)
    logits = rng.standard_normal((60, E)).astype(np.float32)
    sb = (0.2 * rng.standard_normal(E)).astype(np.float32)
    gw = np.zeros((E, 4), np.float32)
    ids, w, margin = oracle.route(None, gw, k, "sigmoid", logits_in=logits, select_bias=sb,
                                  n_groups=G, topk_groups=Kg, group_score_n=n_top)
    keys = scipy.special.expit(logits.astype(np.float64)) + sb.astype(np.float64)
    for t in range(60):
        elig = _brute_groups(keys[t], G, Kg, n_top)
        assert list(ids[t]) == _brute_topk(keys[t], k, elig)


def test_group_limit_reductions_and_negative_keys():
    rng = np.random.default_rng(2)
    logits = rng.standard_normal((30, 16)).astype(np.float32)
    gw = np.zeros((16, 4), np.float32)
    sb = np.full(16, -3.0, np.float32)                # every key negative
    plain = oracle.route(None, gw, 4, "sigmoid", logits_in=logits, select_bias=sb)
    allg = oracle.route(None, gw, 4, "sigmoid", logits_in=logits, select_bias=sb,
                        n_groups=4, topk_groups=4, group_score_n=2)
    oneg = oracle.route(None, gw, 4, "sigmoid", logits_in=logits, select_bias=sb,
                        n_groups=1, topk_groups=1, group_score_n=0)
    for a, b in zip(plain[:2], allg[:2]):
        assert np.array_equal(a, b)
    for a, b in zip(plain[:2], oneg[:2]):
        assert np.array_equal(a, b)
    # ineligible experts are excluded by index: with negative keys a dropped
    # group must still never be picked
    ids, _, _ = oracle.route(None, gw, 4, "sigmoid", logits_in=logits, select_bias=sb,
                             n_groups=4, topk_groups=2, group_score_n=2)
    keys = scipy.special.expit(logits.astype(np.float64)) - 3.0
    for t in range(30):
        elig = _brute_groups(keys[t], 4, 2, 2)
        assert all(elig[e] for e in ids[t])


def test_group_ties_lowest_group():
    logits = np.zeros((1, 8), np.float32)             # all groups tie
    gw = np.zeros((8, 4), np.float32)
    ids, _, margin = oracle.route(None, gw, 2, "sigmoid", logits_in=logits, n_groups=4,
                                  topk_groups=2, group_score_n=2)
    assert list(ids[0]) == [0, 1] and margin[0] == 0.0


def test_margin_is_smallest_decisive_gap():
    logits = np.array([[5.0, 3.0, 2.5, 0.0]], np.float32)
    gw = np.zeros((4, 4), np.float32)
    _, _, m = oracle.route(None, gw, 2, "softmax", logits_in=logits)
    assert m[0] == 0.5                                # cut between 3.0 and 2.5
    _, _, m = oracle.route(None, gw, 3, "softmax", logits_in=logits)
    assert m[0] == 0.5                                # order of 3.0 / 2.5


def test_counts_sum_and_determinism():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((100, 64)).astype(np.float32)
    gw = rng.standard_normal((16, 64)).astype(np.float32)
    a = oracle.route(x, gw, 4)
    b = oracle.route(x, gw, 4)
    assert all(np.array_equal(p, q) for p, q in zip(a, b))
    ids = a[0]
    assert np.bincount(ids.ravel(), minlength=16).sum() == 100 * 4
    assert all(len(set(r)) == 4 for r in ids)
