"""Pins for oracle.topk_gate (Section 2.1: sparse top-k router, Mixtral top-2).

The paper prints no worked example, so the oracle is pinned by: a brute-force
selection written as the definition (repeated scan for the best remaining
expert), crafted ties, library special cases (k=1 = first-max argmax, k=E =
full softmax), the closed form of a two-way softmax (logistic of the logit
gap) and invariants.  A few deliberately wrong variants are checked to fail
those pins, so the pins are known to have teeth.
"""
import math

import numpy as np
import pytest
import scipy.special

from oracle import moe_oracle as O


def brute_gate(logits, k):
    T, E = logits.shape
    idx = np.zeros((T, k), dtype=np.int32)
    w = np.zeros((T, k))
    for t in range(T):
        taken = []
        for j in range(k):
            best = None
            for e in range(E):
                if e in taken:
                    continue
                if best is None or float(logits[t, e]) > float(logits[t, best]):
                    best = e        # strict '>' keeps the lowest index among equals
            taken.append(best)
        z = [math.exp(float(logits[t, e]) - float(logits[t, taken[0]])) for e in taken]
        s = 0.0
        for v in z:
            s += v
        idx[t] = taken
        w[t] = [v / s for v in z]
    return idx, w


def rand_logits(seed, T, E, quant=None):
    rng = np.random.default_rng(seed)
    lg = rng.standard_normal((T, E)).astype(np.float32) * 2
    if quant:                       # coarse grid -> many exact ties
        lg = (np.round(lg * quant) / quant).astype(np.float32)
    return lg


@pytest.mark.parametrize("T,E,k,quant", [(37, 8, 2, None), (50, 8, 2, 2), (19, 64, 6, 1),
                                         (11, 5, 5, 1), (13, 3, 1, 1), (7, 130, 4, 2)])
def test_matches_brute_force(T, E, k, quant):
    lg = rand_logits(100 + E + k, T, E, quant)
    idx, w = O.topk_gate(lg, k)
    bidx, bw = brute_gate(lg, k)
    assert idx.dtype == np.int32
    np.testing.assert_array_equal(idx, bidx)
    np.testing.assert_allclose(w, bw, rtol=1e-14, atol=0)


def test_crafted_ties_go_to_lower_index_and_signed_zero_is_a_tie():
    lg = np.array([[1.0, 3.0, 3.0, 3.0, 0.0],
                   [0.0, -0.0, 0.0, -1.0, -0.0],
                   [-0.0, 0.0, -5.0, -5.0, -5.0],
                   [2.0, 2.0, 2.0, 2.0, 2.0]], dtype=np.float32)
    idx, w = O.topk_gate(lg, 3)
    np.testing.assert_array_equal(idx, [[1, 2, 3], [0, 1, 2], [0, 1, 2], [0, 1, 2]])
    np.testing.assert_allclose(w[3], [1 / 3] * 3, rtol=1e-15)
    np.testing.assert_allclose(w[0], [1 / 3] * 3, rtol=1e-15)


def test_k1_is_first_max_argmax_with_unit_weight():
    lg = rand_logits(5, 200, 16, quant=1)
    idx, w = O.topk_gate(lg, 1)
    np.testing.assert_array_equal(idx[:, 0], np.argmax(lg, axis=1))
    np.testing.assert_array_equal(w, np.ones((200, 1)))


def test_k_equals_E_is_the_full_softmax_in_sorted_order():
    lg = rand_logits(6, 64, 8)
    idx, w = O.topk_gate(lg, 8)
    full = scipy.special.softmax(lg.astype(np.float64), axis=1)
    np.testing.assert_allclose(w, np.take_along_axis(full, idx.astype(np.int64), axis=1), rtol=1e-13)
    assert np.all(np.sort(idx, axis=1) == np.arange(8)[None, :])


def test_top2_weight_is_the_logistic_of_the_logit_gap():
    lg = rand_logits(7, 300, 8)
    idx, w = O.topk_gate(lg, 2)
    top = np.sort(lg.astype(np.float64), axis=1)[:, ::-1]
    gap = top[:, 0] - top[:, 1]
    np.testing.assert_allclose(w[:, 0], 1 / (1 + np.exp(-gap)), rtol=1e-14)
    np.testing.assert_allclose(w[:, 1], 1 / (1 + np.exp(gap)), rtol=1e-13)


def test_renormalised_full_softmax_equals_softmax_over_selected():
    lg = rand_logits(8, 100, 8)
    idx, w = O.topk_gate(lg, 2)
    full = scipy.special.softmax(lg.astype(np.float64), axis=1)
    sel = np.take_along_axis(full, idx.astype(np.int64), axis=1)
    np.testing.assert_allclose(w, sel / sel.sum(axis=1, keepdims=True), rtol=1e-13)


@pytest.mark.parametrize("E,k", [(8, 2), (64, 6)])
def test_invariants(E, k):
    lg = rand_logits(9, 500, E, quant=4)
    idx, w = O.topk_gate(lg, k)
    assert idx.min() >= 0 and idx.max() < E
    assert all(len(set(r)) == k for r in idx.tolist())
    sel = np.take_along_axis(lg, idx.astype(np.int64), axis=1)
    assert np.all(np.diff(sel, axis=1) <= 0)
    assert np.all(np.diff(w, axis=1) <= 0)
    np.testing.assert_allclose(w.sum(axis=1), 1.0, atol=1e-14)
    # shifting a row by a constant changes nothing
    idx2, w2 = O.topk_gate((lg.astype(np.float64) + 3.25), k)
    np.testing.assert_array_equal(idx, idx2)
    np.testing.assert_allclose(w, w2, rtol=1e-13)


def test_large_magnitude_logits_do_not_overflow():
    lg = np.array([[1e4, 1e4 - 1, -1e4, 0]], dtype=np.float32)
    idx, w = O.topk_gate(lg, 2)
    np.testing.assert_array_equal(idx, [[0, 1]])
    np.testing.assert_allclose(w[0, 0], 1 / (1 + math.exp(-1.0)), rtol=1e-14)


def test_rejects_bad_input():
    with pytest.raises(ValueError):
        O.topk_gate(np.array([[0.0, np.nan]], dtype=np.float32), 1)
    with pytest.raises(ValueError):
        O.topk_gate(np.array([[0.0, np.inf]], dtype=np.float32), 1)
    with pytest.raises(ValueError):
        O.topk_gate(np.zeros((2, 4), dtype=np.float32), 5)
    with pytest.raises(ValueError):
        O.topk_gate(np.zeros((2, 4), dtype=np.float32), 0)


# ---- planted mistakes: the pins above must reject plausible wrong gates -----
def _wrong_tie_high_index(lg, k):
    order = np.argsort(-lg[:, ::-1].astype(np.float64), axis=1, kind="stable")
    idx = (lg.shape[1] - 1 - order)[:, :k]
    sel = np.take_along_axis(lg.astype(np.float64), idx, axis=1)
    p = np.exp(sel - sel[:, :1])
    return idx.astype(np.int32), p / p.sum(axis=1, keepdims=True)


def _wrong_softmax_over_all(lg, k):
    idx, _ = O.topk_gate(lg, k)
    full = scipy.special.softmax(lg.astype(np.float64), axis=1)
    return idx, np.take_along_axis(full, idx.astype(np.int64), axis=1)


def test_planted_mistakes_are_caught():
    lg = rand_logits(50, 50, 8, quant=2)
    bidx, bw = brute_gate(lg, 2)
    assert not np.array_equal(_wrong_tie_high_index(lg, 2)[0], bidx)
    assert not np.allclose(_wrong_softmax_over_all(lg, 2)[1], bw, rtol=1e-6)


# ---- gating without renormalisation (softmax over all experts, read at the kept ones) ----

def brute_gate_all(logits, k):
    idx, _ = brute_gate(logits, k)
    T, E = logits.shape
    w = np.zeros((T, k))
    for t in range(T):
        m = max(float(v) for v in logits[t])
        z = [math.exp(float(v) - m) for v in logits[t]]
        s = 0.0
        for v in z:
            s += v
        w[t] = [z[e] / s for e in idx[t]]
    return idx, w


@pytest.mark.parametrize("T,E,k", [(5, 4, 2), (17, 8, 2), (9, 64, 6), (3, 5, 5)])
def test_all_norm_matches_brute_force(T, E, k):
    rng = np.random.default_rng(T * 100 + E)
    lg = rng.normal(size=(T, E)).astype(np.float32)
    idx, w = O.topk_gate(lg, k, norm="all")
    bi, bw = brute_gate_all(lg, k)
    assert np.array_equal(idx, bi)
    np.testing.assert_allclose(w, bw, rtol=1e-13, atol=0)


def test_all_norm_textbook_example():
    # logits = ln(1, 2, 3, 4): the softmax is (0.1, 0.2, 0.3, 0.4)
    lg = np.log(np.array([[1.0, 2.0, 3.0, 4.0]]))
    idx, w = O.topk_gate(lg, 2, norm="all")
    assert idx.tolist() == [[3, 2]]
    np.testing.assert_allclose(w, [[0.4, 0.3]], rtol=1e-14)
    _, ws = O.topk_gate(lg, 2)                       # renormalised over the kept pair
    np.testing.assert_allclose(ws, [[4 / 7, 3 / 7]], rtol=1e-14)


def test_all_norm_is_selected_norm_times_kept_mass_and_same_selection():
    rng = np.random.default_rng(11)
    lg = rng.normal(size=(40, 16)) * 3
    idx_a, w_a = O.topk_gate(lg, 4, norm="all")
    idx_s, w_s = O.topk_gate(lg, 4)
    assert np.array_equal(idx_a, idx_s)
    full = scipy.special.softmax(lg, axis=1)
    mass = np.take_along_axis(full, idx_a, axis=1).sum(axis=1, keepdims=True)
    np.testing.assert_allclose(w_a, w_s * mass, rtol=1e-12)
    np.testing.assert_allclose(w_a, np.take_along_axis(full, idx_a, axis=1), rtol=1e-12)
    assert np.all(w_a.sum(axis=1) < 1.0)
    # k = E: nothing is dropped, both rules give the full softmax
    _, w_full = O.topk_gate(lg, 16, norm="all")
    np.testing.assert_allclose(w_full.sum(axis=1), 1.0, rtol=1e-12)
    np.testing.assert_allclose(w_full, O.topk_gate(lg, 16)[1], rtol=1e-12)


def test_all_norm_uniform_logits_shift_invariance_and_large_magnitudes():
    _, w = O.topk_gate(np.full((3, 8), 2.5), 2, norm="all")
    np.testing.assert_allclose(w, 1 / 8, rtol=1e-14)
    rng = np.random.default_rng(5)
    lg = rng.normal(size=(10, 8))
    np.testing.assert_allclose(O.topk_gate(lg + 1000.0, 2, norm="all")[1], O.topk_gate(lg, 2, norm="all")[1], rtol=1e-9)
    _, w = O.topk_gate(np.array([[900.0, -900.0, 899.0, 0.0]]), 2, norm="all")
    assert np.all(np.isfinite(w))
    np.testing.assert_allclose(w[0, 0] / w[0, 1], math.e, rtol=1e-12)
    with pytest.raises(ValueError):
        O.topk_gate(lg, 2, norm="none")
