"""Pins for oracle.transition_counts (Section 2.4, Section 3.1 "Token Routing
Profile", ILP 2 input R_{e1,e2,l}) and for the placement evaluators (Eq. 1-3,
Eq. 8-9).

Pins: a set-comprehension brute force, the three marginal identities
(row sums = k_{l+1} * P_l, column sums = k_l * P_{l+1}, total = T k_l k_{l+1}),
k=1 against a library contingency table, accumulate-twice = 2x, and for the
evaluators the conservation laws sum_c T_c = sum_e P_e and sum C = sum R plus a
hand-worked 4-expert example.
"""
import numpy as np
import pandas as pd
import pytest

from oracle import moe_oracle as O
from paper_2502_06643_amd import synth


@pytest.mark.parametrize("T,E1,E2,k1,k2", [(40, 8, 8, 2, 2), (25, 5, 9, 1, 3), (30, 16, 4, 6, 2)])
def test_matches_brute_force(T, E1, E2, k1, k2):
    a = synth.random_topk_idx(1, T, E1, k1)
    b = synth.random_topk_idx(2, T, E2, k2)
    R = O.transition_counts(a, b, E1, E2)
    assert R.dtype == np.int64 and R.shape == (E1, E2)
    for e1 in range(E1):
        for e2 in range(E2):
            n = len([(t, j1, j2) for t in range(T) for j1 in range(k1) for j2 in range(k2)
                     if a[t, j1] == e1 and b[t, j2] == e2])
            assert R[e1, e2] == n
    assert not np.array_equal(R, O.transition_counts(b, a, E2, E1)) or E1 == E2 and np.array_equal(R, R.T)


def test_marginals():
    T, E, k1, k2 = 700, 8, 2, 2
    a = synth.random_topk_idx(3, T, E, k1)
    b = synth.random_topk_idx(4, T, E, k2)
    R = O.transition_counts(a, b, E, E)
    P_l = np.bincount(a.reshape(-1), minlength=E)
    P_l1 = np.bincount(b.reshape(-1), minlength=E)
    np.testing.assert_array_equal(R.sum(axis=1), k2 * P_l)
    np.testing.assert_array_equal(R.sum(axis=0), k1 * P_l1)
    assert R.sum() == T * k1 * k2
    # with k_{l+1} = 1 the rows sum to the layer-l expert counts themselves
    R1 = O.transition_counts(a, b[:, :1], E, E)
    np.testing.assert_array_equal(R1.sum(axis=1), P_l)


def test_k1_is_a_contingency_table():
    T, E = 1000, 8
    a = synth.random_topk_idx(5, T, E, 1)
    b = synth.random_topk_idx(6, T, E, 1)
    R = O.transition_counts(a, b, E, E)
    ct = pd.crosstab(pd.Categorical(a[:, 0], categories=range(E)), pd.Categorical(b[:, 0], categories=range(E)),
                     dropna=False).to_numpy()
    np.testing.assert_array_equal(R, ct)
    D = O.transition_counts(a, a, E, E)                      # same layer twice -> diagonal = P
    np.testing.assert_array_equal(D, np.diag(np.bincount(a[:, 0], minlength=E)))


def test_accumulates_in_place():
    a = synth.random_topk_idx(7, 50, 8, 2)
    b = synth.random_topk_idx(8, 50, 8, 2)
    R = O.transition_counts(a, b, 8, 8)
    R2 = O.transition_counts(a, b, 8, 8, R.copy())
    np.testing.assert_array_equal(R2, 2 * R)
    with pytest.raises(ValueError):
        O.transition_counts(a, b, 8, 8, np.zeros((8, 8), dtype=np.int32))
    with pytest.raises(ValueError):
        O.transition_counts(a, b, 4, 8)


def test_empty_batch():
    R = O.transition_counts(np.zeros((0, 2), dtype=np.int32), np.zeros((0, 2), dtype=np.int32), 8, 8)
    assert not R.any()


# --------------------------- evaluators (Eq. 1-3, 8-9) -----------------------
def test_cluster_loads_hand_example_and_conservation():
    P = np.array([50, 30, 15, 5])
    pl = np.array([0, 1, 1, 0])
    np.testing.assert_array_equal(O.cluster_loads(P, pl, 2), [55, 45])          # Eq. 2
    assert O.load_imbalance(P, pl, 2) == pytest.approx(10.0)                     # |55-50|+|45-50|, Eq. 1 & 3
    assert O.load_imbalance(P, np.array([0, 0, 1, 1]), 2) == pytest.approx(60.0)
    rng = np.random.default_rng(0)
    P = rng.integers(0, 1000, 16)
    for G in (1, 2, 4, 8):
        assert O.cluster_loads(P, rng.integers(0, G, 16), G).sum() == P.sum()


def test_cluster_traffic_hand_example_and_conservation():
    R = np.array([[1, 2], [3, 4]])
    np.testing.assert_array_equal(O.cluster_traffic(R, [0, 1], [0, 1], 2), R)
    np.testing.assert_array_equal(O.cluster_traffic(R, [0, 1], [1, 0], 2), R[:, ::-1])   # second map is layer l+1's
    np.testing.assert_array_equal(O.cluster_traffic(R, [0, 0], [0, 1], 2), [[4, 6], [0, 0]])
    rng = np.random.default_rng(1)
    R = rng.integers(0, 100, (8, 8))
    C = O.cluster_traffic(R, rng.integers(0, 4, 8), rng.integers(0, 4, 8), 4)
    assert C.sum() == R.sum()
    assert O.max_pair_cost(np.array([[4, 6], [0, 9]]), np.array([[1.0, 2.0], [2.0, 4.5]])) == pytest.approx(4.0)


def test_top1_only_counts_one_pair_per_token():
    rng = np.random.default_rng(3)
    T, E1, E2 = 200, 8, 6
    a = np.stack([rng.permutation(E1)[:3] for _ in range(T)]).astype(np.int32)
    b = np.stack([rng.permutation(E2)[:2] for _ in range(T)]).astype(np.int32)
    R = O.transition_counts(a, b, E1, E2, top1_only=True)
    # brute force on slot 0 of either layer
    B = np.zeros((E1, E2), dtype=np.int64)
    for t in range(T):
        B[a[t, 0], b[t, 0]] += 1
    assert np.array_equal(R, B)
    assert R.sum() == T
    assert np.array_equal(R.sum(axis=1), np.bincount(a[:, 0], minlength=E1))
    assert np.array_equal(R.sum(axis=0), np.bincount(b[:, 0], minlength=E2))
    # it is the all-pairs table of the first columns, and a subset of the full all-pairs table
    assert np.array_equal(R, O.transition_counts(a[:, :1], b[:, :1], E1, E2))
    assert np.all(R <= O.transition_counts(a, b, E1, E2))
    # k = 1 in both layers: the two modes coincide
    assert np.array_equal(O.transition_counts(a[:, :1], b[:, :1], E1, E2, top1_only=True), R)
    # accumulates in place like the all-pairs mode
    R2 = O.transition_counts(a, b, E1, E2, R=R.copy(), top1_only=True)
    assert np.array_equal(R2, 2 * R)
