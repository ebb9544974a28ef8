"""Pins for oracle.dispatch (Section 1 / Section 2.2: tokens go to the GPU that
owns their expert; Section 3.1: custom, possibly uneven expert->GPU maps; ILP 1
input P_{e,l}).

Pinned by a definitional triple loop (for each GPU, for each of its experts,
for each route in order), by invariants, and by the paper's contiguous map (8
experts on 4 GPUs: GPU g owns experts 2g and 2g+1), for which the bucket order
equals a plain sort by expert.
"""
import numpy as np
import pytest

from oracle import moe_oracle as O
from paper_2502_06643_amd import synth


def brute_dispatch(idx, placement, G):
    T, k = idx.shape
    E = len(placement)
    flat = [int(v) for v in idx.reshape(-1)]
    perm, estart, ecount = [], [0] * E, [0] * E
    gcount = [0] * G
    for g in range(G):
        for e in range(E):
            if placement[e] != g:
                continue
            estart[e] = len(perm)
            for r in range(T * k):
                if flat[r] == e:
                    perm.append(r)
                    ecount[e] += 1
                    gcount[g] += 1
    inv = [0] * (T * k)
    for p, r in enumerate(perm):
        inv[r] = p
    goff = [0]
    for g in range(G):
        goff.append(goff[-1] + gcount[g])
    return perm, inv, ecount, estart, gcount, goff


MAPS = {
    "contiguous": (np.array([0, 0, 1, 1, 2, 2, 3, 3], dtype=np.int32), 4),
    "interleaved": (np.array([3, 0, 2, 1, 0, 3, 1, 2], dtype=np.int32), 4),
    "uneven_1124": (np.array([2, 3, 0, 3, 1, 3, 2, 3], dtype=np.int32), 4),
    "empty_gpu": (np.array([0, 0, 0, 2, 2, 2, 4, 4], dtype=np.int32), 5),
    "single": (np.zeros(8, dtype=np.int32), 1),
}


@pytest.mark.parametrize("name", list(MAPS))
@pytest.mark.parametrize("T,k", [(1, 1), (33, 2), (70, 3)])
def test_matches_brute_force(name, T, k):
    pl, G = MAPS[name]
    idx = synth.random_topk_idx(11 * T + k, T, 8, k)
    x = np.random.default_rng(1).standard_normal((T, 6)).astype(np.float32)
    r = O.dispatch(x, idx, pl, G)
    perm, inv, ecount, estart, gcount, goff = brute_dispatch(idx, pl.tolist(), G)
    np.testing.assert_array_equal(r["perm"], perm)
    np.testing.assert_array_equal(r["inv_perm"], inv)
    np.testing.assert_array_equal(r["expert_counts"], ecount)
    np.testing.assert_array_equal(r["expert_start"], estart)
    np.testing.assert_array_equal(r["gpu_counts"], gcount)
    np.testing.assert_array_equal(r["gpu_offsets"], goff)
    for p in range(T * k):
        assert r["send_buf"][p].tobytes() == x[perm[p] // k].tobytes()
    for v in ("perm", "inv_perm", "expert_counts", "expert_start", "gpu_counts", "gpu_offsets"):
        assert r[v].dtype == np.int32


@pytest.mark.parametrize("E,G,k,T", [(8, 4, 2, 257), (64, 8, 6, 301), (16, 3, 4, 99)])
def test_invariants(E, G, k, T):
    rng = np.random.default_rng(E + G)
    pl = rng.integers(0, G, E).astype(np.int32)
    idx = synth.random_topk_idx(7, T, E, k)
    r = O.dispatch(None, idx, pl, G)
    N = T * k
    assert r["expert_counts"].sum() == N and r["gpu_counts"].sum() == N
    assert r["gpu_offsets"][0] == 0 and r["gpu_offsets"][G] == N
    assert sorted(r["perm"].tolist()) == list(range(N))          # bijection
    np.testing.assert_array_equal(r["inv_perm"][r["perm"]], np.arange(N))
    e_sorted = idx.reshape(-1)[r["perm"]]
    key = pl[e_sorted].astype(np.int64) * E + e_sorted
    assert np.all(np.diff(key) >= 0)
    same = np.diff(key) == 0
    assert np.all(np.diff(r["perm"])[same] > 0)                   # stable inside a key
    np.testing.assert_array_equal(np.bincount(r["perm"] // k, minlength=T), np.full(T, k))
    for e in range(E):                                            # buckets are where they claim
        s, c = r["expert_start"][e], r["expert_counts"][e]
        assert np.all(e_sorted[s:s + c] == e)
        assert r["gpu_offsets"][pl[e]] <= s and s + c <= r["gpu_offsets"][pl[e] + 1]


def test_paper_contiguous_map_equals_plain_sort_by_expert():
    """Section 1: 8 experts over 4 GPUs, GPU 0 <- {0,1}, GPU 1 <- {2,3}, ..."""
    pl = synth.placement_contiguous(8, 4)
    np.testing.assert_array_equal(pl, [0, 0, 1, 1, 2, 2, 3, 3])
    idx = synth.random_topk_idx(3, 500, 8, 2)
    a = O.dispatch(None, idx, pl, 4)
    b = O.dispatch(None, idx, np.zeros(8, dtype=np.int32), 1)
    np.testing.assert_array_equal(a["perm"], b["perm"])
    np.testing.assert_array_equal(a["perm"], np.argsort(idx.reshape(-1), kind="stable"))
    np.testing.assert_array_equal(a["expert_start"], b["expert_start"])
    np.testing.assert_array_equal(a["gpu_offsets"][:4], a["expert_start"][::2])
    np.testing.assert_array_equal(a["gpu_counts"], a["expert_counts"].reshape(4, 2).sum(axis=1))


def test_non_contiguous_map_changes_bucket_order():
    idx = synth.random_topk_idx(4, 200, 8, 2)
    a = O.dispatch(None, idx, MAPS["contiguous"][0], 4)
    b = O.dispatch(None, idx, MAPS["interleaved"][0], 4)
    assert not np.array_equal(a["perm"], b["perm"])
    np.testing.assert_array_equal(a["expert_counts"], b["expert_counts"])   # P does not depend on the map
    assert not np.all(np.diff(b["expert_start"]) >= 0)


def test_bf16_rows_are_bit_copies():
    x = np.random.default_rng(2).integers(0, 65536, (40, 16)).astype(np.uint16)
    idx = synth.random_topk_idx(5, 40, 8, 2)
    r = O.dispatch(x, idx, MAPS["uneven_1124"][0], 4)
    assert r["send_buf"].dtype == np.uint16
    np.testing.assert_array_equal(r["send_buf"], x[r["perm"] // 2])


def test_rejects_bad_contents():
    idx = np.array([[0, 9]], dtype=np.int32)
    with pytest.raises(ValueError):
        O.dispatch(None, idx, np.zeros(8, dtype=np.int32), 1)
    with pytest.raises(ValueError):
        O.dispatch(None, np.array([[0, 1]], dtype=np.int32), np.array([0, 4] + [0] * 6, dtype=np.int32), 4)
