"""GPU parity: moe_transition_counts vs the oracle, bit exact (int64)."""
import numpy as np
import pytest
import torch

from oracle import moe_oracle as O
from paper_2502_06643_amd import synth

pytestmark = pytest.mark.gpu


def run(lib, a, b, E1, E2, R0=None):
    R = torch.zeros((E1, E2), dtype=torch.int64, device="cuda") if R0 is None else torch.from_numpy(R0).cuda()
    lib.moe_transition_counts(torch.from_numpy(a).cuda(), torch.from_numpy(b).cuda(), a.shape[0], a.shape[1], b.shape[1], E1, E2, R)
    torch.cuda.synchronize()
    return R.cpu().numpy()


@pytest.mark.parametrize("T,E1,E2,k1,k2", [(1, 8, 8, 2, 2), (1000, 8, 8, 2, 2), (16384, 8, 8, 2, 2), (5000, 64, 64, 6, 6),
                                           (3000, 5, 9, 1, 3), (2000, 200, 100, 4, 2), (777, 256, 256, 16, 16), (4097, 16, 4, 6, 2)])
def test_matches_oracle(lib, T, E1, E2, k1, k2):
    a = synth.random_topk_idx(T, T, E1, k1)
    b = synth.random_topk_idx(T + 1, T, E2, k2)
    np.testing.assert_array_equal(run(lib, a, b, E1, E2), O.transition_counts(a, b, E1, E2))


def test_accumulates_over_batches_and_large_start_values(lib):
    a = synth.random_topk_idx(1, 3000, 8, 2)
    b = synth.random_topk_idx(2, 3000, 8, 2)
    R0 = np.full((8, 8), (1 << 40) + 3, dtype=np.int64)          # beyond 32 bits: the table really is int64
    ref = O.transition_counts(a, b, 8, 8, R0.copy())
    got = run(lib, a, b, 8, 8, R0.copy())
    np.testing.assert_array_equal(got, ref)
    got2 = run(lib, a, b, 8, 8, got.copy())
    np.testing.assert_array_equal(got2 - got, got - R0)


def test_marginals_at_a_size_the_oracle_loop_would_crawl_through(lib):
    T, E, k = 1 << 20, 8, 2
    a = synth.random_topk_idx(3, T, E, k)
    b = synth.random_topk_idx(4, T, E, k)
    R = run(lib, a, b, E, E)
    np.testing.assert_array_equal(R.sum(axis=1), k * np.bincount(a.reshape(-1), minlength=E))
    np.testing.assert_array_equal(R.sum(axis=0), k * np.bincount(b.reshape(-1), minlength=E))
    assert R.sum() == T * k * k
    # sampled bins one by one
    for e1, e2 in [(0, 0), (3, 5), (7, 1)]:
        n = int(((a == e1).any(axis=1) & (b == e2).any(axis=1)).sum())
        assert R[e1, e2] == n


def run_top1(lib, a, b, E1, E2, R0=None):
    from paper_2502_06643_amd import binding as B
    R = torch.zeros((E1, E2), dtype=torch.int64, device="cuda") if R0 is None else torch.from_numpy(R0).cuda()
    lib.moe_transition_counts_pairs(torch.from_numpy(a).cuda(), torch.from_numpy(b).cuda(), a.shape[0], a.shape[1], b.shape[1], E1, E2,
                                    B.MOE_PAIRS_TOP1, R)
    torch.cuda.synchronize()
    return R.cpu().numpy()


@pytest.mark.parametrize("T,E1,E2,k1,k2", [(1, 8, 8, 2, 2), (1000, 8, 8, 2, 2), (16384, 8, 8, 2, 2), (5000, 64, 64, 6, 6),
                                           (3000, 5, 9, 1, 3), (2000, 200, 100, 4, 2), (777, 256, 256, 16, 16)])
def test_top1_pairs_match_oracle(lib, T, E1, E2, k1, k2):
    a = synth.random_topk_idx(T + 5, T, E1, k1)
    b = synth.random_topk_idx(T + 6, T, E2, k2)
    ref = O.transition_counts(a, b, E1, E2, top1_only=True)
    np.testing.assert_array_equal(run_top1(lib, a, b, E1, E2), ref)
    assert ref.sum() == T
    # accumulates on top of an existing table; the all-pairs entry point is unchanged by the mode
    np.testing.assert_array_equal(run_top1(lib, a, b, E1, E2, ref.copy()), 2 * ref)
    np.testing.assert_array_equal(run(lib, a, b, E1, E2), O.transition_counts(a, b, E1, E2))


def test_many_pairs_per_token_at_a_size_that_takes_the_large_workgroups(lib):
    """top-6 x top-6 over 64 experts, 150000 tokens: more than 512 workgroups of 256 threads would be needed, so the
    launch switches to 1024-thread workgroups.  Marginal identities, the total, and sampled bins counted one by one."""
    T, E, k = 150000, 64, 6
    a = synth.random_topk_idx(23, T, E, k)
    b = synth.random_topk_idx(24, T, E, k)
    R = run(lib, a, b, E, E)
    np.testing.assert_array_equal(R.sum(axis=1), k * np.bincount(a.reshape(-1), minlength=E))
    np.testing.assert_array_equal(R.sum(axis=0), k * np.bincount(b.reshape(-1), minlength=E))
    assert R.sum() == T * k * k
    for e1, e2 in [(0, 0), (13, 50), (63, 1), (31, 32)]:
        assert R[e1, e2] == int(((a == e1).any(axis=1) & (b == e2).any(axis=1)).sum())


def test_top1_pairs_large_batch_marginals(lib):
    T, E, k = 1 << 20, 8, 2
    a = synth.random_topk_idx(13, T, E, k)
    b = synth.random_topk_idx(14, T, E, k)
    R = run_top1(lib, a, b, E, E)
    np.testing.assert_array_equal(R.sum(axis=1), np.bincount(a[:, 0], minlength=E))
    np.testing.assert_array_equal(R.sum(axis=0), np.bincount(b[:, 0], minlength=E))
    assert R[2, 6] == int(((a[:, 0] == 2) & (b[:, 0] == 6)).sum())
