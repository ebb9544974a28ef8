"""GPU parity of the placement evaluators (Eq. 1-3, Eq. 8-9) against the
oracle, and a small end-to-end use of them: profile routing on the GPU (P from
moe_dispatch's expert_counts, R from moe_transition_counts), then score expert
placements with the paper's two objectives and pick a better one than the
contiguous default by exhaustive search (8 experts on 4 GPUs; the ILP solver
itself is out of scope)."""
import itertools

import numpy as np
import pytest
import torch

from oracle import moe_oracle as O
from paper_2502_06643_amd import synth

pytestmark = pytest.mark.gpu


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def gpu_loads(lib, P, pl, G):
    T_c = torch.full((G,), -1, dtype=torch.int64, device="cuda")
    imb = torch.full((1,), -1.0, dtype=torch.float64, device="cuda")
    lib.moe_placement_loads(dev(P.astype(np.int64)), dev(pl.astype(np.int32)), len(P), G, T_c, imb)
    torch.cuda.synchronize()
    return T_c.cpu().numpy(), float(imb.item())


def gpu_traffic(lib, R, pa, pb, G, B=None):
    C = torch.full((G, G), -1, dtype=torch.int64, device="cuda")
    mc = torch.full((1,), -1.0, dtype=torch.float64, device="cuda")
    lib.moe_placement_traffic(dev(R.astype(np.int64)), dev(pa.astype(np.int32)), dev(pb.astype(np.int32)), R.shape[0], R.shape[1], G,
                              C, None if B is None else dev(B.astype(np.float64)), mc)
    torch.cuda.synchronize()
    return C.cpu().numpy(), float(mc.item())


@pytest.mark.parametrize("E,G", [(8, 4), (64, 8), (256, 256), (5, 1), (16, 3)])
def test_loads_match_oracle(lib, E, G):
    rng = np.random.default_rng(E + G)
    P = rng.integers(0, 1 << 40, E)                          # beyond 32 bits
    pl = rng.integers(0, G, E).astype(np.int32)
    T_c, imb = gpu_loads(lib, P, pl, G)
    np.testing.assert_array_equal(T_c, O.cluster_loads(P, pl, G))
    assert imb == pytest.approx(O.load_imbalance(P, pl, G), rel=1e-12)


@pytest.mark.parametrize("E1,E2,G", [(8, 8, 4), (64, 64, 8), (5, 9, 3), (256, 256, 16)])
def test_traffic_matches_oracle(lib, E1, E2, G):
    rng = np.random.default_rng(E1 * G)
    R = rng.integers(0, 1 << 36, (E1, E2))
    pa = rng.integers(0, G, E1).astype(np.int32)
    pb = rng.integers(0, G, E2).astype(np.int32)
    B = rng.uniform(1.0, 9.0, (G, G))                        # e.g. intra-node vs 9x slower inter-node links
    C, mc = gpu_traffic(lib, R, pa, pb, G, B)
    Cref = O.cluster_traffic(R, pa, pb, G)
    np.testing.assert_array_equal(C, Cref)
    assert mc == pytest.approx(O.max_pair_cost(Cref, B), rel=1e-12)
    C2, mc2 = gpu_traffic(lib, R, pa, pb, G, None)
    assert mc2 == pytest.approx(float(Cref.max()), rel=1e-12)
    assert C.sum() == R.sum()                                # Eq. 9 conserves the routed tokens


def test_accumulate_counts_over_batches(lib):
    E = 8
    P = torch.zeros(E, dtype=torch.int64, device="cuda")
    ref = np.zeros(E, dtype=np.int64)
    for b in range(5):
        c = np.random.default_rng(b).integers(0, 1 << 30, E).astype(np.int32)
        lib.moe_accumulate_counts(dev(c), E, P)
        ref += c
    torch.cuda.synchronize()
    np.testing.assert_array_equal(P.cpu().numpy(), ref)


def balanced_maps(E, G):
    """All expert->GPU maps with E/G experts per GPU, up to relabelling of the GPUs."""
    per = E // G

    def rec(remaining, groups):
        if not remaining:
            yield groups
            return
        first = remaining[0]
        for rest in itertools.combinations(remaining[1:], per - 1):
            grp = (first,) + rest
            yield from rec([e for e in remaining if e not in grp], groups + [grp])
    for groups in rec(list(range(E)), []):
        pl = np.empty(E, dtype=np.int32)
        for g, grp in enumerate(groups):
            pl[list(grp)] = g
        yield pl


def test_profile_then_pick_a_better_placement(lib):
    """Two chained layers with the skew and affinity of the C5 recipe at a reduced token count."""
    cfg = synth.config("c5").with_(T=4096)
    E, G, k = cfg.E, 4, cfg.k
    x = synth.make_x(cfg)
    lg0 = synth.make_logits(cfg, x, 0)
    idx0_ref, _ = O.topk_gate(lg0, k)
    lg1 = synth.make_logits(cfg, x, 1, prev_top1=idx0_ref[:, 0])
    i32 = dict(dtype=torch.int32, device="cuda")
    idx = [torch.empty((cfg.T, k), **i32) for _ in range(2)]
    w = torch.empty((cfg.T, k), dtype=torch.float32, device="cuda")
    P = [torch.zeros(E, dtype=torch.int64, device="cuda") for _ in range(2)]
    R = torch.zeros((E, E), dtype=torch.int64, device="cuda")
    contiguous = synth.placement_contiguous(E, G)
    pl_dev = dev(contiguous)
    N = cfg.T * k
    outs = [torch.empty(n, **i32) for n in (N, N, E, E, G, G + 1)]
    ws = torch.empty(lib.moe_dispatch_workspace_bytes(cfg.T, E, k), dtype=torch.uint8, device="cuda")
    for layer, lg in enumerate((lg0, lg1)):
        lib.moe_topk_gate(dev(lg), cfg.T, E, k, idx[layer], w)
        lib.moe_dispatch(None, lib.MOE_BF16, idx[layer], cfg.T, 0, E, k, pl_dev, G, None, outs[0], outs[1], outs[2], outs[3],
                         outs[4], outs[5], ws)
        lib.moe_accumulate_counts(outs[2], E, P[layer])
    lib.moe_transition_counts(idx[0], idx[1], cfg.T, k, k, E, E, R)
    torch.cuda.synchronize()
    P0, P1, Rh = P[0].cpu().numpy(), P[1].cpu().numpy(), R.cpu().numpy()
    idx1_ref, _ = O.topk_gate(lg1, k)
    P0_ref = np.bincount(idx0_ref.reshape(-1), minlength=E).astype(np.int64)
    R_ref = O.transition_counts(idx0_ref, idx1_ref, E, E)
    np.testing.assert_array_equal(P0, P0_ref)
    np.testing.assert_array_equal(Rh, R_ref)

    # objective 1 (Eq. 1): load imbalance of layer 0, contiguous map vs the best balanced map
    base = gpu_loads(lib, P0, contiguous, G)[1]
    best_pl, best = None, None
    for pl in balanced_maps(E, G):
        v = O.load_imbalance(P0_ref, pl, G)                  # the oracle works on its own profile
        if best is None or v < best:
            best, best_pl = v, pl
    assert gpu_loads(lib, P0, best_pl, G)[1] == pytest.approx(best, rel=1e-12)
    assert best < 0.5 * base                                  # the Zipf skew makes the contiguous map badly unbalanced
    # objective 2 (Eq. 8): with layer 0 fixed to that map, place layer 1 to minimise the worst GPU pair
    base2 = gpu_traffic(lib, Rh, best_pl, contiguous, G)[1]
    best2 = min(O.max_pair_cost(O.cluster_traffic(R_ref, best_pl, pl, G), np.ones((G, G))) for pl in balanced_maps(E, G))
    assert best2 <= base2
    print(f"layer-0 imbalance: contiguous {base:.0f} -> best balanced {best:.0f}; "
          f"worst GPU-pair traffic 0->1: contiguous {base2:.0f} -> best {best2:.0f}")
