"""GPU parity: moe_topk_gate vs the oracle on identical logits.  Indices must
match bit for bit; weights within 1e-4 relative (fp32 softmax vs fp64)."""
import numpy as np
import pytest
import torch

from oracle import moe_oracle as O

pytestmark = pytest.mark.gpu


def run_gate(lib, lg, k):
    T, E = lg.shape
    dl = torch.from_numpy(lg).cuda()
    idx = torch.full((T, k), -7, dtype=torch.int32, device="cuda")
    w = torch.full((T, k), -1.0, dtype=torch.float32, device="cuda")
    lib.moe_topk_gate(dl, T, E, k, idx, w)
    torch.cuda.synchronize()
    return idx.cpu().numpy(), w.cpu().numpy()


def check(lib, lg, k):
    oi, ow = O.topk_gate(lg, k)
    gi, gw = run_gate(lib, lg, k)
    np.testing.assert_array_equal(gi, oi)
    # relative to the oracle's weight; weights that underflow to 0 in fp64 must be (near) 0 on the GPU too
    err = float(np.max(np.abs(gw.astype(np.float64) - ow) / np.maximum(ow, 1e-30))) if ow.size else 0.0
    assert err <= 1e-4, err
    return err


@pytest.mark.parametrize("T,E,k", [(1, 8, 2), (257, 8, 2), (4096, 8, 2), (8192, 64, 6), (100, 5, 5), (333, 13, 3),
                                   (77, 130, 4), (65, 256, 16), (1000, 16, 1), (513, 32, 8), (40, 1, 1), (99, 3, 2)])
def test_random_logits(lib, T, E, k):
    rng = np.random.default_rng(T * 1000 + E)
    check(lib, (rng.standard_normal((T, E)) * 3).astype(np.float32), k)


@pytest.mark.parametrize("E,k", [(8, 2), (64, 6), (7, 3)])
def test_many_exact_ties_and_signed_zeros(lib, E, k):
    rng = np.random.default_rng(E)
    lg = np.round(rng.standard_normal((2000, E))).astype(np.float32)        # integers in about [-3,3]: ties everywhere
    lg[lg == 0] = np.where(rng.random((lg == 0).sum()) < 0.5, -0.0, 0.0)
    check(lib, lg, k)
    check(lib, np.zeros((64, E), dtype=np.float32), k)
    check(lib, np.full((64, E), -0.0, dtype=np.float32), k)


def test_extreme_finite_values(lib):
    lg = np.array([[3e38, -3e38, 0, 1e-45, -1e-45, 1, -1, 2]] * 5, dtype=np.float32)
    check(lib, lg, 2)
    check(lib, lg, 8)


def test_large_batch(lib):
    rng = np.random.default_rng(1)
    check(lib, rng.standard_normal((1 << 18, 8)).astype(np.float32), 2)
    check(lib, rng.standard_normal((1 << 15, 64)).astype(np.float32), 6)


def test_config_logits(lib):
    from paper_2502_06643_amd import synth
    for name in ("c1", "c1b", "c2", "c4"):
        cfg = synth.config(name)
        x = synth.make_x(cfg)
        check(lib, synth.make_logits(cfg, x), cfg.k)


# ---- gate weights without renormalisation (softmax over all experts read at the selected ones) ----

def check_all_norm(lib, lg, k):
    from paper_2502_06643_amd import binding as B
    T, E = lg.shape
    oi, ow = O.topk_gate(lg, k, norm="all")
    dl = torch.from_numpy(lg).cuda()
    idx = torch.full((T, k), -7, dtype=torch.int32, device="cuda")
    w = torch.full((T, k), -1.0, dtype=torch.float32, device="cuda")
    lib.moe_topk_gate_norm(dl, T, E, k, B.MOE_NORM_SOFTMAX_ALL, idx, w)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(idx.cpu().numpy(), oi)
    gw = w.cpu().numpy().astype(np.float64)
    err = float(np.max(np.abs(gw - ow) / np.maximum(ow, 1e-30))) if ow.size else 0.0
    assert err <= 1e-4, err
    # the selected-norm entry point is untouched by the variant: same indices, renormalised weights
    si, sw = run_gate(lib, lg, k)
    np.testing.assert_array_equal(si, oi)
    np.testing.assert_allclose(sw.sum(axis=1), 1.0, rtol=1e-5)


@pytest.mark.parametrize("T,E,k", [(1, 8, 2), (257, 8, 2), (4096, 8, 2), (8192, 64, 6), (100, 5, 5), (333, 13, 3),
                                   (77, 130, 4), (65, 256, 16), (1000, 16, 1), (513, 32, 8), (40, 1, 1), (99, 3, 2)])
def test_all_norm_random_logits(lib, T, E, k):
    rng = np.random.default_rng(T * 1000 + E + 1)
    check_all_norm(lib, (rng.standard_normal((T, E)) * 3).astype(np.float32), k)


def test_all_norm_ties_extremes_and_config_logits(lib):
    from paper_2502_06643_amd import synth
    rng = np.random.default_rng(9)
    lg = np.round(rng.standard_normal((2000, 8))).astype(np.float32)
    lg[lg == 0] = np.where(rng.random((lg == 0).sum()) < 0.5, -0.0, 0.0)
    check_all_norm(lib, lg, 2)
    check_all_norm(lib, np.zeros((64, 64), dtype=np.float32), 6)
    check_all_norm(lib, np.array([[80.0, -80.0, 0, 1e-45, -1e-45, 1, -1, 79]] * 5, dtype=np.float32), 2)
    for name in ("c1", "c2", "c4"):
        cfg = synth.config(name)
        check_all_norm(lib, synth.make_logits(cfg, synth.make_x(cfg)), cfg.k)


def test_all_norm_rejects_unknown_rule(lib):
    from paper_2502_06643_amd import binding as B
    lg = torch.zeros((4, 8), device="cuda")
    idx = torch.zeros((4, 2), dtype=torch.int32, device="cuda")
    w = torch.zeros((4, 2), device="cuda")
    with pytest.raises(B.MoeError):
        lib.moe_topk_gate_norm(lg, 4, 8, 2, 7, idx, w)
