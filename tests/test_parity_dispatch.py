"""GPU parity: moe_dispatch vs the oracle.  Everything is integer or a bit
copy, so everything must match exactly."""
import numpy as np
import pytest
import torch

from oracle import moe_oracle as O
from paper_2502_06643_amd import synth
from paper_2502_06643_amd.layer import to_device, to_host

pytestmark = pytest.mark.gpu


def run_dispatch(lib, x, idx, pl, G):
    T, k = idx.shape
    E = len(pl)
    N = T * k
    i32 = dict(dtype=torch.int32, device="cuda")
    d = 0 if x is None else x.shape[1]
    dt = lib.MOE_BF16 if (x is not None and x.dtype == np.uint16) else lib.MOE_F32
    dx = None if x is None else to_device(x)
    send = None if x is None else torch.zeros((N, d), dtype=dx.dtype, device="cuda")
    out = {n: torch.full((s,), -5, **i32) for n, s in
           [("perm", N), ("inv_perm", N), ("expert_counts", E), ("expert_start", E), ("gpu_counts", G), ("gpu_offsets", G + 1)]}
    ws = torch.empty(lib.moe_dispatch_workspace_bytes(T, E, k), dtype=torch.uint8, device="cuda")
    lib.moe_dispatch(dx, dt, torch.from_numpy(idx).cuda(), T, d, E, k, torch.from_numpy(pl).cuda(), G, send,
                     out["perm"], out["inv_perm"], out["expert_counts"], out["expert_start"], out["gpu_counts"],
                     out["gpu_offsets"], ws)
    torch.cuda.synchronize()
    res = {n: v.cpu().numpy() for n, v in out.items()}
    res["send_buf"] = None if x is None else to_host(send)
    return res


def check(lib, x, idx, pl, G):
    ref = O.dispatch(x, idx, pl, G)
    got = run_dispatch(lib, x, idx, pl, G)
    for n in ("expert_counts", "expert_start", "gpu_counts", "gpu_offsets", "perm", "inv_perm"):
        np.testing.assert_array_equal(got[n], ref[n], err_msg=n)
    if x is not None:
        np.testing.assert_array_equal(got["send_buf"], ref["send_buf"])


MAPS8 = {
    "contiguous4": (np.array([0, 0, 1, 1, 2, 2, 3, 3], dtype=np.int32), 4),
    "interleaved4": (np.array([3, 0, 2, 1, 0, 3, 1, 2], dtype=np.int32), 4),
    "uneven_1124": (np.array([2, 3, 0, 3, 1, 3, 2, 3], dtype=np.int32), 4),
    "empty_gpus": (np.array([0, 0, 0, 2, 2, 2, 4, 4], dtype=np.int32), 5),
    "single": (np.zeros(8, dtype=np.int32), 1),
}


@pytest.mark.parametrize("name", list(MAPS8))
@pytest.mark.parametrize("T,k", [(1, 1), (33, 2), (511, 2), (512, 2), (513, 2), (3000, 3), (5000, 8)])
def test_eight_experts(lib, name, T, k):
    pl, G = MAPS8[name]
    idx = synth.random_topk_idx(T + k, T, 8, k)
    x = synth.normal(T, 0, (T, 64), 1.0, "bf16")
    check(lib, x, idx, pl, G)


@pytest.mark.parametrize("E,G,k,T,d,dtype", [(64, 8, 6, 2500, 128, "bf16"), (256, 256, 16, 700, 8, "bf16"),
                                              (5, 3, 5, 1234, 12, "f32"), (130, 7, 4, 999, 260, "f32"),
                                              (8, 4, 2, 256, 128, "f32"), (1, 1, 1, 300, 4, "f32")])
def test_other_shapes(lib, E, G, k, T, d, dtype):
    rng = np.random.default_rng(E * 7 + G)
    pl = rng.integers(0, G, E).astype(np.int32)
    idx = synth.random_topk_idx(E, T, E, k)
    check(lib, synth.normal(E, 0, (T, d), 1.0, dtype), idx, pl, G)


def test_all_routes_to_one_expert_and_index_only_mode(lib):
    idx = np.full((4000, 1), 5, dtype=np.int32)
    check(lib, None, idx, MAPS8["interleaved4"][0], 4)
    idx = synth.random_topk_idx(9, 2100, 8, 2)
    check(lib, None, idx, MAPS8["uneven_1124"][0], 4)


def test_empty_batch(lib):
    got = run_dispatch(lib, None, np.zeros((0, 2), dtype=np.int32), MAPS8["contiguous4"][0], 4)
    assert not got["expert_counts"].any() and not got["gpu_counts"].any() and not got["gpu_offsets"].any()
    assert not got["expert_start"].any()


@pytest.mark.parametrize("T,E,k,G", [(70000, 8, 3, 4), (40000, 64, 6, 8), (16384, 8, 1, 4), (16385, 8, 1, 4), (4097, 8, 1, 2)])
def test_large_batches_take_the_multi_workgroup_path(lib, T, E, k, G):
    """Above 16384 routes the index build runs as count / scan / rank kernels
    over many workgroups instead of one fused workgroup (sizes on both sides
    of the switch); index-only mode."""
    rng = np.random.default_rng(T + E)
    pl = rng.integers(0, G, E).astype(np.int32)
    check(lib, None, synth.random_topk_idx(T % 1000 + E, T, E, k), pl, G)


@pytest.mark.parametrize("name", ["c2", "c2b", "c3", "c4", "c5"])
def test_config_shapes_full_size(lib, name):
    """Full-size batches with the skewed routing of the benchmark configs
    (expert choice comes from the oracle's gate on the config's logits)."""
    cfg = synth.config(name)
    x = synth.make_x(cfg)
    idx, _ = O.topk_gate(synth.make_logits(cfg, x), cfg.k)
    check(lib, x, idx, synth.make_placement(cfg), cfg.G)
